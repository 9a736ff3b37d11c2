// Online assembly of one layer's global KV cache from per-chunk caches
// (Section 4.1 of the paper): one copy of the shared prefix, every chunk's own
// rows appended, keys re-numbered from chunk-local to global positions by one
// more rotary rotation (rotations by p and by delta compose to p + delta).
// Pure data movement plus 2 multiply-adds per key element: bound by HBM.
//
// A wave owns CC_ASM_ROWS consecutive destination rows of one segment, so the
// (cos, sin) of the segment's position shift are loaded once per wave and kept
// in registers.  Per key row a lane moves one 16-byte piece of the low half of
// a head and the matching piece of the high half (the two members of every
// rotary pair meet in one lane); value rows are 16-byte copies.  Loads of eight
// rows are issued before their stores.
#include "cc_internal.h"

namespace {

__device__ __forceinline__ bf16x8 zero8() {
    bf16x8 z;
#pragma unroll
    for (int u = 0; u < 8; ++u) z[u] = (bf16_t)0.0f;
    return z;
}

template <int D_H>
__global__ __launch_bounds__(256) void assemble_kernel(cc_asm_args a, const float2* __restrict__ rope,
                                                       int H_kv, int64_t src_st, int64_t src_sh,
                                                       bf16_t* __restrict__ Kd, bf16_t* __restrict__ Vd,
                                                       int64_t dst_st, int64_t dst_sh) {
    constexpr int HALF = D_H / 2;
    constexpr int UPH = HALF / 8;          // (lo, hi) 16-byte pairs per head
    constexpr int CPH = D_H / 8;           // 16-byte chunks per head
    constexpr int RU = 8;                  // rows in flight
    const int lane = threadIdx.x & 63;
    const int blk = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
    if (blk >= a.n_blocks) return;
    int s = 0;                             // last segment whose first block is <= blk
    for (int lo = 0, hi = a.n_seg - 1; lo <= hi;) {
        const int mid = (lo + hi) >> 1;
        if (a.seg[mid].blk0 <= blk) { s = mid; lo = mid + 1; } else { hi = mid - 1; }
    }
    const cc_asm_seg sg = a.seg[s];
    const int r0 = (blk - sg.blk0) * CC_ASM_ROWS;
    const int r1 = min(sg.len, r0 + CC_ASM_ROWS);
    const bool zero = sg.K == nullptr;

    // ---- keys ----
    for (int u = lane; u < H_kv * UPH; u += 64) {
        const int h = u / UPH, j0 = (u - h * UPH) * 8;
        float2 cs[8];
        if (sg.delta != 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) cs[e] = rope[(int64_t)sg.delta * HALF + j0 + e];
        }
        const bf16_t* src = sg.K + (int64_t)h * src_sh + j0;
        bf16_t* dst = Kd + (int64_t)sg.dst * dst_st + (int64_t)h * dst_sh + j0;
        for (int r = r0; r < r1; r += RU) {
            bf16x8 lo[RU], hi[RU];
#pragma unroll
            for (int i = 0; i < RU; ++i) {
                const int rr = min(r + i, r1 - 1);       // rows past the end repeat the last one
                if (zero) {
                    lo[i] = zero8();
                    hi[i] = zero8();
                } else {
                    lo[i] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(src + (int64_t)rr * src_st));
                    hi[i] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(src + (int64_t)rr * src_st + HALF));
                }
            }
#pragma unroll
            for (int i = 0; i < RU; ++i) {
                if (r + i >= r1) break;
                bf16x8 ol = lo[i], oh = hi[i];
                if (sg.delta != 0) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float x = (float)lo[i][e], y = (float)hi[i][e];
                        ol[e] = (bf16_t)(x * cs[e].x - y * cs[e].y);
                        oh[e] = (bf16_t)(y * cs[e].x + x * cs[e].y);
                    }
                }
                bf16_t* d = dst + (int64_t)(r + i) * dst_st;
                __builtin_nontemporal_store(ol, reinterpret_cast<bf16x8*>(d));
                __builtin_nontemporal_store(oh, reinterpret_cast<bf16x8*>(d + HALF));
            }
        }
    }
    // ---- values ----
    for (int c = lane; c < H_kv * CPH; c += 64) {
        const int h = c / CPH, e0 = (c - h * CPH) * 8;
        const bf16_t* src = sg.V + (int64_t)h * src_sh + e0;
        bf16_t* dst = Vd + (int64_t)sg.dst * dst_st + (int64_t)h * dst_sh + e0;
        for (int r = r0; r < r1; r += RU) {
            bf16x8 v[RU];
#pragma unroll
            for (int i = 0; i < RU; ++i) {
                const int rr = min(r + i, r1 - 1);
                v[i] = zero ? zero8()
                            : __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(src + (int64_t)rr * src_st));
            }
#pragma unroll
            for (int i = 0; i < RU; ++i) {
                if (r + i >= r1) break;
                __builtin_nontemporal_store(v[i], reinterpret_cast<bf16x8*>(dst + (int64_t)(r + i) * dst_st));
            }
        }
    }
}

}  // namespace

void cc_launch_assemble(const cc_asm_args& a, const float2* rope, const cc_model_desc& m,
                        int64_t src_st, int64_t src_sh, const cc_kv_layer& dst, hipStream_t s) {
    if (a.n_blocks <= 0) return;
    dim3 grid((a.n_blocks + 3) / 4), block(256);
    if (m.d_h == 128)
        hipLaunchKernelGGL(assemble_kernel<128>, grid, block, 0, s, a, rope, m.H_kv, src_st, src_sh,
                           (bf16_t*)dst.K, (bf16_t*)dst.V, dst.stride_token, dst.stride_head);
    else
        hipLaunchKernelGGL(assemble_kernel<64>, grid, block, 0, s, a, rope, m.H_kv, src_st, src_sh,
                           (bf16_t*)dst.K, (bf16_t*)dst.V, dst.stride_token, dst.stride_head);
}
