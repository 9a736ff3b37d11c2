// Sparse-query causal GQA attention over the updated KV cache: recomputed row i
// (global position idx[i]) attends to every cache slot j <= idx[i].  This is
// the kernel Section 5.6 of the paper describes as flash attention with sparse
// query indices; the design below is for gfx950.
//
// Work split: one workgroup = one kv head x BT consecutive recomputed tokens;
// the g = H_q/H_kv query heads that share the kv head are packed with the
// tokens on the 32-wide N side of the MFMA tile (32/g tokens per wave), so a
// K/V tile read from LDS serves the whole query group.
//
// Each wave computes S^T = K Q^T (keys on the MFMA row side, query rows on the
// column side).  In the 32x32 accumulator layout a lane then owns ONE query row
// and 16 keys per tile, so the online-softmax maximum and sum are in-lane
// reductions plus one exchange with lane^32, the rescale factor is a per-lane
// scalar, and the probabilities are already laid out as the B operand of
// O^T = V^T P^T: no shuffle between the two contractions.
//
// K and V tiles (64 keys) go from the cache straight into LDS with 16-byte
// global->LDS loads, row-major as they are stored, two stages each.  K
// fragments are plain 16-byte LDS reads; the V^T fragments (contraction index =
// key) come from the row-major V tile through the transposing LDS read
// ds_read_b64_tr_b16, so V is never transposed in registers.  Both tiles are
// XOR-swizzled (by choosing which global chunk a lane fetches) so that the
// fragment reads spread over the 64 LDS banks.
//
// Causality with sorted idx: the key loop of a workgroup ends at the position
// of its last row; the per-row mask only bites between the positions of the
// first and last row of the tile.  Workgroups are issued longest-first and
// workgroup id modulo H_kv picks the kv head, so the workgroups resident on
// one XCD walk the same K/V stream through that XCD's L2.
#include "cc_internal.h"

namespace {

constexpr int BN_KEYS = 64;

__device__ __forceinline__ void dma16(const bf16_t* gsrc, bf16_t* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const void __attribute__((address_space(1)))*)gsrc,
        (void __attribute__((address_space(3)))*)lds_wave_base, 16, 0, 0);
}

// Transposing LDS read.  Within each group of 16 lanes, lane i receives, as
// element e, element (i % 4) of the 8-byte row addressed by lane (i / 4 + 4 e).
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)p);
}

template <int D_H>
__global__ __launch_bounds__(256, 2) void sparse_attn_kernel(
    const bf16_t* __restrict__ q, int M, const int32_t* __restrict__ idx, int H_q, int H_kv,
    const bf16_t* __restrict__ Kc, const bf16_t* __restrict__ Vc, int64_t st, int64_t sh, int N,
    bf16_t* __restrict__ o, int n_row_tiles, float scale_log2) {
    constexpr int KS = D_H / 16;          // k-steps of the QK^T contraction
    constexpr int DT = D_H / 32;          // 32-row tiles of O^T
    constexpr int CPRW = D_H / 8;         // 16-byte chunks per cache row
    constexpr int RPI = 64 / CPRW;        // rows moved by one global->LDS instruction
    constexpr int NI = BN_KEYS / RPI / 4; // such instructions per wave, tile and tensor

    __shared__ __align__(16) bf16_t Ks0[BN_KEYS * D_H];
    __shared__ __align__(16) bf16_t Ks1[BN_KEYS * D_H];
    __shared__ __align__(16) bf16_t Vs0[BN_KEYS * D_H];
    __shared__ __align__(16) bf16_t Vs1[BN_KEYS * D_H];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform (scalar) on purpose
    const int g = H_q / H_kv;
    const int tw = 32 / g;              // tokens per wave
    const int BT = 4 * tw;              // tokens per workgroup
    const int kvh = blockIdx.x % H_kv;
    const int rt = n_row_tiles - 1 - blockIdx.x / H_kv;

    const int qr = lane & 31, hf = lane >> 5;
    const int tok_in_wave = qr / g, hg = qr - tok_in_wave * g;
    const int mi = rt * BT + wave * tw + tok_in_wave;
    const bool valid = tok_in_wave < tw && mi < M;
    const int limit = valid ? idx[mi] : -1;
    const int last_row = min(M - 1, rt * BT + BT - 1);
    const int kmax = idx[last_row];                    // rows are sorted: the block's longest span
    const int n_tiles = kmax / BN_KEYS + 1;
    // Workgroups with the longest key loops decide when the kernel ends: give their
    // waves issue priority over the short ones they share a SIMD with.
    {
        const int q4 = (4 * n_tiles) / ((N + BN_KEYS - 1) / BN_KEYS + 1);
        if (q4 >= 3) __builtin_amdgcn_s_setprio(3);
        else if (q4 == 2) __builtin_amdgcn_s_setprio(2);
        else if (q4 == 1) __builtin_amdgcn_s_setprio(1);
    }

    // wave-wide largest limit (tiles beyond it are skipped by this wave) and smallest
    // limit of a valid row (tiles that end at or below it need no mask)
    int wave_limit = limit;
    for (int off = 32; off > 0; off >>= 1) wave_limit = max(wave_limit, __shfl_xor(wave_limit, off));
    int wave_min = valid ? limit : 0x7fffffff;
    for (int off = 32; off > 0; off >>= 1) wave_min = min(wave_min, __shfl_xor(wave_min, off));

    // ---- Q fragments (B operand of S^T = K Q^T): lane = query row, 8 d's per k-step ----
    bf16x8 qf[KS];
    {
        const bf16_t* qp = q + ((int64_t)(valid ? mi : 0) * H_q + kvh * g + hg) * D_H + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (valid) {
                qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u) qf[ks][u] = (bf16_t)0.0f;
            }
        }
    }

    // ---- global -> LDS: instruction i of this wave moves rows (i*4+wave)*RPI .. +RPI-1;
    //      lane L fills physical chunk L % CPRW of row L / CPRW and fetches the logical
    //      chunk that the swizzle maps there ----
    //   K rows: chunk c sits at slot c ^ kswz(row)           (16-byte fragment reads)
    //   V rows: the 64-byte group dt sits at group dt ^ vswz(row)  (transposing 8-byte reads)
    auto kswz = [](int r) { return D_H == 128 ? (r & 15) : ((r >> 1) & 7); };
    auto vswz = [](int r) { return D_H == 128 ? (r & 3) : ((r >> 1) & 1); };
    const bf16_t* kbase = Kc + (int64_t)kvh * sh;
    const bf16_t* vbase = Vc + (int64_t)kvh * sh;
    const int l_row = lane / CPRW, l_p = lane % CPRW;
    int d_row[NI], k_col[NI], v_col[NI], koff[NI], voff[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int r = (i * 4 + wave) * RPI + l_row;
        d_row[i] = r;
        k_col[i] = (l_p ^ kswz(r)) * 8;
        v_col[i] = ((((l_p >> 2) ^ vswz(r)) << 2) | (l_p & 3)) * 8;
        koff[i] = r * (int)st + k_col[i];     // 32-bit lane offsets from a wave-uniform tile base
        voff[i] = r * (int)st + v_col[i];
    }
    auto dma_tile = [&](bf16_t* ks, bf16_t* vs, int j0) {
        const bf16_t* kb = kbase + (int64_t)j0 * st;
        const bf16_t* vb = vbase + (int64_t)j0 * st;
        if (j0 + BN_KEYS <= N) {
#pragma unroll
            for (int i = 0; i < NI; ++i) dma16(kb + koff[i], ks + (i * 4 + wave) * RPI * D_H);
#pragma unroll
            for (int i = 0; i < NI; ++i) dma16(vb + voff[i], vs + (i * 4 + wave) * RPI * D_H);
        } else {   // last tile of the cache: rows past N-1 are clamped (they are masked anyway)
            const int rmax = N - 1 - j0;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int r = min(d_row[i], rmax);
                dma16(kb + (int64_t)r * st + k_col[i], ks + (i * 4 + wave) * RPI * D_H);
                dma16(vb + (int64_t)r * st + v_col[i], vs + (i * 4 + wave) * RPI * D_H);
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the loads ahead of the tile's math
    };

    // ---- fragment addresses ----
    // K: row kt*32 + qr, logical chunk 2 ks + hf
    const int k_frag_row = qr * D_H;
    const int k_sw = kswz(qr);
    // V^T through the transposing read: lane s of a 16-lane group addresses key
    // (4 hf + s/4) and the 4 d's starting at 16*(group%2) + 4*(s%4); the lane then
    // holds 4 consecutive keys of column d = 32 dt + lane%32.
    const int s16 = lane & 15, dsub = (lane >> 4) & 1;
    const int v_key = 4 * hf + (s16 >> 2);
    const int v_sw = vswz(v_key);
    const int v_lane = v_key * D_H + (2 * dsub + ((s16 & 3) >> 1)) * 8 + (s16 & 1) * 4;

    f32x16 acc_o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[dt][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    auto tile_math = [&](const bf16_t* ks_, const bf16_t* vs_, int j0) {
        // ---- S^T tile: 64 keys x 32 query rows ----
        f32x16 s[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kt][v] = 0.0f;
        // the two 32-key halves are independent accumulation chains: alternate them
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int kc = (ks * 2 + hf) ^ k_sw;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks_ + kt * 32 * D_H + k_frag_row + (kc << 3));
                s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kt], 0, 0, 0);
            }
        }
        // ---- causal mask (only in tiles that reach past the wave's first row),
        //      online softmax in base 2 with the 1/sqrt(d_h) scale folded into the exponent ----
        if (j0 + BN_KEYS - 1 > wave_min) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int key = j0 + kt * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
                    if (key > limit) s[kt][v] = -INFINITY;
                }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kt][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;
        // The reference point m_run of the exponent is only moved when a row's maximum
        // grew by more than 2^8: until then probabilities up to 256 are accumulated
        // (harmless in fp32 / bf16, and the final division by the row sum cancels it),
        // which keeps the 64-element rescale of O out of most tiles.
        const bool grow = mx > m_run + 8.0f;
        if (__any(grow)) {
            const float m_new = grow ? mx : m_run;
            const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.0f : m_new));
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc_o[dt][v] *= alpha;
            m_run = m_new;
        }
        const float m_use = m_run == -INFINITY ? 0.0f : m_run;
        float psum = 0.0f;
        bf16x8 pf[4];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float p = __builtin_amdgcn_exp2f(fmaf(s[kt][v], scale_log2, -m_use));
                psum += p;
                pf[kt * 2 + (v >> 3)][v & 7] = (bf16_t)p;
            }
        l_run += psum;
        // ---- O^T += V^T P^T: slots 0..3 <- keys 16ss+4hf.., slots 4..7 <- keys 16ss+8+4hf.. ----
#pragma unroll
        for (int ss = 0; ss < 4; ++ss) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {      // DT independent accumulation chains
                const bf16_t* vcol = vs_ + v_lane + ((dt ^ v_sw) << 5);
                bf16x4 a0 = lds_read_tr(vcol + (16 * ss) * D_H);
                bf16x4 a1 = lds_read_tr(vcol + (16 * ss + 8) * D_H);
                bf16x8 vf;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    vf[u] = a0[u];
                    vf[4 + u] = a1[u];
                }
                acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ss], acc_o[dt], 0, 0, 0);
            }
        }
    };

    // ---- key loop: the next tile streams into the idle stage while this one is used;
    //      the barrier waits for the loads (vmcnt) and for every wave to leave the stage ----
    dma_tile(Ks0, Vs0, 0);
    __syncthreads();
    for (int t = 0; t < n_tiles; t += 2) {
        const int j0 = t * BN_KEYS;
        if (t + 1 < n_tiles) dma_tile(Ks1, Vs1, j0 + BN_KEYS);
        if (j0 <= wave_limit) tile_math(Ks0, Vs0, j0);
        __syncthreads();
        if (t + 1 < n_tiles) {
            if (t + 2 < n_tiles) dma_tile(Ks0, Vs0, j0 + 2 * BN_KEYS);
            if (j0 + BN_KEYS <= wave_limit) tile_math(Ks1, Vs1, j0 + BN_KEYS);
            __syncthreads();
        }
    }

    // ---- normalise and write: lane holds 4 consecutive d per (dt, v/4) ----
    float l_tot = l_run + __shfl_xor(l_run, 32);
    if (valid) {
        const float inv = 1.0f / l_tot;
        bf16_t* op = o + ((int64_t)mi * H_q + kvh * g + hg) * D_H;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                bf16x4 w;
#pragma unroll
                for (int u = 0; u < 4; ++u) w[u] = (bf16_t)(acc_o[dt][vq * 4 + u] * inv);
                *reinterpret_cast<bf16x4*>(op + dt * 32 + 8 * vq + 4 * hf) = w;
            }
    }
}

}  // namespace

void cc_launch_attention(const bf16_t* q, int M, const int32_t* idx, const cc_model_desc& m,
                         const cc_kv_layer& kv, bf16_t* o, hipStream_t s) {
    if (M <= 0) return;
    const int g = m.H_q / m.H_kv;
    const int BT = 4 * (32 / g);
    const int n_row_tiles = (M + BT - 1) / BT;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)m.d_h);
    dim3 grid(n_row_tiles * m.H_kv), block(256);
    if (m.d_h == 128)
        hipLaunchKernelGGL(sparse_attn_kernel<128>, grid, block, 0, s, q, M, idx, m.H_q, m.H_kv,
                           (const bf16_t*)kv.K, (const bf16_t*)kv.V, kv.stride_token, kv.stride_head,
                           kv.N, o, n_row_tiles, scale_log2);
    else
        hipLaunchKernelGGL(sparse_attn_kernel<64>, grid, block, 0, s, q, M, idx, m.H_q, m.H_kv,
                           (const bf16_t*)kv.K, (const bf16_t*)kv.V, kv.stride_token, kv.stride_head,
                           kv.N, o, n_row_tiles, scale_log2);
}
