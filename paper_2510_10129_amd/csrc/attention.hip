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
// K tiles sit in LDS as [key][d] (XOR-swizzled 16-byte chunks); V tiles are
// transposed on the way in to [d][key] so that the PV contraction index (key)
// is contiguous.  Both are double buffered: the next tile's global loads are
// issued before the current tile's MFMAs.
//
// Causality with sorted idx: the key loop of a workgroup ends at the position
// of its last row; the per-row mask only bites between the positions of the
// first and last row of the tile.  Workgroups are issued longest-first and
// workgroup id modulo H_kv picks the kv head, so the workgroups resident on
// one XCD walk the same K/V stream through that XCD's L2.
#include "cc_internal.h"

namespace {

constexpr int BN_KEYS = 64;

template <int D_H>
__global__ __launch_bounds__(256, 2) void sparse_attn_kernel(
    const bf16_t* __restrict__ q, int M, const int32_t* __restrict__ idx, int H_q, int H_kv,
    const bf16_t* __restrict__ Kc, const bf16_t* __restrict__ Vc, int64_t st, int64_t sh, int N,
    bf16_t* __restrict__ o, int n_row_tiles, float scale_log2) {
    constexpr int KS = D_H / 16;        // k-steps of the QK^T contraction
    constexpr int DT = D_H / 32;        // 32-row tiles of O^T
    constexpr int KCPR = D_H / 8;       // 16-byte chunks per K row
    constexpr int K_CH = BN_KEYS * KCPR / 256;
    constexpr int LPR = D_H / 2;        // lanes per V row when each lane loads 2 elements
    constexpr int V_IT = 8 * LPR / 256; // (key group, d pair) items per thread

    __shared__ __align__(16) bf16_t Ks[2][BN_KEYS * D_H];
    __shared__ __align__(16) bf16_t Vt[2][D_H * BN_KEYS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    // wave-wide largest limit: tiles beyond it are skipped by this wave
    int wave_limit = limit;
    for (int off = 32; off > 0; off >>= 1) wave_limit = max(wave_limit, __shfl_xor(wave_limit, off));

    // wave-wide smallest limit of a valid row: tiles that end at or below it need no mask
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

    // ---- global -> LDS staging: per-lane 32-bit offsets from a wave-uniform tile base ----
    const bf16_t* kbase = Kc + (int64_t)kvh * sh;
    const bf16_t* vbase = Vc + (int64_t)kvh * sh;
    const int k_r0 = tid / KCPR, k_c = (tid % KCPR) * 8;      // chunk i: row k_r0 + i*(256/KCPR)
    const int v_kg0 = tid / LPR, v_d = 2 * (tid % LPR);       // item i: key group v_kg0 + i*(256/LPR)
    int koff[K_CH], k_lds[K_CH], voff[V_IT];
#pragma unroll
    for (int i = 0; i < K_CH; ++i) {
        int r = k_r0 + i * (256 / KCPR);
        koff[i] = r * (int)st + k_c;
        k_lds[i] = r * D_H + (((k_c >> 3) ^ (r & 7)) << 3);
    }
#pragma unroll
    for (int i = 0; i < V_IT; ++i) voff[i] = (v_kg0 + i * (256 / LPR)) * 8 * (int)st + v_d;

    u32x4 rk[K_CH];
    uint32_t rv[V_IT][8];
    auto load_tile = [&](int j0) {
        const bf16_t* kb = kbase + (int64_t)j0 * st;
        const bf16_t* vb = vbase + (int64_t)j0 * st;
        if (j0 + BN_KEYS <= N) {
#pragma unroll
            for (int i = 0; i < K_CH; ++i) rk[i] = *reinterpret_cast<const u32x4*>(kb + koff[i]);
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const bf16_t* vr = vb + (int64_t)kk * st;
#pragma unroll
                for (int i = 0; i < V_IT; ++i) rv[i][kk] = *reinterpret_cast<const uint32_t*>(vr + voff[i]);
            }
        } else {   // last tile of the cache: rows past N-1 are clamped (they are masked anyway)
            const int rmax = N - 1 - j0;
#pragma unroll
            for (int i = 0; i < K_CH; ++i) {
                int r = min(k_r0 + i * (256 / KCPR), rmax);
                rk[i] = *reinterpret_cast<const u32x4*>(kb + (int64_t)r * st + k_c);
            }
#pragma unroll
            for (int i = 0; i < V_IT; ++i)
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    int r = min((v_kg0 + i * (256 / LPR)) * 8 + kk, rmax);
                    rv[i][kk] = *reinterpret_cast<const uint32_t*>(vb + (int64_t)r * st + v_d);
                }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < K_CH; ++i) *reinterpret_cast<u32x4*>(&Ks[buf][k_lds[i]]) = rk[i];
#pragma unroll
        for (int i = 0; i < V_IT; ++i) {
            // rv[i][kk] = (V[key kk][d0], V[key kk][d0+1]); regroup into 8 keys per d
            u32x4 lo, hi;
            lo.x = (rv[i][0] & 0xFFFFu) | (rv[i][1] << 16);
            lo.y = (rv[i][2] & 0xFFFFu) | (rv[i][3] << 16);
            lo.z = (rv[i][4] & 0xFFFFu) | (rv[i][5] << 16);
            lo.w = (rv[i][6] & 0xFFFFu) | (rv[i][7] << 16);
            hi.x = (rv[i][0] >> 16) | (rv[i][1] & 0xFFFF0000u);
            hi.y = (rv[i][2] >> 16) | (rv[i][3] & 0xFFFF0000u);
            hi.z = (rv[i][4] >> 16) | (rv[i][5] & 0xFFFF0000u);
            hi.w = (rv[i][6] >> 16) | (rv[i][7] & 0xFFFF0000u);
            // rows with bit 3 of d set keep their two 8-byte halves swapped, so that the
            // 16 lanes of one LDS read pass (d..d+15, same half) touch 16 distinct slots
            const int d0 = v_d, kg = v_kg0 + i * (256 / LPR);
            if (d0 & 8) {
                lo = u32x4{lo.z, lo.w, lo.x, lo.y};
                hi = u32x4{hi.z, hi.w, hi.x, hi.y};
            }
            *reinterpret_cast<u32x4*>(&Vt[buf][d0 * BN_KEYS + ((kg ^ (d0 & 7)) << 3)]) = lo;
            *reinterpret_cast<u32x4*>(&Vt[buf][(d0 + 1) * BN_KEYS + ((kg ^ ((d0 + 1) & 7)) << 3)]) = hi;
        }
    };

    f32x16 acc_o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[dt][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
        const int cur = t & 1;
        const int j0 = t * BN_KEYS;
        const bool more = t + 1 < n_tiles;
        if (more) load_tile(j0 + BN_KEYS);

        if (j0 <= wave_limit) {
            // ---- S^T tile: 64 keys x 32 query rows ----
            f32x16 s[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) s[kt][v] = 0.0f;
                const int r = kt * 32 + qr;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int kc = ks * 2 + hf;
                    bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[cur][r * D_H + ((kc ^ (r & 7)) << 3)]);
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
            const float m_new = fmaxf(m_run, mx);
            const float m_use = m_new == -INFINITY ? 0.0f : m_new;
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
            // rescale only when some row's maximum moved
            if (__any(m_new != m_run)) {
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
                l_run *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc_o[dt][v] *= alpha;
            }
            l_run += psum;
            m_run = m_new;
            // ---- O^T += V^T P^T ----
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const int d = dt * 32 + qr;
                const bf16_t* vrow = &Vt[cur][d * BN_KEYS];
#pragma unroll
                for (int ss = 0; ss < 4; ++ss) {
                    // slots 0..3 <- keys 16ss+4hf.., slots 4..7 <- keys 16ss+8+4hf..
                    const int hsel = 4 * (hf ^ ((d >> 3) & 1));
                    bf16x4 a0 = *reinterpret_cast<const bf16x4*>(vrow + (((2 * ss) ^ (d & 7)) << 3) + hsel);
                    bf16x4 a1 = *reinterpret_cast<const bf16x4*>(vrow + (((2 * ss + 1) ^ (d & 7)) << 3) + hsel);
                    bf16x8 vf;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        vf[u] = a0[u];
                        vf[4 + u] = a1[u];
                    }
                    acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ss], acc_o[dt], 0, 0, 0);
                }
            }
        }
        if (more) store_tile(cur ^ 1);
        __syncthreads();
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
