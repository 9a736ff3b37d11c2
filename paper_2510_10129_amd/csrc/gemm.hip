// bf16 MFMA GEMMs of the recompute path: C[M,N] = A[M,K] * B[N,K]^T with fp32
// accumulation, where A holds the (few) recomputed rows and B a weight matrix
// stored [out][in].  Four fused epilogues:
//   QKV     bias + rotary embedding at the token's global position, q to the
//           query buffer, k/v scattered into the KV cache rows idx[i]
//   OPROJ   + residual (gathered hidden row) -> fp32 residual stream
//   GATE_UP B tile = 64 gate rows + 64 up rows; writes silu(gate)*up
//   DOWN    + residual stream -> bf16 layer output
//
// Tiling: one workgroup of WAVES_M x WAVES_N waves computes a BM x BN tile with
// v_mfma_f32_32x32x16_bf16; the K loop moves BK = 64 columns per step through a
// double-buffered, XOR-swizzled LDS stage filled by direct global->LDS loads
// (no register staging), one barrier per step.  The accumulators are written back through LDS so that
// every global store is 16 or 32 contiguous bytes per lane along the row.
#include <stdlib.h>

#include "cc_internal.h"

namespace {

constexpr int BK = 64;
constexpr int CPR = BK / 8;   // 16-byte chunks per tile row
constexpr int RG = 32;        // rows staged through LDS at a time in the epilogue

struct BSingle {
    const bf16_t* B;
    int ldb, N;
    template <int BN>
    __device__ __forceinline__ const bf16_t* row(int bn, int r) const {
        int n = bn * BN + r;
        n = n < N ? n : N - 1;
        return B + (int64_t)n * ldb;
    }
};

// rows [0, BN/2) of the tile come from B0 (gate), rows [BN/2, BN) from B1 (up)
struct BDual {
    const bf16_t* B0;
    const bf16_t* B1;
    int ldb, f;
    template <int BN>
    __device__ __forceinline__ const bf16_t* row(int bn, int r) const {
        constexpr int H = BN / 2;
        int n = bn * H + (r < H ? r : r - H);
        n = n < f ? n : f - 1;
        return (r < H ? B0 : B1) + (int64_t)n * ldb;
    }
};

__device__ __forceinline__ void store_bf16x8(bf16_t* dst, const float* v) {
    bf16x8 o;
#pragma unroll
    for (int u = 0; u < 8; ++u) o[u] = (bf16_t)v[u];
    *reinterpret_cast<bf16x8*>(dst) = o;
}

struct EpiQKV {
    const int32_t* idx;
    const bf16_t* bias;
    const float2* rope;
    int H_q, H_kv, d_h, N;
    bf16_t* q_out;
    bf16_t* K;
    bf16_t* V;
    int64_t st, sh;
    template <int BN>
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow) const {
        const int n = bn * BN + cc;
        if (n >= N) return;
        const int head = n / d_h, c = n - head * d_h, half = d_h >> 1;
        const int pos = idx[m];
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = crow[cc + u];
        if (bias) {
            bf16x8 b = *reinterpret_cast<const bf16x8*>(bias + n);
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] += (float)b[u];
        }
        if (head < H_q + H_kv) {
            const bool lo = c < half;
            const int pcc = lo ? cc + half : cc - half;
            const int pn = lo ? n + half : n - half;
            const int j = lo ? c : c - half;
            float p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) p[u] = crow[pcc + u];
            if (bias) {
                bf16x8 b = *reinterpret_cast<const bf16x8*>(bias + pn);
#pragma unroll
                for (int u = 0; u < 8; ++u) p[u] += (float)b[u];
            }
            const float2* cs = rope + (int64_t)pos * half + j;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                float2 t = cs[u];
                v[u] = lo ? v[u] * t.x - p[u] * t.y : v[u] * t.x + p[u] * t.y;
            }
        }
        bf16_t* dst;
        if (head < H_q)
            dst = q_out + (int64_t)m * H_q * d_h + n;
        else if (head < H_q + H_kv)
            dst = K + (int64_t)pos * st + (int64_t)(head - H_q) * sh + c;
        else
            dst = V + (int64_t)pos * st + (int64_t)(head - H_q - H_kv) * sh + c;
        store_bf16x8(dst, v);
    }
};

struct EpiOProj {
    const bf16_t* hidden;
    const int32_t* gather_idx;
    int d;
    float* y;
    template <int BN>
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow) const {
        const int n = bn * BN + cc;
        if (n >= d) return;
        const int64_t src = gather_idx ? (int64_t)gather_idx[m] : (int64_t)m;
        bf16x8 x = *reinterpret_cast<const bf16x8*>(hidden + src * d + n);
        f32x4 a, b;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a[u] = crow[cc + u] + (float)x[u];
            b[u] = crow[cc + 4 + u] + (float)x[4 + u];
        }
        f32x4* dst = reinterpret_cast<f32x4*>(y + (int64_t)m * d + n);
        dst[0] = a;
        dst[1] = b;
    }
};

struct EpiGateUp {
    int f;
    bf16_t* act;
    template <int BN>
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow) const {
        constexpr int H = BN / 2;
        if (cc >= H) return;
        const int n = bn * H + cc;
        if (n >= f) return;
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float g = crow[cc + u], up = crow[cc + H + u];
            v[u] = g / (1.0f + __expf(-g)) * up;
        }
        store_bf16x8(act + (int64_t)m * f + n, v);
    }
};

struct EpiDown {
    const float* y;
    int d;
    bf16_t* out;
    template <int BN>
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow) const {
        const int n = bn * BN + cc;
        if (n >= d) return;
        const f32x4* r = reinterpret_cast<const f32x4*>(y + (int64_t)m * d + n);
        f32x4 a = r[0], b = r[1];
        float v[8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v[u] = crow[cc + u] + a[u];
            v[4 + u] = crow[cc + 4 + u] + b[u];
        }
        store_bf16x8(out + (int64_t)m * d + n, v);
    }
};

// Consecutive workgroup ids go round-robin to the 8 XCDs (each with its own
// L2); give every XCD one contiguous range of tiles so that workgroups sharing
// a weight tile also share an L2.
__device__ __forceinline__ int xcd_remap(int bid, int nb) {
    const int q = nb >> 3, r = nb & 7;
    const int x = bid & 7, local = bid >> 3;
    return x * q + (x < r ? x : r) + local;
}

// 16 bytes per lane straight from global memory into LDS (no VGPR staging, no
// LDS store instruction).  The LDS destination is wave-uniform: lane L lands at
// lds_base + 16*L.  Completion is tracked by vmcnt like any vector load.
__device__ __forceinline__ void dma16(const bf16_t* gsrc, bf16_t* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const void __attribute__((address_space(1)))*)gsrc,
        (void __attribute__((address_space(3)))*)lds_wave_base, 16, 0, 0);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, class BSrc, class Epi>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_nt_kernel(
    const bf16_t* __restrict__ A, int lda, int M, int K, int tiles_m, int tiles_n, BSrc bsrc,
    Epi epi) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int NT = NW * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_CH = BM * CPR / NT, B_CH = BN * CPR / NT;   // DMA instructions per wave and tile
    static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile/threads");
    static_assert(BM % RG == 0 && WM % 32 == 0 && WN % 32 == 0, "wave tile");
    static_assert(RG * (BN + 4) * 4 <= (BM + BN) * BK * 2, "epilogue stage fits in one pipeline stage");

    // Two pipeline stages as separate arrays, so that a DMA into one stage is
    // known not to alias the fragment reads of the other.
    __shared__ __align__(16) bf16_t st0[(BM + BN) * BK];
    __shared__ __align__(16) bf16_t st1[(BM + BN) * BK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
    const int vb = xcd_remap(blockIdx.x, tiles_m * tiles_n);
    const int bm = vb % tiles_m, bn = vb / tiles_m;   // neighbours share the weight tile
    const int m0 = bm * BM;

    // One DMA instruction moves 8 tile rows (8 x 128 B).  Lane L fills physical
    // chunk slot L%8 of row L/8; the XOR swizzle (slot = chunk ^ ((row>>1)&7),
    // conflict-free on the 64-bank LDS for 16-byte fragment reads) is applied by
    // choosing which global chunk the lane fetches.
    const bf16_t* ag[A_CH];
    const bf16_t* bg[B_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int r = (i * NW + wave) * 8 + (lane >> 3);
        int c = (lane & 7) ^ ((r >> 1) & 7);
        int m = m0 + r;
        m = m < M ? m : M - 1;
        ag[i] = A + (int64_t)m * lda + c * 8;
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        int r = (i * NW + wave) * 8 + (lane >> 3);
        int c = (lane & 7) ^ ((r >> 1) & 7);
        bg[i] = bsrc.template row<BN>(bn, r) + c * 8;
    }
    auto dma_tile = [&](bf16_t* stage, int kt) {
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) dma16(ag[i] + k0, stage + (i * NW + wave) * 8 * BK);
#pragma unroll
        for (int i = 0; i < B_CH; ++i) dma16(bg[i] + k0, stage + BM * BK + (i * NW + wave) * 8 * BK);
        // keep the loads at the top of the iteration: the compiler would otherwise sink
        // them below the MFMAs, next to the barrier that waits for them
        __builtin_amdgcn_sched_barrier(0);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int frow = lane & 31, fk = lane >> 5;
    const int fsw = (frow >> 1) & 7;      // rows of a fragment differ by multiples of 32
    auto compute = [&](const bf16_t* stage) {
        const bf16_t* as = stage;
        const bf16_t* bs = stage + BM * BK;
        bf16x8 af[2][TM], bfr[2][TN];
        auto load_frags = [&](int ks, int fb) {
            const int sl = ((ks * 2 + fk) ^ fsw) << 3;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[fb][i] = *reinterpret_cast<const bf16x8*>(as + (wm0 + i * 32 + frow) * BK + sl);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[fb][j] = *reinterpret_cast<const bf16x8*>(bs + (wn0 + j * 32 + frow) * BK + sl);
        };
        load_frags(0, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) load_frags(ks + 1, (ks + 1) & 1);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j],
                                                                        acc[i][j], 0, 0, 0);
        }
        // issue order: the first k-step's fragments, then every MFMA followed by one
        // fragment read of the next k-step, so LDS latency hides behind the matrix pipe
        constexpr int NF = TM + TN, NM = TM * TN;
        __builtin_amdgcn_sched_group_barrier(0x100, NF, 0);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks)
#pragma unroll
            for (int mm = 0; mm < NM; ++mm) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (ks + 1 < BK / 16 && mm < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
    };

    // K loop: while tile kt is multiplied out of one stage, the DMA engine fills
    // the other with tile kt+1; the barrier at the end of the iteration waits for
    // both (vmcnt for the DMA, every wave done reading).
    const int KT = K / BK;
    dma_tile(st0, 0);
    __syncthreads();
    int kt = 0;
    for (; kt + 2 <= KT; kt += 2) {
        dma_tile(st1, kt + 1);
        compute(st0);
        __syncthreads();
        if (kt + 2 < KT) dma_tile(st0, kt + 2);
        compute(st1);
        __syncthreads();
    }
    if (kt < KT) {
        compute(st0);
        __syncthreads();
    }

    // ---- epilogue: accumulators -> LDS (fp32, RG rows at a time) -> fused store ----
    float* stage = reinterpret_cast<float*>(st0);
    constexpr int LDS_LD = BN + 4;
    constexpr int TPR = BN / 8;           // threads per staged row
    constexpr int RPP = NT / TPR;         // rows per pass
#pragma unroll
    for (int rg = 0; rg < BM / RG; ++rg) {
        if (rg) __syncthreads();
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int tr = wm0 + i * 32;
            if (tr / RG == rg) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int r = (tr % RG) + 8 * (v >> 2) + 4 * fk + (v & 3);
                        stage[r * LDS_LD + wn0 + j * 32 + frow] = acc[i][j][v];
                    }
            }
        }
        __syncthreads();
        const int cc = (tid % TPR) * 8;
        for (int r = tid / TPR; r < RG; r += RPP) {
            int m = m0 + rg * RG + r;
            if (m < M) epi.template operator()<BN>(m, bn, cc, stage + r * LDS_LD);
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, class BSrc, class Epi>
void launch_gemm_cfg(const bf16_t* A, int lda, int M, int N_tiles_cols, int K, BSrc bsrc, Epi epi,
                 hipStream_t s) {
    // N_tiles_cols: number of output columns covered by tiles of BN
    auto kern = gemm_nt_kernel<BM, BN, WAVES_M, WAVES_N, BSrc, Epi>;
    constexpr int lds = 0;
    int tiles_m = (M + BM - 1) / BM, tiles_n = (N_tiles_cols + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WAVES_M * WAVES_N * 64), lds, s, A, lda,
                       M, K, tiles_m, tiles_n, bsrc, epi);
}

// Two tile shapes: 256x256 (8 waves of 128x64, least LDS and L1 traffic per
// flop, one workgroup per CU) and 128x128 (4 waves of 64x64, two per CU, about
// 0.88 of the large tile's rate).  A grid runs as a whole number of "rounds" of
// workgroups, so the shape is chosen per launch to minimise rounds x tile cost.
template <class BSrc, class Epi>
void launch_gemm(const bf16_t* A, int lda, int M, int N_tiles_cols, int K, BSrc bsrc, Epi epi,
                 hipStream_t s) {
    static const int n_cu = [] {
        int dev = 0, n = 256;
        if (hipGetDevice(&dev) == hipSuccess)
            (void)hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        return n > 0 ? n : 256;
    }();
    static const char* force = getenv("CC_GEMM_CFG");
    auto cost = [&](int bm, int bn, int per_cu, double eff) {
        const long tiles = (long)((M + bm - 1) / bm) * ((N_tiles_cols + bn - 1) / bn);
        const long slots = (long)n_cu * per_cu;
        const long rounds = (tiles + slots - 1) / slots;
        return (double)rounds * per_cu * bm * bn / eff;
    };
    const double cb = cost(256, 256, 1, 1.00), cs = cost(128, 128, 2, 0.88);
    char pick = cb <= cs ? 'b' : 's';
    if (force) pick = force[0];
    if (pick == 'b')
        launch_gemm_cfg<256, 256, 2, 4>(A, lda, M, N_tiles_cols, K, bsrc, epi, s);
    else
        launch_gemm_cfg<128, 128, 2, 2>(A, lda, M, N_tiles_cols, K, bsrc, epi, s);
}

}  // namespace

void cc_launch_qkv(const bf16_t* xn, int M, const int32_t* idx, const bf16_t* w_qkv,
                   const bf16_t* b_qkv, const cc_model_desc& m, const float2* rope,
                   const cc_kv_layer& kv, bf16_t* q_out, hipStream_t s) {
    if (M <= 0) return;
    const int N = (m.H_q + 2 * m.H_kv) * m.d_h;
    BSingle b{w_qkv, m.d, N};
    EpiQKV e{idx, b_qkv, rope, m.H_q, m.H_kv, m.d_h, N, q_out,
             (bf16_t*)kv.K, (bf16_t*)kv.V, kv.stride_token, kv.stride_head};
    launch_gemm(xn, m.d, M, N, m.d, b, e, s);
}

void cc_launch_oproj(const bf16_t* o, int M, const bf16_t* w_o, const bf16_t* hidden,
                     const int32_t* gather_idx, const cc_model_desc& m, float* y, hipStream_t s) {
    if (M <= 0) return;
    const int K = m.H_q * m.d_h;
    BSingle b{w_o, K, m.d};
    EpiOProj e{hidden, gather_idx, m.d, y};
    launch_gemm(o, K, M, m.d, K, b, e, s);
}

void cc_launch_gate_up(const bf16_t* mn, int M, const bf16_t* w_gate, const bf16_t* w_up,
                       const cc_model_desc& m, bf16_t* act, hipStream_t s) {
    if (M <= 0) return;
    BDual b{w_gate, w_up, m.d, m.f};
    EpiGateUp e{m.f, act};
    // each 128-column tile holds 64 gate + 64 up columns: 2*f tile columns in total
    launch_gemm(mn, m.d, M, 2 * m.f, m.d, b, e, s);
}

void cc_launch_down(const bf16_t* act, int M, const bf16_t* w_down, const float* y,
                    const cc_model_desc& m, bf16_t* out, hipStream_t s) {
    if (M <= 0) return;
    BSingle b{w_down, m.f, m.d};
    EpiDown e{y, m.d, out};
    launch_gemm(act, m.f, M, m.d, m.f, b, e, s);
}
