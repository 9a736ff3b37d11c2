// bf16 MFMA GEMMs of the recompute path: C[M,N] = A[M,K] * B[N,K]^T with fp32
// accumulation, where A holds the (few) recomputed rows and B a weight matrix
// stored [out][in].  Four fused epilogues:
//   QKV     bias + rotary embedding at the token's global position, q to the
//           query buffer, k/v scattered into the KV cache rows idx[i]
//   OPROJ   + residual (gathered hidden row) -> fp32 residual stream
//   GATE_UP B tile = 64 gate rows + 64 up rows; writes silu(gate)*up
//   DOWN    + residual stream -> bf16 layer output
//
// Tiling: one workgroup of WAVES_M x WAVES_N waves computes a BM x BN tile.  Operands
// go from global memory straight into LDS (16-byte global->LDS loads, no register
// staging), XOR-swizzled so that the 16-byte fragment reads are conflict-free on the
// 64-bank LDS.  Three K loops:
//   ring16 (K % 128 == 0; gemm_ring16_kernel, what every projection of the model
//          widths runs) slices of 32 columns in a ring of four LDS slots; a slice is
//          requested three slices (96 columns of MFMA work) before it is read, which
//          hides the L2/fabric latency that a two-stage pipeline exposes; one barrier
//          per slice, waits by explicit vmcnt; v_mfma_f32_16x16x32_bf16 (one k-step per
//          slice) with hand-written fragment reads and hand-counted lgkmcnt waits.
//   ring   (gemm_ring_kernel) the same ring with v_mfma_f32_32x32x16_bf16 and
//          compiler-scheduled fragment reads; kept as a cross-check behind
//          cc_debug_set_launch.
//   staged (any K % 64 == 0; gemm_nt_kernel) two stages of 64 columns, one barrier
//          per stage, 32x32x16 MFMAs.
// The accumulators are written back through LDS so that every global store is
// 16 or 32 contiguous bytes per lane along the row.
#include "cc_internal.h"
#include <type_traits>

namespace {

struct BSingle {
    const bf16_t* B;
    int ldb, N;
    template <int BN>
    __device__ __forceinline__ const bf16_t* row(int bn, int r) const {
        int n = bn * BN + r;
        n = n < N ? n : N - 1;
        return B + (int64_t)n * ldb;
    }
    // ring loop: tile rows [half*BN/2, (half+1)*BN/2) start at base() and there are
    // rows_left() valid rows from there (rows past the end are clamped by the caller)
    template <int BN>
    __device__ __forceinline__ const bf16_t* base(int bn, int half) const {
        int n0 = bn * BN + half * (BN / 2);
        n0 = n0 < N ? n0 : N - 1;
        return B + (int64_t)n0 * ldb;
    }
    template <int BN>
    __device__ __forceinline__ int rows_left(int bn, int half) const {
        const int l = N - bn * BN - half * (BN / 2);
        return l < 1 ? 1 : l;
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
    template <int BN>
    __device__ __forceinline__ const bf16_t* base(int bn, int half) const {
        int n0 = bn * (BN / 2);
        n0 = n0 < f ? n0 : f - 1;
        return (half ? B1 : B0) + (int64_t)n0 * ldb;
    }
    template <int BN>
    __device__ __forceinline__ int rows_left(int bn, int half) const {
        const int l = f - bn * (BN / 2);
        return l < 1 ? 1 : l;
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
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow, int swz) const {
        const int n = bn * BN + cc;
        if (n >= N) return;
        const int head = n / d_h, c = n - head * d_h, half = d_h >> 1;
        const int pos = idx[m];
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = crow[(cc ^ swz) + u];
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
            for (int u = 0; u < 8; ++u) p[u] = crow[(pcc ^ swz) + u];
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
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow, int swz) const {
        const int n = bn * BN + cc;
        if (n >= d) return;
        const int64_t src = gather_idx ? (int64_t)gather_idx[m] : (int64_t)m;
        bf16x8 x = *reinterpret_cast<const bf16x8*>(hidden + src * d + n);
        const float* cr = crow + (cc ^ swz);
        f32x4 a, b;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a[u] = cr[u] + (float)x[u];
            b[u] = cr[4 + u] + (float)x[4 + u];
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
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow, int swz) const {
        constexpr int H = BN / 2;
        if (cc >= H) return;
        const int n = bn * H + cc;
        if (n >= f) return;
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float g = crow[(cc ^ swz) + u], up = crow[((cc + H) ^ swz) + u];
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
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow, int swz) const {
        const int n = bn * BN + cc;
        if (n >= d) return;
        const f32x4* r = reinterpret_cast<const f32x4*>(y + (int64_t)m * d + n);
        f32x4 a = r[0], b = r[1];
        const float* cr = crow + (cc ^ swz);
        float v[8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v[u] = cr[u] + a[u];
            v[4 + u] = cr[4 + u] + b[u];
        }
        store_bf16x8(out + (int64_t)m * d + n, v);
    }
};

// Split-K: workgroup row blockIdx.y of a launch computes the products over its share of K and
// leaves its fp32 tile in a workspace [share][tile slot][256][256] (slot = the tile's index
// within the launch); splitk_finish_kernel adds the shares and applies the launch's own
// epilogue functor.
struct EpiPartial {
    float* ws;
    int64_t share_stride;     // floats per share: slots * 65536
    int slot, m0;             // set by the kernel: this workgroup's slot and first row
    template <int BN>
    __device__ __forceinline__ void operator()(int m, int bn, int cc, const float* crow, int swz) const {
        static_assert(BN == 256, "slots are 256 columns wide");
        float* dst = ws + blockIdx.y * share_stride + (int64_t)slot * 65536 + (m - m0) * 256 + cc;
        const f32x4* cr = reinterpret_cast<const f32x4*>(crow + (cc ^ swz));
        reinterpret_cast<f32x4*>(dst)[0] = cr[0];
        reinterpret_cast<f32x4*>(dst)[1] = cr[1];
    }
};
template <class Epi>
__device__ __forceinline__ Epi epi_for_tile(const Epi& e, int, int) { return e; }
__device__ __forceinline__ EpiPartial epi_for_tile(const EpiPartial& e, int slot, int m0) {
    EpiPartial r = e;
    r.slot = slot;
    r.m0 = m0;
    return r;
}

__device__ __forceinline__ void tile_of_seq(int vb, int tiles_m, int tiles_n, int GM, int* bm, int* bn);

// One workgroup per 8 rows of one tile slot: sums the shares of each 8-column chunk into an LDS
// row, then every thread calls the functor on its chunk (functors may read other chunks of the
// row: the RoPE partner, the up half of a gate/up tile).
template <class Epi>
__global__ __launch_bounds__(256) void splitk_finish_kernel(const float* __restrict__ ws, int64_t share_stride,
                                                            int n_shares, int M, int BM, int vb0, int tiles_m,
                                                            int tiles_n, int GM, Epi epi) {
    constexpr int BN = 256, TPR = BN / 8, ROWS = 256 / TPR;
    __shared__ __align__(16) float stage[ROWS][BN];
    const int r = threadIdx.x / TPR, cc = (threadIdx.x % TPR) * 8;
    int bm, bn;
    tile_of_seq(vb0 + blockIdx.x, tiles_m, tiles_n, GM, &bm, &bn);
    const int row = blockIdx.y * ROWS + r, m = bm * BM + row;
    const bool on = row < BM && m < M;
    if (on) {
        const float* src = ws + (int64_t)blockIdx.x * 65536 + row * 256 + cc;
        f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
        for (int sp = 0; sp < n_shares; ++sp) {
            const f32x4* p = reinterpret_cast<const f32x4*>(src + sp * share_stride);
            a += p[0];
            b += p[1];
        }
        *reinterpret_cast<f32x4*>(&stage[r][cc]) = a;
        *reinterpret_cast<f32x4*>(&stage[r][cc + 4]) = b;
    }
    __syncthreads();
    if (on) epi.template operator()<BN>(m, bn, cc, stage[r], 0);
}

// Consecutive workgroup ids go round-robin to the 8 XCDs (each with its own
// L2).  Every XCD gets one contiguous range of the tile sequence, and the
// sequence walks bands of GM row-tiles column by column, so the workgroups that
// run together on an XCD form a GM x (32/GM) block of tiles: they share GM
// tiles of A and 32/GM tiles of B through that L2.
// tile `vb` of the sequence (bands of GM row-tiles, column by column)
__device__ __forceinline__ void tile_of_seq(int vb, int tiles_m, int tiles_n, int GM, int* bm, int* bn) {
    const int band = GM * tiles_n;
    const int b = vb / band, rb = vb - b * band;
    const int gm = min(GM, tiles_m - b * GM);
    *bm = b * GM + rb % gm;
    *bn = rb / gm;
}
// workgroup `bid` of a launch over tiles vb0 .. vb0 + nb - 1 of the sequence; returns its tile's index
__device__ __forceinline__ int tile_of_block(int bid, int nb, int vb0, int tiles_m, int tiles_n, int GM,
                                             int* bm, int* bn) {
    const int q = nb >> 3, r = nb & 7;
    const int x = bid & 7, local = bid >> 3;
    const int vb = vb0 + x * q + (x < r ? x : r) + local;
    tile_of_seq(vb, tiles_m, tiles_n, GM, bm, bn);
    return vb;
}
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int GM, int* bm,
                                              int* bn) {
    (void)tile_of_block(bid, tiles_m * tiles_n, 0, tiles_m, tiles_n, GM, bm, bn);
}

// 16 bytes per lane straight from global memory into LDS (no VGPR staging, no
// LDS store instruction).  The LDS destination is wave-uniform: lane L lands at
// lds_base + 16*L.  Completion is tracked by vmcnt like any vector load.
__device__ __forceinline__ void dma16(const bf16_t* gsrc, bf16_t* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const void __attribute__((address_space(1)))*)gsrc,
        (void __attribute__((address_space(3)))*)lds_wave_base, 16, 0, 0);
}

// The same with an immediate offset, added to both the LDS and the global address: loads
// that share a wave base need no rewrite of M0 between them.
template <int OFF>
__device__ __forceinline__ void dma16_at(const char* gsrc_minus_off, bf16_t* lds_wave_base) {
    static_assert(OFF >= 0 && OFF < 4096, "the instruction offset is 13 bits signed; a larger value wraps silently");
    __builtin_amdgcn_global_load_lds(
        (const void __attribute__((address_space(1)))*)gsrc_minus_off,
        (void __attribute__((address_space(3)))*)lds_wave_base, 16, OFF, 0);
}
template <int N, int I = 0, class F>
__device__ __forceinline__ void unrolled(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        unrolled<N, I + 1>(f);
    }
}

// Workgroup barrier without the memory fence of __syncthreads() (that fence waits for
// every outstanding global->LDS load; the ring loop waits only for the slice it needs,
// with wait_vm_lds0 just before).  The empty asm statements keep the compiler from
// moving LDS accesses across the barrier.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// s_waitcnt: at most N vector-memory operations outstanding, no LDS operation.
template <int N>
__device__ __forceinline__ void wait_vm_lds0() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4));
}

// Accumulators -> LDS (fp32, RG rows at a time) -> fused store.  `stage` must
// hold RG * (BN + 4) floats and no wave may still be reading operands from it.
template <int BM, int BN, int WAVES_M, int WAVES_N, int RG, class Epi>
__device__ __forceinline__ void store_tile(f32x16 (&acc)[BM / WAVES_M / 32][BN / WAVES_N / 32],
                                           float* stage, int m0, int bn, int M, const Epi& epi) {
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int LDS_LD = BN + 4;
    constexpr int TPR = BN / 8;           // threads per staged row
    constexpr int RPP = NT / TPR;         // rows per pass
    static_assert(RG == 32 || RG == 16, "row group");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
    const int frow = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int rg = 0; rg < BM / RG; ++rg) {
        if (rg) __syncthreads();
        // register v of a 32x32 accumulator tile holds tile row 8*(v>>2) + 4*fk + (v&3):
        // the rows of this group are those of one accumulator tile (or of its half `sub`)
        constexpr int VPG = 16 * RG / 32;                 // accumulator registers per row group
        const int sub = (rg * RG % 32) / RG;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int tr = wm0 + i * 32;                  // first row of this accumulator tile
            if (tr / 32 == rg * RG / 32) {                // wave-uniform
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int vv = 0; vv < VPG; ++vv) {
                        const int v = sub * VPG + vv;
                        const int r = 8 * (v >> 2) + 4 * fk + (v & 3) - sub * RG;
                        stage[r * LDS_LD + wn0 + j * 32 + frow] = acc[i][j][v];
                    }
            }
        }
        __syncthreads();
        const int cc = (tid % TPR) * 8;
        for (int r = tid / TPR; r < RG; r += RPP) {
            int m = m0 + rg * RG + r;
            if (m < M) epi.template operator()<BN>(m, bn, cc, stage + r * LDS_LD, 0);
        }
    }
}

// Ring-loop epilogue.  After the K loop the four ring slots are free; each holds
// one RG-row group of the tile as fp32 [RG][BN] (RG = 32 where a slot is large enough,
// else 16: half an accumulator tile), so a tile leaves in phases of four groups with two
// barriers per phase, and a thread's functor calls of a phase are independent (their
// global loads overlap).  Column c of staged row r sits at c ^ 32*((r>>2)&1): the two
// half-waves of an accumulator store (rows r and r+4) then hit disjoint banks, and
// 8-column chunks stay contiguous for the functors.
template <int BM, int BN, int WAVES_M, int WAVES_N, int RG, class Epi>
__device__ __forceinline__ void store_tile_ring(f32x16 (&acc)[BM / WAVES_M / 32][BN / WAVES_N / 32],
                                                float* s0, float* s1, float* s2, float* s3, int m0,
                                                int bn, int M, const Epi& epi) {
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int GPW = 4 / WAVES_M;      // staged groups per wave and phase
    constexpr int VPG = RG / 2;           // accumulator registers per group and tile
    constexpr int BPP = GPW * RG / 32;    // accumulator row blocks per wave and phase
    constexpr int PHASES = TM / BPP;
    constexpr int TPR = BN / 8;           // threads per staged row
    constexpr int RPP = NT / TPR;         // rows per pass
    static_assert(RG == 32 || RG == 16, "row group");
    static_assert(4 % WAVES_M == 0 && GPW * RG % 32 == 0 && TM % BPP == 0 && RG % RPP == 0, "epilogue shape");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WAVES_M, wn0 = (wave / WAVES_M) * WN;
    const int frow = lane & 31, fk = lane >> 5;
    auto stage = [&](int q) -> float* { return q == 0 ? s0 : q == 1 ? s1 : q == 2 ? s2 : s3; };
#pragma unroll
    for (int p = 0; p < PHASES; ++p) {
        if (p) __syncthreads();
        // register v of a 32x32 accumulator tile holds tile row 8*(v>>2) + 4*fk + (v&3): rows
        // 0..15 are registers 0..7, rows 16..31 registers 8..15; (row>>2)&1 == fk
#pragma unroll
        for (int g = 0; g < GPW; ++g) {
            const int i = p * BPP + g * RG / 32;  // accumulator row block
            const int sub = (g * RG % 32) / RG;   // which half of it (RG = 16)
            float* st = stage(wm * GPW + g);      // slot q holds wave-row q / GPW, group q % GPW
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int vv = 0; vv < VPG; ++vv) {
                    const int v = sub * VPG + vv;
                    const int r = 8 * (v >> 2) + 4 * fk + (v & 3) - sub * RG;
                    st[r * BN + ((wn0 + j * 32 + frow) ^ (fk << 5))] = acc[i][j][v];
                }
        }
        __syncthreads();
        const int cc = (tid % TPR) * 8;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row0 = (q / GPW) * WM + p * BPP * 32 + (q % GPW) * RG;   // tile row of the slot's first row
#pragma unroll
            for (int k = 0; k < RG / RPP; ++k) {
                const int r = tid / TPR + k * RPP;
                const int m = m0 + row0 + r;
                if (m < M) epi.template operator()<BN>(m, bn, cc, stage(q) + r * BN, ((r >> 2) & 1) << 5);
            }
        }
    }
}

// ---------------------------------------------------------------- staged loop
constexpr int BK = 64;
constexpr int CPR = BK / 8;   // 16-byte chunks per tile row

template <int BM, int BN, int WAVES_M, int WAVES_N, class BSrc, class Epi>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_nt_kernel(
    const bf16_t* __restrict__ A, int lda, int M, int K, int tiles_m, int tiles_n, int GM, BSrc bsrc,
    Epi epi) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int NT = NW * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_CH = BM * CPR / NT, B_CH = BN * CPR / NT;   // DMA instructions per wave and tile
    static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile/threads");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
    static_assert(32 * (BN + 4) * 4 <= (BM + BN) * BK * 2, "epilogue stage fits in one pipeline stage");

    // Two pipeline stages as separate arrays, so that a DMA into one stage is
    // known not to alias the fragment reads of the other.
    __shared__ __align__(16) bf16_t st0[(BM + BN) * BK];
    __shared__ __align__(16) bf16_t st1[(BM + BN) * BK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
    int bm, bn;
    tile_of_block(blockIdx.x, tiles_m, tiles_n, GM, &bm, &bn);
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
    store_tile<BM, BN, WAVES_M, WAVES_N, 32>(acc, reinterpret_cast<float*>(st0), m0, bn, M, epi);
}

// ------------------------------------------------------------------ ring loop
constexpr int BKS = 32;   // K columns per slice
constexpr int NS = 4;     // ring slots

template <int BM, int BN, int WAVES_M, int WAVES_N, class BSrc, class Epi>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_ring_kernel(
    const bf16_t* __restrict__ A, int lda, int M, int K, int tiles_m, int tiles_n, int GM, int nb, int vb0,
    BSrc bsrc, Epi epi) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    // DMA instructions per wave and slice.  Where the A_P 16-row pieces of A do not divide among
    // the waves, the first A_FULL waves own A_I pieces and the others A_I - 1; those repeat
    // their last piece so that every wave issues the same number of loads.
    constexpr int A_P = BM / 16;
    constexpr int A_I = (A_P + NW - 1) / NW, B_I = BN / 16 / NW;
    constexpr int A_FULL = A_P - NW * (A_I - 1);
    constexpr int DPS = A_I + B_I;
    constexpr int SL = NW * DPS * 16 * BKS;
    // rows of a staged fp32 group: 32 if that fits in one slot and a wave's row blocks pair up, else 16
    constexpr int RG = (32 * BN * 4 <= SL * 2 && TM % (4 / WAVES_M) == 0) ? 32 : 16;
    static_assert(BM % 16 == 0 && BN % (16 * NW) == 0 && BN % 32 == 0, "tile/waves");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
    static_assert(RG * BN * 4 <= SL * 2, "an fp32 row group fits in one slot");
    static_assert(DPS * (NS - 1) < 64, "vmcnt range");

    // One array per ring slot: the compiler then knows that a DMA into one slot
    // does not alias the fragment reads of another and adds no waits of its own.
    __shared__ __align__(16) bf16_t sl0[SL];
    __shared__ __align__(16) bf16_t sl1[SL];
    __shared__ __align__(16) bf16_t sl2[SL];
    __shared__ __align__(16) bf16_t sl3[SL];
    auto slot = [&](int i) -> bf16_t* { return i == 0 ? sl0 : i == 1 ? sl1 : i == 2 ? sl2 : sl3; };

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
    int bm, bn;
    const int vb = tile_of_block(blockIdx.x, nb, vb0, tiles_m, tiles_n, GM, &bm, &bn);   // this launch covers tiles vb0 .. vb0 + nb - 1
    const int m0 = bm * BM;

    // One DMA instruction moves 16 slice rows (16 x 64 B).  Lane L fills physical
    // chunk slot L%4 of row L/4 and fetches the logical chunk slot ^ ((row>>2)&3):
    // a 16-byte fragment read of 16 consecutive rows then touches every bank once.
    // Wave w loads its A pieces (16 rows each) and B rows w*16*B_I .. of the tile, and a slot
    // holds them wave by wave ([wave][A rows | B rows], DPS KB each): the DPS loads of a wave
    // and slice share one LDS base and differ in their immediate offset only.
    // Global addresses are a wave-uniform base (advanced along K in scalar
    // registers) plus a loop-invariant 32-bit lane offset.
    uint32_t ao[A_I], bo[B_I];
    const int a_rows = M - m0;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
    for (int i = 0; i < A_I; ++i) {
        const int piece = wave_u < A_FULL ? wave_u * A_I + i
                                          : A_FULL * A_I + (wave_u - A_FULL) * (A_I - 1) + (i < A_I - 1 ? i : A_I - 2);
        int r = piece * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        r = r < a_rows ? r : a_rows - 1;
        ao[i] = (uint32_t)((r * lda + c * 8) * 2);
    }
    // B rows: the rows of one wave lie in one half of the tile (BN/2 is a multiple of
    // 16*B_I); each half has its own base (the gate and the up matrix of a fused gate/up tile,
    // or simply row BN/2 of the same matrix).
    static_assert((BN / 2) % (16 * B_I) == 0, "a wave's B rows stay in one half");
    const bool hi_half = wave_u * B_I * 16 >= BN / 2;          // wave-uniform
#pragma unroll
    for (int i = 0; i < B_I; ++i) {
        int r = (wave_u * B_I + i) * 16 - (hi_half ? BN / 2 : 0) + (lane >> 2);   // row within the half
        const int c = (lane & 3) ^ ((r >> 2) & 3);             // same swizzle as for the tile row
        const int left = bsrc.template rows_left<BN>(bn, hi_half ? 1 : 0);
        r = r < left ? r : left - 1;
        bo[i] = (uint32_t)((r * bsrc.ldb + c * 8) * 2);
    }
    // K is this launch's share per workgroup row: row blockIdx.y starts blockIdx.y * K columns in
    const int64_t kz = (int64_t)blockIdx.y * K * 2;
    const char* abase = reinterpret_cast<const char*>(A + (int64_t)m0 * lda) + kz;
    const char* bbase = reinterpret_cast<const char*>(bsrc.template base<BN>(bn, hi_half ? 1 : 0)) + kz;
    const int wbase = wave_u * DPS * 16 * BKS;
    auto scalar_ptr = [](const char* p) -> const char* {   // keeps the base in scalar registers
        const uint64_t u = reinterpret_cast<uint64_t>(p);
        const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)u);
        const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(u >> 32));
        return reinterpret_cast<const char*>((hi << 32) | lo);
    };
    auto dma_slice = [&](bf16_t* s, int sidx) {
        const int64_t kb = (int64_t)sidx * (BKS * 2);
        unrolled<A_I>([&](auto i) {
            const char* ab = scalar_ptr(abase + kb - i.value * 1024);   // the immediate adds it back
            asm volatile("" : "+v"(ao[i.value]));   // keeps the offset a 32-bit register operand of the load
            dma16_at<i.value * 1024>(ab + ao[i.value], s + wbase);
        });
        unrolled<B_I>([&](auto i) {
            const char* bb = scalar_ptr(bbase + kb - (A_I + i.value) * 1024);
            asm volatile("" : "+v"(bo[i.value]));
            dma16_at<(A_I + i.value) * 1024>(bb + bo[i.value], s + wbase);
        });
    };
    // element offset in a slot of tile row r of A (is_b = 0) or B (is_b = 1)
    auto row_at = [](int r, int is_b) {
        constexpr int per_b = 16 * B_I;
        if (is_b) return ((r / per_b) * DPS * 16 + A_I * 16 + r % per_b) * BKS;
        const int piece = r / 16;
        int w, i;
        if (A_FULL == NW || piece < A_FULL * A_I) {
            w = piece / A_I, i = piece % A_I;
        } else {
            const int q = piece - A_FULL * A_I;
            w = A_FULL + q / (A_I > 1 ? A_I - 1 : 1), i = q % (A_I > 1 ? A_I - 1 : 1);
        }
        return (w * DPS * 16 + i * 16 + r % 16) * BKS;
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int frow = lane & 31, fk = lane >> 5;
    const int fsw = (frow >> 2) & 3;      // rows of a fragment differ by multiples of 32
    bf16x8 af[2][TM], bfr[2][TN];
    auto load_frags = [&](const bf16_t* s, int ks, int fb) {
        const int sl = ((ks * 2 + fk) ^ fsw) << 3;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[fb][i] = *reinterpret_cast<const bf16x8*>(s + row_at(wm0 + i * 32 + frow, 0) + sl);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            bfr[fb][j] = *reinterpret_cast<const bf16x8*>(s + row_at(wn0 + j * 32 + frow, 1) + sl);
    };
    auto mfmas = [&](int fb) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[fb][i], bfr[fb][j], acc[i][j], 0, 0, 0);
    };
    constexpr int NF = TM + TN, NM = TM * TN;
    auto pin_interleave = [&]() {   // issue order: every MFMA followed by one fragment read
#pragma unroll
        for (int mm = 0; mm < NM; ++mm) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (mm < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };

    // The two 16-column k-steps of a slice alternate between two fragment
    // register sets, and the stream of k-steps runs on across slice boundaries:
    // the MFMAs of a slice's second k-step are issued after the barrier that opens
    // the next slice, so they cover the latency of its first fragment reads.
    // At a boundary a wave waits until its own loads of the next slice have landed
    // (vmcnt: only the younger slices may be outstanding) and its fragment reads
    // of the current slice have returned; after the barrier the slot just read is
    // free everywhere and is refilled with the slice NS ahead.
    const int KS = K / BKS;            // K % (BKS * NS) == 0, KS >= NS
#pragma unroll
    for (int j = 0; j < NS; ++j) dma_slice(slot(j), j);
    wait_vm_lds0<DPS * (NS - 1)>();
    wg_barrier();
    load_frags(slot(0), 0, 0);
    int s0 = 0;
    for (; s0 + 2 * NS <= KS; s0 += NS) {
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            load_frags(slot(j), 1, 1);
            mfmas(0);
            pin_interleave();
            wait_vm_lds0<DPS * (NS - 2)>();
            wg_barrier();
            dma_slice(slot(j), s0 + j + NS);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(slot((j + 1) % NS), 0, 0);
            mfmas(1);
            pin_interleave();
        }
    }
    // the last NS slices are in flight or landed: no refills
#pragma unroll
    for (int j = 0; j < NS; ++j) {
        load_frags(slot(j), 1, 1);
        mfmas(0);
        pin_interleave();
        if (j + 1 < NS) {
            if (j == 0) wait_vm_lds0<DPS * (NS - 2)>();
            else if (j == 1) wait_vm_lds0<DPS * (NS - 3)>();
            else wait_vm_lds0<0>();
            wg_barrier();
            __builtin_amdgcn_sched_barrier(0);
            load_frags(slot(j + 1), 0, 0);
            mfmas(1);
            pin_interleave();
        } else {
            mfmas(1);
        }
    }
    __syncthreads();   // every wave has finished reading the ring
    store_tile_ring<BM, BN, WAVES_M, WAVES_N, RG>(acc, reinterpret_cast<float*>(sl0), reinterpret_cast<float*>(sl1),
                                              reinterpret_cast<float*>(sl2), reinterpret_cast<float*>(sl3),
                                              m0, bn, M, epi_for_tile(epi, vb - vb0, m0));
}

// The same ring with 16x16x32 MFMAs and hand-written fragment reads (the 256-wide tiles).
template <int BM, int BN, int WAVES_M, int WAVES_N, class BSrc, class Epi>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_ring16_kernel(
    const bf16_t* __restrict__ A, int lda, int M, int K, int tiles_m, int tiles_n, int GM, int nb, int vb0,
    BSrc bsrc, Epi epi) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32;
    constexpr int UM = WM / 16, UN = WN / 16;       // 16x16 accumulator tiles per wave
    // DMA instructions per wave and slice.  Where the A_P 16-row pieces of A do not divide among
    // the waves, the first A_FULL waves own A_I pieces and the others A_I - 1; those repeat
    // their last piece so that every wave issues the same number of loads.
    constexpr int A_P = BM / 16;
    constexpr int A_I = (A_P + NW - 1) / NW, B_I = BN / 16 / NW;
    constexpr int A_FULL = A_P - NW * (A_I - 1);
    constexpr int DPS = A_I + B_I;
    constexpr int SL = NW * DPS * 16 * BKS;
    // rows of a staged fp32 group: 32 if that fits in one slot and a wave's row blocks pair up, else 16
    constexpr int RG = (32 * BN * 4 <= SL * 2 && TM % (4 / WAVES_M) == 0) ? 32 : 16;
    static_assert(BM % 16 == 0 && BN % (16 * NW) == 0 && BN % 32 == 0, "tile/waves");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
    static_assert(RG * BN * 4 <= SL * 2, "an fp32 row group fits in one slot");
    static_assert(DPS * (NS - 1) < 64, "vmcnt range");

    // One array: the fragment reads of this loop are written by hand, so the compiler has no
    // LDS reads to order against the global -> LDS loads.
    __shared__ __align__(16) bf16_t ring[NS * SL];
    auto slot = [&](int i) -> bf16_t* { return ring + i * SL; };

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
    int bm, bn;
    const int vb = tile_of_block(blockIdx.x, nb, vb0, tiles_m, tiles_n, GM, &bm, &bn);   // this launch covers tiles vb0 .. vb0 + nb - 1
    const int m0 = bm * BM;

    // One DMA instruction moves 16 slice rows (16 x 64 B).  Lane L fills physical
    // chunk slot L%4 of row L/4 and fetches the logical chunk slot ^ ((row>>1)&3).  The
    // fragment read of this loop (lane = row L%16, chunk L/16 of 16 consecutive rows) runs at
    // the full LDS rate with this swizzle and at half of it with slot ^ ((row>>2)&3), with
    // slot ^ (row&3) or without one (measured with a read-only kernel on this part; the
    // bank-conflict counter of the loop agrees: half of the active LDS cycles before).
    // Wave w loads its A pieces (16 rows each) and B rows w*16*B_I .. of the tile, and a slot
    // holds them wave by wave ([wave][A rows | B rows], DPS KB each): the DPS loads of a wave
    // and slice share one LDS base and differ in their immediate offset only.
    // Global addresses are a wave-uniform base (advanced along K in scalar
    // registers) plus a loop-invariant 32-bit lane offset.
    uint32_t ao[A_I], bo[B_I];
    const int a_rows = M - m0;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
    for (int i = 0; i < A_I; ++i) {
        const int piece = wave_u < A_FULL ? wave_u * A_I + i
                                          : A_FULL * A_I + (wave_u - A_FULL) * (A_I - 1) + (i < A_I - 1 ? i : A_I - 2);
        int r = piece * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 1) & 3);
        r = r < a_rows ? r : a_rows - 1;
        ao[i] = (uint32_t)((r * lda + c * 8) * 2);
    }
    // B rows: the rows of one wave lie in one half of the tile (BN/2 is a multiple of
    // 16*B_I); each half has its own base (the gate and the up matrix of a fused gate/up tile,
    // or simply row BN/2 of the same matrix).
    static_assert((BN / 2) % (16 * B_I) == 0, "a wave's B rows stay in one half");
    const bool hi_half = wave_u * B_I * 16 >= BN / 2;          // wave-uniform
#pragma unroll
    for (int i = 0; i < B_I; ++i) {
        int r = (wave_u * B_I + i) * 16 - (hi_half ? BN / 2 : 0) + (lane >> 2);   // row within the half
        const int c = (lane & 3) ^ ((r >> 1) & 3);             // same swizzle as for the tile row
        const int left = bsrc.template rows_left<BN>(bn, hi_half ? 1 : 0);
        r = r < left ? r : left - 1;
        bo[i] = (uint32_t)((r * bsrc.ldb + c * 8) * 2);
    }
    // K is this launch's share per workgroup row: row blockIdx.y starts blockIdx.y * K columns in
    const int64_t kz = (int64_t)blockIdx.y * K * 2;
    const char* abase = reinterpret_cast<const char*>(A + (int64_t)m0 * lda) + kz;
    const char* bbase = reinterpret_cast<const char*>(bsrc.template base<BN>(bn, hi_half ? 1 : 0)) + kz;
    const int wbase = wave_u * DPS * 16 * BKS;
    auto scalar_ptr = [](const char* p) -> const char* {   // keeps the base in scalar registers
        const uint64_t u = reinterpret_cast<uint64_t>(p);
        const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)u);
        const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(u >> 32));
        return reinterpret_cast<const char*>((hi << 32) | lo);
    };
    auto dma_one = [&](bf16_t* s, int sidx, auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        const int64_t kb = (int64_t)sidx * (BKS * 2);
        if constexpr (i < A_I) {
            const char* ab = scalar_ptr(abase + kb - i * 1024);   // the immediate adds it back
            asm volatile("" : "+v"(ao[i]));   // keeps the offset a 32-bit register operand of the load
            dma16_at<i * 1024>(ab + ao[i], s + wbase);
        } else {
            const char* bb = scalar_ptr(bbase + kb - i * 1024);
            asm volatile("" : "+v"(bo[i - A_I]));
            dma16_at<i * 1024>(bb + bo[i - A_I], s + wbase);
        }
    };
    auto dma_slice = [&](bf16_t* s, int sidx) __attribute__((always_inline)) {
        unrolled<DPS>([&](auto i) __attribute__((always_inline)) { dma_one(s, sidx, i); });
    };
    // element offset in a slot of tile row r of A (is_b = 0) or B (is_b = 1)
    auto row_at = [](int r, int is_b) {
        constexpr int per_b = 16 * B_I;
        if (is_b) return ((r / per_b) * DPS * 16 + A_I * 16 + r % per_b) * BKS;
        const int piece = r / 16;
        int w, i;
        if (A_FULL == NW || piece < A_FULL * A_I) {
            w = piece / A_I, i = piece % A_I;
        } else {
            const int q = piece - A_FULL * A_I;
            w = A_FULL + q / (A_I > 1 ? A_I - 1 : 1), i = q % (A_I > 1 ? A_I - 1 : 1);
        }
        return (w * DPS * 16 + i * 16 + r % 16) * BKS;
    };

    // ---- 16x16x32 MFMAs: one k-step per slice.  Lane L holds row (column) L%16 and the eight k
    //      values of 16-byte chunk L/16 of the slice row; an accumulator tile is f32x4 with
    //      row 4*(L/16) + v, column L%16 ----
    static_assert(UM % 2 == 0 && UM >= 4 && UN >= 2, "fragment ring");
    static_assert((A_FULL != NW || WM % (16 * A_I) == 0) && WN % (16 * B_I) == 0, "fragment offsets are lane-independent");
    static_assert(DPS <= 2 * UN, "one load per MFMA of a block's first part at most");
    f32x4 acc[UM][UN];
#pragma unroll
    for (int i = 0; i < UM; ++i)
#pragma unroll
        for (int j = 0; j < UN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int frow = lane & 15, fk = lane >> 4;
    const int fsw = (lane >> 1) & 3;
    const int sl = (fk ^ fsw) << 3;
    // A fragments cycle through four registers (two rows ahead of the MFMAs), B fragments of a
    // slice stay for the slice and alternate between two sets from slice to slice
    bf16x8 ar[4], bq[2][UN];
    // byte offset of fragment i (16 rows) from the lane's address of fragment 0
    constexpr auto delta = [](int i, int per, int dps) { return 2 * BKS * (((16 * i) / per) * dps * 16 + (16 * i) % per); };
    const uint32_t ring_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)ring;
    const uint32_t a_lane = ring_base + 2 * (row_at(wm0 + frow, 0) + sl), b_lane = ring_base + 2 * (row_at(wn0 + frow, 1) + sl);
    // slots 0, 1 and 2, 3 share an address register each: the offset field of an LDS read is 16 bits
    static_assert(NS == 4, "slot pairs");
    const uint32_t a_addr[2] = {a_lane, a_lane + 2 * 2 * SL}, b_addr[2] = {b_lane, b_lane + 2 * 2 * SL};
    // Where the pieces of A are not spread evenly (192-row tile) the fragments of a wave are not
    // at the same distances for both wave rows: one address register per fragment and slot pair.
    constexpr bool A_EVEN = A_FULL == NW;
    uint32_t a_fr[A_EVEN ? 1 : UM][2];
    if constexpr (!A_EVEN) {
#pragma unroll
        for (int i = 0; i < UM; ++i) {
            a_fr[i][0] = ring_base + 2 * (row_at(wm0 + i * 16 + frow, 0) + sl);
            a_fr[i][1] = a_fr[i][0] + 2 * 2 * SL;
        }
    }
    auto read_a = [&](auto jc, auto ic) __attribute__((always_inline)) -> bf16x8 {
        constexpr int j = decltype(jc)::value, i = decltype(ic)::value;
        bf16x8 v;
        if constexpr (A_EVEN) {
            constexpr int off = (j & 1) * 2 * SL + delta(i, 16 * A_I, DPS);
            static_assert(off < 65536, "ds offset field");
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(a_addr[j >> 1]), "n"(off));
        } else {
            constexpr int off = (j & 1) * 2 * SL;
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(a_fr[i][j >> 1]), "n"(off));
        }
        return v;
    };
    auto read_b = [&](auto jc, auto ic) __attribute__((always_inline)) -> bf16x8 {
        constexpr int j = decltype(jc)::value, i = decltype(ic)::value;
        constexpr int off = (j & 1) * 2 * SL + delta(i, 16 * B_I, DPS);
        static_assert(off < 65536, "ds offset field");
        bf16x8 v;
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(b_addr[j >> 1]), "n"(off));
        return v;
    };
    // One slice (slot j), straight-line code: [the last two fragment rows of the previous slice,
    // between their MFMAs the first reads of this slice and the refill of the slot freed at the
    // previous barrier], rows 0 .. UM-3 (the A fragment two rows ahead is requested before each
    // row's MFMAs), wait, barrier.  The compiler does not know that a hand-written read fills
    // its registers later: every read is issued and waited for inside this block, and none is
    // in flight at its end.  Reads return in issue order (A0 B0 .. B(UN-1) A1 A2 ...): when a
    // row's MFMAs need their operands, exactly two younger reads may still be out.
    auto block = [&](auto jc, auto firstc, auto dmac, auto vmc, int sidx) __attribute__((always_inline)) {
        constexpr int j = decltype(jc)::value, bb = j & 1;
        constexpr bool first = decltype(firstc)::value, with_dma = decltype(dmac)::value;
        constexpr int VM = decltype(vmc)::value;
        // A fragment i of this slice lives in ar[(i + RO) % 4]; with UM % 4 == 2 the slices of odd
        // slots start two registers on, so that the previous slice's last two stay clear of the
        // first two of this one
        constexpr int RO = (UM % 4) * (j & 1) % 4, RP = (UM % 4) * ((j + NS - 1) & 1) % 4;
        unrolled<2 * UN>([&](auto mc) __attribute__((always_inline)) {
            constexpr int m = decltype(mc)::value, i = UM - 2 + m / UN, n = m % UN;
            if constexpr (!first) acc[i][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ar[(i + RP) % 4], bq[bb ^ 1][n], acc[i][n], 0, 0, 0);
            if constexpr (m == 0) ar[RO % 4] = read_a(jc, std::integral_constant<int, 0>{});
            else if constexpr (m <= UN) bq[bb][m - 1] = read_b(jc, std::integral_constant<int, m - 1>{});
            else if constexpr (m == UN + 1) ar[(1 + RO) % 4] = read_a(jc, std::integral_constant<int, 1>{});
            if constexpr (with_dma && m < DPS) dma_one(slot((j + NS - 1) % NS), sidx, mc);
            if constexpr (!first) __builtin_amdgcn_sched_barrier(0);
        });
        unrolled<UM - 2>([&](auto ic) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            ar[(i + 2 + RO) % 4] = read_a(jc, std::integral_constant<int, i + 2>{});
            asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(ar[(i + RO) % 4]));
            if constexpr (i == 0) {
#pragma unroll
                for (int n = 0; n < UN; ++n) asm volatile("" : "+v"(bq[bb][n]));
            }
            unrolled<UN>([&](auto nc) __attribute__((always_inline)) {
                constexpr int n = decltype(nc)::value;
                acc[i][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ar[(i + RO) % 4], bq[bb][n], acc[i][n], 0, 0, 0);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        // this wave's loads of the next slice have landed (at most VM younger ones may be out) and
        // its last two A fragments have arrived; after the barrier slot j is free everywhere
        asm volatile("s_waitcnt vmcnt(%2) lgkmcnt(0)" : "+v"(ar[(UM - 2 + RO) % 4]), "+v"(ar[(UM - 1 + RO) % 4]) : "n"(VM));
        wg_barrier();
    };
    using T = std::true_type;
    using F = std::false_type;
#define CC_IC(x) std::integral_constant<int, (x)>{}
    const int KS = K / BKS;            // K % (BKS * NS) == 0, KS >= NS
#pragma unroll
    for (int j = 0; j < NS; ++j) dma_slice(slot(j), j);
    wait_vm_lds0<DPS * (NS - 1)>();
    wg_barrier();
    constexpr int VS = DPS * (NS - 2);
    block(CC_IC(0), T{}, F{}, CC_IC(VS), 0);
    int t = 1;
    for (; t + 3 + NS <= KS; t += NS) {      // slices t .. t+3 in slots 1, 2, 3, 0; each refills the slot before its own
        block(CC_IC(1), F{}, T{}, CC_IC(VS), t - 1 + NS);
        block(CC_IC(2), F{}, T{}, CC_IC(VS), t + NS);
        block(CC_IC(3), F{}, T{}, CC_IC(VS), t + 1 + NS);
        block(CC_IC(0), F{}, T{}, CC_IC(VS), t + 2 + NS);
    }
    // t == KS - NS + 1: the last three slices, every load has been issued
    block(CC_IC(1), F{}, F{}, CC_IC(DPS), 0);
    block(CC_IC(2), F{}, F{}, CC_IC(0), 0);
    block(CC_IC(3), F{}, F{}, CC_IC(0), 0);
#undef CC_IC
    // rows UM-2, UM-1 of the last slice (slot NS-1)
    unrolled<2 * UN>([&](auto mc) __attribute__((always_inline)) {
        constexpr int m = decltype(mc)::value, i = UM - 2 + m / UN, n = m % UN;
        constexpr int RL = (UM % 4) * ((NS - 1) & 1) % 4;
        acc[i][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ar[(i + RL) % 4], bq[1][n], acc[i][n], 0, 0, 0);
    });
    __syncthreads();   // every wave has finished reading the ring

    // ---- epilogue: the four slots take one RG-row group each as fp32 [RG][BN] (RG = 32: two
    //      accumulator tiles, where a slot is large enough and a wave's 32-row blocks pair up; else
    //      16: one), a wave's rows leave in phases of 4 / WAVES_M groups.  Column c of staged row r
    //      sits at c ^ 16*((r>>2)&3): the four 16-lane groups of an accumulator store (rows 4 apart)
    //      hit disjoint banks, and 8-column chunks stay contiguous for the functors ----
    {
        constexpr int NT = NW * 64;
        constexpr int GPW = 4 / WAVES_M;          // staged groups per wave and phase
        constexpr int RGS = (32 * BN * 4 <= SL * 2 && TM % GPW == 0) ? 32 : 16;
        constexpr int TPG = RGS / 16;             // accumulator tiles per group
        constexpr int PHASES = UM / (GPW * TPG);
        constexpr int TPR = BN / 8, RPP = NT / TPR;
        static_assert(RGS * BN * 4 <= SL * 2 && 4 % WAVES_M == 0 && UM % (GPW * TPG) == 0 && RGS % RPP == 0, "epilogue shape");
        const int wm = wave % WAVES_M;
        auto stage = [&](int q) -> float* { return reinterpret_cast<float*>(ring + q * SL); };
        const auto e2 = epi_for_tile(epi, vb - vb0, m0);
#pragma unroll
        for (int p = 0; p < PHASES; ++p) {
            if (p) __syncthreads();
#pragma unroll
            for (int g = 0; g < GPW; ++g) {
                float* st = stage(wm * GPW + g);      // slot q holds wave-row q / GPW, group q % GPW
#pragma unroll
                for (int hh = 0; hh < TPG; ++hh) {    // the 16-row accumulator tiles of the group
                    const int i = (p * GPW + g) * TPG + hh;
#pragma unroll
                    for (int jj = 0; jj < UN; ++jj)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int r = 16 * hh + 4 * fk + v;
                            st[r * BN + ((wn0 + jj * 16 + frow) ^ (fk << 4))] = acc[i][jj][v];
                        }
                }
            }
            __syncthreads();
            const int cc = (tid % TPR) * 8;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row0 = (q / GPW) * WM + (p * GPW + q % GPW) * RGS;   // tile row of the slot's first row
#pragma unroll
                for (int k = 0; k < RGS / RPP; ++k) {
                    const int r = tid / TPR + k * RPP;
                    const int m = m0 + row0 + r;
                    if (m < M) e2.template operator()<BN>(m, bn, cc, stage(q) + r * BN, ((r >> 2) & 3) << 4);
                }
            }
        }
    }
}

// Tile shapes: 256x256 (8 waves of 128x64, least LDS and L2 traffic per flop, one
// workgroup per CU), 192x256 (8 waves of 96x64, ring loop only, measured at 0.8 of the
// large tile's rate: it pays where it saves a half-empty round), 256x128 (8 waves of 64x64, one
// per CU, ring loop only) and 128x128 (4 waves of 64x64, two per CU, measured at 0.55 to 0.85 of
// the large tile's rate depending on K).  Every shape runs the 16x16x32 ring loop when K allows
// it, the 256x256 and 128x128 shapes the staged loop otherwise.  A grid runs as a whole number
// of "rounds" of workgroups, so the shape is chosen per launch to minimise rounds x tile
// cost.
template <class BSrc, class Epi>
void launch_gemm(const bf16_t* A, int lda, int M, int N_tiles_cols, int K, int ldb, int gm_big,
                 BSrc bsrc, Epi epi, float* ws, int64_t ws_floats, const cc_launch_override& ovr,
                 hipStream_t s) {
    static const int n_cu = [] {
        int dev = 0, n = 256;
        if (hipGetDevice(&dev) == hipSuccess)
            (void)hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        return n > 0 ? n : 256;
    }();
    // Test overrides (cc_debug_set_launch): tile shape, staged K loop, the 32x32x16 ring loop,
    // band height of the tile order, number of K shares (1 = none).
    const char force = (char)ovr.gemm_tile;                   // 0: the launcher's choice
    const bool mfma16 = !ovr.gemm_mfma32;
    auto rounds_of = [&](int bm, int bn, int per_cu, int shares) {
        const long tiles = (long)((M + bm - 1) / bm) * ((N_tiles_cols + bn - 1) / bn) * shares;
        const long slots = (long)n_cu * per_cu;
        return (tiles + slots - 1) / slots;
    };
    auto cost = [&](int bm, int bn, int per_cu, double eff) {
        return (double)rounds_of(bm, bn, per_cu, 1) * per_cu * bm * bn / eff;
    };
    // ring loop: whole groups of NS slices, 32-bit lane offsets within a tile's rows
    bool ring = K % (BKS * NS) == 0 && (int64_t)lda * 256 * 2 < (1ll << 31) &&
                (int64_t)ldb * 256 * 2 < (1ll << 31);
    if (ovr.gemm_staged) ring = false;
    const double cb = cost(256, 256, 1, 1.00), cm = cost(192, 256, 1, 0.80), ch = cost(256, 128, 1, 0.70),
                 cs = cost(128, 128, 2, 0.67);
    char pick = cb <= cs ? 'b' : 's';
    double best = cb <= cs ? cb : cs;
    if (ring && ch < best) pick = 'h', best = ch;               // these two have no staged variant
    if (ring && cm < best) pick = 'm', best = cm;
    if (force == 'b' || force == 's' || ((force == 'h' || force == 'm') && ring)) pick = force;
    // Split-K for the part of a grid that leaves most CUs idle: the tiles of a last round that
    // fills at most half the chip (all tiles, if there is no full round) are computed by S
    // workgroup rows, each over K/S columns, with S x tiles <= CUs, and a finishing pass; the full
    // rounds before them run as a launch of their own.  256-wide tiles only.  Times in
    // microseconds: 0.75 per 32-column slice of a 256x256 tile, 6 per round for the ends of a tile,
    // the finishing pass at 4 TB/s plus 10 for the two extra launches (measured: QKV at M = 3928,
    // 384 tiles, takes 208 split against 199 with the 192-row tile, so the estimate has to be
    // 10 % below the unsplit one to be taken).
    int S = 1;
    if (ring && ws) {
        const double slice_us = 0.75 * K / BKS / 65536.0;       // per unit of tile area
        auto rem_of = [&](int bm) {
            const long tiles = (long)((M + bm - 1) / bm) * ((N_tiles_cols + 255) / 256);
            return (int)(tiles % n_cu == 0 && tiles > 0 ? n_cu : tiles % n_cu);
        };
        auto split_ok = [&](int bm, int sp, int k_min) {
            const int rem = rem_of(bm);
            return (K / (BKS * NS)) % sp == 0 && K / sp >= k_min && (long)rem * sp <= n_cu &&
                   (double)sp * rem * 65536.0 <= (double)ws_floats;
        };
        if (ovr.gemm_splitk > 0) {
            const int sp = ovr.gemm_splitk;
            const int bm = pick == 'm' ? 192 : 256;
            if (sp > 1 && sp <= 16 && split_ok(bm, sp, BKS * NS)) S = sp, pick = bm == 192 ? 'm' : 'b';
        } else if (!force && !ovr.gemm_staged) {
            double t_best = best * slice_us + 6.0 * rounds_of(pick == 's' ? 128 : pick == 'm' ? 192 : 256,
                                                               (pick == 'b' || pick == 'm') ? 256 : 128,
                                                               pick == 's' ? 2 : 1, 1);
            const double t_unsplit = t_best;
            for (int bm = 256; bm >= 192; bm -= 64) {
                const double tile_us = bm * 256.0 / (bm == 256 ? 1.0 : 0.80) * slice_us;
                const long full_rounds = rounds_of(bm, 256, 1, 1) - 1;
                const int rem = rem_of(bm);
                for (int sp = 2; sp <= 16; ++sp) {
                    if (!split_ok(bm, sp, 512)) continue;
                    const double t = full_rounds * (tile_us + 6.0) + tile_us / sp + 6.0 + 10.0 +
                                     (double)sp * rem * 65536.0 * 4 / 4.0e6;
                    if (t < t_best && t < 0.9 * t_unsplit) t_best = t, S = sp, pick = bm == 256 ? 'b' : 'm';
                }
            }
        }
    }
    const int bm = pick == 's' ? 128 : pick == 'm' ? 192 : 256, bn = (pick == 'b' || pick == 'm') ? 256 : 128;
    const int tiles_m = (M + bm - 1) / bm, tiles_n = (N_tiles_cols + bn - 1) / bn;
    int GM = pick == 's' ? 2 * gm_big : gm_big;
    if (ovr.gemm_gm > 0) GM = ovr.gemm_gm;
    GM = GM < 1 ? 1 : (GM > tiles_m ? tiles_m : GM);
    const int n_tiles = tiles_m * tiles_n;
#define CC_LAUNCH(KERN, BM_, BN_, WM_, WN_, EPI_T, EPI_V, K_, NB_, VB0_, GY_)                              \
    hipLaunchKernelGGL((KERN<BM_, BN_, WM_, WN_, BSrc, EPI_T>), dim3(NB_, GY_), dim3(WM_ * WN_ * 64), 0, s, A, \
                       lda, M, K_, tiles_m, tiles_n, GM, NB_, VB0_, bsrc, EPI_V)
#define CC_LAUNCH_NT(BM_, BN_, WM_, WN_)                                                                    \
    hipLaunchKernelGGL((gemm_nt_kernel<BM_, BN_, WM_, WN_, BSrc, Epi>), dim3(n_tiles), dim3(WM_ * WN_ * 64), 0, \
                       s, A, lda, M, K, tiles_m, tiles_n, GM, bsrc, epi)
    if (S > 1) {
        const int rem = n_tiles % n_cu == 0 ? n_cu : n_tiles % n_cu, full = n_tiles - rem;
        EpiPartial pe{ws, (int64_t)rem * 65536, 0, 0};
        if (pick == 'b' && mfma16) {
            if (full) CC_LAUNCH(gemm_ring16_kernel, 256, 256, 2, 4, Epi, epi, K, full, 0, 1);
            CC_LAUNCH(gemm_ring16_kernel, 256, 256, 2, 4, EpiPartial, pe, K / S, rem, full, S);
        } else if (pick == 'b') {
            if (full) CC_LAUNCH(gemm_ring_kernel, 256, 256, 2, 4, Epi, epi, K, full, 0, 1);
            CC_LAUNCH(gemm_ring_kernel, 256, 256, 2, 4, EpiPartial, pe, K / S, rem, full, S);
        } else if (mfma16) {
            if (full) CC_LAUNCH(gemm_ring16_kernel, 192, 256, 2, 4, Epi, epi, K, full, 0, 1);
            CC_LAUNCH(gemm_ring16_kernel, 192, 256, 2, 4, EpiPartial, pe, K / S, rem, full, S);
        } else {
            if (full) CC_LAUNCH(gemm_ring_kernel, 192, 256, 2, 4, Epi, epi, K, full, 0, 1);
            CC_LAUNCH(gemm_ring_kernel, 192, 256, 2, 4, EpiPartial, pe, K / S, rem, full, S);
        }
        hipLaunchKernelGGL((splitk_finish_kernel<Epi>), dim3(rem, (bm + 7) / 8), dim3(256), 0, s, ws,
                           (int64_t)rem * 65536, S, M, bm, full, tiles_m, tiles_n, GM, epi);
    } else if (pick == 'b') {
        if (ring && mfma16) CC_LAUNCH(gemm_ring16_kernel, 256, 256, 2, 4, Epi, epi, K, n_tiles, 0, 1);
        else if (ring) CC_LAUNCH(gemm_ring_kernel, 256, 256, 2, 4, Epi, epi, K, n_tiles, 0, 1);
        else CC_LAUNCH_NT(256, 256, 2, 4);
    } else if (pick == 'm') {
        if (mfma16) CC_LAUNCH(gemm_ring16_kernel, 192, 256, 2, 4, Epi, epi, K, n_tiles, 0, 1);
        else CC_LAUNCH(gemm_ring_kernel, 192, 256, 2, 4, Epi, epi, K, n_tiles, 0, 1);
    } else if (pick == 'h') {
        if (mfma16) CC_LAUNCH(gemm_ring16_kernel, 256, 128, 4, 2, Epi, epi, K, n_tiles, 0, 1);
        else CC_LAUNCH(gemm_ring_kernel, 256, 128, 4, 2, Epi, epi, K, n_tiles, 0, 1);
    } else {
        if (ring && mfma16) CC_LAUNCH(gemm_ring16_kernel, 128, 128, 2, 2, Epi, epi, K, n_tiles, 0, 1);
        else if (ring) CC_LAUNCH(gemm_ring_kernel, 128, 128, 2, 2, Epi, epi, K, n_tiles, 0, 1);
        else CC_LAUNCH_NT(128, 128, 2, 2);
    }
#undef CC_LAUNCH
#undef CC_LAUNCH_NT
}

}  // namespace

void cc_launch_qkv(const bf16_t* xn, int M, const int32_t* idx, const bf16_t* w_qkv,
                   const bf16_t* b_qkv, const cc_model_desc& m, const float2* rope,
                   const cc_kv_layer& kv, bf16_t* q_out, float* ws, int64_t ws_floats,
                   const cc_launch_override& ovr, hipStream_t s) {
    if (M <= 0) return;
    const int N = (m.H_q + 2 * m.H_kv) * m.d_h;
    BSingle b{w_qkv, m.d, N};
    EpiQKV e{idx, b_qkv, rope, m.H_q, m.H_kv, m.d_h, N, q_out,
             (bf16_t*)kv.K, (bf16_t*)kv.V, kv.stride_token, kv.stride_head};
    launch_gemm(xn, m.d, M, N, m.d, m.d, 4, b, e, ws, ws_floats, ovr, s);
}

void cc_launch_oproj(const bf16_t* o, int M, const bf16_t* w_o, const bf16_t* hidden,
                     const int32_t* gather_idx, const cc_model_desc& m, float* y, float* ws,
                     int64_t ws_floats, const cc_launch_override& ovr, hipStream_t s) {
    if (M <= 0) return;
    const int K = m.H_q * m.d_h;
    BSingle b{w_o, K, m.d};
    EpiOProj e{hidden, gather_idx, m.d, y};
    launch_gemm(o, K, M, m.d, K, K, 4, b, e, ws, ws_floats, ovr, s);
}

void cc_launch_gate_up(const bf16_t* mn, int M, const bf16_t* w_gate, const bf16_t* w_up,
                       const cc_model_desc& m, bf16_t* act, float* ws, int64_t ws_floats,
                       const cc_launch_override& ovr, hipStream_t s) {
    if (M <= 0) return;
    BDual b{w_gate, w_up, m.d, m.f};
    EpiGateUp e{m.f, act};
    // each 128-column tile holds 64 gate + 64 up columns: 2*f tile columns in total
    launch_gemm(mn, m.d, M, 2 * m.f, m.d, m.d, 4, b, e, ws, ws_floats, ovr, s);
}

void cc_launch_down(const bf16_t* act, int M, const bf16_t* w_down, const float* y,
                    const cc_model_desc& m, bf16_t* out, float* ws, int64_t ws_floats,
                    const cc_launch_override& ovr, hipStream_t s) {
    if (M <= 0) return;
    BSingle b{w_down, m.f, m.d};
    EpiDown e{y, m.d, out};
    launch_gemm(act, m.f, M, m.d, m.f, m.f, 8, b, e, ws, ws_floats, ovr, s);
}
