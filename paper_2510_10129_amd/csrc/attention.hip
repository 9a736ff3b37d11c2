// Sparse-query causal GQA attention over the updated KV cache: recomputed row i
// (global position idx[i]) attends to every cache slot j <= idx[i].  This is
// the kernel Section 5.6 of the paper describes as flash attention with sparse
// query indices; the design below is for gfx950.
//
// Work split: the (recomputed token, query head of the group) pairs of one kv
// head form one flat column sequence c = i*g + h (g = H_q/H_kv); a workgroup of
// eight waves owns 256 consecutive columns, a wave 32 of them on the N side of
// the MFMA tile, so a K/V tile read from LDS serves the whole query group and
// no column is padding when g does not divide 32.
//
// Each wave computes S^T = K Q^T (keys on the MFMA row side, query rows on the
// column side).  In the 32x32 accumulator layout a lane then owns ONE query row
// and 16 keys per tile, so the online-softmax maximum and sum are in-lane
// reductions plus one exchange with lane^32, the rescale factor is a per-lane
// scalar, and the probabilities are already laid out as the B operand of
// O^T = V^T P^T: no shuffle between the two contractions.
//
// Two wave groups alternate between the matrix pipe and the vector ALU.  Per
// 64-key tile a wave issues 32 MFMAs and about as many cycles of exponentials,
// sums and conversions, one after the other; two independent waves on a SIMD
// drift into the same phase (both contend for the matrix pipe, then both for
// the vector ALU) and each pipe idles half of the time.  Here the two waves of a
// SIMD belong to the same workgroup, one to group A and one to group B, and
// the workgroup barrier separates phases: while A runs the softmax of tile t, B
// runs P V of tile t-1 and Q K^T of tile t, and the other way round in the next
// phase.  A wave issues its global -> LDS loads at the end of its matrix phase
// (group A the V tiles, group B the K tiles), while its SIMD partner is in the
// vector part of its softmax: next to a partner that keeps the matrix pipe busy
// such a load holds the issuing wave several times as long.
//
// K and V tiles (64 keys) go from the cache straight into LDS with 16-byte
// global->LDS loads, row-major as they are stored, three stages each.  K
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
#include <type_traits>

namespace {

constexpr int BN_KEYS = 64;

// 16 bytes per lane from global memory straight into LDS.  The LDS address is
// wave base (M0) + OFF + 16 * lane and OFF is also added to the global address.
// Rewriting M0 between loads is expensive while MFMAs are in flight (measured:
// several hundred cycles per rewrite with two MFMA-bound waves on a SIMD), so
// the loads of one tile and tensor share one base and differ in OFF only.
template <int OFF>
__device__ __forceinline__ void dma16(const bf16_t* gsrc_minus_off, bf16_t* lds_wave_base) {
    static_assert(OFF >= 0 && OFF < 4096, "the instruction offset is 13 bits signed; a larger value wraps silently");
    __builtin_amdgcn_global_load_lds(
        (const void __attribute__((address_space(1)))*)gsrc_minus_off,
        (void __attribute__((address_space(3)))*)lds_wave_base, 16, OFF, 0);
}
// LDS reads whose place in the instruction stream is fixed by the source order (the
// compiler's scheduler, short of registers, would issue every read right before its use).
// The waits for them are written by hand: LDS operations of a wave return in order, so
// "at most N outstanding" after N younger reads means this one has arrived.
template <int IMM>
__device__ __forceinline__ bf16x4 lds_read_tr_at(uint32_t addr) {
    bf16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(IMM));
    return v;
}
template <int IMM>
__device__ __forceinline__ bf16x8 lds_read_b128_at(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(IMM));
    return v;
}
template <int N>
__device__ __forceinline__ void lds_wait_all_but(bf16x8& x) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N));
}

template <int NI, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < NI) {
        f(std::integral_constant<int, I>{});
        static_for<NI, I + 1>(f);
    }
}

// Transposing LDS read.  Within each group of 16 lanes, lane i receives, as
// element e, element (i % 4) of the 8-byte row addressed by lane (i / 4 + 4 e).
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)p);
}

template <int D_H>
__global__ __launch_bounds__(512, 1) void sparse_attn_kernel(
    const bf16_t* __restrict__ q, int M, const int32_t* __restrict__ idx, int H_q, int H_kv,
    const bf16_t* __restrict__ Kc, const bf16_t* __restrict__ Vc, int64_t st, int64_t sh, int N,
    bf16_t* __restrict__ o, int n_row_tiles, float scale_log2, int n_splits, float* __restrict__ part) {
    constexpr int KS = D_H / 16;          // k-steps of the QK^T contraction
    constexpr int DT = D_H / 32;          // 32-row tiles of O^T
    constexpr int CPRW = D_H / 8;         // 16-byte chunks per cache row
    constexpr int RPI = 64 / CPRW;        // rows moved by one global->LDS instruction
    constexpr int NI = BN_KEYS / RPI / 4; // such instructions per wave, tile and tensor

    constexpr int TILE = BN_KEYS * D_H;   // elements of one K or V tile
    // three stages per tensor: K tile t lives in stage t % 3, V tile t in stage 3 + t % 3
    __shared__ __align__(16) bf16_t smem[6 * TILE];
    auto k_stage = [&](int t) __attribute__((always_inline)) { return smem + (t % 3) * TILE; };
    auto v_stage = [&](int t) __attribute__((always_inline)) { return smem + (3 + t % 3) * TILE; };

    __shared__ int simd_waves[4], group_waves[2];

    const int tid = threadIdx.x, lane = tid & 63;
    // Group and slot of this wave.  The two waves that share a SIMD must land in different
    // groups: the SIMD id comes from the hardware id register (HW_ID bits 5:4), the first
    // wave to register on a SIMD joins group A (0), the second group B (1).  Should the
    // eight waves not sit two per SIMD, the split falls back to wave index order (correct,
    // but the phases of a SIMD's waves then no longer alternate).
    int grp, widx;
    {
        if (tid < 4) simd_waves[tid] = 0;
        if (tid < 2) group_waves[tid] = 0;
        __syncthreads();
        int a = 0, b = 0;
        if (lane == 0) {
            const int simd = __builtin_amdgcn_s_getreg(((2 - 1) << 11) | (4 << 6) | 4);
            a = atomicAdd(&simd_waves[simd & 3], 1) & 1;
            b = atomicAdd(&group_waves[a], 1);
        }
        grp = __builtin_amdgcn_readfirstlane(a);
        widx = __builtin_amdgcn_readfirstlane(b);
        __syncthreads();
        if (group_waves[0] != 4) {
            const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
            grp = w >> 2;
            widx = w & 3;
        }
    }
    const int wave = widx;                              // role in the cooperative tile loads
    const int g = H_q / H_kv;
    const int kvh = blockIdx.x % H_kv;
    const int rt = n_row_tiles - 1 - blockIdx.x / H_kv;

    const int qr = lane & 31, hf = lane >> 5;
    const int col = rt * 256 + (grp * 4 + widx) * 32 + qr;       // flat (token, head) column
    const int mi = col / g, hg = col - mi * g;
    const bool valid = mi < M;
    const int limit = valid ? idx[mi] : -1;
    const int last_row = min(M - 1, (rt * 256 + 255) / g);
    const int kmax = idx[last_row];                    // rows are sorted: the block's longest span
    // Key split: workgroup blockIdx.y of n_splits takes key tiles ta .. ta + n_tiles - 1 of the
    // block's span and leaves unnormalised fp32 partial results for the merge kernel.
    const int all_tiles = kmax / BN_KEYS + 1;
    const int tiles_per = (all_tiles + n_splits - 1) / n_splits;
    const int ta = blockIdx.y * tiles_per;
    const int n_tiles = min(all_tiles - ta, tiles_per);
    const int j_a = ta * BN_KEYS;                      // first key of this workgroup
    const int64_t part_row = valid ? ((int64_t)blockIdx.y * M + mi) * H_q + kvh * g + hg : 0;
    if (n_tiles <= 0) {                                // more splits than tiles: an empty part
        if (valid && hf == 0) {
            float* pm = part + part_row * (D_H + 4) + D_H;
            pm[0] = -INFINITY;
            pm[1] = 0.0f;
        }
        return;
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

    // ---- global -> LDS: instruction i of this wave moves the RPI logical rows
    //      (i*4 + wave)*RPI ..; lane L fills physical chunk L % CPRW of row L / CPRW and
    //      fetches the logical chunk that the swizzle maps there.  In LDS the rows of one
    //      wave's NI instructions are adjacent (physical row rho(r) below), so they are
    //      reached from one base with immediate offsets of 1 KB ----
    //   K rows: chunk c sits at slot c ^ kswz(row)           (16-byte fragment reads)
    //   V rows: the 64-byte group dt sits at group dt ^ vswz(row)  (transposing 8-byte reads)
    // The swizzles use row bits that the instruction index does not touch, so one lane
    // offset per tensor serves every instruction.
    auto kswz = [](int r) { return D_H == 128 ? (r & 15) : ((r >> 1) & 7); };
    auto vswz = [](int r) { return D_H == 128 ? (r & 3) : ((r >> 1) & 1); };
    constexpr auto rho = [](int r) constexpr { return (((r / RPI) % 4) * NI + r / (4 * RPI)) * RPI + r % RPI; };
    static_assert((4 * RPI) % 16 == 0 && NI * 1024 <= 4096, "row bits of the swizzle / immediate offset range");
    const bf16_t* kbase = Kc + (int64_t)kvh * sh;
    const bf16_t* vbase = Vc + (int64_t)kvh * sh;
    const int l_row = lane / CPRW, l_p = lane % CPRW;
    const int r0 = wave * RPI + l_row;                 // logical row of instruction 0
    const int k_col = (l_p ^ kswz(r0)) * 8;
    const int v_col = ((((l_p >> 2) ^ vswz(r0)) << 2) | (l_p & 3)) * 8;
    const int koff = r0 * (int)st + k_col;             // 32-bit lane offsets from a wave-uniform tile base
    const int voff = r0 * (int)st + v_col;
    const int64_t istep = (int64_t)(4 * RPI) * st - 512;   // next instruction: 4 RPI rows on, minus its 1 KB immediate
    const int wave_slot = wave * NI * RPI * D_H;
    auto dma_k = [&](bf16_t* ks, int j0) __attribute__((always_inline)) {
        const bf16_t* kb = kbase + (int64_t)j0 * st;
        if (j0 + BN_KEYS <= N) {
            static_for<NI>([&](auto i) { dma16<i.value * 1024>(kb + i.value * istep + koff, ks + wave_slot); });
        } else {   // last tile of the cache: rows past N-1 are clamped (they are masked anyway)
            const int rmax = N - 1 - j0;
            static_for<NI>([&](auto i) {
                const int64_t r = min(r0 + i.value * 4 * RPI, rmax);
                dma16<i.value * 1024>(kb + r * st + k_col - i.value * 512, ks + wave_slot);
            });
        }
    };
    auto dma_v = [&](bf16_t* vs, int j0) __attribute__((always_inline)) {
        const bf16_t* vb = vbase + (int64_t)j0 * st;
        if (j0 + BN_KEYS <= N) {
            static_for<NI>([&](auto i) { dma16<i.value * 1024>(vb + i.value * istep + voff, vs + wave_slot); });
        } else {
            const int rmax = N - 1 - j0;
            static_for<NI>([&](auto i) {
                const int64_t r = min(r0 + i.value * 4 * RPI, rmax);
                dma16<i.value * 1024>(vb + r * st + v_col - i.value * 512, vs + wave_slot);
            });
        }
    };

    // ---- fragment addresses: LDS byte addresses in the stage this wave reads next (they
    //      move on after every matrix phase); key block and half are immediate offsets ----
    const uint32_t smem_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)smem;
    // K: logical row kt*32 + qr (physical rho(qr) + 8 kt), logical chunk 2 ks + hf
    const int k_sw = kswz(qr);
    uint32_t kaddr[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        kaddr[ks] = smem_base + 2 * (rho(qr) * D_H + (((ks * 2 + hf) ^ k_sw) << 3));
    // V^T through the transposing read: lane s of a 16-lane group addresses key
    // (4 hf + s/4) and the 4 d's starting at 16*(group%2) + 4*(s%4); the lane then
    // holds 4 consecutive keys of column d = 32 dt + lane%32.  Key 16 ss + 8 e + v_key sits
    // in physical row rho(16 ss + 8 e) + rho(v_key) (the two parts use different row bits).
    const int s16 = lane & 15, dsub = (lane >> 4) & 1;
    const int v_key = 4 * hf + (s16 >> 2);
    const int v_sw = vswz(v_key);
    const int v_lane = (2 * dsub + ((s16 & 3) >> 1)) * 8 + (s16 & 1) * 4;
    uint32_t vaddr[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
        vaddr[dt] = smem_base + 2 * (3 * TILE + rho(v_key) * D_H + v_lane + ((dt ^ v_sw) << 5));

    f32x16 acc_o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[dt][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;
    f32x16 s[2];       // S^T tile: 64 keys x 32 query rows
    bf16x8 pf[4];      // its probabilities as B operand of the second contraction

    auto softmax = [&](int j0) __attribute__((always_inline)) {
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
        {   // the other half-wave's maximum of the same query row: lanes i and i + 32 exchange by a
            // register swap (no LDS round trip)
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
            mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * scale_log2;
        }
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
        // four scores at a time: exponentials, their sum and their bf16 pair conversions are
        // finished before the next four start (keeps only four probabilities live)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int kt = c >> 2, v0 = (c & 3) * 4;
            float pv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) pv[u] = __builtin_amdgcn_exp2f(fmaf(s[kt][v0 + u], scale_log2, -m_use));
            psum += (pv[0] + pv[1]) + (pv[2] + pv[3]);
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
            bf16x2 lo = __builtin_convertvector(f32x2{pv[0], pv[1]}, bf16x2);
            bf16x2 hi = __builtin_convertvector(f32x2{pv[2], pv[3]}, bf16x2);
            asm volatile("" : "+v"(lo), "+v"(hi));   // converted here, not gathered at the end
            bf16x8& dst = pf[kt * 2 + (v0 >> 3)];
            dst[(v0 & 7) + 0] = lo[0];
            dst[(v0 & 7) + 1] = lo[1];
            dst[(v0 & 7) + 2] = hi[0];
            dst[(v0 & 7) + 3] = hi[1];
        }
        l_run += psum;
    };
    // End of a phase: all of this wave's global -> LDS loads but the newest tile's
    // (`pending`) have landed, then the workgroup barrier.  The tile
    // reads are written by hand, so no compiler-made wait is needed around the barrier.
    auto phase_end = [&](bool pending) __attribute__((always_inline)) {
        if (pending) __builtin_amdgcn_s_waitcnt((NI & 0xF) | ((NI >> 4) << 14) | (0x7 << 4) | (0xF << 8));
        else __builtin_amdgcn_s_waitcnt((0x7 << 4) | (0xF << 8));
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // Matrix phase of one wave: O^T += V^T P^T for the V tile at vaddr (with_pv), then
    // S^T = K Q^T for the K tile at kaddr.  The other wave of the SIMD is in
    // its softmax, so this wave alone has to keep the matrix pipe fed: the LDS reads of MFMA
    // j + PD are issued before MFMA j.  P V: MFMA j = (ss, dt) = (j / DT, j % DT), DT
    // independent accumulation chains; A slots 0..3 <- keys 16ss+4hf.., 4..7 <- keys
    // 16ss+8+4hf..  Scores: MFMA n = (ks, kt) = (n / 2, n % 2), two chains.
    constexpr int PD = 4;
    auto matrix_phase = [&](auto with_pv) __attribute__((always_inline)) {
        constexpr int NPV = decltype(with_pv)::value ? 4 * DT : 0, NQK = 2 * KS, NALL = NPV + NQK;
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        bf16x8 opnd[NALL];
        // Order of the MFMAs when both contractions run: two of P V, two of Q K^T, and so on, so
        // that an MFMA follows the one whose accumulator it continues four issue slots later, not
        // two (the score tile has only two accumulation chains; back to back they wait for each
        // other's result).
        constexpr auto is_pv = [](int j) constexpr { return NPV != 0 && (j & 3) < 2; };
        constexpr auto pv_of = [](int j) constexpr { return (j >> 2) * 2 + (j & 3); };
        constexpr auto qk_of = [](int j) constexpr { return NPV != 0 ? (j >> 2) * 2 + (j & 3) - 2 : j; };
        static_assert(NPV == 0 || NPV == NQK, "the interleaved order pairs the two contractions one to one");
        // reads of the operands j+1 .. last (a P V operand is two reads)
        constexpr auto reads_after = [](int j, int last) constexpr {
            int n = 0;
            for (int i = j + 1; i <= last; ++i) n += (NPV != 0 && (i & 3) < 2) ? 2 : 1;
            return n;
        };
        auto issue = [&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            if constexpr (j < NALL) {
                if constexpr (is_pv(j)) {
                    constexpr int p = pv_of(j), ss = p / DT, dt = p % DT;
                    constexpr int at = 2 * rho(16 * ss) * D_H;
                    constexpr int at8 = 2 * rho(16 * ss + 8) * D_H;
                    const bf16x4 a0 = lds_read_tr_at<at>(vaddr[dt]);
                    const bf16x4 a1 = lds_read_tr_at<at8>(vaddr[dt]);
                    opnd[j] = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
                } else {
                    constexpr int n = qk_of(j), ks = n / 2, kt = n % 2;
                    opnd[j] = lds_read_b128_at<2 * kt * 8 * D_H>(kaddr[ks]);
                }
            }
        };
        static_for<PD>(issue);
        static_for<NALL>([&](auto jc) __attribute__((always_inline)) {
            constexpr int j = decltype(jc)::value;
            issue(std::integral_constant<int, j + PD>{});
            constexpr int last = j + PD < NALL ? j + PD : NALL - 1;
            lds_wait_all_but<reads_after(j, last)>(opnd[j]);
            if constexpr (is_pv(j)) {
                constexpr int p = pv_of(j), ss = p / DT, dt = p % DT;
                acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[j], pf[ss], acc_o[dt], 0, 0, 0);
            } else {
                constexpr int n = qk_of(j), ks = n / 2, kt = n % 2;
                s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[j], qf[ks], ks == 0 ? zero : s[kt], 0, 0, 0);
            }
        });
    };

    // ---- phases.  P0: A scores(0).  P(2t+1): A softmax(t) | B values(t-1), scores(t).
    //      P(2t+2): A values(t), scores(t+1) | B softmax(t).  A wave issues its loads at the
    //      end of its matrix phase, while its SIMD partner is in the softmax: next to a partner
    //      that keeps the matrix pipe busy a vector-memory instruction takes several times as
    //      long to issue.  Group A loads V(t+2) at the end of P(2t+2) into the stage V(t-1)
    //      left at the end of P(2t+1); it is first read in P(2t+6); group A lets only its newest
    //      tile stay in flight across a barrier, so V(t+2) has landed by the end of P(2t+4).
    //      Group B loads K(t+3) at the end of P(2t+3) into the stage K(t) left at the end of
    //      P(2t+1); first read in P(2t+6), landed by the end of P(2t+5) (group B waits for all
    //      but its newest tile after issuing K(t+4)).  Every wave passes 2 n_tiles + 3
    //      barriers; tiles past a wave's own last key only cost it the barriers and its loads.
    //      The scores of tile my_tiles (computed from whatever its stage holds) are never used.
    const int my_tiles = wave_limit < 0 ? 0 : max(0, min(wave_limit / BN_KEYS + 1 - ta, n_tiles));
    using yes = std::integral_constant<int, 1>;
    using no = std::integral_constant<int, 0>;
    int k_at = 0, v_at = 0;           // stages the address registers point at
    auto advance = [&](bool also_v) __attribute__((always_inline)) {
        const int kd = k_at == 2 ? -4 * TILE : 2 * TILE;
        k_at = k_at == 2 ? 0 : k_at + 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kaddr[ks] += kd;
        if (also_v) {
            const int vd = v_at == 2 ? -4 * TILE : 2 * TILE;
            v_at = v_at == 2 ? 0 : v_at + 1;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) vaddr[dt] += vd;
        }
    };
    if (grp == 0) {
        dma_v(v_stage(0), j_a);
        if (n_tiles > 1) dma_v(v_stage(1), j_a + BN_KEYS);
        phase_end(n_tiles > 1);                            // K(0), V(0) are in place
        if (my_tiles > 0) {                                // P0
            matrix_phase(no{});
            advance(false);
        }
        phase_end(n_tiles > 1);
        for (int t = 0; t < n_tiles; ++t) {
            if (t < my_tiles) softmax(j_a + t * BN_KEYS);
            phase_end(t + 1 < n_tiles);                    // V(t) has landed
            if (t < my_tiles) {
                matrix_phase(yes{});
                advance(true);
            }
            if (t + 2 < n_tiles) dma_v(v_stage(t + 2), j_a + (t + 2) * BN_KEYS);
            phase_end(true);
        }
        phase_end(false);
    } else {
        dma_k(k_stage(0), j_a);
        if (n_tiles > 1) dma_k(k_stage(1), j_a + BN_KEYS);
        if (n_tiles > 2) dma_k(k_stage(2), j_a + 2 * BN_KEYS);
        if (n_tiles > 2) __builtin_amdgcn_s_waitcnt(((2 * NI) & 0xF) | (((2 * NI) >> 4) << 14) | (0x7 << 4) | (0xF << 8));
        phase_end(n_tiles > 1);                            // K(0), V(0) are in place
        phase_end(true);                                   // P0
        if (my_tiles > 0) {                                // P1
            matrix_phase(no{});
            advance(false);
        }
        phase_end(n_tiles > 2);                            // K(1) has landed
        for (int t = 0; t < n_tiles; ++t) {
            if (t < my_tiles) softmax(j_a + t * BN_KEYS);
            phase_end(true);
            if (t < my_tiles) {
                matrix_phase(yes{});
                advance(true);
            }
            if (t + 3 < n_tiles) dma_k(k_stage(t), j_a + (t + 3) * BN_KEYS);
            phase_end(t + 3 < n_tiles);                    // K(t+2) has landed
        }
    }

    // ---- normalise and write: lane holds 4 consecutive d per (dt, v/4) ----
    float l_tot = l_run + __shfl_xor(l_run, 32);
    if (!valid) return;
    if (n_splits == 1) {
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
    } else {
        // part row: d_h unnormalised sums, then the exponent's reference point and the row sum
        float* pp = part + part_row * (D_H + 4);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                f32x4 w;
#pragma unroll
                for (int u = 0; u < 4; ++u) w[u] = acc_o[dt][vq * 4 + u];
                *reinterpret_cast<f32x4*>(pp + dt * 32 + 8 * vq + 4 * hf) = w;
            }
        if (hf == 0) {
            pp[D_H] = m_run;
            pp[D_H + 1] = l_tot;
        }
    }
}

// Merge of a key-split launch: o = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s with m = max m_s.
// One thread per (token, head) row and four output elements.
template <int D_H>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part, int64_t rows,
                                                         int n_splits, bf16_t* __restrict__ o) {
    constexpr int TPR = D_H / 4;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = t / TPR;
    const int d0 = (int)(t % TPR) * 4;
    if (row >= rows) return;
    float m = -INFINITY;
    for (int sp = 0; sp < n_splits; ++sp) m = fmaxf(m, part[(sp * rows + row) * (D_H + 4) + D_H]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float l = 0.0f;
    for (int sp = 0; sp < n_splits; ++sp) {
        const float* pp = part + (sp * rows + row) * (D_H + 4);
        const float ms = pp[D_H];
        if (ms == -INFINITY) continue;                 // an empty part: its sums were never written
        const float w = __builtin_amdgcn_exp2f(ms - m);
        const f32x4 v = *reinterpret_cast<const f32x4*>(pp + d0);
        acc += v * w;
        l += pp[D_H + 1] * w;
    }
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    bf16x4 w;
#pragma unroll
    for (int u = 0; u < 4; ++u) w[u] = (bf16_t)(acc[u] * inv);
    *reinterpret_cast<bf16x4*>(o + row * D_H + d0) = w;
}

}  // namespace

void cc_launch_attention(const bf16_t* q, int M, const int32_t* idx, const cc_model_desc& m,
                         const cc_kv_layer& kv, bf16_t* o, float* part, int64_t part_rows,
                         const cc_launch_override& ovr, hipStream_t s) {
    if (M <= 0) return;
    const int g = m.H_q / m.H_kv;
    const int n_row_tiles = (int)(((int64_t)M * g + 255) / 256);   // 256 (token, head) columns each
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)m.d_h);
    // A grid that does not fill the chip is split along the keys: S workgroups per block, each over
    // 1/S of the block's key tiles, and a merge pass.  Model, in key-tile times: the longest
    // workgroup (t_max / S tiles) or the whole work spread over the CUs, whichever is longer; the
    // work is taken as half of blocks x t_max (spans grow with the position of the block's last
    // token) with 30 % on top for the uneven end, as measured; plus the merge's traffic.
    const int64_t rows = (int64_t)M * m.H_q;
    static const int n_cu = [] {
        int dev = 0, n = 256;
        if (hipGetDevice(&dev) == hipSuccess)
            (void)hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        return n > 0 ? n : 256;
    }();
    const int n_wg = n_row_tiles * m.H_kv;
    const int t_max = (kv.N + BN_KEYS - 1) / BN_KEYS;
    int S = 1;
    if (ovr.attn_splits > 0) {                        // test override (cc_debug_set_launch)
        S = ovr.attn_splits;
    } else if (part && n_wg < 2 * n_cu) {
        const double tile_us = m.d_h == 128 ? 1.9 : 1.0;
        const double spread = 1.3 * 0.5 * (double)n_wg * t_max / n_cu;
        double best = t_max > spread ? t_max : spread;
        for (int sp = 2; sp <= 8 && sp <= t_max; ++sp) {
            if (sp * rows > part_rows) break;
            const double longest = (double)((t_max + sp - 1) / sp);
            const double merge_us = 3.0 + (double)(sp * rows) * (m.d_h + 4) * 4 / 4.0e6;
            const double c = (longest > spread ? longest : spread) + merge_us / tile_us;
            if (c < 0.95 * best) best = c, S = sp;
        }
    }
    if (S < 1 || !part || S * rows > part_rows) S = 1;
    if (S > t_max) S = t_max;
    dim3 grid(n_row_tiles * m.H_kv, S), block(512);
    if (m.d_h == 128)
        hipLaunchKernelGGL(sparse_attn_kernel<128>, grid, block, 0, s, q, M, idx, m.H_q, m.H_kv,
                           (const bf16_t*)kv.K, (const bf16_t*)kv.V, kv.stride_token, kv.stride_head,
                           kv.N, o, n_row_tiles, scale_log2, S, part);
    else
        hipLaunchKernelGGL(sparse_attn_kernel<64>, grid, block, 0, s, q, M, idx, m.H_q, m.H_kv,
                           (const bf16_t*)kv.K, (const bf16_t*)kv.V, kv.stride_token, kv.stride_head,
                           kv.N, o, n_row_tiles, scale_log2, S, part);
    if (S > 1) {
        const int64_t threads = rows * (m.d_h / 4);
        dim3 mg((unsigned)((threads + 255) / 256));
        if (m.d_h == 128) hipLaunchKernelGGL(attn_merge_kernel<128>, mg, dim3(256), 0, s, part, rows, S, o);
        else hipLaunchKernelGGL(attn_merge_kernel<64>, mg, dim3(256), 0, s, part, rows, S, o);
    }
}
