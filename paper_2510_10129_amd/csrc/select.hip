// Token selection on the device: importance scores, top-k candidates with
// lowest-index tie-break, sliding-window grouping and compaction
// (Sections 4.2 and 4.3 of the paper).
#include "cc_internal.h"

// ----------------------------------------------------------------------------
// Importance score per chunk token: sum of the query->chunk attention block
// over its query rows (Section 4.2).  Every column has ONE fp32 accumulator
// and its rows are added in ascending order, so the result is the same bit
// pattern on every run and on any host that adds in that order.
//
// The adds are cheap; the kernel lives on bytes in flight.  A workgroup of four
// waves owns 64 columns.  Rows are taken 64 at a time: wave w issues the loads
// of rows 16w .. 16w+15 of the chunk together (lane = column, 256 contiguous
// bytes per row and wave) and parks them in LDS; wave 0 then walks the 64
// rows of its column in order.  32 KB of LDS per workgroup: five workgroups
// (80 KB of loads in flight) per CU.  Two LDS buffers let the loads of the next chunk
// start while the sums of this one are taken.
// ----------------------------------------------------------------------------
#define CS_ROWS 64
#define CS_RPW (CS_ROWS / 4)   // rows per wave and chunk
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ attn, int Q_a, int T,
                                                     int64_t ld, float* __restrict__ score) {
    __shared__ float tile[2][CS_ROWS][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x * 64 + lane;
    const bool col_ok = t < T;
    const float* p = attn + (col_ok ? t : 0);
    float acc = 0.0f;
    const int n_chunks = (Q_a + CS_ROWS - 1) / CS_ROWS;
    for (int c = 0; c < n_chunks; ++c) {
        const int q0 = c * CS_ROWS + wave * CS_RPW;
        float (*buf)[64] = tile[c & 1];
        float v[CS_RPW];
#pragma unroll
        for (int u = 0; u < CS_RPW; ++u) {      // rows past the end re-read the last row and are not summed
            const int q = min(q0 + u, Q_a - 1);
            v[u] = __builtin_nontemporal_load(p + (int64_t)q * ld);
        }
#pragma unroll
        for (int u = 0; u < CS_RPW; ++u) buf[wave * CS_RPW + u][lane] = v[u];
        // the buffer written now was last read two chunks ago; one barrier per chunk
        // orders both that reuse and this hand-over
        __syncthreads();
        if (wave == 0) {
            const int rows = min(CS_ROWS, Q_a - c * CS_ROWS);
            int r = 0;
            for (; r + 8 <= rows; r += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = buf[r + u][lane];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc = acc + x[u];
            }
            for (; r < rows; ++r) acc = acc + buf[r][lane];
        }
    }
    if (wave == 0 && col_ok) score[t] = acc;
}

void cc_launch_colsum(const float* attn, int Q_a, int T, int64_t ld, float* score, hipStream_t s) {
    hipLaunchKernelGGL(colsum_kernel, dim3((T + 63) / 64), dim3(256), 0, s, attn, Q_a, T, ld, score);
}

// ----------------------------------------------------------------------------
// Importance scores straight from the auxiliary model's batched last-layer
// attention (Section 4.2): batch element c holds the attention of `chunk c +
// query`, [head][query row][key column]; the query -> chunk block starts at
// column col0 and is len columns wide.  Heads are averaged (the attention maps
// of Section 3 are head averages), then the query rows are summed:
//     a(q, j) = (sum over heads, ascending, of A[h][q][col0 + j]) * (1 / H)
//     s(t0 + j) = sum over q, ascending, of a(q, j)
// all in fp32 with one accumulator each, so the result has one bit pattern.
// Same scheme as the column sum above with more loads in flight (a request has
// only T / 64 workgroups): sixteen waves own 64 columns of one batch element,
// wave w forms a(q, .) for four of every 64 query rows (the loads of four rows
// x eight heads are issued together), parks them in LDS, and wave 0 adds the 64
// parked values of its column in order.
// ----------------------------------------------------------------------------
#define BS_WAVES 16
#define BS_RPW (CS_ROWS / BS_WAVES)
__global__ __launch_bounds__(64 * BS_WAVES) void block_scores_kernel(cc_blk_args a, int H, int Q_a, float inv_h,
                                                                     float* __restrict__ score) {
    __shared__ float tile[2][CS_ROWS][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int blk = blockIdx.x;
    int lo = 0, hi = a.n_seg - 1, sidx = 0;
    while (lo <= hi) {                      // last segment whose first workgroup is <= blk
        const int mid = (lo + hi) >> 1;
        if (a.seg[mid].blk0 <= blk) { sidx = mid; lo = mid + 1; } else { hi = mid - 1; }
    }
    const cc_blk_seg sg = a.seg[sidx];
    const int j = (blk - sg.blk0) * 64 + lane;
    const bool col_ok = j < sg.len;
    const float* p = sg.attn + sg.col0 + (col_ok ? j : 0);
    float acc = 0.0f;
    const int n_groups = (Q_a + CS_ROWS - 1) / CS_ROWS;
    for (int c = 0; c < n_groups; ++c) {
        const int q0 = c * CS_ROWS + wave * BS_RPW;
        float (*buf)[64] = tile[c & 1];
        const float* pq[BS_RPW];
        float m[BS_RPW];
#pragma unroll
        for (int u = 0; u < BS_RPW; ++u) {      // rows past the end re-read the last row and are not summed
            pq[u] = p + (int64_t)min(q0 + u, Q_a - 1) * sg.stride_row;
            m[u] = 0.0f;
        }
        for (int h0 = 0; h0 < H; h0 += 8) {
            float v[BS_RPW][8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {       // heads past the end re-read the last head and are not added
                const int64_t ho = (int64_t)min(h0 + i, H - 1) * sg.stride_head;
#pragma unroll
                for (int u = 0; u < BS_RPW; ++u) v[u][i] = __builtin_nontemporal_load(pq[u] + ho);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int u = 0; u < BS_RPW; ++u) m[u] = h0 + i < H ? m[u] + v[u][i] : m[u];
        }
#pragma unroll
        for (int u = 0; u < BS_RPW; ++u) buf[wave * BS_RPW + u][lane] = m[u] * inv_h;
        // the buffer written now was last read two groups ago; one barrier per group
        // orders both that reuse and this hand-over
        __syncthreads();
        if (wave == 0) {
            const int rows = min(CS_ROWS, Q_a - c * CS_ROWS);
            int r = 0;
            for (; r + 8 <= rows; r += 8) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = buf[r + u][lane];
#pragma unroll
                for (int u = 0; u < 8; ++u) acc = acc + x[u];
            }
            for (; r < rows; ++r) acc = acc + buf[r][lane];
        }
    }
    if (wave == 0 && col_ok) score[sg.t0 + j] = acc;
}

void cc_launch_block_scores(const cc_blk_args& a, int H, int Q_a, float* score, hipStream_t s) {
    if (a.n_blocks <= 0) return;
    hipLaunchKernelGGL(block_scores_kernel, dim3(a.n_blocks), dim3(64 * BS_WAVES), 0, s, a, H, Q_a, 1.0f / (float)H, score);
}

// ----------------------------------------------------------------------------
// Top-k + grouping + compaction in one workgroup of 16 waves.
//
// Scores become order-preserving 32-bit keys; the k-th largest key is found by
// a most-significant-digit-first radix search (4 passes of 8 bits: LDS histogram,
// the bin of the k-th key by a suffix sum over the 256 bins); ties at the threshold are ranked by index
// with wave ballots so that the lowest indices win.  Candidates, passing
// window starts and chosen tokens are bitmaps in LDS: a window test is a
// popcount over the words the window spans, and the final compaction is one
// scan over per-word popcounts.
// ----------------------------------------------------------------------------
#define SEL_THREADS 1024
#define SEL_WAVES 16
#define SEL_TCAP 131072
#define SEL_WORDS (SEL_TCAP / 64 + 20)   // bitmap words incl. zero padding past T + window

__device__ __forceinline__ uint32_t score_key(float s) {
    uint32_t u = __float_as_uint(s + 0.0f);   // -0 -> +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// popcount of bits [b0, b1) of a zero-padded bitmap
__device__ __forceinline__ int window_popc(const uint64_t* bm, int b0, int b1) {
    int w0 = b0 >> 6, w1 = (b1 - 1) >> 6;
    int cnt = 0;
    for (int wi = w0; wi <= w1; ++wi) {
        uint64_t word = bm[wi];
        if (wi == w0) word &= ~0ULL << (b0 & 63);
        if (wi == w1) {
            int e = b1 & 63;
            if (e) word &= (1ULL << e) - 1ULL;
        }
        cnt += __popcll(word);
    }
    return cnt;
}

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(
    const float* __restrict__ score, int T, int k, int window, int tau, int grouping,
    int idx_offset, int n_tail, int32_t* __restrict__ idx_out, int32_t* __restrict__ n_out) {
    __shared__ uint64_t cand[SEL_WORDS];
    __shared__ uint64_t pass[SEL_WORDS];
    __shared__ uint64_t marked[SEL_WORDS];
    __shared__ uint32_t word_prefix[SEL_TCAP / 64 + 1];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_tot[SEL_WAVES];
    __shared__ uint32_t sh_prefix, sh_krem, sh_total;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const uint64_t lane_lt = (1ULL << lane) - 1ULL;
    const int n_words = (T + 63) >> 6;

    for (int i = tid; i < SEL_WORDS; i += SEL_THREADS) {
        cand[i] = 0;
        pass[i] = 0;
        marked[i] = 0;
    }
    __syncthreads();

    // ---- threshold key: the k-th largest (0 < k < T) ----
    uint32_t kth = 0, krem = 0;
    const bool all = k >= T, none = k <= 0;
    if (!all && !none) {
        uint32_t prefix = 0, mask = 0;
        krem = (uint32_t)k;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int base = 0; base < T; base += SEL_THREADS) {
                const int t = base + tid;
                if (t < T) {
                    const uint32_t key = score_key(score[t]);
                    if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
                }
            }
            __syncthreads();
            // the digit b of the k-th largest key: the largest b with (keys of larger digit) < krem
            // <= (those + keys of digit b); thread b holds bin b, suffix sums by wave shuffles
            uint32_t h = 0, inc = 0;                    // bin tid; sum of bins tid .. end of this wave
            if (tid < 256) {
                h = inc = hist[tid];
                for (int off = 1; off < 64; off <<= 1) {
                    uint32_t o = __shfl_down(inc, off);
                    if (lane + off < 64) inc += o;
                }
                if (lane == 0) wave_tot[wave] = inc;
            }
            __syncthreads();
            if (tid < 256) {
                uint32_t above = inc - h;               // keys in bins above tid
                for (int w = wave + 1; w < 4; ++w) above += wave_tot[w];
                const bool here = tid == 0 ? above < krem : (above < krem && krem <= above + h);
                if (here) {
                    sh_prefix = prefix | ((uint32_t)tid << shift);
                    sh_krem = krem - above;
                }
            }
            __syncthreads();
            prefix = sh_prefix;
            krem = sh_krem;
            mask |= 255u << shift;
        }
        kth = prefix;
    }

    // ---- candidate bitmap; equal keys are taken in index order ----
    // Wave w owns the contiguous tokens [w * seg, (w + 1) * seg): it counts its keys equal to the
    // threshold, the sixteen counts give every wave the rank of its first such key, and a second
    // walk ranks them 64 at a time by ballot.  One barrier in all.
    {
        const int seg = ((T + SEL_WAVES * 64 - 1) / (SEL_WAVES * 64)) * 64;   // tokens per wave, whole words
        const int t0 = wave * seg, t1 = min(T, t0 + seg);
        uint32_t n_eq = 0;
        if (!all && !none) {
            for (int base = t0; base < t1; base += 64) {
                const int t = base + lane;
                const bool eq = t < t1 && score_key(score[t]) == kth;
                n_eq += (uint32_t)__popcll(__ballot(eq));
            }
        }
        if (lane == 0) wave_tot[wave] = n_eq;
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        for (int base = t0; base < t1; base += 64) {
            const int t = base + lane;
            bool gt = false, eq = false;
            if (t < t1) {
                if (all) {
                    gt = true;
                } else if (!none) {
                    const uint32_t key = score_key(score[t]);
                    gt = key > kth;
                    eq = key == kth;
                }
            }
            const uint64_t be = __ballot(eq);
            const uint32_t rank = before + (uint32_t)__popcll(be & lane_lt);
            const uint64_t bc = __ballot(gt || (eq && rank < krem));
            if (lane == 0) cand[base >> 6] = bc;
            before += (uint32_t)__popcll(be);
        }
        __syncthreads();
    }

    // ---- windows that start at a candidate and hold >= tau candidates ----
    if (grouping) {
        for (int base = 0; base < T; base += SEL_THREADS) {
            int t = base + tid;
            bool ok = false;
            if (t < T && ((cand[t >> 6] >> (t & 63)) & 1ULL))
                ok = window_popc(cand, t, t + window) >= tau;   // bits past T are zero
            uint64_t b = __ballot(ok);
            if (lane == 0) pass[(base >> 6) + wave] = b;
        }
        __syncthreads();
        // a token is chosen when some passing window covers it
        for (int base = 0; base < T; base += SEL_THREADS) {
            int t = base + tid;
            bool ok = false;
            if (t < T) {
                int b0 = t - window + 1;
                ok = window_popc(pass, b0 < 0 ? 0 : b0, t + 1) > 0;
            }
            uint64_t b = __ballot(ok);
            if (lane == 0) marked[(base >> 6) + wave] = b;
        }
    } else {
        for (int i = tid; i < n_words; i += SEL_THREADS) marked[i] = cand[i];
    }
    __syncthreads();

    // ---- exclusive scan of per-word popcounts ----
    uint32_t run = 0;
    for (int base = 0; base < n_words; base += SEL_THREADS) {
        int wi = base + tid;
        uint32_t c = wi < n_words ? (uint32_t)__popcll(marked[wi]) : 0u;
        uint32_t inc = c;
        for (int off = 1; off < 64; off <<= 1) {
            uint32_t o = __shfl_up(inc, off);
            if (lane >= off) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        uint32_t before = run, total = 0;
        for (int w = 0; w < SEL_WAVES; ++w) {
            uint32_t cw = wave_tot[w];
            if (w < wave) before += cw;
            total += cw;
        }
        if (wi < n_words) word_prefix[wi] = before + inc - c;
        run += total;
        __syncthreads();
    }
    const uint32_t n_sel = run;

    // ---- compaction: ascending token order by construction ----
    for (int base = 0; base < T; base += SEL_THREADS) {
        int t = base + tid;
        if (t < T) {
            uint64_t word = marked[t >> 6];
            if ((word >> (t & 63)) & 1ULL) {
                uint32_t pos = word_prefix[t >> 6] + (uint32_t)__popcll(word & ((1ULL << (t & 63)) - 1ULL));
                idx_out[pos] = idx_offset + t;
            }
        }
    }
    for (int j = tid; j < n_tail; j += SEL_THREADS) idx_out[n_sel + j] = idx_offset + T + j;
    if (tid == 0) *n_out = (int32_t)n_sel + n_tail;
    (void)sh_total;
}

void cc_launch_select(const float* score, int T, int k, int window, int tau, int grouping,
                      int idx_offset, int n_tail, int32_t* idx_out, int32_t* n_out, hipStream_t s) {
    hipLaunchKernelGGL(select_kernel, dim3(1), dim3(SEL_THREADS), 0, s, score, T, k, window, tau,
                       grouping, idx_offset, n_tail, idx_out, n_out);
}

// ----------------------------------------------------------------------------
// idx check: strictly ascending (or merely in range when strict == 0), each in
// [lo, hi).  flag receives the number of violations.
// ----------------------------------------------------------------------------
__global__ void check_idx_kernel(const int32_t* __restrict__ idx, int M, int lo, int hi, int strict,
                                 int32_t* __restrict__ flag) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= M) return;
    int v = idx[i];
    bool bad = v < lo || v >= hi;
    if (strict && i > 0 && idx[i - 1] >= v) bad = true;
    if (bad) atomicAdd(flag, 1);
}

void cc_launch_check_idx(const int32_t* idx, int M, int lo, int hi, int strict, int32_t* flag,
                         hipStream_t s) {
    if (M <= 0) return;
    hipLaunchKernelGGL(check_idx_kernel, dim3((M + 255) / 256), dim3(256), 0, s, idx, M, lo, hi,
                       strict, flag);
}
