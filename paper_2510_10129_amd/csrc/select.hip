// Token selection on the device: importance scores, top-k candidates with
// lowest-index tie-break, sliding-window grouping and compaction
// (Sections 4.2 and 4.3 of the paper).
#include "cc_internal.h"

// Order-preserving 32-bit key of a score: a larger score has a larger key.
__device__ __forceinline__ uint32_t score_key(float s) {
    const uint32_t u = __float_as_uint(s + 0.0f);   // -0 -> +0
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);   // negative: all bits flipped; else the sign bit set
}

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
// rows of its column in order.  32 KB of LDS per workgroup: five workgroups per
// CU.  The loads of the next chunk are in flight before this chunk is parked, and
// two LDS buffers let the waves go on while the sums of this one are taken.
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
    // the loads of chunk c + 1 are issued before chunk c is parked: two chunks of loads in flight
    float va[CS_RPW], vb[CS_RPW];
    auto load_chunk = [&](float (&v)[CS_RPW], int c) {
        const int q0 = c * CS_ROWS + wave * CS_RPW;
#pragma unroll
        for (int u = 0; u < CS_RPW; ++u) {      // rows past the end re-read the last row and are not summed
            const int q = min(q0 + u, Q_a - 1);
            v[u] = __builtin_nontemporal_load(p + (int64_t)q * ld);
        }
    };
    auto park_and_sum = [&](const float (&v)[CS_RPW], int c) {
        float (*buf)[64] = tile[c & 1];
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
    };
    load_chunk(va, 0);
    for (int c = 0; c < n_chunks; c += 2) {
        if (c + 1 < n_chunks) load_chunk(vb, c + 1);
        park_and_sum(va, c);
        if (c + 1 < n_chunks) {
            if (c + 2 < n_chunks) load_chunk(va, c + 2);
            park_and_sum(vb, c + 1);
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
// Top-k + grouping + compaction in one workgroup of 16 waves.  One compute unit
// executes all of it, so the work per token is kept to two passes over the
// scores and everything after them runs per 64-token bitmap word.
//
// Scores become order-preserving 32-bit keys; the k-th largest key is found by a
// most-significant-digit-first radix search over 11 + 11 + 10 bits (LDS
// histogram, then the bin of the k-th key by a suffix sum over the bins).
//   scan 1  histogram of the first digit of every key.  The scores of a request
//           sit in a few binades, so neighbouring keys mostly share the digit: a
//           thread merges runs of equal digits among its own keys and adds a run
//           with one LDS atomic (same-address atomics serialise).
//   scan 2  keys above the threshold digit are candidates (one ballot per word);
//           keys of the threshold digit go, with their token index, into a list in
//           LDS.  The two remaining digits are resolved on that list, and the
//           list entries at or above the threshold set their candidate bits.
// A list that would not fit (more than SEL_LIST keys share the threshold digit)
// or a threshold value of which only some keys are taken (equal scores: the lowest
// indices win, ranked with wave ballots and a scan over per-word counts) takes the
// general path: the remaining digits and the candidates from further passes over
// the scores.
// Candidates, passing window starts and chosen tokens are bitmaps in LDS.  For
// windows up to 64 tokens a thread owns a bitmap word: it tests the windows that
// start at the word's candidates with shifts and popcounts, spreads passing
// starts over their windows by doubling shifts, and writes the indices of a
// 16-token quarter of a word from its set bits; longer windows are tested per
// token with popcounts over the words they span.
// ----------------------------------------------------------------------------
#define SEL_THREADS 1024
#define SEL_WAVES 16
#define SEL_TCAP 131072
#define SEL_WORDS (SEL_TCAP / 64 + 20)   // bitmap words incl. zero padding past T + window
#define SEL_BINS 2048
#define SEL_BATCH 8                      // keys a thread loads together
#define SEL_LIST 12288                   // keys of the threshold digit that the LDS list holds

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

// In-place exclusive prefix sum of v[0 .. n) by the whole workgroup; returns the total.
// wave_tot: SEL_WAVES words of LDS.  Ends with a barrier.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t* v, int n, uint32_t* wave_tot) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t run = 0;
    for (int base = 0; base < n; base += SEL_THREADS) {
        const int i = base + tid;
        const uint32_t c = i < n ? v[i] : 0u;
        uint32_t inc = c;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(inc, off);
            if (lane >= off) inc += o;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        // lanes 0..15 of every wave hold the sixteen totals; inclusive prefix over them by shuffles
        uint32_t wt = lane < SEL_WAVES ? wave_tot[lane] : 0u;
        for (int off = 1; off < SEL_WAVES; off <<= 1) {
            const uint32_t o = __shfl_up(wt, off);
            if (lane >= off) wt += o;
        }
        const uint32_t before = run + (wave ? __shfl(wt, wave - 1) : 0u);
        const uint32_t total = __shfl(wt, SEL_WAVES - 1);
        if (i < n) v[i] = before + inc - c;
        run += total;
        __syncthreads();
    }
    return run;
}

// Adds one digit to a thread's run of equal digits; a run that ends goes to the histogram with
// one LDS atomic (same-address atomics serialise, and the scores of a request sit in a few
// binades: measured against one atomic per key, merging runs is a fifth faster).
__device__ __forceinline__ void run_add(uint32_t* hist, uint32_t dgt, uint32_t& run_d, uint32_t& run_n) {
    if (run_n && dgt == run_d) {
        ++run_n;
    } else {
        if (run_n) atomicAdd(&hist[run_d], run_n);
        run_d = dgt;
        run_n = 1;
    }
}

// Histogram (nb = dmask + 1 bins, zeroed here) of digit (key >> shift) & dmask over the keys
// with (key & mask) == prefix.  Thread tid takes tokens tid, tid + 1024, ...; the loads of the
// next batch are issued before the current one is processed.  Ends with a barrier.
__device__ __forceinline__ void hist_of_scores(const float* __restrict__ score, int T, uint32_t prefix,
                                               uint32_t mask, int shift, uint32_t dmask, uint32_t* hist) {
    const int tid = threadIdx.x;
    for (int i = tid; i <= (int)dmask; i += SEL_THREADS) hist[i] = 0;
    __syncthreads();
    constexpr int STEP = SEL_THREADS * SEL_BATCH;
    float cur[SEL_BATCH], nxt[SEL_BATCH];
#pragma unroll
    for (int j = 0; j < SEL_BATCH; ++j) {
        const int t = j * SEL_THREADS + tid;
        cur[j] = t < T ? score[t] : 0.0f;
        nxt[j] = 0.0f;
    }
    uint32_t run_d = 0, run_n = 0;
    for (int base = 0; base < T; base += STEP) {
        if (base + STEP < T) {
#pragma unroll
            for (int j = 0; j < SEL_BATCH; ++j) {
                const int t = base + STEP + j * SEL_THREADS + tid;
                nxt[j] = t < T ? score[t] : 0.0f;
            }
        }
#pragma unroll
        for (int j = 0; j < SEL_BATCH; ++j) {
            const int t = base + j * SEL_THREADS + tid;
            const uint32_t key = score_key(cur[j]);
            if (t < T && (key & mask) == prefix) run_add(hist, (key >> shift) & dmask, run_d, run_n);
        }
#pragma unroll
        for (int j = 0; j < SEL_BATCH; ++j) cur[j] = nxt[j];
    }
    if (run_n) atomicAdd(&hist[run_d], run_n);
    __syncthreads();
}

// The bin b of the krem-th largest entry of a histogram of nb (1024 or 2048) bins: the largest b
// with (entries in bins above b) < krem <= (those + bin b).  Returns b, krem minus the entries
// above b, and the bin's count through sh[0..2].  Thread t holds bins 2t, 2t+1 (nb = 2048) or
// bin t; suffix sums by wave shuffles, then over the waves' totals.  Ends with a barrier.
__device__ __forceinline__ void pick_bin(const uint32_t* hist, int nb, uint32_t krem, uint32_t* wave_tot,
                                         uint32_t* sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = nb / SEL_THREADS;
    const uint32_t h0 = hist[tid * per], h1 = per == 2 ? hist[tid * per + 1] : 0u;
    const uint32_t mine = h0 + h1;
    uint32_t inc = mine;                              // this thread's bins .. end of the wave
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_down(inc, off);
        if (lane + off < 64) inc += o;
    }
    if (lane == 0) wave_tot[wave] = inc;
    __syncthreads();
    // lanes 0..15 of every wave hold the sixteen totals; suffix sums over them by shuffles
    uint32_t wt = lane < SEL_WAVES ? wave_tot[lane] : 0u;
    for (int off = 1; off < SEL_WAVES; off <<= 1) {
        const uint32_t o = __shfl_down(wt, off);
        if (lane + off < SEL_WAVES) wt += o;
    }
    // entries in bins above this thread's: the rest of its wave, then the waves above
    uint32_t above = inc - mine + (wave + 1 < SEL_WAVES ? __shfl(wt, wave + 1) : 0u);
    if (per == 2) {                                   // the upper of the two bins first
        if (above < krem && krem <= above + h1) {
            sh[0] = (uint32_t)(tid * 2 + 1);
            sh[1] = krem - above;
            sh[2] = h1;
        }
        above += h1;
    }
    if (above < krem && krem <= above + h0) {
        sh[0] = (uint32_t)(tid * per);
        sh[1] = krem - above;
        sh[2] = h0;
    }
    __syncthreads();
}

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(
    const float* __restrict__ score, int T, int k, int window, int tau, int grouping,
    int idx_offset, int n_tail, int32_t* __restrict__ idx_out, int32_t* __restrict__ n_out) {
    __shared__ uint64_t cand[SEL_WORDS];
    __shared__ uint64_t pass[SEL_WORDS];
    uint64_t* const marked = cand;      // the chosen-token bitmap takes the candidates' place once the windows are judged
    __shared__ uint32_t word_prefix[SEL_TCAP / 64 + 1];
    __shared__ uint32_t hist[SEL_BINS];
    __shared__ uint32_t list_t[SEL_LIST];       // token index and low 21 key bits of the keys of the threshold digit
    __shared__ uint32_t list_low[SEL_LIST];
    __shared__ uint32_t wave_tot[SEL_WAVES];
    __shared__ uint32_t sh[3];
    __shared__ uint32_t sh_list_n;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const uint64_t lane_lt = (1ULL << lane) - 1ULL;
    const int n_words = (T + 63) >> 6;

    // the bitmaps are read up to `window` bits past T: clear the words that the phases below
    // do not write
    for (int i = n_words + tid; i < n_words + 20 && i < SEL_WORDS; i += SEL_THREADS) {
        cand[i] = 0;
        pass[i] = 0;
    }
    if (tid == 0) sh_list_n = 0;

    // ---- threshold key: the k-th largest (0 < k < T) ----
    uint32_t kth = 0, krem = 0;
    bool rank_ties = false, have_cand = false;
    const bool all = k >= T, none = k <= 0;
    if (!all && !none) {
        // scan 1: first digit (bits 31..21)
        hist_of_scores(score, T, 0u, 0u, 21, 2047u, hist);
        pick_bin(hist, 2048, (uint32_t)k, wave_tot, sh);
        const uint32_t b0 = sh[0];
        krem = sh[1];
        uint32_t bin_count = sh[2];
        uint32_t prefix = b0 << 21, mask = 2047u << 21;
        if (bin_count <= SEL_LIST) {
            // scan 2: candidates above the threshold digit; the keys of that digit into the list
            constexpr int STEP = SEL_THREADS * SEL_BATCH;
            float cur[SEL_BATCH], nxt[SEL_BATCH];
#pragma unroll
            for (int j = 0; j < SEL_BATCH; ++j) {
                const int t = j * SEL_THREADS + tid;
                cur[j] = t < T ? score[t] : 0.0f;
                nxt[j] = 0.0f;
            }
            for (int base = 0; base < T; base += STEP) {
                if (base + STEP < T) {
#pragma unroll
                    for (int j = 0; j < SEL_BATCH; ++j) {
                        const int t = base + STEP + j * SEL_THREADS + tid;
                        nxt[j] = t < T ? score[t] : 0.0f;
                    }
                }
#pragma unroll
                for (int j = 0; j < SEL_BATCH; ++j) {
                    const int r0 = base + j * SEL_THREADS;       // first token of this row of the batch
                    if (r0 < T) {                                // workgroup-uniform
                        const int t = r0 + tid;
                        const uint32_t key = score_key(cur[j]);
                        const uint32_t dgt = key >> 21;
                        const bool gt = t < T && dgt > b0, eq = t < T && dgt == b0;
                        const uint64_t bg = __ballot(gt), be = __ballot(eq);
                        if (lane == 0 && (r0 >> 6) + wave < n_words) cand[(r0 >> 6) + wave] = bg;
                        if (be) {
                            uint32_t at = 0;
                            if (lane == 0) at = atomicAdd(&sh_list_n, (uint32_t)__popcll(be));
                            at = __shfl(at, 0) + (uint32_t)__popcll(be & lane_lt);
                            if (eq) {
                                list_t[at] = (uint32_t)t;
                                list_low[at] = key & 0x1FFFFFu;
                            }
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < SEL_BATCH; ++j) cur[j] = nxt[j];
            }
            __syncthreads();
            const int n_list = (int)sh_list_n;                   // == bin_count
            // second and third digit (bits 20..10, 9..0) on the list
            uint32_t lprefix = 0, lmask = 0;
#pragma unroll 1
            for (int p = 1; p < 3; ++p) {
                const int shift = p == 1 ? 10 : 0;
                const uint32_t dmask = p == 1 ? 2047u : 1023u;
                for (int i = tid; i <= (int)dmask; i += SEL_THREADS) hist[i] = 0;
                __syncthreads();
                uint32_t run_d = 0, run_n = 0;
                for (int i = tid; i < n_list; i += SEL_THREADS) {
                    const uint32_t low = list_low[i];
                    if ((low & lmask) == lprefix) run_add(hist, (low >> shift) & dmask, run_d, run_n);
                }
                if (run_n) atomicAdd(&hist[run_d], run_n);
                __syncthreads();
                pick_bin(hist, (int)dmask + 1, krem, wave_tot, sh);
                lprefix |= sh[0] << shift;
                lmask |= dmask << shift;
                krem = sh[1];
                bin_count = sh[2];
            }
            kth = prefix | lprefix;
            // bin_count keys equal the threshold and krem of them are candidates
            rank_ties = krem < bin_count;
            if (!rank_ties) {
                for (int i = tid; i < n_list; i += SEL_THREADS)
                    if (list_low[i] >= lprefix) {
                        const uint32_t t = list_t[i];
                        atomicOr(reinterpret_cast<unsigned long long*>(&cand[t >> 6]), 1ULL << (t & 63));
                    }
                have_cand = true;
            }
        } else {
            // general path: the other two digits from passes over all scores
#pragma unroll 1
            for (int p = 1; p < 3; ++p) {
                const int shift = p == 1 ? 10 : 0;
                const uint32_t dmask = p == 1 ? 2047u : 1023u;
                hist_of_scores(score, T, prefix, mask, shift, dmask, hist);
                pick_bin(hist, (int)dmask + 1, krem, wave_tot, sh);
                prefix |= sh[0] << shift;
                mask |= dmask << shift;
                krem = sh[1];
                bin_count = sh[2];
            }
            kth = prefix;
            rank_ties = krem < bin_count;
        }
    }

    // ---- candidate bitmap, general path: word (r0 >> 6) + wave is written by wave `wave` ----
    if (!have_cand) {
        if (rank_ties) {
            // threshold keys per word, exclusive scan over the words = rank of a word's first one
            for (int base = 0; base < T; base += SEL_THREADS) {
                const int t = base + tid;
                const bool eq = t < T && score_key(score[t]) == kth;
                const uint64_t be = __ballot(eq);
                if (lane == 0 && (base >> 6) + wave < n_words) word_prefix[(base >> 6) + wave] = (uint32_t)__popcll(be);
            }
            __syncthreads();
            (void)block_exclusive_scan(word_prefix, n_words, wave_tot);
        }
        for (int base = 0; base < T; base += SEL_THREADS * SEL_BATCH) {
            float sv[SEL_BATCH];
#pragma unroll
            for (int j = 0; j < SEL_BATCH; ++j) {
                const int t = base + j * SEL_THREADS + tid;
                sv[j] = t < T ? score[t] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < SEL_BATCH; ++j) {
                const int r0 = base + j * SEL_THREADS;
                if (r0 < T) {                                // workgroup-uniform
                    const int t = r0 + tid;
                    const int wi = (r0 >> 6) + wave;
                    const uint32_t key = score_key(sv[j]);
                    const bool eq = t < T && !all && !none && key == kth;
                    bool take = t < T && (all || (!none && key > kth));
                    if (rank_ties) {
                        const uint64_t be = __ballot(eq);
                        const uint32_t before = wi < n_words ? word_prefix[wi] : 0u;
                        if (eq && before + (uint32_t)__popcll(be & lane_lt) < krem) take = true;
                    } else if (eq) {
                        take = true;
                    }
                    const uint64_t bc = __ballot(take);
                    if (lane == 0 && wi < n_words) cand[wi] = bc;
                }
            }
        }
    }
    __syncthreads();

    // ---- windows that start at a candidate and hold >= tau candidates; a token is chosen when
    //      some passing window covers it ----
    if (grouping && window <= 64) {
        const uint64_t wmask = window == 64 ? ~0ULL : (1ULL << window) - 1ULL;
        // a wave takes a word, lane = token: the window's tokens are bits lane .. lane + window - 1
        // of the 128 bits (word i, word i + 1), fetched as two 32-bit funnel shifts
        const uint32_t m0 = (uint32_t)wmask, m1 = (uint32_t)(wmask >> 32);
        const uint32_t* c32 = reinterpret_cast<const uint32_t*>(cand);
        for (int i = wave; i < n_words; i += SEL_WAVES) {
            const uint32_t* wp = c32 + 2 * i + (lane >> 5);      // word n_words is zero padding
            const uint32_t w0 = wp[0], w1 = wp[1], w2 = wp[2];
            const uint32_t sh5 = lane & 31;
            const uint32_t v0 = __builtin_amdgcn_alignbit(w1, w0, sh5), v1 = __builtin_amdgcn_alignbit(w2, w1, sh5);
            const int cnt = __popc(v0 & m0) + __popc(v1 & m1);
            const uint64_t b = __ballot((v0 & 1u) && cnt >= tau);
            if (lane == 0) pass[i] = b;
        }
        __syncthreads();
        for (int i = tid; i < n_words; i += SEL_THREADS) {
            // bits (lo, hi) = tokens 64(i-1) .. 64i+63; OR of the shifts by 0 .. window-1, by doubling
            uint64_t lo = i ? pass[i - 1] : 0ULL, hi = pass[i];
            for (int covered = 1; covered < window;) {
                const int st = min(covered, window - covered);  // 1 <= st <= 32
                hi |= (hi << st) | (lo >> (64 - st));
                lo |= lo << st;
                covered += st;
            }
            if (i == n_words - 1 && (T & 63)) hi &= (1ULL << (T & 63)) - 1ULL;   // windows are cut at T
            marked[i] = hi;
        }
    } else if (grouping) {
        for (int base = 0; base < T; base += SEL_THREADS) {
            int t = base + tid;
            bool ok = false;
            if (t < T && ((cand[t >> 6] >> (t & 63)) & 1ULL))
                ok = window_popc(cand, t, t + window) >= tau;   // bits past T are zero
            uint64_t b = __ballot(ok);
            if (lane == 0 && (base >> 6) + wave < n_words) pass[(base >> 6) + wave] = b;
        }
        __syncthreads();
        for (int base = 0; base < T; base += SEL_THREADS) {
            int t = base + tid;
            bool ok = false;
            if (t < T) {
                int b0 = t - window + 1;
                ok = window_popc(pass, b0 < 0 ? 0 : b0, t + 1) > 0;
            }
            uint64_t b = __ballot(ok);
            if (lane == 0 && (base >> 6) + wave < n_words) marked[(base >> 6) + wave] = b;
        }
    }                                   // without grouping the candidates are the chosen tokens
    __syncthreads();

    // ---- exclusive scan of per-word popcounts ----
    for (int i = tid; i < n_words; i += SEL_THREADS) word_prefix[i] = (uint32_t)__popcll(marked[i]);
    __syncthreads();
    const uint32_t n_sel = block_exclusive_scan(word_prefix, n_words, wave_tot);

    // ---- compaction: a thread writes the indices of a 16-token quarter of a word ----
    for (int q = tid; q < 4 * n_words; q += SEL_THREADS) {
        const uint64_t word = marked[q >> 2];
        const int sb = 16 * (q & 3);
        uint32_t sub = (uint32_t)(word >> sb) & 0xFFFFu;
        uint32_t pos = word_prefix[q >> 2] + (uint32_t)__popcll(word & ((1ULL << sb) - 1ULL));
        const int t0 = idx_offset + 64 * (q >> 2) + sb;
        while (sub) {
            const int b = __ffs((int)sub) - 1;
            sub &= sub - 1;
            idx_out[pos++] = t0 + b;
        }
    }
    for (int j = tid; j < n_tail; j += SEL_THREADS) idx_out[n_sel + j] = idx_offset + T + j;
    if (tid == 0) *n_out = (int32_t)n_sel + n_tail;
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
