/*
 * cacheclip.h - C ABI of the MI355X (gfx950) selective KV-recompute prefill library.
 *
 * The two top-level calls follow the paper's statement of the online phase
 * (Section 4 overview): cc_select turns the auxiliary model's query->chunk
 * attention block into the list of cache slots to recompute (Sections 4.2 and
 * 4.3), and cc_recompute_layer recomputes those slots in one decoder layer of
 * the primary model with full-attention position ids and overwrites their
 * entries in the global KV cache (Section 4.3, "KV cache update"; the sparse
 * query attention is the kernel Section 5.6 names).  The cc_step_* calls expose
 * the individual stages of cc_recompute_layer on caller-provided buffers.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses on the GPU the context was
 *     created on; "host" pointers are ordinary host memory.  The library never
 *     frees or keeps caller buffers past the call.
 *   - bf16 data is passed as `const void*` / `void*`: 2-byte brain-float, the
 *     upper half of an IEEE binary32.  All matrices are row-major with the
 *     contraction (input-feature) dimension contiguous: W[out][in], y = W x.
 *   - Every call only enqueues work on the context's HIP stream and returns;
 *     nothing synchronises unless stated.  Calls on one context must not
 *     overlap on different host threads.
 *   - Return value: CC_OK (0) or a negative cc_status.  On error nothing has
 *     been enqueued and no output was written; cc_last_error() gives the text.
 *   - Launch shapes (GEMM tile, K loop, split-K shares, key splits of the
 *     attention) are chosen per call from the sizes; cc_debug_set_launch (at
 *     the end of this file) overrides the choice for tests.
 *   - Every cache slot below kv->N must hold finite values, also the slots no
 *     row attends to: a masked key enters the value contraction as probability
 *     zero times its V row, and zero times NaN or infinity is NaN.
 *     cc_assemble_cache writes zeros to the slots it does not fill.
 */
#ifndef CACHECLIP_H
#define CACHECLIP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t cc_status;
enum {
    CC_OK = 0,
    CC_ERR_NULL = -1,      /* a required pointer is NULL */
    CC_ERR_SHAPE = -2,     /* a size or shape the kernels do not support */
    CC_ERR_IDX = -3,       /* idx not strictly ascending / out of range (CC_FLAG_CHECK_IDX only) */
    CC_ERR_WORKSPACE = -4, /* the call needs more rows/slots than the context was created for */
    CC_ERR_HIP = -5        /* a HIP runtime call failed */
};

typedef struct cc_ctx cc_ctx;

/* Shape of the primary model's decoder layer and the capacity of the context. */
typedef struct cc_model_desc {
    int32_t d;         /* hidden width; multiple of 64, at most 16384 */
    int32_t H_q;       /* query heads */
    int32_t H_kv;      /* key/value heads; divides H_q, H_q / H_kv <= 32 */
    int32_t d_h;       /* head dim: 64 or 128 */
    int32_t f;         /* SwiGLU inner width; multiple of 64 */
    float rope_base;   /* rotary base: pair (j, j + d_h/2) turns by pos * base^(-2j/d_h) */
    float rms_eps;     /* RMSNorm epsilon */
    int32_t N_cap;     /* most cache slots (positions) any call will address */
    int32_t M_cap;     /* most rows any cc_recompute_layer call will recompute */
    int32_t T_cap;     /* most chunk tokens any cc_select call will score (<= 131072) */
} cc_model_desc;

/* One layer's slice of the global KV cache (Section 4.1: concatenated chunk
 * caches behind one copy of the shared prefix; slot j holds position j).
 * K and V are dev bf16; element (j, h, c) is at j*stride_token + h*stride_head + c
 * (strides in elements, c contiguous, stride_head % 8 == 0, stride_token % 8 == 0).
 * The rows listed in idx are overwritten; every other row is only read. */
typedef struct cc_kv_layer {
    void* K;
    void* V;
    int64_t stride_token;
    int64_t stride_head;
    int32_t N;             /* valid slots: idx values must be < N <= N_cap */
} cc_kv_layer;

/* One decoder layer's weights, all dev bf16, read-only. */
typedef struct cc_layer_weights {
    const void* w_in_norm;   /* [d]                     RMSNorm before attention */
    const void* w_qkv;       /* [(H_q+2H_kv)*d_h, d]    rows: all q heads, then k heads, then v heads */
    const void* b_qkv;       /* [(H_q+2H_kv)*d_h] or NULL */
    const void* w_o;         /* [d, H_q*d_h] */
    const void* w_post_norm; /* [d]                     RMSNorm before the MLP */
    const void* w_gate;      /* [f, d] */
    const void* w_up;        /* [f, d] */
    const void* w_down;      /* [d, f] */
} cc_layer_weights;

enum {
    CC_FLAG_NO_GROUPING = 1, /* cc_select: return the top-k candidates themselves (the paper's
                                "without grouping" ablation) */
    CC_FLAG_CHECK_IDX = 2    /* cc_recompute_layer / cc_step_*: verify idx (and gather_idx) on the
                                device first; this synchronises the stream */
};

/* Creates a context on the current HIP device: the rotary table for N_cap
 * positions and the scratch rows for M_cap recomputed tokens are allocated
 * here, once.  `hip_stream` is a hipStream_t (NULL = the default stream) on
 * which every later call enqueues.  The context owns only its own workspace. */
cc_status cc_create(cc_ctx** out, const cc_model_desc* desc, void* hip_stream);
cc_status cc_destroy(cc_ctx* ctx);
cc_status cc_set_stream(cc_ctx* ctx, void* hip_stream);
/* Text of the last error on this context (ctx == NULL: of the last failed cc_create or
 * context-free call on this thread). */
const char* cc_last_error(const cc_ctx* ctx);

/*
 * Token selection (Sections 4.2-4.3).
 *   attn   dev fp32 [Q_a, T], row stride ld (elements): the query->chunk block of the
 *          auxiliary model's last-layer attention (prefix and query columns already
 *          removed, heads already reduced).  Values must be finite and >= 0.
 *   score[t] = sum over the Q_a rows, added in fp32 in ascending row order.
 *   k = floor(T * recomp_bp / 10000) candidates = the k largest scores, equal
 *          scores going to the lower index.
 *   grouping: a window of `window` tokens (cut off at T) is looked at wherever its
 *          first token is a candidate; if it holds >= tau candidates all its tokens are
 *          chosen.  tau = 0 means ceil(5*window/8) (5 at the paper's window of 8).
 *   idx_out dev int32, capacity >= T + n_tail: receives idx_offset + t for every
 *          chosen t, ascending, then idx_offset + T .. idx_offset + T + n_tail - 1
 *          (the user-query slots, always recomputed).
 *   n_out  dev int32: number of entries written.
 *   n_out_host  host pointer or NULL: if given, the count is also copied there and
 *          the call waits for it (the one host synchronisation of a request).
 * Requires 1 <= T <= T_cap, Q_a >= 1, ld >= T, 1 <= window <= 1024,
 * 0 <= tau <= window, recomp_bp <= 10000.
 */
cc_status cc_select(cc_ctx* ctx, const float* attn, int32_t Q_a, int32_t T, int64_t ld,
                    uint32_t recomp_bp, int32_t window, int32_t tau, int32_t flags,
                    int32_t idx_offset, int32_t n_tail,
                    int32_t* idx_out, int32_t* n_out, int32_t* n_out_host);

/*
 * cc_select for callers that cannot allocate device memory or create a context: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as cc_select, except: no context (the work is enqueued on
 * `hip_stream`, a hipStream_t or NULL for the default stream, of the current device), no
 * host copy of the count, and the scores between the two kernels live in a static device
 * array inside the library (1 MiB per GPU, held until the process ends) instead of a
 * context's workspace.  T may be at most 131072; a larger T returns CC_ERR_WORKSPACE.
 * The call allocates and frees nothing and does not synchronise.  Every call on one GPU
 * uses that GPU's one array: calls that may overlap on a GPU (different streams, different
 * threads) race on it and must be serialised by the caller; calls on one stream are
 * ordered.  The error text of a failed call is read with cc_last_error(NULL).
 */
cc_status cc_select_noalloc(void* hip_stream, const float* attn, int32_t Q_a, int32_t T, int64_t ld,
                            uint32_t recomp_bp, int32_t window, int32_t tau, int32_t flags,
                            int32_t idx_offset, int32_t n_tail, int32_t* idx_out, int32_t* n_out);

/* One batch element of the auxiliary model's last-layer attention (Section 4.2:
 * the chunks are processed as `chunk c + query` in one batch): fp32 attention
 * weights with the query tokens as rows.  Element (head h, query row q, key
 * column col) is attn[h*stride_head + q*stride_row + col] (strides in elements,
 * device memory, read only).  The query -> chunk block is columns col0 ..
 * col0 + len - 1: whatever lies before it (a shared prefix) and behind it (the
 * query tokens themselves) is excluded, as the paper prescribes. */
typedef struct cc_aux_block {
    const float* attn;
    int64_t stride_head;
    int64_t stride_row;
    int32_t col0;
    int32_t len;            /* chunk tokens, >= 1 */
} cc_aux_block;

/* Importance scores from the batched attention tensors (Section 4.2; head average
 * as in Section 3, then the reduction over the query dimension):
 *   score[t0_c + j] = sum_q ( (sum_h attn_c[h][q][col0_c + j]) * (1/H) ),
 * t0_c = len_0 + ... + len_{c-1}; fp32, heads and rows added in ascending order
 * with one accumulator each (reproducible bit pattern).
 *   blocks  host array of n_blocks descriptors (read during the call only)
 *   H, Q_a  heads and query rows of every block, >= 1
 *   score   dev fp32 [sum of len]
 * Enqueues on the context's stream; no host synchronisation. */
cc_status cc_step_block_scores(cc_ctx* ctx, const cc_aux_block* blocks, int32_t n_blocks, int32_t H,
                               int32_t Q_a, float* score);

/* cc_select with the scores taken from the batched attention tensors
 * (cc_step_block_scores, T = sum of len <= T_cap) instead of a [Q_a, T] block.
 * Other arguments, outputs and errors as for cc_select. */
cc_status cc_select_blocks(cc_ctx* ctx, const cc_aux_block* blocks, int32_t n_blocks, int32_t H,
                           int32_t Q_a, uint32_t recomp_bp, int32_t window, int32_t tau,
                           int32_t flags, int32_t idx_offset, int32_t n_tail, int32_t* idx_out,
                           int32_t* n_out, int32_t* n_out_host);

/* First stage of cc_select on its own: score dev fp32 [T] (Section 4.2, reduction
 * over the query dimension). */
cc_status cc_step_column_scores(cc_ctx* ctx, const float* attn, int32_t Q_a, int32_t T,
                                int64_t ld, float* score);

/*
 * Selective recompute of one decoder layer (Section 4.3).
 *   hidden      dev bf16 [rows, d]: layer inputs.
 *   gather_idx  dev int32 [M] row of `hidden` for each recomputed token, or NULL when
 *               `hidden` is already the compact [M, d] output of the layer below.
 *   kv          this layer's cache; rows idx[i] of K and V are overwritten with the
 *               rotated key / value of token i (bf16, round to nearest even).
 *   idx         dev int32 [M], strictly ascending, each in [0, kv->N): the cache slot
 *               and, equally, the global position of token i.
 *   out         dev bf16 [M, d]: the layer output of the recomputed rows.
 * Row i attends, causally, over every slot j <= idx[i] of the updated cache
 * (stale rows, the shared prefix and every fresh row), grouped-query style: query
 * head h reads kv head h / (H_q/H_kv).  M = 0 is allowed and does nothing.
 */
cc_status cc_recompute_layer(cc_ctx* ctx, const void* hidden, int64_t rows,
                             const int32_t* gather_idx, const cc_kv_layer* kv,
                             const int32_t* idx, int32_t M, const cc_layer_weights* w,
                             void* out, int32_t flags);

/* ---- the stages of cc_recompute_layer, on caller buffers (all dev) ---- */

/* Gather + RMSNorm: xn[i] = bf16( x * rsqrt(mean(x^2)+eps) * w_norm ), x = hidden[gather_idx[i]]
 * (or hidden[i] when gather_idx is NULL).  xn bf16 [M, d]. */
cc_status cc_step_gather_rmsnorm(cc_ctx* ctx, const void* hidden, int64_t rows,
                                 const int32_t* gather_idx, int32_t M, const void* w_norm,
                                 void* xn);
/* QKV projection of xn [M, d], bias, rotary embedding of q and k at position idx[i],
 * q -> q_out bf16 [M, H_q*d_h], k and v -> rows idx[i] of the cache. */
cc_status cc_step_qkv_rope_scatter(cc_ctx* ctx, const void* xn, int32_t M, const int32_t* idx,
                                   const void* w_qkv, const void* b_qkv,
                                   const cc_kv_layer* kv, void* q_out, int32_t flags);
/* Sparse-query causal GQA attention: q bf16 [M, H_q*d_h] (already rotated) at
 * positions idx over cache slots 0..idx[i]; o bf16 [M, H_q*d_h]. */
cc_status cc_step_sparse_attention(cc_ctx* ctx, const void* q, int32_t M, const int32_t* idx,
                                   const cc_kv_layer* kv, void* o, int32_t flags);
/* y[i] = x[i] + W_o o[i], x gathered as above; y fp32 [M, d]. */
cc_status cc_step_oproj_residual(cc_ctx* ctx, const void* o, int32_t M, const void* w_o,
                                 const void* hidden, int64_t rows, const int32_t* gather_idx,
                                 float* y);
/* out[i] = bf16( y + W_down( silu(W_gate m) * (W_up m) ) ), m = RMSNorm(y; w_post_norm). */
cc_status cc_step_mlp(cc_ctx* ctx, const float* y, int32_t M, const void* w_post_norm,
                      const void* w_gate, const void* w_up, const void* w_down, void* out);

/*
 * Online cache assembly (Section 4.1): the per-chunk caches, each precomputed alone
 * behind the shared prefix at local positions 0 .. P+len-1, are concatenated into one
 * layer's global cache with a single copy of the prefix and re-numbered positions.
 *   chunks   host array of n_chunks descriptors (read during the call only).  K and V
 *            are dev bf16 [P + len, H_kv, d_h]; element (t, h, c) is at
 *            t*stride_token + h*stride_head + c (strides in elements, shared by all
 *            chunks, multiples of 8; pointers 16-byte aligned).
 *   dst rows 0 .. P-1               <- rows 0 .. P-1 of chunk 0 (K and V as stored)
 *   dst row  P + start_c + t        <- row P + t of chunk c, start_c = len_0 + .. + len_{c-1}:
 *            V copied; K turned by start_c more positions (pair (j, j + d_h/2) by the
 *            angle start_c * base^(-2j/d_h), fp32, rounded to bf16 nearest-even), which
 *            moves it from local position P + t to global position P + start_c + t.
 *   dst rows P + T .. P + T + n_tail - 1 (the user-query slots) <- zeros.
 * Requires P >= 0, every len >= 1, P + T + n_tail <= dst->N.  dst must not overlap a chunk.
 */
typedef struct cc_chunk_kv {
    const void* K;
    const void* V;
    int32_t len;
} cc_chunk_kv;
cc_status cc_assemble_cache(cc_ctx* ctx, const cc_chunk_kv* chunks, int32_t n_chunks, int32_t P,
                            int64_t stride_token, int64_t stride_head, int32_t n_tail,
                            const cc_kv_layer* dst);

/* ---- timing of the library's own kernels on its stream ---- */
enum {
    CC_K_COLSUM = 0, CC_K_SELECT, CC_K_GATHER_NORM, CC_K_QKV, CC_K_ATTN, CC_K_OPROJ,
    CC_K_POST_NORM, CC_K_GATE_UP, CC_K_DOWN, CC_K_ASSEMBLE, CC_K_COPY, CC_K_BLOCK_SCORES,
    CC_K_COUNT
};
/* While enabled, every kernel launch is bracketed by HIP events on the stream. */
cc_status cc_profile_enable(cc_ctx* ctx, int32_t on);
/* Synchronises the stream, then writes, per kernel kind, the summed duration in
 * milliseconds (ms[CC_K_COUNT], host) and the number of launches (count[CC_K_COUNT],
 * host) since the last read, and resets them. */
cc_status cc_profile_read(cc_ctx* ctx, float* ms, int32_t* count);

/* Measurement support, not a step of the method: copies `bytes` (a multiple of 16,
 * both pointers dev and 16-byte aligned, buffers not overlapping) with a plain
 * 16-bytes-per-lane kernel.  Hardware counters of HBM traffic (bytes fetched / written
 * per dispatch) are calibrated against this kernel, whose traffic is known: `bytes`
 * read and `bytes` written. */
cc_status cc_calib_copy(cc_ctx* ctx, void* dst, const void* src, int64_t bytes);

/*
 * Test support: overrides the launch shapes that the library otherwise picks from
 * the sizes of a call, so that a test can send the same inputs through every tile
 * shape and loop.  Every choice computes the same result up to the fp32 summation
 * order; a value that does not fit a call (a tile shape without a variant for the
 * call's K, more shares than K allows or the workspace holds) is ignored for that
 * call.  The override stays until the next cc_debug_set_launch on this context;
 * o == NULL restores the library's own choices.  All-zero fields mean "no override".
 */
typedef struct cc_launch_override {
    int32_t gemm_tile;    /* 0, or 'b' 256x256, 'm' 192x256, 'h' 256x128, 's' 128x128 */
    int32_t gemm_staged;  /* 1: the two-stage K loop (64 columns per stage) instead of the ring */
    int32_t gemm_mfma32;  /* 1: the ring loop with 32x32x16 MFMAs instead of 16x16x32 */
    int32_t gemm_gm;      /* > 0: row tiles per band of the XCD-aware tile order */
    int32_t gemm_splitk;  /* > 0: shares of K (1 = never split) */
    int32_t attn_splits;  /* > 0: key splits of the attention launch (1 = never split) */
} cc_launch_override;
cc_status cc_debug_set_launch(cc_ctx* ctx, const cc_launch_override* o);

#ifdef __cplusplus
}
#endif
#endif /* CACHECLIP_H */
