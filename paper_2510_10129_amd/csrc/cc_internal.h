// Internal declarations shared by the HIP translation units of the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "cacheclip.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct cc_event_pair {
    hipEvent_t a, b;
    int kind;
};

struct cc_ctx {
    cc_model_desc m;
    hipStream_t stream;
    int device;
    std::string err;

    // workspace (device)
    float2* rope;      // [N_cap][d_h/2] (cos, sin)
    bf16_t* xn;        // [M_cap][d]          normalised layer input
    bf16_t* q;         // [M_cap][H_q*d_h]    rotated queries
    bf16_t* o;         // [M_cap][H_q*d_h]    attention output
    float* y;          // [M_cap][d]          residual stream after attention
    bf16_t* mn;        // [M_cap][d]          normalised MLP input
    bf16_t* act;       // [M_cap][f]          silu(gate)*up
    float* attn_part;  // [attn_part_rows][d_h + 4]  partial results of a key-split attention launch
    int64_t attn_part_rows;
    float* gemm_part;  // [gemm_part_floats]  fp32 shares of a split-K projection
    int64_t gemm_part_floats;
    float* score;      // [T_cap]
    int32_t* n_sel;    // [1]
    int32_t* flag;     // [1] idx check result
    int32_t* pinned;   // host pinned [2]
    cc_launch_override ovr;   // test overrides of the launch shapes (all zero: none)

    // profiling
    bool prof;
    std::vector<cc_event_pair> used;
    std::vector<cc_event_pair> pool;
    float prof_ms[CC_K_COUNT];
    int32_t prof_n[CC_K_COUNT];
};

// Brackets one kernel launch with events when profiling is on.
struct cc_prof_scope {
    cc_ctx* c;
    cc_event_pair p;
    bool on;
    cc_prof_scope(cc_ctx* ctx, int kind);
    ~cc_prof_scope();
};

// ---- kernel launchers (each only enqueues on `s`) ----
// The projections take a workspace `ws` of `ws_floats` floats (may be NULL) for split-K launches.
// One launch of the assembly kernel covers up to CC_ASM_SEGS source segments.
#define CC_ASM_SEGS 64
#define CC_ASM_ROWS 16      // destination rows per wave
struct cc_asm_seg {
    const bf16_t* K;        // first source row (NULL: write zeros)
    const bf16_t* V;
    int32_t dst;            // first destination row
    int32_t len;            // rows
    int32_t delta;          // positions to turn the keys by
    int32_t blk0;           // first wave-block of this segment within the launch
};
struct cc_asm_args {
    cc_asm_seg seg[CC_ASM_SEGS];
    int32_t n_seg, n_blocks;
};
void cc_launch_assemble(const cc_asm_args& a, const float2* rope, const cc_model_desc& m,
                        int64_t src_st, int64_t src_sh, const cc_kv_layer& dst, hipStream_t s);
// One launch of the block-score kernel covers up to CC_BLK_SEGS batch elements.
#define CC_BLK_SEGS 64
struct cc_blk_seg {
    const float* attn;      // element (h, q, col) at attn[h*stride_head + q*stride_row + col]
    int64_t stride_head, stride_row;
    int32_t col0, len;      // query -> chunk block: columns col0 .. col0 + len - 1
    int32_t t0;             // first score it produces
    int32_t blk0;           // first workgroup (64 columns each) of this element within the launch
};
struct cc_blk_args {
    cc_blk_seg seg[CC_BLK_SEGS];
    int32_t n_seg, n_blocks;
};
void cc_launch_block_scores(const cc_blk_args& a, int H, int Q_a, float* score, hipStream_t s);
void cc_launch_copy(void* dst, const void* src, int64_t bytes, hipStream_t s);
void cc_launch_rope_table(float2* table, int n_pos, int d_h, double base, hipStream_t s);
void cc_launch_colsum(const float* attn, int Q_a, int T, int64_t ld, float* score, hipStream_t s);
void cc_launch_select(const float* score, int T, int k, int window, int tau, int grouping,
                      int idx_offset, int n_tail, int32_t* idx_out, int32_t* n_out, hipStream_t s);
void cc_launch_check_idx(const int32_t* idx, int M, int lo, int hi, int strict, int32_t* flag,
                         hipStream_t s);
void cc_launch_gather_rmsnorm(const bf16_t* hidden, const int32_t* gather_idx, int M, int d,
                              const bf16_t* w, float eps, bf16_t* xn, hipStream_t s);
void cc_launch_rmsnorm_f32(const float* y, int M, int d, const bf16_t* w, float eps, bf16_t* out,
                           hipStream_t s);
void cc_launch_qkv(const bf16_t* xn, int M, const int32_t* idx, const bf16_t* w_qkv,
                   const bf16_t* b_qkv, const cc_model_desc& m, const float2* rope,
                   const cc_kv_layer& kv, bf16_t* q_out, float* ws, int64_t ws_floats,
                   const cc_launch_override& ovr, hipStream_t s);
// `part` ([part_rows][d_h + 4] fp32, may be NULL) lets a launch with few workgroups split the keys.
void cc_launch_attention(const bf16_t* q, int M, const int32_t* idx, const cc_model_desc& m,
                         const cc_kv_layer& kv, bf16_t* o, float* part, int64_t part_rows,
                         const cc_launch_override& ovr, hipStream_t s);
void cc_launch_oproj(const bf16_t* o, int M, const bf16_t* w_o, const bf16_t* hidden,
                     const int32_t* gather_idx, const cc_model_desc& m, float* y, float* ws,
                     int64_t ws_floats, const cc_launch_override& ovr, hipStream_t s);
void cc_launch_gate_up(const bf16_t* mn, int M, const bf16_t* w_gate, const bf16_t* w_up,
                       const cc_model_desc& m, bf16_t* act, float* ws, int64_t ws_floats,
                       const cc_launch_override& ovr, hipStream_t s);
void cc_launch_down(const bf16_t* act, int M, const bf16_t* w_down, const float* y,
                    const cc_model_desc& m, bf16_t* out, float* ws, int64_t ws_floats,
                    const cc_launch_override& ovr, hipStream_t s);
