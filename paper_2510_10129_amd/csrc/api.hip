// C ABI of the library: argument checks, workspace, stream and kernel timing.
// Every compute step runs in the HIP kernels of this directory.
#include <math.h>
#include <algorithm>
#include <mutex>
#include <string.h>

#include "cc_internal.h"

// Scratch of cc_select_noalloc: the importance scores between its two kernels live here
// instead of in a context's workspace.  One copy per GPU, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; the device address it yields (one
// per device) is what kernels, copies and fills are given.
#define CC_NOALLOC_T_MAX 131072
#define CC_NOALLOC_SCRATCH_BYTES (1u << 20)       // scores [T_MAX] fp32 in the first half; the rest is spare
static __device__ __align__(256) unsigned char scratch[CC_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local std::string g_create_err;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};            // device address of `scratch` on each device

// Device address of the scratch array on the current device, resolved once per device with
// that device current.
hipError_t scratch_on_current_device(void** out, int* dev_out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    if (dev_out) *dev_out = dev;
    return hipSuccess;
}

cc_status fail(cc_ctx* c, cc_status code, const std::string& msg) {
    if (c) c->err = msg; else g_create_err = msg;
    return code;
}

#define CC_HIP(c, call)                                                                       \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail((c), CC_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

cc_status check_model(const cc_model_desc& m, std::string* why) {
    auto bad = [&](const char* s) { *why = s; return CC_ERR_SHAPE; };
    if (m.d < 64 || m.d % 64 || m.d > 16384) return bad("d must be a multiple of 64 in [64, 16384]");
    if (m.f < 64 || m.f % 64) return bad("f must be a positive multiple of 64");
    if (m.d_h != 64 && m.d_h != 128) return bad("d_h must be 64 or 128");
    if (m.H_q < 1 || m.H_kv < 1 || m.H_q % m.H_kv) return bad("H_kv must divide H_q");
    if (m.H_q / m.H_kv > 32) return bad("H_q / H_kv must be <= 32");
    if (!(m.rope_base > 1.0f)) return bad("rope_base must be > 1");
    if (!(m.rms_eps >= 0.0f)) return bad("rms_eps must be >= 0");
    if (m.N_cap < 1 || m.M_cap < 1 || m.T_cap < 1) return bad("capacities must be >= 1");
    if (m.T_cap > 131072) return bad("T_cap must be <= 131072");
    return CC_OK;
}

cc_status check_kv(cc_ctx* c, const cc_kv_layer* kv) {
    if (!kv || !kv->K || !kv->V) return fail(c, CC_ERR_NULL, "kv, kv->K and kv->V must not be NULL");
    if (kv->N < 1 || kv->N > c->m.N_cap)
        return fail(c, CC_ERR_WORKSPACE, "kv->N must be in [1, N_cap]");
    if (kv->stride_head < c->m.d_h || kv->stride_head % 8 ||
        kv->stride_token < (int64_t)c->m.d_h * c->m.H_kv || kv->stride_token % 8)
        return fail(c, CC_ERR_SHAPE, "kv strides must be multiples of 8 and cover [H_kv, d_h]");
    if (!aligned16(kv->K) || !aligned16(kv->V))
        return fail(c, CC_ERR_SHAPE, "kv->K and kv->V must be 16-byte aligned");
    return CC_OK;
}

cc_status check_rows(cc_ctx* c, int32_t M) {
    if (M < 0) return fail(c, CC_ERR_SHAPE, "M must be >= 0");
    if (M > c->m.M_cap) return fail(c, CC_ERR_WORKSPACE, "M exceeds M_cap");
    return CC_OK;
}

// Optional device-side check of idx / gather_idx; synchronises the stream.
cc_status check_idx_sync(cc_ctx* c, const int32_t* idx, int M, int hi, int strict, const char* what) {
    if (M <= 0 || !idx) return CC_OK;
    CC_HIP(c, hipMemsetAsync(c->flag, 0, sizeof(int32_t), c->stream));
    cc_launch_check_idx(idx, M, 0, hi, strict, c->flag, c->stream);
    CC_HIP(c, hipMemcpyAsync(c->pinned, c->flag, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    CC_HIP(c, hipStreamSynchronize(c->stream));
    if (c->pinned[0] != 0)
        return fail(c, CC_ERR_IDX, std::string(what) + (strict ? " must be strictly ascending and in range"
                                                                : " must be in range"));
    return CC_OK;
}

}  // namespace

cc_prof_scope::cc_prof_scope(cc_ctx* ctx, int kind) : c(ctx), on(ctx->prof) {
    if (!on) return;
    if (c->pool.empty()) {
        cc_event_pair np;
        if (hipEventCreate(&np.a) != hipSuccess || hipEventCreate(&np.b) != hipSuccess) {
            on = false;
            return;
        }
        p = np;
    } else {
        p = c->pool.back();
        c->pool.pop_back();
    }
    p.kind = kind;
    (void)hipEventRecord(p.a, c->stream);
}

cc_prof_scope::~cc_prof_scope() {
    if (!on) return;
    (void)hipEventRecord(p.b, c->stream);
    c->used.push_back(p);
}

extern "C" {

const char* cc_last_error(const cc_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

cc_status cc_create(cc_ctx** out, const cc_model_desc* desc, void* hip_stream) {
    if (!out || !desc) return fail(nullptr, CC_ERR_NULL, "out and desc must not be NULL");
    *out = nullptr;
    std::string why;
    if (check_model(*desc, &why) != CC_OK) return fail(nullptr, CC_ERR_SHAPE, why);
    cc_ctx* c = new cc_ctx();
    c->m = *desc;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->prof = false;
    memset(&c->ovr, 0, sizeof(c->ovr));
    memset(c->prof_ms, 0, sizeof(c->prof_ms));
    memset(c->prof_n, 0, sizeof(c->prof_n));
    c->rope = nullptr; c->xn = nullptr; c->q = nullptr; c->o = nullptr; c->y = nullptr;
    c->mn = nullptr; c->act = nullptr; c->attn_part = nullptr; c->gemm_part = nullptr; c->score = nullptr; c->n_sel = nullptr; c->flag = nullptr;
    c->pinned = nullptr;
    const cc_model_desc& m = c->m;
    const size_t Mc = (size_t)m.M_cap, nq = (size_t)m.H_q * m.d_h;
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) {
        // resolves the scratch of cc_select_noalloc on this device now, so that a later call
        // from a region that must not touch the runtime's loader (graph capture) finds it
        void* sp = nullptr;
        e = scratch_on_current_device(&sp, nullptr);
    }
    auto alloc = [&](void** p, size_t bytes) {
        if (e == hipSuccess) e = hipMalloc(p, bytes);
    };
    alloc((void**)&c->rope, (size_t)m.N_cap * (m.d_h / 2) * sizeof(float2));
    alloc((void**)&c->xn, Mc * m.d * 2);
    alloc((void**)&c->q, Mc * nq * 2);
    alloc((void**)&c->o, Mc * nq * 2);
    alloc((void**)&c->y, Mc * m.d * 4);
    alloc((void**)&c->mn, Mc * m.d * 2);
    alloc((void**)&c->act, Mc * m.f * 2);
    // room for up to 8 key splits of the attention while the launch is small enough to want them
    c->attn_part_rows = (int64_t)std::min<size_t>(Mc * m.H_q * 8, 196608);
    alloc((void**)&c->attn_part, (size_t)c->attn_part_rows * (m.d_h + 4) * 4);
    // shares of a split-K projection: up to 8 x [M_cap][widest padded output], at most 128 MB
    {
        const size_t widest = std::max<size_t>(std::max<size_t>((size_t)m.d, nq + 2 * (size_t)m.H_kv * m.d_h), 2 * (size_t)m.f);
        c->gemm_part_floats = (int64_t)std::min<size_t>(8 * Mc * ((widest + 255) / 256 * 256), (size_t)32 << 20);
    }
    alloc((void**)&c->gemm_part, (size_t)c->gemm_part_floats * 4);
    alloc((void**)&c->score, (size_t)m.T_cap * 4);
    alloc((void**)&c->n_sel, 4);
    alloc((void**)&c->flag, 4);
    if (e == hipSuccess) e = hipHostMalloc((void**)&c->pinned, 2 * sizeof(int32_t), hipHostMallocDefault);
    if (e != hipSuccess) {
        std::string msg = std::string("workspace allocation: ") + hipGetErrorString(e);
        cc_destroy(c);
        return fail(nullptr, CC_ERR_HIP, msg);
    }
    cc_launch_rope_table(c->rope, m.N_cap, m.d_h, (double)m.rope_base, c->stream);
    e = hipGetLastError();
    if (e != hipSuccess) {
        std::string msg = std::string("rope table launch: ") + hipGetErrorString(e);
        cc_destroy(c);
        return fail(nullptr, CC_ERR_HIP, msg);
    }
    *out = c;
    return CC_OK;
}

cc_status cc_destroy(cc_ctx* c) {
    if (!c) return CC_OK;
    (void)hipStreamSynchronize(c->stream);
    for (auto& p : c->used) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    for (auto& p : c->pool) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
    (void)hipFree(c->rope); (void)hipFree(c->xn); (void)hipFree(c->q); (void)hipFree(c->o);
    (void)hipFree(c->y); (void)hipFree(c->mn); (void)hipFree(c->act); (void)hipFree(c->attn_part); (void)hipFree(c->gemm_part);
    (void)hipFree(c->score);
    (void)hipFree(c->n_sel); (void)hipFree(c->flag);
    if (c->pinned) (void)hipHostFree(c->pinned);
    delete c;
    return CC_OK;
}

cc_status cc_set_stream(cc_ctx* c, void* hip_stream) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    c->stream = static_cast<hipStream_t>(hip_stream);
    return CC_OK;
}

cc_status cc_step_column_scores(cc_ctx* c, const float* attn, int32_t Q_a, int32_t T, int64_t ld,
                                float* score) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!attn || !score) return fail(c, CC_ERR_NULL, "attn and score must not be NULL");
    if (Q_a < 1 || T < 1 || ld < T) return fail(c, CC_ERR_SHAPE, "need Q_a >= 1, T >= 1, ld >= T");
    {
        cc_prof_scope ps(c, CC_K_COLSUM);
        cc_launch_colsum(attn, Q_a, T, ld, score, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

// Validates the descriptors, enqueues the block-score launches (CC_BLK_SEGS batch elements
// each) and returns the number of scores in *T_out.
static cc_status block_scores(cc_ctx* c, const cc_aux_block* blocks, int32_t n_blocks, int32_t H,
                              int32_t Q_a, int64_t T_max, float* score, int32_t* T_out) {
    if (!blocks || !score) return fail(c, CC_ERR_NULL, "blocks and score must not be NULL");
    if (n_blocks < 1 || H < 1 || Q_a < 1) return fail(c, CC_ERR_SHAPE, "need n_blocks >= 1, H >= 1, Q_a >= 1");
    int64_t T = 0;
    for (int i = 0; i < n_blocks; ++i) {
        const cc_aux_block& b = blocks[i];
        if (!b.attn) return fail(c, CC_ERR_NULL, "a block's attn must not be NULL");
        if (b.len < 1 || b.col0 < 0 || b.stride_row < (int64_t)b.col0 + b.len ||
            b.stride_head < (int64_t)(Q_a - 1) * b.stride_row + b.col0 + b.len)
            return fail(c, CC_ERR_SHAPE, "a block needs len >= 1, col0 >= 0, stride_row >= col0 + len and non-overlapping heads");
        T += b.len;
        if (T > T_max) return fail(c, T_max == (int64_t)c->m.T_cap ? CC_ERR_WORKSPACE : CC_ERR_SHAPE, "sum of len exceeds the score capacity");
    }
    int32_t t0 = 0;
    for (int i0 = 0; i0 < n_blocks; i0 += CC_BLK_SEGS) {
        cc_blk_args a;
        a.n_seg = std::min<int>(CC_BLK_SEGS, n_blocks - i0);
        a.n_blocks = 0;
        for (int i = 0; i < a.n_seg; ++i) {
            const cc_aux_block& b = blocks[i0 + i];
            a.seg[i] = cc_blk_seg{b.attn, b.stride_head, b.stride_row, b.col0, b.len, t0, a.n_blocks};
            a.n_blocks += (b.len + 63) / 64;
            t0 += b.len;
        }
        cc_prof_scope ps(c, CC_K_BLOCK_SCORES);
        cc_launch_block_scores(a, H, Q_a, score, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    *T_out = (int32_t)T;
    return CC_OK;
}

cc_status cc_step_block_scores(cc_ctx* c, const cc_aux_block* blocks, int32_t n_blocks, int32_t H,
                               int32_t Q_a, float* score) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    int32_t T = 0;
    return block_scores(c, blocks, n_blocks, H, Q_a, INT32_MAX, score, &T);
}

cc_status cc_select_blocks(cc_ctx* c, const cc_aux_block* blocks, int32_t n_blocks, int32_t H,
                           int32_t Q_a, uint32_t recomp_bp, int32_t window, int32_t tau,
                           int32_t flags, int32_t idx_offset, int32_t n_tail, int32_t* idx_out,
                           int32_t* n_out, int32_t* n_out_host) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!idx_out || !n_out) return fail(c, CC_ERR_NULL, "idx_out and n_out must not be NULL");
    if (recomp_bp > 10000u) return fail(c, CC_ERR_SHAPE, "recomp_bp must be <= 10000");
    if (window < 1 || window > 1024) return fail(c, CC_ERR_SHAPE, "window must be in [1, 1024]");
    if (tau < 0 || tau > window) return fail(c, CC_ERR_SHAPE, "tau must be in [0, window]");
    if (n_tail < 0 || idx_offset < 0) return fail(c, CC_ERR_SHAPE, "idx_offset and n_tail must be >= 0");
    int32_t T = 0;
    cc_status st = block_scores(c, blocks, n_blocks, H, Q_a, c->m.T_cap, c->score, &T);
    if (st != CC_OK) return st;
    const int k = (int)(((int64_t)T * (int64_t)recomp_bp) / 10000);
    const int tau_eff = tau > 0 ? tau : (5 * window + 7) / 8;
    {
        cc_prof_scope ps(c, CC_K_SELECT);
        cc_launch_select(c->score, T, k, window, tau_eff, (flags & CC_FLAG_NO_GROUPING) ? 0 : 1,
                         idx_offset, n_tail, idx_out, n_out, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    if (n_out_host) {
        CC_HIP(c, hipMemcpyAsync(c->pinned + 1, n_out, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        CC_HIP(c, hipStreamSynchronize(c->stream));
        *n_out_host = c->pinned[1];
    }
    return CC_OK;
}

cc_status cc_select(cc_ctx* c, const float* attn, int32_t Q_a, int32_t T, int64_t ld,
                    uint32_t recomp_bp, int32_t window, int32_t tau, int32_t flags,
                    int32_t idx_offset, int32_t n_tail, int32_t* idx_out, int32_t* n_out,
                    int32_t* n_out_host) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!attn || !idx_out || !n_out) return fail(c, CC_ERR_NULL, "attn, idx_out and n_out must not be NULL");
    if (Q_a < 1 || T < 1 || ld < T) return fail(c, CC_ERR_SHAPE, "need Q_a >= 1, T >= 1, ld >= T");
    if (T > c->m.T_cap) return fail(c, CC_ERR_WORKSPACE, "T exceeds T_cap");
    if (recomp_bp > 10000u) return fail(c, CC_ERR_SHAPE, "recomp_bp must be <= 10000");
    if (window < 1 || window > 1024) return fail(c, CC_ERR_SHAPE, "window must be in [1, 1024]");
    if (tau < 0 || tau > window) return fail(c, CC_ERR_SHAPE, "tau must be in [0, window]");
    if (n_tail < 0 || idx_offset < 0) return fail(c, CC_ERR_SHAPE, "idx_offset and n_tail must be >= 0");
    const int k = (int)(((int64_t)T * (int64_t)recomp_bp) / 10000);
    const int tau_eff = tau > 0 ? tau : (5 * window + 7) / 8;
    {
        cc_prof_scope ps(c, CC_K_COLSUM);
        cc_launch_colsum(attn, Q_a, T, ld, c->score, c->stream);
    }
    {
        cc_prof_scope ps(c, CC_K_SELECT);
        cc_launch_select(c->score, T, k, window, tau_eff, (flags & CC_FLAG_NO_GROUPING) ? 0 : 1,
                         idx_offset, n_tail, idx_out, n_out, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    if (n_out_host) {
        CC_HIP(c, hipMemcpyAsync(c->pinned + 1, n_out, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        CC_HIP(c, hipStreamSynchronize(c->stream));
        *n_out_host = c->pinned[1];
    }
    return CC_OK;
}

cc_status cc_select_noalloc(void* hip_stream, const float* attn, int32_t Q_a, int32_t T, int64_t ld,
                            uint32_t recomp_bp, int32_t window, int32_t tau, int32_t flags,
                            int32_t idx_offset, int32_t n_tail, int32_t* idx_out, int32_t* n_out) {
    if (!attn || !idx_out || !n_out) return fail(nullptr, CC_ERR_NULL, "attn, idx_out and n_out must not be NULL");
    if (Q_a < 1 || T < 1 || ld < T) return fail(nullptr, CC_ERR_SHAPE, "need Q_a >= 1, T >= 1, ld >= T");
    if (T > CC_NOALLOC_T_MAX)
        return fail(nullptr, CC_ERR_WORKSPACE, "T exceeds 131072, the most chunk tokens the static scratch holds scores for");
    if (recomp_bp > 10000u) return fail(nullptr, CC_ERR_SHAPE, "recomp_bp must be <= 10000");
    if (window < 1 || window > 1024) return fail(nullptr, CC_ERR_SHAPE, "window must be in [1, 1024]");
    if (tau < 0 || tau > window) return fail(nullptr, CC_ERR_SHAPE, "tau must be in [0, window]");
    if (n_tail < 0 || idx_offset < 0) return fail(nullptr, CC_ERR_SHAPE, "idx_offset and n_tail must be >= 0");
    void* sp = nullptr;
    hipError_t e = scratch_on_current_device(&sp, nullptr);
    if (e != hipSuccess)
        return fail(nullptr, CC_ERR_HIP, std::string("address of the static scratch: ") + hipGetErrorString(e));
    float* score = static_cast<float*>(sp);           // [T]: every entry below T is written before it is read
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int k = (int)(((int64_t)T * (int64_t)recomp_bp) / 10000);
    const int tau_eff = tau > 0 ? tau : (5 * window + 7) / 8;
    cc_launch_colsum(attn, Q_a, T, ld, score, stream);
    cc_launch_select(score, T, k, window, tau_eff, (flags & CC_FLAG_NO_GROUPING) ? 0 : 1, idx_offset, n_tail,
                     idx_out, n_out, stream);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(nullptr, CC_ERR_HIP, std::string("launch: ") + hipGetErrorString(e));
    return CC_OK;
}

cc_status cc_step_gather_rmsnorm(cc_ctx* c, const void* hidden, int64_t rows,
                                 const int32_t* gather_idx, int32_t M, const void* w_norm, void* xn) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!hidden || !w_norm || !xn) return fail(c, CC_ERR_NULL, "hidden, w_norm and xn must not be NULL");
    if (M < 0 || rows < 1 || (!gather_idx && rows < M)) return fail(c, CC_ERR_SHAPE, "bad M / rows");
    if (!aligned16(hidden) || !aligned16(w_norm) || !aligned16(xn))
        return fail(c, CC_ERR_SHAPE, "buffers must be 16-byte aligned");
    {
        cc_prof_scope ps(c, CC_K_GATHER_NORM);
        cc_launch_gather_rmsnorm((const bf16_t*)hidden, gather_idx, M, c->m.d, (const bf16_t*)w_norm,
                                 c->m.rms_eps, (bf16_t*)xn, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

cc_status cc_step_qkv_rope_scatter(cc_ctx* c, const void* xn, int32_t M, const int32_t* idx,
                                   const void* w_qkv, const void* b_qkv, const cc_kv_layer* kv,
                                   void* q_out, int32_t flags) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!xn || !idx || !w_qkv || !q_out) return fail(c, CC_ERR_NULL, "xn, idx, w_qkv and q_out must not be NULL");
    cc_status st = check_kv(c, kv);
    if (st != CC_OK) return st;
    if (M < 0) return fail(c, CC_ERR_SHAPE, "M must be >= 0");
    if (!aligned16(xn) || !aligned16(w_qkv) || !aligned16(q_out) || (b_qkv && !aligned16(b_qkv)))
        return fail(c, CC_ERR_SHAPE, "buffers must be 16-byte aligned");
    if (flags & CC_FLAG_CHECK_IDX) {
        st = check_idx_sync(c, idx, M, kv->N, 1, "idx");
        if (st != CC_OK) return st;
    }
    {
        cc_prof_scope ps(c, CC_K_QKV);
        cc_launch_qkv((const bf16_t*)xn, M, idx, (const bf16_t*)w_qkv, (const bf16_t*)b_qkv, c->m,
                      c->rope, *kv, (bf16_t*)q_out, c->gemm_part, c->gemm_part_floats, c->ovr, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

cc_status cc_step_sparse_attention(cc_ctx* c, const void* q, int32_t M, const int32_t* idx,
                                   const cc_kv_layer* kv, void* o, int32_t flags) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!q || !idx || !o) return fail(c, CC_ERR_NULL, "q, idx and o must not be NULL");
    cc_status st = check_kv(c, kv);
    if (st != CC_OK) return st;
    if (M < 0) return fail(c, CC_ERR_SHAPE, "M must be >= 0");
    if (!aligned16(q) || !aligned16(o)) return fail(c, CC_ERR_SHAPE, "buffers must be 16-byte aligned");
    if (flags & CC_FLAG_CHECK_IDX) {
        st = check_idx_sync(c, idx, M, kv->N, 1, "idx");
        if (st != CC_OK) return st;
    }
    {
        cc_prof_scope ps(c, CC_K_ATTN);
        cc_launch_attention((const bf16_t*)q, M, idx, c->m, *kv, (bf16_t*)o, c->attn_part, c->attn_part_rows, c->ovr, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

cc_status cc_step_oproj_residual(cc_ctx* c, const void* o, int32_t M, const void* w_o,
                                 const void* hidden, int64_t rows, const int32_t* gather_idx, float* y) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!o || !w_o || !hidden || !y) return fail(c, CC_ERR_NULL, "o, w_o, hidden and y must not be NULL");
    if (M < 0 || rows < 1 || (!gather_idx && rows < M)) return fail(c, CC_ERR_SHAPE, "bad M / rows");
    if (!aligned16(o) || !aligned16(w_o) || !aligned16(hidden) || !aligned16(y))
        return fail(c, CC_ERR_SHAPE, "buffers must be 16-byte aligned");
    {
        cc_prof_scope ps(c, CC_K_OPROJ);
        cc_launch_oproj((const bf16_t*)o, M, (const bf16_t*)w_o, (const bf16_t*)hidden, gather_idx,
                        c->m, y, c->gemm_part, c->gemm_part_floats, c->ovr, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

cc_status cc_step_mlp(cc_ctx* c, const float* y, int32_t M, const void* w_post_norm,
                      const void* w_gate, const void* w_up, const void* w_down, void* out) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!y || !w_post_norm || !w_gate || !w_up || !w_down || !out)
        return fail(c, CC_ERR_NULL, "y, weights and out must not be NULL");
    cc_status st = check_rows(c, M);
    if (st != CC_OK) return st;
    if (!aligned16(y) || !aligned16(w_post_norm) || !aligned16(w_gate) || !aligned16(w_up) ||
        !aligned16(w_down) || !aligned16(out))
        return fail(c, CC_ERR_SHAPE, "buffers must be 16-byte aligned");
    {
        cc_prof_scope ps(c, CC_K_POST_NORM);
        cc_launch_rmsnorm_f32(y, M, c->m.d, (const bf16_t*)w_post_norm, c->m.rms_eps, c->mn, c->stream);
    }
    {
        cc_prof_scope ps(c, CC_K_GATE_UP);
        cc_launch_gate_up(c->mn, M, (const bf16_t*)w_gate, (const bf16_t*)w_up, c->m, c->act, c->gemm_part,
                          c->gemm_part_floats, c->ovr, c->stream);
    }
    {
        cc_prof_scope ps(c, CC_K_DOWN);
        cc_launch_down(c->act, M, (const bf16_t*)w_down, y, c->m, (bf16_t*)out, c->gemm_part, c->gemm_part_floats,
                       c->ovr, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

cc_status cc_recompute_layer(cc_ctx* c, const void* hidden, int64_t rows, const int32_t* gather_idx,
                             const cc_kv_layer* kv, const int32_t* idx, int32_t M,
                             const cc_layer_weights* w, void* out, int32_t flags) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!hidden || !idx || !w || !out) return fail(c, CC_ERR_NULL, "hidden, idx, w and out must not be NULL");
    if (!w->w_in_norm || !w->w_qkv || !w->w_o || !w->w_post_norm || !w->w_gate || !w->w_up || !w->w_down)
        return fail(c, CC_ERR_NULL, "every weight pointer except b_qkv must be set");
    cc_status st = check_kv(c, kv);
    if (st != CC_OK) return st;
    st = check_rows(c, M);
    if (st != CC_OK) return st;
    if (M > kv->N) return fail(c, CC_ERR_SHAPE, "M exceeds the number of cache slots");
    if (rows < 1 || (!gather_idx && rows < M)) return fail(c, CC_ERR_SHAPE, "hidden has fewer rows than M");
    if (M == 0) return CC_OK;
    if (flags & CC_FLAG_CHECK_IDX) {
        st = check_idx_sync(c, idx, M, kv->N, 1, "idx");
        if (st != CC_OK) return st;
        if (gather_idx) {
            int hi = rows > 0x7fffffff ? 0x7fffffff : (int)rows;
            st = check_idx_sync(c, gather_idx, M, hi, 0, "gather_idx");
            if (st != CC_OK) return st;
        }
    }
    st = cc_step_gather_rmsnorm(c, hidden, rows, gather_idx, M, w->w_in_norm, c->xn);
    if (st != CC_OK) return st;
    st = cc_step_qkv_rope_scatter(c, c->xn, M, idx, w->w_qkv, w->b_qkv, kv, c->q, 0);
    if (st != CC_OK) return st;
    st = cc_step_sparse_attention(c, c->q, M, idx, kv, c->o, 0);
    if (st != CC_OK) return st;
    st = cc_step_oproj_residual(c, c->o, M, w->w_o, hidden, rows, gather_idx, c->y);
    if (st != CC_OK) return st;
    return cc_step_mlp(c, c->y, M, w->w_post_norm, w->w_gate, w->w_up, w->w_down, out);
}

cc_status cc_assemble_cache(cc_ctx* c, const cc_chunk_kv* chunks, int32_t n_chunks, int32_t P,
                            int64_t stride_token, int64_t stride_head, int32_t n_tail,
                            const cc_kv_layer* dst) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!chunks) return fail(c, CC_ERR_NULL, "chunks must not be NULL");
    cc_status st = check_kv(c, dst);
    if (st != CC_OK) return st;
    if (n_chunks < 1 || P < 0 || n_tail < 0) return fail(c, CC_ERR_SHAPE, "need n_chunks >= 1, P >= 0, n_tail >= 0");
    if (stride_head < c->m.d_h || stride_head % 8 || stride_token < (int64_t)c->m.d_h * c->m.H_kv ||
        stride_token % 8)
        return fail(c, CC_ERR_SHAPE, "chunk strides must be multiples of 8 and cover [H_kv, d_h]");
    int64_t T = 0;
    for (int i = 0; i < n_chunks; ++i) {
        if (!chunks[i].K || !chunks[i].V) return fail(c, CC_ERR_NULL, "chunk K and V must not be NULL");
        if (chunks[i].len < 1) return fail(c, CC_ERR_SHAPE, "every chunk length must be >= 1");
        if (!aligned16(chunks[i].K) || !aligned16(chunks[i].V))
            return fail(c, CC_ERR_SHAPE, "chunk K and V must be 16-byte aligned");
        T += chunks[i].len;
    }
    if ((int64_t)P + T + n_tail > dst->N) return fail(c, CC_ERR_SHAPE, "P + T + n_tail exceeds dst->N");
    // segments: the prefix (from chunk 0), every chunk's own rows, the zeroed tail
    std::vector<cc_asm_seg> segs;
    auto blocks_of = [](int len) { return (len + CC_ASM_ROWS - 1) / CC_ASM_ROWS; };
    if (P > 0) segs.push_back({(const bf16_t*)chunks[0].K, (const bf16_t*)chunks[0].V, 0, P, 0, 0});
    int32_t start = 0;
    for (int i = 0; i < n_chunks; ++i) {
        segs.push_back({(const bf16_t*)chunks[i].K + (int64_t)P * stride_token,
                        (const bf16_t*)chunks[i].V + (int64_t)P * stride_token, P + start, chunks[i].len,
                        start, 0});
        start += chunks[i].len;
    }
    if (n_tail > 0) segs.push_back({nullptr, nullptr, P + start, n_tail, 0, 0});
    {
        cc_prof_scope ps(c, CC_K_ASSEMBLE);
        for (size_t s0 = 0; s0 < segs.size(); s0 += CC_ASM_SEGS) {
            cc_asm_args a;
            a.n_seg = (int32_t)std::min<size_t>(CC_ASM_SEGS, segs.size() - s0);
            int32_t nb = 0;
            for (int i = 0; i < a.n_seg; ++i) {
                a.seg[i] = segs[s0 + i];
                a.seg[i].blk0 = nb;
                nb += blocks_of(a.seg[i].len);
            }
            for (int i = a.n_seg; i < CC_ASM_SEGS; ++i) a.seg[i] = {nullptr, nullptr, 0, 0, 0, nb};
            a.n_blocks = nb;
            cc_launch_assemble(a, c->rope, c->m, stride_token, stride_head, *dst, c->stream);
        }
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

cc_status cc_calib_copy(cc_ctx* c, void* dst, const void* src, int64_t bytes) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!dst || !src) return fail(c, CC_ERR_NULL, "dst and src must not be NULL");
    if (bytes < 0 || bytes % 16 || !aligned16(dst) || !aligned16(src))
        return fail(c, CC_ERR_SHAPE, "bytes must be a non-negative multiple of 16, pointers 16-byte aligned");
    {
        cc_prof_scope ps(c, CC_K_COPY);
        cc_launch_copy(dst, src, bytes, c->stream);
    }
    CC_HIP(c, hipGetLastError());
    return CC_OK;
}

cc_status cc_debug_set_launch(cc_ctx* c, const cc_launch_override* o) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!o) {
        memset(&c->ovr, 0, sizeof(c->ovr));
        return CC_OK;
    }
    const int t = o->gemm_tile;
    if (t != 0 && t != 'b' && t != 'm' && t != 'h' && t != 's')
        return fail(c, CC_ERR_SHAPE, "gemm_tile must be 0, 'b', 'm', 'h' or 's'");
    if (o->gemm_gm < 0 || o->gemm_splitk < 0 || o->gemm_splitk > 16 || o->attn_splits < 0 || o->attn_splits > 64)
        return fail(c, CC_ERR_SHAPE, "override values must be >= 0, gemm_splitk <= 16, attn_splits <= 64");
    c->ovr = *o;
    return CC_OK;
}

cc_status cc_profile_enable(cc_ctx* c, int32_t on) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    c->prof = on != 0;
    return CC_OK;
}

cc_status cc_profile_read(cc_ctx* c, float* ms, int32_t* count) {
    if (!c) return fail(nullptr, CC_ERR_NULL, "ctx must not be NULL");
    if (!ms || !count) return fail(c, CC_ERR_NULL, "ms and count must not be NULL");
    CC_HIP(c, hipStreamSynchronize(c->stream));
    for (auto& p : c->used) {
        float t = 0.0f;
        if (hipEventElapsedTime(&t, p.a, p.b) == hipSuccess) {
            c->prof_ms[p.kind] += t;
            c->prof_n[p.kind] += 1;
        }
        c->pool.push_back(p);
    }
    c->used.clear();
    for (int i = 0; i < CC_K_COUNT; ++i) {
        ms[i] = c->prof_ms[i];
        count[i] = c->prof_n[i];
        c->prof_ms[i] = 0.0f;
        c->prof_n[i] = 0;
    }
    return CC_OK;
}

}  // extern "C"
