// Row-wise HBM-bound kernels: gather + RMSNorm of the selected hidden rows,
// RMSNorm of the fp32 residual stream, and the rotary table.
#include "cc_internal.h"

__device__ __forceinline__ float block_sum_256(float v, float* red) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float t = red[0] + red[1] + red[2] + red[3];
    __syncthreads();
    return t;
}

// One workgroup per recomputed token: reads row gather_idx[i] of `hidden`
// (16 bytes per lane, whole 128-byte lines per 8 lanes), reduces the mean
// square in fp32, and writes the normalised bf16 row.  The second sweep over
// the row is served from cache.
__global__ __launch_bounds__(256) void gather_rmsnorm_kernel(
    const bf16_t* __restrict__ hidden, const int32_t* __restrict__ gather_idx, int d,
    const bf16_t* __restrict__ w, float eps, bf16_t* __restrict__ xn) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    const int64_t src = gather_idx ? (int64_t)gather_idx[i] : (int64_t)i;
    const bf16x8* row = reinterpret_cast<const bf16x8*>(hidden + src * d);
    const bf16x8* wv = reinterpret_cast<const bf16x8*>(w);
    bf16x8* dst = reinterpret_cast<bf16x8*>(xn + (int64_t)i * d);
    const int nchunk = d >> 3;
    float ss = 0.0f;
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        bf16x8 v = row[c];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            float f = (float)v[u];
            ss += f * f;
        }
    }
    float tot = block_sum_256(ss, red);
    float r = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        bf16x8 v = row[c], g = wv[c], o;
#pragma unroll
        for (int u = 0; u < 8; ++u) o[u] = (bf16_t)((float)v[u] * r * (float)g[u]);
        dst[c] = o;
    }
}

void cc_launch_gather_rmsnorm(const bf16_t* hidden, const int32_t* gather_idx, int M, int d,
                              const bf16_t* w, float eps, bf16_t* xn, hipStream_t s) {
    if (M <= 0) return;
    hipLaunchKernelGGL(gather_rmsnorm_kernel, dim3(M), dim3(256), 0, s, hidden, gather_idx, d, w,
                       eps, xn);
}

// RMSNorm of the fp32 residual rows y [M, d] -> bf16.
__global__ __launch_bounds__(256) void rmsnorm_f32_kernel(const float* __restrict__ y, int d,
                                                          const bf16_t* __restrict__ w, float eps,
                                                          bf16_t* __restrict__ out) {
    __shared__ float red[4];
    const int i = blockIdx.x;
    const f32x4* row = reinterpret_cast<const f32x4*>(y + (int64_t)i * d);
    const bf16x4* wv = reinterpret_cast<const bf16x4*>(w);
    bf16x4* dst = reinterpret_cast<bf16x4*>(out + (int64_t)i * d);
    const int nchunk = d >> 2;
    float ss = 0.0f;
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        f32x4 v = row[c];
        ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
    float tot = block_sum_256(ss, red);
    float r = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        f32x4 v = row[c];
        bf16x4 g = wv[c], o;
#pragma unroll
        for (int u = 0; u < 4; ++u) o[u] = (bf16_t)(v[u] * r * (float)g[u]);
        dst[c] = o;
    }
}

void cc_launch_rmsnorm_f32(const float* y, int M, int d, const bf16_t* w, float eps, bf16_t* out,
                           hipStream_t s) {
    if (M <= 0) return;
    hipLaunchKernelGGL(rmsnorm_f32_kernel, dim3(M), dim3(256), 0, s, y, d, w, eps, out);
}

// Rotary table: entry (p, j) = (cos, sin) of p * base^(-2j/d_h), evaluated in
// fp64 and stored as fp32.
__global__ void rope_table_kernel(float2* __restrict__ table, int n_pos, int half, double log2_base) {
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (int64_t)n_pos * half) return;
    int p = (int)(e / half), j = (int)(e % half);
    double inv = exp2(-(double)j / (double)half * log2_base);   // base^(-2j/d_h), d_h = 2*half
    double ang = (double)p * inv;
    table[e] = make_float2((float)cos(ang), (float)sin(ang));
}

void cc_launch_rope_table(float2* table, int n_pos, int d_h, double base, hipStream_t s) {
    int half = d_h / 2;
    int64_t n = (int64_t)n_pos * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, table,
                       n_pos, half, log2(base));
}
