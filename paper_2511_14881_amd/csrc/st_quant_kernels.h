// Publish-time int8 quantisation with one global scale (Sec. 4.2): global min / max over the whole
// embedding table, s = max(|min|, |max|) / 127 (1 for an all-zero table), q = round-half-even(x / s)
// kept inside [-127, 127].  Zero maps to zero, so inner products of quantised rows need no offset
// terms, and every row's scale is s.
//
// Two passes over the table, both bound by HBM: the min / max reduction reads 4 bytes per value,
// the second pass reads them again and writes 1 byte per value (9 bytes per value in all).
#pragma once
#include "st_device.h"

namespace st {

// Order-preserving map of a float onto unsigned integers (for atomicMin / atomicMax).
__device__ inline uint32_t float_order(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float order_float(uint32_t u)
{
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u);
}

// mm[0] = running minimum, mm[1] = running maximum, both in the ordered encoding.
__global__ void quant_init_kernel(uint32_t* mm)
{
    if (threadIdx.x == 0) {
        mm[0] = 0xFFFFFFFFu;
        mm[1] = 0u;
    }
}

constexpr int kQuantThreads = 256;

// x is 16-byte aligned; n values.  Grid-stride over float4, the last n % 4 values by thread 0 of
// workgroup 0; one pair of atomics per workgroup.
__global__ __launch_bounds__(kQuantThreads) void quant_minmax_kernel(const float* __restrict__ x, int64_t n,
                                                                      uint32_t* __restrict__ mm)
{
    __shared__ float s_mn[kQuantThreads / 64], s_mx[kQuantThreads / 64];
    const int tid = threadIdx.x;
    float mn = __builtin_inff(), mx = -__builtin_inff();
    const int64_t n4 = n >> 2;
    const float4* x4 = reinterpret_cast<const float4*>(x);
    for (int64_t i = (int64_t)blockIdx.x * kQuantThreads + tid; i < n4; i += (int64_t)gridDim.x * kQuantThreads) {
        const float4 v = x4[i];
        mn = fminf(fminf(mn, v.x), fminf(fminf(v.y, v.z), v.w));
        mx = fmaxf(fmaxf(mx, v.x), fmaxf(fmaxf(v.y, v.z), v.w));
    }
    if (blockIdx.x == 0 && tid == 0)
        for (int64_t i = n4 << 2; i < n; ++i) {
            mn = fminf(mn, x[i]);
            mx = fmaxf(mx, x[i]);
        }
    for (int o = 32; o > 0; o >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
    }
    if ((tid & 63) == 0) {
        s_mn[tid >> 6] = mn;
        s_mx[tid >> 6] = mx;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kQuantThreads / 64; ++w) {
            mn = fminf(mn, s_mn[w]);
            mx = fmaxf(mx, s_mx[w]);
        }
        if (mn <= mx) {  // this workgroup saw at least one value
            atomicMin(&mm[0], float_order(mn));
            atomicMax(&mm[1], float_order(mx));
        }
    }
}

__device__ inline int quant_one(float x, float s)
{
    float v = rintf(__fdiv_rn(x, s));  // ties to even
    v = fminf(fmaxf(v, -127.0f), 127.0f);
    return (int)v;
}

// Second pass: 16 values per thread and step (four float4 loads, one 16-byte store); the tail of
// n % 16 values by workgroup 0.  Also writes the row scales and decodes min / max for the caller.
__global__ __launch_bounds__(kQuantThreads) void quant_apply_kernel(const float* __restrict__ x, int64_t n,
                                                                     int64_t n_rows, const uint32_t* __restrict__ mm,
                                                                     int8_t* __restrict__ q, float* __restrict__ row_scale,
                                                                     float* __restrict__ minmax_out)
{
    const int tid = threadIdx.x;
    float mn = 0.0f, mx = 0.0f;
    if (n > 0) {
        mn = order_float(mm[0]);
        mx = order_float(mm[1]);
    }
    const float a = fmaxf(fabsf(mn), fabsf(mx));
    const float s = a > 0.0f ? __fdiv_rn(a, 127.0f) : 1.0f;
    const int64_t gtid = (int64_t)blockIdx.x * kQuantThreads + tid, gsize = (int64_t)gridDim.x * kQuantThreads;
    const int64_t n16 = n >> 4;
    const float4* x4 = reinterpret_cast<const float4*>(x);
    int4* q16 = reinterpret_cast<int4*>(q);
    for (int64_t i = gtid; i < n16; i += gsize) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = x4[i * 4 + u];
        int w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            w[u] = (quant_one(v[u].x, s) & 255) | ((quant_one(v[u].y, s) & 255) << 8) |
                   ((quant_one(v[u].z, s) & 255) << 16) | ((quant_one(v[u].w, s) & 255) << 24);
        q16[i] = make_int4(w[0], w[1], w[2], w[3]);
    }
    if (blockIdx.x == 0)
        for (int64_t i = (n16 << 4) + tid; i < n; i += kQuantThreads) q[i] = (int8_t)quant_one(x[i], s);
    for (int64_t r = gtid; r < n_rows; r += gsize) row_scale[r] = s;
    if (gtid == 0) {
        minmax_out[0] = mn;
        minmax_out[1] = mx;
    }
}

// Plain streaming read for bandwidth measurements: every thread reads 16-byte pieces a whole
// grid apart (four in flight per step) and folds them into one word, so that nothing but the
// loads remains; one word per workgroup is written.  The measured rate of this kernel is the
// practical ceiling the HBM-bound kernels of the library are compared with.
constexpr int kStreamThreads = 256;
__global__ __launch_bounds__(kStreamThreads) void stream_read_kernel(const int4* __restrict__ src, int64_t n16,
                                                                     uint32_t* __restrict__ sink)
{
    const int64_t stride = (int64_t)gridDim.x * kStreamThreads;
    int64_t i = (int64_t)blockIdx.x * kStreamThreads + threadIdx.x;
    int acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const int4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const int4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o);
    __shared__ int s_part[kStreamThreads / 64];
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int v = 0;
        for (int w = 0; w < kStreamThreads / 64; ++w) v ^= s_part[w];
        sink[blockIdx.x] = (uint32_t)v;
    }
}

}  // namespace st
