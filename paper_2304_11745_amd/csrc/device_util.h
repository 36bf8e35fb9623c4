// Small device helpers shared by the streaming kernels (element conversion, activations).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include "kernels.h"

// every kernel of the library is enqueued through this macro (see LaunchTimer in kernels.h)
#define GACER_LAUNCH(kernel, grid, block, shmem, stream, ...)                                                                \
    do {                                                                                                                     \
        if (gacer::launch_timer)                                                                                             \
            hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, gacer::launch_timer->start, gacer::launch_timer->stop, \
                                  0, __VA_ARGS__);                                                                           \
        else                                                                                                                 \
            hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                                             \
    } while (0)

namespace gacer {

// Division of an index by a run-time extent d that the launcher knows: the launcher prepares (mul, shift) with
// n / d == (n * mul) >> (32 + shift) for every 0 <= n < 2^31 -- mul = ceil(2^(31 + c) / d), c = ceil(log2 d), shift = c - 1;
// the error term n * (mul * d - 2^(31+c)) stays below 2^(31+c) because n < 2^31 <= 2^(31+c) / d -- and the kernel spends
// one multiply-high and a shift instead of the dozens of instructions of a division.  d = 1 is marked by mul = 0.
inline void divisor(int d, unsigned (&out)[2])
{
    if (d <= 1) { out[0] = 0u; out[1] = 0u; return; }
    int c = 0;
    while ((1ll << c) < d) ++c;
    const unsigned long long two_k = 1ull << (31 + c);
    out[0] = (unsigned)((two_k + (unsigned long long)d - 1) / (unsigned long long)d);
    out[1] = (unsigned)(c - 1);
}
__device__ __forceinline__ int div_by(int n, const unsigned (&d)[2])
{
    return d[0] ? (int)(__umulhi((unsigned)n, d[0]) >> d[1]) : n;
}

__device__ __forceinline__ float ld_f32(const float *p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld_f32(const unsigned short *p, int64_t i) { return __uint_as_float(((unsigned)p[i]) << 16); }

__device__ __forceinline__ unsigned short to_bf16(float f)      // round to nearest even (hardware conversion)
{
    return __builtin_bit_cast(unsigned short, (__bf16)f);
}
__device__ __forceinline__ void st_f32(float *p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_f32(unsigned short *p, int64_t i, float v) { p[i] = to_bf16(v); }

// hard-sigmoid min(max(v + 3, 0), 6) / 6, and hard-swish = v times that (act is ACT_HSIGMOID or ACT_HSWISH).  The sixth is a
// multiplication by the rounded constant: four instructions, small enough to sit in every unrolled epilogue (a correctly
// rounded division is a dozen more per element, and kernels that never take this branch still pay for fetching around it).
__device__ __forceinline__ float hard_act(float v, int act)
{
    asm volatile("");                           // keeps the (launch-uniform) branch around this a branch: as selects, every element of every kernel would pay for it
    const float s = __fmul_rn(__builtin_amdgcn_fmed3f(__fadd_rn(v, 3.f), 0.f, 6.f), 0.16666667163372039794921875f);
    return act == ACT_HSWISH ? __fmul_rn(v, s) : s;
}

__device__ __forceinline__ float activate(float v, int act)
{
    if (act == ACT_RELU) return __builtin_fmaxf(v, 0.f);
    if (act == ACT_RELU6) return __builtin_amdgcn_fmed3f(v, 0.f, 6.f);
    if (act == ACT_GELU) return __fmul_rn(__fmul_rn(0.5f, v), __fadd_rn(1.f, erff(__fmul_rn(v, 0.70710678118654752440f))));
    if (act == ACT_HSWISH || act == ACT_HSIGMOID) return hard_act(v, act);
    return v;
}

// Activation of N values at once: `act` is uniform over the launch, so one branch is taken per group of values instead of
// one per value (per value, the compiler threads every element through its own run of scalar branches).
template <int N> __device__ __forceinline__ void activate_n(float *v, int act)
{
    if (act == ACT_RELU) {
#pragma unroll
        for (int q = 0; q < N; ++q) v[q] = __builtin_fmaxf(v[q], 0.f);
    } else if (act == ACT_RELU6) {
#pragma unroll
        for (int q = 0; q < N; ++q) v[q] = __builtin_amdgcn_fmed3f(v[q], 0.f, 6.f);
    } else if (act != ACT_NONE) {
#pragma unroll
        for (int q = 0; q < N; ++q) v[q] = activate(v[q], act);
    }
}

// 16-byte vector of V elements of type T, unpacked to / packed from float.
template <typename T, int V> struct Vec;
template <> struct Vec<float, 4> {
    float4 raw;
    __device__ __forceinline__ float get(int i) const { return i == 0 ? raw.x : i == 1 ? raw.y : i == 2 ? raw.z : raw.w; }
    __device__ __forceinline__ void set(int i, float v) { if (i == 0) raw.x = v; else if (i == 1) raw.y = v; else if (i == 2) raw.z = v; else raw.w = v; }
};
template <> struct Vec<unsigned short, 8> {
    uint4 raw;
    __device__ __forceinline__ float get(int i) const
    {
        const unsigned wd = (i >> 1) == 0 ? raw.x : (i >> 1) == 1 ? raw.y : (i >> 1) == 2 ? raw.z : raw.w;
        return __uint_as_float((i & 1) ? (wd & 0xFFFF0000u) : (wd << 16));
    }
    __device__ __forceinline__ void set(int i, float v)
    {
        const unsigned b = to_bf16(v);
        unsigned &wd = (i >> 1) == 0 ? raw.x : (i >> 1) == 1 ? raw.y : (i >> 1) == 2 ? raw.z : raw.w;
        wd = (i & 1) ? ((wd & 0x0000FFFFu) | (b << 16)) : ((wd & 0xFFFF0000u) | b);
    }
};
template <> struct Vec<float, 1> {
    float raw;
    __device__ __forceinline__ float get(int) const { return raw; }
    __device__ __forceinline__ void set(int, float v) { raw = v; }
};
template <> struct Vec<unsigned short, 1> {
    unsigned short raw;
    __device__ __forceinline__ float get(int) const { return __uint_as_float(((unsigned)raw) << 16); }
    __device__ __forceinline__ void set(int, float v) { raw = to_bf16(v); }
};

template <typename T, int V> __device__ __forceinline__ Vec<T, V> ld_vec(const T *p, int64_t i)
{
    Vec<T, V> v;
    v.raw = *(const decltype(v.raw) *)(p + i);
    return v;
}
template <typename T, int V> __device__ __forceinline__ void st_vec(T *p, int64_t i, const Vec<T, V> &v)
{
    *(decltype(v.raw) *)(p + i) = v.raw;
}


// Buffer descriptors let every global load be unconditional: a masked element gets an offset beyond the
// descriptor's range and the hardware returns zero (zero padding of the image border, of the K tail and of
// ragged tile edges), so the main loop has no branches and loads can stay in flight across MFMA blocks.
typedef int i32x4 __attribute__((ext_vector_type(4)));
static constexpr unsigned OOB = 0x80000000u;     // tensors are smaller than 2 GiB (checked when tenants load)

// The descriptor must live in scalar registers: its inputs are wave-uniform by construction, which
// readfirstlane makes visible to the compiler (integer divisions are otherwise computed per lane).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, int64_t bytes)
{
    int rec = bytes > 0x7FFFFFFF ? 0x7FFFFFFF : (bytes < 0 ? 0 : (int)bytes);
    rec = __builtin_amdgcn_readfirstlane(rec);
    const uint64_t u = (uint64_t)p;
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)u);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(u >> 32));
    return __builtin_amdgcn_make_buffer_rsrc((void *)(((uint64_t)hi << 32) | lo), 0, rec, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned off)
{
    const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    return make_uint4((unsigned)v.x, (unsigned)v.y, (unsigned)v.z, (unsigned)v.w);
}
__device__ __forceinline__ uint2 buf_load8(__amdgpu_buffer_rsrc_t r, unsigned off)
{
    typedef int i32x2 __attribute__((ext_vector_type(2)));
    const i32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
    return make_uint2((unsigned)v.x, (unsigned)v.y);
}
template <typename T> __device__ __forceinline__ T buf_load1(__amdgpu_buffer_rsrc_t r, unsigned off);
template <> __device__ __forceinline__ float buf_load1<float>(__amdgpu_buffer_rsrc_t r, unsigned off)
{
    return __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
}
template <> __device__ __forceinline__ unsigned short buf_load1<unsigned short>(__amdgpu_buffer_rsrc_t r, unsigned off)
{
    return (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)off, 0, 0);
}

}  // namespace gacer
