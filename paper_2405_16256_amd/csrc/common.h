// Shared device helpers for the gfx950 kernels: storage types, bf16 rounding,
// buffer resources, wave reductions.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <stdint.h>

namespace hh {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(2 * sizeof(int)))) int i32x2;

constexpr int WAVE = 64;

// ---- bf16 <-> fp32 (round to nearest even; inputs here are finite) ----------
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// two floats -> packed pair of bf16 (lo in bits 0..15): one v_cvt_pk_bf16_f32, round to nearest even
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
    const f32x2 v = {lo, hi};
    const bf16x2 b = __builtin_convertvector(v, bf16x2);
    uint32_t u;
    __builtin_memcpy(&u, &b, 4);
    return u;
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack_bf2(f, 0.f) & 0xFFFFu); }
__device__ __forceinline__ float lo_bf(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float hi_bf(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }

// ---- 16-byte vectors of the storage type, widened to float -----------------
template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int N = 4;
    typedef float4 Raw;
    __device__ static __forceinline__ Raw raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
    __device__ static __forceinline__ void widen(const Raw& v, float* f) { f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w; }
    __device__ static __forceinline__ void load(const float* p, float* f) { widen(raw(p), f); }
    __device__ static __forceinline__ void store(float* p, const float* f) {
        *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
    }
};
template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    typedef uint4 Raw;
    __device__ static __forceinline__ Raw raw(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
    __device__ static __forceinline__ void widen(const Raw& v, float* f) {
        f[0] = lo_bf(v.x); f[1] = hi_bf(v.x); f[2] = lo_bf(v.y); f[3] = hi_bf(v.y);
        f[4] = lo_bf(v.z); f[5] = hi_bf(v.z); f[6] = lo_bf(v.w); f[7] = hi_bf(v.w);
    }
    __device__ static __forceinline__ void load(const bf16_t* p, float* f) { widen(raw(p), f); }
    __device__ static __forceinline__ void store(bf16_t* p, const float* f) {
        uint4 v;
        v.x = pack_bf2(f[0], f[1]); v.y = pack_bf2(f[2], f[3]);
        v.z = pack_bf2(f[4], f[5]); v.w = pack_bf2(f[6], f[7]);
        *reinterpret_cast<uint4*>(p) = v;
    }
};

// ---- buffer resources: out-of-range loads return 0, stores are dropped ------
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// ---- dynamic LDS above the 48 KB default -------------------------------------
// The limit is an attribute of the (kernel, device) pair.  `done` is the calling launcher's own record (one
// bit per device, one record per kernel instantiation) of where it has been raised already.
inline hipError_t allow_lds(const void* kern, int bytes, std::atomic<uint64_t>& done) {
    if (bytes <= 48 * 1024) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_relaxed) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_relaxed);
    return e;
}

// ---- wave / block reductions -----------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}
// sum over a workgroup of NW waves; `red` is NW floats of LDS; all threads get the result
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();  // protects `red` from a previous use
    if ((threadIdx.x & (WAVE - 1)) == 0) red[threadIdx.x / WAVE] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NW; i++) s += red[i];
    return s;
}

}  // namespace hh
