// Device-side helpers shared by the kernel files of the GRAWA update (gfx950, wave64): bf16
// widening, wave and block reductions in fp64, global-memory accessors with wave-uniform row
// bases, gradient loads by dtype and vector width, and the launch-side choice between streaming
// and cached accesses.
#pragma once
#include <hip/hip_ext.h>

#include "grawa_internal.h"

#define GRAWA_BLOCK 256
#define GRAWA_WAVE 64
#define GRAWA_CELL 256 // columns per block of the one-column-per-lane passes

// ---------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_one(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Move a double between lanes with a DPP control word (both 32-bit halves).
template <int CTRL> __device__ __forceinline__ double dpp_move_f64(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes of a wave; every lane gets the total.  Within a row of 16 lanes:
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror; across the four
// rows: two butterfly exchanges.
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_move_f64<0xB1>(v);  // lane ^ 1
    v += dpp_move_f64<0x4E>(v);  // lane ^ 2
    v += dpp_move_f64<0x141>(v); // other quad of the half row
    v += dpp_move_f64<0x140>(v); // other half of the row
    v += __shfl_xor(v, 16, GRAWA_WAVE);
    v += __shfl_xor(v, 32, GRAWA_WAVE);
    return v;
}

__device__ __forceinline__ double wave_min(double v)
{
    for (int m = 1; m < GRAWA_WAVE; m <<= 1) v = fmin(v, __shfl_xor(v, m, GRAWA_WAVE));
    return v;
}

// Sum over a 256-thread block through LDS; every thread gets the result.  `sm` holds one
// double per wave.
__device__ __forceinline__ double block_sum(double v, double *sm)
{
    v = wave_sum(v);
    const int w = threadIdx.x / GRAWA_WAVE;
    __syncthreads();
    if ((threadIdx.x & (GRAWA_WAVE - 1)) == 0) sm[w] = v;
    __syncthreads();
    double t = 0.0;
    for (int i = 0; i < GRAWA_BLOCK / GRAWA_WAVE; ++i) t += sm[i];
    return t;
}

typedef float v2f __attribute__((ext_vector_type(2)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Global-memory accessors for the one-element-per-lane kernels.  An address is a wave-uniform
// 64-bit base plus a 32-bit lane byte offset; the base is pinned in a scalar register pair so
// that the access is issued in that form instead of with a 64-bit address computed per lane.
// NT = streaming (non-temporal) access.
#define GRAWA_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ uint64_t uniform_base(const void *p)
{
    uint64_t a = reinterpret_cast<uint64_t>(p);
    asm volatile("" : "+s"(a));
    return a;
}
// A float read through the scalar unit from memory this kernel never writes.
__device__ __forceinline__ float ld_uniform_f32(uint64_t base, int64_t index)
{
    return ((const __attribute__((address_space(4))) float *)base)[index];
}
template <bool NT, typename T> __device__ __forceinline__ T ld_lane(uint64_t base, unsigned byte_off)
{
    const GRAWA_GLOBAL T *p = (const GRAWA_GLOBAL T *)(base + byte_off);
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT, typename T> __device__ __forceinline__ void st_lane(uint64_t base, unsigned byte_off, T v)
{
    GRAWA_GLOBAL T *p = (GRAWA_GLOBAL T *)(base + byte_off);
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// acc + v^2 with the value widened first: one fp64 fused multiply-add.
__device__ __forceinline__ double sq_add(float v, double acc)
{
    const double d = (double)v;
    return fma(d, d, acc);
}

// Gradient element access.  VEC8 = elements per 8-byte load (norm pass).
template <typename GT> struct Grad;

template <> struct Grad<float> {
    static constexpr int VEC8 = 2;
    static __device__ __forceinline__ float one(const float *p) { return *p; }
    template <bool NT> static __device__ __forceinline__ float lane(uint64_t base, unsigned off)
    {
        return ld_lane<NT, float>(base, off);
    }
    // 8 bytes (2 floats) at p, 8-byte aligned, streaming load; and their squares added to acc.
    // The square of a widened fp32 (or bf16) value is exact in fp64, so no gradient magnitude
    // that the input type can hold underflows or overflows here.
    typedef v2f Vec8;
    static __device__ __forceinline__ Vec8 load8(const float *p)
    {
        return __builtin_nontemporal_load(reinterpret_cast<const v2f *>(p));
    }
    static __device__ __forceinline__ double sumsq8(Vec8 q, double acc)
    {
        acc = sq_add(q.x, acc);
        acc = sq_add(q.y, acc);
        return acc;
    }
};

template <> struct Grad<uint16_t> { // bfloat16 bit patterns
    static constexpr int VEC8 = 4;
    static __device__ __forceinline__ float one(const uint16_t *p) { return bf16_one(*p); }
    template <bool NT> static __device__ __forceinline__ float lane(uint64_t base, unsigned off)
    {
        return bf16_one(ld_lane<NT, uint16_t>(base, off));
    }
    // 8 bytes (4 bf16) at p, 8-byte aligned, streaming load; and their squares added to acc
    typedef v2u Vec8;
    static __device__ __forceinline__ Vec8 load8(const uint16_t *p)
    {
        return __builtin_nontemporal_load(reinterpret_cast<const v2u *>(p));
    }
    static __device__ __forceinline__ double sumsq8(Vec8 q, double acc)
    {
        acc = sq_add(bf16_lo(q.x), acc);
        acc = sq_add(bf16_hi(q.x), acc);
        acc = sq_add(bf16_lo(q.y), acc);
        acc = sq_add(bf16_hi(q.y), acc);
        return acc;
    }
};

// V gradient elements (V * sizeof(GT) = 4 or 8 bytes, naturally aligned) widened to float.
template <typename GT, int V, bool NT> struct GradVec;
template <bool NT> struct GradVec<float, 1, NT> {
    static __device__ __forceinline__ void load(const float *p, float (&f)[1]) { f[0] = NT ? __builtin_nontemporal_load(p) : *p; }
};
template <bool NT> struct GradVec<float, 4, NT> {
    static __device__ __forceinline__ void load(const float *p, float (&f)[4])
    {
        typedef float v4f __attribute__((ext_vector_type(4)));
        const v4f *q = reinterpret_cast<const v4f *>(p);
        const v4f w = NT ? __builtin_nontemporal_load(q) : *q;
        f[0] = w.x;
        f[1] = w.y;
        f[2] = w.z;
        f[3] = w.w;
    }
};
template <bool NT> struct GradVec<uint16_t, 2, NT> {
    static __device__ __forceinline__ void load(const uint16_t *p, float (&f)[2])
    {
        const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
        const uint32_t w = NT ? __builtin_nontemporal_load(q) : *q;
        f[0] = bf16_lo(w);
        f[1] = bf16_hi(w);
    }
};
template <bool NT> struct GradVec<uint16_t, 4, NT> {
    static __device__ __forceinline__ void load(const uint16_t *p, float (&f)[4])
    {
        const v2u *q = reinterpret_cast<const v2u *>(p);
        const v2u w = NT ? __builtin_nontemporal_load(q) : *q;
        f[0] = bf16_lo(w.x);
        f[1] = bf16_hi(w.x);
        f[2] = bf16_lo(w.y);
        f[3] = bf16_hi(w.y);
    }
};
template <int V> struct FloatVec { typedef float T __attribute__((ext_vector_type(V))); };
template <> struct FloatVec<1> { typedef float T; };
template <int V> __device__ __forceinline__ float vec_get(const typename FloatVec<V>::T &v, int c)
{
    if constexpr (V == 1) return v;
    else return v[c];
}
template <int V> __device__ __forceinline__ void vec_set(typename FloatVec<V>::T &v, int c, float f)
{
    if constexpr (V == 1) v = f;
    else v[c] = f;
}

#define GRAWA_STREAMING_MIN_BYTES ((int64_t)512 << 20)

// Streaming accesses are used only when no cache line is shared between two rows or written
// in two parts: base pointers and row pitches are multiples of 128 bytes.
static inline bool rows_line_aligned(const void *base, int64_t ld, int elem_bytes)
{
    return (reinterpret_cast<uintptr_t>(base) % 128u) == 0 && ((ld * elem_bytes) % 128) == 0;
}
