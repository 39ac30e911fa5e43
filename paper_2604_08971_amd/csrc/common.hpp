// Shared host/device helpers of the gfx950 library (not used by the CPU oracle).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "sentryfuse.h"

namespace sf {

// ---- error reporting -------------------------------------------------------
char *err_buf();                       // thread-local, 512 bytes
int32_t fail(int32_t code, const char *fmt, ...);
int32_t check_launch(const char *what);   // wraps hipGetLastError()

// ---- optional per-kernel timing (measurement aid, off by default) -----------
// While a kernel class is being profiled, every launch of that class is
// bracketed by a pair of HIP events on the launch stream.
struct ProfScope {
    ProfScope(int kernel_class, hipStream_t st);
    ~ProfScope();
    int slot;
    hipStream_t st;
};

// ---- descriptor ------------------------------------------------------------
struct Dims {
    int B, L, d, Hq, Hk, dh, F, nl, P, dtype, act, U, ffn_pad, n_sample;
    unsigned flags;
    float eps;
};
// Validates the descriptor; returns SF_OK and fills `out`.
int32_t read_desc(const sf_desc *desc, Dims &out);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t elem_size(int dtype) { return dtype == SF_BF16 ? 2 : 4; }

// Bump allocator over the caller's workspace.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <class T> T *take(size_t n) {
        size_t o = off;
        off = align_up(off + n * sizeof(T), 256);
        return base ? reinterpret_cast<T *>(base + o) : nullptr;
    }
};

// ---- device helpers ----------------------------------------------------------
// The 16-bit storage and matrix-core type of this build of the library: bfloat16 (libsentryfuse.so, dtype SF_BF16)
// or, compiled with -DSF_HALF_F16, IEEE binary16 (libsentryfuse_f16.so, dtype SF_F16) - the same kernels and entry
// points; both convert from fp32 with round-to-nearest-even and accumulate in fp32.
#ifdef SF_HALF_F16
typedef _Float16 h16;
#define SF_MFMA16 __builtin_amdgcn_mfma_f32_32x32x16_f16
#define SF_FDOT2 __builtin_amdgcn_fdot2
#define SF_DTYPE_16 SF_F16
#define SF_DTYPE_16_OTHER SF_BF16
#else
typedef __bf16 h16;
#define SF_MFMA16 __builtin_amdgcn_mfma_f32_32x32x16_bf16
#define SF_FDOT2 __builtin_amdgcn_fdot2_f32_bf16
#define SF_DTYPE_16 SF_BF16
#define SF_DTYPE_16_OTHER SF_F16
#endif
typedef __attribute__((ext_vector_type(8))) h16 h16x8;
typedef __attribute__((ext_vector_type(4))) h16 h16x4;
typedef __attribute__((ext_vector_type(2))) h16 h16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(h16 x) { return (float)x; }
template <class T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ h16 from_f32<h16>(float x) { return (h16)x; }   // RNE

// Two fp32 values -> two 16-bit values in one register (a in the low half), round to nearest even
__device__ __forceinline__ uint32_t pack2_h16(float a, float b)
{
#ifdef SF_HALF_F16
    const h16x2 v = {(h16)a, (h16)b};
    return __builtin_bit_cast(uint32_t, v);
#else
    // written out: the compiler converts the elements one by one and merges them with a byte permute
    uint32_t r;
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
#endif
}

// Order-preserving map of fp32 to uint32 (larger float <=> larger key).
__device__ __forceinline__ uint32_t sortable_key(float f)
{
    uint32_t u = __float_as_uint(f + 0.0f);      // -0 and +0 compare equal, as floats do
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace sf
