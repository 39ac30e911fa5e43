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
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__bf16 x) { return (float)x; }
template <class T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ __bf16 from_f32<__bf16>(float x) { return (__bf16)x; }   // RNE

// Order-preserving map of fp32 to uint32 (larger float <=> larger key).
__device__ __forceinline__ uint32_t sortable_key(float f)
{
    uint32_t u = __float_as_uint(f + 0.0f);      // -0 and +0 compare equal, as floats do
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace sf
