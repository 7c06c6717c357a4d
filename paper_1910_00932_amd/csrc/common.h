// Shared host/device helpers of the HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdio.h>
#include "../../include/tsm.h"

namespace tsm {

// ---- error reporting -------------------------------------------------------
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);
// Checks the launch error state of the calling thread after a kernel launch.
int check_launch(const char* what);
bool profiling_active();   // per-launch timing is on (every launch must then stay on the profiled stream)

#define TSM_TRY(expr)                 \
    do {                              \
        int _rc = (expr);             \
        if (_rc != TSM_OK) return _rc; \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }
inline size_t dtype_size(int dtype) { return dtype == TSM_BF16 ? 2 : 4; }

// fold for a channel count; returns <0 status on an invalid fold_div.
inline int fold_of(int C, int fold_div, int* fold) {
    if (fold_div == 0) { *fold = 0; return TSM_OK; }
    if (fold_div < 0 || fold_div == 1) return TSM_ERR_FOLD;
    int f = C / fold_div;
    if (2 * f > C) return TSM_ERR_FOLD;
    *fold = f;
    return TSM_OK;
}

// Bump allocator over the caller's workspace.
struct Arena {
    char* base;
    size_t cap, used;
    Arena(void* p, size_t bytes) : base((char*)p), cap(bytes), used(0) {}
    void* take(size_t bytes) {
        size_t a = align_up(bytes);
        void* r = base ? base + used : nullptr;
        used += a;
        return r;
    }
    template <typename T> T* take_n(size_t n) { return (T*)take(n * sizeof(T)); }
    bool ok() const { return used <= cap; }
};

// ---- bf16 as raw 16 bits ----------------------------------------------------
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// Round to nearest even with the hardware converter (v_cvt_pk_bf16_f32): two floats -> two packed bf16,
// `lo` in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    f32x2_t v = {lo, hi};
    bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int VEC = 4;  // elements per 16-byte vector
    __device__ static __forceinline__ float ld(float v) { return v; }
    __device__ static __forceinline__ float st(float v) { return v; }
};
template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    __device__ static __forceinline__ float ld(bf16_t v) { return bf16_to_f32(v); }
    __device__ static __forceinline__ bf16_t st(float v) { return f32_to_bf16(v); }
};

// 16-byte vector of T
template <typename T> struct alignas(16) Vec16 { T v[16 / sizeof(T)]; };

}  // namespace tsm
