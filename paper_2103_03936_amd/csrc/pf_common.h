// Shared host/device helpers for the gfx950 low-rank layer kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pufferfish.h"

#include <initializer_list>

namespace pf {

// true when one of the (non-NULL) pointers is not a multiple of `a` bytes
inline bool any_misaligned(std::initializer_list<const void *> ps, uintptr_t a)
{
    for (const void *q : ps)
        if (((uintptr_t)q & (a - 1)) != 0) return true;
    return false;
}


typedef long long i64;

// ------------------------------------------------------------------ types
struct bf16_t {
    uint16_t v;
};

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));

// Two floats -> two bf16 (round to nearest even, NaN stays NaN) packed lo | hi << 16: one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2_hw_t v = {lo, hi};
    union {
        bf16x2_hw_t b;
        uint32_t u;
    } c;
    c.b = __builtin_convertvector(v, bf16x2_hw_t);
    return c.u;
}

__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) { return (uint16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return bf16_bits_to_float(x.v); }

template <typename T>
__device__ __forceinline__ T from_float(float f);
template <>
__device__ __forceinline__ float from_float<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float f)
{
    bf16_t r;
    r.v = float_to_bf16_bits(f);
    return r;
}

typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;

// Transposing LDS read (ds_read_b64_tr_b16): within each group of 16 lanes, lane 4 q + c receives element c of
// the 8-byte chunks addressed by lanes q, q + 4, q + 8, q + 12.  Pointing lane q + 4 e at &tile[m0 + e][c0 + 4 q]
// hands lane i the four rows m0 .. m0 + 3 of column c0 + i; two such reads make one MFMA fragment:
// the 8 consecutive rows r0 + 8 (lane / 32) + 0..7 of column c0 + lane % 32 of a row-major bf16 LDS tile.
__device__ __forceinline__ bf16x8_t lds_frag_tr(const uint16_t *tile, int pitch, int r0, int c0, int lane)
{
    const int g = lane >> 4, i = lane & 15;
    const uint16_t *p = tile + (r0 + 8 * (g >> 1) + (i >> 2)) * pitch + c0 + 16 * (g & 1) + 4 * (i & 3);
    typedef __attribute__((address_space(3))) bf16x4_t *lds_ptr;
    const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)p);
    const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr)(p + 4 * pitch));
    bf16x8_t r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        r[e] = lo[e];
        r[4 + e] = hi[e];
    }
    return r;
}

// ------------------------------------------------------------ host helpers
int set_hip_error(hipError_t e); // records e for pf_last_hip_error(), returns PF_ERR_LAUNCH

struct TimingScope {
    TimingScope(const char *name, hipStream_t s);
    ~TimingScope();
    int slot;
    hipStream_t stream;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Bump allocator over the caller's workspace.
struct Workspace {
    char *base;
    size_t size, used;
    Workspace(void *p, size_t n) : base((char *)p), size(n), used(0) {}
    template <typename T>
    T *take(size_t count)
    {
        size_t bytes = align_up(count * sizeof(T));
        T *r = (T *)(base + used);
        used += bytes;
        return r;
    }
    // false once the pieces handed out exceed the buffer: a plan and its call disagree
    bool ok() const { return used <= size; }
};

} // namespace pf

// Launch `kernel` on `stream`, bracketed by timing events when enabled.  Evaluates to a
// pf_status in `status_var` (PF_OK or PF_ERR_LAUNCH).
#define PF_LAUNCH(status_var, name, kernel, grid, block, stream, ...)                    \
    do {                                                                                  \
        if ((status_var) == PF_OK) {                                                      \
            pf::TimingScope pf_ts_(name, stream);                                         \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);              \
            hipError_t pf_e_ = hipGetLastError();                                         \
            if (pf_e_ != hipSuccess) (status_var) = pf::set_hip_error(pf_e_);             \
        }                                                                                 \
    } while (0)
