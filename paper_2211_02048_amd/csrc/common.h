// Internal helpers of the gfx950 library: error reporting, argument checks,
// storage-type traits and 16-byte vector access.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "sige.h"

namespace sige {

typedef _Float16 f16;
typedef __bf16 bf16;

int fail(int code, const char* fmt, ...);  // records a thread-local message, returns code
void clear_error();

#define SIGE_REQUIRE(cond, code, ...)                 \
    do {                                              \
        if (!(cond)) return sige::fail(code, __VA_ARGS__); \
    } while (0)

#define SIGE_LAUNCH_CHECK(name)                                                          \
    do {                                                                                 \
        hipError_t e_ = hipGetLastError();                                               \
        if (e_ != hipSuccess)                                                            \
            return sige::fail(SIGE_ERR_HIP, "%s: launch failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

// Overrides of the launch heuristics set through sige_set_knob (-1 = automatic); process-wide,
// read on the host when a call is planned.
extern int g_knobs[SIGE_KNOB_COUNT];
inline int knob(sige_knob k) { return g_knobs[k]; }

// reduce_mask.hip: the compaction pass over lists that sige_mark_blocks left marked (flags -> ordered
// lists, flags cleared), for consumers of marked lists that cannot build the lists themselves
int compact_marked_lists(const char* who, const sige_block_list* lists, int n, hipStream_t st);

inline size_t dtype_size(sige_dtype dt) { return dt == SIGE_F32 ? 4 : 2; }
inline bool dtype_ok(sige_dtype dt) { return dt == SIGE_F32 || dt == SIGE_F16 || dt == SIGE_BF16; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks shared by every call that takes a geometry; fills tile sizes.
int check_geom(const sige_geom* g, const char* who, int* tile_h, int* tile_w);
// Resolves (count, max_blocks, n_blocks) into the number of blocks to launch for.
int check_blocks(const int32_t* count, int32_t max_blocks, int32_t n_blocks, const char* who,
                 int* launch_blocks);

// ---- device side ---------------------------------------------------------------

template <typename T> struct Vec16;                    // a 16-byte vector of T
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<f16> { static constexpr int N = 8; };
template <> struct Vec16<bf16> { static constexpr int N = 8; };

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; }

// Unpack a 16-byte vector into floats / pack floats back with one rounding each.
template <typename T> __device__ __forceinline__ void unpack(const uint4& u, float* f);
template <> __device__ __forceinline__ void unpack<float>(const uint4& u, float* f)
{
    f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
    f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
}
template <> __device__ __forceinline__ void unpack<f16>(const uint4& u, float* f)
{
    union { uint4 v; f16 h[8]; } c; c.v = u;
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)c.h[i];
}
template <> __device__ __forceinline__ void unpack<bf16>(const uint4& u, float* f)
{
    // bf16 -> fp32 is a 16-bit shift, exact
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
    f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
    f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
}
template <typename T> __device__ __forceinline__ uint4 pack(const float* f);
template <> __device__ __forceinline__ uint4 pack<float>(const float* f)
{
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                      __float_as_uint(f[3]));
}
template <> __device__ __forceinline__ uint4 pack<f16>(const float* f)
{
    union { uint4 v; f16 h[8]; } c;
#pragma unroll
    for (int i = 0; i < 8; ++i) c.h[i] = (f16)f[i];
    return c.v;
}
template <> __device__ __forceinline__ uint4 pack<bf16>(const float* f)
{
    union { uint4 v; bf16 h[8]; } c;
#pragma unroll
    for (int i = 0; i < 8; ++i) c.h[i] = (bf16)f[i];
    return c.v;
}

// Streaming (non-temporal) 16-byte load: data that is read exactly once.
__device__ __forceinline__ uint4 load_stream(const uint4* p)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// f[i] = act(sc[i] * f[i] + sh[i]) for the N elements of one vector.  The activation is chosen once
// per vector, not per element, so that the N independent chains sit in one basic block and overlap.
// SiLU as v * rcp(1 + exp2(-v * log2 e)): two hardware transcendentals (about 1 ulp each) and no
// full-precision division, so that the fused gather stays bandwidth bound.  exp2 overflows to
// +inf for very negative v, whose reciprocal is 0: the result is -0, as it should be.
template <int N>
__device__ __forceinline__ void scale_shift_act(float (&f)[N], const float (&sc)[N], const float (&sh)[N], int act)
{
    if (act == SIGE_ACT_SILU) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float v = fmaf(sc[i], f[i], sh[i]);
            f[i] = v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * -1.4426950408889634f));
        }
    } else if (act == SIGE_ACT_RELU) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float v = fmaf(sc[i], f[i], sh[i]);
            f[i] = v > 0.0f ? v : 0.0f;
        }
    } else if (act == SIGE_ACT_LEAKY_RELU) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const float v = fmaf(sc[i], f[i], sh[i]);
            f[i] = v > 0.0f ? v : 0.2f * v;
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) f[i] = fmaf(sc[i], f[i], sh[i]);
    }
}

// A single activation (used where the value is not a plain scale-shift result).
__device__ __forceinline__ float activate(float v, int act)
{
    if (act == SIGE_ACT_SILU) return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * -1.4426950408889634f));
    if (act == SIGE_ACT_RELU) return v > 0.0f ? v : 0.0f;
    if (act == SIGE_ACT_LEAKY_RELU) return v > 0.0f ? v : 0.2f * v;
    return v;
}

inline bool act_ok(int act) { return act >= SIGE_ACT_NONE && act <= SIGE_ACT_LEAKY_RELU; }

__device__ __forceinline__ bool aligned16_dev(const void* p)
{
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// Forces a kernel argument into a scalar register here.  Left alone, the compiler fetches the fields
// of a large by-value argument struct in small groups right before their first use, each group a
// dependent round trip to the scalar cache; pinned at the top of a kernel they arrive together.
#define SIGE_PIN_S(x) asm volatile("" ::"s"(x))

// Number of blocks a kernel may touch: the host value when given, else the device count.
__device__ __forceinline__ int effective_blocks(const int32_t* count, int max_blocks, int n_host)
{
    if (n_host >= 0) return n_host;
    int c = *count;
    return c < max_blocks ? c : max_blocks;
}

// Number of blocks and the origin of block n, fetched together: the count and the index row are
// independent loads, so they are issued back to back and awaited once instead of one after the
// other (row n exists whenever n < max_blocks, whatever the count says).  The empty asm pins the
// loads above the early exit that depends on the count.
__device__ __forceinline__ int blocks_and_origin(const int32_t* count, int max_blocks, int n_host,
                                                 const int32_t* indices, int n, int& y0, int& x0)
{
    y0 = indices[2 * n];
    x0 = indices[2 * n + 1];
    int n_eff = effective_blocks(count, max_blocks, n_host);
    asm volatile("" : "+v"(y0), "+v"(x0), "+v"(n_eff));
    return n_eff;
}

// N consecutive fp32 parameters starting at p + off (off a multiple of N): as 16-byte vectors when p
// is 16-byte aligned, element by element otherwise.
template <int N>
__device__ __forceinline__ void load_f32_run(const float* p, int off, float (&out)[N])
{
    typedef float vec4 __attribute__((ext_vector_type(4)));
    if ((reinterpret_cast<uintptr_t>(p) & 15u) == 0) {
#pragma unroll
        for (int i = 0; i < N / 4; ++i) {
            const vec4 q = *(const vec4*)(p + off + 4 * i);
            out[4 * i] = q.x; out[4 * i + 1] = q.y; out[4 * i + 2] = q.z; out[4 * i + 3] = q.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = p[off + i];
    }
}

// Division by a divisor known on the host: q = floor(x / d) for any 0 <= x < 2^32 and d >= 1 from one
// high multiply and one correction (m = floor(2^32 / d), 0 for d == 1).  The compiler's expansion of
// a 32-bit division is about thirty instructions, several of them quarter-rate multiplies, and the
// prologues of the small kernels are instruction bound.
struct FastDiv { int d; unsigned m; };
inline FastDiv fast_div(int d)
{
    FastDiv f;
    f.d = d;
    f.m = d <= 1 ? 0u : (unsigned)((1ull << 32) / (unsigned)d);
    return f;
}
__device__ __forceinline__ void divmod(int x, const FastDiv f, int& q, int& r)
{
    if (f.m == 0u) { q = x; r = 0; return; }     // d == 1
    unsigned qq = __umulhi((unsigned)x, f.m);
    unsigned rr = (unsigned)x - qq * (unsigned)f.d;
    if (rr >= (unsigned)f.d) { ++qq; rr -= (unsigned)f.d; }
    q = (int)qq;
    r = (int)rr;
}

}  // namespace sige
