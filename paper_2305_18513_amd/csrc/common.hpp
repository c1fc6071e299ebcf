// Shared host/device helpers of the gfx950 kernels (wave64, DPP cross-lane ops).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "slimfit.h"

namespace slimfit {

constexpr int kWave = 64;

// ---- host-side helpers (api.cpp) --------------------------------------------
int32_t check_device_range(const void *p, size_t bytes);   // pointer checks, see slimfit.h
// Declared at the top of every entry point that takes a stream: while that stream is being captured into a
// graph the pointer look-ups (runtime queries a capture does not allow) are skipped for this thread's call.
struct StreamScope {
    explicit StreamScope(void *stream);
    ~StreamScope();
    StreamScope(const StreamScope &) = delete;
    StreamScope &operator=(const StreamScope &) = delete;
private:
    bool prev_;
};
int32_t launch_status();                                    // hipGetLastError -> status

// short rows that keep few entries have a kernel of their own (prune_short.hip)
constexpr int kShortPruneMaxCols = 256;
constexpr int kShortPruneMaxK = 16;                     // bf16 rows
constexpr int kShortPruneMaxKF32 = 9;                   // fp32 rows
bool prune_short_eligible(const void *p, int32_t dt, int64_t rows, int cols, int k);
void launch_prune_short(const void *p, int32_t dt, int64_t rows, int cols, int k, int mode, float tau, void *vals,
                        uint16_t *idx, int32_t *counts, hipStream_t st);
void launch_softmax_prune_short(const void *logits, int32_t dt, int64_t rows, int cols, int k, void *probs, void *vals,
                                uint16_t *idx, hipStream_t st);

inline bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline bool dtype_ok(int32_t dt) { return dt == SLIMFIT_F32 || dt == SLIMFIT_BF16; }
inline size_t dtype_size(int32_t dt) { return dt == SLIMFIT_F32 ? 4 : 2; }

#if defined(__HIPCC__)
// ---- 128/64-bit global access, optionally non-temporal (streamed once) ----------
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <bool NT, typename V>
__device__ __forceinline__ V load_global(const V *p)
{
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT, typename V>
__device__ __forceinline__ void store_global(V *p, V v)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// ---- DPP lane exchange --------------------------------------------------------
// A DPP "row" is 16 consecutive lanes.  The controls used here only permute
// inside a row, so every source lane exists.
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(float, dpp_u32<CTRL>(__builtin_bit_cast(uint32_t, v)));
}

// max over groups of G consecutive lanes (G = 4..64, power of two); every lane
// of a group receives the group's result.
template <int G>
__device__ __forceinline__ float group_max_f32(float v)
{
    static_assert(G == 4 || G == 8 || G == 16 || G == 32 || G == 64, "group size");
    v = fmaxf(v, dpp_f32<kDppXor1>(v));
    v = fmaxf(v, dpp_f32<kDppXor2>(v));
    if (G >= 8) v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
    if (G >= 16) v = fmaxf(v, dpp_f32<kDppMirror>(v));
    if (G >= 32) v = fmaxf(v, __shfl_xor(v, 16, kWave));
    if (G >= 64) v = fmaxf(v, __shfl_xor(v, 32, kWave));
    return v;
}

// the same with the group size a wave-uniform run-time value (4, 8, 16, 32 or 64)
__device__ __forceinline__ float group_max_f32_dyn(float v, int G)
{
    v = fmaxf(v, dpp_f32<kDppXor1>(v));
    v = fmaxf(v, dpp_f32<kDppXor2>(v));
    if (G >= 8) v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
    if (G >= 16) v = fmaxf(v, dpp_f32<kDppMirror>(v));
    if (G >= 32) v = fmaxf(v, __shfl_xor(v, 16, kWave));
    if (G >= 64) v = fmaxf(v, __shfl_xor(v, 32, kWave));
    return v;
}

// Alg. 2 with one scale per block: code = clamp(round_half_even(x * mult), qmin, qmax)
// -- one fp32 multiply -- where mult = qmax / a and the stored scale = a / qmax for a
// block whose largest magnitude is a (two IEEE fp32 divisions); a block of zeros, or one
// whose multiplier would overflow, gets scale 0 and codes 0.
template <int BITS>
__device__ __forceinline__ int quantise_one(float x, float mult)
{
    constexpr float qmax = (float)((1 << (BITS - 1)) - 1);
    constexpr float qmin = -(float)(1 << (BITS - 1));
    float r = __builtin_rintf(x * mult);
    r = fminf(fmaxf(r, qmin), qmax);
    return (int)r;
}
template <int BITS>
__device__ __forceinline__ void block_scale(float a, float &mult, float &scale)
{
    constexpr float qmax = (float)((1 << (BITS - 1)) - 1);
    mult = 0.0f;
    scale = 0.0f;
    if (a > 0.0f) {
        mult = qmax / a;
        if (__builtin_isinf(mult)) mult = 0.0f;
        else scale = a / qmax;
    }
}
// field i of BITS bits of a packed word, sign-extended
template <int BITS>
__device__ __forceinline__ int code_field(uint32_t word, int i)
{
    const int sh = i * BITS;
    return (int)(word << (32 - BITS - sh)) >> (32 - BITS);
}

// Whole-wave reductions of unsigned keys; the result is wave-uniform (SGPR).
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = max(v, dpp_u32<kDppXor1>(v));
    v = max(v, dpp_u32<kDppXor2>(v));
    v = max(v, dpp_u32<kDppHalfMirror>(v));
    v = max(v, dpp_u32<kDppMirror>(v));
    uint32_t a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    uint32_t c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    return max(max(a, b), max(c, d));
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
    v = min(v, dpp_u32<kDppXor1>(v));
    v = min(v, dpp_u32<kDppXor2>(v));
    v = min(v, dpp_u32<kDppHalfMirror>(v));
    v = min(v, dpp_u32<kDppMirror>(v));
    uint32_t a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    uint32_t c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    return min(min(a, b), min(c, d));
}

// number of set bits of `mask` strictly below this lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// ---- bf16 -----------------------------------------------------------------------
__device__ __forceinline__ float bf16_widen(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// fp32 -> bf16, round to nearest even, denormals kept, NaN stays NaN.  gfx950 has the conversion in
// hardware (one instruction for a pair); the integer form is kept for comparison.
#ifndef SLIMFIT_HW_BF16_CVT
#define SLIMFIT_HW_BF16_CVT 1
#endif
__device__ __forceinline__ uint32_t bf16_narrow(float f)
{
#if SLIMFIT_HW_BF16_CVT
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
#else
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u) : r;
#endif
}

// two at once, a in the low half
__device__ __forceinline__ uint32_t bf16_narrow2(float a, float b)
{
#if SLIMFIT_HW_BF16_CVT
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const bf16x2_t h = __builtin_convertvector(f32x2_t{a, b}, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
#else
    return bf16_narrow(a) | (bf16_narrow(b) << 16);
#endif
}

// Order-preserving map float -> uint32 (larger float <=> larger key) and back.
__device__ __forceinline__ uint32_t float_to_key(float f)
{
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k)
{
    uint32_t u = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __builtin_bit_cast(float, u);
}
#endif  // __HIPCC__

}  // namespace slimfit
