// Low-bit caching of saved activations (Alg. 2; Sec. 4 and 5): fused
// quantise + pack and unpack + dequantise for gfx950.
//
// Layout: every lane owns one 16-byte vector of the flat tensor (4 fp32 or
// 8 bf16 elements) per step; consecutive lanes own consecutive vectors, so a
// wave's load is one contiguous 1 KiB run.  A quantisation block of `block`
// elements is therefore G = block / V consecutive lanes, and the block's
// absolute maximum is a DPP butterfly over those lanes -- no LDS, no second
// pass over the data.  A workgroup covers kUnroll such steps so that each lane
// has kUnroll independent 128-bit loads in flight.
//
// Producer fusion: the same tiles can also carry the GELU whose input is being
// cached.  Forward, the lane that holds x for the quantiser also writes
// GELU(x), so the activation is read once for both; backward, the dequantised
// x^ never reaches memory: the lane multiplies the incoming gradient by
// GELU'(x^) and writes the input gradient.
#include "common.hpp"

namespace slimfit {
namespace {

// Tunables (compile-time): vectors per lane in the two kernels, and whether
// the bulk streams bypass the caches' retention (each byte is touched once).
#ifndef SLIMFIT_QUANT_UNROLL
#define SLIMFIT_QUANT_UNROLL 4
#endif
#ifndef SLIMFIT_DEQUANT_UNROLL
#define SLIMFIT_DEQUANT_UNROLL 2
#endif
#ifndef SLIMFIT_QUANT_NT
#define SLIMFIT_QUANT_NT 1
#endif

#ifndef SLIMFIT_QUANT_THREADS
#define SLIMFIT_QUANT_THREADS 256
#endif
#ifndef SLIMFIT_DEQUANT_THREADS
#define SLIMFIT_DEQUANT_THREADS 512
#endif
constexpr int kThreads = SLIMFIT_QUANT_THREADS;      // quantiser workgroup
constexpr int kThreadsD = SLIMFIT_DEQUANT_THREADS;   // dequantiser workgroup
constexpr int kUnrollQ = SLIMFIT_QUANT_UNROLL;
constexpr int kUnrollD = SLIMFIT_DEQUANT_UNROLL;
constexpr bool kNT = SLIMFIT_QUANT_NT != 0;

template <typename T> struct Vec;
template <> struct Vec<float> {
    static constexpr int V = 4;
    using raw = f32x4;
    __device__ static void unpack(const raw &r, float (&f)[4]) { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
    __device__ static raw pack(const float (&f)[4]) { return raw{f[0], f[1], f[2], f[3]}; }
    __device__ static float load1(const float *p) { return *p; }
    __device__ static void store1(float *p, float v) { *p = v; }
};
template <> struct Vec<uint16_t> {   // bf16 bit patterns
    static constexpr int V = 8;
    using raw = u32x4;
    __device__ static void unpack(const raw &r, float (&f)[8])
    {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
            f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
        }
    }
    __device__ static raw pack(const float (&f)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = bf16_narrow2(f[2 * i], f[2 * i + 1]);
        return raw{w[0], w[1], w[2], w[3]};
    }
    __device__ static float load1(const uint16_t *p) { return bf16_widen(*p); }
    __device__ static void store1(uint16_t *p, float v) { *p = (uint16_t)bf16_narrow(v); }
};

// Exact (erf) GELU and its derivative in fp32.
// 1 + erf(x / sqrt 2) is built from erfc(t), t = |x| / sqrt 2:  2 - erfc(t) for
// x >= 0 and erfc(t) itself for x < 0, which also keeps the left tail free of
// cancellation.  erfc(t) = exp(-t * Q(t)) with Q(t) = -ln(erfc t) / t, a smooth
// function (Q(0) = 2 / sqrt pi) replaced by a degree-8 polynomial fitted to it
// on [0, 4.2] (weighted least squares at Chebyshev nodes, weight erfc(t) * t);
// beyond 4.2 erfc is below 3e-9 and t is clamped.  In fp32 with fused
// multiply-adds and the hardware exp2 the absolute error of erfc stays under
// 1.5e-7 (checked against fp64 on 3 M points), one branch-free path of about 16
// instructions where the library erff takes two divergent ones of about 40.
__device__ __forceinline__ float erfc_nonneg(float t)
{
    t = fminf(t, 4.2f);
    float q = -8.094536919e-06f;
    q = fmaf(q, t, 1.064909658e-04f);
    q = fmaf(q, t, -5.896771888e-04f);
    q = fmaf(q, t, 1.580125120e-03f);
    q = fmaf(q, t, -6.248015670e-05f);
    q = fmaf(q, t, -1.921485045e-02f);
    q = fmaf(q, t, 1.027984564e-01f);
    q = fmaf(q, t, 6.366162197e-01f);
    q = fmaf(q, t, 1.128379327e+00f);
    return __builtin_amdgcn_exp2f(-(q * t) * 1.44269504088896340736f);
}
__device__ __forceinline__ float twice_normal_cdf(float x)        // 1 + erf(x / sqrt 2)
{
    const float e = erfc_nonneg(fabsf(x) * 0.70710678118654752440f);
    return x >= 0.0f ? 2.0f - e : e;
}
__device__ __forceinline__ float gelu_f32(float x) { return (0.5f * x) * twice_normal_cdf(x); }
__device__ __forceinline__ float gelu_slope_f32(float x)
{
    const float pdf = __builtin_amdgcn_exp2f(((-0.5f * x) * x) * 1.44269504088896340736f) * 0.39894228040143267794f;
    return 0.5f * twice_normal_cdf(x) + x * pdf;
}

// One workgroup tile of quantise + pack.  INSIDE: the whole tile lies below n, so
// the code is straight-line (all loads issue back to back, no per-lane bounds);
// otherwise every access is guarded and elements past n count as 0.
// T: element type, BITS: 4|8, BLOCKED: per-block scale, G: lanes per block,
// GELU: also write GELU(x) to y
template <typename T, int BITS, bool BLOCKED, int G, bool INSIDE, bool GELU>
__device__ __forceinline__ void quant_tile(const T *__restrict__ x, int64_t n, float fixed_mult,
                                           uint8_t *__restrict__ codes, float *__restrict__ scales,
                                           T *__restrict__ y)
{
    constexpr int V = Vec<T>::V;
    constexpr int OUT_BYTES = V * BITS / 8;            // packed bytes per lane-vector: 2, 4 or 8
    constexpr int kUnroll = kUnrollQ;
    const int64_t first_vec = (int64_t)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;

    float f[kUnroll][V];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t e0 = (first_vec + (int64_t)u * kThreads) * V;
        if (INSIDE || e0 + V <= n) {
            typename Vec<T>::raw r = load_global<kNT>(reinterpret_cast<const typename Vec<T>::raw *>(x + e0));
            Vec<T>::unpack(r, f[u]);
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) f[u][i] = (e0 + i < n) ? Vec<T>::load1(x + e0 + i) : 0.0f;
        }
    }

    if (GELU) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t e0 = (first_vec + (int64_t)u * kThreads) * V;
            float g[V];
#pragma unroll
            for (int i = 0; i < V; ++i) g[i] = gelu_f32(f[u][i]);
            if (INSIDE || e0 + V <= n) {
                store_global<kNT>(reinterpret_cast<typename Vec<T>::raw *>(y + e0), Vec<T>::pack(g));
            } else {
                for (int i = 0; i < V && e0 + i < n; ++i) Vec<T>::store1(y + e0 + i, g[i]);
            }
        }
    }

#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t e0 = (first_vec + (int64_t)u * kThreads) * V;
        float mult = fixed_mult;
        if (BLOCKED) {
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < V; ++i) a = fmaxf(a, fabsf(f[u][i]));
            a = group_max_f32<G>(a);                   // all lanes take part (no divergence above)
            float scale;
            block_scale<BITS>(a, mult, scale);
            if ((threadIdx.x & (G - 1)) == 0 && (INSIDE || e0 < n)) scales[e0 / (V * G)] = scale;
        }
        if (!INSIDE && e0 >= n) continue;

        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const uint32_t c = (uint32_t)quantise_one<BITS>(f[u][i], mult) & ((1u << BITS) - 1u);
            w[(i * BITS) / 32] |= c << ((i * BITS) % 32);
        }
        uint8_t *dst = codes + (e0 * BITS) / 8;
        if (INSIDE || e0 + V <= n) {
            if (OUT_BYTES == 2) store_global<kNT>(reinterpret_cast<uint16_t *>(dst), (uint16_t)w[0]);
            else if (OUT_BYTES == 4) store_global<kNT>(reinterpret_cast<uint32_t *>(dst), w[0]);
            else store_global<kNT>(reinterpret_cast<u32x2 *>(dst), u32x2{w[0], w[1]});
        } else {
            const int nbytes = (int)(((n - e0) * BITS + 7) / 8);   // elements past n quantised 0
            for (int b = 0; b < nbytes; ++b) dst[b] = (uint8_t)(w[b / 4] >> (8 * (b % 4)));
        }
    }
}

template <typename T, int BITS, bool BLOCKED, int G, bool GELU>
__global__ __launch_bounds__(kThreads) void quant_pack_kernel(const T *__restrict__ x, int64_t n, float fixed_mult,
                                                              uint8_t *__restrict__ codes, float *__restrict__ scales,
                                                              T *__restrict__ y)
{
    constexpr int64_t TILE = (int64_t)kThreads * kUnrollQ * Vec<T>::V;
    if (((int64_t)blockIdx.x + 1) * TILE <= n)         // workgroup-uniform
        quant_tile<T, BITS, BLOCKED, G, true, GELU>(x, n, fixed_mult, codes, scales, y);
    else
        quant_tile<T, BITS, BLOCKED, G, false, GELU>(x, n, fixed_mult, codes, scales, y);
}

// GELU: y receives dy * GELU'(x^) instead of x^
template <typename T, int BITS, bool BLOCKED, bool INSIDE, bool GELU>
__device__ __forceinline__ void dequant_tile(const uint8_t *__restrict__ codes, const float *__restrict__ scales,
                                             int64_t n, int block_shift, float fixed_step, T *__restrict__ y,
                                             const T *__restrict__ dy)
{
    constexpr int V = Vec<T>::V;
    constexpr int IN_BYTES = V * BITS / 8;
    constexpr int kUnroll = kUnrollD;
    const int64_t first_vec = (int64_t)blockIdx.x * (kThreadsD * kUnroll) + threadIdx.x;

    uint32_t w[kUnroll][2];
    float s[kUnroll];
    float grad[GELU ? kUnroll : 1][V];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t e0 = (first_vec + (int64_t)u * kThreadsD) * V;
        w[u][0] = w[u][1] = 0u;
        s[u] = fixed_step;
        if (!INSIDE && e0 >= n) continue;
        if (GELU) {
            if (INSIDE || e0 + V <= n) {
                typename Vec<T>::raw r = load_global<kNT>(reinterpret_cast<const typename Vec<T>::raw *>(dy + e0));
                Vec<T>::unpack(r, grad[u]);
            } else {
#pragma unroll
                for (int i = 0; i < V; ++i) grad[u][i] = (e0 + i < n) ? Vec<T>::load1(dy + e0 + i) : 0.0f;
            }
        }
        const uint8_t *src = codes + (e0 * BITS) / 8;
        if (INSIDE || e0 + V <= n) {
            if (IN_BYTES == 2) w[u][0] = load_global<kNT>(reinterpret_cast<const uint16_t *>(src));
            else if (IN_BYTES == 4) w[u][0] = load_global<kNT>(reinterpret_cast<const uint32_t *>(src));
            else { u32x2 t = load_global<kNT>(reinterpret_cast<const u32x2 *>(src)); w[u][0] = t.x; w[u][1] = t.y; }
        } else {
            const int nbytes = (int)(((n - e0) * BITS + 7) / 8);
            for (int b = 0; b < nbytes; ++b) w[u][b / 4] |= (uint32_t)src[b] << (8 * (b % 4));
        }
        if (BLOCKED) s[u] = scales[e0 >> block_shift];      // block is a power of two
    }

#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t e0 = (first_vec + (int64_t)u * kThreadsD) * V;
        if (!INSIDE && e0 >= n) continue;
        float f[V];
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const uint32_t word = w[u][(i * BITS) / 32];
            const int sh = (i * BITS) % 32;
            const int c = (int)(word << (32 - BITS - sh)) >> (32 - BITS);   // sign-extending field extract
            f[i] = (float)c * s[u];                                        // one fp32 multiply
            if (GELU) f[i] = grad[u][i] * gelu_slope_f32(f[i]);
        }
        if (INSIDE || e0 + V <= n) {
            store_global<kNT>(reinterpret_cast<typename Vec<T>::raw *>(y + e0), Vec<T>::pack(f));
        } else {
            for (int i = 0; i < V && e0 + i < n; ++i) Vec<T>::store1(y + e0 + i, f[i]);
        }
    }
}

template <typename T, int BITS, bool BLOCKED, bool GELU>
__global__ __launch_bounds__(kThreadsD) void dequant_unpack_kernel(const uint8_t *__restrict__ codes,
                                                                  const float *__restrict__ scales, int64_t n,
                                                                  int block_shift, float fixed_step,
                                                                  T *__restrict__ y, const T *__restrict__ dy)
{
    constexpr int64_t TILE = (int64_t)kThreadsD * kUnrollD * Vec<T>::V;
    if (((int64_t)blockIdx.x + 1) * TILE <= n)         // workgroup-uniform
        dequant_tile<T, BITS, BLOCKED, true, GELU>(codes, scales, n, block_shift, fixed_step, y, dy);
    else
        dequant_tile<T, BITS, BLOCKED, false, GELU>(codes, scales, n, block_shift, fixed_step, y, dy);
}

inline unsigned grid_for(int64_t n, int V, int unroll, int threads)
{
    const int64_t per_block = (int64_t)threads * unroll * V;
    return (unsigned)((n + per_block - 1) / per_block);
}

template <typename T, int BITS, bool GELU>
void launch_quant(const void *x, int64_t n, int mode, int block, int frac_bits, uint8_t *codes, float *scales, void *y,
                  hipStream_t st)
{
    constexpr int V = Vec<T>::V;
    const dim3 grid(grid_for(n, V, kUnrollQ, kThreads)), tb(kThreads);
    const T *xp = static_cast<const T *>(x);
    T *yp = static_cast<T *>(y);
    if (mode == SLIMFIT_Q_FIXED) {
        quant_pack_kernel<T, BITS, false, 4, GELU><<<grid, tb, 0, st>>>(xp, n, __builtin_ldexpf(1.0f, frac_bits), codes,
                                                                        nullptr, yp);
        return;
    }
    switch (block / V) {
    case 4: quant_pack_kernel<T, BITS, true, 4, GELU><<<grid, tb, 0, st>>>(xp, n, 0.0f, codes, scales, yp); break;
    case 8: quant_pack_kernel<T, BITS, true, 8, GELU><<<grid, tb, 0, st>>>(xp, n, 0.0f, codes, scales, yp); break;
    case 16: quant_pack_kernel<T, BITS, true, 16, GELU><<<grid, tb, 0, st>>>(xp, n, 0.0f, codes, scales, yp); break;
    case 32: quant_pack_kernel<T, BITS, true, 32, GELU><<<grid, tb, 0, st>>>(xp, n, 0.0f, codes, scales, yp); break;
    default: quant_pack_kernel<T, BITS, true, 64, GELU><<<grid, tb, 0, st>>>(xp, n, 0.0f, codes, scales, yp); break;
    }
}

template <typename T, int BITS, bool GELU>
void launch_dequant(const uint8_t *codes, const float *scales, int64_t n, int mode, int block, int frac_bits, void *y,
                    const void *dy, hipStream_t st)
{
    constexpr int V = Vec<T>::V;
    const dim3 grid(grid_for(n, V, kUnrollD, kThreadsD)), tb(kThreadsD);
    T *yp = static_cast<T *>(y);
    const T *gp = static_cast<const T *>(dy);
    if (mode == SLIMFIT_Q_FIXED)
        dequant_unpack_kernel<T, BITS, false, GELU><<<grid, tb, 0, st>>>(codes, nullptr, n, 0,
                                                                         __builtin_ldexpf(1.0f, -frac_bits), yp, gp);
    else
        dequant_unpack_kernel<T, BITS, true, GELU><<<grid, tb, 0, st>>>(codes, scales, n, __builtin_ctz((unsigned)block),
                                                                        0.0f, yp, gp);
}

int32_t validate(int32_t dt, int64_t n, int32_t mode, int32_t bits, int32_t block, int32_t frac_bits)
{
    if (!dtype_ok(dt) || n < 0) return SLIMFIT_ERR_INVALID_ARG;
    if (mode != SLIMFIT_Q_FIXED && mode != SLIMFIT_Q_BLOCK) return SLIMFIT_ERR_INVALID_ARG;
    if (bits != 4 && bits != 8) return SLIMFIT_ERR_UNSUPPORTED;
    if (mode == SLIMFIT_Q_FIXED && (frac_bits < -32 || frac_bits > 32)) return SLIMFIT_ERR_UNSUPPORTED;
    if (mode == SLIMFIT_Q_BLOCK && block != 32 && block != 64 && block != 128 && block != 256)
        return SLIMFIT_ERR_UNSUPPORTED;
    // one workgroup per >= 1024 elements: the grid must fit a 31-bit launch dimension
    if (n > ((int64_t)1 << 40)) return SLIMFIT_ERR_UNSUPPORTED;
    return SLIMFIT_OK;
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

extern "C" size_t slimfit_packed_bytes(int64_t n, int32_t bits)
{
    if (n < 0 || (bits != 4 && bits != 8)) return 0;
    return (size_t)((n * bits + 7) / 8);
}

extern "C" int64_t slimfit_num_blocks(int64_t n, int32_t block)
{
    if (n < 0 || block <= 0) return 0;
    return (n + block - 1) / block;
}

namespace {

template <bool GELU>
int32_t quant_entry(const void *x, int32_t dt, int64_t n, int32_t mode, int32_t bits, int32_t block, int32_t frac_bits,
                    void *y, uint8_t *codes, float *scales, void *stream)
{
    int32_t rc = validate(dt, n, mode, bits, block, frac_bits);
    if (rc != SLIMFIT_OK) return rc;
    if (n == 0) return SLIMFIT_OK;
    if (!x || !codes || (mode == SLIMFIT_Q_BLOCK && !scales) || (GELU && !y)) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(x, 16) || !aligned_to(codes, 16) || (mode == SLIMFIT_Q_BLOCK && !aligned_to(scales, 16)) ||
        (GELU && !aligned_to(y, 16)))
        return SLIMFIT_ERR_ALIGNMENT;
    if ((rc = check_device_range(x, (size_t)n * dtype_size(dt))) != SLIMFIT_OK) return rc;
    if (GELU && (rc = check_device_range(y, (size_t)n * dtype_size(dt))) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(codes, slimfit_packed_bytes(n, bits))) != SLIMFIT_OK) return rc;
    if (mode == SLIMFIT_Q_BLOCK &&
        (rc = check_device_range(scales, (size_t)slimfit_num_blocks(n, block) * 4)) != SLIMFIT_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == SLIMFIT_F32) {
        if (bits == 4) launch_quant<float, 4, GELU>(x, n, mode, block, frac_bits, codes, scales, y, st);
        else launch_quant<float, 8, GELU>(x, n, mode, block, frac_bits, codes, scales, y, st);
    } else {
        if (bits == 4) launch_quant<uint16_t, 4, GELU>(x, n, mode, block, frac_bits, codes, scales, y, st);
        else launch_quant<uint16_t, 8, GELU>(x, n, mode, block, frac_bits, codes, scales, y, st);
    }
    return launch_status();
}

template <bool GELU>
int32_t dequant_entry(const uint8_t *codes, const float *scales, int64_t n, int32_t mode, int32_t bits, int32_t block,
                      int32_t frac_bits, const void *dy, void *y, int32_t dt, void *stream)
{
    int32_t rc = validate(dt, n, mode, bits, block, frac_bits);
    if (rc != SLIMFIT_OK) return rc;
    if (n == 0) return SLIMFIT_OK;
    if (!y || !codes || (mode == SLIMFIT_Q_BLOCK && !scales) || (GELU && !dy)) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(y, 16) || !aligned_to(codes, 16) || (mode == SLIMFIT_Q_BLOCK && !aligned_to(scales, 16)) ||
        (GELU && !aligned_to(dy, 16)))
        return SLIMFIT_ERR_ALIGNMENT;
    if ((rc = check_device_range(y, (size_t)n * dtype_size(dt))) != SLIMFIT_OK) return rc;
    if (GELU && (rc = check_device_range(dy, (size_t)n * dtype_size(dt))) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(codes, slimfit_packed_bytes(n, bits))) != SLIMFIT_OK) return rc;
    if (mode == SLIMFIT_Q_BLOCK &&
        (rc = check_device_range(scales, (size_t)slimfit_num_blocks(n, block) * 4)) != SLIMFIT_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == SLIMFIT_F32) {
        if (bits == 4) launch_dequant<float, 4, GELU>(codes, scales, n, mode, block, frac_bits, y, dy, st);
        else launch_dequant<float, 8, GELU>(codes, scales, n, mode, block, frac_bits, y, dy, st);
    } else {
        if (bits == 4) launch_dequant<uint16_t, 4, GELU>(codes, scales, n, mode, block, frac_bits, y, dy, st);
        else launch_dequant<uint16_t, 8, GELU>(codes, scales, n, mode, block, frac_bits, y, dy, st);
    }
    return launch_status();
}

}  // namespace

extern "C" int32_t slimfit_quant_pack(const void *x, int32_t dt, int64_t n, int32_t mode, int32_t bits, int32_t block,
                                      int32_t frac_bits, uint8_t *codes, float *scales, void *stream)
{
    StreamScope capture_aware(stream);
    return quant_entry<false>(x, dt, n, mode, bits, block, frac_bits, nullptr, codes, scales, stream);
}

extern "C" int32_t slimfit_dequant_unpack(const uint8_t *codes, const float *scales, int64_t n, int32_t mode,
                                          int32_t bits, int32_t block, int32_t frac_bits, void *y, int32_t dt,
                                          void *stream)
{
    StreamScope capture_aware(stream);
    return dequant_entry<false>(codes, scales, n, mode, bits, block, frac_bits, nullptr, y, dt, stream);
}

extern "C" int32_t slimfit_gelu_quant_pack(const void *x, int32_t dt, int64_t n, int32_t mode, int32_t bits,
                                           int32_t block, int32_t frac_bits, void *y, uint8_t *codes, float *scales,
                                           void *stream)
{
    StreamScope capture_aware(stream);
    if (x && x == y) return SLIMFIT_ERR_INVALID_ARG;                    // the kernels are compiled for distinct buffers
    return quant_entry<true>(x, dt, n, mode, bits, block, frac_bits, y, codes, scales, stream);
}

extern "C" int32_t slimfit_gelu_backward_dequant(const uint8_t *codes, const float *scales, int64_t n, int32_t mode,
                                                 int32_t bits, int32_t block, int32_t frac_bits, const void *dy,
                                                 void *dx, int32_t dt, void *stream)
{
    StreamScope capture_aware(stream);
    if (dy && dy == dx) return SLIMFIT_ERR_INVALID_ARG;
    return dequant_entry<true>(codes, scales, n, mode, bits, block, frac_bits, dy, dx, dt, stream);
}
