// LayerNorm around the pruned cache of its standardised input (Sec. 4):
//
//   layernorm_forward_kernel          y = x~ * gamma + beta and the row
//                                     statistics (mean, 1/sqrt(Var + eps)) that
//                                     let the whole-tensor pruner form x~ on the
//                                     fly instead of reading a stored copy;
//   layernorm_backward_kernel         the input gradient of an active LayerNorm
//                                     (the same formula with every x~ present,
//                                     formed from x and the row statistics);
//   param_grad_*_kernel               gamma^ and beta^ of an active LayerNorm
//                                     (column sums over all rows, two stages);
//   layernorm_forward_quant_kernel    the forward pass that also writes the low-bit
//                                     cache of its input (Alg. 2), one read of x;
//   layernorm_backward_dequant_kernel the input gradient straight from that cache;
//   layernorm_backward_pruned_kernel  the input gradient of a frozen LayerNorm,
//                                     x^ = H g - sum g - x~ sum(g x~),
//                                     g = gamma y^ / (H sqrt(Var + eps)), with
//                                     x~ given as the (value, flat index) pairs
//                                     Alg. 5 kept: the dense x~ is never rebuilt
//                                     in memory.
//
// Both give a row of H elements to one wave: lane l holds the 16-byte vectors
// l, l+64, ... of the row (NV of them), sums run over the lanes with DPP in a
// fixed order, and nothing is read twice.  The backward kernel stages g and
// then the output row in the wave's LDS region so that the kept pairs, which
// arrive in index order and not in lane order, can be applied to it; the row's
// pairs are found through row pointers (survivors ahead of every row), which
// the pruner emits alongside the pairs.
#include "common.hpp"

namespace slimfit {
namespace {

#ifndef SLIMFIT_LN_THREADS
#define SLIMFIT_LN_THREADS 256
#endif
constexpr int kThreads = SLIMFIT_LN_THREADS;
constexpr int kWaves = kThreads / kWave;
constexpr int kMaxH = 4096;                 // NV <= 16 vectors of 4 per lane

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add_f32(float v)      // absent sources contribute +0
{
    return v + __builtin_bit_cast(float,
                                  __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
// sum of one float per lane, in a fixed order; result uniform
__device__ __forceinline__ float wave_sum_f32(float v)
{
    v = dpp_add_f32<0x111, 0xF>(v);        // row_shr:1
    v = dpp_add_f32<0x112, 0xF>(v);        // row_shr:2
    v = dpp_add_f32<0x114, 0xF>(v);        // row_shr:4
    v = dpp_add_f32<0x118, 0xF>(v);        // row_shr:8
    v = dpp_add_f32<0x142, 0xA>(v);        // row_bcast:15 into rows 1 and 3
    v = dpp_add_f32<0x143, 0xC>(v);        // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// lane's vectors of a row; vectors past the row's end read as zeros
template <int NV>
__device__ __forceinline__ void load_row(const float *__restrict__ row, int nvec, int lane, f32x4 (&v)[NV], bool stream)
{
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        v[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (q < nvec) {
            const f32x4 *src = reinterpret_cast<const f32x4 *>(row) + q;
            v[i] = stream ? __builtin_nontemporal_load(src) : *src;
        }
    }
}

// A 16-byte vector of a row as E floats: 4 fp32 elements, or 8 bf16 elements widened (exactly) on the
// way in and rounded to nearest even on the way out.  gamma / beta / statistics are always fp32.
template <typename T> struct RowIO;
template <> struct RowIO<float> {
    static constexpr int E = 4;
    __device__ static void load(const float *row, int q, float (&f)[4])
    {
        const f32x4 r = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(row) + q);
        f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    }
    __device__ static void store(float *row, int q, const float (&f)[4])
    {
        __builtin_nontemporal_store(f32x4{f[0], f[1], f[2], f[3]}, reinterpret_cast<f32x4 *>(row) + q);
    }
};
template <> struct RowIO<uint16_t> {
    static constexpr int E = 8;
    __device__ static void load(const uint16_t *row, int q, float (&f)[8])
    {
        const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row) + q);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
            f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
        }
    }
    __device__ static void store(uint16_t *row, int q, const float (&f)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = bf16_narrow2(f[2 * i], f[2 * i + 1]);
        __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4 *>(row) + q);
    }
};
// the fp32 parameters (or any fp32 row) that go with vector q of E elements
template <int E>
__device__ __forceinline__ void load_f32(const float *g, int q, float (&f)[E])
{
#pragma unroll
    for (int c = 0; c < E / 4; ++c) {
        const f32x4 r = reinterpret_cast<const f32x4 *>(g)[q * (E / 4) + c];
        f[4 * c] = r.x; f[4 * c + 1] = r.y; f[4 * c + 2] = r.z; f[4 * c + 3] = r.w;
    }
}
// lane's vectors of a row (vectors past the row's end hold zeros)
template <typename T, int NV>
__device__ __forceinline__ void load_row_t(const T *row, int nvec, int lane, float (&v)[NV][RowIO<T>::E])
{
    constexpr int E = RowIO<T>::E;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
#pragma unroll
        for (int e = 0; e < E; ++e) v[i][e] = 0.0f;
        if (q < nvec) RowIO<T>::load(row, q, v[i]);
    }
}
template <int E, int NV>
__device__ __forceinline__ void load_params(const float *g, int nvec, int lane, float (&v)[NV][E])
{
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
#pragma unroll
        for (int e = 0; e < E; ++e) v[i][e] = 0.0f;
        if (q < nvec) load_f32<E>(g, q, v[i]);
    }
}
// pairwise sum of a vector's E values, the same tree for every vector
template <int E>
__device__ __forceinline__ float sum_vec(const float (&f)[E])
{
    float s = (f[0] + f[1]) + (f[2] + f[3]);
    if constexpr (E == 8) s += (f[4] + f[5]) + (f[6] + f[7]);
    return s;
}

// Shared front end of the two forward kernels: statistics of the row held in v.
template <int E, int NV>
__device__ __forceinline__ void row_statistics(const float (&v)[NV][E], int nvec, int lane, int H, float eps, float &mu,
                                               float &rs)
{
    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) part += sum_vec<E>(v[i]);
    mu = wave_sum_f32(part) / (float)H;
    part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const bool in = i * kWave + lane < nvec;             // padding vectors must not add mu^2
        float sq[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const float d = v[i][e] - mu;
            sq[e] = d * d;
        }
        part += in ? sum_vec<E>(sq) : 0.0f;
    }
    const float var = wave_sum_f32(part) / (float)H;
    rs = 1.0f / __builtin_sqrtf(var + eps);
}
template <typename T, int NV>
__device__ __forceinline__ void store_normalised(T *yrow, const float (&v)[NV][RowIO<T>::E],
                                                 const float (&ga)[NV][RowIO<T>::E], const float (&be)[NV][RowIO<T>::E],
                                                 int nvec, int lane, float mu, float rs)
{
    constexpr int E = RowIO<T>::E;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
            float o[E];
#pragma unroll
            for (int e = 0; e < E; ++e) o[e] = ((v[i][e] - mu) * rs) * ga[i][e] + be[i][e];
            RowIO<T>::store(yrow, q, o);
        }
    }
}

template <typename T, int NV>
__global__ void __launch_bounds__(kThreads)
layernorm_forward_kernel(const T *__restrict__ x, const float *__restrict__ gamma, const float *__restrict__ beta,
                         int64_t rows, int H, float eps, T *__restrict__ y, float *__restrict__ mean,
                         float *__restrict__ rstd)
{
    constexpr int E = RowIO<T>::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int nvec = H / E;
    float v[NV][E], ga[NV][E], be[NV][E];
    load_row_t<T, NV>(x + r * (int64_t)H, nvec, lane, v);
    load_params<E, NV>(gamma, nvec, lane, ga);
    load_params<E, NV>(beta, nvec, lane, be);
    float mu, rs;
    row_statistics<E, NV>(v, nvec, lane, H, eps, mu, rs);
    if (lane == 0) {
        mean[r] = mu;
        rstd[r] = rs;
    }
    store_normalised<T, NV>(y + r * (int64_t)H, v, ga, be, nvec, lane, mu, rs);
}

template <typename T, int NV>
__global__ void __launch_bounds__(kThreads)
layernorm_backward_pruned_kernel(const float *__restrict__ vals, const int32_t *__restrict__ idx,
                                 const int32_t *__restrict__ row_ptr, int64_t k, const float *__restrict__ rstd,
                                 const float *__restrict__ gamma, const T *__restrict__ dy, int64_t rows, int H,
                                 T *__restrict__ dx)
{
    constexpr int E = RowIO<T>::E;
    extern __shared__ __align__(16) float lds[];             // kWaves rows of H floats
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r = (int64_t)blockIdx.x * kWaves + wave;
    if (r >= rows) return;
    float *buf = lds + (size_t)wave * H;
    const int nvec = H / E;
    const int64_t e0 = r * (int64_t)H;

    float g[NV][E], ga[NV][E];
    load_row_t<T, NV>(dy + e0, nvec, lane, g);
    load_params<E, NV>(gamma, nvec, lane, ga);

    // the row's pairs: [row_ptr[r], row_ptr[r + 1]) of the index-ordered list
    int64_t p0 = min(max((int64_t)row_ptr[r], (int64_t)0), k);
    int64_t p1 = min(max((int64_t)row_ptr[r + 1], p0), min(k, p0 + H));

    const float scale = rstd[r] / (float)H;
    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
#pragma unroll
        for (int e = 0; e < E; ++e) g[i][e] = (ga[i][e] * g[i][e]) * scale;
        part += sum_vec<E>(g[i]);
        const int q = i * kWave + lane;
        if (q < nvec) {
#pragma unroll
            for (int c = 0; c < E / 4; ++c)
                reinterpret_cast<f32x4 *>(buf)[q * (E / 4) + c] = f32x4{g[i][4 * c], g[i][4 * c + 1], g[i][4 * c + 2], g[i][4 * c + 3]};
        }
    }
    const float sum_g = wave_sum_f32(part);
    __builtin_amdgcn_wave_barrier();                          // LDS serves a wave's accesses in order

    // the row's pairs: the first kKeep * 64 stay in registers for both uses below
    constexpr int kKeep = 4;
    int kept_col[kKeep];
    float kept_val[kKeep];
#pragma unroll
    for (int u = 0; u < kKeep; ++u) {
        const int64_t s = p0 + u * kWave + lane;
        kept_col[u] = -1;
        kept_val[u] = 0.0f;
        if (s < p1) {
            const int64_t c = (int64_t)idx[s] - e0;
            kept_col[u] = (c >= 0 && c < H) ? (int)c : -1;
            kept_val[u] = vals[s];
        }
    }
    part = 0.0f;
#pragma unroll
    for (int u = 0; u < kKeep; ++u)
        if (kept_col[u] >= 0) part += buf[kept_col[u]] * kept_val[u];
    for (int64_t s = p0 + kKeep * kWave + lane; s < p1; s += kWave) {
        const int64_t c = (int64_t)idx[s] - e0;
        if (c >= 0 && c < H) part += buf[c] * vals[s];
    }
    const float sum_gx = wave_sum_f32(part);
    __builtin_amdgcn_wave_barrier();

    const float fH = (float)H;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
#pragma unroll
            for (int c = 0; c < E / 4; ++c)
                reinterpret_cast<f32x4 *>(buf)[q * (E / 4) + c] =
                    f32x4{fH * g[i][4 * c] - sum_g, fH * g[i][4 * c + 1] - sum_g, fH * g[i][4 * c + 2] - sum_g,
                          fH * g[i][4 * c + 3] - sum_g};
        }
    }
    __builtin_amdgcn_wave_barrier();
    // distinct columns: no two lanes touch one slot
#pragma unroll
    for (int u = 0; u < kKeep; ++u)
        if (kept_col[u] >= 0) buf[kept_col[u]] -= kept_val[u] * sum_gx;
    for (int64_t s = p0 + kKeep * kWave + lane; s < p1; s += kWave) {
        const int64_t c = (int64_t)idx[s] - e0;
        if (c >= 0 && c < H) buf[c] -= vals[s] * sum_gx;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
            float o[E];
            load_f32<E>(buf, q, o);
            RowIO<T>::store(dx + e0, q, o);
        }
    }
}

// Shared back end of the two dense backward kernels: xt holds x~ (zeros in padding vectors), g holds y^.
template <typename T, int NV>
__device__ __forceinline__ void backward_from_xt(float (&xt)[NV][RowIO<T>::E], float (&g)[NV][RowIO<T>::E],
                                                 const float (&ga)[NV][RowIO<T>::E], int nvec, int lane, int H, float rs,
                                                 T *dxrow)
{
    constexpr int E = RowIO<T>::E;
    const float scale = rs / (float)H;
    float part_g = 0.0f, part_gx = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        float gx[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            g[i][e] = (ga[i][e] * g[i][e]) * scale;
            gx[e] = g[i][e] * xt[i][e];
        }
        part_g += sum_vec<E>(g[i]);
        part_gx += sum_vec<E>(gx);
    }
    const float sum_g = wave_sum_f32(part_g);
    const float sum_gx = wave_sum_f32(part_gx);
    const float fH = (float)H;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
            float o[E];
#pragma unroll
            for (int e = 0; e < E; ++e) o[e] = (fH * g[i][e] - sum_g) - xt[i][e] * sum_gx;
            RowIO<T>::store(dxrow, q, o);
        }
    }
}

template <typename T, int NV>
__global__ void __launch_bounds__(kThreads)
layernorm_backward_kernel(const T *__restrict__ x, const float *__restrict__ mean, const float *__restrict__ rstd,
                          const float *__restrict__ gamma, const T *__restrict__ dy, int64_t rows, int H,
                          T *__restrict__ dx)
{
    constexpr int E = RowIO<T>::E;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int nvec = H / E;
    float xt[NV][E], g[NV][E], ga[NV][E];
    load_row_t<T, NV>(x + r * (int64_t)H, nvec, lane, xt);
    load_row_t<T, NV>(dy + r * (int64_t)H, nvec, lane, g);
    load_params<E, NV>(gamma, nvec, lane, ga);
    const float mu = mean[r], rs = rstd[r];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const bool in = i * kWave + lane < nvec;                 // padding vectors hold zeros: x~ must be 0 there too
#pragma unroll
        for (int e = 0; e < E; ++e) xt[i][e] = in ? (xt[i][e] - mu) * rs : 0.0f;
    }
    backward_from_xt<T, NV>(xt, g, ga, nvec, lane, H, rs, dx + r * (int64_t)H);
}

// ---- LayerNorm with the low-bit cache of its input fused in ------------------------------
// Forward: the wave that holds a row for the statistics also quantises it (Alg. 2, one
// scale per `block` consecutive elements = G = block / 4 consecutive lanes of one of its
// vectors, the block maximum a DPP butterfly) and stores codes and scales, so the input is
// read once for both.  H is a multiple of block, hence every block lies inside one row
// and the codes are those of the flat quantiser.
// Backward: x^ = code * scale is rebuilt in registers and goes straight into the dense
// input-gradient formula; it is never stored.
// the E codes of a vector, element i in bits [i*BITS, (i+1)*BITS) of the 64-bit result (two words)
template <int BITS, int E>
__device__ __forceinline__ void pack_codes(const float (&f)[E], float mult, uint32_t (&w)[2])
{
    w[0] = w[1] = 0u;
#pragma unroll
    for (int i = 0; i < E; ++i) {
        const uint32_t c = (uint32_t)quantise_one<BITS>(f[i], mult) & ((1u << BITS) - 1u);
        w[(i * BITS) / 32] |= c << ((i * BITS) % 32);
    }
}

template <typename T, int NV, int BITS>
__global__ void __launch_bounds__(kThreads)
layernorm_forward_quant_kernel(const T *__restrict__ x, const float *__restrict__ gamma,
                               const float *__restrict__ beta, int64_t rows, int H, float eps, int G, int block_shift,
                               T *__restrict__ y, float *__restrict__ mean, float *__restrict__ rstd,
                               uint8_t *__restrict__ codes, float *__restrict__ scales)
{
    constexpr int E = RowIO<T>::E;
    constexpr int OUT_BYTES = E * BITS / 8;                  // 2, 4 or 8
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;                                   // whole waves leave: the lane exchanges below stay complete
    const int nvec = H / E;
    const int64_t e0 = r * (int64_t)H;
    float v[NV][E], ga[NV][E], be[NV][E];
    load_row_t<T, NV>(x + e0, nvec, lane, v);
    load_params<E, NV>(gamma, nvec, lane, ga);
    load_params<E, NV>(beta, nvec, lane, be);

    // the cache: codes and scales of this row's blocks (writing it after y instead makes no measurable difference)
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < E; ++e) a = fmaxf(a, fabsf(v[i][e]));
        a = group_max_f32_dyn(a, G);
        float mult, scale;
        block_scale<BITS>(a, mult, scale);
        if (q < nvec) {
            const int64_t el = e0 + (int64_t)q * E;
            if ((lane & (G - 1)) == 0) scales[el >> block_shift] = scale;
            uint32_t w[2];
            pack_codes<BITS, E>(v[i], mult, w);
            uint8_t *dst = codes + (el * BITS) / 8;
            if (OUT_BYTES == 2) __builtin_nontemporal_store((uint16_t)w[0], reinterpret_cast<uint16_t *>(dst));
            else if (OUT_BYTES == 4) __builtin_nontemporal_store(w[0], reinterpret_cast<uint32_t *>(dst));
            else __builtin_nontemporal_store(u32x2{w[0], w[1]}, reinterpret_cast<u32x2 *>(dst));
        }
    }

    float mu, rs;
    row_statistics<E, NV>(v, nvec, lane, H, eps, mu, rs);
    if (lane == 0) {
        mean[r] = mu;
        rstd[r] = rs;
    }
    store_normalised<T, NV>(y + e0, v, ga, be, nvec, lane, mu, rs);
}

template <typename T, int NV, int BITS>
__global__ void __launch_bounds__(kThreads)
layernorm_backward_dequant_kernel(const uint8_t *__restrict__ codes, const float *__restrict__ scales, int block_shift,
                                  const float *__restrict__ mean, const float *__restrict__ rstd,
                                  const float *__restrict__ gamma, const T *__restrict__ dy, int64_t rows, int H,
                                  T *__restrict__ dx)
{
    constexpr int E = RowIO<T>::E;
    constexpr int IN_BYTES = E * BITS / 8;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int nvec = H / E;
    const int64_t e0 = r * (int64_t)H;
    float g[NV][E], ga[NV][E], xt[NV][E];
    uint32_t w[NV][2];
    float sc[NV];
    load_row_t<T, NV>(dy + e0, nvec, lane, g);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        w[i][0] = w[i][1] = 0u;
        sc[i] = 0.0f;
        if (q < nvec) {
            const int64_t el = e0 + (int64_t)q * E;
            const uint8_t *src = codes + (el * BITS) / 8;
            if (IN_BYTES == 2) w[i][0] = __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(src));
            else if (IN_BYTES == 4) w[i][0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(src));
            else {
                const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(src));
                w[i][0] = t.x;
                w[i][1] = t.y;
            }
            sc[i] = scales[el >> block_shift];
        }
    }
    load_params<E, NV>(gamma, nvec, lane, ga);
    const float mu = mean[r], rs = rstd[r];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const bool in = i * kWave + lane < nvec;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const float xh = (float)code_field<BITS>(w[i][(e * BITS) / 32], e % (32 / BITS)) * sc[i];   // one fp32 multiply
            xt[i][e] = in ? (xh - mu) * rs : 0.0f;
        }
    }
    backward_from_xt<T, NV>(xt, g, ga, nvec, lane, H, rs, dx + e0);
}

// ---- parameter gradients of an active LayerNorm: column sums over all rows --------------
// gamma^_j = sum_r x~_rj * y^_rj,  beta^_j = sum_r y^_rj.  A workgroup owns a slab of
// kSlabRows consecutive rows and a group of 256 columns: lane l of every wave holds the
// 16-byte column vector l of the group (a wave reads 1 KiB of a row at a time), the four
// waves take every fourth row of the slab, accumulate in fp32 and are added in wave order
// through LDS; one partial per slab and column goes to the workspace.  The second kernel adds
// the slabs' partials in fp64 in a fixed order.  No atomics: the result does not depend on
// scheduling.  (Smaller slabs fill the chip better but leave more partials to the second
// kernel, which then dominates: 64-row slabs of whole rows took 0.093 ms, 16-row ones 0.185.)
constexpr int kSlabRows = 256;
constexpr int kGroupVecs = kWave;           // column vectors per workgroup: 256 columns (fp32), 512 (bf16)

template <typename T>
__global__ void __launch_bounds__(kThreads)
param_grad_partials_kernel(const T *__restrict__ x, const float *__restrict__ mean, const float *__restrict__ rstd,
                           const T *__restrict__ dy, int64_t rows, int H, int groups, float *__restrict__ partials)
{
    constexpr int E = RowIO<T>::E;
    __shared__ float red_g[kWaves][kWave][E], red_b[kWaves][kWave][E];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nvec = H / E;
    const int64_t slab = blockIdx.x / groups;
    const int group = blockIdx.x % groups;
    const int q = group * kGroupVecs + lane;                   // this lane's column vector
    const bool mine = q < nvec;
    const int64_t r0 = slab * kSlabRows;
    const int n_rows = (int)min((int64_t)kSlabRows, rows - r0);
    float sg[E], sb[E];
#pragma unroll
    for (int e = 0; e < E; ++e) sg[e] = sb[e] = 0.0f;
    constexpr int kRowsInFlight = 4;
    for (int i0 = wave; i0 < n_rows; i0 += kWaves * kRowsInFlight) {          // wave-uniform
        float xv[kRowsInFlight][E], gv[kRowsInFlight][E];
        float mu[kRowsInFlight], rs[kRowsInFlight];
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            const int64_t r = min(r0 + i0 + u * kWaves, rows - 1);            // a row past the slab is re-read, not used
            mu[u] = mean[r];                                                  // uniform: scalar loads
            rs[u] = rstd[r];
#pragma unroll
            for (int e = 0; e < E; ++e) xv[u][e] = gv[u][e] = 0.0f;
            if (mine) {
                RowIO<T>::load(x + r * (int64_t)H, q, xv[u]);
                RowIO<T>::load(dy + r * (int64_t)H, q, gv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            if (i0 + u * kWaves < n_rows) {                                   // wave-uniform; rows add in order
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    sg[e] += ((xv[u][e] - mu[u]) * rs[u]) * gv[u][e];
                    sb[e] += gv[u][e];
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < E; ++e) {
        red_g[wave][lane][e] = sg[e];
        red_b[wave][lane][e] = sb[e];
    }
    __syncthreads();
    if (wave == 0 && mine) {
        // partials: [slab][2][H]
        float *pg = partials + slab * 2 * H + (int64_t)q * E, *pb = pg + H;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float tg = red_g[0][lane][e], tb = red_b[0][lane][e];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) {
                tg += red_g[w][lane][e];
                tb += red_b[w][lane][e];
            }
            pg[e] = tg;
            pb[e] = tb;
        }
    }
}

// 32 columns (of the 2H outputs: gamma^ then beta^) per workgroup; the 8 groups of 32 threads take every
// eighth slab each and their fp64 sums are added in group order.
constexpr int kFinishCols = 32;
constexpr int kFinishGroups = kThreads / kFinishCols;
__global__ void __launch_bounds__(kThreads)
param_grad_finish_kernel(const float *__restrict__ partials, int64_t slabs, int H, float *__restrict__ dgamma,
                         float *__restrict__ dbeta)
{
    __shared__ double part[kFinishGroups][kFinishCols];
    const int c = threadIdx.x % kFinishCols, grp = threadIdx.x / kFinishCols;
    const int col = blockIdx.x * kFinishCols + c;               // 0 .. 2H-1; 2H is a multiple of 8, not always of 32
    double acc = 0.0;
    if (col < 2 * H)
        for (int64_t s = grp; s < slabs; s += kFinishGroups) acc += (double)partials[s * 2 * H + col];
    part[grp][c] = acc;
    __syncthreads();
    if (grp == 0 && col < 2 * H) {
        double total = 0.0;
#pragma unroll
        for (int g = 0; g < kFinishGroups; ++g) total += part[g][c];
        if (col < H) dgamma[col] = (float)total;
        else dbeta[col - H] = (float)total;
    }
}

int32_t validate(int64_t rows, int64_t H, int32_t dt = SLIMFIT_F32)
{
    if (!dtype_ok(dt)) return SLIMFIT_ERR_INVALID_ARG;
    const int64_t epv = dt == SLIMFIT_F32 ? 4 : 8;             // elements per 16-byte vector
    if (rows < 0 || H < epv || H % epv != 0) return SLIMFIT_ERR_INVALID_ARG;
    if (H > kMaxH || rows * H > 0x7FFFFFFFLL) return SLIMFIT_ERR_UNSUPPORTED;
    return SLIMFIT_OK;
}

int32_t validate_quant(int64_t H, int32_t bits, int32_t block)
{
    if (bits != 4 && bits != 8) return SLIMFIT_ERR_UNSUPPORTED;
    if (block != 32 && block != 64 && block != 128 && block != 256) return SLIMFIT_ERR_UNSUPPORTED;
    if (H % block != 0) return SLIMFIT_ERR_UNSUPPORTED;        // a block must not straddle two rows
    return SLIMFIT_OK;
}

// vectors a lane has to hold for rows of H elements
int lane_vectors(int64_t H, int32_t dt = SLIMFIT_F32)
{
    const int64_t epv = dt == SLIMFIT_F32 ? 4 : 8;
    return (int)((H / epv + kWave - 1) / kWave);
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

#define SLIMFIT_LN_DISPATCH(NVEXPR, CALL)        \
    do {                                         \
        const int nv_ = (NVEXPR);                \
        if (nv_ <= 1) { constexpr int NV = 1; CALL; }        \
        else if (nv_ <= 2) { constexpr int NV = 2; CALL; }   \
        else if (nv_ <= 3) { constexpr int NV = 3; CALL; }   \
        else if (nv_ <= 4) { constexpr int NV = 4; CALL; }   \
        else if (nv_ <= 8) { constexpr int NV = 8; CALL; }   \
        else { constexpr int NV = 16; CALL; }                \
    } while (0)
// the same over the element type: CALL sees the type TT and NV (a bf16 row of 4096 elements is 8 vectors a lane)
#define SLIMFIT_LN_DISPATCH_T(DT, H, CALL)                                        \
    do {                                                                          \
        if ((DT) == SLIMFIT_F32) { using TT = float; SLIMFIT_LN_DISPATCH(lane_vectors(H, DT), CALL); }         \
        else { using TT = uint16_t; SLIMFIT_LN_DISPATCH(lane_vectors(H, DT), CALL); }                          \
    } while (0)

extern "C" int32_t slimfit_layernorm_forward(const void *x, int32_t dt, const float *gamma, const float *beta,
                                             int64_t rows, int64_t H, float eps, void *y, float *mean, float *rstd,
                                             void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(rows, H, dt);
    if (rc != SLIMFIT_OK) return rc;
    if (!(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    if (rows == 0) return SLIMFIT_OK;
    if (!x || !gamma || !beta || !y || !mean || !rstd || x == y) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(x, 16) || !aligned_to(y, 16) || !aligned_to(gamma, 16) || !aligned_to(beta, 16) ||
        !aligned_to(mean, 4) || !aligned_to(rstd, 4))
        return SLIMFIT_ERR_ALIGNMENT;
    const size_t nbytes = (size_t)rows * (size_t)H * dtype_size(dt);
    if ((rc = check_device_range(x, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(y, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(gamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(beta, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((rows + kWaves - 1) / kWaves);
    SLIMFIT_LN_DISPATCH_T(dt, H, (layernorm_forward_kernel<TT, NV><<<grid, kThreads, 0, s>>>(
                                     static_cast<const TT *>(x), gamma, beta, rows, (int)H, eps, static_cast<TT *>(y), mean,
                                     rstd)));
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_backward_pruned(const float *vals, const int32_t *idx, const int32_t *row_ptr,
                                                     int64_t k, const float *rstd, const float *gamma, const void *dy,
                                                     int32_t dt, int64_t rows, int64_t H, void *dx, void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(rows, H, dt);
    if (rc != SLIMFIT_OK) return rc;
    if (k < 0 || k > rows * H) return SLIMFIT_ERR_INVALID_ARG;
    if (rows == 0) return SLIMFIT_OK;
    if (!row_ptr || !rstd || !gamma || !dy || !dx || dy == dx || (k > 0 && (!vals || !idx)))
        return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(dy, 16) || !aligned_to(dx, 16) || !aligned_to(gamma, 16) || !aligned_to(rstd, 4) ||
        !aligned_to(row_ptr, 4) || (k > 0 && (!aligned_to(vals, 4) || !aligned_to(idx, 4))))
        return SLIMFIT_ERR_ALIGNMENT;
    const int64_t n = rows * H;
    const size_t nbytes = (size_t)n * dtype_size(dt);
    if ((rc = check_device_range(dy, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dx, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(gamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(row_ptr, (size_t)(rows + 1) * 4)) != SLIMFIT_OK) return rc;
    if (k > 0) {
        if ((rc = check_device_range(vals, (size_t)k * 4)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(idx, (size_t)k * 4)) != SLIMFIT_OK) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((rows + kWaves - 1) / kWaves);
    const size_t lds_bytes = (size_t)kWaves * (size_t)H * 4;              // at most 64 KB
    SLIMFIT_LN_DISPATCH_T(dt, H, (layernorm_backward_pruned_kernel<TT, NV><<<grid, kThreads, lds_bytes, s>>>(
                                     vals, idx, row_ptr, k, rstd, gamma, static_cast<const TT *>(dy), rows, (int)H,
                                     static_cast<TT *>(dx))));
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_param_grads_workspace(int64_t rows, int64_t H, size_t *bytes)
{
    int32_t rc = validate(rows, H);
    if (rc != SLIMFIT_OK) return rc;
    if (!bytes) return SLIMFIT_ERR_INVALID_ARG;
    const int64_t slabs = (rows + kSlabRows - 1) / kSlabRows;
    *bytes = (size_t)(slabs > 0 ? slabs : 1) * 2 * (size_t)H * 4;
    return SLIMFIT_OK;
}

extern "C" int32_t slimfit_layernorm_param_grads(const void *x, int32_t dt, const float *mean, const float *rstd,
                                                 const void *dy, int64_t rows, int64_t H, float *dgamma, float *dbeta,
                                                 void *workspace, size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(rows, H, dt);
    if (rc != SLIMFIT_OK) return rc;
    if (!dgamma || !dbeta || !workspace || (rows > 0 && (!x || !mean || !rstd || !dy))) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(dgamma, 4) || !aligned_to(dbeta, 4) || !aligned_to(workspace, 16) ||
        (rows > 0 && (!aligned_to(x, 16) || !aligned_to(dy, 16) || !aligned_to(mean, 4) || !aligned_to(rstd, 4))))
        return SLIMFIT_ERR_ALIGNMENT;
    size_t need = 0;
    slimfit_layernorm_param_grads_workspace(rows, H, &need);
    if (workspace_bytes < need) return SLIMFIT_ERR_WORKSPACE;
    if ((rc = check_device_range(dgamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dbeta, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(workspace, need)) != SLIMFIT_OK) return rc;
    if (rows > 0) {
        const size_t nbytes = (size_t)rows * (size_t)H * dtype_size(dt);
        if ((rc = check_device_range(x, nbytes)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(dy, nbytes)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t slabs = (rows + kSlabRows - 1) / kSlabRows;
    float *partials = static_cast<float *>(workspace);
    const int64_t epv = dt == SLIMFIT_F32 ? 4 : 8;
    const int groups = (int)((H / epv + kGroupVecs - 1) / kGroupVecs);
    if (slabs > 0) {
        if (dt == SLIMFIT_F32)
            param_grad_partials_kernel<float><<<(unsigned)(slabs * groups), kThreads, 0, s>>>(
                static_cast<const float *>(x), mean, rstd, static_cast<const float *>(dy), rows, (int)H, groups, partials);
        else
            param_grad_partials_kernel<uint16_t><<<(unsigned)(slabs * groups), kThreads, 0, s>>>(
                static_cast<const uint16_t *>(x), mean, rstd, static_cast<const uint16_t *>(dy), rows, (int)H, groups,
                partials);
    }
    const unsigned fgrid = (unsigned)((2 * H + kFinishCols - 1) / kFinishCols);
    param_grad_finish_kernel<<<fgrid, kThreads, 0, s>>>(partials, slabs, (int)H, dgamma, dbeta);
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_backward(const void *x, int32_t dt, const float *mean, const float *rstd,
                                              const float *gamma, const void *dy, int64_t rows, int64_t H, void *dx,
                                              void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(rows, H, dt);
    if (rc != SLIMFIT_OK) return rc;
    if (rows == 0) return SLIMFIT_OK;
    if (!x || !mean || !rstd || !gamma || !dy || !dx || dx == x || dx == dy) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(x, 16) || !aligned_to(dy, 16) || !aligned_to(dx, 16) || !aligned_to(gamma, 16) ||
        !aligned_to(mean, 4) || !aligned_to(rstd, 4))
        return SLIMFIT_ERR_ALIGNMENT;
    const size_t nbytes = (size_t)rows * (size_t)H * dtype_size(dt);
    if ((rc = check_device_range(x, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dy, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dx, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(gamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((rows + kWaves - 1) / kWaves);
    SLIMFIT_LN_DISPATCH_T(dt, H, (layernorm_backward_kernel<TT, NV><<<grid, kThreads, 0, s>>>(
                                     static_cast<const TT *>(x), mean, rstd, gamma, static_cast<const TT *>(dy), rows, (int)H,
                                     static_cast<TT *>(dx))));
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_forward_quant_pack(const void *x, int32_t dt, const float *gamma,
                                                        const float *beta, int64_t rows, int64_t H, float eps,
                                                        int32_t bits, int32_t block, void *y, float *mean, float *rstd,
                                                        uint8_t *codes, float *scales, void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(rows, H, dt);
    if (rc != SLIMFIT_OK) return rc;
    if ((rc = validate_quant(H, bits, block)) != SLIMFIT_OK) return rc;
    if (!(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    if (rows == 0) return SLIMFIT_OK;
    if (!x || !gamma || !beta || !y || !mean || !rstd || !codes || !scales || x == y) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(x, 16) || !aligned_to(y, 16) || !aligned_to(gamma, 16) || !aligned_to(beta, 16) ||
        !aligned_to(mean, 4) || !aligned_to(rstd, 4) || !aligned_to(codes, 16) || !aligned_to(scales, 16))
        return SLIMFIT_ERR_ALIGNMENT;
    const int64_t n = rows * H;
    const size_t nbytes = (size_t)n * dtype_size(dt);
    if ((rc = check_device_range(x, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(y, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(gamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(beta, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(codes, (size_t)(n * bits / 8))) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(scales, (size_t)(n / block) * 4)) != SLIMFIT_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((rows + kWaves - 1) / kWaves);
    const int G = block / (dt == SLIMFIT_F32 ? 4 : 8), shift = __builtin_ctz((unsigned)block);
    if (bits == 4)
        SLIMFIT_LN_DISPATCH_T(dt, H, (layernorm_forward_quant_kernel<TT, NV, 4><<<grid, kThreads, 0, s>>>(
                                         static_cast<const TT *>(x), gamma, beta, rows, (int)H, eps, G, shift,
                                         static_cast<TT *>(y), mean, rstd, codes, scales)));
    else
        SLIMFIT_LN_DISPATCH_T(dt, H, (layernorm_forward_quant_kernel<TT, NV, 8><<<grid, kThreads, 0, s>>>(
                                         static_cast<const TT *>(x), gamma, beta, rows, (int)H, eps, G, shift,
                                         static_cast<TT *>(y), mean, rstd, codes, scales)));
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_backward_dequant(const uint8_t *codes, const float *scales, int32_t bits,
                                                      int32_t block, const float *mean, const float *rstd,
                                                      const float *gamma, const void *dy, int32_t dt, int64_t rows,
                                                      int64_t H, void *dx, void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(rows, H, dt);
    if (rc != SLIMFIT_OK) return rc;
    if ((rc = validate_quant(H, bits, block)) != SLIMFIT_OK) return rc;
    if (rows == 0) return SLIMFIT_OK;
    if (!codes || !scales || !mean || !rstd || !gamma || !dy || !dx || dx == dy) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(codes, 16) || !aligned_to(scales, 16) || !aligned_to(dy, 16) || !aligned_to(dx, 16) ||
        !aligned_to(gamma, 16) || !aligned_to(mean, 4) || !aligned_to(rstd, 4))
        return SLIMFIT_ERR_ALIGNMENT;
    const int64_t n = rows * H;
    const size_t nbytes = (size_t)n * dtype_size(dt);
    if ((rc = check_device_range(dy, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dx, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(gamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(codes, (size_t)(n * bits / 8))) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(scales, (size_t)(n / block) * 4)) != SLIMFIT_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((rows + kWaves - 1) / kWaves);
    const int shift = __builtin_ctz((unsigned)block);
    if (bits == 4)
        SLIMFIT_LN_DISPATCH_T(dt, H, (layernorm_backward_dequant_kernel<TT, NV, 4><<<grid, kThreads, 0, s>>>(
                                         codes, scales, shift, mean, rstd, gamma, static_cast<const TT *>(dy), rows, (int)H,
                                         static_cast<TT *>(dx))));
    else
        SLIMFIT_LN_DISPATCH_T(dt, H, (layernorm_backward_dequant_kernel<TT, NV, 8><<<grid, kThreads, 0, s>>>(
                                         codes, scales, shift, mean, rstd, gamma, static_cast<const TT *>(dy), rows, (int)H,
                                         static_cast<TT *>(dx))));
    return launch_status();
}
