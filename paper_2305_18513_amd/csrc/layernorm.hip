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

constexpr int kThreads = 256;
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

template <int NV>
__global__ void __launch_bounds__(kThreads)
layernorm_forward_kernel(const float *__restrict__ x, const float *__restrict__ gamma, const float *__restrict__ beta,
                         int64_t rows, int H, float eps, float *__restrict__ y, float *__restrict__ mean,
                         float *__restrict__ rstd)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int nvec = H / 4;
    f32x4 v[NV], ga[NV], be[NV];
    load_row<NV>(x + r * (int64_t)H, nvec, lane, v, true);
    load_row<NV>(gamma, nvec, lane, ga, false);
    load_row<NV>(beta, nvec, lane, be, false);

    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) part += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    const float mu = wave_sum_f32(part) / (float)H;
    part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const bool in = i * kWave + lane < nvec;             // padding vectors must not add mu^2
        const float a = v[i].x - mu, b = v[i].y - mu, c = v[i].z - mu, d = v[i].w - mu;
        part += in ? (a * a + b * b) + (c * c + d * d) : 0.0f;
    }
    const float var = wave_sum_f32(part) / (float)H;
    const float rs = 1.0f / __builtin_sqrtf(var + eps);
    if (lane == 0) {
        mean[r] = mu;
        rstd[r] = rs;
    }
    f32x4 *dst = reinterpret_cast<f32x4 *>(y + r * (int64_t)H);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
            f32x4 o;
            o.x = ((v[i].x - mu) * rs) * ga[i].x + be[i].x;
            o.y = ((v[i].y - mu) * rs) * ga[i].y + be[i].y;
            o.z = ((v[i].z - mu) * rs) * ga[i].z + be[i].z;
            o.w = ((v[i].w - mu) * rs) * ga[i].w + be[i].w;
            __builtin_nontemporal_store(o, dst + q);
        }
    }
}

template <int NV>
__global__ void __launch_bounds__(kThreads)
layernorm_backward_pruned_kernel(const float *__restrict__ vals, const int32_t *__restrict__ idx,
                                 const int32_t *__restrict__ row_ptr, int64_t k, const float *__restrict__ rstd,
                                 const float *__restrict__ gamma, const float *__restrict__ dy, int64_t rows, int H,
                                 float *__restrict__ dx)
{
    extern __shared__ __align__(16) float lds[];             // kWaves rows of H floats
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r = (int64_t)blockIdx.x * kWaves + wave;
    if (r >= rows) return;
    float *buf = lds + (size_t)wave * H;
    const int nvec = H / 4;
    const int64_t e0 = r * (int64_t)H;

    f32x4 g[NV], ga[NV];
    load_row<NV>(dy + e0, nvec, lane, g, true);
    load_row<NV>(gamma, nvec, lane, ga, false);

    // the row's pairs: [row_ptr[r], row_ptr[r + 1]) of the index-ordered list
    int64_t p0 = min(max((int64_t)row_ptr[r], (int64_t)0), k);
    int64_t p1 = min(max((int64_t)row_ptr[r + 1], p0), min(k, p0 + H));

    const float scale = rstd[r] / (float)H;
    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        g[i].x = (ga[i].x * g[i].x) * scale;
        g[i].y = (ga[i].y * g[i].y) * scale;
        g[i].z = (ga[i].z * g[i].z) * scale;
        g[i].w = (ga[i].w * g[i].w) * scale;
        part += (g[i].x + g[i].y) + (g[i].z + g[i].w);
        const int q = i * kWave + lane;
        if (q < nvec) reinterpret_cast<f32x4 *>(buf)[q] = g[i];
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
            f32x4 o;
            o.x = fH * g[i].x - sum_g;
            o.y = fH * g[i].y - sum_g;
            o.z = fH * g[i].z - sum_g;
            o.w = fH * g[i].w - sum_g;
            reinterpret_cast<f32x4 *>(buf)[q] = o;
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
    f32x4 *dst = reinterpret_cast<f32x4 *>(dx + e0);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) __builtin_nontemporal_store(reinterpret_cast<const f32x4 *>(buf)[q], dst + q);
    }
}

// ---- input gradient of an active LayerNorm: the row formula with every x~ present ----------
template <int NV>
__global__ void __launch_bounds__(kThreads)
layernorm_backward_kernel(const float *__restrict__ x, const float *__restrict__ mean, const float *__restrict__ rstd,
                          const float *__restrict__ gamma, const float *__restrict__ dy, int64_t rows, int H,
                          float *__restrict__ dx)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int nvec = H / 4;
    f32x4 xt[NV], g[NV], ga[NV];
    load_row<NV>(x + r * (int64_t)H, nvec, lane, xt, true);
    load_row<NV>(dy + r * (int64_t)H, nvec, lane, g, true);
    load_row<NV>(gamma, nvec, lane, ga, false);
    const float mu = mean[r], rs = rstd[r];
    const float scale = rs / (float)H;
    float part_g = 0.0f, part_gx = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const bool in = i * kWave + lane < nvec;                 // padding vectors hold zeros: x~ must be 0 there too
        xt[i].x = in ? (xt[i].x - mu) * rs : 0.0f;
        xt[i].y = in ? (xt[i].y - mu) * rs : 0.0f;
        xt[i].z = in ? (xt[i].z - mu) * rs : 0.0f;
        xt[i].w = in ? (xt[i].w - mu) * rs : 0.0f;
        g[i].x = (ga[i].x * g[i].x) * scale;
        g[i].y = (ga[i].y * g[i].y) * scale;
        g[i].z = (ga[i].z * g[i].z) * scale;
        g[i].w = (ga[i].w * g[i].w) * scale;
        part_g += (g[i].x + g[i].y) + (g[i].z + g[i].w);
        part_gx += (g[i].x * xt[i].x + g[i].y * xt[i].y) + (g[i].z * xt[i].z + g[i].w * xt[i].w);
    }
    const float sum_g = wave_sum_f32(part_g);
    const float sum_gx = wave_sum_f32(part_gx);
    const float fH = (float)H;
    f32x4 *dst = reinterpret_cast<f32x4 *>(dx + r * (int64_t)H);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
            f32x4 o;
            o.x = (fH * g[i].x - sum_g) - xt[i].x * sum_gx;
            o.y = (fH * g[i].y - sum_g) - xt[i].y * sum_gx;
            o.z = (fH * g[i].z - sum_g) - xt[i].z * sum_gx;
            o.w = (fH * g[i].w - sum_g) - xt[i].w * sum_gx;
            __builtin_nontemporal_store(o, dst + q);
        }
    }
}

// ---- LayerNorm with the low-bit cache of its input fused in ------------------------------
// Forward: the wave that holds a row for the statistics also quantises it (Alg. 2, one
// scale per `block` consecutive elements = G = block / 4 consecutive lanes of one of its
// vectors, the block maximum a DPP butterfly) and stores codes and scales, so the input is
// read once for both.  H is a multiple of block, hence every block lies inside one row
// and the codes are those of the flat quantiser.
// Backward: x^ = code * scale is rebuilt in registers and goes straight into the dense
// input-gradient formula; it is never stored.
template <int BITS>
__device__ __forceinline__ uint32_t pack4(const f32x4 &v, float mult)
{
    constexpr uint32_t m = (1u << BITS) - 1u;
    return ((uint32_t)quantise_one<BITS>(v.x, mult) & m) | (((uint32_t)quantise_one<BITS>(v.y, mult) & m) << BITS) |
           (((uint32_t)quantise_one<BITS>(v.z, mult) & m) << (2 * BITS)) |
           (((uint32_t)quantise_one<BITS>(v.w, mult) & m) << (3 * BITS));
}

template <int NV, int BITS>
__global__ void __launch_bounds__(kThreads)
layernorm_forward_quant_kernel(const float *__restrict__ x, const float *__restrict__ gamma,
                               const float *__restrict__ beta, int64_t rows, int H, float eps, int G, int block_shift,
                               float *__restrict__ y, float *__restrict__ mean, float *__restrict__ rstd,
                               uint8_t *__restrict__ codes, float *__restrict__ scales)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;                                   // whole waves leave: the lane exchanges below stay complete
    const int nvec = H / 4;
    const int64_t e0 = r * (int64_t)H;
    f32x4 v[NV], ga[NV], be[NV];
    load_row<NV>(x + e0, nvec, lane, v, true);
    load_row<NV>(gamma, nvec, lane, ga, false);
    load_row<NV>(beta, nvec, lane, be, false);

    // the cache: codes and scales of this row's blocks
    auto write_cache = [&]() {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        float a = fmaxf(fmaxf(fabsf(v[i].x), fabsf(v[i].y)), fmaxf(fabsf(v[i].z), fabsf(v[i].w)));
        a = group_max_f32_dyn(a, G);
        float mult, scale;
        block_scale<BITS>(a, mult, scale);
        if (q < nvec) {
            const int64_t e = e0 + (int64_t)q * 4;
            if ((lane & (G - 1)) == 0) scales[e >> block_shift] = scale;
            const uint32_t w = pack4<BITS>(v[i], mult);
            if (BITS == 4) __builtin_nontemporal_store((uint16_t)w, reinterpret_cast<uint16_t *>(codes + e / 2));
            else __builtin_nontemporal_store(w, reinterpret_cast<uint32_t *>(codes + e));
        }
    }
    };
    write_cache();       // before or after the y stores makes no measurable difference

    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) part += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    const float mu = wave_sum_f32(part) / (float)H;
    part = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const bool in = i * kWave + lane < nvec;
        const float a = v[i].x - mu, b = v[i].y - mu, c = v[i].z - mu, d = v[i].w - mu;
        part += in ? (a * a + b * b) + (c * c + d * d) : 0.0f;
    }
    const float var = wave_sum_f32(part) / (float)H;
    const float rs = 1.0f / __builtin_sqrtf(var + eps);
    if (lane == 0) {
        mean[r] = mu;
        rstd[r] = rs;
    }
    f32x4 *dst = reinterpret_cast<f32x4 *>(y + e0);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
            f32x4 o;
            o.x = ((v[i].x - mu) * rs) * ga[i].x + be[i].x;
            o.y = ((v[i].y - mu) * rs) * ga[i].y + be[i].y;
            o.z = ((v[i].z - mu) * rs) * ga[i].z + be[i].z;
            o.w = ((v[i].w - mu) * rs) * ga[i].w + be[i].w;
            __builtin_nontemporal_store(o, dst + q);
        }
    }
}

template <int NV, int BITS>
__global__ void __launch_bounds__(kThreads)
layernorm_backward_dequant_kernel(const uint8_t *__restrict__ codes, const float *__restrict__ scales, int block_shift,
                                  const float *__restrict__ mean, const float *__restrict__ rstd,
                                  const float *__restrict__ gamma, const float *__restrict__ dy, int64_t rows, int H,
                                  float *__restrict__ dx)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int nvec = H / 4;
    const int64_t e0 = r * (int64_t)H;
    f32x4 g[NV], ga[NV];
    uint32_t w[NV];
    float sc[NV];
    load_row<NV>(dy + e0, nvec, lane, g, true);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        w[i] = 0u;
        sc[i] = 0.0f;
        if (q < nvec) {
            const int64_t e = e0 + (int64_t)q * 4;
            if (BITS == 4) w[i] = __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(codes + e / 2));
            else w[i] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(codes + e));
            sc[i] = scales[e >> block_shift];
        }
    }
    load_row<NV>(gamma, nvec, lane, ga, false);
    const float mu = mean[r], rs = rstd[r];
    const float scale = rs / (float)H;
    f32x4 xt[NV];
    float part_g = 0.0f, part_gx = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const bool in = i * kWave + lane < nvec;
        xt[i].x = in ? ((float)code_field<BITS>(w[i], 0) * sc[i] - mu) * rs : 0.0f;
        xt[i].y = in ? ((float)code_field<BITS>(w[i], 1) * sc[i] - mu) * rs : 0.0f;
        xt[i].z = in ? ((float)code_field<BITS>(w[i], 2) * sc[i] - mu) * rs : 0.0f;
        xt[i].w = in ? ((float)code_field<BITS>(w[i], 3) * sc[i] - mu) * rs : 0.0f;
        g[i].x = (ga[i].x * g[i].x) * scale;
        g[i].y = (ga[i].y * g[i].y) * scale;
        g[i].z = (ga[i].z * g[i].z) * scale;
        g[i].w = (ga[i].w * g[i].w) * scale;
        part_g += (g[i].x + g[i].y) + (g[i].z + g[i].w);
        part_gx += (g[i].x * xt[i].x + g[i].y * xt[i].y) + (g[i].z * xt[i].z + g[i].w * xt[i].w);
    }
    const float sum_g = wave_sum_f32(part_g);
    const float sum_gx = wave_sum_f32(part_gx);
    const float fH = (float)H;
    f32x4 *dst = reinterpret_cast<f32x4 *>(dx + e0);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int q = i * kWave + lane;
        if (q < nvec) {
            f32x4 o;
            o.x = (fH * g[i].x - sum_g) - xt[i].x * sum_gx;
            o.y = (fH * g[i].y - sum_g) - xt[i].y * sum_gx;
            o.z = (fH * g[i].z - sum_g) - xt[i].z * sum_gx;
            o.w = (fH * g[i].w - sum_g) - xt[i].w * sum_gx;
            __builtin_nontemporal_store(o, dst + q);
        }
    }
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
constexpr int kGroupVecs = kWave;           // column vectors per workgroup: 256 columns

__global__ void __launch_bounds__(kThreads)
param_grad_partials_kernel(const float *__restrict__ x, const float *__restrict__ mean, const float *__restrict__ rstd,
                           const float *__restrict__ dy, int64_t rows, int H, int groups, float *__restrict__ partials)
{
    __shared__ f32x4 red_g[kWaves][kWave], red_b[kWaves][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nvec = H / 4;
    const int64_t slab = blockIdx.x / groups;
    const int group = blockIdx.x % groups;
    const int q = group * kGroupVecs + lane;                   // this lane's column vector
    const bool mine = q < nvec;
    const int64_t r0 = slab * kSlabRows;
    const int n_rows = (int)min((int64_t)kSlabRows, rows - r0);
    f32x4 sg = {0.0f, 0.0f, 0.0f, 0.0f}, sb = {0.0f, 0.0f, 0.0f, 0.0f};
    constexpr int kRowsInFlight = 4;
    for (int i0 = wave; i0 < n_rows; i0 += kWaves * kRowsInFlight) {          // wave-uniform
        f32x4 xv[kRowsInFlight], gv[kRowsInFlight];
        float mu[kRowsInFlight], rs[kRowsInFlight];
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            const int64_t r = min(r0 + i0 + u * kWaves, rows - 1);            // a row past the slab is re-read, not used
            mu[u] = mean[r];                                                  // uniform: scalar loads
            rs[u] = rstd[r];
            xv[u] = gv[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if (mine) {
                xv[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(x + r * (int64_t)H) + q);
                gv[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(dy + r * (int64_t)H) + q);
            }
        }
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            if (i0 + u * kWaves < n_rows) {                                   // wave-uniform; rows add in order
                sg.x += ((xv[u].x - mu[u]) * rs[u]) * gv[u].x;
                sg.y += ((xv[u].y - mu[u]) * rs[u]) * gv[u].y;
                sg.z += ((xv[u].z - mu[u]) * rs[u]) * gv[u].z;
                sg.w += ((xv[u].w - mu[u]) * rs[u]) * gv[u].w;
                sb.x += gv[u].x;
                sb.y += gv[u].y;
                sb.z += gv[u].z;
                sb.w += gv[u].w;
            }
        }
    }
    red_g[wave][lane] = sg;
    red_b[wave][lane] = sb;
    __syncthreads();
    if (wave == 0 && mine) {
        f32x4 tg = red_g[0][lane], tb = red_b[0][lane];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) {
            tg += red_g[w][lane];
            tb += red_b[w][lane];
        }
        // partials: [slab][2][H]
        reinterpret_cast<f32x4 *>(partials + slab * 2 * H)[q] = tg;
        reinterpret_cast<f32x4 *>(partials + slab * 2 * H + H)[q] = tb;
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

int32_t validate(int64_t rows, int64_t H)
{
    if (rows < 0 || H < 4 || H % 4 != 0) return SLIMFIT_ERR_INVALID_ARG;
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
int lane_vectors(int64_t H) { return (int)((H / 4 + kWave - 1) / kWave); }

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

extern "C" int32_t slimfit_layernorm_forward(const float *x, const float *gamma, const float *beta, int64_t rows,
                                             int64_t H, float eps, float *y, float *mean, float *rstd, void *stream)
{
    int32_t rc = validate(rows, H);
    if (rc != SLIMFIT_OK) return rc;
    if (!(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    if (rows == 0) return SLIMFIT_OK;
    if (!x || !gamma || !beta || !y || !mean || !rstd || x == y) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(x, 16) || !aligned_to(y, 16) || !aligned_to(gamma, 16) || !aligned_to(beta, 16) ||
        !aligned_to(mean, 4) || !aligned_to(rstd, 4))
        return SLIMFIT_ERR_ALIGNMENT;
    const size_t nbytes = (size_t)rows * (size_t)H * 4;
    if ((rc = check_device_range(x, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(y, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(gamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(beta, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((rows + kWaves - 1) / kWaves);
    SLIMFIT_LN_DISPATCH(lane_vectors(H), (layernorm_forward_kernel<NV><<<grid, kThreads, 0, s>>>(
                                             x, gamma, beta, rows, (int)H, eps, y, mean, rstd)));
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_backward_pruned(const float *vals, const int32_t *idx, const int32_t *row_ptr,
                                                     int64_t k, const float *rstd, const float *gamma, const float *dy,
                                                     int64_t rows, int64_t H, float *dx, void *stream)
{
    int32_t rc = validate(rows, H);
    if (rc != SLIMFIT_OK) return rc;
    if (k < 0 || k > rows * H) return SLIMFIT_ERR_INVALID_ARG;
    if (rows == 0) return SLIMFIT_OK;
    if (!row_ptr || !rstd || !gamma || !dy || !dx || dy == dx || (k > 0 && (!vals || !idx)))
        return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(dy, 16) || !aligned_to(dx, 16) || !aligned_to(gamma, 16) || !aligned_to(rstd, 4) ||
        !aligned_to(row_ptr, 4) || (k > 0 && (!aligned_to(vals, 4) || !aligned_to(idx, 4))))
        return SLIMFIT_ERR_ALIGNMENT;
    const int64_t n = rows * H;
    if ((rc = check_device_range(dy, (size_t)n * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dx, (size_t)n * 4)) != SLIMFIT_OK) return rc;
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
    SLIMFIT_LN_DISPATCH(lane_vectors(H), (layernorm_backward_pruned_kernel<NV><<<grid, kThreads, lds_bytes, s>>>(
                                             vals, idx, row_ptr, k, rstd, gamma, dy, rows, (int)H, dx)));
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

extern "C" int32_t slimfit_layernorm_param_grads(const float *x, const float *mean, const float *rstd, const float *dy,
                                                 int64_t rows, int64_t H, float *dgamma, float *dbeta, void *workspace,
                                                 size_t workspace_bytes, void *stream)
{
    int32_t rc = validate(rows, H);
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
        const size_t nbytes = (size_t)rows * (size_t)H * 4;
        if ((rc = check_device_range(x, nbytes)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(dy, nbytes)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t slabs = (rows + kSlabRows - 1) / kSlabRows;
    float *partials = static_cast<float *>(workspace);
    const int groups = (int)((H / 4 + kGroupVecs - 1) / kGroupVecs);
    if (slabs > 0)
        param_grad_partials_kernel<<<(unsigned)(slabs * groups), kThreads, 0, s>>>(x, mean, rstd, dy, rows, (int)H, groups,
                                                                                   partials);
    const unsigned fgrid = (unsigned)((2 * H + kFinishCols - 1) / kFinishCols);
    param_grad_finish_kernel<<<fgrid, kThreads, 0, s>>>(partials, slabs, (int)H, dgamma, dbeta);
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_backward(const float *x, const float *mean, const float *rstd, const float *gamma,
                                              const float *dy, int64_t rows, int64_t H, float *dx, void *stream)
{
    int32_t rc = validate(rows, H);
    if (rc != SLIMFIT_OK) return rc;
    if (rows == 0) return SLIMFIT_OK;
    if (!x || !mean || !rstd || !gamma || !dy || !dx || dx == x || dx == dy) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(x, 16) || !aligned_to(dy, 16) || !aligned_to(dx, 16) || !aligned_to(gamma, 16) ||
        !aligned_to(mean, 4) || !aligned_to(rstd, 4))
        return SLIMFIT_ERR_ALIGNMENT;
    const size_t nbytes = (size_t)rows * (size_t)H * 4;
    if ((rc = check_device_range(x, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dy, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dx, nbytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(gamma, (size_t)H * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(mean, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(rstd, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned grid = (unsigned)((rows + kWaves - 1) / kWaves);
    SLIMFIT_LN_DISPATCH(lane_vectors(H), (layernorm_backward_kernel<NV><<<grid, kThreads, 0, s>>>(
                                             x, mean, rstd, gamma, dy, rows, (int)H, dx)));
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_forward_quant_pack(const float *x, const float *gamma, const float *beta,
                                                        int64_t rows, int64_t H, float eps, int32_t bits, int32_t block,
                                                        float *y, float *mean, float *rstd, uint8_t *codes,
                                                        float *scales, void *stream)
{
    int32_t rc = validate(rows, H);
    if (rc != SLIMFIT_OK) return rc;
    if ((rc = validate_quant(H, bits, block)) != SLIMFIT_OK) return rc;
    if (!(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    if (rows == 0) return SLIMFIT_OK;
    if (!x || !gamma || !beta || !y || !mean || !rstd || !codes || !scales || x == y) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(x, 16) || !aligned_to(y, 16) || !aligned_to(gamma, 16) || !aligned_to(beta, 16) ||
        !aligned_to(mean, 4) || !aligned_to(rstd, 4) || !aligned_to(codes, 16) || !aligned_to(scales, 16))
        return SLIMFIT_ERR_ALIGNMENT;
    const int64_t n = rows * H;
    const size_t nbytes = (size_t)n * 4;
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
    const int G = block / 4, shift = __builtin_ctz((unsigned)block);
    if (bits == 4)
        SLIMFIT_LN_DISPATCH(lane_vectors(H), (layernorm_forward_quant_kernel<NV, 4><<<grid, kThreads, 0, s>>>(
                                                 x, gamma, beta, rows, (int)H, eps, G, shift, y, mean, rstd, codes, scales)));
    else
        SLIMFIT_LN_DISPATCH(lane_vectors(H), (layernorm_forward_quant_kernel<NV, 8><<<grid, kThreads, 0, s>>>(
                                                 x, gamma, beta, rows, (int)H, eps, G, shift, y, mean, rstd, codes, scales)));
    return launch_status();
}

extern "C" int32_t slimfit_layernorm_backward_dequant(const uint8_t *codes, const float *scales, int32_t bits,
                                                      int32_t block, const float *mean, const float *rstd,
                                                      const float *gamma, const float *dy, int64_t rows, int64_t H,
                                                      float *dx, void *stream)
{
    int32_t rc = validate(rows, H);
    if (rc != SLIMFIT_OK) return rc;
    if ((rc = validate_quant(H, bits, block)) != SLIMFIT_OK) return rc;
    if (rows == 0) return SLIMFIT_OK;
    if (!codes || !scales || !mean || !rstd || !gamma || !dy || !dx || dx == dy) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(codes, 16) || !aligned_to(scales, 16) || !aligned_to(dy, 16) || !aligned_to(dx, 16) ||
        !aligned_to(gamma, 16) || !aligned_to(mean, 4) || !aligned_to(rstd, 4))
        return SLIMFIT_ERR_ALIGNMENT;
    const int64_t n = rows * H;
    const size_t nbytes = (size_t)n * 4;
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
        SLIMFIT_LN_DISPATCH(lane_vectors(H), (layernorm_backward_dequant_kernel<NV, 4><<<grid, kThreads, 0, s>>>(
                                                 codes, scales, shift, mean, rstd, gamma, dy, rows, (int)H, dx)));
    else
        SLIMFIT_LN_DISPATCH(lane_vectors(H), (layernorm_backward_dequant_kernel<NV, 8><<<grid, kThreads, 0, s>>>(
                                                 codes, scales, shift, mean, rstd, gamma, dy, rows, (int)H, dx)));
    return launch_status();
}
