// Pruning of score rows to (values, indices) and its inverse (Alg. 5 and the
// appendix on pruning), for gfx950.
//
// The paper sorts the whole input to find the largest 10 %.  A sort is not
// needed for that: the kept set is {p > T} plus the first few {p == T} in
// column order, where T is the k-th largest value of the row.  One wavefront
// owns one row at a time and keeps it in registers (lane l holds columns
// l, l+64, ...).  T is found by bisection over the order-preserving integer
// image of the floats between the row's minimum and maximum; every probe is
// one v_cmp per held element whose lane mask is popcounted on the scalar
// unit, and the search stops as soon as a probe is passed by exactly k
// entries.  Survivors are compacted in ascending column order with
// mask-prefix counts (mbcnt), so no LDS and no atomics are involved.
// Rows wider than the register path are handled by a workgroup-per-row
// kernel with the same logic that re-reads the row from cache for each probe.
#include "common.hpp"

#include <cfloat>
#include <cmath>

namespace slimfit {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
constexpr int kMaxRegSlots = 16;             // register path: cols <= 64 * 16

template <typename T> struct Elem;
template <> struct Elem<float> {
    __device__ static float load(const float *p) { return *p; }
    __device__ static float raw(float f) { return f; }
    __device__ static float zero() { return 0.0f; }
};
template <> struct Elem<uint16_t> {
    __device__ static float load(const uint16_t *p) { return bf16_widen(*p); }
    __device__ static uint16_t raw(float f) { return (uint16_t)(__builtin_bit_cast(uint32_t, f) >> 16); }
    __device__ static uint16_t zero() { return 0; }
};

__device__ __forceinline__ int popc64(uint64_t m) { return __builtin_popcountll(m); }

// ---------------------------------------------------------------------------
// register path: one wave per row, M slots per lane
// ---------------------------------------------------------------------------
template <typename T, int M>
__global__ __launch_bounds__(kThreads) void prune_rows_kernel(const T *__restrict__ p, int64_t rows, int cols, int k,
                                                              int mode, float tau, T *__restrict__ vals,
                                                              uint16_t *__restrict__ idx, int32_t *__restrict__ counts)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * kWavesPerBlock;
    const float ninf = -__builtin_inff(), pinf = __builtin_inff();

    for (int64_t row = wave0; row < rows; row += n_waves) {      // wave-uniform trip count
        const T *src = p + row * (int64_t)cols;
        float f[M];
        bool valid[M];
        // every load is issued (absent columns re-read the last one) so that
        // all of a row's loads are in flight together
#pragma unroll
        for (int j = 0; j < M; ++j) {
            const int col = j * kWave + lane;
            valid[j] = col < cols;
            f[j] = Elem<T>::load(src + (valid[j] ? col : cols - 1));
        }
        float lmax = ninf, lmin = pinf;
#pragma unroll
        for (int j = 0; j < M; ++j) {
            f[j] = valid[j] ? f[j] : ninf;
            lmax = fmaxf(lmax, f[j]);
            lmin = fminf(lmin, valid[j] ? f[j] : pinf);
        }

        auto count_ge = [&](float t) {
            int c = 0;
#pragma unroll
            for (int j = 0; j < M; ++j) c += popc64(__builtin_amdgcn_ballot_w64(f[j] >= t));
            return c;
        };

        int kk = k;                  // pairs to keep for this row
        float T_cut = 0.0f;
        int c_ge = 0;
        bool have_cut = false;
        if (mode == SLIMFIT_PRUNE_THRESHOLD) {
            const int c_tau = count_ge(tau);
            if (c_tau <= k) { kk = c_tau; T_cut = tau; c_ge = c_tau; have_cut = true; }
        }
        if (!have_cut) {
            uint32_t lo = wave_min_u32(float_to_key(lmin));
            uint32_t hi = wave_max_u32(float_to_key(lmax));
            const int c_hi = count_ge(key_to_float(hi));
            if (c_hi >= kk) {
                lo = hi;
                c_ge = c_hi;
            } else {
                c_ge = cols;                                     // every entry is >= the minimum
                while (hi - lo > 1u) {                           // at most 32 probes
                    const uint32_t mid = lo + ((hi - lo) >> 1);
                    const int c = count_ge(key_to_float(mid));
                    if (c >= kk) {
                        lo = mid;
                        c_ge = c;
                        if (c == kk) break;                      // the probe separates exactly kk entries
                    } else {
                        hi = mid;
                    }
                }
            }
            T_cut = key_to_float(lo);
        }

        // which entries survive
        bool sel[M];
        if (c_ge == kk) {
#pragma unroll
            for (int j = 0; j < M; ++j) sel[j] = valid[j] && f[j] >= T_cut;
        } else {
            // more than kk entries reach the cut value: all above it, then the
            // equal ones by ascending column until kk are taken
            int c_gt = 0;
#pragma unroll
            for (int j = 0; j < M; ++j) c_gt += popc64(__builtin_amdgcn_ballot_w64(f[j] > T_cut));
            const int need = kk - c_gt;
            int seen = 0;
#pragma unroll
            for (int j = 0; j < M; ++j) {
                const bool eq = valid[j] && f[j] == T_cut;
                const uint64_t eqm = __builtin_amdgcn_ballot_w64(eq);
                const int rank = seen + (int)lanes_below(eqm);
                sel[j] = valid[j] && (f[j] > T_cut || (eq && rank < need));
                seen += popc64(eqm);
            }
        }

        // compaction in ascending column order
        T *ov = vals + row * (int64_t)k;
        uint16_t *oi = idx + row * (int64_t)k;
        int base = 0;
#pragma unroll
        for (int j = 0; j < M; ++j) {
            const uint64_t m = __builtin_amdgcn_ballot_w64(sel[j]);
            const int pos = base + (int)lanes_below(m);
            if (sel[j] && pos < k) {
                ov[pos] = Elem<T>::raw(f[j]);
                oi[pos] = (uint16_t)(j * kWave + lane);
            }
            base += popc64(m);
        }
        for (int s = kk + lane; s < k; s += kWave) {             // THRESHOLD: unused slots
            ov[s] = Elem<T>::zero();
            oi[s] = 0xFFFFu;
        }
        if (counts && lane == 0) counts[row] = kk;
    }
}

// ---------------------------------------------------------------------------
// wide rows: one workgroup per row, the row is re-read for every probe
// ---------------------------------------------------------------------------
struct BlockScratch {
    uint32_t u[kWavesPerBlock];
    int i[kWavesPerBlock];
};

__device__ __forceinline__ int block_sum_int(int v, BlockScratch &s)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    __syncthreads();                         // previous use of the scratch is over
    if ((threadIdx.x & 63) == 0) s.i[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) t += s.i[w];
    return t;
}

__device__ __forceinline__ uint32_t block_max_u32(uint32_t v, BlockScratch &s)
{
    v = wave_max_u32(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s.u[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t t = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) t = max(t, s.u[w]);
    return t;
}

// exclusive prefix of `flag` over the workgroup in thread order; *total = sum
__device__ __forceinline__ int block_prefix(bool flag, int *total, BlockScratch &s)
{
    const uint64_t m = __builtin_amdgcn_ballot_w64(flag);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s.i[wave] = popc64(m);
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        const int c = s.i[w];
        before += (w < wave) ? c : 0;
        all += c;
    }
    *total = all;
    return before + (int)lanes_below(m);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void prune_rows_wide_kernel(const T *__restrict__ p, int64_t rows, int cols,
                                                                   int k, int mode, float tau, T *__restrict__ vals,
                                                                   uint16_t *__restrict__ idx,
                                                                   int32_t *__restrict__ counts)
{
    __shared__ BlockScratch scratch;
    const int tid = threadIdx.x;
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {        // block-uniform
        const T *src = p + row * (int64_t)cols;

        auto count_ge = [&](float t) {
            int c = 0;
            for (int col = tid; col < cols; col += kThreads) c += Elem<T>::load(src + col) >= t ? 1 : 0;
            return block_sum_int(c, scratch);
        };

        int kk = k;
        float T_cut = 0.0f;
        int c_ge = 0;
        bool have_cut = false;
        if (mode == SLIMFIT_PRUNE_THRESHOLD) {
            const int c_tau = count_ge(tau);
            if (c_tau <= k) { kk = c_tau; T_cut = tau; c_ge = c_tau; have_cut = true; }
        }
        if (!have_cut) {
            float lmax = -__builtin_inff(), lmin = __builtin_inff();
            for (int col = tid; col < cols; col += kThreads) {
                const float v = Elem<T>::load(src + col);
                lmax = fmaxf(lmax, v);
                lmin = fminf(lmin, v);
            }
            uint32_t hi = block_max_u32(float_to_key(lmax), scratch);
            uint32_t lo = ~block_max_u32(~float_to_key(lmin), scratch);
            const int c_hi = count_ge(key_to_float(hi));
            if (c_hi >= kk) {
                lo = hi;
                c_ge = c_hi;
            } else {
                c_ge = cols;
                while (hi - lo > 1u) {                                     // at most 32 probes, block-uniform
                    const uint32_t mid = lo + ((hi - lo) >> 1);
                    const int c = count_ge(key_to_float(mid));
                    if (c >= kk) {
                        lo = mid;
                        c_ge = c;
                        if (c == kk) break;
                    } else {
                        hi = mid;
                    }
                }
            }
            T_cut = key_to_float(lo);
        }

        int need = 0x7FFFFFFF;                                             // equal entries still to take
        if (c_ge != kk) {
            int c = 0;
            for (int col = tid; col < cols; col += kThreads) c += Elem<T>::load(src + col) > T_cut ? 1 : 0;
            need = kk - block_sum_int(c, scratch);
        }

        T *ov = vals + row * (int64_t)k;
        uint16_t *oi = idx + row * (int64_t)k;
        int base = 0, seen_eq = 0;
        for (int c0 = 0; c0 < cols; c0 += kThreads) {                      // tiles in column order
            const int col = c0 + tid;
            const bool in = col < cols;
            const float v = in ? Elem<T>::load(src + col) : 0.0f;
            bool s;
            if (c_ge == kk) {
                s = in && v >= T_cut;
            } else {
                const bool eq = in && v == T_cut;
                int n_eq;
                const int rank = seen_eq + block_prefix(eq, &n_eq, scratch);
                s = in && (v > T_cut || (eq && rank < need));
                seen_eq += n_eq;
            }
            int n_sel;
            const int pos = base + block_prefix(s, &n_sel, scratch);
            if (s && pos < k) {
                ov[pos] = Elem<T>::raw(v);
                oi[pos] = (uint16_t)col;
            }
            base += n_sel;
        }
        for (int s = kk + tid; s < k; s += kThreads) {
            ov[s] = Elem<T>::zero();
            oi[s] = 0xFFFFu;
        }
        if (counts && tid == 0) counts[row] = kk;
    }
}

// ---------------------------------------------------------------------------
// restore: zeros, then scatter (two launches in stream order)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void zero_fill_kernel(uint4 *__restrict__ out16, int64_t n16,
                                                             uint8_t *__restrict__ tail, int n_tail)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t j = i; j < n16; j += stride) out16[j] = make_uint4(0u, 0u, 0u, 0u);
    if (i < n_tail) tail[i] = 0;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void scatter_kernel(const T *__restrict__ vals, const uint16_t *__restrict__ idx,
                                                           const int32_t *__restrict__ counts, int64_t rows, int cols,
                                                           int k, T *__restrict__ out)
{
    const int64_t total = rows * (int64_t)k;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        const int64_t row = i / k;
        const int s = (int)(i - row * k);
        const int cnt = counts ? counts[row] : k;
        const int col = idx[i];
        if (s < cnt && col < cols) out[row * (int64_t)cols + col] = vals[i];
    }
}

template <typename T>
void launch_prune(const void *p, int64_t rows, int cols, int k, int mode, float tau, void *vals, uint16_t *idx,
                  int32_t *counts, hipStream_t st)
{
    const T *pp = static_cast<const T *>(p);
    T *vv = static_cast<T *>(vals);
    const int slots = (cols + kWave - 1) / kWave;
    if (slots > kMaxRegSlots) {
        const unsigned grid = (unsigned)(rows < 16384 ? rows : 16384);
        prune_rows_wide_kernel<T><<<grid, kThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts);
        return;
    }
    const int64_t blocks_needed = (rows + kWavesPerBlock - 1) / kWavesPerBlock;
    const unsigned grid = (unsigned)(blocks_needed < 16384 ? blocks_needed : 16384);
#define SLIMFIT_PRUNE_CASE(MM) \
    prune_rows_kernel<T, MM><<<grid, kThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts)
    if (slots <= 1) SLIMFIT_PRUNE_CASE(1);
    else if (slots <= 2) SLIMFIT_PRUNE_CASE(2);
    else if (slots <= 3) SLIMFIT_PRUNE_CASE(3);
    else if (slots <= 4) SLIMFIT_PRUNE_CASE(4);
    else if (slots <= 6) SLIMFIT_PRUNE_CASE(6);
    else if (slots <= 8) SLIMFIT_PRUNE_CASE(8);
    else if (slots <= 12) SLIMFIT_PRUNE_CASE(12);
    else SLIMFIT_PRUNE_CASE(16);
#undef SLIMFIT_PRUNE_CASE
}

int32_t validate(int32_t dt, int64_t rows, int32_t cols, int32_t k)
{
    if (!dtype_ok(dt) || rows < 0 || cols < 1 || k < 1 || k > cols) return SLIMFIT_ERR_INVALID_ARG;
    if (cols > 65536) return SLIMFIT_ERR_UNSUPPORTED;
    if (rows > ((int64_t)1 << 40)) return SLIMFIT_ERR_UNSUPPORTED;
    return SLIMFIT_OK;
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

extern "C" int32_t slimfit_keep_count(int32_t cols, int32_t keep_ppm)
{
    if (cols < 0 || keep_ppm < 0 || keep_ppm > 1000000) return -1;
    return (int32_t)(((int64_t)cols * (int64_t)keep_ppm) / 1000000);
}

extern "C" int32_t slimfit_prune_scores(const void *p, int32_t dt, int64_t rows, int32_t cols, int32_t k, int32_t mode,
                                        float tau, void *vals, uint16_t *idx, int32_t *counts, void *stream)
{
    int32_t rc = validate(dt, rows, cols, k);
    if (rc != SLIMFIT_OK) return rc;
    if (mode != SLIMFIT_PRUNE_TOPK && mode != SLIMFIT_PRUNE_THRESHOLD) return SLIMFIT_ERR_INVALID_ARG;
    if (rows == 0) return SLIMFIT_OK;
    if (!p || !vals || !idx) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    if (!aligned_to(p, esz) || !aligned_to(vals, esz) || !aligned_to(idx, 2) || (counts && !aligned_to(counts, 4)))
        return SLIMFIT_ERR_ALIGNMENT;
    if ((rc = check_device_range(p, (size_t)rows * (size_t)cols * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(vals, (size_t)rows * (size_t)k * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(idx, (size_t)rows * (size_t)k * 2)) != SLIMFIT_OK) return rc;
    if (counts && (rc = check_device_range(counts, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    // every finite value passes a threshold of -inf; the kernels mark absent
    // columns with -inf, so use the lowest finite value instead
    if (mode == SLIMFIT_PRUNE_THRESHOLD && tau == -INFINITY) tau = -FLT_MAX;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == SLIMFIT_F32) launch_prune<float>(p, rows, cols, k, mode, tau, vals, idx, counts, st);
    else launch_prune<uint16_t>(p, rows, cols, k, mode, tau, vals, idx, counts, st);
    return launch_status();
}

extern "C" int32_t slimfit_restore_scores(const void *vals, const uint16_t *idx, const int32_t *counts, int32_t dt,
                                          int64_t rows, int32_t cols, int32_t k, void *out, void *stream)
{
    int32_t rc = validate(dt, rows, cols, k);
    if (rc != SLIMFIT_OK) return rc;
    if (rows == 0) return SLIMFIT_OK;
    if (!vals || !idx || !out) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    if (!aligned_to(out, 16) || !aligned_to(vals, esz) || !aligned_to(idx, 2) || (counts && !aligned_to(counts, 4)))
        return SLIMFIT_ERR_ALIGNMENT;
    const size_t out_bytes = (size_t)rows * (size_t)cols * esz;
    if ((rc = check_device_range(out, out_bytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(vals, (size_t)rows * (size_t)k * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(idx, (size_t)rows * (size_t)k * 2)) != SLIMFIT_OK) return rc;
    if (counts && (rc = check_device_range(counts, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t n16 = (int64_t)(out_bytes / 16);
    const int n_tail = (int)(out_bytes % 16);
    int64_t zb = (n16 + kThreads - 1) / kThreads;
    if (zb < 1) zb = 1;
    if (zb > 65536) zb = 65536;
    zero_fill_kernel<<<(unsigned)zb, kThreads, 0, st>>>(static_cast<uint4 *>(out), n16,
                                                         static_cast<uint8_t *>(out) + n16 * 16, n_tail);
    const int64_t total = rows * (int64_t)k;
    int64_t sb = (total + kThreads - 1) / kThreads;
    if (sb > 65536) sb = 65536;
    if (dt == SLIMFIT_F32)
        scatter_kernel<float><<<(unsigned)sb, kThreads, 0, st>>>(static_cast<const float *>(vals), idx, counts, rows,
                                                                 cols, k, static_cast<float *>(out));
    else
        scatter_kernel<uint16_t><<<(unsigned)sb, kThreads, 0, st>>>(static_cast<const uint16_t *>(vals), idx, counts,
                                                                    rows, cols, k, static_cast<uint16_t *>(out));
    return launch_status();
}
