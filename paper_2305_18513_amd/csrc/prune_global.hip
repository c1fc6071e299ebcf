// Alg. 5 applied to a whole flattened tensor (the form the paper uses for the
// standardised input of LayerNorm: keep int(numel * 0.1) entries with their
// indices, restore by zeros + scatter).
//
// A full sort is not needed to know which k entries a descending sort would put
// first: an exact radix select finds the k-th largest key T and how many keys
// equal to T belong to the kept set, and one more sweep emits the survivors in
// ascending index order (ties at T go to the lowest indices).
//
//   keys      order-preserving unsigned images of the elements: |x| as the IEEE
//             bit pattern without its sign (by magnitude) or the usual signed
//             fold with -0 mapped onto +0 (by value); 32 bits for fp32, 16 for
//             bf16.
//   select    most significant digit first, 12 bits a digit (4096 bins): every
//             workgroup histograms its share of the tensor in LDS (ds_add),
//             adds the non-empty bins to one global histogram, and a single
//             workgroup walks the bins from the top to fix the digit and the
//             count still to take below it.  fp32 takes 12+12+8 bits, bf16
//             12+4.  Later digits only count the keys that match the prefix, so
//             their LDS traffic is a few percent of the first sweep's.
//   count     per tile (4096 fp32 / 8192 bf16 elements): keys above T, keys
//             equal to T.
//   scan      one workgroup turns those into each tile's first output slot and
//             the number of ties it may still keep.
//   write     every tile ranks its survivors with a packed wave prefix sum and
//             stores (value, index) pairs at their final places.
//
// The tensors this path is meant for (some 10^6..10^8 elements) stay resident
// in the 256 MB memory-side cache between sweeps, so HBM sees the input about
// once; the cost is the chain of short dependent launches.  No kernel waits on
// another workgroup.
#include "common.hpp"

namespace slimfit {
namespace {

constexpr int kTileThreads = 256;          // count / write kernels: 4 waves
constexpr int kVecPerThread = 4;           // 16-byte vectors a thread holds
constexpr int kDigitBits = 12;
constexpr int kMaxBins = 1 << kDigitBits;
constexpr int kHistThreads = 1024;
constexpr int kSelectThreads = 1024;
constexpr int kScanThreads = 1024;
constexpr int64_t kMinTile = 4096;         // smallest tile (fp32); sizes the workspace

struct State {                             // first 64 bytes of the workspace
    uint32_t prefix;                       // key bits fixed so far
    uint32_t mask;                         // which bits those are
    uint32_t k_rem;                        // entries still to take among the keys matching prefix
    uint32_t T;                            // k-th largest key (after the last digit)
    uint32_t take_eq;                      // how many keys equal to T are kept
    uint32_t pad[11];
};
static_assert(sizeof(State) == 64, "state block");

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int EPV = 4;          // elements per 16-byte vector
    static constexpr int KEYBITS = 32;
};
template <> struct Elem<uint16_t> {
    static constexpr int EPV = 8;
    static constexpr int KEYBITS = 16;
};

// raw element bits -> key (larger key <=> earlier in the descending order)
template <typename T, bool MAG> __device__ __forceinline__ uint32_t make_key(uint32_t bits);
template <> __device__ __forceinline__ uint32_t make_key<float, true>(uint32_t b) { return b << 1; }
template <> __device__ __forceinline__ uint32_t make_key<float, false>(uint32_t b)
{
    b = (b == 0x80000000u) ? 0u : b;                      // -0 orders as +0
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
template <> __device__ __forceinline__ uint32_t make_key<uint16_t, true>(uint32_t h) { return (h << 1) & 0xFFFFu; }
template <> __device__ __forceinline__ uint32_t make_key<uint16_t, false>(uint32_t h)
{
    h = (h == 0x8000u) ? 0u : h;
    return h ^ ((h & 0x8000u) ? 0xFFFFu : 0x8000u);
}

__device__ __forceinline__ uint32_t raw_bits(const float *p) { return __builtin_bit_cast(uint32_t, *p); }
__device__ __forceinline__ uint32_t raw_bits(const uint16_t *p) { return *p; }

// The EPV raw elements of vector `v` (element offset v*EPV); returns how many of
// them lie inside [0, n).  A vector that straddles n is read element by element.
template <typename T>
__device__ __forceinline__ int load_vec(const T *x, int64_t n, int64_t v, uint32_t (&bits)[Elem<T>::EPV])
{
    constexpr int EPV = Elem<T>::EPV;
    const int64_t e0 = v * EPV;
    if (e0 + EPV <= n) {
        const u32x4 w = *reinterpret_cast<const u32x4 *>(x + e0);
        if constexpr (EPV == 4) {
            bits[0] = w.x; bits[1] = w.y; bits[2] = w.z; bits[3] = w.w;
        } else {
            bits[0] = w.x & 0xFFFFu; bits[1] = w.x >> 16;
            bits[2] = w.y & 0xFFFFu; bits[3] = w.y >> 16;
            bits[4] = w.z & 0xFFFFu; bits[5] = w.z >> 16;
            bits[6] = w.w & 0xFFFFu; bits[7] = w.w >> 16;
        }
        return EPV;
    }
    int valid = 0;
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
        bits[e] = 0u;
        if (e0 + e < n) {
            bits[e] = raw_bits(x + e0 + e);
            ++valid;
        }
    }
    return valid;
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v)            // absent sources contribute 0
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}
// inclusive prefix sum over the 64 lanes of a wave
__device__ __forceinline__ uint32_t wave_scan_u32(uint32_t v)
{
    v += dpp_or_zero<0x111, 0xF>(v);       // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);       // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);       // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);       // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);       // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);       // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ uint32_t wave_total_u32(uint32_t inclusive)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)inclusive, 63);
}

// ---- state / histogram reset ------------------------------------------------------
__global__ void __launch_bounds__(kSelectThreads) init_kernel(State *st, uint32_t *hist, uint32_t k)
{
    for (int i = threadIdx.x; i < kMaxBins; i += kSelectThreads) hist[i] = 0u;
    if (threadIdx.x == 0) {
        st->prefix = 0u;
        st->mask = 0u;
        st->k_rem = k;
        st->T = 0u;
        st->take_eq = 0u;
    }
}

// ---- one digit of the select: histogram of the keys that match the prefix ------------
template <typename T, bool MAG>
__global__ void __launch_bounds__(kHistThreads)
hist_kernel(const T *__restrict__ x, int64_t n, const State *__restrict__ st, uint32_t *__restrict__ hist, int shift,
            int nbins)
{
    constexpr int EPV = Elem<T>::EPV;
    __shared__ uint32_t bins[kMaxBins];
    for (int i = threadIdx.x; i < nbins; i += kHistThreads) bins[i] = 0u;
    const uint32_t prefix = st->prefix, mask = st->mask;
    const uint32_t digit_mask = (uint32_t)nbins - 1u;
    __syncthreads();

    const int64_t nvec = (n + EPV - 1) / EPV;
    const int64_t chunk = (int64_t)kHistThreads * kVecPerThread;
    for (int64_t base = (int64_t)blockIdx.x * chunk; base < nvec; base += (int64_t)gridDim.x * chunk) {
        uint32_t bits[kVecPerThread][EPV];
        int valid[kVecPerThread];
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) {
            const int64_t v = base + (int64_t)j * kHistThreads + threadIdx.x;
            valid[j] = 0;
            if (v < nvec) valid[j] = load_vec<T>(x, n, v, bits[j]);
        }
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                if (e < valid[j]) {
                    const uint32_t key = make_key<T, MAG>(bits[j][e]);
                    if ((key & mask) == prefix) atomicAdd(&bins[(key >> shift) & digit_mask], 1u);
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nbins; i += kHistThreads) {
        const uint32_t c = bins[i];
        if (c) atomicAdd(&hist[i], c);
    }
}

// exclusive prefix sum of one value per thread over a workgroup of NT threads
// (NT/64 waves); `total` receives the workgroup's sum.  Two barriers.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_sums, uint32_t &total)
{
    constexpr int NW = NT / kWave;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint32_t incl = wave_scan_u32(v);
    __syncthreads();                                       // wave_sums may still be read from a previous call
    if (lane == kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t before = 0u, sum = 0u;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t s = wave_sums[w];
        before += (w < wave) ? s : 0u;
        sum += s;
    }
    total = sum;
    return before + incl - v;
}

// Walk the bins from the highest digit down: the digit of the k-th largest key
// is the first one whose running count reaches k_rem.  Clears the histogram.
__global__ void __launch_bounds__(kSelectThreads)
select_kernel(State *st, uint32_t *hist, int shift, int nbins, int last)
{
    __shared__ uint32_t wave_sums[kSelectThreads / kWave];
    constexpr int PER = kMaxBins / kSelectThreads;         // 4 bins a thread, highest first
    const uint32_t prefix = st->prefix, mask = st->mask, k_rem = st->k_rem;
    uint32_t h[PER];
    uint32_t mine = 0u;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int r = threadIdx.x * PER + j;               // rank from the top
        const int b = nbins - 1 - r;
        h[j] = 0u;
        if (b >= 0) {
            h[j] = hist[b];
            hist[b] = 0u;
        }
        mine += h[j];
    }
    uint32_t total;
    uint32_t above = block_exclusive_scan<kSelectThreads>(mine, wave_sums, total);
    (void)total;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int b = nbins - 1 - (threadIdx.x * PER + j);
        if (b >= 0 && above < k_rem && k_rem <= above + h[j]) {     // exactly one (thread, j) when k_rem <= #matching keys
            const uint32_t new_prefix = prefix | ((uint32_t)b << shift);
            const uint32_t left = k_rem - above;
            st->prefix = new_prefix;
            st->mask = mask | (((uint32_t)nbins - 1u) << shift);
            st->k_rem = left;
            if (last) {
                st->T = new_prefix;
                st->take_eq = left;
            }
        }
        above += h[j];
    }
}

// vector index of (tile, wave, group j, lane): a wave owns 4 x 64 consecutive vectors
__device__ __forceinline__ int64_t tile_vec(int64_t tile, int wave, int j, int lane)
{
    return tile * (int64_t)(kTileThreads * kVecPerThread) + (int64_t)((wave * kVecPerThread + j) * kWave + lane);
}

// ---- per tile: keys above T, keys equal to T -------------------------------------------
template <typename T, bool MAG>
__global__ void __launch_bounds__(kTileThreads)
count_kernel(const T *__restrict__ x, int64_t n, const State *__restrict__ st, u32x2 *__restrict__ tile_cnt)
{
    constexpr int EPV = Elem<T>::EPV;
    __shared__ uint32_t wave_gt[kTileThreads / kWave], wave_eq[kTileThreads / kWave];
    const uint32_t Tk = st->T;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t nvec = (n + EPV - 1) / EPV;
    uint32_t bits[kVecPerThread][EPV];
    int valid[kVecPerThread];
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const int64_t v = tile_vec(blockIdx.x, wave, j, lane);
        valid[j] = 0;
        if (v < nvec) valid[j] = load_vec<T>(x, n, v, bits[j]);
    }
    uint32_t gt = 0u, eq = 0u;
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (e < valid[j]) {
                const uint32_t key = make_key<T, MAG>(bits[j][e]);
                gt += key > Tk ? 1u : 0u;
                eq += key == Tk ? 1u : 0u;
            }
        }
    }
    const uint32_t packed = wave_total_u32(wave_scan_u32(gt | (eq << 16)));     // a wave holds at most 2048 elements
    if (lane == 0) {
        wave_gt[wave] = packed & 0xFFFFu;
        wave_eq[wave] = packed >> 16;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        u32x2 c = {0u, 0u};
#pragma unroll
        for (int w = 0; w < kTileThreads / kWave; ++w) {
            c.x += wave_gt[w];
            c.y += wave_eq[w];
        }
        tile_cnt[blockIdx.x] = c;
    }
}

// ---- tile counts -> first output slot and tie budget of every tile ----------------------
__global__ void __launch_bounds__(kScanThreads)
scan_kernel(const State *__restrict__ st, const u32x2 *__restrict__ tile_cnt, u32x2 *__restrict__ tile_base,
            int64_t ntiles)
{
    __shared__ uint32_t wave_sums[kScanThreads / kWave];
    const uint32_t take_eq = st->take_eq;
    uint32_t gt_carry = 0u, eq_carry = 0u;
    for (int64_t base = 0; base < ntiles; base += kScanThreads) {
        const int64_t t = base + threadIdx.x;
        u32x2 c = {0u, 0u};
        if (t < ntiles) c = tile_cnt[t];
        uint32_t gt_total, eq_total;
        const uint32_t gt_before = gt_carry + block_exclusive_scan<kScanThreads>(c.x, wave_sums, gt_total);
        const uint32_t eq_before = eq_carry + block_exclusive_scan<kScanThreads>(c.y, wave_sums, eq_total);
        if (t < ntiles) {
            u32x2 b;
            b.x = gt_before + min(eq_before, take_eq);
            b.y = take_eq > eq_before ? take_eq - eq_before : 0u;
            tile_base[t] = b;
        }
        gt_carry += gt_total;
        eq_carry += eq_total;
    }
}

template <typename T> __device__ __forceinline__ void store_raw(T *p, uint32_t bits);
template <> __device__ __forceinline__ void store_raw<float>(float *p, uint32_t bits) { *p = __builtin_bit_cast(float, bits); }
template <> __device__ __forceinline__ void store_raw<uint16_t>(uint16_t *p, uint32_t bits) { *p = (uint16_t)bits; }

// ---- emit the survivors of a tile in ascending index order ------------------------------
template <typename T, bool MAG>
__global__ void __launch_bounds__(kTileThreads)
write_kernel(const T *__restrict__ x, int64_t n, const State *__restrict__ st, const u32x2 *__restrict__ tile_base,
             T *__restrict__ vals, int32_t *__restrict__ idx, uint32_t k)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int NW = kTileThreads / kWave;
    __shared__ uint32_t wave_gt[NW], wave_eq[NW];
    const uint32_t Tk = st->T;
    const u32x2 tb = tile_base[blockIdx.x];
    const uint32_t out_base = tb.x, budget = tb.y;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t nvec = (n + EPV - 1) / EPV;

    uint32_t bits[kVecPerThread][EPV];
    int valid[kVecPerThread];
    uint32_t packed[kVecPerThread];                         // per vector: keys above T | keys equal T << 16
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const int64_t v = tile_vec(blockIdx.x, wave, j, lane);
        valid[j] = 0;
        if (v < nvec) valid[j] = load_vec<T>(x, n, v, bits[j]);
    }
    uint32_t incl[kVecPerThread];
    uint32_t wave_packed = 0u;
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        uint32_t gt = 0u, eq = 0u;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (e < valid[j]) {
                const uint32_t key = make_key<T, MAG>(bits[j][e]);
                gt += key > Tk ? 1u : 0u;
                eq += key == Tk ? 1u : 0u;
            }
        }
        packed[j] = gt | (eq << 16);
        incl[j] = wave_scan_u32(packed[j]);                 // at most 512 per group and field
        wave_packed += wave_total_u32(incl[j]);
    }
    if (lane == 0) {
        wave_gt[wave] = wave_packed & 0xFFFFu;
        wave_eq[wave] = wave_packed >> 16;
    }
    __syncthreads();
    uint32_t run_gt = 0u, run_eq = 0u;                      // survivors / ties of this tile ahead of the current group
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        run_gt += (w < wave) ? wave_gt[w] : 0u;
        run_eq += (w < wave) ? wave_eq[w] : 0u;
    }
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const uint32_t excl = incl[j] - packed[j];
        uint32_t my_gt = run_gt + (excl & 0xFFFFu);
        uint32_t my_eq = run_eq + (excl >> 16);
        const int64_t e0 = tile_vec(blockIdx.x, wave, j, lane) * EPV;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (e < valid[j]) {
                const uint32_t key = make_key<T, MAG>(bits[j][e]);
                const bool above = key > Tk;
                const bool tie = key == Tk;
                if (above || (tie && my_eq < budget)) {
                    const uint32_t pos = out_base + my_gt + min(my_eq, budget);
                    if (pos < k) {                          // always true for consistent counts; guards the stores
                        store_raw<T>(vals + pos, bits[j][e]);
                        idx[pos] = (int32_t)(e0 + e);
                    }
                }
                my_gt += above ? 1u : 0u;
                my_eq += tie ? 1u : 0u;
            }
        }
        const uint32_t group = wave_total_u32(incl[j]);
        run_gt += group & 0xFFFFu;
        run_eq += group >> 16;
    }
}

// ---- restore: zeros, then scatter ---------------------------------------------------------
__global__ void __launch_bounds__(kTileThreads) zero_kernel(u32x4 *__restrict__ out, int64_t nvec16, uint8_t *tail, int tail_bytes)
{
    const int64_t v = (int64_t)blockIdx.x * (kTileThreads * kVecPerThread) + threadIdx.x;
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const int64_t i = v + (int64_t)j * kTileThreads;
        if (i < nvec16) out[i] = z;
    }
    if (blockIdx.x == 0 && (int)threadIdx.x < tail_bytes) tail[threadIdx.x] = 0;
}

template <typename T>
__global__ void __launch_bounds__(kTileThreads)
scatter_kernel(const T *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int64_t n, T *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * kTileThreads + threadIdx.x;
    if (i >= k) return;
    const int32_t at = idx[i];
    if (at >= 0 && (int64_t)at < n) out[at] = vals[i];
}

template <typename T, bool MAG>
void launch_select(const T *x, int64_t n, uint32_t k, T *vals, int32_t *idx, State *st, uint32_t *hist, u32x2 *tile_cnt,
                   u32x2 *tile_base, hipStream_t s)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int KEYBITS = Elem<T>::KEYBITS;
    const int64_t nvec = (n + EPV - 1) / EPV;
    const int64_t chunk = (int64_t)kHistThreads * kVecPerThread;
    const int64_t nchunks = (nvec + chunk - 1) / chunk;
    const unsigned hist_grid = (unsigned)(nchunks < 1024 ? nchunks : 1024);
    const int64_t tile_vecs = (int64_t)kTileThreads * kVecPerThread;
    const int64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;

    init_kernel<<<1, kSelectThreads, 0, s>>>(st, hist, k);
    int hi = KEYBITS;
    while (hi > 0) {
        const int bits = hi >= kDigitBits ? kDigitBits : hi;
        const int shift = hi - bits;
        hist_kernel<T, MAG><<<hist_grid, kHistThreads, 0, s>>>(x, n, st, hist, shift, 1 << bits);
        select_kernel<<<1, kSelectThreads, 0, s>>>(st, hist, shift, 1 << bits, shift == 0 ? 1 : 0);
        hi = shift;
    }
    count_kernel<T, MAG><<<(unsigned)ntiles, kTileThreads, 0, s>>>(x, n, st, tile_cnt);
    scan_kernel<<<1, kScanThreads, 0, s>>>(st, tile_cnt, tile_base, ntiles);
    write_kernel<T, MAG><<<(unsigned)ntiles, kTileThreads, 0, s>>>(x, n, st, tile_base, vals, idx, k);
}

size_t workspace_bytes_for(int64_t n)
{
    const int64_t ntiles = (n + kMinTile - 1) / kMinTile;
    return sizeof(State) + (size_t)kMaxBins * 4 + (size_t)ntiles * 16;
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

extern "C" int32_t slimfit_prune_global_workspace(int64_t n, size_t *bytes)
{
    if (!bytes || n < 0 || n > 0x7FFFFFFFLL) return SLIMFIT_ERR_INVALID_ARG;
    *bytes = workspace_bytes_for(n);
    return SLIMFIT_OK;
}

extern "C" int32_t slimfit_prune_global(const void *x, int32_t dt, int64_t n, int64_t k, int32_t by_magnitude,
                                        void *vals, int32_t *idx, void *workspace, size_t workspace_bytes,
                                        void *stream)
{
    if (!dtype_ok(dt) || n < 0 || k < 0 || k > n) return SLIMFIT_ERR_INVALID_ARG;
    if (n > 0x7FFFFFFFLL) return SLIMFIT_ERR_UNSUPPORTED;                 // indices are int32
    if (k == 0) return SLIMFIT_OK;
    if (!x || !vals || !idx || !workspace) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    if (!aligned_to(x, 16) || !aligned_to(vals, esz) || !aligned_to(idx, 4) || !aligned_to(workspace, 16))
        return SLIMFIT_ERR_ALIGNMENT;
    const size_t need = workspace_bytes_for(n);
    if (workspace_bytes < need) return SLIMFIT_ERR_WORKSPACE;
    int32_t rc;
    if ((rc = check_device_range(x, (size_t)n * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(vals, (size_t)k * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(idx, (size_t)k * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(workspace, need)) != SLIMFIT_OK) return rc;

    char *ws = static_cast<char *>(workspace);
    State *st = reinterpret_cast<State *>(ws);
    uint32_t *hist = reinterpret_cast<uint32_t *>(ws + sizeof(State));
    const int64_t slots = (n + kMinTile - 1) / kMinTile;
    u32x2 *tile_cnt = reinterpret_cast<u32x2 *>(ws + sizeof(State) + (size_t)kMaxBins * 4);
    u32x2 *tile_base = tile_cnt + slots;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t kk = (uint32_t)k;
    if (dt == SLIMFIT_F32) {
        const float *xf = static_cast<const float *>(x);
        float *vf = static_cast<float *>(vals);
        if (by_magnitude) launch_select<float, true>(xf, n, kk, vf, idx, st, hist, tile_cnt, tile_base, s);
        else launch_select<float, false>(xf, n, kk, vf, idx, st, hist, tile_cnt, tile_base, s);
    } else {
        const uint16_t *xh = static_cast<const uint16_t *>(x);
        uint16_t *vh = static_cast<uint16_t *>(vals);
        if (by_magnitude) launch_select<uint16_t, true>(xh, n, kk, vh, idx, st, hist, tile_cnt, tile_base, s);
        else launch_select<uint16_t, false>(xh, n, kk, vh, idx, st, hist, tile_cnt, tile_base, s);
    }
    return launch_status();
}

extern "C" int32_t slimfit_restore_global(const void *vals, const int32_t *idx, int64_t k, int32_t dt, int64_t n,
                                          void *out, void *stream)
{
    if (!dtype_ok(dt) || n < 0 || k < 0 || k > n) return SLIMFIT_ERR_INVALID_ARG;
    if (n > 0x7FFFFFFFLL) return SLIMFIT_ERR_UNSUPPORTED;
    if (n == 0) return SLIMFIT_OK;
    if (!out || (k > 0 && (!vals || !idx))) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    if (!aligned_to(out, 16) || (k > 0 && (!aligned_to(vals, esz) || !aligned_to(idx, 4)))) return SLIMFIT_ERR_ALIGNMENT;
    int32_t rc;
    if ((rc = check_device_range(out, (size_t)n * esz)) != SLIMFIT_OK) return rc;
    if (k > 0) {
        if ((rc = check_device_range(vals, (size_t)k * esz)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(idx, (size_t)k * 4)) != SLIMFIT_OK) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t bytes = (size_t)n * esz;
    const int64_t nvec16 = (int64_t)(bytes / 16);
    const int tail_bytes = (int)(bytes % 16);
    const int64_t per_block = (int64_t)kTileThreads * kVecPerThread;
    int64_t zblocks = (nvec16 + per_block - 1) / per_block;
    if (zblocks < 1) zblocks = 1;
    zero_kernel<<<(unsigned)zblocks, kTileThreads, 0, s>>>(static_cast<u32x4 *>(out), nvec16,
                                                          static_cast<uint8_t *>(out) + (size_t)nvec16 * 16, tail_bytes);
    if (k > 0) {
        const unsigned sblocks = (unsigned)((k + kTileThreads - 1) / kTileThreads);
        if (dt == SLIMFIT_F32)
            scatter_kernel<float><<<sblocks, kTileThreads, 0, s>>>(static_cast<const float *>(vals), idx, k, n,
                                                                   static_cast<float *>(out));
        else
            scatter_kernel<uint16_t><<<sblocks, kTileThreads, 0, s>>>(static_cast<const uint16_t *>(vals), idx, k, n,
                                                                      static_cast<uint16_t *>(out));
    }
    return launch_status();
}
