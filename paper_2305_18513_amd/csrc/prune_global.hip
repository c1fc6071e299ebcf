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
//   digit 1   every workgroup histograms the top 12 key bits of its share of
//             the tensor in LDS (ds_add) and adds the non-empty bins to one
//             global histogram; a single workgroup walks the 4096 bins from the
//             top and fixes the bin that holds T and the count still to take
//             from it.
//   bracket   if that bin is small enough (the usual case: a bin is 1/16 of a
//             binade, 1-2 % of a bell-shaped tensor), one sweep counts, per
//             tile, the keys above the bin and files the bin's own keys in the
//             tile's slot of a key list (1/16 of the tile's size; slots are
//             granted from an LDS counter, no global atomics).  The remaining
//             digits (8+12 bits for fp32, 4 for bf16) and the per-tile counts
//             of keys above / equal to T then read the lists only, a wave per
//             tile.  A bin too large for the lists (heavy ties, constant
//             tensors), or a tile whose slot overflows because the bin's keys
//             are bunched, takes the plain route instead: every further digit
//             and the count sweep read the tensor again.
//   scan      one workgroup turns the tile counts into each tile's first output
//             slot and the number of ties it may still keep.
//   write     every tile ranks its survivors with a packed wave prefix sum and
//             stores (value, index) pairs at their final places, plus the
//             optional tile pointers (survivors ahead of every 4096 elements)
//             that let the restoring process run as one pass.
//
// Both routes run the same launches; a kernel looks at the route flag in the
// state block and either returns or picks its source.  No kernel waits on
// another workgroup, and the single-workgroup steps (digit selection, scan) are
// launches of their own: letting the last workgroup of a sweep do them needs an
// agent-scope release in every workgroup, which on this part writes back the
// XCD's whole L2 and made the sweeps 2-25x slower when it was tried.  The tensor is read three times on the list route (digit
// 1, bracket, write) and 2 + number of digits times on the plain one.
#include "common.hpp"

#include <type_traits>

namespace slimfit {
namespace {

constexpr int kTileThreads = 256;          // tile kernels: 4 waves
constexpr int kVecPerThread = 4;           // 16-byte vectors a thread holds
constexpr int kDigitBits = 12;
constexpr int kMaxBins = 1 << kDigitBits;
constexpr int kHistThreads = 1024;
constexpr int kSelectThreads = 1024;
constexpr int kScanThreads = 1024;
constexpr int64_t kPtrTile = SLIMFIT_GLOBAL_TILE;   // granularity of the tile pointers; smallest kernel tile

struct State {                             // first 64 bytes of the workspace
    uint32_t prefix;                       // key bits fixed so far
    uint32_t mask;                         // which bits those are
    uint32_t k_rem;                        // entries still to take among the keys matching prefix
    uint32_t T;                            // k-th largest key (after the last digit)
    uint32_t take_eq;                      // how many keys equal to T are kept
    uint32_t route;                        // 1: digits after the first and the counts read the candidate list
    uint32_t overflow;                     // 1: a tile's list ran out of slots; the lists are not used after all
    uint32_t pad[9];
};
#ifndef SLIMFIT_PG_HIST_GRID
#define SLIMFIT_PG_HIST_GRID 256          // workgroups of a histogram sweep: each adds its non-empty bins with global atomics
#endif
#ifndef SLIMFIT_PG_NT
#define SLIMFIT_PG_NT 0
#endif
constexpr int kListShare = 16;             // a tile's key list holds 1/16 of the tile's element count
__device__ __forceinline__ bool use_list(const State *st) { return st->route != 0u && st->overflow == 0u; }

// bf16 elements that enter the selection widened to fp32: the rows of a bf16 tensor that is standardised
// on the way in (the standardised values are fp32, and so are the kept values)
struct Bf16Row {
    uint16_t h;
};
template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int EPV = 4;          // elements per 16-byte vector
    static constexpr int KEYBITS = 32;
    using Out = float;                     // type of the kept values
    using Key = float;                     // type whose key / digit plan applies
};
template <> struct Elem<uint16_t> {
    static constexpr int EPV = 8;
    static constexpr int KEYBITS = 16;
    static constexpr bool WIDEN = false;
    using Out = uint16_t;
    using Key = uint16_t;
};
template <> struct Elem<Bf16Row> {
    static constexpr int EPV = 8;
    static constexpr int KEYBITS = 32;
    static constexpr bool WIDEN = true;    // raw bits are the fp32 pattern of the widened element
    using Out = float;
    using Key = float;
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
template <> __device__ __forceinline__ uint32_t make_key<Bf16Row, true>(uint32_t b) { return make_key<float, true>(b); }
template <> __device__ __forceinline__ uint32_t make_key<Bf16Row, false>(uint32_t b) { return make_key<float, false>(b); }

__device__ __forceinline__ uint32_t raw_bits(const float *p) { return __builtin_bit_cast(uint32_t, *p); }
__device__ __forceinline__ uint32_t raw_bits(const uint16_t *p) { return *p; }
__device__ __forceinline__ uint32_t raw_bits(const Bf16Row *p) { return (uint32_t)p->h << 16; }
// the eight halves of a 16-byte vector, as they are or widened to fp32 bit patterns
template <bool WIDEN>
__device__ __forceinline__ void split_halves(const u32x4 &w, uint32_t (&bits)[8])
{
    const uint32_t q[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bits[2 * i] = WIDEN ? q[i] << 16 : q[i] & 0xFFFFu;
        bits[2 * i + 1] = WIDEN ? q[i] & 0xFFFF0000u : q[i] >> 16;
    }
}

// The EPV raw elements of vector `v` (element offset v*EPV); returns how many of
// them lie inside [0, n).  A vector that straddles n is read element by element.
template <typename T, bool NT = false>
__device__ __forceinline__ int load_vec(const T *x, int64_t n, int64_t v, uint32_t (&bits)[Elem<T>::EPV])
{
    constexpr int EPV = Elem<T>::EPV;
    const int64_t e0 = v * EPV;
    if (e0 + EPV <= n) {
        const u32x4 w = load_global<NT>(reinterpret_cast<const u32x4 *>(x + e0));
        if constexpr (EPV == 4) {
            bits[0] = w.x; bits[1] = w.y; bits[2] = w.z; bits[3] = w.w;
        } else {
            split_halves<Elem<T>::WIDEN>(w, bits);
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

// INSIDE: the caller has established (uniformly for the workgroup) that every vector it touches lies
// wholly below n, so the load is unconditional and the code after it is straight-line; otherwise the
// vector may straddle n or lie past it.
template <typename T, bool INSIDE, bool NT = false>
__device__ __forceinline__ int load_tile_vec(const T *x, int64_t n, int64_t nvec, int64_t v,
                                             uint32_t (&bits)[Elem<T>::EPV])
{
    constexpr int EPV = Elem<T>::EPV;
    if constexpr (INSIDE) {
        const u32x4 w = load_global<NT>(reinterpret_cast<const u32x4 *>(x + v * EPV));
        if constexpr (EPV == 4) {
            bits[0] = w.x; bits[1] = w.y; bits[2] = w.z; bits[3] = w.w;
        } else {
            split_halves<Elem<T>::WIDEN>(w, bits);
        }
        return EPV;
    } else {
#pragma unroll
        for (int e = 0; e < EPV; ++e) bits[e] = 0u;
        return v < nvec ? load_vec<T, NT>(x, n, v, bits) : 0;
    }
}

// Optional standardisation on the way in (fp32 tensors): element j of row r
// enters the selection as x~ = fl(fl(x - mean[r]) * rstd[r]), two fp32 operations
// that every sweep repeats bit for bit, so the LayerNorm's standardised input is
// pruned without ever being stored.  r = j / H by a multiply-high with a magic
// number (exact for j < 2^31: magic = ceil(2^(31+l) / H), l = ceil(log2 H),
// r = mulhi(j, magic) >> (l - 1)).
struct Std {
    const float *mean, *rstd;
    uint32_t magic, shift;
    uint32_t wave_uniform;       // H is a multiple of 64 vectors: the 64 vectors a wave loads together share a row
    uint32_t last_row;
    uint32_t H;
    int32_t *row_ptr;            // optional output: survivors ahead of every row (rows + 1 entries)
};
// Applied to a vector after all of the thread's loads have been issued, so that
// the loads still overlap.
template <typename T, bool STD>
__device__ __forceinline__ void standardise(uint32_t (&bits)[Elem<T>::EPV], int valid, int64_t v, const Std &sd)
{
    constexpr int EPV = Elem<T>::EPV;
    if constexpr (STD) {
        // H is a multiple of EPV: a vector lies in one row.  No branch on `valid`: a vector past the end
        // takes the last row's statistics and its result is never looked at, and the statistic loads of
        // all of a thread's vectors can be issued together.
        (void)valid;
        uint32_t row = min(__umulhi((uint32_t)(v * EPV), sd.magic) >> sd.shift, sd.last_row);
        if (sd.wave_uniform) row = (uint32_t)__builtin_amdgcn_readfirstlane((int)row);   // scalar loads
        const float mu = sd.mean[row], rs = sd.rstd[row];
#pragma unroll
        for (int e = 0; e < EPV; ++e)
            bits[e] = __builtin_bit_cast(uint32_t, (__builtin_bit_cast(float, bits[e]) - mu) * rs);
    }
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
        st->route = 0u;
        st->overflow = 0u;
    }
}

// ---- one digit of the select: histogram of the keys that match the prefix ------------
// Source: the tensor (first digit, and every digit on the plain route) or the
// candidate list.
template <typename T, bool MAG, bool STD, bool FIRST>
__global__ void __launch_bounds__(kHistThreads)
hist_kernel(const T *__restrict__ x, int64_t n, const State *__restrict__ st, uint32_t *__restrict__ hist,
            const u32x2 *__restrict__ tile_cnt, const uint32_t *__restrict__ lists, int64_t ntiles, int shift, int nbins, Std sd)
{
    constexpr int EPV = Elem<T>::EPV;
    __shared__ uint32_t bins[kMaxBins];
    for (int i = threadIdx.x; i < nbins; i += kHistThreads) bins[i] = 0u;
    const uint32_t prefix = st->prefix, mask = st->mask;
    const uint32_t digit_mask = (uint32_t)nbins - 1u;
    const bool listed = use_list(st);
    __syncthreads();

    if (listed) {
        // a wave per tile list; the tile's count sits in the second word of its counters
        constexpr int64_t kSlot = (int64_t)kTileThreads * kVecPerThread * EPV / kListShare;
        const int lane = threadIdx.x & (kWave - 1);
        const int64_t waves = (int64_t)gridDim.x * (kHistThreads / kWave);
        for (int64_t t = (int64_t)blockIdx.x * (kHistThreads / kWave) + (threadIdx.x >> 6); t < ntiles; t += waves) {
            const uint32_t cnt = min(tile_cnt[t].y, (uint32_t)kSlot);
            const uint32_t *keys = lists + t * kSlot;
            for (uint32_t i = lane; i < cnt; i += kWave) {
                const uint32_t key = keys[i];
                if ((key & mask) == prefix) atomicAdd(&bins[(key >> shift) & digit_mask], 1u);
            }
        }
    } else {
        const int64_t nvec = (n + EPV - 1) / EPV;
        const int64_t nfull = n / EPV;                            // vectors wholly below n
        const int64_t chunk = (int64_t)kHistThreads * kVecPerThread;
        auto sweep = [&](auto inside_tag, int64_t base) {
            constexpr bool INSIDE = decltype(inside_tag)::value;
            uint32_t bits[kVecPerThread][EPV];
            int valid[kVecPerThread];
#pragma unroll
            for (int j = 0; j < kVecPerThread; ++j) {
                const int64_t v = base + (int64_t)j * kHistThreads + threadIdx.x;
                valid[j] = load_tile_vec<T, INSIDE, SLIMFIT_PG_NT != 0>(x, n, nvec, v, bits[j]);
            }
#pragma unroll
            for (int j = 0; j < kVecPerThread; ++j)
                standardise<T, STD>(bits[j], valid[j], base + (int64_t)j * kHistThreads + threadIdx.x, sd);
#pragma unroll
            for (int j = 0; j < kVecPerThread; ++j) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    if (INSIDE || e < valid[j]) {
                        const uint32_t key = make_key<T, MAG>(bits[j][e]);
                        // the first digit counts every key: no prefix to match, no branch around the ds_add
                        if (FIRST || (key & mask) == prefix) atomicAdd(&bins[(key >> shift) & digit_mask], 1u);
                    }
                }
            }
        };
        for (int64_t base = (int64_t)blockIdx.x * chunk; base < nvec; base += (int64_t)gridDim.x * chunk) {
            if (base + chunk <= nfull) sweep(std::true_type{}, base);      // workgroup-uniform
            else sweep(std::false_type{}, base);
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
// After the first digit it also picks the route: the candidate list is used
// when the chosen bin fits into it.
__global__ void __launch_bounds__(kSelectThreads)
select_kernel(State *st, uint32_t *hist, int shift, int nbins, int first, int last, uint32_t cap)
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
            if (first) st->route = (!last && h[j] <= cap) ? 1u : 0u;
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

// ---- list route: per tile, keys above the chosen bin; the bin's own keys go to the tile's list ----
// Leaves tile_cnt[tile] = (keys above the bin, keys filed).
template <typename T, bool MAG, bool STD, bool INSIDE>
__device__ __forceinline__ void
bracket_tile(const T *__restrict__ x, int64_t n, State *st, u32x2 *__restrict__ tile_cnt, uint32_t *__restrict__ lists, Std sd)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr uint32_t kSlot = kTileThreads * kVecPerThread * EPV / kListShare;
    __shared__ uint32_t wave_gt[kTileThreads / kWave];
    __shared__ uint32_t filed;
    if (st->route == 0u) return;
    const uint32_t prefix = st->prefix, mask = st->mask;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t nvec = (n + EPV - 1) / EPV;
    if (threadIdx.x == 0) filed = 0u;
    uint32_t bits[kVecPerThread][EPV];
    int valid[kVecPerThread];
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const int64_t v = tile_vec(blockIdx.x, wave, j, lane);
        valid[j] = load_tile_vec<T, INSIDE>(x, n, nvec, v, bits[j]);
    }
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) standardise<T, STD>(bits[j], valid[j], tile_vec(blockIdx.x, wave, j, lane), sd);
    uint32_t gt = 0u, in_bin = 0u;
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (INSIDE || e < valid[j]) {
                const uint32_t top = make_key<T, MAG>(bits[j][e]) & mask;
                gt += top > prefix ? 1u : 0u;
                in_bin += top == prefix ? 1u : 0u;
            }
        }
    }
    const uint32_t packed = gt | (in_bin << 16);            // a wave holds at most 2048 elements
    const uint32_t incl = wave_scan_u32(packed);
    const uint32_t wave_total = wave_total_u32(incl);
    if (lane == 0) wave_gt[wave] = wave_total & 0xFFFFu;
    const uint32_t wave_filed = wave_total >> 16;
    __syncthreads();                                        // `filed` is zero
    if (wave_filed) {                                       // wave-uniform
        uint32_t base = 0u;
        if (lane == 0) base = atomicAdd(&filed, wave_filed);
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
        uint32_t slot = base + ((incl - packed) >> 16);
        uint32_t *keys = lists + (int64_t)blockIdx.x * kSlot;
#pragma unroll
        for (int j = 0; j < kVecPerThread; ++j) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                if (INSIDE || e < valid[j]) {
                    const uint32_t key = make_key<T, MAG>(bits[j][e]);
                    if ((key & mask) == prefix) {
                        if (slot < kSlot) keys[slot] = key;
                        ++slot;
                    }
                }
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        u32x2 c = {0u, min(filed, kSlot)};
#pragma unroll
        for (int w = 0; w < kTileThreads / kWave; ++w) c.x += wave_gt[w];
        tile_cnt[blockIdx.x] = c;
        if (filed > kSlot) st->overflow = 1u;
    }
}

template <typename T, bool MAG, bool STD>
__global__ void __launch_bounds__(kTileThreads)
bracket_kernel(const T *__restrict__ x, int64_t n, State *st, u32x2 *__restrict__ tile_cnt, uint32_t *__restrict__ lists, Std sd)
{
    // workgroup-uniform: the whole tile lies below n
    constexpr int64_t kTileElems = (int64_t)kTileThreads * kVecPerThread * Elem<T>::EPV;
    if (((int64_t)blockIdx.x + 1) * kTileElems <= n)
        bracket_tile<T, MAG, STD, true>(x, n, st, tile_cnt, lists, sd);
    else
        bracket_tile<T, MAG, STD, false>(x, n, st, tile_cnt, lists, sd);
}

// ---- per tile: keys above T, keys equal to T -------------------------------------------
// plain route: from the tensor; list route: the list's keys are added to the
// counts that bracket_kernel left.
template <typename T, bool MAG, bool STD, bool INSIDE>
__device__ __forceinline__ void
count_tile(const T *__restrict__ x, int64_t n, const State *__restrict__ st, u32x2 *__restrict__ tile_cnt,
             const uint32_t *__restrict__ lists, int64_t ntiles, Std sd)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr uint32_t kTileElems = kTileThreads * kVecPerThread * EPV;
    __shared__ uint32_t wave_gt[kTileThreads / kWave], wave_eq[kTileThreads / kWave];
    const uint32_t Tk = st->T;
    if (use_list(st)) {                                     // a wave per tile list
        constexpr int64_t kSlot = (int64_t)kTileElems / kListShare;
        const int64_t t = (int64_t)blockIdx.x * (kTileThreads / kWave) + (threadIdx.x >> 6);
        if (t >= ntiles) return;
        const int lane_ = threadIdx.x & (kWave - 1);
        const u32x2 c = tile_cnt[t];
        const uint32_t cnt = min(c.y, (uint32_t)kSlot);
        const uint32_t *keys = lists + t * kSlot;
        uint32_t gt_ = 0u, eq_ = 0u;
        for (uint32_t i = lane_; i < cnt; i += kWave) {
            const uint32_t key = keys[i];
            gt_ += key > Tk ? 1u : 0u;
            eq_ += key == Tk ? 1u : 0u;
        }
        const uint32_t sums = wave_total_u32(wave_scan_u32(gt_ | (eq_ << 16)));
        if (lane_ == 0) {
            u32x2 r;
            r.x = c.x + (sums & 0xFFFFu);
            r.y = sums >> 16;
            tile_cnt[t] = r;
        }
        return;
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t nvec = (n + EPV - 1) / EPV;
    uint32_t bits[kVecPerThread][EPV];
    int valid[kVecPerThread];
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const int64_t v = tile_vec(blockIdx.x, wave, j, lane);
        valid[j] = load_tile_vec<T, INSIDE>(x, n, nvec, v, bits[j]);
    }
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) standardise<T, STD>(bits[j], valid[j], tile_vec(blockIdx.x, wave, j, lane), sd);
    uint32_t gt = 0u, eq = 0u;
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (INSIDE || e < valid[j]) {
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

template <typename T, bool MAG, bool STD>
__global__ void __launch_bounds__(kTileThreads)
count_kernel(const T *__restrict__ x, int64_t n, const State *__restrict__ st, u32x2 *__restrict__ tile_cnt,
             const uint32_t *__restrict__ lists, int64_t ntiles, Std sd)
{
    // workgroup-uniform: the whole tile lies below n
    constexpr int64_t kTileElems = (int64_t)kTileThreads * kVecPerThread * Elem<T>::EPV;
    if (((int64_t)blockIdx.x + 1) * kTileElems <= n)
        count_tile<T, MAG, STD, true>(x, n, st, tile_cnt, lists, ntiles, sd);
    else
        count_tile<T, MAG, STD, false>(x, n, st, tile_cnt, lists, ntiles, sd);
}

// ---- tile counts -> first output slot and tie budget of every tile ----------------------
// One workgroup.  Loads and stores are 16 bytes a lane, lanes side by side (a
// lane that fetched 16 consecutive tiles of its own made the kernel's one CU
// request every cache line 16 times over and took twice as long).  A pass covers
// 2 * kScanThreads tiles, thread t owning tiles 2t and 2t+1 of it; a round
// issues the loads of kScanPasses passes at once and then scans them in turn,
// carrying the totals.
constexpr int kScanPasses = 8;
__device__ __forceinline__ void block_exclusive_scan2(uint32_t a, uint32_t b, uint32_t *sums_a, uint32_t *sums_b,
                                                      uint32_t &before_a, uint32_t &before_b, uint32_t &total_a,
                                                      uint32_t &total_b)
{
    constexpr int NW = kScanThreads / kWave;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const uint32_t ia = wave_scan_u32(a), ib = wave_scan_u32(b);
    __syncthreads();                                       // the sums of the previous pass have been read
    if (lane == kWave - 1) {
        sums_a[wave] = ia;
        sums_b[wave] = ib;
    }
    __syncthreads();
    uint32_t ba = 0u, bb = 0u, ta = 0u, tb = 0u;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t sa = sums_a[w], sb = sums_b[w];
        ba += (w < wave) ? sa : 0u;
        bb += (w < wave) ? sb : 0u;
        ta += sa;
        tb += sb;
    }
    before_a = ba + ia - a;
    before_b = bb + ib - b;
    total_a = ta;
    total_b = tb;
}
__global__ void __launch_bounds__(kScanThreads)
scan_kernel(const State *__restrict__ st, const u32x2 *__restrict__ tile_cnt, u32x2 *__restrict__ tile_base,
            int64_t ntiles)
{
    __shared__ uint32_t sums_gt[kScanThreads / kWave], sums_eq[kScanThreads / kWave];
    const uint32_t take_eq = st->take_eq;
    auto base_of = [&](uint32_t gt_b, uint32_t eq_b) {
        u32x2 r;
        r.x = gt_b + min(eq_b, take_eq);
        r.y = take_eq > eq_b ? take_eq - eq_b : 0u;
        return r;
    };
    uint32_t gt_carry = 0u, eq_carry = 0u;
    for (int64_t base = 0; base < ntiles; base += (int64_t)kScanPasses * 2 * kScanThreads) {
        u32x2 c0[kScanPasses], c1[kScanPasses];
#pragma unroll
        for (int p = 0; p < kScanPasses; ++p) {
            const int64_t t = base + (int64_t)p * 2 * kScanThreads + 2 * threadIdx.x;
            c0[p] = u32x2{0u, 0u};
            c1[p] = u32x2{0u, 0u};
            if (t + 1 < ntiles) {                           // tile_cnt is 128-byte aligned and t is even
                const u32x4 v = *reinterpret_cast<const u32x4 *>(tile_cnt + t);
                c0[p] = u32x2{v.x, v.y};
                c1[p] = u32x2{v.z, v.w};
            } else if (t < ntiles) {
                c0[p] = tile_cnt[t];
            }
        }
#pragma unroll
        for (int p = 0; p < kScanPasses; ++p) {
            const int64_t t = base + (int64_t)p * 2 * kScanThreads + 2 * threadIdx.x;
            if (base + (int64_t)p * 2 * kScanThreads >= ntiles) break;          // uniform
            uint32_t gt_before, eq_before, gt_total, eq_total;
            block_exclusive_scan2(c0[p].x + c1[p].x, c0[p].y + c1[p].y, sums_gt, sums_eq, gt_before, eq_before, gt_total,
                                  eq_total);
            gt_before += gt_carry;
            eq_before += eq_carry;
            const u32x2 b0 = base_of(gt_before, eq_before);
            const u32x2 b1 = base_of(gt_before + c0[p].x, eq_before + c0[p].y);
            if (t + 1 < ntiles) {
                *reinterpret_cast<u32x4 *>(tile_base + t) = u32x4{b0.x, b0.y, b1.x, b1.y};
            } else if (t < ntiles) {
                tile_base[t] = b0;
            }
            gt_carry += gt_total;
            eq_carry += eq_total;
        }
    }
}

template <typename T> __device__ __forceinline__ void store_raw(T *p, uint32_t bits);
template <> __device__ __forceinline__ void store_raw<float>(float *p, uint32_t bits) { *p = __builtin_bit_cast(float, bits); }
template <> __device__ __forceinline__ void store_raw<uint16_t>(uint16_t *p, uint32_t bits) { *p = (uint16_t)bits; }

// ---- emit the survivors of a tile in ascending index order ------------------------------
template <typename T, bool MAG, bool STD, bool INSIDE>
__device__ __forceinline__ void
write_tile(const T *__restrict__ x, int64_t n, const State *__restrict__ st, const u32x2 *__restrict__ tile_base,
             typename Elem<T>::Out *__restrict__ vals, int32_t *__restrict__ idx, int32_t *__restrict__ tile_ptr, uint32_t k,
             Std sd)
{
    constexpr int EPV = Elem<T>::EPV;
    constexpr int NW = kTileThreads / kWave;
    constexpr int64_t kWaveElems = (int64_t)kWave * kVecPerThread * EPV;       // 1024 (fp32) / 2048 (bf16)
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
        valid[j] = load_tile_vec<T, INSIDE>(x, n, nvec, v, bits[j]);
    }
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) standardise<T, STD>(bits[j], valid[j], tile_vec(blockIdx.x, wave, j, lane), sd);
    uint32_t incl[kVecPerThread];
    uint32_t wave_packed = 0u;
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        uint32_t gt = 0u, eq = 0u;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (INSIDE || e < valid[j]) {
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
    if (tile_ptr) {
        const int64_t wave_start = (int64_t)blockIdx.x * (kWaveElems * NW) + wave * kWaveElems;
        if (lane == 0 && wave_start % kPtrTile == 0 && wave_start < n)
            tile_ptr[wave_start / kPtrTile] = (int32_t)(out_base + run_gt + min(run_eq, budget));
        if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) tile_ptr[(n + kPtrTile - 1) / kPtrTile] = (int32_t)k;
    }
    if constexpr (STD) {
        if (sd.row_ptr && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) sd.row_ptr[sd.last_row + 1u] = (int32_t)k;
    }
#pragma unroll
    for (int j = 0; j < kVecPerThread; ++j) {
        const uint32_t excl = incl[j] - packed[j];
        uint32_t my_gt = run_gt + (excl & 0xFFFFu);
        uint32_t my_eq = run_eq + (excl >> 16);
        const int64_t e0 = tile_vec(blockIdx.x, wave, j, lane) * EPV;
        if constexpr (STD) {
            if (sd.row_ptr && valid[j]) {                       // rows start on vector boundaries
                const uint32_t row = __umulhi((uint32_t)e0, sd.magic) >> sd.shift;
                if ((uint32_t)e0 == row * sd.H) sd.row_ptr[row] = (int32_t)(out_base + my_gt + min(my_eq, budget));
            }
        }
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (INSIDE || e < valid[j]) {
                const uint32_t key = make_key<T, MAG>(bits[j][e]);
                const bool above = key > Tk;
                const bool tie = key == Tk;
                if (above || (tie && my_eq < budget)) {
                    const uint32_t pos = out_base + my_gt + min(my_eq, budget);
                    if (pos < k) {                          // always true for consistent counts; guards the stores
                        store_raw<typename Elem<T>::Out>(vals + pos, bits[j][e]);
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

template <typename T, bool MAG, bool STD>
__global__ void __launch_bounds__(kTileThreads)
write_kernel(const T *__restrict__ x, int64_t n, const State *__restrict__ st, const u32x2 *__restrict__ tile_base,
             typename Elem<T>::Out *__restrict__ vals, int32_t *__restrict__ idx, int32_t *__restrict__ tile_ptr, uint32_t k,
             Std sd)
{
    // workgroup-uniform: the whole tile lies below n
    constexpr int64_t kTileElems = (int64_t)kTileThreads * kVecPerThread * Elem<T>::EPV;
    if (((int64_t)blockIdx.x + 1) * kTileElems <= n)
        write_tile<T, MAG, STD, true>(x, n, st, tile_base, vals, idx, tile_ptr, k, sd);
    else
        write_tile<T, MAG, STD, false>(x, n, st, tile_base, vals, idx, tile_ptr, k, sd);
}

// ---- restore without tile pointers: zeros, then scatter -----------------------------------
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

// ---- restore with tile pointers: each 4096-element tile of the output is built in LDS
// (zeros + its own records) and written once ------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(kTileThreads)
restore_tiles_kernel(const T *__restrict__ vals, const int32_t *__restrict__ idx, const int32_t *__restrict__ tile_ptr,
                     int64_t k, int64_t n, T *__restrict__ out)
{
    constexpr int PER16 = 16 / (int)sizeof(T);
    constexpr int kVecs = (int)kPtrTile / PER16;
    __shared__ alignas(16) T tile[kPtrTile];
    const int tid = threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.x * kPtrTile;
    const int m = (int)min(kPtrTile, n - t0);                  // >= 1 by the launch size

    int64_t p0 = tile_ptr[blockIdx.x], p1 = tile_ptr[blockIdx.x + 1];
    p0 = min(max(p0, (int64_t)0), k);                          // pointers that do not fit the record arrays are cut
    p1 = min(max(p1, p0), min(k, p0 + kPtrTile));
    const int n_rec = (int)(p1 - p0);

    // the first records of every thread are fetched before the tile is cleared,
    // so their latency overlaps the zero-fill and the barrier
    constexpr int PRE = 2;
    int pre_at[PRE];
    T pre_val[PRE];
#pragma unroll
    for (int u = 0; u < PRE; ++u) {
        const int j = tid + u * kTileThreads;
        pre_at[u] = -1;
        pre_val[u] = T(0);
        if (j < n_rec) {
            const int64_t at = (int64_t)idx[p0 + j] - t0;
            pre_at[u] = (at >= 0 && at < m) ? (int)at : -1;
            pre_val[u] = vals[p0 + j];
        }
    }
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int v = tid; v < kVecs; v += kTileThreads) reinterpret_cast<u32x4 *>(tile)[v] = z;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PRE; ++u)
        if (pre_at[u] >= 0) tile[pre_at[u]] = pre_val[u];
    for (int j = tid + PRE * kTileThreads; j < n_rec; j += kTileThreads) {
        const int64_t at = (int64_t)idx[p0 + j] - t0;
        if (at >= 0 && at < m) tile[at] = vals[p0 + j];
    }
    __syncthreads();
    const int full = m / PER16;                                // whole 16-byte vectors inside the tensor
    u32x4 *dst = reinterpret_cast<u32x4 *>(out + t0);
    for (int v = tid; v < full; v += kTileThreads)
        __builtin_nontemporal_store(reinterpret_cast<const u32x4 *>(tile)[v], dst + v);
    for (int e = full * PER16 + tid; e < m; e += kTileThreads) out[t0 + e] = tile[e];
}

// Workspace: state | histogram | tile counts | tile bases | tile key lists.
struct Workspace {
    State *st;
    uint32_t *hist;
    u32x2 *tile_cnt, *tile_base;
    uint32_t *lists;
    uint32_t route_cap;                    // largest bin that is sent to the lists: half of their slots
    size_t bytes;
};
Workspace carve(void *base, int64_t n)
{
    Workspace w;
    const size_t slots = (size_t)((n + kPtrTile - 1) / kPtrTile);        // >= kernel tiles of either dtype
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = static_cast<char *>(base) + off;
        off += (bytes + 127) / 128 * 128;
        return p;
    };
    w.st = reinterpret_cast<State *>(take(sizeof(State)));
    w.hist = reinterpret_cast<uint32_t *>(take((size_t)kMaxBins * 4));
    w.tile_cnt = reinterpret_cast<u32x2 *>(take(slots * 8));
    w.tile_base = reinterpret_cast<u32x2 *>(take(slots * 8));
    // a bf16 tile spans two pointer tiles and owns both their list slots
    w.lists = reinterpret_cast<uint32_t *>(take((slots + 1) * (size_t)(kPtrTile / kListShare) * 4));
    w.route_cap = (uint32_t)(n / (2 * kListShare));
    w.bytes = off;
    return w;
}
size_t workspace_bytes_for(int64_t n)
{
    static char origin[1];                 // only offsets are taken
    return carve(origin, n).bytes;
}

// digits from the top: fp32 12 | 8 | 12, bf16 12 | 4.  The middle digit is kept
// narrow because every workgroup adds its non-empty bins to the global
// histogram with atomics, and on the list route the second digit still sees
// every filed key.
template <typename T> struct Digits;
template <> struct Digits<float> {
    static constexpr int N = 3;
    static constexpr int bits[3] = {12, 8, 12};
};
template <> struct Digits<uint16_t> {
    static constexpr int N = 2;
    static constexpr int bits[3] = {12, 4, 0};
};

template <typename T, bool MAG, bool STD>
void launch_select(const T *x, int64_t n, uint32_t k, typename Elem<T>::Out *vals, int32_t *idx, int32_t *tile_ptr,
                   const Workspace &w, const Std &sd, hipStream_t s)
{
    using DigitPlan = Digits<typename Elem<T>::Key>;
    constexpr int EPV = Elem<T>::EPV;
    const int64_t nvec = (n + EPV - 1) / EPV;
    const int64_t chunk = (int64_t)kHistThreads * kVecPerThread;
    const int64_t nchunks = (nvec + chunk - 1) / chunk;
    const unsigned hist_grid = (unsigned)(nchunks < SLIMFIT_PG_HIST_GRID ? nchunks : SLIMFIT_PG_HIST_GRID);
    const int64_t tile_vecs = (int64_t)kTileThreads * kVecPerThread;
    const int64_t ntiles = (nvec + tile_vecs - 1) / tile_vecs;

    init_kernel<<<1, kSelectThreads, 0, s>>>(w.st, w.hist, k);
    int hi = Elem<T>::KEYBITS;
    for (int d = 0; d < DigitPlan::N; ++d) {
        const int bits = DigitPlan::bits[d];
        const int shift = hi - bits;
        const bool first = d == 0, last = d == DigitPlan::N - 1;
        if (first)
            hist_kernel<T, MAG, STD, true><<<hist_grid, kHistThreads, 0, s>>>(x, n, w.st, w.hist, w.tile_cnt, w.lists,
                                                                             ntiles, shift, 1 << bits, sd);
        else
            hist_kernel<T, MAG, STD, false><<<hist_grid, kHistThreads, 0, s>>>(x, n, w.st, w.hist, w.tile_cnt, w.lists,
                                                                              ntiles, shift, 1 << bits, sd);
        select_kernel<<<1, kSelectThreads, 0, s>>>(w.st, w.hist, shift, 1 << bits, first ? 1 : 0, last ? 1 : 0,
                                                   w.route_cap);
        if (first && !last)
            bracket_kernel<T, MAG, STD><<<(unsigned)ntiles, kTileThreads, 0, s>>>(x, n, w.st, w.tile_cnt, w.lists, sd);
        hi = shift;
    }
    count_kernel<T, MAG, STD><<<(unsigned)ntiles, kTileThreads, 0, s>>>(x, n, w.st, w.tile_cnt, w.lists, ntiles, sd);
    scan_kernel<<<1, kScanThreads, 0, s>>>(w.st, w.tile_cnt, w.tile_base, ntiles);
    write_kernel<T, MAG, STD><<<(unsigned)ntiles, kTileThreads, 0, s>>>(x, n, w.st, w.tile_base, vals, idx, tile_ptr, k,
                                                                         sd);
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

extern "C" int64_t slimfit_global_tile_ptr_len(int64_t n)
{
    if (n < 0 || n > 0x7FFFFFFFLL) return -1;
    return (n + kPtrTile - 1) / kPtrTile + 1;
}

namespace {

// Shared body of the two pruning entry points.  H == 0: plain; otherwise the
// tensor is rows of H elements standardised with mean / rstd on the way in.
int32_t prune_global_entry(const void *x, int32_t dt, int64_t n, int64_t H, const float *mean, const float *rstd,
                           int64_t k, int32_t by_magnitude, void *vals, int32_t *idx, int32_t *tile_ptr,
                           int32_t *row_ptr, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dtype_ok(dt) || n < 0 || k < 0 || k > n) return SLIMFIT_ERR_INVALID_ARG;
    if (n > 0x7FFFFFFFLL) return SLIMFIT_ERR_UNSUPPORTED;                 // indices are int32
    const bool standardised = H != 0;
    const int64_t epv = dt == SLIMFIT_F32 ? 4 : 8;            // a row has to be whole 16-byte vectors
    if (standardised && (H < epv || H % epv != 0 || n % H != 0)) return SLIMFIT_ERR_INVALID_ARG;
    if (k == 0) return SLIMFIT_OK;
    if (!x || !vals || !idx || !workspace || (standardised && (!mean || !rstd))) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    const size_t vsz = standardised ? 4 : esz;                // standardised values are fp32 whatever the input
    if (!aligned_to(x, 16) || !aligned_to(vals, vsz) || !aligned_to(idx, 4) || !aligned_to(workspace, 16) ||
        (tile_ptr && !aligned_to(tile_ptr, 4)) || (row_ptr && !aligned_to(row_ptr, 4)) ||
        (standardised && (!aligned_to(mean, 4) || !aligned_to(rstd, 4))))
        return SLIMFIT_ERR_ALIGNMENT;
    const Workspace w = carve(workspace, n);
    if (workspace_bytes < w.bytes) return SLIMFIT_ERR_WORKSPACE;
    int32_t rc;
    if ((rc = check_device_range(x, (size_t)n * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(vals, (size_t)k * vsz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(idx, (size_t)k * 4)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(workspace, w.bytes)) != SLIMFIT_OK) return rc;
    if (tile_ptr && (rc = check_device_range(tile_ptr, (size_t)slimfit_global_tile_ptr_len(n) * 4)) != SLIMFIT_OK)
        return rc;
    Std sd = {nullptr, nullptr, 0u, 0u, 0u, 0u, 0u, nullptr};
    if (standardised) {
        const size_t rows = (size_t)(n / H);
        if ((rc = check_device_range(mean, rows * 4)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(rstd, rows * 4)) != SLIMFIT_OK) return rc;
        if (row_ptr && (rc = check_device_range(row_ptr, (rows + 1) * 4)) != SLIMFIT_OK) return rc;
        int l = 0;
        while (((int64_t)1 << l) < H) ++l;                              // ceil(log2 H) >= 2
        const uint64_t pow = (uint64_t)1 << (31 + l);
        sd.mean = mean;
        sd.rstd = rstd;
        sd.magic = (uint32_t)((pow + (uint64_t)H - 1) / (uint64_t)H);   // < 2^32 because H > 2^(l-1)
        sd.shift = (uint32_t)(l - 1);
        sd.wave_uniform = (H % (kWave * epv) == 0) ? 1u : 0u;           // the 64 vectors a wave loads together share a row
        sd.last_row = (uint32_t)(rows - 1);
        sd.H = (uint32_t)H;
        sd.row_ptr = row_ptr;
    }

    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t kk = (uint32_t)k;
    if (dt == SLIMFIT_F32) {
        const float *xf = static_cast<const float *>(x);
        float *vf = static_cast<float *>(vals);
        if (standardised) {
            if (by_magnitude) launch_select<float, true, true>(xf, n, kk, vf, idx, tile_ptr, w, sd, s);
            else launch_select<float, false, true>(xf, n, kk, vf, idx, tile_ptr, w, sd, s);
        } else {
            if (by_magnitude) launch_select<float, true, false>(xf, n, kk, vf, idx, tile_ptr, w, sd, s);
            else launch_select<float, false, false>(xf, n, kk, vf, idx, tile_ptr, w, sd, s);
        }
    } else if (standardised) {
        const Bf16Row *xr = static_cast<const Bf16Row *>(x);
        float *vf = static_cast<float *>(vals);
        if (by_magnitude) launch_select<Bf16Row, true, true>(xr, n, kk, vf, idx, tile_ptr, w, sd, s);
        else launch_select<Bf16Row, false, true>(xr, n, kk, vf, idx, tile_ptr, w, sd, s);
    } else {
        const uint16_t *xh = static_cast<const uint16_t *>(x);
        uint16_t *vh = static_cast<uint16_t *>(vals);
        if (by_magnitude) launch_select<uint16_t, true, false>(xh, n, kk, vh, idx, tile_ptr, w, sd, s);
        else launch_select<uint16_t, false, false>(xh, n, kk, vh, idx, tile_ptr, w, sd, s);
    }
    return launch_status();
}

}  // namespace

extern "C" int32_t slimfit_prune_global(const void *x, int32_t dt, int64_t n, int64_t k, int32_t by_magnitude,
                                        void *vals, int32_t *idx, int32_t *tile_ptr, void *workspace,
                                        size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    return prune_global_entry(x, dt, n, 0, nullptr, nullptr, k, by_magnitude, vals, idx, tile_ptr, nullptr, workspace,
                              workspace_bytes, stream);
}

extern "C" int32_t slimfit_prune_global_standardized(const void *x, int32_t dt, int64_t n, int64_t H,
                                                     const float *mean, const float *rstd, int64_t k,
                                                     int32_t by_magnitude, void *vals, int32_t *idx,
                                                     int32_t *tile_ptr, int32_t *row_ptr, void *workspace,
                                                     size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    if (H == 0) return SLIMFIT_ERR_INVALID_ARG;
    return prune_global_entry(x, dt, n, H, mean, rstd, k, by_magnitude, vals, idx, tile_ptr, row_ptr, workspace,
                              workspace_bytes, stream);
}

extern "C" int32_t slimfit_restore_global(const void *vals, const int32_t *idx, const int32_t *tile_ptr, int64_t k,
                                          int32_t dt, int64_t n, void *out, void *stream)
{
    StreamScope capture_aware(stream);
    if (!dtype_ok(dt) || n < 0 || k < 0 || k > n) return SLIMFIT_ERR_INVALID_ARG;
    if (n > 0x7FFFFFFFLL) return SLIMFIT_ERR_UNSUPPORTED;
    if (n == 0) return SLIMFIT_OK;
    if (!out || (k > 0 && (!vals || !idx))) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    if (!aligned_to(out, 16) || (k > 0 && (!aligned_to(vals, esz) || !aligned_to(idx, 4))) ||
        (tile_ptr && !aligned_to(tile_ptr, 4)))
        return SLIMFIT_ERR_ALIGNMENT;
    int32_t rc;
    if ((rc = check_device_range(out, (size_t)n * esz)) != SLIMFIT_OK) return rc;
    if (k > 0) {
        if ((rc = check_device_range(vals, (size_t)k * esz)) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(idx, (size_t)k * 4)) != SLIMFIT_OK) return rc;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (tile_ptr && k > 0) {
        const int64_t tiles = (n + kPtrTile - 1) / kPtrTile;
        if ((rc = check_device_range(tile_ptr, (size_t)(tiles + 1) * 4)) != SLIMFIT_OK) return rc;
        if (dt == SLIMFIT_F32)
            restore_tiles_kernel<float><<<(unsigned)tiles, kTileThreads, 0, s>>>(
                static_cast<const float *>(vals), idx, tile_ptr, k, n, static_cast<float *>(out));
        else
            restore_tiles_kernel<uint16_t><<<(unsigned)tiles, kTileThreads, 0, s>>>(
                static_cast<const uint16_t *>(vals), idx, tile_ptr, k, n, static_cast<uint16_t *>(out));
        return launch_status();
    }
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
