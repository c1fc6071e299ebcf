// Pruning of score rows to (values, indices) and its inverse (Alg. 5 and the
// appendix on pruning), for gfx950.
//
// The paper sorts the whole input to find the largest 10 %.  A sort is not
// needed for that: the kept set is {p > T} plus the first few {p == T} in
// column order, where T is the k-th largest value of the row.  Three kernels:
//   prune_rows_kernel       rows of up to 1024 columns, one wavefront per row,
//                           the row held in registers (lane l: columns l, l+64, ...)
//   prune_rows_block_kernel rows of up to 16384 columns, one workgroup per row,
//                           the row held in the workgroup's registers
//   prune_rows_wide_kernel  wider rows still, one workgroup per row, the row
//                           re-read from cache for every probe
//   restore_tile_kernel     the restoring process: zeros + scatter in one pass
//   softmax_backward_tile_kernel  the Softmax input gradient from the kept pairs
#include "common.hpp"

#include <cfloat>
#include <cmath>

namespace slimfit {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;
#ifndef SLIMFIT_PRUNE_WAVES
#define SLIMFIT_PRUNE_WAVES 4
#endif
constexpr int kRowWaves = SLIMFIT_PRUNE_WAVES;          // waves per workgroup of the register-path kernel
constexpr int kRowThreads = kRowWaves * kWave;
#ifndef SLIMFIT_PRUNE_WAVE_SLOTS
#define SLIMFIT_PRUNE_WAVE_SLOTS 32
#endif
constexpr int kMaxRegSlots = SLIMFIT_PRUNE_WAVE_SLOTS;   // one-wave path: cols <= 64 * this (16, 32 or 64)
#ifndef SLIMFIT_PRUNE_BLOCKS
#define SLIMFIT_PRUNE_BLOCKS (1 << 30)
#endif
constexpr int64_t kMaxPruneBlocks = SLIMFIT_PRUNE_BLOCKS;

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
//
// Finding the cut value T (the k-th largest entry of the row):
//   1. lane-local, then wave-wide minimum and maximum (DPP butterflies);
//   2. a 256-bin histogram of the row in the wave's private LDS region, bins
//      of equal width in the order-preserving integer image of the floats,
//      bin 0 holding the largest values (ds_add, one per element);
//   3. a wave prefix sum over the bins locates the bin that holds the k-th
//      largest entry; if the entries above that bin plus the bin's own are
//      exactly k, its lower edge separates the kept set and the search is over
//      (about half of all softmax rows);
//   4. otherwise a bisection inside that bin (1/256 of the row's range; one or
//      two probes on average), each probe one v_cmp per held element whose
//      lane mask is popcounted on the scalar unit, ending as soon as a probe is
//      passed by exactly k entries or the bracket is a single value (ties).
// Survivors are compacted in ascending column order with mask-prefix counts
// (mbcnt) into (value, column) records in LDS when k <= 64; a wave owns 8
// consecutive rows and stores their records as two contiguous runs, so the
// output leaves in full cache lines instead of a dozen masked stores per row.
// Launch shape: one 8-row unit per wave (no persistent loop; the chip streams
// best with many short workgroups).
constexpr int kBins = 256;
constexpr int kStage = 64;           // largest k whose output is staged in LDS
#ifndef SLIMFIT_PRUNE_ROWS_PER_UNIT
#define SLIMFIT_PRUNE_ROWS_PER_UNIT 8
#endif
constexpr int kRowsPerUnit = SLIMFIT_PRUNE_ROWS_PER_UNIT;   // consecutive rows a wave stages before it stores them

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_zero_i32(int v)          // absent sources contribute 0
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, false);
}
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;

// wave-wide maximum of unsigned keys, result uniform.  Sources that a DPP
// control does not reach contribute 0, the identity of an unsigned max.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_zero_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_umax(uint32_t v)
{
    v = max(v, dpp_zero_u32<kDppXor1, 0xF>(v));
    v = max(v, dpp_zero_u32<kDppXor2, 0xF>(v));
    v = max(v, dpp_zero_u32<kDppHalfMirror, 0xF>(v));
    v = max(v, dpp_zero_u32<kDppMirror, 0xF>(v));
    v = max(v, dpp_zero_u32<kDppBcast15, 0xA>(v));
    v = max(v, dpp_zero_u32<kDppBcast31, 0xC>(v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ int wave_scan_i32(int v)
{
    v += dpp_zero_i32<kDppRowShr1, 0xF>(v);
    v += dpp_zero_i32<kDppRowShr2, 0xF>(v);
    v += dpp_zero_i32<kDppRowShr4, 0xF>(v);
    v += dpp_zero_i32<kDppRowShr8, 0xF>(v);
    v += dpp_zero_i32<kDppBcast15, 0xA>(v);
    v += dpp_zero_i32<kDppBcast31, 0xC>(v);
    return v;
}

// sum of one float per lane, in a fixed order; result uniform
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add_f32(float v)      // absent sources contribute +0
{
    return v + __builtin_bit_cast(float, dpp_zero_i32<CTRL, ROW_MASK>(__builtin_bit_cast(int, v)));
}
__device__ __forceinline__ float wave_sum_f32(float v)
{
    v = dpp_add_f32<kDppRowShr1, 0xF>(v);
    v = dpp_add_f32<kDppRowShr2, 0xF>(v);
    v = dpp_add_f32<kDppRowShr4, 0xF>(v);
    v = dpp_add_f32<kDppRowShr8, 0xF>(v);
    v = dpp_add_f32<kDppBcast15, 0xA>(v);
    v = dpp_add_f32<kDppBcast31, 0xC>(v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

#ifndef SLIMFIT_PRUNE_SHORT
#define SLIMFIT_PRUNE_SHORT 1          // rows of <= 256 columns keeping <= 16 entries take the short-row kernel
#endif
#ifndef SLIMFIT_SOFTMAX_SHORT
#define SLIMFIT_SOFTMAX_SHORT 1        // the fused softmax takes the short-row kernel under the same conditions
#endif
#ifndef SLIMFIT_PRUNE_NT
#define SLIMFIT_PRUNE_NT 1             // row loads are streamed once
#endif
#ifndef SLIMFIT_PRUNE_NT_STORE
#define SLIMFIT_PRUNE_NT_STORE 1       // so are the staged output stores
#endif

template <typename T> __device__ __forceinline__ float load_elem_stream(const T *p);
template <> __device__ __forceinline__ float load_elem_stream<float>(const float *p)
{
    return SLIMFIT_PRUNE_NT ? __builtin_nontemporal_load(p) : *p;
}
template <> __device__ __forceinline__ float load_elem_stream<uint16_t>(const uint16_t *p)
{
    return bf16_widen(SLIMFIT_PRUNE_NT ? __builtin_nontemporal_load(p) : *p);
}

// LDS staging of one wave: the (value bits, column) records of the kept entries
// of kRowsPerUnit consecutive rows, in output order (row stride k).
struct StageRec {
    uint32_t v, c;
};
struct alignas(16) WaveStage {
    StageRec rec[kRowsPerUnit * kStage];
};

// Places the kept entries of one row in ascending column order, either as
// records in the staging area (STAGED; at most k <= kStage per row) or directly
// in global memory.  pred(j) is this lane's "entry j is kept" flag.  Every caller
// derives the flags from the same comparisons that counted kk <= k entries, so a
// position never reaches k.  first: index of the row's first output slot (in the
// staging area, or 0).
template <typename T, int M, bool STAGED, typename Pred>
__device__ __forceinline__ void emit_row(Pred pred, const float (&f)[M], int lane, int k, int kk, T *ov, uint16_t *oi,
                                         StageRec *rec, uint32_t first)
{
    uint32_t base = first;
#pragma unroll
    for (int j = 0; j < M; ++j) {
        const bool s = pred(j);
        const uint64_t m = __builtin_amdgcn_ballot_w64(s);
        const uint32_t pos =
            __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, base));
        if (s) {
            if (STAGED) {
                rec[pos].v = __builtin_bit_cast(uint32_t, f[j]);
                rec[pos].c = (uint32_t)(j * kWave + lane);
            } else {
                ov[pos] = Elem<T>::raw(f[j]);
                oi[pos] = (uint16_t)(j * kWave + lane);
            }
        }
        base += (uint32_t)popc64(m);
    }
    for (int s = kk + lane; s < k; s += kWave) {             // THRESHOLD: unused slots
        if (STAGED) {
            rec[first + s].v = 0u;
            rec[first + s].c = 0xFFFFu;
        } else {
            ov[s] = Elem<T>::zero();
            oi[s] = 0xFFFFu;
        }
    }
}

// T: element type; M: slots per lane; FULL: cols == 64*M (no absent columns);
// STAGED: k <= kStage, outputs of kRowsPerUnit rows leave as contiguous runs;
// SOFTMAX: the rows are logits: the row's softmax is written to `probs`, the
// kept set is decided on the logits (which order the row as the probabilities
// do, without their rounding) and the kept values are the probabilities.
template <typename T, int M, bool FULL, bool STAGED, bool SOFTMAX>
__global__ __launch_bounds__(kRowThreads) void prune_rows_kernel(const T *__restrict__ p, int64_t rows, int cols, int k,
                                                              int mode, float tau, T *__restrict__ vals,
                                                              uint16_t *__restrict__ idx, int32_t *__restrict__ counts,
                                                              T *__restrict__ probs)
{
    // keys of bf16 inputs have 16 zero low bits: work in units of 2^16 there
    constexpr int KEY_SHIFT = sizeof(T) == 2 ? 16 : 0;
    constexpr uint32_t UNIT = 1u << KEY_SHIFT;
    constexpr uint32_t KEY_MASK = ~(UNIT - 1u);
    __shared__ uint32_t s_hist[kRowWaves][kBins];
    __shared__ WaveStage s_stage[STAGED ? kRowWaves : 1];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);      // uniform: rows and pointers stay scalar
    uint32_t *hist = s_hist[wave];
    StageRec *rec = s_stage[STAGED ? wave : 0].rec;
    const float ninf = -__builtin_inff(), pinf = __builtin_inff(), qnan = __builtin_nanf("");

    // a unit is kRowsPerUnit consecutive rows owned by one wave; a workgroup owns
    // kRowWaves consecutive units, so its output is one contiguous run
    const int64_t n_units = (rows + kRowsPerUnit - 1) / kRowsPerUnit;
    const int64_t unit0 = (int64_t)blockIdx.x * kRowWaves + wave;
    const int64_t unit_stride = (int64_t)gridDim.x * kRowWaves;

    // byte offsets of this lane's columns inside a row: 32 bits, so that a load is a scalar row
    // address plus a vector offset and no 64-bit address is formed per element
    bool valid[M];
    uint32_t coff[M];
#pragma unroll
    for (int j = 0; j < M; ++j) {
        const int col = j * kWave + lane;
        valid[j] = FULL || col < cols;
        coff[j] = (uint32_t)(valid[j] ? col : cols - 1) * (uint32_t)sizeof(T);   // absent columns re-read the last one
    }
    auto load_col = [&](const T *row, int j) {
        return load_elem_stream<T>(reinterpret_cast<const T *>(reinterpret_cast<const char *>(row) + coff[j]));
    };

    float nxt[M];
    for (int64_t unit = unit0; unit < n_units; unit += unit_stride) {        // wave-uniform trip counts
        const int64_t row0 = unit * kRowsPerUnit;
        const int n_here = (int)min((int64_t)kRowsPerUnit, rows - row0);
        int my_count = 0;                                                    // lane i keeps row i's count
        // the launch gives every wave one unit (the loop only runs on for row counts beyond the grid
        // limit), so rows are prefetched inside a unit only
        const T *next_src = p + row0 * (int64_t)cols;                        // row whose loads are in flight
#pragma unroll
        for (int j = 0; j < M; ++j) nxt[j] = load_col(next_src, j);
        for (int i = 0; i < n_here; ++i) {
            const int64_t row = row0 + i;
            // absent columns hold NaN from here on: every ordered comparison with them is false and
            // fmaxf / fminf pass them over, so the predicates below need no validity term (a ballot of a
            // compound predicate costs two extra vector instructions per slot)
            float f[M];
#pragma unroll
            for (int j = 0; j < M; ++j) f[j] = (FULL || valid[j]) ? nxt[j] : qnan;
            if (i + 1 < n_here) {        // the next row's loads fly during this row's work
                next_src += cols;
#pragma unroll
                for (int j = 0; j < M; ++j) nxt[j] = load_col(next_src, j);
            }

            float pv[M];                 // SOFTMAX: the row's probabilities, in the output dtype's values
            if constexpr (SOFTMAX) {
                float lm = ninf;
#pragma unroll
                for (int j = 0; j < M; ++j) lm = fmaxf(lm, f[j]);
                const float row_max = key_to_float(wave_umax(float_to_key(lm)));
                float part = 0.0f;
#pragma unroll
                for (int j = 0; j < M; ++j) {
                    const float e = __builtin_amdgcn_exp2f((f[j] - row_max) * 1.44269504088896340736f);
                    pv[j] = (FULL || valid[j]) ? e : 0.0f;
                    part += pv[j];
                }
                const float inv = 1.0f / wave_sum_f32(part);      // IEEE division
                T *prow = probs + row * (int64_t)cols;
#pragma unroll
                for (int j = 0; j < M; ++j) {
                    float pj = pv[j] * inv;
                    if (sizeof(T) == 2) pj = bf16_widen(bf16_narrow(pj));
                    pv[j] = pj;
                    if (FULL || valid[j])
                        store_global<SLIMFIT_PRUNE_NT_STORE != 0>(prow + j * kWave + lane, Elem<T>::raw(pj));
                }
            }
            const float(&kept_value)[M] = SOFTMAX ? pv : f;

            auto count_ge = [&](float t) {
                int c = 0;
#pragma unroll
                for (int j = 0; j < M; ++j) c += popc64(__builtin_amdgcn_ballot_w64(f[j] >= t));
                return c;
            };

            int kk = k;                  // pairs to keep for this row
            float T_cut = 0.0f, T_exact = 0.0f;
            int c_ge = 0;
            bool have_cut = false;
            if (mode == SLIMFIT_PRUNE_THRESHOLD) {
                const int c_tau = count_ge(tau);
                if (c_tau <= k) { kk = c_tau; T_cut = T_exact = tau; c_ge = c_tau; have_cut = true; }
            }
            if (!have_cut) {
                // 1. extrema as order-preserving keys (the minimum as a maximum of complements)
                float lmax = ninf, lmin = pinf;
#pragma unroll
                for (int j = 0; j < M; ++j) {
                    lmax = fmaxf(lmax, f[j]);
                    lmin = fminf(lmin, f[j]);
                }
                uint32_t hi = wave_umax(float_to_key(lmax));
                uint32_t lo = ~wave_umax(~float_to_key(lmin));
                // a key below that of +0 means a set sign bit somewhere in the row
                const bool any_neg = lo < 0x80000000u;
                // -0 is folded onto +0 so that integer order agrees with float comparison
                if (hi == 0x7FFFFFFFu) hi = 0x80000000u;
                if (lo == 0x7FFFFFFFu) lo = 0x80000000u;
                // bf16: the keys of negative values end in 0xFFFF, those of the others in 0x0000;
                // dropping the low bits keeps the order and puts every key on a multiple of UNIT
                hi &= KEY_MASK;
                lo &= KEY_MASK;
                const uint32_t range = (hi - lo) >> KEY_SHIFT;
                const int width_bits = 32 - __builtin_clz(range | 1u);
                const int sh = KEY_SHIFT + (width_bits > 8 ? width_bits - 8 : 0);   // bin = (hi - key) >> sh < 256

                // 2. histogram
                reinterpret_cast<uint4 *>(hist)[lane] = make_uint4(0u, 0u, 0u, 0u);
                __builtin_amdgcn_wave_barrier();
                if (!any_neg) {
                    const uint32_t hi_bits = hi ^ 0x80000000u;   // keys of non-negative floats are their bits
#pragma unroll
                    for (int j = 0; j < M; ++j) {
                        const uint32_t b = ((hi_bits - __builtin_bit_cast(uint32_t, f[j])) >> sh) & (kBins - 1);
                        if (FULL || valid[j]) atomicAdd(&hist[b], 1u);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < M; ++j) {
                        const uint32_t b = ((hi - (float_to_key(f[j] + 0.0f) & KEY_MASK)) >> sh) & (kBins - 1);
                        if (FULL || valid[j]) atomicAdd(&hist[b], 1u);
                    }
                }
                __builtin_amdgcn_wave_barrier();
                const uint4 h4 = reinterpret_cast<const uint4 *>(hist)[lane];    // bins 4*lane .. 4*lane+3

                // 3. the bin holding the kk-th largest entry
                const int s4 = (int)(h4.x + h4.y + h4.z + h4.w);
                const int incl = wave_scan_i32(s4);
                const uint64_t reached = __builtin_amdgcn_ballot_w64(incl >= kk);
                const int L = reached ? __builtin_ctzll(reached) : 63;          // always reached for finite input
                // the crossing lane's four bins are resolved on the scalar unit
                const int e_L = __builtin_amdgcn_readlane(incl - s4, L);         // entries in bins before lane L's
                const int h0 = __builtin_amdgcn_readlane((int)h4.x, L), h1 = __builtin_amdgcn_readlane((int)h4.y, L);
                const int h2 = __builtin_amdgcn_readlane((int)h4.z, L), h3 = __builtin_amdgcn_readlane((int)h4.w, L);
                const int c0 = e_L + h0, c1 = c0 + h1, c2 = c1 + h2, c3 = c2 + h3;
                const int sub = c0 >= kk ? 0 : (c1 >= kk ? 1 : (c2 >= kk ? 2 : 3));
                const int c_bin = sub == 0 ? c0 : (sub == 1 ? c1 : (sub == 2 ? c2 : c3));   // entries >= the bin's lower edge
                const int B = 4 * L + sub;
                // keys of bin B: (hi - (B+1)<<sh, hi - B<<sh]
                const uint64_t span = (uint64_t)(B + 1) << sh;
                uint32_t blo = span > (uint64_t)(hi - lo) ? lo : (uint32_t)(hi - (uint32_t)span + UNIT);
                uint32_t bhi = hi - ((uint32_t)B << sh) + UNIT;  // exclusive
                c_ge = c_bin;
                // 4. bisection inside the bin
                if (c_ge != kk) {
                    while (bhi - blo > UNIT) {                    // at most 32 probes
                        const uint32_t mid = blo + (((bhi - blo) >> (KEY_SHIFT + 1)) << KEY_SHIFT);
                        const int c = count_ge(key_to_float(mid));
                        if (c >= kk) {
                            blo = mid;
                            c_ge = c;
                            if (c == kk) break;                  // the probe separates exactly kk entries
                        } else {
                            bhi = mid;
                        }
                    }
                }
                T_cut = key_to_float(blo);
                // the value itself when blo is the key of a row entry (negative bf16 values
                // have the dropped low bits set); only the tie path below compares for equality
                T_exact = key_to_float((blo & 0x80000000u) ? blo : (blo | (UNIT - 1u)));
            }

            T *ov = vals + row * (int64_t)k;
            uint16_t *oi = idx + row * (int64_t)k;
            const uint32_t first = STAGED ? (uint32_t)(i * k) : 0u;
            if (c_ge == kk) {
                emit_row<T, M, STAGED>([&](int j) { return f[j] >= T_cut; }, kept_value, lane, k, kk, ov, oi, rec,
                                       first);
            } else {
                // more than kk entries reach the cut value: all above it, then the
                // equal ones by ascending column until kk are taken
                int c_gt = 0;
#pragma unroll
                for (int j = 0; j < M; ++j) c_gt += popc64(__builtin_amdgcn_ballot_w64(f[j] > T_exact));
                const int need = kk - c_gt;
                bool sel[M];
                int seen = 0;
#pragma unroll
                for (int j = 0; j < M; ++j) {
                    const bool eq = f[j] == T_exact;
                    const uint64_t eqm = __builtin_amdgcn_ballot_w64(eq);
                    const int rank = seen + (int)lanes_below(eqm);
                    sel[j] = f[j] > T_exact || (eq && rank < need);
                    seen += popc64(eqm);
                }
                emit_row<T, M, STAGED>([&](int j) { return sel[j]; }, kept_value, lane, k, kk, ov, oi, rec, first);
            }
            my_count = lane == i ? kk : my_count;
        }
        if (STAGED) {                            // the unit's records leave as two contiguous runs
            __builtin_amdgcn_wave_barrier();
            T *ov = vals + row0 * (int64_t)k;
            uint16_t *oi = idx + row0 * (int64_t)k;
            const int n_out = n_here * k;
            for (int t = lane; t < n_out; t += kWave) {
                const StageRec r = rec[t];
                store_global<SLIMFIT_PRUNE_NT_STORE != 0>(ov + t, Elem<T>::raw(__builtin_bit_cast(float, r.v)));
                store_global<SLIMFIT_PRUNE_NT_STORE != 0>(oi + t, (uint16_t)r.c);
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (counts && lane < n_here) counts[row0 + lane] = my_count;
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
    v = __builtin_amdgcn_readlane(wave_scan_i32(v), kWave - 1);          // the wave's sum, by DPP
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

// ---------------------------------------------------------------------------
// rows of 1025 .. 16384 columns: one workgroup per row, the row held in registers
// ---------------------------------------------------------------------------
// The algorithm of the one-wave kernel with workgroup-wide steps: thread t holds columns t, t + 256, ...
// (S slots), the 256-bin histogram lives in LDS with one bin per thread, counts and extrema go through
// LDS between the four waves, and the survivors' positions come from a table of per-(slot, wave)
// counts that is prefix-summed once.  The row is read from memory once.  Every branch around a
// barrier depends on workgroup-wide results only.
__device__ __forceinline__ int block_inclusive_scan_i32(int v, BlockScratch &s)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    int incl = wave_scan_i32(v);
    __syncthreads();                         // previous use of the scratch is over
    if (lane == kWave - 1) s.i[wave] = incl;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) incl += (w < wave) ? s.i[w] : 0;
    return incl;
}
// table[0 .. n) (n <= kThreads) -> its exclusive prefix sums, in place
__device__ __forceinline__ void block_scan_table(int *table, int n, BlockScratch &s)
{
    __syncthreads();                         // the table is complete
    const int v = (int)threadIdx.x < n ? table[threadIdx.x] : 0;
    const int incl = block_inclusive_scan_i32(v, s);
    if ((int)threadIdx.x < n) table[threadIdx.x] = incl - v;
    __syncthreads();
}

template <typename T, int S>
__global__ __launch_bounds__(kThreads) void prune_rows_block_kernel(const T *__restrict__ p, int64_t rows, int cols,
                                                                    int k, int mode, float tau, T *__restrict__ vals,
                                                                    uint16_t *__restrict__ idx,
                                                                    int32_t *__restrict__ counts)
{
    static_assert(S <= 64 && S * kWavesPerBlock <= kThreads, "slots");
    constexpr int KEY_SHIFT = sizeof(T) == 2 ? 16 : 0;
    constexpr uint32_t UNIT = 1u << KEY_SHIFT;
    constexpr uint32_t KEY_MASK = ~(UNIT - 1u);
    __shared__ BlockScratch scratch;
    __shared__ uint32_t hist[kBins];
    __shared__ int table[S * kWavesPerBlock];                  // entry s * 4 + wave
    __shared__ int found[2];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const float ninf = -__builtin_inff(), pinf = __builtin_inff(), qnan = __builtin_nanf("");

    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {        // workgroup-uniform
        const T *src = p + row * (int64_t)cols;
        float f[S];                                                        // absent columns hold NaN
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int col = s * kThreads + tid;
            f[s] = col < cols ? load_elem_stream<T>(src + col) : qnan;
        }
        auto count_ge = [&](float t) {
            int c = 0;
#pragma unroll
            for (int s = 0; s < S; ++s) c += f[s] >= t ? 1 : 0;
            return block_sum_int(c, scratch);
        };

        int kk = k;
        float T_cut = 0.0f, T_exact = 0.0f;
        int c_ge = 0;
        bool have_cut = false;
        if (mode == SLIMFIT_PRUNE_THRESHOLD) {
            const int c_tau = count_ge(tau);
            if (c_tau <= k) { kk = c_tau; T_cut = T_exact = tau; c_ge = c_tau; have_cut = true; }
        }
        if (!have_cut) {
            float lmax = ninf, lmin = pinf;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                lmax = fmaxf(lmax, f[s]);
                lmin = fminf(lmin, f[s]);
            }
            // both extrema through LDS in one exchange (the minimum as a maximum of complements); the histogram
            // and the search result are cleared in the same step
            const uint32_t wmax = wave_max_u32(float_to_key(lmax)), wmin = wave_max_u32(~float_to_key(lmin));
            __syncthreads();                                               // previous use of the scratch is over
            if (lane == 0) {
                scratch.u[wave] = wmax;
                scratch.i[wave] = (int)wmin;
            }
            hist[tid] = 0u;                                                // kBins == kThreads
            if (tid == 0) {
                found[0] = kBins - 1;
                found[1] = cols;
            }
            __syncthreads();
            uint32_t hi = 0u, lo = 0u;
#pragma unroll
            for (int w = 0; w < kWavesPerBlock; ++w) {
                hi = max(hi, scratch.u[w]);
                lo = max(lo, (uint32_t)scratch.i[w]);
            }
            lo = ~lo;
            if (hi == 0x7FFFFFFFu) hi = 0x80000000u;                       // -0 is folded onto +0
            if (lo == 0x7FFFFFFFu) lo = 0x80000000u;
            hi &= KEY_MASK;
            lo &= KEY_MASK;
            const uint32_t range = (hi - lo) >> KEY_SHIFT;
            const int width_bits = 32 - __builtin_clz(range | 1u);
            const int sh = KEY_SHIFT + (width_bits > 8 ? width_bits - 8 : 0);   // bin = (hi - key) >> sh < 256
#pragma unroll
            for (int s = 0; s < S; ++s) {
                if (s * kThreads + tid < cols) {
                    const uint32_t b = ((hi - (float_to_key(f[s] + 0.0f) & KEY_MASK)) >> sh) & (kBins - 1);
                    atomicAdd(&hist[b], 1u);
                }
            }
            __syncthreads();
            const int h = (int)hist[tid];
            const int incl = block_inclusive_scan_i32(h, scratch);         // entries in bins 0 .. tid
            if (incl >= kk && incl - h < kk) {                             // the bin holding the kk-th largest entry
                found[0] = tid;
                found[1] = incl;
            }
            __syncthreads();
            const int B = found[0];
            c_ge = found[1];
            const uint64_t span = (uint64_t)(B + 1) << sh;
            uint32_t blo = span > (uint64_t)(hi - lo) ? lo : (uint32_t)(hi - (uint32_t)span + UNIT);
            uint32_t bhi = hi - ((uint32_t)B << sh) + UNIT;               // exclusive
            if (c_ge != kk) {
                while (bhi - blo > UNIT) {                                 // workgroup-uniform: c is a workgroup sum
                    const uint32_t mid = blo + (((bhi - blo) >> (KEY_SHIFT + 1)) << KEY_SHIFT);
                    const int c = count_ge(key_to_float(mid));
                    if (c >= kk) {
                        blo = mid;
                        c_ge = c;
                        if (c == kk) break;
                    } else {
                        bhi = mid;
                    }
                }
            }
            T_cut = key_to_float(blo);
            T_exact = key_to_float((blo & 0x80000000u) ? blo : (blo | (UNIT - 1u)));
        }

        // which slots of this thread are kept (bit s)
        uint64_t keep = 0;
        if (c_ge == kk) {
#pragma unroll
            for (int s = 0; s < S; ++s) keep |= (uint64_t)(f[s] >= T_cut ? 1 : 0) << s;
        } else {
            // more than kk entries reach the cut value: all above it, then the equal ones by ascending
            // column until kk are taken
            int c = 0;
#pragma unroll
            for (int s = 0; s < S; ++s) c += f[s] > T_exact ? 1 : 0;
            const int need = kk - block_sum_int(c, scratch);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const uint64_t eqm = __builtin_amdgcn_ballot_w64(f[s] == T_exact);
                if (lane == 0) table[s * kWavesPerBlock + wave] = popc64(eqm);
            }
            block_scan_table(table, S * kWavesPerBlock, scratch);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const bool eq = f[s] == T_exact;
                const uint64_t eqm = __builtin_amdgcn_ballot_w64(eq);
                const int rank = table[s * kWavesPerBlock + wave] + (int)lanes_below(eqm);
                keep |= (uint64_t)((f[s] > T_exact || (eq && rank < need)) ? 1 : 0) << s;
            }
            __syncthreads();                                               // the table is reused below
        }

        // positions in ascending column order: slot-major, then wave, then lane
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const uint64_t m = __builtin_amdgcn_ballot_w64(((keep >> s) & 1u) != 0);
            if (lane == 0) table[s * kWavesPerBlock + wave] = popc64(m);
        }
        block_scan_table(table, S * kWavesPerBlock, scratch);
        T *ov = vals + row * (int64_t)k;
        uint16_t *oi = idx + row * (int64_t)k;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const bool sel = ((keep >> s) & 1u) != 0;
            const uint64_t m = __builtin_amdgcn_ballot_w64(sel);
            const int pos = table[s * kWavesPerBlock + wave] + (int)lanes_below(m);
            if (sel && pos < k) {
                ov[pos] = Elem<T>::raw(f[s]);
                oi[pos] = (uint16_t)(s * kThreads + tid);
            }
        }
        for (int s = kk + tid; s < k; s += kThreads) {                     // THRESHOLD: unused slots
            ov[s] = Elem<T>::zero();
            oi[s] = 0xFFFFu;
        }
        if (counts && tid == 0) counts[row] = kk;
        __syncthreads();                                                   // LDS is reused by the next row
    }
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
// restore (Alg. 5, restoring process): zeros, then scatter -- fused
// ---------------------------------------------------------------------------
// The dense output is produced in flat tiles of kTile elements.  A workgroup
// zero-fills its tile in LDS, scatters into it the records of the rows that
// intersect the tile (their (value, column) pairs are one contiguous run of the
// record arrays), and streams the tile out with 16-byte stores.  Every output
// byte is written exactly once; no zero-fill pass over HBM.
#ifndef SLIMFIT_RESTORE_TILE
#define SLIMFIT_RESTORE_TILE 4096
#endif
constexpr int kTile = SLIMFIT_RESTORE_TILE;

template <typename T>
__global__ __launch_bounds__(kThreads) void restore_tile_kernel(const T *__restrict__ vals,
                                                                const uint16_t *__restrict__ idx,
                                                                const int32_t *__restrict__ counts, int64_t rows,
                                                                int cols, int k, T *__restrict__ out)
{
    __shared__ alignas(16) T tile[kTile];
    constexpr int PER16 = 16 / (int)sizeof(T);                  // elements per 16-byte vector
    constexpr int kVecs = kTile / PER16;
    const int tid = threadIdx.x;
    const int64_t total = rows * (int64_t)cols;
    const int64_t t0 = (int64_t)blockIdx.x * kTile;
    const int n = (int)min((int64_t)kTile, total - t0);         // >= 1 by the launch size

    const int64_t r_lo = t0 / cols, r_hi = (t0 + n - 1) / cols; // rows touching this tile
    const int n_rec = (int)(r_hi - r_lo + 1) * k;
    const int64_t rec0 = r_lo * (int64_t)k;

    // a record's place in the tile, or -1 if it is unused / lies outside
    auto place = [&](int j, int col, int cnt_or_neg) {
        const int rl = j / k;
        const int s = j - rl * k;
        const int cnt = cnt_or_neg < 0 ? k : cnt_or_neg;
        const int64_t at = (r_lo + rl) * (int64_t)cols + col - t0;
        return (s < cnt && col < cols && at >= 0 && at < n) ? (int)at : -1;
    };

    // the first records of every thread are fetched before the tile is cleared,
    // so their latency overlaps the zero-fill and the barrier
    constexpr int PRE = 2;
    int pre_col[PRE], pre_cnt[PRE];
    T pre_val[PRE];
#pragma unroll
    for (int u = 0; u < PRE; ++u) {
        const int j = tid + u * kThreads;
        pre_col[u] = 0;
        pre_cnt[u] = -1;
        pre_val[u] = T(0);
        if (j < n_rec) {
            pre_col[u] = idx[rec0 + j];
            pre_val[u] = vals[rec0 + j];
            if (counts) pre_cnt[u] = counts[r_lo + j / k];
        }
    }

    for (int v = tid; v < kVecs; v += kThreads) reinterpret_cast<uint4 *>(tile)[v] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();

#pragma unroll
    for (int u = 0; u < PRE; ++u) {
        const int j = tid + u * kThreads;
        if (j < n_rec) {
            const int at = place(j, pre_col[u], pre_cnt[u]);
            if (at >= 0) tile[at] = pre_val[u];
        }
    }
    for (int j = tid + PRE * kThreads; j < n_rec; j += kThreads) {
        const int at = place(j, idx[rec0 + j], counts ? counts[r_lo + j / k] : -1);
        if (at >= 0) tile[at] = vals[rec0 + j];
    }
    __syncthreads();

    T *dst = out + t0;                                          // 16-byte aligned: kTile * sizeof(T) is
    const int n_vec = n / PER16;
    for (int v = tid; v < n_vec; v += kThreads)
        store_global<true>(reinterpret_cast<u32x4 *>(dst) + v, reinterpret_cast<const u32x4 *>(tile)[v]);
    for (int e = n_vec * PER16 + tid; e < n; e += kThreads) dst[e] = tile[e];
}

// ---------------------------------------------------------------------------
// softmax backward from the kept probabilities
// ---------------------------------------------------------------------------
// ds_j = p^_j (dp_j - sum_i p^_i dp_i) with p^ the restored row: zero wherever
// nothing was kept.  Same tiling as the restore kernel (a workgroup owns kTile
// consecutive output elements, builds them in LDS and streams them out), with a
// wave per intersecting row: its lanes fetch the row's records, gather dp at
// the kept columns, sum the products over the wave in a fixed order and drop
// p^_j (dp_j - sum) into the tile.  A row that straddles two tiles is summed by
// both workgroups (identically).  kBackRows rows of a wave are in flight at once.
template <typename T> struct Narrow;
template <> struct Narrow<float> {
    __device__ static float from(float f) { return f; }
};
template <> struct Narrow<uint16_t> {
    __device__ static uint16_t from(float f) { return (uint16_t)bf16_narrow(f); }
};

constexpr int kBackRows = 4;

template <typename T>
__global__ __launch_bounds__(kThreads) void softmax_backward_tile_kernel(const T *__restrict__ vals,
                                                                         const uint16_t *__restrict__ idx,
                                                                         const int32_t *__restrict__ counts,
                                                                         const T *__restrict__ dp, int64_t rows,
                                                                         int cols, int k, T *__restrict__ out)
{
    __shared__ alignas(16) T tile[kTile];
    constexpr int PER16 = 16 / (int)sizeof(T);
    constexpr int kVecs = kTile / PER16;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t total = rows * (int64_t)cols;
    const int64_t t0 = (int64_t)blockIdx.x * kTile;
    const int n = (int)min((int64_t)kTile, total - t0);         // >= 1 by the launch size
    const int64_t r_lo = t0 / cols, r_hi = (t0 + n - 1) / cols; // rows touching this tile
    const int n_rows = (int)(r_hi - r_lo + 1);

    for (int v = tid; v < kVecs; v += kThreads) reinterpret_cast<uint4 *>(tile)[v] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();

    for (int rb = wave * kBackRows; rb < n_rows; rb += kWavesPerBlock * kBackRows) {
        // first chunk of up to kBackRows rows: records, then the gathered dp, all loads issued before any use
        int col[kBackRows];
        float v[kBackRows], d[kBackRows];
        bool ok[kBackRows];
        int cnt[kBackRows];
#pragma unroll
        for (int u = 0; u < kBackRows; ++u) {
            const int64_t r = r_lo + rb + u;
            const bool row_ok = rb + u < n_rows;
            cnt[u] = row_ok ? (counts ? min(counts[r], k) : k) : 0;
            ok[u] = lane < cnt[u];
            col[u] = 0xFFFF;
            v[u] = 0.0f;
            if (ok[u]) {
                col[u] = idx[r * (int64_t)k + lane];
                v[u] = Elem<T>::load(vals + r * (int64_t)k + lane);
            }
        }
#pragma unroll
        for (int u = 0; u < kBackRows; ++u) {
            ok[u] = ok[u] && col[u] < cols;
            d[u] = ok[u] ? Elem<T>::load(dp + (r_lo + rb + u) * (int64_t)cols + col[u]) : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kBackRows; ++u) {
            if (rb + u >= n_rows) break;                        // wave-uniform
            const int64_t r = r_lo + rb + u;
            const T *rv = vals + r * (int64_t)k;
            const uint16_t *ri = idx + r * (int64_t)k;
            const T *rd = dp + r * (int64_t)cols;
            float part = ok[u] ? v[u] * d[u] : 0.0f;
            for (int s = lane + kWave; s < cnt[u]; s += kWave) {        // records past the first 64
                const int c = ri[s];
                if (c < cols) part = fmaf(Elem<T>::load(rv + s), Elem<T>::load(rd + c), part);
            }
            const float dot = wave_sum_f32(part);
            const int64_t base = r * (int64_t)cols - t0;                // the row's start relative to the tile
            if (ok[u]) {
                const int64_t at = base + col[u];
                if (at >= 0 && at < n) tile[at] = Narrow<T>::from(v[u] * (d[u] - dot));
            }
            for (int s = lane + kWave; s < cnt[u]; s += kWave) {
                const int c = ri[s];
                const int64_t at = base + c;
                if (c < cols && at >= 0 && at < n)
                    tile[at] = Narrow<T>::from(Elem<T>::load(rv + s) * (Elem<T>::load(rd + c) - dot));
            }
        }
    }
    __syncthreads();

    T *dst = out + t0;
    const int n_vec = n / PER16;
    for (int e = tid; e < n_vec; e += kThreads)
        store_global<true>(reinterpret_cast<u32x4 *>(dst) + e, reinterpret_cast<const u32x4 *>(tile)[e]);
    for (int e = n_vec * PER16 + tid; e < n; e += kThreads) dst[e] = tile[e];
}

// The same for rows that keep few pairs (k <= kSmallK): a wave per row would leave most lanes idle, so
// the records of all the tile's rows are spread over the threads instead.  Three phases: every record's
// product p^ * dp goes to LDS; groups of eight lanes add the k products of a row each (lane g takes
// products g, g+8, ..., then three lane exchanges inside the group: a fixed order); the LDS buffer is then
// cleared and refilled as the output tile.  A thread keeps its first two records in registers across the
// phases; further ones are fetched again.
#ifndef SLIMFIT_SMB_SMALL_BELOW
#define SLIMFIT_SMB_SMALL_BELOW 33           // rows keeping fewer pairs than this take the record-spread kernel
                                             // (k = 9: 2.2x faster than a wave per row; k = 38: 1 % slower)
#endif
constexpr int kSmallK = 64;
constexpr int kSmallRecs = kTile + 2 * kSmallK;              // records of the rows touching one tile: k <= cols
constexpr int kSmallMinCols = 32;                            // at most kTile / 32 + 2 rows touch a tile
constexpr int kSmallRows = kTile / kSmallMinCols + 2;

template <typename T>
__global__ __launch_bounds__(kThreads) void softmax_backward_small_kernel(const T *__restrict__ vals,
                                                                          const uint16_t *__restrict__ idx,
                                                                          const int32_t *__restrict__ counts,
                                                                          const T *__restrict__ dp, int64_t rows,
                                                                          int cols, int k, T *__restrict__ out)
{
    __shared__ alignas(16) float buf[kSmallRecs];            // products first, the output tile afterwards
    __shared__ float dots[kSmallRows];
    T *tile = reinterpret_cast<T *>(buf);
    constexpr int PER16 = 16 / (int)sizeof(T);
    constexpr int kVecs = kTile / PER16;
    const int tid = threadIdx.x;
    const int64_t total = rows * (int64_t)cols;
    const int64_t t0 = (int64_t)blockIdx.x * kTile;
    const int n = (int)min((int64_t)kTile, total - t0);
    const int64_t r_lo = t0 / cols, r_hi = (t0 + n - 1) / cols;
    const int n_rows = (int)(r_hi - r_lo + 1);               // <= kSmallRows because cols >= kSmallMinCols
    const int n_rec = n_rows * k;                            // <= kSmallRecs
    const int64_t rec0 = r_lo * (int64_t)k;

    // record j of the tile: row r_lo + j / k, slot j % k; used (and its column, value, gradient) or not
    auto fetch = [&](int j, int &rl, int &col, float &v, float &d) {
        rl = j / k;
        const int sl = j - rl * k;
        const int64_t r = r_lo + rl;
        const int cnt = counts ? counts[r] : k;
        col = -1;
        v = d = 0.0f;
        if (sl < cnt) {
            const int c = idx[rec0 + j];
            if (c < cols) {
                col = c;
                v = Elem<T>::load(vals + rec0 + j);
                d = Elem<T>::load(dp + r * (int64_t)cols + c);
            }
        }
    };
    constexpr int PRE = 2;
    int pre_rl[PRE], pre_col[PRE];
    float pre_v[PRE], pre_d[PRE];
#pragma unroll
    for (int u = 0; u < PRE; ++u) {
        const int j = tid + u * kThreads;
        pre_rl[u] = 0;
        pre_col[u] = -1;
        pre_v[u] = pre_d[u] = 0.0f;
        if (j < n_rec) fetch(j, pre_rl[u], pre_col[u], pre_v[u], pre_d[u]);
    }
#pragma unroll
    for (int u = 0; u < PRE; ++u) {
        const int j = tid + u * kThreads;
        if (j < n_rec) buf[j] = pre_v[u] * pre_d[u];          // an unused record contributes +0
    }
    for (int j = tid + PRE * kThreads; j < n_rec; j += kThreads) {
        int rl, col;
        float v, d;
        fetch(j, rl, col, v, d);
        buf[j] = v * d;
    }
    __syncthreads();

    // the row sums: eight lanes a row (the exchanges stay inside a group of eight, whose lanes share rl)
    for (int rl = tid >> 3; rl < n_rows; rl += kThreads / 8) {
        const int g = tid & 7;
        float part = 0.0f;
        for (int sl = g; sl < k; sl += 8) part += buf[rl * k + sl];
        part += dpp_f32<kDppXor1>(part);
        part += dpp_f32<kDppXor2>(part);
        part += dpp_f32<kDppHalfMirror>(part);
        if (g == 0) dots[rl] = part;
    }
    __syncthreads();

    for (int v = tid; v < kVecs; v += kThreads) reinterpret_cast<uint4 *>(tile)[v] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();

    auto place = [&](int rl, int col, float v, float d) {
        if (col < 0) return;
        const int64_t at = (r_lo + rl) * (int64_t)cols + col - t0;
        if (at >= 0 && at < n) tile[at] = Narrow<T>::from(v * (d - dots[rl]));
    };
#pragma unroll
    for (int u = 0; u < PRE; ++u) place(pre_rl[u], pre_col[u], pre_v[u], pre_d[u]);
    for (int j = tid + PRE * kThreads; j < n_rec; j += kThreads) {
        int rl, col;
        float v, d;
        fetch(j, rl, col, v, d);
        place(rl, col, v, d);
    }
    __syncthreads();

    T *dst = out + t0;
    const int n_vec = n / PER16;
    for (int e = tid; e < n_vec; e += kThreads)
        store_global<true>(reinterpret_cast<u32x4 *>(dst) + e, reinterpret_cast<const u32x4 *>(tile)[e]);
    for (int e = n_vec * PER16 + tid; e < n; e += kThreads) dst[e] = tile[e];
}

template <typename T, bool SOFTMAX>
void launch_prune(const void *p, int64_t rows, int cols, int k, int mode, float tau, void *vals, uint16_t *idx,
                  int32_t *counts, void *probs, hipStream_t st)
{
    const T *pp = static_cast<const T *>(p);
    T *vv = static_cast<T *>(vals);
    T *pr = static_cast<T *>(probs);
    constexpr int32_t dt = sizeof(T) == 4 ? SLIMFIT_F32 : SLIMFIT_BF16;
    if (!SOFTMAX && SLIMFIT_PRUNE_SHORT && prune_short_eligible(p, dt, rows, cols, k)) {
        launch_prune_short(p, dt, rows, cols, k, mode, tau, vals, idx, counts, st);
        return;
    }
    if (SOFTMAX && SLIMFIT_SOFTMAX_SHORT && prune_short_eligible(p, dt, rows, cols, k) && aligned_to(probs, 16)) {
        launch_softmax_prune_short(p, dt, rows, cols, k, probs, vals, idx, st);      // (the dense rows leave in 16-byte stores)
        return;
    }
    const int slots = (cols + kWave - 1) / kWave;
    if (slots > kMaxRegSlots) {                       // never with SOFTMAX: the entry point rejects such rows
        const int bslots = (cols + kThreads - 1) / kThreads;              // slots per thread of a whole workgroup
        const unsigned bgrid = (unsigned)(rows < (1 << 20) ? rows : (1 << 20));
        if (bslots <= 8) prune_rows_block_kernel<T, 8><<<bgrid, kThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts);
        else if (bslots <= 16) prune_rows_block_kernel<T, 16><<<bgrid, kThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts);
        else if (bslots <= 32) prune_rows_block_kernel<T, 32><<<bgrid, kThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts);
        else if (bslots <= 64) prune_rows_block_kernel<T, 64><<<bgrid, kThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts);
        else {
            const unsigned grid = (unsigned)(rows < 16384 ? rows : 16384);
            prune_rows_wide_kernel<T><<<grid, kThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts);
        }
        return;
    }
    const int64_t rows_per_block = (int64_t)kRowWaves * kRowsPerUnit;
    const int64_t blocks_needed = (rows + rows_per_block - 1) / rows_per_block;
    const unsigned grid = (unsigned)(blocks_needed < kMaxPruneBlocks ? blocks_needed : kMaxPruneBlocks);
#define SLIMFIT_PRUNE_LAUNCH(MM, FF, SS)                                                                       \
    prune_rows_kernel<T, MM, FF, SS, SOFTMAX><<<grid, kRowThreads, 0, st>>>(pp, rows, cols, k, mode, tau, vv, idx, counts, pr)
#define SLIMFIT_PRUNE_CASE(MM)                                                                                  \
    do {                                                                                                        \
        const bool full = cols == MM * kWave, staged = k <= kStage;                                             \
        if (full && staged) SLIMFIT_PRUNE_LAUNCH(MM, true, true);                                               \
        else if (full) SLIMFIT_PRUNE_LAUNCH(MM, true, false);                                                   \
        else if (staged) SLIMFIT_PRUNE_LAUNCH(MM, false, true);                                                 \
        else SLIMFIT_PRUNE_LAUNCH(MM, false, false);                                                            \
    } while (0)
    if (slots <= 1) SLIMFIT_PRUNE_CASE(1);
    else if (slots <= 2) SLIMFIT_PRUNE_CASE(2);
    else if (slots <= 3) SLIMFIT_PRUNE_CASE(3);
    else if (slots <= 4) SLIMFIT_PRUNE_CASE(4);
    else if (slots <= 6) SLIMFIT_PRUNE_CASE(6);
    else if (slots <= 8) SLIMFIT_PRUNE_CASE(8);
    else if (slots <= 12) SLIMFIT_PRUNE_CASE(12);
    else if (slots <= 16) SLIMFIT_PRUNE_CASE(16);
#if SLIMFIT_PRUNE_WAVE_SLOTS >= 32
    else if (slots <= 24) SLIMFIT_PRUNE_LAUNCH(24, false, false);       // wide rows: no staging, ragged or not
    else if (slots <= 32) SLIMFIT_PRUNE_LAUNCH(32, false, false);
#endif
#if SLIMFIT_PRUNE_WAVE_SLOTS >= 64
    else if (slots <= 48) SLIMFIT_PRUNE_LAUNCH(48, false, false);
    else if (slots <= 64) SLIMFIT_PRUNE_LAUNCH(64, false, false);
#endif
#undef SLIMFIT_PRUNE_CASE
#undef SLIMFIT_PRUNE_LAUNCH
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
    StreamScope capture_aware(stream);
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
    if (dt == SLIMFIT_F32) launch_prune<float, false>(p, rows, cols, k, mode, tau, vals, idx, counts, nullptr, st);
    else launch_prune<uint16_t, false>(p, rows, cols, k, mode, tau, vals, idx, counts, nullptr, st);
    return launch_status();
}

extern "C" int32_t slimfit_softmax_prune(const void *logits, int32_t dt, int64_t rows, int32_t cols, int32_t k,
                                         void *probs, void *vals, uint16_t *idx, void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(dt, rows, cols, k);
    if (rc != SLIMFIT_OK) return rc;
    if (cols > kMaxRegSlots * kWave) return SLIMFIT_ERR_UNSUPPORTED;      // the row has to fit one wave's registers
    if (rows == 0) return SLIMFIT_OK;
    if (!logits || !probs || !vals || !idx || logits == probs) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    if (!aligned_to(logits, esz) || !aligned_to(probs, esz) || !aligned_to(vals, esz) || !aligned_to(idx, 2))
        return SLIMFIT_ERR_ALIGNMENT;
    if ((rc = check_device_range(logits, (size_t)rows * (size_t)cols * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(probs, (size_t)rows * (size_t)cols * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(vals, (size_t)rows * (size_t)k * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(idx, (size_t)rows * (size_t)k * 2)) != SLIMFIT_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dt == SLIMFIT_F32)
        launch_prune<float, true>(logits, rows, cols, k, SLIMFIT_PRUNE_TOPK, 0.0f, vals, idx, nullptr, probs, st);
    else
        launch_prune<uint16_t, true>(logits, rows, cols, k, SLIMFIT_PRUNE_TOPK, 0.0f, vals, idx, nullptr, probs, st);
    return launch_status();
}

extern "C" int32_t slimfit_restore_scores(const void *vals, const uint16_t *idx, const int32_t *counts, int32_t dt,
                                          int64_t rows, int32_t cols, int32_t k, void *out, void *stream)
{
    StreamScope capture_aware(stream);
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
    const int64_t total = rows * (int64_t)cols;
    const int64_t tiles = (total + kTile - 1) / kTile;
    if (tiles > 0x7FFFFFFF) return SLIMFIT_ERR_UNSUPPORTED;
    if (dt == SLIMFIT_F32)
        restore_tile_kernel<float><<<(unsigned)tiles, kThreads, 0, st>>>(static_cast<const float *>(vals), idx, counts,
                                                                         rows, cols, k, static_cast<float *>(out));
    else
        restore_tile_kernel<uint16_t><<<(unsigned)tiles, kThreads, 0, st>>>(static_cast<const uint16_t *>(vals), idx,
                                                                            counts, rows, cols, k,
                                                                            static_cast<uint16_t *>(out));
    return launch_status();
}

extern "C" int32_t slimfit_softmax_backward_pruned(const void *vals, const uint16_t *idx, const int32_t *counts,
                                                   const void *dp, int32_t dt, int64_t rows, int32_t cols, int32_t k,
                                                   void *ds, void *stream)
{
    StreamScope capture_aware(stream);
    int32_t rc = validate(dt, rows, cols, k);
    if (rc != SLIMFIT_OK) return rc;
    if (rows == 0) return SLIMFIT_OK;
    if (!vals || !idx || !dp || !ds || dp == ds) return SLIMFIT_ERR_INVALID_ARG;
    const size_t esz = dtype_size(dt);
    if (!aligned_to(ds, 16) || !aligned_to(dp, esz) || !aligned_to(vals, esz) || !aligned_to(idx, 2) ||
        (counts && !aligned_to(counts, 4)))
        return SLIMFIT_ERR_ALIGNMENT;
    const size_t dense_bytes = (size_t)rows * (size_t)cols * esz;
    if ((rc = check_device_range(ds, dense_bytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dp, dense_bytes)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(vals, (size_t)rows * (size_t)k * esz)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(idx, (size_t)rows * (size_t)k * 2)) != SLIMFIT_OK) return rc;
    if (counts && (rc = check_device_range(counts, (size_t)rows * 4)) != SLIMFIT_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t total = rows * (int64_t)cols;
    const int64_t tiles = (total + kTile - 1) / kTile;
    if (tiles > 0x7FFFFFFF) return SLIMFIT_ERR_UNSUPPORTED;
    const bool small = k <= kSmallK && cols >= kSmallMinCols && k < SLIMFIT_SMB_SMALL_BELOW;
    if (dt == SLIMFIT_F32) {
        const float *v = static_cast<const float *>(vals), *g = static_cast<const float *>(dp);
        float *o = static_cast<float *>(ds);
        if (small) softmax_backward_small_kernel<float><<<(unsigned)tiles, kThreads, 0, st>>>(v, idx, counts, g, rows, cols, k, o);
        else softmax_backward_tile_kernel<float><<<(unsigned)tiles, kThreads, 0, st>>>(v, idx, counts, g, rows, cols, k, o);
    } else {
        const uint16_t *v = static_cast<const uint16_t *>(vals), *g = static_cast<const uint16_t *>(dp);
        uint16_t *o = static_cast<uint16_t *>(ds);
        if (small) softmax_backward_small_kernel<uint16_t><<<(unsigned)tiles, kThreads, 0, st>>>(v, idx, counts, g, rows, cols, k, o);
        else softmax_backward_tile_kernel<uint16_t><<<(unsigned)tiles, kThreads, 0, st>>>(v, idx, counts, g, rows, cols, k, o);
    }
    return launch_status();
}
