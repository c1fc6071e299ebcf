// Pruning of short score rows that keep few entries (Alg. 5 applied per row; the
// appendix on pruning), for gfx950: rows of at most 256 columns, k <= 16 (bf16)
// or k <= 9 (fp32).
//
// With 197-column rows a wave that owns one row at a time spends most of its
// instructions on per-row bookkeeping (wave reductions, a bin scan, scalar
// popcounts) that does not shrink with the row.  Here nothing is done per row by
// a whole wave.  G lanes (2 or 4) share a row, so a wave works on R = 64 / G
// consecutive rows at once, and every lane owns one contiguous segment of its
// row (E = ceil(cols / G) entries):
//
//   stage    the wave's R consecutive rows are one contiguous, 16-byte aligned
//            piece of the tensor: copied to LDS with 16-byte non-temporal loads
//            (the only pass over HBM);
//   select   each lane keeps the largest CH keys of its segment in a sorted
//            register list: inserting a key is one v_max plus CH-1 v_med3
//            (new s[i] = median(s[i-1], s[i], key)), no branch, no cross-lane step.
//            A key carries the entry's column below its value (bf16: the 16 value
//            bits and the column; fp32: the upper 24 bits of the value's image and
//            the column), so ties go to the lower column and the list itself names
//            the columns.
//   merge    the G sorted lists of a row are merged by DPP exchanges inside the
//            quad (the partner's j-th largest can only land at position >= j).
//   fp32     24 value bits decide the kept set exactly unless the k-th and the
//            (k+1)-th largest agree in all of them (or, with a threshold, an entry
//            agrees with the threshold in all of them): about 0.1 % of 197-column
//            softmax rows, 1.5 % of their waves.  A wave that has such a row repeats the selection on the full
//            32-bit images (no columns), then walks its segment once more to
//            place the kept columns: the exact route, same result.
//   output   the kept columns are sorted in registers, staged in LDS in output
//            order and leave as contiguous runs; fp32 values (and bf16 ones when
//            a sign bit was seen, so that -0 stays -0) are re-read from the staged
//            rows.
//
// Keys: the bit patterns themselves, read as signed integers, order positive
// entries correctly and put zeros and negative entries below them, which is all
// a row needs whose kept entries are positive (every softmax row).  A wave that
// meets a row whose k-th largest entry is not positive starts over with
// sign * magnitude keys (-0 and +0 coincide, as float comparison has it).
#include "common.hpp"

#include <climits>
#include <utility>

namespace slimfit {
namespace {

#ifndef SLIMFIT_SHORT_NT
#define SLIMFIT_SHORT_NT 1             // the rows are streamed once
#endif
#ifndef SLIMFIT_SHORT_NT_STORE
#define SLIMFIT_SHORT_NT_STORE 0       // the pairs leave through the cache: plain stores are acknowledged sooner
#endif
#ifndef SLIMFIT_SHORT_FORCE_EXACT
#define SLIMFIT_SHORT_FORCE_EXACT 0    // tests of the exact route: take it for every wave
#endif

__device__ __forceinline__ int med3_i32(int a, int b, int c)
{
    // written as an instruction: max(min(a, b), min(max(a, b), c)) compiles to the same v_med3_i32, but chains
    // of it take the optimiser minutes to analyse
    int d;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// (a & mask) | b in one instruction; mask sits in a register because the three-operand encoding takes no literal
__device__ __forceinline__ int and_or_i32(int a, int mask, int b)
{
    int d;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(mask), "s"(b));
    return d;
}

// s is sorted in descending order; afterwards it holds the CH largest of s + {key}
template <int CH>
__device__ __forceinline__ void chain_insert(int (&s)[CH], int key)
{
#pragma unroll
    for (int i = CH - 1; i >= 1; --i) s[i] = med3_i32(s[i - 1], s[i], key);
    s[0] = max(s[0], key);
}

// the same for b[0] >= b[1] >= ...: b[j] cannot land above position j
template <int CH>
__device__ __forceinline__ void chain_merge(int (&m)[CH], const int (&b)[CH])
{
#pragma unroll
    for (int j = 0; j < CH; ++j) {
#pragma unroll
        for (int i = CH - 1; i >= (j > 1 ? j : 1); --i) m[i] = med3_i32(m[i - 1], m[i], b[j]);
        if (j == 0) m[0] = max(m[0], b[0]);
    }
}

// every lane of a row ends with the merged list of the row's G lanes
template <int G, int CH>
__device__ __forceinline__ void merge_row(int (&m)[CH])
{
    int b[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) b[i] = (int)dpp_u32<kDppXor1>((uint32_t)m[i]);
    chain_merge<CH>(m, b);
    if constexpr (G == 4) {
#pragma unroll
        for (int i = 0; i < CH; ++i) b[i] = (int)dpp_u32<kDppXor2>((uint32_t)m[i]);
        chain_merge<CH>(m, b);
    }
}

// ascending, in place (odd-even transposition)
template <int N>
__device__ __forceinline__ void sort_ascending(uint32_t (&c)[N])
{
#pragma unroll
    for (int round = 0; round < N; ++round) {
#pragma unroll
        for (int i = round & 1; i + 1 < N; i += 2) {
            const uint32_t lo = min(c[i], c[i + 1]), hi = max(c[i], c[i + 1]);
            c[i] = lo;
            c[i + 1] = hi;
        }
    }
}

// sign * magnitude of a float's bits (-0 -> 0)
__device__ __forceinline__ int signed_key_f32(uint32_t u)
{
    const int s = (int)u >> 31;
    return (int)(((u & 0x7FFFFFFFu) ^ (uint32_t)s) - (uint32_t)s);
}
// the same for 16 bits held sign-extended
__device__ __forceinline__ int signed_key_16(int v)
{
    const int s = v >> 31;
    return ((v & 0x7FFF) ^ s) - s;
}

struct ShortArgs {
    int64_t rows;
    int cols, k, mode;
    float tau;
    uint32_t div_magic;            // t / k == (t * div_magic) >> 16 for t < 64 * k
};

constexpr uint32_t kNoPair = 0xFFFF0000u;              // staging slot of an unused output position: column 0xFFFF

template <int... J, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, J...>, F f)
{
    (f(std::integral_constant<int, J>{}), ...);
}

// T: float or bf16 bits; G: lanes a row; K: largest k served; NV: 16-byte vectors a lane holds
template <typename T, int G, int K, int NV>
struct ShortRows {
    static constexpr bool BF = sizeof(T) == 2;
    static constexpr int R = kWave / G;
    static constexpr int CHP = BF ? K : K + 1;                 // list length: fp32 also wants the (k+1)-th largest
    static constexpr int TAG_BITS = BF ? 7 : 6;                // entry's rank inside the lane's segment
    static constexpr int N_OUT = (R * K + kWave - 1) / kWave;  // output pairs a lane stores

    // Visits the lane's entries e = 0 .. E-1 in column order: f(e, bits, ok) with the entry's bits (fp32: its
    // 32; bf16: its 16, zero-extended, or sign-extended when SEXT) and ok = "this lane has an entry e".  seg:
    // the lane's segment among the staged rows (LDS).  Blocks of kBlk entries; two register buffers take
    // turns, so a block's LDS reads are in flight while the one before it is worked on (f may hold asm
    // statements, which a run-time trip count cannot be unrolled around: blocks by hand).
    static constexpr int kBlk = 8;
    template <bool SEXT, typename F>
    static __device__ __forceinline__ void for_each_entry(const T *seg, int E, int len, int e_all, F f)
    {
        auto bits_at = [&](int e) -> int {
            if constexpr (BF) return SEXT ? (int)(int16_t)seg[e] : (int)seg[e];
            else return (int)__builtin_bit_cast(uint32_t, seg[e]);
        };
        const int n_blk = e_all / kBlk;                    // blocks every lane has in full
        int A[kBlk], B[kBlk];
        if (n_blk > 0) {
#pragma unroll
            for (int u = 0; u < kBlk; ++u) A[u] = bits_at(u);
        }
        for (int bi = 0; bi < n_blk; bi += 2) {
            if (bi + 1 < n_blk) {
#pragma unroll
                for (int u = 0; u < kBlk; ++u) B[u] = bits_at((bi + 1) * kBlk + u);
            }
#pragma unroll
            for (int u = 0; u < kBlk; ++u) f(bi * kBlk + u, A[u], true);
            if (bi + 1 < n_blk) {
                if (bi + 2 < n_blk) {
#pragma unroll
                    for (int u = 0; u < kBlk; ++u) A[u] = bits_at((bi + 2) * kBlk + u);
                }
#pragma unroll
                for (int u = 0; u < kBlk; ++u) f((bi + 1) * kBlk + u, B[u], true);
            }
        }
        // the ragged end: entries some lanes do not have.  Such a lane reads a few entries past its segment
        // (the next row's, or at most three entries past the staged rows: still inside the wave's LDS).
        for (int e0 = n_blk * kBlk; e0 < E; e0 += kBlk) {
#pragma unroll
            for (int u = 0; u < kBlk; ++u) {
                if (e0 + u < E) A[u] = bits_at(e0 + u);    // wave-uniform
            }
#pragma unroll
            for (int u = 0; u < kBlk; ++u) {
                if (e0 + u < E) f(e0 + u, A[u], e0 + u < len);
            }
        }
    }

    // NEG: keys are sign * magnitude.  Without it the bit patterns themselves serve as (signed) keys, which orders
    // the positive entries correctly and puts everything else (zeros of either sign, negative values in reversed
    // order) below them: enough whenever every kept entry is positive.  The plain pass notices when that fails for
    // one of the wave's rows and returns false before it has written anything; the caller then runs the signed pass.
    // between(): called once, after the kept columns are staged and before the kept values are fetched from the
    // staged rows (FROM_ROWS: always from there); the fused softmax rewrites the rows in between.
    struct Nothing {
        __device__ void operator()() const {}
    };
    template <bool NEG, bool FROM_ROWS = false, typename Between = Nothing>
    static __device__ bool run(const ShortArgs &a, const T *rows_lds, uint32_t *oc, int lane, int n_here, int64_t row0,
                               T *__restrict__ vals, uint16_t *__restrict__ idx, int32_t *__restrict__ counts,
                               Between between = Between())
    {
        const int cols = a.cols, k = a.k;
        const int r = lane / G, q = lane % G;
        const int E = (cols + G - 1) / G;                  // entries a lane
        const int len = min(max(cols - q * E, 0), E);      // this lane's
        const int e_all = max(cols - (G - 1) * E, 0);      // the last lane's: the shortest segment
        const T *seg = rows_lds + r * cols + q * E;
        constexpr int TAG_TOP = (1 << TAG_BITS) - 1;
        constexpr uint32_t COL_MASK = (1u << (TAG_BITS + 2)) - 1u;      // rank in the segment, lane of the row

        // ---- selection on keys that carry the column ---------------------------------
        int m[CHP];
#pragma unroll
        for (int i = 0; i < CHP; ++i) m[i] = INT_MIN;
        int value_mask = (int)~COL_MASK;
        asm("" : "+v"(value_mask));                        // in a register, not a literal at every use
        for_each_entry<NEG>(seg, E, len, e_all, [&](int e, int bits, bool ok) {
            // the tag is wave-uniform: the earlier entry of the segment ranks higher
            int key;
            if constexpr (BF) key = (int)(((uint32_t)(NEG ? signed_key_16(bits) : bits) << 16) | (uint32_t)(TAG_TOP - e));
            else key = and_or_i32(NEG ? signed_key_f32((uint32_t)bits) : bits, value_mask, TAG_TOP - e);
            chain_insert<CHP>(m, ok ? key : INT_MIN);
        });
#pragma unroll
        for (int i = 0; i < CHP; ++i) m[i] |= (G - 1 - q) << TAG_BITS;     // lanes of lower columns rank higher
        merge_row<G, CHP>(m);

        auto column_of = [&](int key) {
            const int low = key & (int)COL_MASK;
            return (G - 1 - (low >> TAG_BITS)) * E + (TAG_TOP - (low & TAG_TOP));
        };
        int kk = k;
        bool exact = false;                                 // this row has to take the exact route (fp32 only)
        uint32_t c[K];                                      // kept (column << 16 | bf16 value bits), kNoPair beyond kk
        if constexpr (!NEG) {
            // all kept entries positive?  With k entries kept: the k-th largest is; with fewer (a threshold run): tau is.
            int cut_value = 0;
#pragma unroll
            for (int i = 0; i < K; ++i) cut_value = (i == k - 1) ? m[i] >> (BF ? 16 : TAG_BITS + 2) : cut_value;
            const bool plain_ok = cut_value > 0 || (a.mode == SLIMFIT_PRUNE_THRESHOLD && a.tau > 0.0f);
            if (__builtin_amdgcn_ballot_w64(!plain_ok) != 0) return false;
        }
        if constexpr (BF) {
            auto bits_of = [&](int key) -> uint32_t {
                const int k16 = key >> 16;
                if constexpr (NEG) return k16 < 0 ? ((uint32_t)(-k16) | 0x8000u) : (uint32_t)k16;
                else return (uint32_t)k16 & 0xFFFFu;
            };
            if (a.mode == SLIMFIT_PRUNE_THRESHOLD) {
                int n = 0;
#pragma unroll
                for (int i = 0; i < K; ++i) n += (i < k && bf16_widen(bits_of(m[i])) >= a.tau) ? 1 : 0;
                kk = n;
            }
#pragma unroll
            for (int i = 0; i < K; ++i)
                c[i] = i < kk ? ((uint32_t)min(column_of(m[i]), cols - 1) << 16) | bits_of(m[i]) : kNoPair;
        } else {
            int cut_v = INT_MIN, next_v = INT_MIN;          // value bits of the k-th and the (k+1)-th largest
#pragma unroll
            for (int i = 0; i < CHP; ++i) {
                cut_v = (i == k - 1) ? m[i] >> (TAG_BITS + 2) : cut_v;
                next_v = (i == k) ? m[i] >> (TAG_BITS + 2) : next_v;
            }
            exact = cut_v == next_v;
            if (a.mode == SLIMFIT_PRUNE_THRESHOLD) {
                const int tau_v = signed_key_f32(__builtin_bit_cast(uint32_t, a.tau)) >> (TAG_BITS + 2);
                int n = 0;
                bool unsure = false;
#pragma unroll
                for (int i = 0; i < K; ++i) {
                    const int v = m[i] >> (TAG_BITS + 2);
                    n += (i < k && v > tau_v) ? 1 : 0;
                    unsure = unsure || (i < k && v == tau_v);
                }
                if (n < k) exact = false;                   // fewer than k pass: the kept set is {entries >= tau}
                kk = n;
                exact = exact || unsure;
            }
#pragma unroll
            for (int i = 0; i < K; ++i) c[i] = i < kk ? (uint32_t)min(column_of(m[i]), cols - 1) << 16 : kNoPair;
        }

        uint32_t *orow = oc + r * k;
        const bool any_exact = !BF && (SLIMFIT_SHORT_FORCE_EXACT || __builtin_amdgcn_ballot_w64(exact) != 0);
        if (!any_exact) {
            sort_ascending<K>(c);
#pragma unroll
            for (int i = 0; i < K; ++i)
                if (i % G == q && i < k) orow[i] = c[i];
        }
        if constexpr (!BF) {
            if (any_exact) {
                // ---- the exact route: full 32-bit images, then a second walk over the registers ----
                constexpr int CH = K + 1;
                int s[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i) s[i] = INT_MIN;
                auto full_key = [&](int bits) { return NEG ? signed_key_f32((uint32_t)bits) : bits; };
                for_each_entry<NEG>(seg, E, len, e_all,
                                    [&](int e, int bits, bool ok) { chain_insert<CH>(s, ok ? full_key(bits) : INT_MIN); });
                int mm[CH];
#pragma unroll
                for (int i = 0; i < CH; ++i) mm[i] = s[i];
                merge_row<G, CH>(mm);
                int cut = INT_MIN, cut_next = INT_MIN;
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    cut = (i == k - 1) ? mm[i] : cut;
                    cut_next = (i == k) ? mm[i] : cut_next;
                }
                bool take_all_equal = cut_next != cut;      // exactly k entries reach the cut
                kk = k;
                if (a.mode == SLIMFIT_PRUNE_THRESHOLD) {
                    const int tau_key = signed_key_f32(__builtin_bit_cast(uint32_t, a.tau));
                    int n = 0;
#pragma unroll
                    for (int i = 0; i < K; ++i) n += (i < k && mm[i] >= tau_key) ? 1 : 0;
                    if (n < k) {                            // fewer than k pass: all of them are kept
                        kk = n;
                        cut = tau_key;
                        take_all_equal = true;
                    }
                }
                // from its own list a lane knows how many of its entries are above the cut and how many equal it
                int gt = 0, eq = 0;
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    gt += s[i] > cut ? 1 : 0;
                    eq += s[i] == cut ? 1 : 0;
                }
                int gt_of[G], eq_of[G];                     // the same of every lane of the row
                if constexpr (G == 4) {
                    gt_of[0] = (int)dpp_u32<0x00>((uint32_t)gt); gt_of[1] = (int)dpp_u32<0x55>((uint32_t)gt);
                    gt_of[2] = (int)dpp_u32<0xAA>((uint32_t)gt); gt_of[3] = (int)dpp_u32<0xFF>((uint32_t)gt);
                    eq_of[0] = (int)dpp_u32<0x00>((uint32_t)eq); eq_of[1] = (int)dpp_u32<0x55>((uint32_t)eq);
                    eq_of[2] = (int)dpp_u32<0xAA>((uint32_t)eq); eq_of[3] = (int)dpp_u32<0xFF>((uint32_t)eq);
                } else {
                    gt_of[0] = (int)dpp_u32<0xA0>((uint32_t)gt); gt_of[1] = (int)dpp_u32<0xF5>((uint32_t)gt);
                    eq_of[0] = (int)dpp_u32<0xA0>((uint32_t)eq); eq_of[1] = (int)dpp_u32<0xF5>((uint32_t)eq);
                }
                int gt_all = 0;
#pragma unroll
                for (int g = 0; g < G; ++g) gt_all += gt_of[g];
                int need = take_all_equal ? INT_MAX : kk - gt_all;      // equal entries still to hand out, lower columns first
                int base = 0, take_eq = 0;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const int t = min(max(need, 0), eq_of[g]);
                    if (g < q) base += gt_of[g] + t;
                    if (g == q) take_eq = t;
                    need = need == INT_MAX ? need : need - t;
                }
                // the same keys as in the selection, so the columns placed here are exactly the entries counted above
                uint32_t *out = orow + base;
                const int col0 = q * E;
                int seen = 0;
                for_each_entry<NEG>(seg, E, len, e_all, [&](int e, int bits, bool ok) {
                    const int key = full_key(bits);
                    const bool is_eq = ok && key == cut;
                    if ((ok && key > cut) || (is_eq && seen < take_eq)) *out++ = (uint32_t)(col0 + e) << 16;
                    seen += is_eq ? 1 : 0;
                });
            }
        }

        // ---- the wave's pairs in output order ----
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        between();
        const int n_out = n_here * k;
        constexpr bool REREAD = !BF || NEG || FROM_ROWS;    // values come from the staged rows again
        T *ov = vals + row0 * (int64_t)k;
        uint16_t *oi = idx + row0 * (int64_t)k;
        uint32_t w[N_OUT];
        T v[N_OUT];
#pragma unroll
        for (int it = 0; it < N_OUT; ++it) {
            const int t = it * kWave + lane;
            w[it] = t < n_out ? oc[t] : kNoPair;
        }
#pragma unroll
        for (int it = 0; it < N_OUT; ++it) {
            const uint32_t t = (uint32_t)(it * kWave + lane);
            const uint32_t rl = min((t * a.div_magic) >> 16, (uint32_t)(R - 1));
            v[it] = T(0);
            if constexpr (REREAD) {
                const T x = rows_lds[rl * (uint32_t)cols + min(w[it] >> 16, (uint32_t)cols - 1u)];
                if (w[it] != kNoPair) v[it] = x;
            } else {
                v[it] = (T)(w[it] & 0xFFFFu);
            }
        }
#pragma unroll
        for (int it = 0; it < N_OUT; ++it) {
            const int t = it * kWave + lane;
            if (t < n_out) {
                store_global<SLIMFIT_SHORT_NT_STORE != 0>(ov + t, v[it]);
                store_global<SLIMFIT_SHORT_NT_STORE != 0>(oi + t, (uint16_t)(w[it] >> 16));
            }
        }
        if (counts && q == 0 && r < n_here) counts[row0 + r] = kk;
        return true;
    }
};

// NV: 16-byte vectors a lane holds while the rows are staged (the wave's rows are 64 * cols bytes: NV >= cols / 16)
template <typename T, int G, int K, int NV>
__global__ __launch_bounds__(kWave) void prune_rows_short_kernel(const T *__restrict__ p, ShortArgs a,
                                                                 T *__restrict__ vals, uint16_t *__restrict__ idx,
                                                                 int32_t *__restrict__ counts)
{
    using S = ShortRows<T, G, K, NV>;
    extern __shared__ uint4 short_lds[];
    constexpr int R = S::R;
    constexpr int PER16 = 16 / (int)sizeof(T);
    static_assert(R * sizeof(T) % 16 == 0, "the wave's rows are a whole number of 16-byte vectors");
    const int lane = threadIdx.x;
    const int cols = a.cols, k = a.k;
    char *slab = reinterpret_cast<char *>(short_lds);
    const int slab_bytes = (R * cols * (int)sizeof(T) + 15) & ~15;
    uint32_t *oc = reinterpret_cast<uint32_t *>(slab + slab_bytes);        // R * k output slots
    u32x4 *dst_v = reinterpret_cast<u32x4 *>(slab);

    // The wave's R consecutive rows are one contiguous, 16-byte aligned piece of 64 * cols bytes.  No branch
    // around a load: lanes past the end of a short last piece re-read its last vector (and store it again where
    // it belongs), which keeps all NV loads in flight together.
    const int64_t row0 = (int64_t)blockIdx.x * R;
    const int n_here = (int)min((int64_t)R, a.rows - row0);        // >= 1 by the launch size
    const int n_elem = n_here * cols;
    const int n_vec = n_elem / PER16;
    const u32x4 *src_v = reinterpret_cast<const u32x4 *>(p + row0 * (int64_t)cols);
    if (n_vec > (NV - 1) * kWave) {
        // (wave-uniform) the piece fills all NV rounds but perhaps the last: no index arithmetic on the others
        u32x4 v[NV];
        const int last = min((NV - 1) * kWave + lane, n_vec - 1);
#pragma unroll
        for (int u = 0; u < NV - 1; ++u) v[u] = load_global<SLIMFIT_SHORT_NT != 0>(src_v + u * kWave + lane);
        v[NV - 1] = load_global<SLIMFIT_SHORT_NT != 0>(src_v + last);
#pragma unroll
        for (int u = 0; u < NV - 1; ++u) dst_v[u * kWave + lane] = v[u];
        dst_v[last] = v[NV - 1];
    } else if (n_vec > 0) {
        // fewer rounds (narrow rows for this NV, or a short last piece): lanes past the end re-read the last vector
        // (and store it again where it belongs), which keeps the loads free of branches
        u32x4 v[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) v[u] = load_global<SLIMFIT_SHORT_NT != 0>(src_v + min(u * kWave + lane, n_vec - 1));
#pragma unroll
        for (int u = 0; u < NV; ++u) dst_v[min(u * kWave + lane, n_vec - 1)] = v[u];
    }
    {
        const int ei = n_vec * PER16 + lane;           // fewer than PER16 entries are left over (short last piece only)
        if (ei < n_elem) reinterpret_cast<T *>(slab)[ei] = p[row0 * (int64_t)cols + ei];
    }
    // unused output slots read as "no pair"
    for (int t = lane; t < R * k; t += kWave) oc[t] = kNoPair;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const T *rows_lds = reinterpret_cast<const T *>(slab);
    if (!S::template run<false>(a, rows_lds, oc, lane, n_here, row0, vals, idx, counts))
        S::template run<true>(a, rows_lds, oc, lane, n_here, row0, vals, idx, counts);
}

// ---------------------------------------------------------------------------------------------------------------
// Row softmax and Alg. 5 in one pass over short rows of logits: the kept set is decided on the logits (which order
// a row exactly as its probabilities do), the dense probabilities are written once, and the kept values are the
// numbers the dense row holds.  The rows are staged and selected as above; before the kept values are fetched each
// lane turns its part of its row into probabilities in place (row maximum and sum of exponentials by exchanges
// between the row's G lanes; hardware exp2; four running sums a lane, so that no sum is longer than a quarter of
// the lane's part; one IEEE division a row), and the wave's rows leave for `probs` as they came, as one contiguous
// piece.
template <typename T, int G, int K, int NV>
__global__ __launch_bounds__(kWave) void softmax_prune_short_kernel(const T *__restrict__ p, ShortArgs a,
                                                                    T *__restrict__ probs, T *__restrict__ vals,
                                                                    uint16_t *__restrict__ idx)
{
    using S = ShortRows<T, G, K, NV>;
    extern __shared__ uint4 short_lds[];
    constexpr bool BF = sizeof(T) == 2;
    constexpr int R = S::R;
    constexpr int PER16 = 16 / (int)sizeof(T);
    const int lane = threadIdx.x;
    const int cols = a.cols, k = a.k;
    char *slab = reinterpret_cast<char *>(short_lds);
    const int slab_bytes = (R * cols * (int)sizeof(T) + 15) & ~15;
    uint32_t *oc = reinterpret_cast<uint32_t *>(slab + slab_bytes);        // R * k output slots
    u32x4 *slab_v = reinterpret_cast<u32x4 *>(slab);

    const int64_t row0 = (int64_t)blockIdx.x * R;
    const int n_here = (int)min((int64_t)R, a.rows - row0);        // >= 1 by the launch size
    const int n_elem = n_here * cols;
    const int n_vec = n_elem / PER16;
    const u32x4 *src_v = reinterpret_cast<const u32x4 *>(p + row0 * (int64_t)cols);
    if (n_vec > 0) {
        // lanes past the end of a short last piece re-read its last vector (and store it again where it belongs)
        u32x4 v[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) v[u] = load_global<SLIMFIT_SHORT_NT != 0>(src_v + min(u * kWave + lane, n_vec - 1));
#pragma unroll
        for (int u = 0; u < NV; ++u) slab_v[min(u * kWave + lane, n_vec - 1)] = v[u];
    }
    {
        const int ei = n_vec * PER16 + lane;           // fewer than PER16 entries are left over (short last piece only)
        if (ei < n_elem) reinterpret_cast<T *>(slab)[ei] = p[row0 * (int64_t)cols + ei];
    }
    for (int t = lane; t < R * k; t += kWave) oc[t] = kNoPair;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    auto to_probabilities = [&]() {
        const int r = lane / G, q = lane % G;
        const int E = (cols + G - 1) / G;
        const int len = min(max(cols - q * E, 0), E);
        const int e_all = max(cols - (G - 1) * E, 0);
        T *seg = reinterpret_cast<T *>(slab) + r * cols + q * E;
        auto value = [](int bits) { return __builtin_bit_cast(float, BF ? (uint32_t)bits << 16 : (uint32_t)bits); };
        constexpr float kLog2e = 1.44269504088896340736f;
        float mx = -__builtin_inff();
        S::template for_each_entry<false>(seg, E, len, e_all, [&](int, int bits, bool ok) {
            const float x = value(bits);
            mx = ok ? fmaxf(mx, x) : mx;
        });
        mx = fmaxf(mx, dpp_f32<kDppXor1>(mx));
        if constexpr (G == 4) mx = fmaxf(mx, dpp_f32<kDppXor2>(mx));
        // (a lane of a row past the tensor's end, or one without entries, holds -inf here: its results are not used)
        float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
        S::template for_each_entry<false>(seg, E, len, e_all, [&](int e, int bits, bool ok) {
            const float t = __builtin_amdgcn_exp2f((value(bits) - mx) * kLog2e);
            const float s = s0 + (ok ? t : 0.0f);           // the four sums take turns
            s0 = s1; s1 = s2; s2 = s3; s3 = s;
            if constexpr (!BF) {
                if (ok) seg[e] = t;                         // fp32 rows keep the exponential in place of the logit
            }
        });
        float sum = (s0 + s1) + (s2 + s3);
        sum += dpp_f32<kDppXor1>(sum);
        if constexpr (G == 4) sum += dpp_f32<kDppXor2>(sum);
        const float inv = 1.0f / sum;                       // IEEE division
        if constexpr (!BF) {                                // (the lane reads back what it wrote itself: LDS keeps a wave's order)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        S::template for_each_entry<false>(seg, E, len, e_all, [&](int e, int bits, bool ok) {
            const float pj = (BF ? __builtin_amdgcn_exp2f((value(bits) - mx) * kLog2e) : value(bits)) * inv;
            if (ok) {
                if constexpr (BF) seg[e] = (T)bf16_narrow(pj);
                else seg[e] = pj;
            }
        });
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // the dense rows leave as they came: one contiguous piece, 16 bytes a lane
        u32x4 *dst_v = reinterpret_cast<u32x4 *>(probs + row0 * (int64_t)cols);
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int v = u * kWave + lane;
            if (v < n_vec) store_global<true>(dst_v + v, slab_v[v]);
        }
        const int ei = n_vec * PER16 + lane;
        if (ei < n_elem) probs[row0 * (int64_t)cols + ei] = reinterpret_cast<const T *>(slab)[ei];
    };

    const T *rows_lds = reinterpret_cast<const T *>(slab);
    if (!S::template run<false, true>(a, rows_lds, oc, lane, n_here, row0, vals, idx, nullptr, to_probabilities))
        S::template run<true, true>(a, rows_lds, oc, lane, n_here, row0, vals, idx, nullptr, to_probabilities);
}

template <typename T, int G, int K, int NV>
void launch_softmax_short(const T *p, const ShortArgs &a, T *probs, T *vals, uint16_t *idx, hipStream_t st)
{
    constexpr int R = kWave / G;
    const int64_t blocks = (a.rows + R - 1) / R;
    const size_t lds = (size_t)((R * a.cols * (int)sizeof(T) + 15) & ~15) + (size_t)R * (size_t)a.k * 4u;
    softmax_prune_short_kernel<T, G, K, NV><<<(unsigned)blocks, kWave, lds, st>>>(p, a, probs, vals, idx);
}

template <typename T, int G, int K>
void launch_softmax_short_nv(const T *p, const ShortArgs &a, T *probs, T *vals, uint16_t *idx, hipStream_t st)
{
    constexpr int R = kWave / G;
    constexpr int S = R * (int)sizeof(T) / 64;
    const int nv = (a.cols * S * 4 + kWave - 1) / kWave;
    if (nv <= 4 * S) launch_softmax_short<T, G, K, 4 * S>(p, a, probs, vals, idx, st);
    else if (nv <= 8 * S) launch_softmax_short<T, G, K, 8 * S>(p, a, probs, vals, idx, st);
    else if (nv <= 12 * S + 1) launch_softmax_short<T, G, K, 12 * S + 1>(p, a, probs, vals, idx, st);
    else launch_softmax_short<T, G, K, 16 * S>(p, a, probs, vals, idx, st);
}

template <typename T, int G>
void launch_softmax_short_k(const T *p, const ShortArgs &a, T *probs, T *vals, uint16_t *idx, hipStream_t st)
{
    if (a.k <= 2) launch_softmax_short_nv<T, G, 2>(p, a, probs, vals, idx, st);
    else if (a.k <= 4) launch_softmax_short_nv<T, G, 4>(p, a, probs, vals, idx, st);
    else if (a.k <= 6) launch_softmax_short_nv<T, G, 6>(p, a, probs, vals, idx, st);
    else if (a.k <= 9) launch_softmax_short_nv<T, G, 9>(p, a, probs, vals, idx, st);
    else if constexpr (sizeof(T) == 2) {
        if (a.k <= 12) launch_softmax_short_nv<T, G, 12>(p, a, probs, vals, idx, st);
        else launch_softmax_short_nv<T, G, 16>(p, a, probs, vals, idx, st);
    }
}

template <typename T, int G, int K, int NV>
void launch_short(const T *p, const ShortArgs &a, T *vals, uint16_t *idx, int32_t *counts, hipStream_t st)
{
    constexpr int R = kWave / G;
    const int64_t blocks = (a.rows + R - 1) / R;
#ifndef SLIMFIT_SHORT_LDS_PAD
#define SLIMFIT_SHORT_LDS_PAD 0        // timing experiments only: LDS a wave claims beyond what it uses
#endif
    const size_t lds = (size_t)((R * a.cols * (int)sizeof(T) + 15) & ~15) + (size_t)R * (size_t)a.k * 4u + SLIMFIT_SHORT_LDS_PAD;
    prune_rows_short_kernel<T, G, K, NV><<<(unsigned)blocks, kWave, lds, st>>>(p, a, vals, idx, counts);
}

template <typename T, int G, int K>
void launch_short_nv(const T *p, const ShortArgs &a, T *vals, uint16_t *idx, int32_t *counts, hipStream_t st)
{
    constexpr int R = kWave / G;
    const int nv = (R * a.cols * (int)sizeof(T) / 16 + kWave - 1) / kWave;      // rounds of 64 vectors a piece takes
    if (nv <= 4) launch_short<T, G, K, 4>(p, a, vals, idx, counts, st);
    else if (nv <= 8) launch_short<T, G, K, 8>(p, a, vals, idx, counts, st);
    else if (nv <= 13) launch_short<T, G, K, 13>(p, a, vals, idx, counts, st);   // 197 columns
    else launch_short<T, G, K, 16>(p, a, vals, idx, counts, st);
}

template <typename T, int G>
void launch_short_k(const T *p, const ShortArgs &a, T *vals, uint16_t *idx, int32_t *counts, hipStream_t st)
{
    if (a.k <= 2) launch_short_nv<T, G, 2>(p, a, vals, idx, counts, st);
    else if (a.k <= 4) launch_short_nv<T, G, 4>(p, a, vals, idx, counts, st);
    else if (a.k <= 6) launch_short_nv<T, G, 6>(p, a, vals, idx, counts, st);
    else if (a.k <= 9) launch_short_nv<T, G, 9>(p, a, vals, idx, counts, st);
    else if constexpr (sizeof(T) == 2) {               // (fp32 rows that keep more than 9 entries are not routed here)
        if (a.k <= 12) launch_short_nv<T, G, 12>(p, a, vals, idx, counts, st);
        else launch_short_nv<T, G, 16>(p, a, vals, idx, counts, st);
    }
}

}  // namespace

// Measured against the wave-per-row kernel on 64 .. 250 columns: bf16 rows gain at every k <= 16 (1.2 - 4 times
// faster), fp32 rows up to k = 9 (1.2 - 1.8 times); fp32 rows that keep 12 or 16 entries lose 15 - 45 %, the
// list insertion growing with k.
bool prune_short_eligible(const void *p, int32_t dt, int64_t rows, int cols, int k)
{
    const int k_max = dt == SLIMFIT_BF16 ? kShortPruneMaxK : kShortPruneMaxKF32;
    // (the rows are staged with 16-byte loads)
    return cols <= kShortPruneMaxCols && k <= k_max && aligned_to(p, 16) && rows <= (int64_t)0x7FFFFFFF * 16;
}

void launch_softmax_prune_short(const void *logits, int32_t dt, int64_t rows, int cols, int k, void *probs, void *vals,
                                uint16_t *idx, hipStream_t st)
{
    ShortArgs a;
    a.rows = rows;
    a.cols = cols;
    a.k = k;
    a.mode = SLIMFIT_PRUNE_TOPK;
    a.tau = 0.0f;
    a.div_magic = 65536u / (uint32_t)k + 1u;
    if (dt == SLIMFIT_F32)
        launch_softmax_short_k<float, 4>(static_cast<const float *>(logits), a, static_cast<float *>(probs),
                                         static_cast<float *>(vals), idx, st);
    else
        launch_softmax_short_k<uint16_t, 2>(static_cast<const uint16_t *>(logits), a, static_cast<uint16_t *>(probs),
                                            static_cast<uint16_t *>(vals), idx, st);
}

void launch_prune_short(const void *p, int32_t dt, int64_t rows, int cols, int k, int mode, float tau, void *vals,
                        uint16_t *idx, int32_t *counts, hipStream_t st)
{
    ShortArgs a;
    a.rows = rows;
    a.cols = cols;
    a.k = k;
    a.mode = mode;
    a.tau = tau;
    a.div_magic = 65536u / (uint32_t)k + 1u;
#ifndef SLIMFIT_SHORT_G_F32
#define SLIMFIT_SHORT_G_F32 4
#endif
    if (dt == SLIMFIT_F32)
        launch_short_k<float, SLIMFIT_SHORT_G_F32>(static_cast<const float *>(p), a, static_cast<float *>(vals), idx, counts, st);
    else
#ifndef SLIMFIT_SHORT_G_BF16
#define SLIMFIT_SHORT_G_BF16 2
#endif
        launch_short_k<uint16_t, SLIMFIT_SHORT_G_BF16>(static_cast<const uint16_t *>(p), a, static_cast<uint16_t *>(vals), idx, counts, st);
}

}  // namespace slimfit
