// Training-dynamics freeze score (Eq. 1, Sec. 3.1): for every layer the mean
// of |W^t - W^{t-1}| / |W^{t-1}|, all layers in one launch.
//
// The layers of a model differ in size by three orders of magnitude (a
// LayerNorm vector next to a 4H x H matrix), so the work is cut into chunks of
// kChunk elements; chunk c of the launch belongs to exactly one layer.  Stage
// one streams both tensors of a chunk with 128-bit loads and writes one fp64
// partial sum; stage two adds the partials of each layer in a fixed order.
// No atomics, so the score is bit-identical from run to run.
//
// The workspace holds a header, the layer table (pointers, sizes, first chunk)
// and the partials.  The table is written by tiny kernels that receive up to
// kPlanBatch layers by value, which keeps planning asynchronous and free of
// host staging memory.
#include "common.hpp"

#include <mutex>
#include <vector>

namespace slimfit {
namespace {

#ifndef SLIMFIT_DELTA_CHUNK
#define SLIMFIT_DELTA_CHUNK 16384
#endif
#ifndef SLIMFIT_DELTA_NT
#define SLIMFIT_DELTA_NT 1                   // both tensors are streamed once
#endif
#ifndef SLIMFIT_DELTA_THREADS
#define SLIMFIT_DELTA_THREADS 256
#endif
constexpr int kThreads = SLIMFIT_DELTA_THREADS;
constexpr int kChunk = SLIMFIT_DELTA_CHUNK;  // elements per workgroup
constexpr bool kNT = SLIMFIT_DELTA_NT != 0;
#ifndef SLIMFIT_DELTA_APPLY_NT
#define SLIMFIT_DELTA_APPLY_NT 1             // the new weights are not read again before the caches have turned over
#endif
constexpr bool kApplyNT = SLIMFIT_DELTA_APPLY_NT != 0;
#ifndef SLIMFIT_DELTA_APPLY_SPLIT
#define SLIMFIT_DELTA_APPLY_SPLIT 1         // 2 or 4 parts per chunk: no faster
#endif
constexpr int kApplySplit = SLIMFIT_DELTA_APPLY_SPLIT;
constexpr uint32_t kMagic = 0x534C4644u;     // "SLFD"
constexpr int kPlanBatch = 32;

struct Header {                              // 64 bytes at the start of the workspace
    uint32_t magic;
    int32_t n_layers;
    int64_t total_chunks;
    int32_t prev_dt, cur_dt;
    int64_t pad[5];
};
static_assert(sizeof(Header) == 64, "header size");

struct LayerEntry {                          // 32 bytes
    const void *w_prev;
    const void *w_cur;
    int64_t numel;
    int64_t first_chunk;
};

struct PlanBatch {
    LayerEntry e[kPlanBatch];
};

inline size_t table_bytes(int32_t L) { return (sizeof(Header) + sizeof(LayerEntry) * (size_t)L + 255) & ~(size_t)255; }

__global__ void plan_write_kernel(char *ws, Header h, int first, int count, PlanBatch batch)
{
    LayerEntry *table = reinterpret_cast<LayerEntry *>(ws + sizeof(Header));
    const int t = threadIdx.x;
    if (t < count) table[first + t] = batch.e[t];
    if (first == 0 && t == 0) *reinterpret_cast<Header *>(ws) = h;
}

template <typename T> struct Load4;
template <> struct Load4<float> {
    __device__ static void vec(const float *p, float (&f)[4])
    {
        f32x4 r = load_global<kNT>(reinterpret_cast<const f32x4 *>(p));
        f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    }
    __device__ static float one(const float *p) { return *p; }
};
template <> struct Load4<uint16_t> {
    __device__ static void vec(const uint16_t *p, float (&f)[4])
    {
        u32x2 r = load_global<kNT>(reinterpret_cast<const u32x2 *>(p));
        f[0] = __builtin_bit_cast(float, r.x << 16); f[1] = __builtin_bit_cast(float, r.x & 0xFFFF0000u);
        f[2] = __builtin_bit_cast(float, r.y << 16); f[3] = __builtin_bit_cast(float, r.y & 0xFFFF0000u);
    }
    __device__ static float one(const uint16_t *p) { return bf16_widen(*p); }
};

// W^t = W^{t-1} + delta written back over W^{t-1}: one fp32 addition, bf16 weights rounded once more
template <typename T> struct Store4;
template <> struct Store4<float> {
    __device__ static void vec(float *p, const float (&f)[4])
    {
        store_global<kApplyNT>(reinterpret_cast<f32x4 *>(p), f32x4{f[0], f[1], f[2], f[3]});
    }
    __device__ static void one(float *p, float v) { *p = v; }
};
template <> struct Store4<uint16_t> {
    __device__ static void vec(uint16_t *p, const float (&f)[4])
    {
        store_global<kApplyNT>(reinterpret_cast<u32x2 *>(p), u32x2{bf16_narrow2(f[0], f[1]), bf16_narrow2(f[2], f[3])});
    }
    __device__ static void one(uint16_t *p, float v) { *p = (uint16_t)bf16_narrow(v); }
};

template <bool IS_DELTA>
__device__ __forceinline__ float term(float wp, float c, float eps)
{
    const float d = IS_DELTA ? c : c - wp;
    const float den = fmaxf(fabsf(wp), eps);
    const float q = fabsf(d) / den;            // IEEE fp32 division
    return d == 0.0f ? 0.0f : q;               // an unchanged weight contributes nothing
}

// fixed-order sum over the workgroup; valid in thread 0
__device__ __forceinline__ double block_sum(double v, double *lds)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) lds[wave] = v;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += lds[w];
    return s;
}

// APPLY (with IS_DELTA): the chunk of W^{t-1} is overwritten with W^{t-1} + delta after its terms are taken,
// so the score needs no copy of the previous weights and the update costs no pass of its own.
#ifndef SLIMFIT_DELTA_APPLY_THREADS
#define SLIMFIT_DELTA_APPLY_THREADS 1024      // 4 vectors of each tensor per thread: 0.62 ms against 0.67 ms with 256 threads x 16
#endif
constexpr int kApplyThreads = SLIMFIT_DELTA_APPLY_THREADS;
template <typename TP, typename TC, bool IS_DELTA, bool APPLY = false>
__global__ __launch_bounds__(APPLY ? kApplyThreads : kThreads) void layer_delta_partials_kernel(const char *__restrict__ ws, int32_t L,
                                                                        int64_t total_chunks, float eps,
                                                                        double *__restrict__ partials)
{
    constexpr int THREADS = APPLY ? kApplyThreads : kThreads;
    constexpr int kVecs = kChunk / 4 / THREADS;              // 16-byte vectors a thread holds of each tensor
    __shared__ double lds[THREADS / kWave];
    const Header *h = reinterpret_cast<const Header *>(ws);
    constexpr int32_t kPrevDt = sizeof(TP) == 2 ? SLIMFIT_BF16 : SLIMFIT_F32;
    constexpr int32_t kCurDt = sizeof(TC) == 2 ? SLIMFIT_BF16 : SLIMFIT_F32;
    if (h->magic != kMagic || h->n_layers != L || h->total_chunks != total_chunks || h->prev_dt != kPrevDt ||
        h->cur_dt != kCurDt)
        return;                                                          // no matching plan: touch nothing
    const LayerEntry *table = reinterpret_cast<const LayerEntry *>(ws + sizeof(Header));
    const int64_t chunk = blockIdx.x;

    // layer owning this chunk: the last entry whose first_chunk <= chunk
    int lo = 0, hi = L - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (table[mid].first_chunk <= chunk) lo = mid; else hi = mid - 1;
    }
    const LayerEntry e = table[lo];
    const int64_t off = (chunk - e.first_chunk) * kChunk;
    const int64_t len = min((int64_t)kChunk, e.numel - off);        // >= 1 by construction
    const TP *wp = static_cast<const TP *>(e.w_prev) + off;
    const TC *wc = static_cast<const TC *>(e.w_cur) + off;

    double acc = 0.0;
    if (len == kChunk) {
        // APPLY: the chunk goes in kApplySplit parts, and each part's new weights leave before its
        // terms (a division and an fp64 addition each) are worked out
        constexpr int kParts = APPLY ? kApplySplit : 1;
        constexpr int kPer = kVecs / kParts;
#pragma unroll
        for (int part = 0; part < kParts; ++part) {
            float p[kPer][4], c[kPer][4];
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                const int v = ((part * kPer + i) * THREADS + threadIdx.x) * 4;
                Load4<TP>::vec(wp + v, p[i]);
                Load4<TC>::vec(wc + v, c[i]);
            }
            if (APPLY) {
                TP *wn = const_cast<TP *>(wp);
#pragma unroll
                for (int i = 0; i < kPer; ++i) {
                    const int v = ((part * kPer + i) * THREADS + threadIdx.x) * 4;
                    float n4[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) n4[j] = p[i][j] + c[i][j];
                    Store4<TP>::vec(wn + v, n4);
                }
            }
#pragma unroll
            for (int i = 0; i < kPer; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc += (double)term<IS_DELTA>(p[i][j], c[i][j], eps);
        }
    } else {
        for (int64_t j = threadIdx.x; j < len; j += THREADS) {
            const float a = Load4<TP>::one(wp + j), b = Load4<TC>::one(wc + j);
            acc += (double)term<IS_DELTA>(a, b, eps);
            if (APPLY) Store4<TP>::one(const_cast<TP *>(wp) + j, a + b);
        }
    }
    const double s = block_sum(acc, lds);
    if (threadIdx.x == 0) partials[chunk] = s;
}

__global__ __launch_bounds__(kWave) void layer_delta_finish_kernel(const char *__restrict__ ws, int32_t L,
                                                                   int64_t total_chunks, int32_t prev_dt,
                                                                   int32_t cur_dt,
                                                                   const double *__restrict__ partials,
                                                                   float *__restrict__ d_out)
{
    const int layer = blockIdx.x;
    const Header *h = reinterpret_cast<const Header *>(ws);
    if (h->magic != kMagic || h->n_layers != L || h->total_chunks != total_chunks || h->prev_dt != prev_dt ||
        h->cur_dt != cur_dt) {
        if (threadIdx.x == 0) d_out[layer] = __builtin_nanf("");
        return;
    }
    const LayerEntry *table = reinterpret_cast<const LayerEntry *>(ws + sizeof(Header));
    const LayerEntry e = table[layer];
    const int64_t n_chunks = (e.numel + kChunk - 1) / kChunk;
    double acc = 0.0;
    for (int64_t c = threadIdx.x; c < n_chunks; c += kWave) acc += partials[e.first_chunk + c];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);
    if (threadIdx.x == 0) d_out[layer] = e.numel > 0 ? (float)(acc / (double)e.numel) : 0.0f;
}

struct Layout {
    int64_t total_chunks = 0;
    size_t bytes = 0;
};

int32_t layout_of(int32_t L, const int64_t *numel, Layout *out)
{
    if (L < 0) return SLIMFIT_ERR_INVALID_ARG;
    if (L > 0 && !numel) return SLIMFIT_ERR_INVALID_ARG;
    int64_t chunks = 0;
    for (int32_t i = 0; i < L; ++i) {
        if (numel[i] < 0) return SLIMFIT_ERR_INVALID_ARG;
        if (numel[i] > ((int64_t)1 << 40)) return SLIMFIT_ERR_UNSUPPORTED;
        chunks += (numel[i] + kChunk - 1) / kChunk;
    }
    if (chunks > 0x7FFFFFFF) return SLIMFIT_ERR_UNSUPPORTED;       // one chunk per workgroup
    out->total_chunks = chunks;
    out->bytes = table_bytes(L) + sizeof(double) * (size_t)chunks;
    return SLIMFIT_OK;
}

// own_scratch: the workspace is the library's own device array (no allocation to look up)
int32_t check_workspace(const Layout &lay, const void *ws, size_t ws_bytes, bool own_scratch = false)
{
    if (!ws || ws_bytes < lay.bytes) return SLIMFIT_ERR_WORKSPACE;
    if (!aligned_to(ws, 256)) return SLIMFIT_ERR_ALIGNMENT;
    return own_scratch ? SLIMFIT_OK : check_device_range(ws, lay.bytes);
}

// ---- the workspace of slimfit_layer_delta_static ---------------------------------------------------------
// A fixed device array, one copy per GPU the library's code is loaded on, alive until the process ends.  Its
// name is a host-side handle, not a device address: the address on the current device is looked up once per
// device with hipGetSymbolAddress and kept; kernels and checks only ever see that address.
constexpr size_t kStaticScratchBytes = SLIMFIT_LAYER_DELTA_STATIC_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];            // guarded by g_scratch_mutex

int32_t static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return SLIMFIT_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return SLIMFIT_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return SLIMFIT_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SLIMFIT_OK;
}

template <typename TP, typename TC>
void launch_partials(bool is_delta, bool apply, unsigned grid, hipStream_t st, const char *ws, int32_t L, int64_t chunks,
                     float eps, double *partials)
{
    if (apply)
        layer_delta_partials_kernel<TP, TC, true, true><<<grid, kApplyThreads, 0, st>>>(ws, L, chunks, eps, partials);
    else if (is_delta)
        layer_delta_partials_kernel<TP, TC, true><<<grid, kThreads, 0, st>>>(ws, L, chunks, eps, partials);
    else
        layer_delta_partials_kernel<TP, TC, false><<<grid, kThreads, 0, st>>>(ws, L, chunks, eps, partials);
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

extern "C" int32_t slimfit_layer_delta_workspace(int32_t L, const int64_t *numel, size_t *bytes)
{
    if (!bytes) return SLIMFIT_ERR_INVALID_ARG;
    Layout lay;
    int32_t rc = layout_of(L, numel, &lay);
    if (rc != SLIMFIT_OK) return rc;
    *bytes = lay.bytes;
    return SLIMFIT_OK;
}

static int32_t plan_entry(const void *const *w_prev, int32_t prev_dt, const void *const *w_cur, int32_t cur_dt,
                          const int64_t *numel, int32_t L, void *workspace, size_t workspace_bytes, void *stream,
                          bool own_scratch)
{
    if (!dtype_ok(prev_dt) || !dtype_ok(cur_dt)) return SLIMFIT_ERR_INVALID_ARG;
    Layout lay;
    int32_t rc = layout_of(L, numel, &lay);
    if (rc != SLIMFIT_OK) return rc;
    if (L == 0) return SLIMFIT_OK;
    if (!w_prev || !w_cur) return SLIMFIT_ERR_INVALID_ARG;
    for (int32_t i = 0; i < L; ++i) {
        if (numel[i] == 0) continue;
        if (!w_prev[i] || !w_cur[i]) return SLIMFIT_ERR_INVALID_ARG;
        if (!aligned_to(w_prev[i], 16) || !aligned_to(w_cur[i], 16)) return SLIMFIT_ERR_ALIGNMENT;
    }
    if ((rc = check_workspace(lay, workspace, workspace_bytes, own_scratch)) != SLIMFIT_OK) return rc;
    for (int32_t i = 0; i < L; ++i) {
        if ((rc = check_device_range(w_prev[i], (size_t)numel[i] * dtype_size(prev_dt))) != SLIMFIT_OK) return rc;
        if ((rc = check_device_range(w_cur[i], (size_t)numel[i] * dtype_size(cur_dt))) != SLIMFIT_OK) return rc;
    }

    hipStream_t st = static_cast<hipStream_t>(stream);
    Header h = {};
    h.magic = kMagic;
    h.n_layers = L;
    h.total_chunks = lay.total_chunks;
    h.prev_dt = prev_dt;
    h.cur_dt = cur_dt;
    int64_t next_chunk = 0;
    for (int32_t first = 0; first < L; first += kPlanBatch) {
        PlanBatch batch = {};
        const int count = (L - first < kPlanBatch) ? (L - first) : kPlanBatch;
        for (int t = 0; t < count; ++t) {
            const int32_t i = first + t;
            batch.e[t].w_prev = w_prev[i];
            batch.e[t].w_cur = w_cur[i];
            batch.e[t].numel = numel[i];
            batch.e[t].first_chunk = next_chunk;
            next_chunk += (numel[i] + kChunk - 1) / kChunk;
        }
        plan_write_kernel<<<1, kWave, 0, st>>>(static_cast<char *>(workspace), h, first, count, batch);
    }
    return launch_status();
}

extern "C" int32_t slimfit_layer_delta_plan(const void *const *w_prev, int32_t prev_dt, const void *const *w_cur,
                                            int32_t cur_dt, const int64_t *numel, int32_t L, void *workspace,
                                            size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    return plan_entry(w_prev, prev_dt, w_cur, cur_dt, numel, L, workspace, workspace_bytes, stream, false);
}

static int32_t run_entry(const int64_t *numel, int32_t L, int32_t prev_dt, int32_t cur_dt, int32_t cur_is_delta, bool apply,
                         float eps, float *d_out, void *workspace, size_t workspace_bytes, void *stream,
                         bool own_scratch = false)
{
    if (!dtype_ok(prev_dt) || !dtype_ok(cur_dt) || !(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    Layout lay;
    int32_t rc = layout_of(L, numel, &lay);
    if (rc != SLIMFIT_OK) return rc;
    if (L == 0) return SLIMFIT_OK;
    if (!d_out) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(d_out, 4)) return SLIMFIT_ERR_ALIGNMENT;
    if ((rc = check_workspace(lay, workspace, workspace_bytes, own_scratch)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(d_out, sizeof(float) * (size_t)L)) != SLIMFIT_OK) return rc;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const char *ws = static_cast<const char *>(workspace);
    double *partials = reinterpret_cast<double *>(static_cast<char *>(workspace) + table_bytes(L));
    const unsigned grid = (unsigned)lay.total_chunks;
    const bool is_delta = cur_is_delta != 0;
    if (grid > 0) {
        if (prev_dt == SLIMFIT_F32 && cur_dt == SLIMFIT_F32)
            launch_partials<float, float>(is_delta, apply, grid, st, ws, L, lay.total_chunks, eps, partials);
        else if (prev_dt == SLIMFIT_BF16 && cur_dt == SLIMFIT_F32)
            launch_partials<uint16_t, float>(is_delta, apply, grid, st, ws, L, lay.total_chunks, eps, partials);
        else if (prev_dt == SLIMFIT_F32 && cur_dt == SLIMFIT_BF16)
            launch_partials<float, uint16_t>(is_delta, apply, grid, st, ws, L, lay.total_chunks, eps, partials);
        else
            launch_partials<uint16_t, uint16_t>(is_delta, apply, grid, st, ws, L, lay.total_chunks, eps, partials);
    }
    layer_delta_finish_kernel<<<(unsigned)L, kWave, 0, st>>>(ws, L, lay.total_chunks, prev_dt, cur_dt, partials, d_out);
    return launch_status();
}

extern "C" int32_t slimfit_layer_delta_run(const int64_t *numel, int32_t L, int32_t prev_dt, int32_t cur_dt,
                                           int32_t cur_is_delta, float eps, float *d_out, void *workspace,
                                           size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    return run_entry(numel, L, prev_dt, cur_dt, cur_is_delta, false, eps, d_out, workspace, workspace_bytes, stream);
}

extern "C" int32_t slimfit_layer_delta_apply_run(const int64_t *numel, int32_t L, int32_t w_dt, int32_t delta_dt, float eps,
                                                 float *d_out, void *workspace, size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    return run_entry(numel, L, w_dt, delta_dt, 1, true, eps, d_out, workspace, workspace_bytes, stream);
}

extern "C" int32_t slimfit_layer_delta(const void *const *w_prev, int32_t prev_dt, const void *const *w_cur,
                                       int32_t cur_dt, int32_t cur_is_delta, const int64_t *numel, int32_t L,
                                       float eps, float *d_out, void *workspace, size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    // validate the run-only arguments first so that nothing is enqueued on error
    if (!(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    if (L > 0 && !d_out) return SLIMFIT_ERR_INVALID_ARG;
    if (L > 0 && !aligned_to(d_out, 4)) return SLIMFIT_ERR_ALIGNMENT;
    if (L > 0 && check_device_range(d_out, sizeof(float) * (size_t)L) != SLIMFIT_OK) return SLIMFIT_ERR_POINTER;
    int32_t rc = slimfit_layer_delta_plan(w_prev, prev_dt, w_cur, cur_dt, numel, L, workspace, workspace_bytes, stream);
    if (rc != SLIMFIT_OK) return rc;
    return slimfit_layer_delta_run(numel, L, prev_dt, cur_dt, cur_is_delta, eps, d_out, workspace, workspace_bytes,
                                   stream);
}

extern "C" int32_t slimfit_layer_delta_static(const void *const *w_prev, int32_t prev_dt, const void *const *w_cur,
                                              int32_t cur_dt, int32_t cur_is_delta, const int64_t *numel, int32_t L,
                                              float eps, float *d_out, void *stream)
{
    StreamScope capture_aware(stream);
    if (!(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    if (L > 0 && !d_out) return SLIMFIT_ERR_INVALID_ARG;
    if (L > 0 && !aligned_to(d_out, 4)) return SLIMFIT_ERR_ALIGNMENT;
    Layout lay;
    int32_t rc = layout_of(L, numel, &lay);
    if (rc != SLIMFIT_OK) return rc;
    if (lay.bytes > kStaticScratchBytes) return SLIMFIT_ERR_WORKSPACE;     // beyond the fixed array: use slimfit_layer_delta
    if (L == 0) return SLIMFIT_OK;
    if (check_device_range(d_out, sizeof(float) * (size_t)L) != SLIMFIT_OK) return SLIMFIT_ERR_POINTER;
    void *ws = nullptr;
    if ((rc = static_scratch(&ws)) != SLIMFIT_OK) return rc;
    // the table and every partial the finishing kernel reads are rewritten by this call: nothing has to be cleared
    rc = plan_entry(w_prev, prev_dt, w_cur, cur_dt, numel, L, ws, kStaticScratchBytes, stream, true);
    if (rc != SLIMFIT_OK) return rc;
    return run_entry(numel, L, prev_dt, cur_dt, cur_is_delta, false, eps, d_out, ws, kStaticScratchBytes, stream, true);
}

extern "C" int32_t slimfit_apply_update_layer_delta(void *const *w, int32_t w_dt, const void *const *delta,
                                                    int32_t delta_dt, const int64_t *numel, int32_t L, float eps,
                                                    float *d_out, void *workspace, size_t workspace_bytes, void *stream)
{
    StreamScope capture_aware(stream);
    if (!(eps >= 0.0f)) return SLIMFIT_ERR_INVALID_ARG;
    if (L > 0 && !d_out) return SLIMFIT_ERR_INVALID_ARG;
    if (L > 0 && !aligned_to(d_out, 4)) return SLIMFIT_ERR_ALIGNMENT;
    if (L > 0 && w && delta && numel)
        for (int32_t i = 0; i < L; ++i)
            if (numel[i] > 0 && w[i] == delta[i]) return SLIMFIT_ERR_INVALID_ARG;      // the update must not alias the weights
    if (L > 0 && check_device_range(d_out, sizeof(float) * (size_t)L) != SLIMFIT_OK) return SLIMFIT_ERR_POINTER;
    int32_t rc = slimfit_layer_delta_plan(w, w_dt, delta, delta_dt, numel, L, workspace, workspace_bytes, stream);
    if (rc != SLIMFIT_OK) return rc;
    return slimfit_layer_delta_apply_run(numel, L, w_dt, delta_dt, eps, d_out, workspace, workspace_bytes, stream);
}
