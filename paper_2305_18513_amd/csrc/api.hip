// Host side of the C ABI: status text, pointer checks and the inter-layer
// scheduling routines (Alg. 1; Sec. 3.2), which run on the host because the
// distance vector has one entry per layer (about a hundred).
#include "common.hpp"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <numeric>
#include <vector>

namespace slimfit {

static std::atomic<int32_t> g_pointer_checks{1};
static thread_local bool t_capturing = false;      // the entry point running on this thread launches into a capture

StreamScope::StreamScope(void *stream) : prev_(t_capturing)
{
    if (!g_pointer_checks.load(std::memory_order_relaxed)) return;
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &status) != hipSuccess) {
        (void)hipGetLastError();                 // e.g. the legacy stream while another stream captures: not ours to judge
        status = hipStreamCaptureStatusNone;
    }
    t_capturing = prev_ || status == hipStreamCaptureStatusActive;
}

StreamScope::~StreamScope() { t_capturing = prev_; }

int32_t launch_status()
{
    return hipGetLastError() == hipSuccess ? SLIMFIT_OK : SLIMFIT_ERR_HIP;
}

int32_t check_device_range(const void *p, size_t bytes)
{
    if (!g_pointer_checks.load(std::memory_order_relaxed) || t_capturing || bytes == 0) return SLIMFIT_OK;
    if (!p) return SLIMFIT_ERR_INVALID_ARG;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();                 // clear the sticky error of a failed lookup
        return SLIMFIT_ERR_POINTER;
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) return SLIMFIT_ERR_POINTER;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) != hipSuccess) {
        (void)hipGetLastError();
        return SLIMFIT_ERR_POINTER;
    }
    const char *lo = static_cast<const char *>(base);
    const char *q = static_cast<const char *>(p);
    if (q < lo || bytes > size || (size_t)(q - lo) > size - bytes) return SLIMFIT_ERR_POINTER;
    return SLIMFIT_OK;
}

}  // namespace slimfit

using namespace slimfit;

extern "C" const char *slimfit_status_string(int32_t status)
{
    switch (status) {
    case SLIMFIT_OK: return "ok";
    case SLIMFIT_ERR_INVALID_ARG: return "invalid argument";
    case SLIMFIT_ERR_UNSUPPORTED: return "unsupported value";
    case SLIMFIT_ERR_ALIGNMENT: return "misaligned pointer";
    case SLIMFIT_ERR_WORKSPACE: return "workspace missing or too small";
    case SLIMFIT_ERR_HIP: return "HIP runtime error";
    case SLIMFIT_ERR_POINTER: return "not device memory, or buffer too small for the call";
    default: return "unknown status";
    }
}

extern "C" int32_t slimfit_version(void) { return 100; }   // 0.1.0

extern "C" int32_t slimfit_set_pointer_checks(int32_t on)
{
    return g_pointer_checks.exchange(on ? 1 : 0);
}

extern "C" int32_t slimfit_freeze_count(int32_t L, double F)
{
    if (L < 0 || !(F >= 0.0) || !(F <= 1.0)) return -1;
    const double prod = (double)L * F;            // the pseudo code's L*F in double
    return (int32_t)prod;                         // int(): truncation
}

extern "C" int32_t slimfit_ils_select(const float *d, int32_t L, int32_t n_freeze, int32_t *frozen_idx, uint8_t *mask)
{
    if (L < 0 || n_freeze < 0 || n_freeze > L) return SLIMFIT_ERR_INVALID_ARG;
    if ((L > 0 && !d) || (n_freeze > 0 && !frozen_idx)) return SLIMFIT_ERR_INVALID_ARG;
    if (mask) std::fill(mask, mask + L, (uint8_t)0);
    if (n_freeze == 0) return SLIMFIT_OK;
    std::vector<int32_t> order((size_t)L);
    std::iota(order.begin(), order.end(), 0);
    // ascending distance, ties by layer index, NaN after everything else
    auto before = [d](int32_t a, int32_t b) {
        const bool na = std::isnan(d[a]), nb = std::isnan(d[b]);
        if (na != nb) return nb;
        if (!na && d[a] != d[b]) return d[a] < d[b];
        return a < b;
    };
    std::partial_sort(order.begin(), order.begin() + n_freeze, order.end(), before);
    for (int32_t s = 0; s < n_freeze; ++s) {
        frozen_idx[s] = order[(size_t)s];
        if (mask) mask[order[(size_t)s]] = 1;
    }
    return SLIMFIT_OK;
}

extern "C" int32_t slimfit_ils_select_blocks(const float *d, int32_t L, int32_t group, int32_t n_freeze,
                                             int32_t *frozen_blocks, uint8_t *mask)
{
    if (L < 0 || group < 1 || n_freeze < 0) return SLIMFIT_ERR_INVALID_ARG;
    const int32_t nb = (int32_t)(((int64_t)L + group - 1) / group);
    if (n_freeze > nb || (L > 0 && !d) || (n_freeze > 0 && !frozen_blocks)) return SLIMFIT_ERR_INVALID_ARG;
    if (mask) std::fill(mask, mask + L, (uint8_t)0);
    if (n_freeze == 0) return SLIMFIT_OK;
    auto first_layer = [group](int32_t b) { return (int64_t)b * group; };
    auto end_layer = [group, L](int32_t b) { return std::min<int64_t>((int64_t)b * group + group, L); };
    std::vector<double> mean((size_t)nb);
    for (int32_t b = 0; b < nb; ++b) {
        double sum = 0.0;                                    // layer order, double
        for (int64_t i = first_layer(b); i < end_layer(b); ++i) sum += (double)d[i];
        mean[(size_t)b] = sum / (double)(end_layer(b) - first_layer(b));
    }
    std::vector<int32_t> order((size_t)nb);
    std::iota(order.begin(), order.end(), 0);
    auto before = [&mean](int32_t a, int32_t b) {
        const double ma = mean[(size_t)a], mb = mean[(size_t)b];
        const bool na = std::isnan(ma), nb_ = std::isnan(mb);
        if (na != nb_) return nb_;
        if (!na && ma != mb) return ma < mb;
        return a < b;
    };
    std::partial_sort(order.begin(), order.begin() + n_freeze, order.end(), before);
    for (int32_t s = 0; s < n_freeze; ++s) {
        const int32_t b = order[(size_t)s];
        frozen_blocks[s] = b;
        if (mask)
            for (int64_t i = first_layer(b); i < end_layer(b); ++i) mask[i] = 1;
    }
    return SLIMFIT_OK;
}

extern "C" int32_t slimfit_ils_update(float *d, const float *new_scores, const uint8_t *frozen_mask, int32_t L)
{
    if (L < 0) return SLIMFIT_ERR_INVALID_ARG;
    if (L == 0) return SLIMFIT_OK;
    if (!d || !new_scores || !frozen_mask) return SLIMFIT_ERR_INVALID_ARG;
    for (int32_t i = 0; i < L; ++i)
        if (!frozen_mask[i]) d[i] = new_scores[i];
    return SLIMFIT_OK;
}

// ---- the other two freezing schedules of the paper's ablation -------------------------
namespace {

// SplitMix64: the state advances by the 64-bit golden ratio, the output is the
// state passed through two xor-shift-multiply rounds and a final xor-shift.
inline uint64_t splitmix64(uint64_t &state)
{
    state += 0x9E3779B97F4A7C15ull;
    uint64_t z = state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

}  // namespace

extern "C" int32_t slimfit_schedule_random(int32_t L, int32_t n_freeze, uint64_t seed, uint64_t iteration,
                                           int32_t *frozen_idx, uint8_t *mask)
{
    if (L < 0 || n_freeze < 0 || n_freeze > L) return SLIMFIT_ERR_INVALID_ARG;
    if (n_freeze > 0 && !frozen_idx) return SLIMFIT_ERR_INVALID_ARG;
    if (mask) std::fill(mask, mask + L, (uint8_t)0);
    std::vector<int32_t> pool((size_t)L);
    std::iota(pool.begin(), pool.end(), 0);
    uint64_t state = seed ^ (iteration * 0xD6E8FEB86659FD93ull);
    for (int32_t i = 0; i < n_freeze; ++i) {                 // the first n_freeze steps of a Fisher-Yates shuffle
        const uint64_t span = (uint64_t)(L - i);
        const size_t j = (size_t)i + (size_t)(splitmix64(state) % span);
        std::swap(pool[(size_t)i], pool[j]);
        frozen_idx[i] = pool[(size_t)i];
        if (mask) mask[pool[(size_t)i]] = 1;
    }
    return SLIMFIT_OK;
}

extern "C" int32_t slimfit_schedule_progressive(int32_t L, int32_t n_freeze, int32_t *frozen_idx, uint8_t *mask)
{
    if (L < 0 || n_freeze < 0 || n_freeze > L) return SLIMFIT_ERR_INVALID_ARG;
    if (n_freeze > 0 && !frozen_idx) return SLIMFIT_ERR_INVALID_ARG;
    if (mask)
        for (int32_t i = 0; i < L; ++i) mask[i] = i < n_freeze ? 1 : 0;
    for (int32_t i = 0; i < n_freeze; ++i) frozen_idx[i] = i;
    return SLIMFIT_OK;
}
