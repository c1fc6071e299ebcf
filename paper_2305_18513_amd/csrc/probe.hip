// A plain streaming kernel with a chosen read : write ratio -- the yardstick for "what could a perfect
// kernel of this traffic mix reach on this GPU".  Every thread reads RATIO 16-byte vectors with
// non-temporal loads (consecutive lanes, consecutive vectors: each load of a wave is one contiguous
// 1 KiB run), adds them and writes one vector with a non-temporal store.  Nothing of the method is
// computed here.
#include "common.hpp"

namespace slimfit {
namespace {

constexpr int kThreads = 256;

template <int RATIO>
__global__ __launch_bounds__(kThreads) void stream_probe_kernel(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst,
                                                                int64_t out_vecs)
{
    const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (o >= out_vecs) return;
    const f32x4 *in = src + (int64_t)blockIdx.x * kThreads * RATIO + threadIdx.x;
    f32x4 v[RATIO];
#pragma unroll
    for (int r = 0; r < RATIO; ++r) v[r] = __builtin_nontemporal_load(in + r * kThreads);
    f32x4 s = v[0];
#pragma unroll
    for (int r = 1; r < RATIO; ++r) s += v[r];
    __builtin_nontemporal_store(s, dst + o);
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

extern "C" int32_t slimfit_stream_probe(const void *src, void *dst, int64_t out_vecs, int32_t ratio, void *stream)
{
    if (out_vecs < 0 || ratio < 1 || ratio > 16) return SLIMFIT_ERR_INVALID_ARG;
    if (out_vecs == 0) return SLIMFIT_OK;
    if (!src || !dst || src == dst) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(src, 16) || !aligned_to(dst, 16)) return SLIMFIT_ERR_ALIGNMENT;
    const int64_t blocks = (out_vecs + kThreads - 1) / kThreads;
    if (blocks > 0x7FFFFFFF) return SLIMFIT_ERR_UNSUPPORTED;
    int32_t rc;
    // the last workgroup's threads past out_vecs return before loading, so the source needs blocks' worth only
    // up to the last live thread; ask for whole workgroups to keep the rule simple
    if ((rc = check_device_range(src, (size_t)blocks * kThreads * (size_t)ratio * 16)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dst, (size_t)out_vecs * 16)) != SLIMFIT_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const f32x4 *s = static_cast<const f32x4 *>(src);
    f32x4 *d = static_cast<f32x4 *>(dst);
    const unsigned grid = (unsigned)blocks;
    switch (ratio) {
#define SLIMFIT_PROBE_CASE(R) case R: stream_probe_kernel<R><<<grid, kThreads, 0, st>>>(s, d, out_vecs); break;
        SLIMFIT_PROBE_CASE(1) SLIMFIT_PROBE_CASE(2) SLIMFIT_PROBE_CASE(3) SLIMFIT_PROBE_CASE(4)
        SLIMFIT_PROBE_CASE(5) SLIMFIT_PROBE_CASE(6) SLIMFIT_PROBE_CASE(7) SLIMFIT_PROBE_CASE(8)
        SLIMFIT_PROBE_CASE(9) SLIMFIT_PROBE_CASE(10) SLIMFIT_PROBE_CASE(11) SLIMFIT_PROBE_CASE(12)
        SLIMFIT_PROBE_CASE(13) SLIMFIT_PROBE_CASE(14) SLIMFIT_PROBE_CASE(15) SLIMFIT_PROBE_CASE(16)
#undef SLIMFIT_PROBE_CASE
    }
    return launch_status();
}
