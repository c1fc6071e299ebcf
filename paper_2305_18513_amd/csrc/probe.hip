// A plain streaming kernel with a chosen read : write ratio -- the yardstick for "what could a perfect
// kernel of this traffic mix reach on this GPU".  Every thread keeps four 16-byte non-temporal loads in
// flight (consecutive lanes, consecutive vectors: each load of a wave is one contiguous 1 KiB run) and
// writes, for each vector it read, 16 / ratio bytes made from it, side by side with its neighbours' --
// the shape of a quantiser or a pruner (many short stores next to one another).  One long store per
// `ratio` loads, the other way to the same mix, measured 4-5 % slower and is not kept.  Nothing of the
// method is computed here.
#include "common.hpp"

namespace slimfit {
namespace {

constexpr int kThreads = 256;
constexpr int kVecs = 4;                   // loads a thread has in flight
typedef float f32x2 __attribute__((ext_vector_type(2)));

// what is written for one source vector v = (x, y, z, w), s = ((x + y) + z) + w in fp32
template <int RATIO> struct Out;
template <> struct Out<1> {                // the vector itself
    using type = f32x4;
    __device__ static type make(const f32x4 &v) { return v; }
};
template <> struct Out<2> {                // (x + y, z + w)
    using type = f32x2;
    __device__ static type make(const f32x4 &v) { return f32x2{v.x + v.y, v.z + v.w}; }
};
template <> struct Out<4> {                // s
    using type = float;
    __device__ static type make(const f32x4 &v) { return ((v.x + v.y) + v.z) + v.w; }
};
template <> struct Out<8> {                // the upper 16 bits of s
    using type = uint16_t;
    __device__ static type make(const f32x4 &v) { return (uint16_t)(__builtin_bit_cast(uint32_t, Out<4>::make(v)) >> 16); }
};
template <> struct Out<16> {               // the upper 8 bits of s
    using type = uint8_t;
    __device__ static type make(const f32x4 &v) { return (uint8_t)(__builtin_bit_cast(uint32_t, Out<4>::make(v)) >> 24); }
};

template <int RATIO>
__global__ __launch_bounds__(kThreads) void stream_probe_kernel(const f32x4 *__restrict__ src,
                                                                typename Out<RATIO>::type *__restrict__ dst, int64_t in_vecs)
{
    const int64_t first = (int64_t)blockIdx.x * (kThreads * kVecs);
    const int64_t base = first + threadIdx.x;
    if (first + kThreads * kVecs <= in_vecs) {             // workgroup-uniform: no test around any load
        f32x4 v[kVecs];
#pragma unroll
        for (int j = 0; j < kVecs; ++j) v[j] = __builtin_nontemporal_load(src + base + j * kThreads);
#pragma unroll
        for (int j = 0; j < kVecs; ++j) __builtin_nontemporal_store(Out<RATIO>::make(v[j]), dst + base + j * kThreads);
    } else {
        for (int j = 0; j < kVecs; ++j) {
            const int64_t i = base + j * kThreads;
            if (i < in_vecs) dst[i] = Out<RATIO>::make(src[i]);
        }
    }
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

extern "C" int32_t slimfit_stream_probe(const void *src, void *dst, int64_t in_vecs, int32_t ratio, void *stream)
{
    StreamScope capture_aware(stream);
    if (in_vecs < 0 || (ratio != 1 && ratio != 2 && ratio != 4 && ratio != 8 && ratio != 16)) return SLIMFIT_ERR_INVALID_ARG;
    if (in_vecs == 0) return SLIMFIT_OK;
    if (!src || !dst || src == dst) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(src, 16) || !aligned_to(dst, 16)) return SLIMFIT_ERR_ALIGNMENT;
    const int64_t per_block = (int64_t)kThreads * kVecs;
    const int64_t blocks = (in_vecs + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFF) return SLIMFIT_ERR_UNSUPPORTED;
    int32_t rc;
    if ((rc = check_device_range(src, (size_t)in_vecs * 16)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dst, (size_t)in_vecs * (16 / (size_t)ratio))) != SLIMFIT_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const f32x4 *s = static_cast<const f32x4 *>(src);
    const unsigned grid = (unsigned)blocks;
    switch (ratio) {
#define SLIMFIT_PROBE_CASE(R)                                                                                    \
    case R:                                                                                                      \
        stream_probe_kernel<R><<<grid, kThreads, 0, st>>>(s, static_cast<Out<R>::type *>(dst), in_vecs);         \
        break;
        SLIMFIT_PROBE_CASE(1) SLIMFIT_PROBE_CASE(2) SLIMFIT_PROBE_CASE(4) SLIMFIT_PROBE_CASE(8) SLIMFIT_PROBE_CASE(16)
#undef SLIMFIT_PROBE_CASE
    }
    return launch_status();
}
