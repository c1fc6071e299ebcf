// A plain streaming kernel with a chosen read : write ratio -- the yardstick for "what could a perfect
// kernel of this traffic mix reach on this GPU".  Every thread keeps four 16-byte non-temporal loads in
// flight (consecutive lanes, consecutive vectors: each load of a wave is one contiguous 1 KiB run) and
// writes, for each vector it read, 16 / ratio bytes made from it, side by side with its neighbours' --
// the shape of a quantiser or a pruner (many short stores next to one another).  One long store per
// `ratio` loads, the other way to the same mix, measured 4-5 % slower and is not kept.  Two more shapes:
// ratio 0 only reads (one float per wavefront is written: a scoring pass), and ratio -2, -4, -8 write that
// many 16-byte vectors per vector read (a dequantiser: few bytes in, many out; one thread per output vector).
// Nothing of the method is computed here.
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

// ratio 0: the sum of a wavefront's 4 * 64 vectors' components, lanes added in a fixed butterfly order
__global__ __launch_bounds__(kThreads) void stream_probe_read_kernel(const f32x4 *__restrict__ src, float *__restrict__ dst,
                                                                     int64_t in_vecs)
{
    const int64_t first = (int64_t)blockIdx.x * (kThreads * kVecs);
    const int64_t base = first + threadIdx.x;
    float s = 0.0f;
    if (first + kThreads * kVecs <= in_vecs) {
        f32x4 v[kVecs];
#pragma unroll
        for (int j = 0; j < kVecs; ++j) v[j] = __builtin_nontemporal_load(src + base + j * kThreads);
#pragma unroll
        for (int j = 0; j < kVecs; ++j) s += Out<4>::make(v[j]);
    } else {
        for (int j = 0; j < kVecs; ++j) {
            const int64_t i = base + j * kThreads;
            if (i < in_vecs) s += Out<4>::make(src[i]);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) dst[(int64_t)blockIdx.x * (kThreads / kWave) + (threadIdx.x >> 6)] = s;
}

// ratio -M: one thread per OUTPUT vector, the way a dequantiser is laid out: it reads the 16 / M source bytes that
// stand behind its vector (2 bytes at M = 8: a wavefront's loads are one contiguous 128-byte run) and stores 16.
// Output vector o = s + (0, 1, 2, 3), s the sum of the 16-bit words of source piece o as a float (exact).
#ifndef SLIMFIT_PROBE_GROW_THREADS
#define SLIMFIT_PROBE_GROW_THREADS 512
#endif
constexpr int kGrowThreads = SLIMFIT_PROBE_GROW_THREADS;
constexpr int kGrowVecs = 2;               // output vectors a thread produces
template <int M> struct Piece;
template <> struct Piece<8> {
    using type = uint16_t;
    __device__ static float sum(type p) { return (float)p; }
};
template <> struct Piece<4> {
    using type = uint32_t;
    __device__ static float sum(type p) { return (float)((p & 0xFFFFu) + (p >> 16)); }
};
template <> struct Piece<2> {
    using type = u32x2;
    __device__ static float sum(type p) { return (float)((p.x & 0xFFFFu) + (p.x >> 16) + (p.y & 0xFFFFu) + (p.y >> 16)); }
};
template <int M>
__global__ __launch_bounds__(kGrowThreads) void stream_probe_write_kernel(const typename Piece<M>::type *__restrict__ src,
                                                                          f32x4 *__restrict__ dst, int64_t out_vecs)
{
    const int64_t first = (int64_t)blockIdx.x * (kGrowThreads * kGrowVecs);
    if (first + kGrowThreads * kGrowVecs <= out_vecs) {    // workgroup-uniform: no test around any load
        typename Piece<M>::type p[kGrowVecs];
#pragma unroll
        for (int u = 0; u < kGrowVecs; ++u) p[u] = __builtin_nontemporal_load(src + first + u * kGrowThreads + threadIdx.x);
#pragma unroll
        for (int u = 0; u < kGrowVecs; ++u) {
            const float s = Piece<M>::sum(p[u]);
            __builtin_nontemporal_store(f32x4{s, s + 1.0f, s + 2.0f, s + 3.0f}, dst + first + u * kGrowThreads + threadIdx.x);
        }
    } else {
        for (int u = 0; u < kGrowVecs; ++u) {
            const int64_t o = first + u * kGrowThreads + threadIdx.x;
            if (o < out_vecs) {
                const float s = Piece<M>::sum(src[o]);
                dst[o] = f32x4{s, s + 1.0f, s + 2.0f, s + 3.0f};
            }
        }
    }
}

}  // namespace
}  // namespace slimfit

using namespace slimfit;

extern "C" int32_t slimfit_stream_probe(const void *src, void *dst, int64_t in_vecs, int32_t ratio, void *stream)
{
    StreamScope capture_aware(stream);
    const bool shrink = ratio == 1 || ratio == 2 || ratio == 4 || ratio == 8 || ratio == 16;
    const bool grow = ratio == -2 || ratio == -4 || ratio == -8;
    if (in_vecs < 0 || !(shrink || grow || ratio == 0)) return SLIMFIT_ERR_INVALID_ARG;
    if (in_vecs == 0) return SLIMFIT_OK;
    if (!src || !dst || src == dst) return SLIMFIT_ERR_INVALID_ARG;
    if (!aligned_to(src, 16) || !aligned_to(dst, 16)) return SLIMFIT_ERR_ALIGNMENT;
    const int64_t per_block = grow ? (int64_t)kGrowThreads * kGrowVecs : (int64_t)kThreads * kVecs;
    const int64_t work = grow ? in_vecs * (int64_t)(-ratio) : in_vecs;      // output vectors / source vectors
    const int64_t blocks = (work + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFF) return SLIMFIT_ERR_UNSUPPORTED;
    // bytes written: shrink 16 / ratio per vector; read-only one float per wavefront; grow whole workgroup tiles
    const size_t dst_bytes = shrink ? (size_t)in_vecs * (16 / (size_t)ratio)
                             : grow ? (size_t)in_vecs * (size_t)(-ratio) * 16
                                    : (size_t)blocks * (kThreads / kWave) * 4;
    int32_t rc;
    if ((rc = check_device_range(src, (size_t)in_vecs * 16)) != SLIMFIT_OK) return rc;
    if ((rc = check_device_range(dst, dst_bytes)) != SLIMFIT_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const f32x4 *s = static_cast<const f32x4 *>(src);
    const unsigned grid = (unsigned)blocks;
    switch (ratio) {
    case 0: stream_probe_read_kernel<<<grid, kThreads, 0, st>>>(s, static_cast<float *>(dst), in_vecs); break;
    case -2: stream_probe_write_kernel<2><<<grid, kGrowThreads, 0, st>>>(static_cast<const u32x2 *>(src), static_cast<f32x4 *>(dst), work); break;
    case -4: stream_probe_write_kernel<4><<<grid, kGrowThreads, 0, st>>>(static_cast<const uint32_t *>(src), static_cast<f32x4 *>(dst), work); break;
    case -8: stream_probe_write_kernel<8><<<grid, kGrowThreads, 0, st>>>(static_cast<const uint16_t *>(src), static_cast<f32x4 *>(dst), work); break;
#define SLIMFIT_PROBE_CASE(R)                                                                                    \
    case R:                                                                                                      \
        stream_probe_kernel<R><<<grid, kThreads, 0, st>>>(s, static_cast<Out<R>::type *>(dst), in_vecs);         \
        break;
        SLIMFIT_PROBE_CASE(1) SLIMFIT_PROBE_CASE(2) SLIMFIT_PROBE_CASE(4) SLIMFIT_PROBE_CASE(8) SLIMFIT_PROBE_CASE(16)
#undef SLIMFIT_PROBE_CASE
    }
    return launch_status();
}
