// Measurement probes of libtstgemm: three kernels that do nothing but exercise a resource a gather-add kernel is bound
// by, so that a benchmark can put the rate the machine actually delivers next to the figure it prices against.
//   * k_probe_lds: every wavefront issues conflict-free ds_read_b128 instructions (64 lanes x 16 bytes, the gather of
//     the large-M kernel without anything around it), 2 workgroups of 16 wavefronts per compute unit as in that kernel;
//   * k_probe_stream: a grid-stride read of a buffer with 16-byte loads, the access pattern of the small-M kernel's
//     list walk without the gathers.
//   * k_probe_tile_copy: the tile exchange of the tiled kernels without the gathers between two exchanges -- every
//     workgroup (16 wavefronts, 2 per compute unit) copies 64 KiB pieces of a buffer into its LDS, 16-byte loads, a
//     barrier, 16-byte LDS writes, a barrier, again and again.
// None is part of the sparse ternary GEMM path; the caller times them (events on the stream).
#include "tstgemm_internal.h"

namespace tst {

// Written only under a condition that never holds, which keeps the loads of the probes alive; external linkage, or the
// compiler drops the store, and with it the whole stream kernel, as dead.
__device__ float g_probe_sink;

namespace {

typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 1024;
constexpr int kProbeReadsPerIter = 8;

__global__ void __launch_bounds__(kProbeThreads, 8) k_probe_lds(int iters)
{
    __shared__ __attribute__((aligned(16))) char lds[64 * 1024];
    for (int i = threadIdx.x; i < 16 * 1024; i += kProbeThreads) reinterpret_cast<float *>(lds)[i] = (float)i;
    __syncthreads();
    const int addr = (int)(uintptr_t)(__attribute__((address_space(3))) char *)lds + (threadIdx.x & 63) * 16;
    float sink = 0.f;
    for (int it = 0; it < iters; ++it) {
        float4v a, b, c, d, e, f, g, h;
        asm volatile("ds_read_b128 %0, %8 offset:0\n\tds_read_b128 %1, %8 offset:1024\n\t"
                     "ds_read_b128 %2, %8 offset:2048\n\tds_read_b128 %3, %8 offset:3072\n\t"
                     "ds_read_b128 %4, %8 offset:4096\n\tds_read_b128 %5, %8 offset:5120\n\t"
                     "ds_read_b128 %6, %8 offset:6144\n\tds_read_b128 %7, %8 offset:7168\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d), "=&v"(e), "=&v"(f), "=&v"(g), "=&v"(h)
                     : "v"(addr)
                     : "memory");
        sink += a.x + h.w;
    }
    if (sink == 12345.678f) g_probe_sink = sink;
}

__global__ void __launch_bounds__(256) k_probe_stream(const float4v *__restrict__ src, size_t pieces)
{
    float4v s = {0.f, 0.f, 0.f, 0.f};
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    // four independent loads per round, so that a lane has 64 bytes in flight
    for (; i + 3 * stride < pieces; i += 4 * stride) {
        const float4v a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        s += a + b + c + d;
    }
    for (; i < pieces; i += stride) s += src[i];
    if (s.x + s.y + s.z + s.w == 12345.678f) g_probe_sink = s.x;
}

// One workgroup: `iters` times { 64 KiB of src -> registers, barrier, registers -> LDS, barrier }, the exchange of
// k_large / k_small with nothing between two exchanges.  Workgroup w starts at tile w and steps through the n_tiles
// tiles of the buffer, so at any time the workgroups read different tiles, as the K slices of a call do.
__global__ void __launch_bounds__(kProbeThreads, 8) k_probe_tile_copy(const char *__restrict__ src, int n_tiles, int iters)
{
    constexpr int kTile = 64 * 1024, kPieces = kTile / (kProbeThreads * 16);
    __shared__ __attribute__((aligned(16))) char lds[kTile];
    const int piece = threadIdx.x * 16;
    int tile = blockIdx.x % n_tiles;
    for (int it = 0; it < iters; ++it) {
        float4v st[kPieces];
#pragma unroll
        for (int i = 0; i < kPieces; ++i)
            st[i] = *reinterpret_cast<const float4v *>(src + (size_t)tile * kTile + piece + i * kProbeThreads * 16);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kPieces; ++i) *reinterpret_cast<float4v *>(lds + piece + i * kProbeThreads * 16) = st[i];
        __syncthreads();
        if (++tile == n_tiles) tile = 0;
    }
    const float v = reinterpret_cast<const float *>(lds)[(threadIdx.x * 29) & 16383];
    if (v == 12345.678f) g_probe_sink = v;
}

}  // namespace
}  // namespace tst

extern "C" {

int tstgemm_probe_lds_read(int iters, int64_t *bytes_read, void *stream)
{
    if (iters < 1 || iters > (1 << 20)) return TSTGEMM_EINVAL;
    const int grid = 2 * tst::compute_units();
    hipLaunchKernelGGL(tst::k_probe_lds, dim3(grid), dim3(tst::kProbeThreads), 0, static_cast<hipStream_t>(stream), iters);
    if (hipGetLastError() != hipSuccess) return TSTGEMM_EHIP;
    if (bytes_read)
        *bytes_read = (int64_t)grid * tst::kProbeThreads * 16 * tst::kProbeReadsPerIter * (int64_t)iters;
    return TSTGEMM_OK;
}

int tstgemm_probe_stream_read(const void *buf, size_t bytes, void *stream)
{
    if (!buf || bytes < 16 || (reinterpret_cast<uintptr_t>(buf) & 15)) return TSTGEMM_EINVAL;
    const int grid = 8 * tst::compute_units();
    hipLaunchKernelGGL(tst::k_probe_stream, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const tst::float4v *>(buf), bytes / 16);
    return hipGetLastError() == hipSuccess ? TSTGEMM_OK : TSTGEMM_EHIP;
}

int tstgemm_probe_tile_copy(const void *buf, size_t bytes, int iters, int64_t *bytes_copied, void *stream)
{
    constexpr size_t kTile = 64 * 1024;
    if (!buf || bytes < kTile || (reinterpret_cast<uintptr_t>(buf) & 15) || iters < 1 || iters > (1 << 20)) return TSTGEMM_EINVAL;
    const size_t tiles = bytes / kTile;
    const int n_tiles = tiles > 0x7fffffffu ? 0x7fffffff : (int)tiles;
    const int grid = 2 * tst::compute_units();
    hipLaunchKernelGGL(tst::k_probe_tile_copy, dim3(grid), dim3(tst::kProbeThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const char *>(buf), n_tiles, iters);
    if (hipGetLastError() != hipSuccess) return TSTGEMM_EHIP;
    if (bytes_copied) *bytes_copied = (int64_t)grid * (int64_t)kTile * iters;
    return TSTGEMM_OK;
}

}  // extern "C"
