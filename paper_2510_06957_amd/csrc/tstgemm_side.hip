// Side kernels of the tiled gather-add paths of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper):
// k_pack_x, which lays X out as transposed row tiles before the main kernel, and k_reduce, which adds the K slices of a
// split-K run in a fixed order, adds the bias (once, last), applies the optional PReLU and writes Y.
#include <atomic>

#include "tstgemm_internal.h"

namespace tst {
namespace {

typedef float float4v __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------------------------------
// k_pack_x: X (rows m_begin .. m_begin + rows) -> xt[tile][k_pad][TM], zero padded.  One workgroup per (K-block,
// 64 rows): 64 x 64 floats go through the LDS so that both the reads (along k) and the writes (along rows) are
// contiguous.  VEC: rows of X are 16-byte aligned and K is a multiple of 4.
constexpr int kPackThreads = 256;

template <bool VEC>
__global__ void __launch_bounds__(kPackThreads)
k_pack_x(const float *__restrict__ X, float *__restrict__ xt, int rows, int K, int k_pad, int TM)
{
    __shared__ float t[64][65];
    const int kb = blockIdx.x, m0 = blockIdx.y * 64;
    const int c = threadIdx.x & 15, r = threadIdx.x >> 4;
    const int k = kb * 64 + 4 * c;
    // The four loads are issued unconditionally, so that they are all in flight together: rows beyond the last one
    // read the last row, pieces beyond K read the start of the row, and both are zeroed afterwards.
    float4v v[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int m = m0 + r + 16 * p;
        const float *src = X + (size_t)min(m, rows - 1) * K;
        if constexpr (VEC) {
            v[p] = *reinterpret_cast<const float4v *>(src + (k < K ? k : 0));   // K % 4 == 0: inside or outside as a whole
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[p][j] = src[k + j < K ? k + j : 0];
        }
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int row = r + 16 * p;
        const bool row_ok = m0 + row < rows;
#pragma unroll
        for (int j = 0; j < 4; ++j) t[4 * c + j][row] = (row_ok && k + j < K) ? v[p][j] : 0.f;
    }
    __syncthreads();
    const int kk = threadIdx.x >> 2, q = threadIdx.x & 3;
    if (16 * q >= TM) return;   // TM = 32 or 16: one tile, the rows beyond it do not exist
    const int tile = m0 / TM, r0 = m0 % TM;
    float *dst = xt + ((size_t)tile * k_pad + (size_t)kb * 64 + kk) * TM + r0 + 16 * q;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float4v o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = t[kk][16 * q + 4 * i + j];
        *reinterpret_cast<float4v *>(dst + 4 * i) = o;
    }
}

// ------------------------------------------------------------------------------------------------------------------
// k_reduce: Y = (slice 0 + slice 1 + ... in this order) + b, then the optional PReLU.  The partial sums of a workgroup tile are stored
// [column][row]; one workgroup of k_reduce takes kReduceRows rows x C columns of a tile, adds the slices, turns the
// block round in the LDS and stores rows of Y.  C = 16 NCW columns, TM rows per tile.  The partial sums are read
// once and were written past the caches, so they are loaded as non-temporal data.
constexpr int kReduceThreads = 256;
constexpr int kReduceRows = 32;
constexpr int kMaxSlices = kMaxKSlices;

template <int C>
__global__ void __launch_bounds__(kReduceThreads)
k_reduce(const float *__restrict__ P, const float *__restrict__ b, const float *__restrict__ alpha, int alpha_stride,
         float *__restrict__ Y, int M, int N, int n_colgroups, int k_slices, int TM)
{
    __shared__ float t[C][kReduceRows + 1];
    constexpr int kRowQuads = kReduceRows / 4;                   // threads along the rows of a column
    constexpr int kColsPerPass = kReduceThreads / kRowQuads;
    static_assert(C % kColsPerPass == 0 || kColsPerPass % C == 0, "column passes");
    const int sub_per_tile = TM / kReduceRows;
    const int group = blockIdx.x / sub_per_tile, sub = blockIdx.x % sub_per_tile;
    const int mt = group / n_colgroups, cg = group % n_colgroups;
    const size_t tile_floats = (size_t)C * TM;
    const float *base = P + (size_t)group * k_slices * tile_floats + (size_t)sub * kReduceRows;
    const int rr = (threadIdx.x % kRowQuads) * 4;
#pragma unroll
    for (int pass = 0; pass < (C + kColsPerPass - 1) / kColsPerPass; ++pass) {
        const int c = pass * kColsPerPass + threadIdx.x / kRowQuads;
        if (C < kColsPerPass && c >= C) break;
        const float *src = base + (size_t)c * TM + rr;
        // all slices are requested before the first addition; the additions then run in slice order
        float4v part[kMaxSlices];
#pragma unroll
        for (int s = 0; s < kMaxSlices; ++s)
            part[s] = __builtin_nontemporal_load(
                reinterpret_cast<const float4v *>(src + (size_t)(s < k_slices ? s : 0) * tile_floats));
        float4v sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kMaxSlices; ++s)
            if (s < k_slices) sum += part[s];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[c][rr + i] = sum[i];
    }
    __syncthreads();
    constexpr int kQuads = C / 4;                          // float4 pieces of an output row
    constexpr int kRowsPerPass = kReduceThreads / kQuads;
    const int q = threadIdx.x % kQuads;
    const int n = cg * C + 4 * q;
    const bool vec = (N % 4 == 0) && (n + 4 <= N) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
    float bias[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bias[j] = (b != nullptr && n + j < N) ? b[n + j] : 0.f;
#pragma unroll
    for (int pass = 0; pass < (kReduceRows + kRowsPerPass - 1) / kRowsPerPass; ++pass) {
        const int r = pass * kRowsPerPass + threadIdx.x / kQuads;
        const int m = mt * TM + sub * kReduceRows + r;
        if (r >= kReduceRows || m >= M) continue;
        float *dst = Y + (size_t)m * N + n;
        if (vec) {
            float4v o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = activate(t[4 * q + j][r] + bias[j], alpha, alpha_stride, n + j);
            *reinterpret_cast<float4v *>(dst) = o;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (n + j < N) dst[j] = activate(t[4 * q + j][r] + bias[j], alpha, alpha_stride, n + j);
        }
    }
}

}  // namespace

// Compute units of the current device; remembered per device (read-only facts about the machine).
int compute_units()
{
    constexpr int kDevices = 64;
    static std::atomic<int> cus[kDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    const bool cached = dev >= 0 && dev < kDevices;
    int n = cached ? cus[dev].load(std::memory_order_relaxed) : 0;
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        if (cached) cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}


hipError_t launch_pack(const float *X, float *xt, int rows, int K, int k_pad, int TM, hipStream_t stream)
{
    if (TM < 64 && ((TM != 32 && TM != 16) || rows > TM)) return hipErrorInvalidValue;   // short tiles: a single tile only
    const long long chunks = TM < 64 ? 1 : ((long long)rows + TM - 1) / TM * (TM / 64);
    if (chunks > 65535 || k_pad % 64 != 0) return hipErrorInvalidValue;
    const bool vec = (K % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    const dim3 grid((unsigned)(k_pad / 64), (unsigned)chunks);
    if (vec)
        hipLaunchKernelGGL((k_pack_x<true>), grid, dim3(kPackThreads), 0, stream, X, xt, rows, K, k_pad, TM);
    else
        hipLaunchKernelGGL((k_pack_x<false>), grid, dim3(kPackThreads), 0, stream, X, xt, rows, K, k_pad, TM);
    return hipGetLastError();
}

hipError_t launch_reduce(int C, const float *partials, const float *b, const Activation &act, float *Y, int M, int N,
                         int m_tiles, int n_colgroups, int k_slices, int TM, hipStream_t stream)
{
    const long long blocks = (long long)m_tiles * n_colgroups * (TM / kReduceRows);
    if (blocks > 0x7fffffffLL || k_slices > kMaxKSlices) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(kReduceThreads);
    switch (C) {
    case 16:
        hipLaunchKernelGGL((k_reduce<16>), grid, block, 0, stream, partials, b, act.alpha, act.alpha_stride, Y, M, N,
                           n_colgroups, k_slices, TM);
        break;
    case 32:
        hipLaunchKernelGGL((k_reduce<32>), grid, block, 0, stream, partials, b, act.alpha, act.alpha_stride, Y, M, N,
                           n_colgroups, k_slices, TM);
        break;
    case 64:
        hipLaunchKernelGGL((k_reduce<64>), grid, block, 0, stream, partials, b, act.alpha, act.alpha_stride, Y, M, N,
                           n_colgroups, k_slices, TM);
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace tst
