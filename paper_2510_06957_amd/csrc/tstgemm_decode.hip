// Small-M (decode) kernel of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper), M <= 8.
//
// With so few rows the operation moves more index bytes than it does additions (the paper's
// operational-intensity argument, Sec. 4), so the kernel is shaped around streaming the TCSC
// index arrays (Sec. 2) from HBM exactly once, fully coalesced, in their original form:
//   * all of X (M x K fp32) is kept in the LDS, transposed to xs[k][m], so one gathered index
//     yields the M operands of all rows at once;
//   * one wavefront per column; its 64 lanes split the column's +1 list and then its -1 list
//     (the paper's "horizontal" SIMD scheme, Sec. 3: partial sums per lane, one horizontal sum
//     at the end), reading 4 consecutive indices per lane with a 16-byte load;
//   * the M per-lane partial sums are folded across the wavefront by a halving exchange, the
//     bias is added once, last (then the optional PReLU), and one lane per row stores the result.
#include "tstgemm_internal.h"

namespace tst {
namespace {

constexpr int kDecodeThreads = 1024;
constexpr int kDecodeMaxLds = 150 * 1024;
typedef int int4v __attribute__((ext_vector_type(4)));

// Butterfly sum over the 64 lanes of each of the MM values; every lane ends with all totals.
template <int MM> __device__ __forceinline__ void wave_sum(float (&v)[MM])
{
#pragma unroll
    for (int m = 0; m < MM; ++m) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v[m] += __shfl_xor(v[m], d, 64);
    }
}

template <int MM>
__global__ void __launch_bounds__(kDecodeThreads)
k_decode(const float *__restrict__ X, const int32_t *__restrict__ csp, const int32_t *__restrict__ csn,
         const int32_t *__restrict__ rip, const int32_t *__restrict__ rin, const float *__restrict__ b,
         const float *__restrict__ alpha, int alpha_stride, float *__restrict__ Y, int K, int N)
{
    extern __shared__ __attribute__((aligned(16))) float xs[];   // [K + 1][MM], row K is all zero
    for (int k = threadIdx.x; k <= K; k += kDecodeThreads) {
#pragma unroll
        for (int m = 0; m < MM; ++m) xs[k * MM + m] = k < K ? X[(size_t)m * K + k] : 0.f;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int waves_total = gridDim.x * (kDecodeThreads / 64);
    for (int n = blockIdx.x * (kDecodeThreads / 64) + wave; n < N; n += waves_total) {
        float acc[MM];
#pragma unroll
        for (int m = 0; m < MM; ++m) acc[m] = 0.f;
#pragma unroll
        for (int sign = 0; sign < 2; ++sign) {
            const int32_t *__restrict__ rows = sign ? rin : rip;
            const int p0 = sign ? csn[n] : csp[n], p1 = sign ? csn[n + 1] : csp[n + 1];
            // 16-byte aligned sweep over [p0, p1): slots outside the range gather the zero row K
            for (int i = (p0 & ~3) + lane * 4; i < p1; i += 256) {
                const int4v q = *reinterpret_cast<const int4v *>(rows + i);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = (i + e >= p0 && i + e < p1) ? q[e] : K;
#pragma unroll
                    for (int m = 0; m < MM; ++m) {
                        if (sign) acc[m] -= xs[k * MM + m]; else acc[m] += xs[k * MM + m];
                    }
                }
            }
        }
        wave_sum<MM>(acc);
        const float bias = b ? b[n] : 0.f;
#pragma unroll
        for (int m = 0; m < MM; ++m)
            if (lane == m) Y[(size_t)m * N + n] = activate(acc[m] + bias, alpha, alpha_stride, n);
    }
}

int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

template <int MM>
hipError_t launch(const float *X, const tcsc *t, const float *b, const Activation &act, float *Y, hipStream_t stream)
{
    const DeviceTcsc d = device_view(t);
    const size_t lds = (size_t)(t->K + 1) * MM * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_decode<MM>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kDecodeMaxLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int per_cu = lds * 2 <= (size_t)160 * 1024 ? 2 : 1;
    int grid = compute_units() * per_cu;
    const int need = (t->N + kDecodeThreads / 64 - 1) / (kDecodeThreads / 64);
    if (grid > need) grid = need;
    hipError_t e;
    if (g_event_before && (e = hipEventRecord(g_event_before, stream)) != hipSuccess) return e;
    hipLaunchKernelGGL((k_decode<MM>), dim3(grid), dim3(kDecodeThreads), lds, stream, X, d.col_start_pos,
                       d.col_start_neg, d.row_index_pos, d.row_index_neg, b, act.alpha, act.alpha_stride, Y, t->K, t->N);
    e = hipGetLastError();
    if (e == hipSuccess && g_event_after) e = hipEventRecord(g_event_after, stream);
    return e;
}

}  // namespace

bool decode_supported(int M, int K) { return M <= 8 && (size_t)(K + 1) * M * sizeof(float) <= (size_t)kDecodeMaxLds; }

hipError_t launch_decode(const float *X, const tcsc *t, const float *b, const Activation &act, float *Y, int M,
                         hipStream_t stream)
{
    switch (M) {
    case 1: return launch<1>(X, t, b, act, Y, stream);
    case 2: return launch<2>(X, t, b, act, Y, stream);
    case 3: return launch<3>(X, t, b, act, Y, stream);
    case 4: return launch<4>(X, t, b, act, Y, stream);
    case 5: return launch<5>(X, t, b, act, Y, stream);
    case 6: return launch<6>(X, t, b, act, Y, stream);
    case 7: return launch<7>(X, t, b, act, Y, stream);
    case 8: return launch<8>(X, t, b, act, Y, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tst
