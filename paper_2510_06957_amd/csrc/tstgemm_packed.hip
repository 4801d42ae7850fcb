// Small-M kernel (M <= 8) of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper) on the paper's "value
// compression" encoding of W (Sec. 3): five consecutive rows of a column in one byte, read as a base-3 number.
//
// The encoding is dense: 1.6 bits per entry of W whatever the density, against 32 bits per NON-zero entry for
// TCSC, i.e. a tenth of the index bytes at 50 % density -- the one thing the M <= 8 path is bound by.  The price,
// as the paper notes, is that the zeros take part in the work.
//
//   * a lane owns one column, a wavefront 64 columns and a slice of K; a lane loads 16 bytes = 16 groups = 80 rows
//     of its column at a time (device layout packed[chunk][column][16], so the lanes of a wavefront read
//     consecutive 16-byte pieces), one load ahead of its use;
//   * every byte goes through a 243-entry table in the LDS (the paper's decoding table) that yields the five
//     weights as signed bytes; a weight becomes a float and the entry is accumulated as one fused multiply-add
//     x * w with w in {-1, 0, +1}: the product is exact, so the arithmetic is that of the additions and
//     subtractions of BaseTCSC (Sec. 2) plus additions of +-0.  (Only for finite X: 0 * inf is not 0.)
//   * the K slice is the same for all lanes of a wavefront, so the X entries are wave-uniform: they come through
//     the scalar cache into SGPRs and enter the multiply-add as scalar operands -- no LDS traffic, no staging, no
//     barrier inside the loop;
//   * a workgroup is 64 columns x 16 slices of K (pieces dealt round-robin to the wavefronts); the slices are
//     added in slice order through the LDS, the bias is added once, last;
//   * when N / 64 workgroups leave half of the chip idle and there are enough rows of X to pay for a second launch, K is
//     also dealt to several workgroups per column group, which hand their sums (as tiles of 64 columns x 32 rows)
//     to the reduction kernel of the tiled paths: fixed order, bias last, no atomics.
#include "tstgemm_internal.h"

namespace tst {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kRowsPerChunk = 5 * kChunk5;            // 80 rows of W per 16-byte piece
constexpr int kPartRows = 32;                         // rows of a tile handed to the reduction kernel (its granularity)
constexpr int kXRows = 3;                             // rows of X whose entries are held in scalar registers at a time
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(4))) float *const_f32_ptr;   // read through the scalar cache

// A quarter of a 16-byte piece: four codes = 20 rows of W (first row k, wave-uniform) x MM rows of X.
// CLAMP: the 20 rows reach beyond K; such rows have weight 0 (their digits are 0), and the X entry they are
// multiplied with is taken from row K - 1 instead, so that nothing outside X is read (a vector load, one row per
// lane, and 20 lane reads: clamped scalar addresses would cost the compiler hundreds of scalar registers).
template <int MM, bool CLAMP>
__device__ __forceinline__ void run_quarter(float (&acc)[MM], unsigned codes, const uint2v *lut, const_f32_ptr X, int K, int k,
                                            int lane)
{
    float w[20];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint2v e = lut[(codes >> (8 * j)) & 0xffu];
#pragma unroll
        for (int r = 0; r < 4; ++r) w[5 * j + r] = (float)(int)(signed char)(e.x >> (8 * r));
        w[5 * j + 4] = (float)(int)(signed char)e.y;
    }
    // X entries in blocks of at most kXRows rows of X x 20 rows of W (60 scalar registers); the compiler must not
    // gather the scalar loads of several blocks in one place (it would run out of scalar registers)
#pragma unroll
    for (int m0 = 0; m0 < MM; m0 += kXRows) {
        asm volatile("" ::: "memory");
        float x[kXRows][20];
#pragma unroll
        for (int m = m0; m < MM && m < m0 + kXRows; ++m) {
            if constexpr (CLAMP) {
                // lane r fetches the entry of row k + r (clamped), then the 20 values are spread to all lanes
                const float mine = reinterpret_cast<const float *>(reinterpret_cast<uintptr_t>(X))[(size_t)m * K + min(k + lane, K - 1)];
#pragma unroll
                for (int r = 0; r < 20; ++r) x[m - m0][r] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mine), r));
            } else {
                const const_f32_ptr xm = X + (size_t)m * K + k;
#pragma unroll
                for (int r = 0; r < 20; ++r) x[m - m0][r] = xm[r];
            }
        }
        asm volatile("" ::: "memory");
#pragma unroll
        for (int m = m0; m < MM && m < m0 + kXRows; ++m)
#pragma unroll
            for (int r = 0; r < 20; ++r) acc[m] = __builtin_fmaf(x[m - m0][r], w[r], acc[m]);
    }
}

// One 16-byte piece: 16 codes x 5 rows x MM rows of X, all 80 rows below K.  k0: first row of W of the piece.
template <int MM>
__device__ __forceinline__ void run_piece(float (&acc)[MM], const uint4v &codes, const uint2v *lut, const_f32_ptr X,
                                          int K, int k0)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) run_quarter<MM, false>(acc, codes[q], lut, X, K, k0 + 20 * q, 0);
}

// The last piece of a column when K is not a multiple of 80.  Runs at most once per wavefront.
template <int MM>
__device__ __forceinline__ void run_last_piece(float (&acc)[MM], const uint4v &codes, const uint2v *lut, const_f32_ptr X, int K,
                                               int k0, int lane)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int k = k0 + 20 * q;
        if (k + 20 <= K) run_quarter<MM, false>(acc, codes[q], lut, X, K, k, lane);
        else if (k < K) run_quarter<MM, true>(acc, codes[q], lut, X, K, k, lane);
    }
}

template <int MM>
__global__ void __launch_bounds__(kThreads)
k_packed(const float *__restrict__ X, const uint8_t *__restrict__ packed, const float *__restrict__ b,
         float *__restrict__ Y, float *__restrict__ partials, int K, int N, int n_pad, int n_chunks, int k_parts)
{
    __shared__ uint2v lut[256];                 // code -> five weights as signed bytes
    __shared__ float sums[kWaves][MM][64];      // the K slices of the workgroup
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_colgroups = n_pad / 64;
    const int cg = blockIdx.x % n_colgroups, part = blockIdx.x / n_colgroups;
    const int n = cg * 64 + lane;               // < n_pad
    const int first = part * kWaves + wave, step = k_parts * kWaves;   // this wavefront's pieces: first, first + step, ...

    if (threadIdx.x < 256) {
        // digits of the code, first row most significant; digit 1 -> +1, digit 2 -> -1 (0xff as a signed byte)
        unsigned rest = threadIdx.x, lo = 0, hi = 0;
#pragma unroll
        for (int j = 4; j >= 0; --j) {
            const unsigned d = rest % 3;
            rest /= 3;
            const unsigned w = d == 0 ? 0u : d == 1 ? 1u : 0xffu;
            if (j == 4) hi = w; else lo |= w << (8 * j);
        }
        uint2v e = {lo, hi};
        if (threadIdx.x >= 243) e = uint2v{0u, 0u};   // not a code
        lut[threadIdx.x] = e;
    }
    __syncthreads();

    float acc[MM];
#pragma unroll
    for (int m = 0; m < MM; ++m) acc[m] = 0.f;
    const const_f32_ptr Xs = reinterpret_cast<const_f32_ptr>(reinterpret_cast<uintptr_t>(X));
    const uint8_t *col = packed + (size_t)n * kChunk5;
    const size_t chunk_stride = (size_t)n_pad * kChunk5;
    uint4v next = {0u, 0u, 0u, 0u};
    if (first < n_chunks) next = *reinterpret_cast<const uint4v *>(col + (size_t)first * chunk_stride);
    for (int c = first; c < n_chunks; c += step) {
        const uint4v codes = next;
        if (c + step < n_chunks) next = *reinterpret_cast<const uint4v *>(col + (size_t)(c + step) * chunk_stride);
        const int k0 = c * kRowsPerChunk;
        if (k0 + kRowsPerChunk <= K) run_piece<MM>(acc, codes, lut, Xs, K, k0);
        else run_last_piece<MM>(acc, codes, lut, Xs, K, k0, lane);
    }

    // slice sums -> LDS, added in slice order; bias once, last
#pragma unroll
    for (int m = 0; m < MM; ++m) sums[wave][m][lane] = acc[m];
    __syncthreads();
    if (threadIdx.x < 64 * MM) {
        const int m = threadIdx.x >> 6;
        float sum = 0.f;
#pragma unroll
        for (int s = 0; s < kWaves; ++s) sum += sums[s][m][lane];
        if (k_parts == 1) {
            if (n < N) Y[(size_t)m * N + n] = sum + (b != nullptr ? b[n] : 0.f);
        } else {
            // a tile of the reduction kernel: [column group][part][64 columns][32 rows], rows >= MM unused
            partials[(((size_t)cg * k_parts + part) * 64 + lane) * kPartRows + m] = sum;
        }
    }
}

template <int MM> hipError_t launch(const float *X, const tcsc *t, const float *b, float *Y, const Call &c)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    const hipStream_t stream = c.stream;
    float *const partials = reinterpret_cast<float *>(c.ws);   // may be absent: K is then not dealt to several workgroups
    const int n_colgroups = l.n_pad / 64;
    // parts of K per column group: only if the column groups leave at least half of the compute units idle (with 172
    // groups on 256 units three parts were slower than one) and a column holds enough work (rows of X x pieces) to
    // outweigh the second launch; every wavefront must still get a piece
    int k_parts = c.k_slices;
    if (k_parts == 0) {
        const int cus = compute_units();
        k_parts = (2 * n_colgroups <= cus && MM * l.n_chunks5 >= 400) ? cus / n_colgroups : 1;
        if (k_parts > 4) k_parts = 4;
    }
    if (k_parts > l.n_chunks5 / kWaves) k_parts = l.n_chunks5 / kWaves;
    if (partials == nullptr || (size_t)n_colgroups * k_parts * 64 * kPartRows * sizeof(float) > c.ws_bytes) k_parts = 1;
    if (k_parts < 1) k_parts = 1;
    hipError_t e;
    if ((e = c.record_before()) != hipSuccess) return e;
    hipLaunchKernelGGL((k_packed<MM>), dim3((unsigned)(n_colgroups * k_parts)), dim3(kThreads), 0, stream, X, d.packed, b, Y,
                       partials, l.K, l.N, l.n_pad, l.n_chunks5, k_parts);
    e = hipGetLastError();
    if (e == hipSuccess) e = c.record_after();
    if (e != hipSuccess || k_parts == 1) return e;
    return launch_reduce(64, partials, b, Activation{nullptr, 0}, Y, MM, l.N, 1, n_colgroups, k_parts, kPartRows, stream);
}

}  // namespace

hipError_t launch_packed(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c)
{
    switch (M) {
    case 1: return launch<1>(X, t, b, Y, c);
    case 2: return launch<2>(X, t, b, Y, c);
    case 3: return launch<3>(X, t, b, Y, c);
    case 4: return launch<4>(X, t, b, Y, c);
    case 5: return launch<5>(X, t, b, Y, c);
    case 6: return launch<6>(X, t, b, Y, c);
    case 7: return launch<7>(X, t, b, Y, c);
    case 8: return launch<8>(X, t, b, Y, c);
    default: return hipErrorInvalidValue;
    }
}

// At most 4 workgroups per group of 64 columns write partial sums of kPartRows rows each.
size_t packed_partial_bytes(int N)
{
    const size_t n_colgroups = ((size_t)N + 63) / 64;
    return n_colgroups * kMaxKSlices * 64 * kPartRows * sizeof(float);
}

}  // namespace tst
