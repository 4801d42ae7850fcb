// Small-M (decode) kernel of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper), M <= 8.
//
// With so few rows the operation moves more index bytes than it does additions (the paper's
// operational-intensity argument, Sec. 4), so the kernel is shaped around streaming the TCSC
// index arrays (Sec. 2) from HBM exactly once, fully coalesced, in their original form:
//   * X (M x K fp32) is kept in the LDS, transposed to xs[k][m], so one gathered index yields
//     the M operands of all rows at once (for M > 4 in two planes of at most four rows of X each: a gather
//     is then a 16-byte read per plane that can start at any of the 16 bank groups, not only at every other).  If all of X does not fit, K is cut into chunks of
//     as many rows as fit (the paper's K-blocking, Sec. 3, with the LDS in the place of the L1
//     cache) and the chunks are taken one after the other; the lists are ascending, so the
//     part of a list that falls into a chunk is contiguous and a cursor per list is enough;
//   * one wavefront per column; its 64 lanes split the column's +1 list and then its -1 list
//     (the paper's "horizontal" SIMD scheme, Sec. 3: partial sums per lane, one horizontal sum
//     at the end), reading 4 consecutive indices per lane with a 16-byte load -- or 8, from the
//     padded 16-bit copy of the lists that the upload pass makes when K <= 65535: the kernel is
//     bound by the bytes of the lists, a row number below 65536 does not need 32 bits, and with
//     every list padded to whole 16-byte pieces (pad value K, the row of zeros; the paper's
//     dummy-zero padding, Sec. 3) no entry has to be masked;
//   * the M per-lane partial sums are folded across the wavefront by a halving exchange, the
//     bias is added once, last (then the optional PReLU), and one lane per row stores the result.
// The same kernel also runs on the paper's inverted-index form (Sec. 3): one merged list per column
// whose entries carry their sign (i for +1, ~i for -1); the sign bit is flipped into the operand.
#include <atomic>

#include "tstgemm_internal.h"

namespace tst {
namespace {

constexpr int kDecodeThreads = 1024;
constexpr int kDecodeWaves = kDecodeThreads / 64;
constexpr int kDecodeMaxLds = 150 * 1024;   // ... for X
constexpr int kSlotColumns = 64;            // columns whose two list sums a workgroup keeps in the LDS at a time
typedef int int4v __attribute__((ext_vector_type(4)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));

// Butterfly sum over the 64 lanes of each of the MM values; every lane ends with all totals.
template <int MM> __device__ __forceinline__ void wave_sum(float (&v)[MM])
{
#pragma unroll
    for (int m = 0; m < MM; ++m) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v[m] += __shfl_xor(v[m], d, 64);
    }
}

// xs: plane p holds rows 4p .. 4p+3 of X (the last plane the rest) as plane[k][width]; every plane has kc + 1 rows, the
// last one zero.  Offset (in floats) of element (k, m) for a view whose row 0 is row k_lo of X.
template <int MM> __device__ __forceinline__ int xs_at(int k, int m, int kc1)
{
    const int p = m >> 2, width = (MM - 4 * p) < 4 ? (MM - 4 * p) : 4;
    return 4 * p * kc1 + k * width + (m & 3);
}

// Rows of X a chunk holds for MM rows of X: all of the LDS budget but one row of zeros.
template <int MM> constexpr int chunk_rows() { return kDecodeMaxLds / (MM * (int)sizeof(float)) - 1; }

// The part of the ascending list rows[p .. p1) with row numbers below k_hi: gathered and added to (MODE 1: subtracted
// from) acc; p moves to the first entry that was not consumed.  MODE 2: a merged list of the inverted-index form
// (Sec. 3), an entry i >= 0 adds row i, an entry ~i < 0 subtracts row i: the sign bit of the entry is flipped into the
// operand, no branch.  k_lo is the first row of X in the LDS: xs[xs_at(k - k_lo, m)] is X[m][k] for k in [k_lo, k_hi);
// row k_zero holds zeros.  The sweep is 16-byte aligned, in rounds of 256
// entries per wavefront; slots in front of p or behind the last consumed entry gather the row of zeros.
// CHUNKED = false: the chunk is all of K, nothing can be late.
template <int MM, int MODE, bool CHUNKED>
__device__ __forceinline__ void run_sublist(float (&acc)[MM], const int32_t *__restrict__ rows, int &p, int p1, int k_hi,
                                            int k_zero, const float *xs, int k_lo, int kc1, int lane)
{
    // The 16 bytes of a lane for the round that starts at entry `at`.  The load is unconditional (so that the next
    // round can be in flight while this one is gathered): lanes behind the end of the list read the piece at its
    // end instead (the arrays have that much slack), and every slot outside [p, p1) is masked below anyway.
    const int last_piece = p1 & ~3;
    auto fetch = [&](int at) {
        return *reinterpret_cast<const int4v *>(rows + min(at + lane * 4, last_piece));
    };
    int4v ahead = fetch(p & ~3);
    while (p < p1) {
        const int i = (p & ~3) + lane * 4;
        const int4v q = ahead;
        ahead = fetch((p & ~3) + 256);
        int first_late = 4;   // first slot of this lane that belongs to a later chunk
#pragma unroll
        for (int e = 3; e >= 0; --e) {
            const bool live = i + e >= p && i + e < p1;
            const int row = MODE == 2 ? (q[e] ^ (q[e] >> 31)) : q[e];
            const unsigned flip = MODE == 2 ? ((unsigned)q[e] & 0x80000000u) : 0u;
            const bool late = CHUNKED && live && row >= k_hi;
            if (late) first_late = e;
            const int k = (live && !late) ? row : k_zero;
#pragma unroll
            for (int m = 0; m < MM; ++m) {
                const float x = xs[xs_at<MM>(k - k_lo, m, kc1)];
                if (MODE == 1) acc[m] -= x;
                else if (MODE == 2) acc[m] += __uint_as_float(__float_as_uint(x) ^ flip);
                else acc[m] += x;
            }
        }
        const unsigned long long late_lanes = CHUNKED ? __ballot(first_late < 4) : 0ull;
        if (late_lanes == 0) {
            p = (p & ~3) + 256;   // the whole round was consumed (or lay behind p1)
        } else {
            const int l = __builtin_ctzll(late_lanes);
            p = (p & ~3) + 4 * l + __builtin_amdgcn_readlane(first_late, l);
            return;               // the rest of the list belongs to later chunks
        }
    }
    p = p1;
}

// A list of the padded 16-bit copy, entries [p, p1), both multiples of 8: a lane takes 8 consecutive entries (16 bytes)
// per round, a wavefront 512; every entry is a row number or K, the row of zeros, so nothing has to be masked.  All of
// X is in the LDS (this form is not used with chunks of K).  NEG: subtract.
template <int MM, bool NEG>
__device__ __forceinline__ void run_list16(float (&acc)[MM], const uint16_t *__restrict__ rows, int p, int p1, const float *xs,
                                           int kc1, int lane)
{
    if (p >= p1) return;
    const int last_piece = p1 - 8;
    auto fetch = [&](int at) {   // unconditional: a lane behind the end reads the last piece again and does not use it
        return *reinterpret_cast<const uint4v *>(rows + min(at + lane * 8, last_piece));
    };
    uint4v ahead = fetch(p);
    for (int at = p; at < p1; at += 512) {
        const uint4v q = ahead;
        ahead = fetch(at + 512);   // the next round is on its way while this one is gathered
        if (at + lane * 8 < p1) {
            // four entries at a time: all their gathers are issued before the first addition (left to itself the
            // compiler waits for the two reads of an entry right behind them, one entry in flight per wavefront)
#pragma unroll
            for (int e0 = 0; e0 < 8; e0 += 4) {
                float x[4][MM];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = (int)((q[(e0 + e) >> 1] >> (16 * (e & 1))) & 0xffffu);
#pragma unroll
                    for (int m = 0; m < MM; ++m) x[e][m] = xs[xs_at<MM>(row, m, kc1)];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int m = 0; m < MM; ++m) {
                        if (NEG) acc[m] -= x[e][m]; else acc[m] += x[e][m];
                    }
            }
        }
    }
}

// FORM 0: csp / csn / rip / rin are the TCSC arrays; FORM 1: rip is the merged list of the inverted-index form (column
// n at col_start_pos[n] + col_start_neg[n]), rin unused; FORM 2 (not with CHUNKED): csp / csn / rip / rin are the
// pointers and the entries of the padded 16-bit copy of the lists.
template <int MM, bool CHUNKED, int FORM>
__global__ void __launch_bounds__(kDecodeThreads)
k_decode(const float *__restrict__ X, const int32_t *__restrict__ csp, const int32_t *__restrict__ csn,
         const void *__restrict__ rip_, const void *__restrict__ rin_, const float *__restrict__ b,
         const float *__restrict__ alpha, int alpha_stride, float *__restrict__ Y, int K, int N, int kc, int deal_lists)
{
    static_assert(!(FORM == 2 && CHUNKED), "the padded 16-bit lists need all of X in the LDS");
    constexpr bool SIGNED = FORM == 1;
    const int32_t *rip = static_cast<const int32_t *>(rip_), *rin = static_cast<const int32_t *>(rin_);
    extern __shared__ __attribute__((aligned(16))) float xs[];   // planes of [kc + 1][<= 4], row kc is all zero
    const int kc1 = kc + 1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int waves_total = gridDim.x * kDecodeWaves;
    const int n_chunks = CHUNKED ? (K + kc - 1) / kc : 1;
    const int n_batches = (N + waves_total - 1) / waves_total;

    // Row k of the chunk in the LDS: one write per plane (16 bytes for a full plane: a plane's row k is 16-byte
    // aligned), not one per row of X -- with single floats 16 bytes apart four lanes share a bank.
    auto store_row = [&](int k, const float (&x)[MM]) {
#pragma unroll
        for (int p0 = 0; p0 < MM; p0 += 4) {
            constexpr int kFull = 4;
            const int width = MM - p0 < kFull ? MM - p0 : kFull;
            float *dst = xs + xs_at<MM>(k, p0, kc1);
            if (width == 4) *reinterpret_cast<float4v *>(dst) = float4v{x[p0], x[p0 + 1 < MM ? p0 + 1 : p0], x[p0 + 2 < MM ? p0 + 2 : p0], x[p0 + 3 < MM ? p0 + 3 : p0]};
            else if (width == 3) { dst[0] = x[p0]; dst[1] = x[p0 + 1 < MM ? p0 + 1 : p0]; dst[2] = x[p0 + 2 < MM ? p0 + 2 : p0]; }   // rows of 12 bytes: no alignment to speak of
            else if (width == 2) *reinterpret_cast<float2v *>(dst) = float2v{x[p0], x[p0 + 1 < MM ? p0 + 1 : p0]};
            else dst[0] = x[p0];
        }
    };
    // The chunk of X a workgroup works on, transposed into the LDS.  For one or two rows of X, where the call is short
    // and this is a visible part of it, all requests of a thread go out before its first write (with a write behind
    // each request a thread waited for memory once per 1024 rows of the chunk: four times for K = 4096, about 1 us of
    // a 14 us call), and where the rows of X are 16-byte aligned a thread takes four consecutive k with one 16-byte
    // load.  With more rows of X neither changed the time of a call (M = 4, M = 8), so they keep the plain loop.
    auto load_chunk = [&](int c) {
        const int k_lo = c * kc, len = min(kc, K - k_lo);
        const float *Xc = X + k_lo;
        if constexpr (MM <= 2 && !CHUNKED) {
            const bool aligned = (((unsigned)K | (unsigned)len) & 3u) == 0 && (reinterpret_cast<uintptr_t>(X) & 15u) == 0;
            if (aligned) {
                for (int k4 = 4 * threadIdx.x; k4 < len; k4 += 4 * kDecodeThreads) {
                    float4v x4[MM];
#pragma unroll
                    for (int m = 0; m < MM; ++m) x4[m] = *reinterpret_cast<const float4v *>(Xc + (size_t)m * K + k4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float x[MM];
#pragma unroll
                        for (int m = 0; m < MM; ++m) x[m] = x4[m][i];
                        store_row(k4 + i, x);
                    }
                }
            } else {
                for (int k0 = threadIdx.x; k0 < len; k0 += 4 * kDecodeThreads) {
                    float x[4][MM];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int m = 0; m < MM; ++m) {
                            const int k = k0 + i * kDecodeThreads;
                            x[i][m] = k < len ? Xc[(size_t)m * K + k] : 0.f;
                        }
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (k0 + i * kDecodeThreads < len) store_row(k0 + i * kDecodeThreads, x[i]);
                }
            }
        } else {
            for (int k = threadIdx.x; k < len; k += kDecodeThreads) {
                float x[MM];
#pragma unroll
                for (int m = 0; m < MM; ++m) x[m] = Xc[(size_t)m * K + k];
                store_row(k, x);
            }
        }
    };
    if (threadIdx.x < MM) xs[xs_at<MM>(kc, threadIdx.x, kc1)] = 0.f;
    if (!CHUNKED) load_chunk(0);   // all of X fits: loaded once, for all columns of this workgroup
    __syncthreads();

    if (FORM == 2 && deal_lists) {
        // Lists, not columns, are dealt to the wavefronts: a workgroup takes a run of columns, wavefront w the lists
        // w, w + 16, ... of the run (list 2 c: the +1 list of its column c, 2 c + 1: the -1 list), and the two sums of
        // a column meet in the LDS.  The launch takes this when whole columns per wavefront would leave much of the
        // chip idle (N = 11008: 2.7 columns per wavefront of a chip-filling grid, so a third of the grid is left out and
        // 88 compute units do twice the work of the others) and the second sum over the wavefront per column is cheap
        // (one or two rows of X).
        float *const slot = xs + (size_t)MM * kc1;   // [kSlotColumns][2][MM] behind the planes of X
        const int per_wg = (N + (int)gridDim.x - 1) / (int)gridDim.x;
        const int c_begin = min(N, (int)blockIdx.x * per_wg), c_end = min(N, c_begin + per_wg);
        for (int c0 = c_begin; c0 < c_end; c0 += kSlotColumns) {
            const int columns = min(kSlotColumns, c_end - c0);
            for (int u = wave; u < 2 * columns; u += kDecodeWaves) {
                const int n = c0 + (u >> 1);
                float acc[MM];
#pragma unroll
                for (int m = 0; m < MM; ++m) acc[m] = 0.f;
                if (u & 1) run_list16<MM, true>(acc, static_cast<const uint16_t *>(rin_), csn[n], csn[n + 1], xs, kc1, lane);
                else run_list16<MM, false>(acc, static_cast<const uint16_t *>(rip_), csp[n], csp[n + 1], xs, kc1, lane);
                wave_sum<MM>(acc);
#pragma unroll
                for (int m = 0; m < MM; ++m)
                    if (lane == m) slot[u * MM + m] = acc[m];
            }
            __syncthreads();
            // Y = (sum of the +1 list) + (minus the sum of the -1 list) + b, bias last; consecutive threads take
            // consecutive columns
            for (int i = threadIdx.x; i < columns * MM; i += kDecodeThreads) {
                const int m = i / columns, c = i - m * columns, n = c0 + c;
                const float sum = slot[2 * c * MM + m] + slot[(2 * c + 1) * MM + m];
                Y[(size_t)m * N + n] = activate(sum + (b ? b[n] : 0.f), alpha, alpha_stride, n);
            }
            if (c0 + kSlotColumns < c_end) __syncthreads();   // the slots are written again
        }
        return;
    }
    // Every wavefront of the workgroup goes through the same number of batches and chunks (the barriers inside);
    // a wavefront without a column in the last batch just has empty lists.
    for (int batch = 0; batch < n_batches; ++batch) {
        const int n = batch * waves_total + blockIdx.x * kDecodeWaves + wave;
        const bool have = n < N;
        int pp = have ? csp[n] : 0, pp1 = have ? csp[n + 1] : 0;
        int pn = have ? csn[n] : 0, pn1 = have ? csn[n + 1] : 0;
        if (SIGNED) { pp += pn; pp1 += pn1; pn = pn1 = 0; }
        float acc[MM];
#pragma unroll
        for (int m = 0; m < MM; ++m) acc[m] = 0.f;
        if constexpr (FORM == 2) {
            run_list16<MM, false>(acc, static_cast<const uint16_t *>(rip_), pp, pp1, xs, kc1, lane);
            run_list16<MM, true>(acc, static_cast<const uint16_t *>(rin_), pn, pn1, xs, kc1, lane);
        } else
        for (int c = 0; c < n_chunks; ++c) {
            if (CHUNKED) {
                __syncthreads();   // everybody is done with the previous chunk
                load_chunk(c);
                __syncthreads();
            }
            const int k_lo = c * kc;
            const int k_hi = (c + 1 == n_chunks) ? 0x7fffffff : k_lo + kc;
            if (SIGNED) {
                run_sublist<MM, 2, CHUNKED>(acc, rip, pp, pp1, k_hi, k_lo + kc, xs, k_lo, kc1, lane);
            } else {
                run_sublist<MM, 0, CHUNKED>(acc, rip, pp, pp1, k_hi, k_lo + kc, xs, k_lo, kc1, lane);
                run_sublist<MM, 1, CHUNKED>(acc, rin, pn, pn1, k_hi, k_lo + kc, xs, k_lo, kc1, lane);
            }
        }
        if (!have) continue;
        wave_sum<MM>(acc);
        const float bias = b ? b[n] : 0.f;
#pragma unroll
        for (int m = 0; m < MM; ++m)
            if (lane == m) Y[(size_t)m * N + n] = activate(acc[m] + bias, alpha, alpha_stride, n);
    }
}

template <int MM, bool CHUNKED, int FORM>
hipError_t launch_kernel(const float *X, const tcsc *t, const float *b, float *Y, int kc, size_t lds, const Call &c)   // lds: bytes for X
{
    const DeviceTcsc d = device_view(t);
    const hipStream_t stream = c.stream;
    const Activation &act = c.act;
    // the kernel's LDS limit is an attribute of the function on a device: set once per device (bit = device number;
    // devices beyond 63 set it on every call)
    static std::atomic<unsigned long long> attr_devices{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    const unsigned long long bit = (dev >= 0 && dev < 64) ? 1ull << dev : 0;
    if ((attr_devices.load(std::memory_order_relaxed) & bit) == 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_decode<MM, CHUNKED, FORM>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kDecodeMaxLds + kSlotColumns * 2 * MM * (int)sizeof(float));
        if (e != hipSuccess) return e;
        attr_devices.fetch_or(bit, std::memory_order_relaxed);
    }
    // Whole columns per wavefront, every wavefront the same number, one after the other (with 1.3 columns per
    // wavefront a full grid would leave two thirds of the wavefronts, and of the loads in flight, idle during the
    // second round), or -- 16-bit lists, one or two rows of X -- the lists of a run of columns dealt to the wavefronts
    // of a workgroup, which fills every compute unit alike at the price of a second sum over the wavefront per column
    // (measured, M = 1: N = 11008 13.0 -> 12.5 us, N = 16384, where whole columns fit exactly, 15.9 -> 16.7 us; M = 8:
    // 24.5 -> 28.0 us).  The second is taken when the first would use less than 85 % of the slots of its rounds.
    const size_t lds_dealt = lds + (size_t)kSlotColumns * 2 * MM * sizeof(float);
    const int need = (t->N + kDecodeWaves - 1) / kDecodeWaves;
    int per_cu = lds * 2 <= (size_t)160 * 1024 ? 2 : 1;
    int grid = compute_units() * per_cu;
    if (grid > need) grid = need;
    const int rounds = (need + grid - 1) / grid;
    int deal_lists = 0;
    if (FORM == 2 && MM <= 2 && (double)need < 0.85 * (double)rounds * (double)grid) {
        deal_lists = 1;
        lds = lds_dealt;
        per_cu = lds * 2 <= (size_t)160 * 1024 ? 2 : 1;
        grid = compute_units() * per_cu;
        const int lists_need = (t->N + kDecodeWaves / 2 - 1) / (kDecodeWaves / 2);   // at least one list per wavefront
        if (grid > lists_need) grid = lists_need;
    } else {
        grid = (need + rounds - 1) / rounds;
    }
    hipError_t e;
    if ((e = c.record_before()) != hipSuccess) return e;
    const int32_t *cs_pos = FORM == 2 ? d.col_start16_pos : d.col_start_pos;
    const int32_t *cs_neg = FORM == 2 ? d.col_start16_neg : d.col_start_neg;
    const void *lists_pos = FORM == 1 ? static_cast<const void *>(d.signed_index)
                            : FORM == 2 ? static_cast<const void *>(d.row_index16_pos)
                                        : static_cast<const void *>(d.row_index_pos);
    const void *lists_neg = FORM == 2 ? static_cast<const void *>(d.row_index16_neg) : static_cast<const void *>(d.row_index_neg);
    hipLaunchKernelGGL((k_decode<MM, CHUNKED, FORM>), dim3(grid), dim3(kDecodeThreads), lds, stream, X, cs_pos, cs_neg,
                       lists_pos, lists_neg, b, act.alpha, act.alpha_stride, Y, t->K, t->N, kc, deal_lists);
    e = hipGetLastError();
    if (e == hipSuccess) e = c.record_after();
    return e;
}

template <int MM, int FORM>
hipError_t launch(const float *X, const tcsc *t, const float *b, float *Y, const Call &c)
{
    const int kc = t->K < chunk_rows<MM>() ? t->K : chunk_rows<MM>();
    const size_t lds = (size_t)(kc + 1) * MM * sizeof(float);
    if (t->K > kc)   // K in chunks: the 32-bit lists (the padded 16-bit ones are for X whole in the LDS)
        return launch_kernel<MM, true, FORM == 2 ? 0 : FORM>(X, t, b, Y, kc, lds, c);
    return launch_kernel<MM, false, FORM>(X, t, b, Y, kc, lds, c);
}

template <int FORM>
hipError_t launch_m(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c)
{
    switch (M) {
    case 1: return launch<1, FORM>(X, t, b, Y, c);
    case 2: return launch<2, FORM>(X, t, b, Y, c);
    case 3: return launch<3, FORM>(X, t, b, Y, c);
    case 4: return launch<4, FORM>(X, t, b, Y, c);
    case 5: return launch<5, FORM>(X, t, b, Y, c);
    case 6: return launch<6, FORM>(X, t, b, Y, c);
    case 7: return launch<7, FORM>(X, t, b, Y, c);
    case 8: return launch<8, FORM>(X, t, b, Y, c);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool decode_supported(int M) { return M <= 8; }

hipError_t launch_decode(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c)
{
    // the padded 16-bit copy of the lists, if the matrix has one (K <= 65535): half the bytes
    if (t->layout.has_lists16 && !c.decode_wide_lists) return launch_m<2>(X, t, b, Y, M, c);
    return launch_m<0>(X, t, b, Y, M, c);
}

hipError_t launch_decode_signed(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c)
{
    return launch_m<1>(X, t, b, Y, M, c);
}

}  // namespace tst
