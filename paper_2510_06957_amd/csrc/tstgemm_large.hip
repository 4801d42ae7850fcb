// Large-M kernel of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper) for gfx950.
//
// Arithmetic is that of BaseTCSC (Sec. 2): every output is a sum of gathered X entries
// (+1 list) minus a sum of gathered X entries (-1 list), bias added once at the end; no
// multiplications.  The mapping to the machine is this library's own:
//
//   * one lane owns R consecutive rows of X (R = 1, 2 or 4), a wavefront therefore owns a
//     tile of TM = 64 R rows, and walks the index lists of its columns with the index held
//     in a scalar register: one index serves all TM rows (the paper's "vertical" SIMD scheme
//     and its M-unrolling, Sec. 3, carried to 64 lanes);
//   * K is cut into blocks of 64 (the paper's blocking idea, Sec. 3 "Blocking"); the
//     workgroup keeps the X tile of the current block transposed in the LDS, tile[k][row], so
//     the gather of one index is a single conflict-free ds_read (b32/b64/b128) per lane;
//   * the next block's tile is fetched from global memory into registers while the current one
//     is consumed, and written to the second LDS buffer afterwards (one barrier per block);
//   * accumulators stay in VGPRs over all K-blocks; the bias add and the store are fused.
//
// Index lists come from the K-blocked stream written by the re-blocking pass: per column and
// K-block a +1 list and a -1 list in 8-slot chunks, fetched with 32-byte scalar loads.
#include "tstgemm_internal.h"

namespace tst {
namespace {

typedef int int8v __attribute__((ext_vector_type(8)));

template <int R> struct RowVec;
template <> struct RowVec<1> { typedef float type; };
template <> struct RowVec<2> { typedef float __attribute__((ext_vector_type(2))) type; };
template <> struct RowVec<4> { typedef float __attribute__((ext_vector_type(4))) type; };
typedef float float4v __attribute__((ext_vector_type(4)));

template <int R> __device__ __forceinline__ float lane_of(const typename RowVec<R>::type &v, int r)
{
    if constexpr (R == 1) return v; else return v[r];
}

// acc (+/-)= tile[idx][rows of this lane]
template <int R, bool NEG>
__device__ __forceinline__ void gather(typename RowVec<R>::type &acc, const char *tile_lane, int idx)
{
    typedef typename RowVec<R>::type V;
    const V v = *reinterpret_cast<const V *>(tile_lane + idx * (64 * R * 4));
    if constexpr (NEG) acc -= v; else acc += v;
}

// One list (n entries, stored in chunks of 8 slots at p; p and n are wave-uniform).
template <int R, bool NEG>
__device__ __forceinline__ void run_list(typename RowVec<R>::type &acc, const int32_t *__restrict__ p, int n,
                                         const char *tile_lane)
{
    while (n >= kChunk) {
        const int8v c = *reinterpret_cast<const int8v *>(p);
#pragma unroll
        for (int i = 0; i < kChunk; ++i) gather<R, NEG>(acc, tile_lane, c[i]);
        p += kChunk;
        n -= kChunk;
    }
    if (n > 0) {   // partial chunk: 4 entries in slots 0..3 if n&4, 2 in slots 4..5 if n&2, 1 in slot 6 if n&1
        const int8v c = *reinterpret_cast<const int8v *>(p);
        if (n & 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) gather<R, NEG>(acc, tile_lane, c[i]);
        }
        if (n & 2) {
            gather<R, NEG>(acc, tile_lane, c[4]);
            gather<R, NEG>(acc, tile_lane, c[5]);
        }
        if (n & 1) gather<R, NEG>(acc, tile_lane, c[6]);
    }
}

// R rows per lane, NW wavefronts per workgroup, NCW columns per wavefront.
template <int R, int NW, int NCW>
__global__ void __launch_bounds__(NW * 64)
k_large(const float *__restrict__ X, const int32_t *__restrict__ seg_count, const int64_t *__restrict__ col_ptr,
        const int32_t *__restrict__ stream, const float *__restrict__ b, float *__restrict__ Y, int M, int K, int N,
        int n_pad, int n_kblocks, int n_colgroups)
{
    typedef typename RowVec<R>::type V;
    constexpr int TM = 64 * R;            // rows of X per workgroup tile
    constexpr int RB = TM * 4;            // bytes of one tile row (one k, TM rows)
    constexpr int TILE = kKBlock * RB;    // bytes of one buffer
    constexpr int NT = NW * 64;
    constexpr int CPT = TM * (kKBlock / 4) / NT;   // 16-byte pieces of X each thread stages per K-block
    static_assert(CPT >= 1 && CPT * NT == TM * (kKBlock / 4), "staging must tile the block exactly");

    __shared__ __attribute__((aligned(16))) char lds[2 * TILE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cg = blockIdx.x % n_colgroups, mt = blockIdx.x / n_colgroups;
    const int m0 = mt * TM;
    const int c0 = (cg * NW + wave) * NCW;   // < n_pad by construction of the grid

    // ---- staging role of this thread: row `srow` of the tile, k-segment `sseg`
    const int srow = threadIdx.x % TM, sseg = threadIdx.x / TM;
    const int gm = m0 + srow;
    const float *xrow = X + (size_t)(gm < M ? gm : 0) * K;
    const bool vec_ok = (K % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    float4v st[CPT];

    auto stage_load = [&](int kb) {
        const int k0 = kb * kKBlock + sseg * (4 * CPT);
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int k = k0 + 4 * i;
            float4v v = {0.f, 0.f, 0.f, 0.f};
            if (gm < M) {
                if (vec_ok && k + 4 <= K) {
                    v = *reinterpret_cast<const float4v *>(xrow + k);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (k + j < K) v[j] = xrow[k + j];
                }
            }
            st[i] = v;
        }
    };
    auto stage_store = [&](int buf) {
        char *base = lds + buf * TILE + (sseg * (4 * CPT)) * RB + srow * 4;
#pragma unroll
        for (int i = 0; i < CPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<float *>(base + (4 * i + j) * RB) = st[i][j];
    };

    // ---- compute role: columns c0 .. c0+NCW-1, rows m0 + R*lane .. + R-1
    V acc[NCW];
    const int32_t *sp[NCW];
#pragma unroll
    for (int j = 0; j < NCW; ++j) {
        if constexpr (R == 1) acc[j] = 0.f; else acc[j] = V(0.f);
        sp[j] = stream + col_ptr[c0 + j];
    }

    stage_load(0);
    stage_store(0);
    __syncthreads();

    for (int kb = 0; kb < n_kblocks; ++kb) {
        const bool more = kb + 1 < n_kblocks;
        if (more) stage_load(kb + 1);
        const char *tile_lane = lds + (kb & 1) * TILE + lane * (R * 4);
        const int32_t *cnt = seg_count + (size_t)kb * n_pad + c0;
#pragma unroll
        for (int j = 0; j < NCW; ++j) {
            const int c = cnt[j];
            const int np = c & 0xffff, nn = (c >> 16) & 0xffff;
            run_list<R, false>(acc[j], sp[j], np, tile_lane);
            sp[j] += (np + kChunk - 1) & ~(kChunk - 1);
            run_list<R, true>(acc[j], sp[j], nn, tile_lane);
            sp[j] += (nn + kChunk - 1) & ~(kChunk - 1);
        }
        if (more) stage_store((kb + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: Y = acc + b, bias added once, last
    float bias[NCW];
#pragma unroll
    for (int j = 0; j < NCW; ++j) bias[j] = (b != nullptr && c0 + j < N) ? b[c0 + j] : 0.f;
    const bool store_vec = NCW == 4 && (N % 4 == 0) && (c0 + 4 <= N) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int m = m0 + lane * R + r;
        if (m >= M) continue;
        float *yrow = Y + (size_t)m * N + c0;
        if constexpr (NCW == 4) {
            if (store_vec) {
                float4v o;
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = lane_of<R>(acc[j], r) + bias[j];
                *reinterpret_cast<float4v *>(yrow) = o;
                continue;
            }
        }
#pragma unroll
        for (int j = 0; j < NCW; ++j)
            if (c0 + j < N) yrow[j] = lane_of<R>(acc[j], r) + bias[j];
    }
}

template <int R, int NW, int NCW>
hipError_t launch(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    constexpr int TM = 64 * R;
    const int n_colgroups = l.n_pad / (NW * NCW);
    const int m_tiles = (M + TM - 1) / TM;
    const long long grid = (long long)n_colgroups * m_tiles;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_large<R, NW, NCW>), dim3((unsigned)grid), dim3(NW * 64), 0, stream, X, d.seg_count, d.col_ptr,
                       d.stream, b, Y, M, l.K, l.N, l.n_pad, l.n_kblocks, n_colgroups);
    return hipGetLastError();
}

// Columns per wavefront: as many as still leave about two workgroups per compute unit.
template <int R> hipError_t pick(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream)
{
    constexpr int NW = 16;
    const long long m_tiles = (M + 64 * R - 1) / (64 * R);
    const long long target = 512;
    if (m_tiles * (t->layout.n_pad / (NW * 4)) >= target) return launch<R, NW, 4>(X, t, b, Y, M, stream);
    if (m_tiles * (t->layout.n_pad / (NW * 2)) >= target) return launch<R, NW, 2>(X, t, b, Y, M, stream);
    return launch<R, NW, 1>(X, t, b, Y, M, stream);
}

}  // namespace

hipError_t launch_large(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream)
{
    if (M <= 64) return pick<1>(X, t, b, Y, M, stream);
    if (M <= 128) return pick<2>(X, t, b, Y, M, stream);
    return pick<4>(X, t, b, Y, M, stream);
}

}  // namespace tst
