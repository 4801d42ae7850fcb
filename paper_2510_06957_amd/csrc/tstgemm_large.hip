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
//   * accumulators stay in VGPRs over all K-blocks of the workgroup's K slice; the bias add and
//     the store are fused;
//   * when rows x columns alone give too few workgroups to fill the chip, K is cut into up to
//     8 slices handled by different workgroups; each writes its partial sums to the workspace,
//     and the workgroup that arrives last adds the slices in slice order, adds the bias and
//     stores Y -- a fixed summation order, so results do not depend on timing.
//
// Index lists come from the K-blocked stream written by the re-blocking pass: per K-block and
// column a +1 list and a -1 list in 8-slot chunks.  The lists of a wavefront's columns are
// contiguous, so the wavefront fetches them as one 1 KiB window (16 bytes per lane, one vector
// load) a whole K-block ahead and then broadcasts one index at a time out of the window into a
// scalar register (v_readlane): no memory latency sits between two gathers.  The list lengths
// and the window position travel the same way, two K-blocks ahead.
#include "tstgemm_internal.h"

namespace tst {

int g_cols_per_wave = 0, g_k_slices = 0;

namespace {

constexpr int NW = 16;   // wavefronts per workgroup
typedef int int4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

template <int R> struct RowVec;
template <> struct RowVec<1> { typedef float type; };
template <> struct RowVec<2> { typedef float __attribute__((ext_vector_type(2))) type; };
template <> struct RowVec<4> { typedef float __attribute__((ext_vector_type(4))) type; };

template <int R> __device__ __forceinline__ float lane_of(const typename RowVec<R>::type &v, int r)
{
    if constexpr (R == 1) return v; else return v[r];
}
template <int R> __device__ __forceinline__ typename RowVec<R>::type zero_vec()
{
    if constexpr (R == 1) return 0.f; else return typename RowVec<R>::type(0.f);
}

// acc (+/-)= tile[idx[i]][rows of this lane], i < COUNT.  All gathers are issued before the first addition so that
// COUNT LDS reads are in flight at once.
template <int R, bool NEG, int COUNT>
__device__ __forceinline__ void gather(typename RowVec<R>::type &acc, const char *tile_lane, const int (&idx)[COUNT])
{
    typedef typename RowVec<R>::type V;
    V v[COUNT];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < COUNT; ++i) v[i] = *reinterpret_cast<const V *>(tile_lane + idx[i] * (64 * R * 4));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < COUNT; ++i) {
        if constexpr (NEG) acc -= v[i]; else acc += v[i];
    }
}

constexpr int kWindowChunks = 32;                       // chunks per window: 64 lanes x 4 slots

// The 1 KiB of index stream starting at wp, four consecutive slots per lane.
__device__ __forceinline__ int4v load_window(const int32_t *wp, int lane)
{
    return *reinterpret_cast<const int4v *>(wp + 4 * lane);
}

// The eight slots of chunk cc of the window: slots 0..3 sit in lane 2*cc, slots 4..7 in lane 2*cc+1.  Chunks behind
// the window (a wavefront whose lists of one K-block exceed 1 KiB: rare) are read straight from the stream with a
// scalar load.  cc and wp are wave-uniform.
__device__ __forceinline__ void chunk_slots(int (&idx)[kChunk], const int4v &win, const int32_t *__restrict__ wp, int cc)
{
    if (__builtin_expect(cc < kWindowChunks, 1)) {
        const int l0 = 2 * cc, l1 = l0 + 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            idx[i] = __builtin_amdgcn_readlane(win[i], l0);
            idx[4 + i] = __builtin_amdgcn_readlane(win[i], l1);
        }
    } else {
        const int32_t *p = wp + (size_t)cc * kChunk;
#pragma unroll
        for (int i = 0; i < kChunk; ++i) idx[i] = p[i];
    }
}

// One list of n entries starting at chunk `cc` of the window `win` (which starts at wp in the stream); on return cc
// is the chunk behind the list.  n and cc are wave-uniform.
template <int R, bool NEG>
__device__ __forceinline__ void run_list(typename RowVec<R>::type &acc, int n, int &cc, const int4v &win,
                                         const int32_t *__restrict__ wp, const char *tile_lane)
{
    while (n >= kChunk) {
        int idx[kChunk];
        chunk_slots(idx, win, wp, cc);
        gather<R, NEG, kChunk>(acc, tile_lane, idx);
        n -= kChunk;
        ++cc;
    }
    if (n > 0) {   // partial chunk: 4 entries in slots 0..3 if n&4, 2 in slots 4..5 if n&2, 1 in slot 6 if n&1
        int idx[kChunk];
        chunk_slots(idx, win, wp, cc);
        if (n & 4) {
            const int four[4] = {idx[0], idx[1], idx[2], idx[3]};
            gather<R, NEG, 4>(acc, tile_lane, four);
        }
        if (n & 2) {
            const int two[2] = {idx[4], idx[5]};
            gather<R, NEG, 2>(acc, tile_lane, two);
        }
        if (n & 1) {
            const int one[1] = {idx[6]};
            gather<R, NEG, 1>(acc, tile_lane, one);
        }
        ++cc;
    }
}

struct LargeArgs {
    const float *X;
    const int32_t *seg_count;
    const uint32_t *seg_ptr;
    const int32_t *stream;
    const float *b;
    float *Y;
    float *partials;
    int32_t *counters;
    int M, K, N, n_pad, n_kblocks, n_colgroups, k_slices, kb_per_slice;
};

// R rows per lane, NCW columns per wavefront; VEC: X rows are 16-byte aligned and K is a multiple of 4, so X is
// staged with 16-byte loads (otherwise element by element).
template <int R, int NCW, bool VEC>
__global__ void __launch_bounds__(NW * 64) k_large(const LargeArgs a)
{
    typedef typename RowVec<R>::type V;
    constexpr int TM = 64 * R;            // rows of X per workgroup tile
    constexpr int RB = TM * 4;            // bytes of one tile row (one k, TM rows)
    constexpr int TILE = kKBlock * RB;    // bytes of one buffer
    constexpr int NT = NW * 64;
    constexpr int CPT = TM * (kKBlock / 4) / NT;   // 16-byte pieces of X each thread stages per K-block
    static_assert(CPT >= 1 && CPT * NT == TM * (kKBlock / 4), "staging must tile the block exactly");

    __shared__ __attribute__((aligned(16))) char lds[2 * TILE];
    __shared__ int last_flag;

    const float *__restrict__ X = a.X;
    const int32_t *__restrict__ stream = a.stream;
    const int M = a.M, K = a.K, N = a.N, n_pad = a.n_pad;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cg = blockIdx.x % a.n_colgroups;
    const int rest = blockIdx.x / a.n_colgroups;
    const int slice = rest % a.k_slices, mt = rest / a.k_slices;
    const int m0 = mt * TM;
    const int c0 = (cg * NW + wave) * NCW;   // < n_pad by construction of the grid
    const int kb0 = min(slice * a.kb_per_slice, a.n_kblocks);
    const int kb1 = min(kb0 + a.kb_per_slice, a.n_kblocks);

    // ---- staging role of this thread: row `srow` of the tile, k-segment `sseg`
    const int srow = threadIdx.x % TM, sseg = threadIdx.x / TM;
    const int gm = m0 + srow;
    const bool row_ok = gm < M;
    const float *xrow = X + (size_t)(row_ok ? gm : M - 1) * K;
    float4v st[CPT];

    // All loads are issued unconditionally (out-of-range rows and columns read a clamped, valid address and are
    // zeroed afterwards): the wait counters then know exactly how many loads are in flight behind a given one.
    auto stage_load = [&](int kb) {
        const int k0 = kb * kKBlock + sseg * (4 * CPT);
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int k = k0 + 4 * i;
            float4v v;
            if constexpr (VEC) {
                const bool ok = row_ok && k < K;   // K % 4 == 0: a piece is inside or outside as a whole
                v = *reinterpret_cast<const float4v *>(xrow + (k < K ? k : 0));
                if (!ok) v = float4v{0.f, 0.f, 0.f, 0.f};
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float x = xrow[k + j < K ? k + j : 0];
                    v[j] = (row_ok && k + j < K) ? x : 0.f;
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
#pragma unroll
    for (int j = 0; j < NCW; ++j) acc[j] = zero_vec<R>();

    if (kb0 < kb1) {
        // List lengths and window position of (kb, c0 .. c0+NCW-1) come through ONE vector load: lane j < NCW reads
        // the packed counts of column c0+j, lane NCW the position of the first chunk (the pattern repeats every
        // 2*NCW lanes).  A scalar load would share its wait counter with the LDS gathers.
        const int32_t *meta_base = (lane & NCW) ? reinterpret_cast<const int32_t *>(a.seg_ptr) + c0
                                                : a.seg_count + c0 + (lane & (NCW - 1));
        auto load_meta = [&](int kb) { return meta_base[(size_t)kb * n_pad]; };
        auto clamp_kb = [&](int kb) { return kb < kb1 ? kb : kb1 - 1; };
        int meta = load_meta(kb0);
        stage_load(kb0);
        int cnt[NCW];
#pragma unroll
        for (int j = 0; j < NCW; ++j) cnt[j] = __builtin_amdgcn_readlane(meta, j);
        const int32_t *__restrict__ wp = stream + (size_t)(uint32_t)__builtin_amdgcn_readlane(meta, NCW) * kChunk;
        int4v win = load_window(wp, lane);
        meta = load_meta(clamp_kb(kb0 + 1));
        stage_store(0);
        __syncthreads();

        for (int kb = kb0; kb < kb1; ++kb) {
            // requests for the next K-block (tile, window) and the one after it (list lengths, window position);
            // behind the last block they repeat the last one and are not used
            const bool more = kb + 1 < kb1;
            stage_load(clamp_kb(kb + 1));
            int cnt_next[NCW];
#pragma unroll
            for (int j = 0; j < NCW; ++j) cnt_next[j] = __builtin_amdgcn_readlane(meta, j);
            const int32_t *__restrict__ wp_next =
                stream + (size_t)(uint32_t)__builtin_amdgcn_readlane(meta, NCW) * kChunk;
            const int4v win_next = load_window(wp_next, lane);
            meta = load_meta(clamp_kb(kb + 2));

            const char *tile_lane = lds + ((kb - kb0) & 1) * TILE + lane * (R * 4);
            int cc = 0;
#pragma unroll
            for (int j = 0; j < NCW; ++j) {
                run_list<R, false>(acc[j], cnt[j] & 0xffff, cc, win, wp, tile_lane);
                run_list<R, true>(acc[j], (cnt[j] >> 16) & 0xffff, cc, win, wp, tile_lane);
            }
            wp = wp_next;
            win = win_next;
#pragma unroll
            for (int j = 0; j < NCW; ++j) cnt[j] = cnt_next[j];
            if (more) stage_store((kb + 1 - kb0) & 1);
            __syncthreads();
        }
    }

    // ---- split K: publish this slice's partial sums; the last workgroup of the group sums all slices in order
    if (a.k_slices > 1) {
        const int group = mt * a.n_colgroups + cg;
        constexpr size_t kSliceFloats = (size_t)NW * NCW * TM;
        float *gbase = a.partials + (size_t)group * a.k_slices * kSliceFloats + (size_t)(wave * NCW) * TM + lane * R;
#pragma unroll
        for (int j = 0; j < NCW; ++j)
            *reinterpret_cast<V *>(gbase + (size_t)slice * kSliceFloats + (size_t)j * TM) = acc[j];
        // Release / acquire through one thread: the barrier orders the workgroup's stores before thread 0's
        // device-scope fence, and thread 0's fence after the counter update before the workgroup's loads.
        __syncthreads();
        if (threadIdx.x == 0) {
            __threadfence();
            const int arrived = atomicAdd(&a.counters[group], 1);
            const int last = arrived == a.k_slices - 1;
            if (last) {
                a.counters[group] = 0;   // ready for the next call
                __threadfence();
            }
            last_flag = last;
        }
        __syncthreads();
        if (!last_flag) return;
#pragma unroll
        for (int j = 0; j < NCW; ++j) {
            V sum = zero_vec<R>();
            for (int s = 0; s < a.k_slices; ++s)
                sum += *reinterpret_cast<const V *>(gbase + (size_t)s * kSliceFloats + (size_t)j * TM);
            acc[j] = sum;
        }
    }

    // ---- epilogue: Y = acc + b, bias added once, last
    float bias[NCW];
#pragma unroll
    for (int j = 0; j < NCW; ++j) bias[j] = (a.b != nullptr && c0 + j < N) ? a.b[c0 + j] : 0.f;
    const bool store_vec =
        NCW == 4 && (N % 4 == 0) && (c0 + 4 <= N) && ((reinterpret_cast<uintptr_t>(a.Y) & 15) == 0);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int m = m0 + lane * R + r;
        if (m >= M) continue;
        float *yrow = a.Y + (size_t)m * N + c0;
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

template <int R, int NCW>
hipError_t launch(const float *X, const tcsc *t, const float *b, float *Y, int M, int k_slices, hipStream_t stream)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    constexpr int TM = 64 * R;
    LargeArgs a;
    a.X = X; a.seg_count = d.seg_count; a.seg_ptr = d.seg_ptr; a.stream = d.stream; a.b = b; a.Y = Y;
    a.partials = d.partials; a.counters = d.counters;
    a.M = M; a.K = l.K; a.N = l.N; a.n_pad = l.n_pad; a.n_kblocks = l.n_kblocks;
    a.n_colgroups = l.n_pad / (NW * NCW);
    const long long m_tiles = (M + TM - 1) / TM;
    const long long groups = m_tiles * a.n_colgroups;
    if (k_slices > 1 && groups * k_slices > kMaxSplitGroups) k_slices = (int)(kMaxSplitGroups / groups);
    if (k_slices < 1) k_slices = 1;
    a.k_slices = k_slices;
    a.kb_per_slice = (l.n_kblocks + k_slices - 1) / k_slices;
    const long long grid = groups * k_slices;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool vec = (l.K % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    if (vec)
        hipLaunchKernelGGL((k_large<R, NCW, true>), dim3((unsigned)grid), dim3(NW * 64), 0, stream, a);
    else
        hipLaunchKernelGGL((k_large<R, NCW, false>), dim3((unsigned)grid), dim3(NW * 64), 0, stream, a);
    return hipGetLastError();
}

// Launch shape: 4 columns per wavefront (64 per workgroup); K is sliced only when rows x columns alone leave
// compute units idle, into as few slices as fill them.
template <int R> hipError_t pick(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream)
{
    const tcsc_layout_t &l = t->layout;
    const int ncw = g_cols_per_wave ? g_cols_per_wave : 4;
    const long long m_tiles = (M + 64 * R - 1) / (64 * R);
    const long long groups = m_tiles * (l.n_pad / (NW * ncw));
    int k_slices = g_k_slices;
    if (k_slices == 0) {
        const int cus = compute_units();
        k_slices = groups >= cus ? 1 : (int)((cus + groups - 1) / groups);
        if (k_slices > 8) k_slices = 8;
    }
    if (k_slices > l.n_kblocks) k_slices = l.n_kblocks;
    switch (ncw) {
    case 1: return launch<R, 1>(X, t, b, Y, M, k_slices, stream);
    case 2: return launch<R, 2>(X, t, b, Y, M, k_slices, stream);
    default: return launch<R, 4>(X, t, b, Y, M, k_slices, stream);
    }
}

}  // namespace

hipError_t launch_large(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream)
{
    if (M <= 64) return pick<1>(X, t, b, Y, M, stream);
    if (M <= 128) return pick<2>(X, t, b, Y, M, stream);
    return pick<4>(X, t, b, Y, M, stream);
}

}  // namespace tst
