// Large-M kernel of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper) for gfx950.
//
// Arithmetic is that of BaseTCSC (Sec. 2): every output is a sum of gathered X entries
// (+1 list) minus a sum of gathered X entries (-1 list), bias added once at the end; no
// multiplications.  The mapping to the machine is this library's own:
//
//   * one lane owns R consecutive rows of X (R = 1, 2 or 4), a wavefront therefore owns a
//     tile of TM = 64 R rows, and walks the index lists of its columns with a wave-uniform
//     index: one index serves all TM rows (the paper's "vertical" SIMD scheme and its
//     M-unrolling, Sec. 3, carried to 64 lanes);
//   * K is cut into blocks of 64 (the paper's blocking idea, Sec. 3 "Blocking"); the
//     workgroup keeps the X tile of the current block transposed in the LDS, tile[k][row], so
//     the gather of one index is a single conflict-free ds_read (b32/b64/b128) per lane;
//   * gathers are issued eight at a time and added after one wait; the latency of a group is
//     covered by the other wavefronts (the kernel is built for 8 wavefronts per SIMD: at most
//     64 VGPRs, two workgroups of 16 wavefronts per compute unit);
//   * a list piece (one column, one K-block, one sign) arrives as a 64-bit row set; the scalar
//     unit turns it into row numbers with find-first-set / clear-bit, so an index costs two
//     SALU instructions and neither VALU work, LDS traffic nor memory latency.  The sets of
//     a wavefront's columns for the next K-block are fetched one K-block ahead with one vector
//     load and moved to scalar registers with a few v_readlane at the block border;
//   * the X tile itself is not prefetched: two workgroups share a compute unit, one computes
//     while the other exchanges its tile between two barriers;
//   * accumulators stay in VGPRs over all K-blocks of the workgroup's K slice; the bias add and
//     the store are fused;
//   * when rows x columns alone give too few workgroups to fill the chip, K is cut into up to
//     8 slices handled by different workgroups; each writes its partial sums to the workspace,
//     and the workgroup that arrives last adds the slices in slice order, adds the bias and
//     stores Y -- a fixed summation order, so results do not depend on timing.
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

// A stage of the kernel covers half a K-block: 32 rows of W, one 32-bit half of a 64-bit row set.
constexpr int kStageRows = kKBlock / 2;

// Smallest member of a non-empty row set, removed from the set: two SALU instructions (find-first-set, clear bit).
__device__ __forceinline__ int pop_lowest(uint32_t &set)
{
    const int k = __builtin_ctz(set);
    asm("s_bitset0_b32 %0, %1" : "+s"(set) : "s"(k));
    return k;
}

// LDS layout of an X tile: tile row k (one column of X, TM = 64 R consecutive rows of X) starts at k * stride,
// stride = 4 TM + 16 bytes.  The 16 bytes of padding rotate the banks by four from one tile row to the next, so
// that the transposing writes of the staging (lanes that differ in k and in the X row) hit 64 different banks,
// while a gather (all lanes the same k, consecutive X rows) stays contiguous and 16-byte aligned.
template <int R> constexpr int tile_stride() { return 256 * R + 16; }

// This lane's R rows of tile row k: address = k * stride + lane_base in one VALU instruction (k is wave-uniform).
template <int R>
__device__ __forceinline__ typename RowVec<R>::type tile_row(const char *tile, int lane_base, int stride_vgpr, int k)
{
    int off;
    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(off) : "s"(k), "v"(stride_vgpr), "v"(lane_base));
    return *reinterpret_cast<const typename RowVec<R>::type *>(tile + off);
}

// What a gather needs besides the row number: the tile, this lane's byte offset inside a tile row (plus the offset of
// the buffer in use), and the row stride held in a VGPR (the multiply-add takes only one scalar operand).
struct TileView {
    const char *tile;
    int lane_base;
    int stride_vgpr;
};

// acc (+/-)= tile[k][rows of this lane] for the COUNT smallest members k of `set` (removed from it; the set has at
// least COUNT members).  All gathers are issued before the first addition, so COUNT LDS reads are in flight at once;
// with 8 wavefronts per SIMD the other wavefronts keep the LDS busy while this one adds.
template <int R, bool NEG, int COUNT>
__device__ __forceinline__ void gather(typename RowVec<R>::type &acc, const TileView &t, uint32_t &set)
{
    typedef typename RowVec<R>::type V;
    V v[COUNT];
#pragma unroll
    for (int i = 0; i < COUNT; ++i) v[i] = tile_row<R>(t.tile, t.lane_base, t.stride_vgpr, pop_lowest(set));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < COUNT; ++i) {
        if constexpr (NEG) acc -= v[i]; else acc += v[i];
    }
}

// One list: every member of the row set is gathered and added to (NEG: subtracted from) acc, in ascending row order,
// in groups of 8 and a remainder of 4 + 2 + 1.  The set is wave-uniform.
template <int R, bool NEG>
__device__ __forceinline__ void run_list(typename RowVec<R>::type &acc, uint32_t set, const TileView &t)
{
    int n = __builtin_popcount(set);
    while (n >= 8) {
        gather<R, NEG, 8>(acc, t, set);
        n -= 8;
    }
    if (n & 4) gather<R, NEG, 4>(acc, t, set);
    if (n & 2) gather<R, NEG, 2>(acc, t, set);
    if (n & 1) gather<R, NEG, 1>(acc, t, set);
}

struct LargeArgs {
    const float *X;
    const unsigned long long *masks;
    const float *b;
    float *Y;
    float *partials;
    int32_t *counters;
    int M, K, N, n_pad, n_kblocks, n_colgroups, k_slices, kb_per_slice;
    int wg_slots;   // workgroups of one dispatch round: blocks i and i + wg_slots tend to share a compute unit
};

// R rows per lane, NCW columns per wavefront; VEC: X rows are 16-byte aligned and K is a multiple of 4, so X is
// staged with 16-byte loads (otherwise element by element).
template <int R, int NCW, bool VEC>
__global__ void __launch_bounds__(NW * 64, 8) k_large(const LargeArgs a)
{
    typedef typename RowVec<R>::type V;
    constexpr int TM = 64 * R;            // rows of X per workgroup tile
    constexpr int RB = tile_stride<R>();         // bytes from one tile row (one k, TM rows) to the next
    constexpr int TILE = kStageRows * RB;        // bytes of one buffer
    constexpr int NT = NW * 64;
    constexpr int PIECES = kStageRows / 4;       // 16-byte pieces of an X row per stage
    constexpr int ROWS_PER_PASS = NT / PIECES;   // X rows the workgroup fetches with one load per thread
    constexpr int CPT = (TM + ROWS_PER_PASS - 1) / ROWS_PER_PASS;   // loads per thread and stage
    __shared__ __attribute__((aligned(16))) char lds[2 * TILE];
    __shared__ int last_flag;

    const float *__restrict__ X = a.X;
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

    // ---- staging role of this thread.  A stage needs 32 consecutive floats (8 pieces of 16 bytes) of every X row
    // of the tile.  Four neighbouring lanes fetch 64 contiguous bytes of one row, so a wavefront load touches 16
    // rows; thread t owns piece (t & 3) + 4 * ((t >> 2) / ROWS...) -- in short: row srow + i * ROWS_PER_PASS, piece
    // spiece, for i < CPT.
    const int spiece = (threadIdx.x & 3) + 4 * ((threadIdx.x >> 2) / ROWS_PER_PASS % (PIECES / 4));
    const int srow = (threadIdx.x >> 2) % ROWS_PER_PASS + ROWS_PER_PASS * ((threadIdx.x >> 2) / ROWS_PER_PASS / (PIECES / 4));
    static_assert(PIECES == 8 && NT % PIECES == 0, "staging layout");
    float4v st[CPT];

    // Loads are issued unconditionally (out-of-range rows and columns read a clamped, valid address and are zeroed
    // afterwards): the wait counters then know exactly how many loads are in flight behind a given one.
    // Byte offsets of this thread's X rows from the first row of the tile, as 32-bit values next to a wave-uniform
    // 64-bit base (rows beyond M point at the last valid row and are zeroed after the load).
    const char *xtile = reinterpret_cast<const char *>(X + (size_t)m0 * K);
    uint32_t xoff[CPT];
    bool xok[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int row = srow + i * (NT / 4 / (PIECES / 4));
        xok[i] = row < TM && m0 + row < M;
        xoff[i] = (uint32_t)(min(row, M - 1 - m0)) * (uint32_t)K * 4u;
    }
    auto stage_load = [&](int stage) {
        const int k = stage * kStageRows + 4 * spiece;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            float4v v;
            if constexpr (VEC) {
                const bool ok = xok[i] && k < K;   // K % 4 == 0: a piece is inside or outside as a whole
                v = *reinterpret_cast<const float4v *>(xtile + (xoff[i] + (uint32_t)(k < K ? k : 0) * 4u));
                if (!ok) v = float4v{0.f, 0.f, 0.f, 0.f};
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float x = *reinterpret_cast<const float *>(xtile + (xoff[i] + (uint32_t)(k + j < K ? k + j : 0) * 4u));
                    v[j] = (xok[i] && k + j < K) ? x : 0.f;
                }
            }
            st[i] = v;
        }
    };
    auto stage_store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int row = srow + i * (NT / 4 / (PIECES / 4));
            if (row < TM) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<float *>(lds + buf * TILE + (4 * spiece + j) * RB + row * 4) = st[i][j];
            }
        }
    };

    // ---- compute role: columns c0 .. c0+NCW-1, rows m0 + R*lane .. + R-1
    V acc[NCW];
#pragma unroll
    for (int j = 0; j < NCW; ++j) acc[j] = zero_vec<R>();

    if (kb0 < kb1) {
        // Row sets of (kb, c0 .. c0+NCW-1): 4*NCW consecutive dwords (column j: +1 set low/high half, -1 set low/high
        // half), fetched by lanes 0 .. 4*NCW-1 of one vector load a K-block ahead.  A scalar load would share its
        // wait counter with the LDS reads.
        const uint32_t *set_words = reinterpret_cast<const uint32_t *>(a.masks) + (size_t)c0 * 4 + (lane & (4 * NCW - 1));
        auto load_sets = [&](int kb) { return (int)set_words[(size_t)kb * n_pad * 4]; };
        int sets_ahead = load_sets(kb0);   // the sets of the block the NEXT stage works on (here: of the first stage)
        TileView view;
        view.tile = lds;
        view.stride_vgpr = RB;
        const int lane_base = lane * (R * 4);
        const int wg_parity = (blockIdx.x / a.wg_slots) & 1;

        // Stages: two per K-block (its low and its high 32 rows), double-buffered in the LDS.  While a stage is
        // computed the X tile of the next one sits in registers (requested at the start of the stage) and is written
        // to the other buffer at the end; one barrier per stage.
        const int s0 = 2 * kb0, s1 = 2 * kb1;
        stage_load(s0);
        stage_store(0);
        __syncthreads();
        for (int stage = s0; stage < s1; ++stage) {
            const int half = stage & 1;
            // The two workgroups that share a compute unit take turns in issue priority, stage by stage: the
            // hardware would otherwise always prefer the older one, which then finishes long before the other.
            if ((((stage - s0) >> 1) + wg_parity) & 1) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
            // Every stage issues the same three requests in the same order (tile of the next stage, row sets of the
            // next stage's block -- the same block again after a low half), without branches around them, so that
            // the wait counters can tell the sets of this stage have arrived without waiting for the new requests.
            const int sets_cur = sets_ahead;
            const int next_stage = stage + 1 < s1 ? stage + 1 : stage;   // behind the last stage: repeated, not used
            stage_load(next_stage);
            sets_ahead = load_sets(next_stage >> 1);
            view.lane_base = lane_base + ((stage - s0) & 1) * TILE;
#pragma unroll
            for (int j = 0; j < NCW; ++j) {
                const uint32_t pos = (uint32_t)__builtin_amdgcn_readlane(sets_cur, 4 * j + half);
                const uint32_t neg = (uint32_t)__builtin_amdgcn_readlane(sets_cur, 4 * j + 2 + half);
                run_list<R, false>(acc[j], pos, view);
                run_list<R, true>(acc[j], neg, view);
            }
            if (stage + 1 < s1) stage_store(((stage - s0) & 1) ^ 1);
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
        // All slices of a column are requested before the first addition (one memory round trip instead of
        // k_slices); the additions then run in slice order.
        constexpr int kMaxSlices = 8;
#pragma unroll
        for (int j = 0; j < NCW; ++j) {
            V part[kMaxSlices];
#pragma unroll
            for (int s = 0; s < kMaxSlices; ++s)
                part[s] = *reinterpret_cast<const V *>(gbase + (size_t)(s < a.k_slices ? s : 0) * kSliceFloats +
                                                       (size_t)j * TM);
            V sum = zero_vec<R>();
#pragma unroll
            for (int s = 0; s < kMaxSlices; ++s)
                if (s < a.k_slices) sum += part[s];
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
    a.X = X; a.masks = d.masks; a.b = b; a.Y = Y;
    a.partials = d.partials; a.counters = d.counters;
    a.M = M; a.K = l.K; a.N = l.N; a.n_pad = l.n_pad; a.n_kblocks = l.n_kblocks;
    a.n_colgroups = l.n_pad / (NW * NCW);
    const long long m_tiles = (M + TM - 1) / TM;
    const long long groups = m_tiles * a.n_colgroups;
    if (k_slices > 1 && groups * k_slices > kMaxSplitGroups) k_slices = (int)(kMaxSplitGroups / groups);
    if (k_slices < 1) k_slices = 1;
    a.k_slices = k_slices;
    a.kb_per_slice = (l.n_kblocks + k_slices - 1) / k_slices;
    a.wg_slots = compute_units();
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
        const int slots = 2 * compute_units();   // two workgroups per compute unit
        k_slices = groups >= slots ? 1 : (int)((slots + groups - 1) / groups);
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
