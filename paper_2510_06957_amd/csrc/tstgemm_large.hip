// Large-M kernel (M > 64) of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper) for gfx950.
//
// Arithmetic is that of BaseTCSC (Sec. 2): every output is a sum of gathered X entries
// (+1 list) minus a sum of gathered X entries (-1 list), bias added once at the end; no
// multiplications.  The mapping to the machine is this library's own:
//
//   * a pre-pass (k_pack_x, tstgemm_side.hip) copies X into the workspace as row tiles, transposed:
//     xt[tile][k][row], a tile being TM = 64 R consecutive rows of X (R = 2 or 4), K padded to whole
//     K-blocks, rows beyond M and entries beyond K zero.  A K-block of a tile (64 x TM floats) is then one
//     contiguous piece of memory that goes into the LDS with plain 16-byte copies, and the
//     strided walk over the rows of X happens once per call instead of once per workgroup;
//   * in k_large one lane owns R consecutive rows of X, a wavefront therefore owns a whole tile,
//     and walks the index lists of its NCW columns with a wave-uniform index: one index serves
//     all TM rows (the paper's "vertical" SIMD scheme and its M-unrolling, Sec. 3, carried to
//     64 lanes); the gather of one index is a single conflict-free ds_read (b32/b64/b128);
//   * K is cut into blocks of 64 (the paper's blocking idea, Sec. 3 "Blocking"); a workgroup
//     (16 wavefronts = 16 NCW columns) keeps one K-block of its tile in the LDS;
//   * a list piece (one column, one K-block, one sign) arrives as a 64-bit row set, fetched by
//     the scalar unit; the scalar unit turns it into row numbers with find-first-set /
//     clear-bit, so an index costs two SALU instructions and neither VALU work, LDS traffic nor
//     memory latency.  A piece is walked in groups of 8 gathers (4 in the shape with 8 columns per
//     wavefront) and then groups of 4, 2 and 1 for what is left: nothing but members of the list is
//     gathered (the paper pads its interleaved groups with a dummy zero index, Sec. 3; here a
//     padded gather costs as many vector instructions as a real one, and those are what the kernel
//     is bound by);
//   * the gathers of a group are all issued before the first addition, at a raised wavefront
//     priority; the latency of a group is covered by the other wavefronts: the kernel is built for
//     8 wavefronts per SIMD (at most 64 VGPRs, two workgroups per compute unit).  While one
//     workgroup exchanges its tile between two barriers, the other one computes;
//   * accumulators stay in VGPRs over all K-blocks of the workgroup's K slice; the bias add and
//     the store are fused;
//   * when rows x columns alone give too few workgroups to fill the chip, K is cut into up to
//     8 slices handled by different workgroups; each writes its partial sums to the workspace,
//     past the caches, and k_reduce (tstgemm_side.hip) adds the slices in slice order, adds the bias and stores Y
//     -- a fixed summation order, so results do not depend on timing, and no atomics or fences.
#include "tstgemm_internal.h"

namespace tst {

namespace {

constexpr int NW = 16;        // wavefronts per workgroup
constexpr int NT = NW * 64;   // threads per workgroup
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;
typedef const __attribute__((address_space(4))) u64 *const_u64_ptr;   // read through the scalar cache

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

// A tile row (one k, TM = 64 R rows of X) is 256 R bytes: 2^(8 + log2 R).
template <int R> constexpr int row_shift() { return R == 4 ? 10 : R == 2 ? 9 : 8; }

__device__ __forceinline__ int members(u64 set)
{
    int n;
    asm("s_bcnt1_i32_b64 %0, %1" : "=s"(n) : "s"(set) : "scc");
    return n;
}

// The read phase of a group: COUNT times { k = smallest member of `set`, removed from the set (find-first-set and
// clear-bit on the scalar unit); address = (k << row_shift) + lane_base (one VALU instruction); ds_read of this lane's R
// rows of tile row k }.  lane_base is the LDS address of this lane's part of tile row 0.  One asm statement, so that
// nothing is scheduled or inserted between the instructions; the address register is reused (an LDS instruction takes
// its address when it is issued).  The set must have at least COUNT members.  While it issues its reads the wavefront
// runs at a raised priority (s_setprio): the LDS port is the scarcest unit, so a wavefront that has reads to queue goes
// before the ones that are adding (measured: C2 78.3 -> 75.8 us, C3b 31.6 -> 29.7 us, M = 4096 at 50 % 1.7 % faster;
// levels 1, 2 and 3 do the same, keeping the priority up between the groups is slower).
#define TST_READ(i, width) \
    "s_ff1_i32_b64 %[k], %[set]\n\ts_bitset0_b64 %[set], %[k]\n\tv_lshl_add_u32 %[a], %[k], %[sh], %[base]\n\t" \
    "ds_read_" width " %[v" #i "], %[a]\n\t"
#define TST_R1(w) TST_READ(0, w)
#define TST_R2(w) TST_R1(w) TST_READ(1, w)
#define TST_R3(w) TST_R2(w) TST_READ(2, w)
#define TST_R4(w) TST_R3(w) TST_READ(3, w)
#define TST_R5(w) TST_R4(w) TST_READ(4, w)
#define TST_R6(w) TST_R5(w) TST_READ(5, w)
#define TST_R7(w) TST_R6(w) TST_READ(6, w)
#define TST_R8(w) TST_R7(w) TST_READ(7, w)
// only the value registers a group of COUNT uses are operands, so that a smaller group holds fewer registers
#define TST_O1 , [v0] "=&v"(v[0])
#define TST_O2 TST_O1, [v1] "=&v"(v[1])
#define TST_O3 TST_O2, [v2] "=&v"(v[2])
#define TST_O4 TST_O3, [v3] "=&v"(v[3])
#define TST_O5 TST_O4, [v4] "=&v"(v[4])
#define TST_O6 TST_O5, [v5] "=&v"(v[5])
#define TST_O7 TST_O6, [v6] "=&v"(v[6])
#define TST_O8 TST_O7, [v7] "=&v"(v[7])
#define TST_ASM(reads, outs) \
    asm volatile("s_setprio 1\n\t" reads "s_setprio 0\n\t" \
                 : [set] "+s"(set), [k] "=&s"(k), [a] "=&v"(a) outs : [sh] "n"(row_shift<R>()), [base] "v"(lane_base) : "memory")
template <int R, int COUNT>
__device__ __forceinline__ void read_rows(typename RowVec<R>::type (&v)[8], int lane_base, u64 &set)
{
    int k, a;
    static_assert(COUNT >= 1 && COUNT <= 8, "group sizes");
#define TST_GROUP(w) \
    if constexpr (COUNT == 8) TST_ASM(TST_R8(w), TST_O8); \
    else if constexpr (COUNT == 7) TST_ASM(TST_R7(w), TST_O7); \
    else if constexpr (COUNT == 6) TST_ASM(TST_R6(w), TST_O6); \
    else if constexpr (COUNT == 5) TST_ASM(TST_R5(w), TST_O5); \
    else if constexpr (COUNT == 4) TST_ASM(TST_R4(w), TST_O4); \
    else if constexpr (COUNT == 3) TST_ASM(TST_R3(w), TST_O3); \
    else if constexpr (COUNT == 2) TST_ASM(TST_R2(w), TST_O2); \
    else TST_ASM(TST_R1(w), TST_O1);
    if constexpr (R == 4) { TST_GROUP("b128") } else if constexpr (R == 2) { TST_GROUP("b64") } else { TST_GROUP("b32") }
#undef TST_GROUP
}

// The reads of a group return in order, so "at most LEFT reads outstanding" means that all but the youngest LEFT have
// arrived.  The wait is an asm statement that takes the values it makes valid as read-write operands: whatever uses or
// copies them is data-dependent on the wait and cannot be placed in front of it.  (A scalar load in flight at the same
// time only makes the wait longer: the counter is the number of LDS reads and scalar loads outstanding together.)
template <int LEFT, typename V> __device__ __forceinline__ void arrived(V &x, V &y)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(y) : "n"(LEFT));
}
template <int LEFT, typename V> __device__ __forceinline__ void arrived(V &x)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(LEFT));
}

// acc (+/-)= tile[k][rows of this lane] for the COUNT smallest members k of `set` (removed from it).  All gathers are
// issued before the first addition, so COUNT LDS reads are in flight at once; the additions take the values in pairs
// (second of a pair first), which halves the number of waits, and a last single one if COUNT is odd.
template <int R, bool NEG, int COUNT, int I>
__device__ __forceinline__ void add_arrived(typename RowVec<R>::type &acc, typename RowVec<R>::type (&v)[8])
{
    if constexpr (I + 1 < COUNT) {
        arrived<COUNT - 2 - I>(v[I], v[I + 1]);
        if constexpr (NEG) { acc -= v[I + 1]; acc -= v[I]; } else { acc += v[I + 1]; acc += v[I]; }
    } else if constexpr (I < COUNT) {
        arrived<0>(v[I]);
        if constexpr (NEG) acc -= v[I]; else acc += v[I];
    }
}

template <int R, bool NEG, int COUNT>
__device__ __forceinline__ void gather(typename RowVec<R>::type &acc, int lane_base, u64 &set)
{
    typedef typename RowVec<R>::type V;
    V v[8];
    read_rows<R, COUNT>(v, lane_base, set);
    add_arrived<R, NEG, COUNT, 0>(acc, v);
    add_arrived<R, NEG, COUNT, 2>(acc, v);
    add_arrived<R, NEG, COUNT, 4>(acc, v);
    add_arrived<R, NEG, COUNT, 6>(acc, v);
}

// One list: every member of the row set is gathered and added to (NEG: subtracted from) acc, in ascending row order,
// in groups of GMAX and then groups of 4, 2 and 1 for what is left, so that nothing but members of the list is gathered.
// GMAX = 4: half the registers for values in flight, for the launch shape with eight columns per wavefront, whose
// lists are short.  The set is wave-uniform.
template <int R, bool NEG, int GMAX>
__device__ __forceinline__ void run_list(typename RowVec<R>::type &acc, u64 set, int lane_base)
{
    static_assert(GMAX == 8 || GMAX == 4, "group sizes");
    int n = members(set);
    while (n >= GMAX) {
        gather<R, NEG, GMAX>(acc, lane_base, set);
        n -= GMAX;
    }
    // n is now in [0, GMAX): groups of 4, 2 and 1 by the bits of n.  Independent tests instead of an else-chain keep the
    // accumulators in place (with one group of exactly n behind nested branches the compiler gave the sums different
    // registers on the paths and copied them: 259 spilled registers in the 4-column kernel).
    if constexpr (GMAX == 8) {
        if (n & 4) gather<R, NEG, 4>(acc, lane_base, set);
    }
    if (n & 2) gather<R, NEG, 2>(acc, lane_base, set);
    if (n & 1) gather<R, NEG, 1>(acc, lane_base, set);
}

// ------------------------------------------------------------------------------------------------------------------
struct LargeArgs {
    const float *xt;
    const u64 *masks;
    const float *b;
    const float *alpha;   // PReLU slopes or nullptr
    float *Y;
    float *partials;   // [tile][k_slices][16 NCW columns][TM rows] when k_slices > 1
    int M, N, n_pad, n_kblocks, n_colgroups, k_slices, kb_per_slice;
    int remap;   // workgroups per XCD when the grid is spread evenly over the 8 XCDs, else 0
    int alpha_stride;
};

// What a workgroup does with its sums: the partial tile of its K slice for k_reduce (the tile as it sits in the
// registers, [column][row], so that a wavefront stores 64 R contiguous floats per column), or, when K is not sliced,
// Y = acc + b (bias added once, last), then the optional PReLU.
template <int R, int NCW>
__device__ __forceinline__ void finish(const LargeArgs &a, const typename RowVec<R>::type (&acc)[NCW], int mt, int cg,
                                       int slice, int wave, int lane, int c0)
{
    typedef typename RowVec<R>::type V;
    constexpr int TM = 64 * R;
    const int M = a.M, N = a.N;
    const int m0 = mt * TM;
    if (a.k_slices > 1) {
        constexpr size_t kTileFloats = (size_t)NW * NCW * TM;
        float *dst = a.partials + ((size_t)(mt * a.n_colgroups + cg) * a.k_slices + slice) * kTileFloats +
                     (size_t)(wave * NCW) * TM + lane * R;
#pragma unroll
        for (int j = 0; j < NCW; ++j) __builtin_nontemporal_store(acc[j], reinterpret_cast<V *>(dst + (size_t)j * TM));
        return;
    }
    float bias[NCW];
#pragma unroll
    for (int j = 0; j < NCW; ++j) bias[j] = (a.b != nullptr && c0 + j < N) ? a.b[c0 + j] : 0.f;
    const bool store_vec = NCW % 4 == 0 && (N % 4 == 0) && (c0 + NCW <= N) && ((reinterpret_cast<uintptr_t>(a.Y) & 15) == 0);
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int m = m0 + lane * R + r;
        if (m >= M) continue;
        float *yrow = a.Y + (size_t)m * N + c0;
        if constexpr (NCW % 4 == 0) {
            if (store_vec) {
#pragma unroll
                for (int j0 = 0; j0 < NCW; j0 += 4) {
                    float4v o;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        o[j] = activate(lane_of<R>(acc[j0 + j], r) + bias[j0 + j], a.alpha, a.alpha_stride, c0 + j0 + j);
                    *reinterpret_cast<float4v *>(yrow + j0) = o;
                }
                continue;
            }
        }
#pragma unroll
        for (int j = 0; j < NCW; ++j)
            if (c0 + j < N) yrow[j] = activate(lane_of<R>(acc[j], r) + bias[j], a.alpha, a.alpha_stride, c0 + j);
    }
}

// R rows per lane, NCW columns per wavefront, gather groups of at most GMAX.
template <int R, int NCW, int GMAX>
__global__ void __launch_bounds__(NT, 8) k_large(const LargeArgs a)
{
    typedef typename RowVec<R>::type V;
    constexpr int TM = 64 * R;                 // rows of X per workgroup tile
    constexpr int RB = TM * 4;                 // bytes of a tile row
    constexpr int STAGE = kKBlock * RB;        // bytes of one K-block of the tile
    constexpr int LPT = STAGE / (NT * 16);     // 16-byte pieces per thread and K-block
    static_assert(LPT >= 1 && STAGE % (NT * 16) == 0, "staging layout");
    __shared__ __attribute__((aligned(16))) char tile[STAGE];   // tile rows 0 .. 63 of the current K-block

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // Consecutive workgroup numbers go to different XCDs (each with its own L2).  Workgroups that share a K slice of
    // a tile read the same part of xt, so they are renumbered to land on the same XCD.
    int wg = blockIdx.x;
    if (a.remap) wg = (wg & 7) * a.remap + (wg >> 3);
    const int cg = wg % a.n_colgroups;
    const int rest = wg / a.n_colgroups;
    const int slice = rest % a.k_slices, mt = rest / a.k_slices;
    const int c0 = (cg * NW + wave) * NCW;   // < n_pad by construction of the grid
    const int kb0 = min(slice * a.kb_per_slice, a.n_kblocks);
    const int kb1 = min(kb0 + a.kb_per_slice, a.n_kblocks);

    V acc[NCW];
#pragma unroll
    for (int j = 0; j < NCW; ++j) acc[j] = zero_vec<R>();

    if (kb0 < kb1) {
        // ---- staging: K-block kb of the tile is STAGE contiguous bytes of xt; thread t copies pieces t, t + NT, ...
        const char *xtile = reinterpret_cast<const char *>(a.xt) + (size_t)mt * a.n_kblocks * STAGE;
        const int piece = threadIdx.x * 16;
        float4v st[LPT];
        auto stage_load = [&](int kb) {
#pragma unroll
            for (int i = 0; i < LPT; ++i)
                st[i] = *reinterpret_cast<const float4v *>(xtile + (size_t)kb * STAGE + (piece + i * NT * 16));
        };
        auto stage_store = [&]() {
#pragma unroll
            for (int i = 0; i < LPT; ++i) *reinterpret_cast<float4v *>(tile + piece + i * NT * 16) = st[i];
        };
        // ---- row sets of (kb, c0 .. c0+NCW-1): 2 NCW consecutive 64-bit words (column j: +1 set, -1 set)
        const const_u64_ptr sets_base =
            reinterpret_cast<const_u64_ptr>(reinterpret_cast<uintptr_t>(a.masks)) + (size_t)c0 * 2;
        const size_t sets_stride = (size_t)a.n_pad * 2;
        u64 sets[2 * NCW];
        auto load_sets = [&](int kb) {
#pragma unroll
            for (int i = 0; i < 2 * NCW; ++i) sets[i] = sets_base[(size_t)kb * sets_stride + i];
        };

        load_sets(kb0);
        stage_load(kb0);
        stage_store();
        __syncthreads();
        // LDS address of this lane's rows in tile row 0 (the asm reads take plain LDS addresses)
        const int lane_base = (int)(uintptr_t)(__attribute__((address_space(3))) char *)tile + lane * (R * 4);
        for (int kb = kb0; kb < kb1; ++kb) {
#pragma unroll
            for (int j = 0; j < NCW; ++j) {
                run_list<R, false, GMAX>(acc[j], sets[2 * j], lane_base);
                run_list<R, true, GMAX>(acc[j], sets[2 * j + 1], lane_base);
            }
            if (kb + 1 == kb1) break;
            // Exchange the tile.  The requests for the next K-block go out before the barrier, into the registers
            // the gathers no longer need, so their latency runs while the slower wavefronts finish; the barrier
            // itself only has to order this wavefront's LDS reads (complete: their values have been added) before
            // the other wavefronts' writes, so it does not wait for the requests.
            load_sets(kb + 1);
            stage_load(kb + 1);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            stage_store();
            __syncthreads();
        }
    }

    finish<R, NCW>(a, acc, mt, cg, slice, wave, lane, c0);
}

// One slab: `rows` rows of X (first row X) -> the same rows of Y.  The slab's tiles fit wp.xt.
template <int R, int NCW, int GMAX = 8>
hipError_t launch(const float *X, const tcsc *t, const float *b, float *Y, int rows, int k_slices, const WorkspacePlan &wp,
                  const Call &c)
{
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    constexpr int TM = 64 * R;
    const int k_pad = l.n_kblocks * kKBlock;
    const long long m_tiles = (rows + TM - 1) / TM;
    if (m_tiles * TM > wp.slab_rows) return hipErrorInvalidValue;

    hipError_t e = launch_pack(X, wp.xt, rows, l.K, k_pad, TM, c.stream);
    if (e != hipSuccess) return e;

    LargeArgs a;
    a.xt = wp.xt; a.masks = d.masks; a.b = b; a.Y = Y;
    a.alpha = c.act.alpha; a.alpha_stride = c.act.alpha_stride;
    a.partials = wp.partials;
    a.M = rows; a.N = l.N; a.n_pad = l.n_pad; a.n_kblocks = l.n_kblocks;
    if constexpr (NCW == 8) {
        // 128 columns per workgroup; K is not sliced in this shape (it is taken when rows x columns fill the chip)
        if (l.n_pad % (NW * NCW) != 0) return hipErrorInvalidValue;
        k_slices = 1;
    }
    a.n_colgroups = l.n_pad / (NW * NCW);
    const long long groups = m_tiles * a.n_colgroups;
    if (k_slices > kMaxKSlices) k_slices = kMaxKSlices;
    const size_t slice_bytes = (size_t)groups * NW * NCW * TM * sizeof(float);
    if (k_slices > 1 && slice_bytes * k_slices > wp.partial_bytes) k_slices = (int)(wp.partial_bytes / slice_bytes);
    if (k_slices < 1) k_slices = 1;
    a.k_slices = k_slices;
    a.kb_per_slice = (l.n_kblocks + k_slices - 1) / k_slices;
    const long long grid = groups * k_slices;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    a.remap = (grid % 8 == 0) ? (int)(grid / 8) : 0;
    if ((e = c.record_before()) != hipSuccess) return e;
    hipLaunchKernelGGL((k_large<R, NCW, GMAX>), dim3((unsigned)grid), dim3(NT), 0, c.stream, a);
    e = hipGetLastError();
    if (e == hipSuccess) e = c.record_after();
    if (e != hipSuccess || k_slices == 1) return e;
    return launch_reduce(NW * NCW, wp.partials, b, c.act, Y, rows, l.N, (int)m_tiles, a.n_colgroups, k_slices, TM, c.stream);
}

// Columns per wavefront and K slices for `m_tiles` row tiles processed together.
// 4 columns per wavefront (64 per workgroup); K is sliced only when rows x columns alone leave compute units idle, into
// as few slices as fill them.  With 8 columns per wavefront (128 per workgroup, gather groups of at most 4) a workgroup
// exchanges its tile half as often per column; that shape is taken when the column count allows it, rows x columns
// fill the chip without slicing K, and the estimate below says it is faster.  Measured on M = 4096, K = 4096,
// N = 8192 (whole rounds of workgroups in both shapes), time in us against the density d: 3760 d + 520 with 4
// columns, 3966 d + 316 with 8 -- 4 % faster at d = 0.5, 31 % at 1/16; the estimate scales these with the number of
// rounds of workgroups each shape needs (a last round that is partly filled costs a whole one).
struct Shape {
    int ncw, k_slices;
};
inline Shape choose_shape(const tcsc_layout_t &l, long long m_tiles, const Call &c)
{
    const bool wide_fits = l.n_pad % (NW * 8) == 0;
    const double density = (double)(l.nnz_pos + l.nnz_neg) / ((double)l.K * (double)l.N);
    const double gain8 = (3760.0 * density + 520.0) / (3966.0 * density + 316.0);   // time of a 64-column pair / time of a 128-column workgroup
    const int slots = 2 * compute_units();   // two workgroups per compute unit
    int ncw = c.cols_per_wave ? c.cols_per_wave : 4;
    if (c.cols_per_wave == 0 && wide_fits) {
        const long long groups8 = m_tiles * (l.n_pad / (NW * 8)), groups4 = 2 * groups8;
        const long long rounds8 = (groups8 + slots - 1) / slots, rounds4 = (groups4 + slots - 1) / slots;
        if (groups8 >= slots && 2.0 * (double)rounds8 <= (double)rounds4 * gain8) ncw = 8;
        // one workgroup per compute unit only: still ahead where the lists are very short (measured: 10 % at a
        // density of 1/16 on M = 2048, N = 4096 and on M = 1024, N = 8192; a tie at 1/8; 7 % behind at 1/2)
        else if (groups8 < slots && 2 * groups8 >= slots && gain8 >= 1.3) ncw = 8;
    }
    if (ncw == 8 && !wide_fits) ncw = 4;
    int k_slices = 1;
    if (ncw != 8) {
        k_slices = c.k_slices ? c.k_slices : slices_to_fill(m_tiles * (l.n_pad / (NW * ncw)), slots);
        if (k_slices > l.n_kblocks) k_slices = l.n_kblocks;
    }
    return Shape{ncw, k_slices};
}

// X is processed in slabs of as many row tiles as the workspace holds next to the partial sums (one slab if the
// workspace has room for everything the call's launch shape needs).
template <int R>
hipError_t pick(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c)
{
    const tcsc_layout_t &l = t->layout;
    constexpr int TM = 64 * R;
    const size_t tile_bytes = (size_t)l.n_kblocks * kKBlock * TM * sizeof(float);
    const long long m_tiles_all = ((long long)M + TM - 1) / TM;
    const Shape whole = choose_shape(l, m_tiles_all, c);
    const size_t partial_want =
        whole.k_slices > 1 ? (size_t)whole.k_slices * m_tiles_all * TM * l.n_pad * sizeof(float) : 0;
    WorkspacePlan wp = plan_workspace(c, tile_bytes, m_tiles_all, TM, partial_want);
    if (wp.slab_rows < TM) return kErrWorkspace;
    long long slab_rows = wp.slab_rows;
    if (slab_rows > 65535LL * 64) slab_rows = 65535LL * 64 / TM * TM;
    if (c.slab_tiles > 0 && slab_rows > (long long)c.slab_tiles * TM) slab_rows = (long long)c.slab_tiles * TM;
    for (long long m_begin = 0; m_begin < M; m_begin += slab_rows) {
        const int rows = (int)((M - m_begin) < slab_rows ? (M - m_begin) : slab_rows);
        const Shape s = choose_shape(l, (rows + TM - 1) / TM, c);
        const float *Xs = X + (size_t)m_begin * l.K;
        float *Ys = Y + (size_t)m_begin * l.N;
        hipError_t e;
        switch (s.ncw) {
        case 1: e = launch<R, 1>(Xs, t, b, Ys, rows, s.k_slices, wp, c); break;
        case 2: e = launch<R, 2>(Xs, t, b, Ys, rows, s.k_slices, wp, c); break;
        case 8: e = launch<R, 8, 4>(Xs, t, b, Ys, rows, s.k_slices, wp, c); break;
        default: e = launch<R, 4>(Xs, t, b, Ys, rows, s.k_slices, wp, c); break;
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

hipError_t launch_large(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c)
{
    if (M <= 128) return pick<2>(X, t, b, Y, M, c);
    return pick<4>(X, t, b, Y, M, c);
}

// Scratch memory of the large-M path: the least it runs with, and what one slab of every shape it would choose needs.
void large_workspace_bytes(int M, int K, int n_pad, size_t *min_bytes, size_t *best_bytes)
{
    const int TM = M <= 128 ? 128 : 256;
    const long long n_kblocks = ((long long)K + kKBlock - 1) / kKBlock;
    const size_t tile_bytes = (size_t)n_kblocks * kKBlock * TM * sizeof(float);
    const long long m_tiles = ((long long)M + TM - 1) / TM;
    // the most K slices any built-in shape takes: 64-column workgroups
    long long k_slices = slices_to_fill(m_tiles * (n_pad / (NW * 4)), 2 * compute_units());
    if (k_slices > n_kblocks) k_slices = n_kblocks;
    const size_t partial = k_slices > 1 ? (size_t)k_slices * m_tiles * TM * n_pad * sizeof(float) : 0;
    *min_bytes = tile_bytes;
    *best_bytes = ((size_t)m_tiles * tile_bytes + 255) / 256 * 256 + partial;
}

}  // namespace tst
