// Small-tile kernel of the sparse ternary GEMM  Y = X W + b  (Eq. 1 of the paper) for 8 < M <= 64.
//
// Arithmetic is that of BaseTCSC (Sec. 2): gather-add the +1 list, gather-subtract the -1 list, bias added once at
// the end; no multiplications.  With at most 64 rows of X a wavefront has more lanes than rows, so the mapping
// differs from the large-M kernel's:
//
//   * the 64 lanes form G groups (G = 4 for M <= 64, 8 for M <= 32, 16 for M <= 16); a lane owns 4 consecutive rows of
//     X, a group all TM = 256 / G rows of the tile;
//   * the G groups take G consecutive members of the SAME list at a time (the paper's "horizontal" scheme, Sec. 3,
//     between the groups; its "vertical" scheme inside a group): one ds_read_b128 of the wavefront gathers G tile
//     rows, one per group, and every group keeps its own partial sums, which are added across the groups once, at the
//     end of the K slice (a fixed order);
//   * the members come straight from the TCSC arrays (Sec. 2): the lists are ascending, so the piece of a list that
//     falls into a block of rows of W (the paper's blocking, Sec. 3) is a slice of row_index_pos / _neg; the
//     re-blocking pass stores where the slices start (list_cuts, a cut every 256 rows).  A lane loads 4 consecutive
//     row numbers with one 16-byte load, 4 G per wavefront; a row number costs one VALU instruction (shift and add to
//     the lane's LDS address) and no scalar work.  There are two walks of a slice.  The plain one (run_short_slice)
//     takes a slice in steps of 4 G entries, the last one padded with the row of zeros, entries requested one step
//     ahead: fewest instructions per slice, which is what counts where slices are a step or less.  The other one
//     (run_slice), for longer slices: the vector ALU's issue slots are what the kernel fills, and behind them it
//     waits for the loads of the entries -- a wavefront's loads return in order, and a step cannot start before its
//     entries are there -- so a step costs the vector ALU nothing but its four addresses and sixteen additions, the
//     partly filled step takes only the gathers it needs, the entries of a step are requested two steps ahead and
//     the first entries of a slice two slices ahead, behind every other request of the slice that issues them;
//   * the workgroup (16 wavefronts = 16 NCW columns) keeps one block of the packed X tile in the LDS (64 KiB:
//     256 rows of W at TM = 64, 512 at TM = 32, 1024 at TM = 16; tile[k][TM]) with a row of zeros in front of it for the slots behind
//     the end of a slice; two workgroups share a compute unit, one computes while the other exchanges its tile;
//   * split K, packing pre-pass and reduction as in the large-M path.
#include "tstgemm_internal.h"

namespace tst {
namespace {

constexpr int NW = 16;        // wavefronts per workgroup
constexpr int NT = NW * 64;   // threads per workgroup
constexpr int STAGE = 65536;                  // bytes of one block of the tile
constexpr int LPT = STAGE / (NT * 16);        // 16-byte pieces per thread and block
typedef float float4v __attribute__((ext_vector_type(4)));
typedef int int4v __attribute__((ext_vector_type(4)));
typedef int4v int4v_unaligned __attribute__((aligned(4)));   // the lists start at any entry: 4-byte aligned 16-byte loads
typedef const __attribute__((address_space(4))) int32_t *const_i32_ptr;   // read through the scalar cache
typedef const __attribute__((address_space(3))) float4v *lds_f4_ptr;

// Geometry for G lane groups.
template <int G> struct Geo {
    static constexpr int L = 64 / G;            // lanes per group
    static constexpr int TM = 4 * L;            // rows of X per tile
    static constexpr int RB = TM * 4;           // bytes of a tile row
    static constexpr int SH = G == 4 ? 8 : G == 8 ? 7 : 6;   // log2(RB)
    static constexpr int ROWS = STAGE / RB;     // rows of W per block
    static constexpr int CUTS = ROWS / kCutRows;   // list cuts per block
    static constexpr int CH = 4 * G;            // list entries per wavefront and step
    static constexpr int PR = TM < 32 ? 32 : TM;   // rows of a partial tile (the reduction kernel works in units of 32 rows)
    static_assert((1 << SH) == RB && 2 * CH <= kIndexSlack, "geometry");
};

struct SmallArgs {
    const float *xt;            // xt[k_pad][TM]: the one tile of X, packed
    const int32_t *cuts;        // [n_cuts + 1][n_pad][2]
    const int32_t *rip, *rin;   // row_index_pos / row_index_neg
    const float *b;
    const float *alpha;
    float *Y;
    float *partials;            // [colgroup][k_slices][16 NCW columns][PR rows] when k_slices > 1
    int M, N, n_pad, n_cuts, n_blocks, n_colgroups, k_slices, blocks_per_slice;
    int remap, alpha_stride;
};

// The lists are read through buffer loads: the address is a scalar descriptor (the array), a scalar byte offset (the
// step; below 4 GiB, which small_supported() checks) and a lane offset, so a load costs no vector instruction.  The
// loads are asm statements and so are the waits for them: a wavefront's loads return in order, the kernel keeps
// several in flight at once (two steps of the slice in hand, the first steps of the next two slices), and which of
// them a step needs follows from the order they were issued in, which the code below fixes -- the compiler, which
// does not know how many of the conditional ones are in flight, can only wait for all of them.
typedef int4v rsrc_t;
__device__ __forceinline__ rsrc_t list_rsrc(const int32_t *list)
{
    // raw buffer, no stride, no range limit to speak of; 32-bit data (the word an untyped load ignores but must be valid)
    const uintptr_t p = reinterpret_cast<uintptr_t>(list);
    return rsrc_t{(int)(uint32_t)p, (int)(uint32_t)((p >> 32) & 0xffffu), 0x7fffffff, 0x00020000};
}
__device__ __forceinline__ void list_load(int4v &q, rsrc_t list, int lane_offset, unsigned at)   // at: byte offset, < 4 GiB
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=&v"(q) : "v"(lane_offset), "s"(list), "s"(at) : "memory");
}
// At most LEFT loads outstanding: all but the youngest LEFT have arrived.  The wait takes the value it makes valid as
// a read-write operand, so that whatever uses or copies it is data-dependent on the wait.
template <int LEFT> __device__ __forceinline__ void loaded(int4v &q)
{
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(q) : "n"(LEFT));
}
// A slice of n entries is walked as  n % CH  entries first (the partly filled step, if any) and whole steps of CH
// entries behind it.  A whole step: lane group g takes entries 4 g .. 4 g + 3, one 16-byte load per lane.  The partly
// filled step takes s = ceil(entries / G) gathers instead of four (two or four are issued): lane group g takes entries
// s g .. s g + s - 1, so a lane still loads its entries with one 16-byte load (what lies behind its s entries, or
// behind the end of the slice, is loaded and not used; the index arrays have that much slack).
// This lane's entries of the first step of a slice of n entries that starts at entry `first` of the list.
template <int G> __device__ __forceinline__ void load_head(int4v &q, rsrc_t list, int first, int n, int g)
{
    const int head = n & (Geo<G>::CH - 1);
    const int slots = head ? (head + G - 1) / G : 4;
    list_load(q, list, __mul24(g, 4 * slots), 4u * (unsigned)first);
}

// LDS reads as asm statements: nothing is scheduled between the instructions of one statement, and the waits are
// placed by hand.  The reads return in order, so "at most LEFT outstanding" means that all but the youngest LEFT have
// arrived.  A wait takes the values it makes valid as read-write operands: whatever uses or copies them is
// data-dependent on the wait and cannot be placed in front of it.  (A scalar load in flight at the same time only
// makes a wait longer.)  Every read is waited for before the slice ends.
template <int LEFT> __device__ __forceinline__ void arrived(float4v &x, float4v &y)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(y) : "n"(LEFT));
}
template <int LEFT> __device__ __forceinline__ void arrived(float4v &x, float4v &y, float4v &sums)
{
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(x), "+v"(y), "+v"(sums) : "n"(LEFT));   // ... and behind what was added before
}
// The four gathers of a whole step: address = (row number << SH) + base (one VALU instruction; base is the lane's
// LDS address of row 0 of the W block minus the block's first row times the row size), then the 16-byte read; the
// address register is reused (an LDS instruction takes its address when it is issued).  While it queues its reads
// the wavefront runs at a raised priority (about 1 % faster).  The statement starts with the wait for the entries
// (at most LEFT younger loads still in flight), so the registers it reads are the ones the load wrote.
#define TST_STEP(wait) \
    asm volatile(wait "s_setprio 1\n\t" \
                 "v_lshl_add_u32 %[a], %[q0], %[sh], %[base]\n\tds_read_b128 %[v0], %[a]\n\t" \
                 "v_lshl_add_u32 %[a], %[q1], %[sh], %[base]\n\tds_read_b128 %[v1], %[a]\n\t" \
                 "v_lshl_add_u32 %[a], %[q2], %[sh], %[base]\n\tds_read_b128 %[v2], %[a]\n\t" \
                 "v_lshl_add_u32 %[a], %[q3], %[sh], %[base]\n\tds_read_b128 %[v3], %[a]\n\t" \
                 "s_setprio 0" \
                 : [a] "=&v"(a), [v0] "=&v"(v[0]), [v1] "=&v"(v[1]), [v2] "=&v"(v[2]), [v3] "=&v"(v[3]) \
                 : [q0] "v"(q[0]), [q1] "v"(q[1]), [q2] "v"(q[2]), [q3] "v"(q[3]), [sh] "n"(SH), [base] "v"(base) \
                 : "memory")
template <int SH, int LEFT> __device__ __forceinline__ void read_step(float4v (&v)[4], const int4v &q, int base)
{
    int a;
    static_assert(LEFT >= -1 && LEFT <= 2, "waits");
    if constexpr (LEFT == 2) TST_STEP("s_waitcnt vmcnt(2)\n\t");
    else if constexpr (LEFT == 1) TST_STEP("s_waitcnt vmcnt(1)\n\t");
    else if constexpr (LEFT == 0) TST_STEP("s_waitcnt vmcnt(0)\n\t");
    else TST_STEP("");   // the entries are there already
}
#undef TST_STEP
// Two or four gathers at ready-made addresses (the partly filled step).
__device__ __forceinline__ void read_two(float4v (&v)[4], int a0, int a1)
{
    asm volatile("s_setprio 1\n\tds_read_b128 %[v0], %[a0]\n\tds_read_b128 %[v1], %[a1]\n\ts_setprio 0"
                 : [v0] "=&v"(v[0]), [v1] "=&v"(v[1]) : [a0] "v"(a0), [a1] "v"(a1) : "memory");
}
__device__ __forceinline__ void read_four(float4v (&v)[4], int a0, int a1, int a2, int a3)
{
    asm volatile("s_setprio 1\n\tds_read_b128 %[v0], %[a0]\n\tds_read_b128 %[v1], %[a1]\n\t"
                 "ds_read_b128 %[v2], %[a2]\n\tds_read_b128 %[v3], %[a3]\n\ts_setprio 0"
                 : [v0] "=&v"(v[0]), [v1] "=&v"(v[1]), [v2] "=&v"(v[2]), [v3] "=&v"(v[3])
                 : [a0] "v"(a0), [a1] "v"(a1), [a2] "v"(a2), [a3] "v"(a3) : "memory");
}

// A slice of n entries of a list r, from entry `first` on; h holds this lane's entries of its first step, requested
// two slices ago and arrived.  Once they have become LDS addresses, `next` requests into the same registers what
// the slice after the next one starts with (load_head).  Order of the requests: the whole steps of this slice one
// after the other, each two steps ahead of its use, and `next` right behind the last of them -- so a step never
// waits for more than its own entries and what was requested before them, and at the start of every slice exactly
// two requests are in flight, its own and the next slice's.  zero_row is the lane's address in the row of zeros in
// front of the block: in a slot of the partly filled step where its lane group has no entry a lane gathers that.
template <int G, bool NEG, typename Next>
__device__ __forceinline__ void run_slice(float4v &acc, const int4v &h, rsrc_t r, int first, int n, int base,
                                          int zero_row, int g, Next next)
{
    constexpr int CH = Geo<G>::CH, SH = Geo<G>::SH;
    const int head = n & (CH - 1);
    unsigned at = 4u * (unsigned)(first + head);   // byte offset of the first whole step (below 4 GiB)
    int left = (n - head) / CH;    // whole steps to go
    int4v qa, qb;                  // the entries of the two steps behind the one in hand
    asm volatile("" : "=v"(qa), "=v"(qb));   // (defined as far as the compiler is concerned: no code to initialise them)
    float4v v[4];
    auto sums2 = [&]() {
        arrived<0>(v[0], v[1]);
        if constexpr (NEG) { acc -= v[0]; acc -= v[1]; } else { acc += v[0]; acc += v[1]; }
    };
    auto sums4 = [&]() {
        arrived<2>(v[0], v[1]);
        if constexpr (NEG) { acc -= v[0]; acc -= v[1]; } else { acc += v[0]; acc += v[1]; }
        arrived<0>(v[2], v[3], acc);
        if constexpr (NEG) { acc -= v[2]; acc -= v[3]; } else { acc += v[2]; acc += v[3]; }
    };
    const int lane16 = 16 * g;
    const int slots = (head + G - 1) / G;   // wave-uniform: gathers of the partly filled step, 0 if there is none
    if (head) {
        const int mine = min(head - __mul24(g, slots), slots);   // this lane group has entries in slots 0 .. mine - 1
        const int a0 = mine > 0 ? (h[0] << SH) + base : zero_row;
        const int a1 = mine > 1 ? (h[1] << SH) + base : zero_row;
        // two independent tests, not an else: the sums stay where they are on both paths
        if (slots <= 2) read_two(v, a0, a1);
        if (slots > 2) {
            const int a2 = mine > 2 ? (h[2] << SH) + base : zero_row;
            const int a3 = mine > 3 ? (h[3] << SH) + base : zero_row;
            read_four(v, a0, a1, a2, a3);
        }
    }
    // (a slice without a partly filled step, one in CH, has the entries of its first whole step in h; they are
    // requested once more, which keeps the steps below the same for every slice)
    if (left > 0) list_load(qa, r, lane16, at);
    if (left > 1) list_load(qb, r, lane16, at + 4 * CH);
    if (left <= 2) next();
    if (head) {
        if (slots <= 2) sums2();
        if (slots > 2) sums4();
    }
    // Whole steps, two per turn.  In flight when a step is about to start: its own entries, those of the step behind
    // it if there is one, and `next` once the last step's entries have been requested: two younger requests when two
    // steps are left, one otherwise.  The wait is for "at most one younger" in every case: with two steps left it then
    // also waits for the entries of the last step, requested a step ago, and the loop has one path instead of two.
    for (; left > 0; left -= 2, at += 8 * CH) {   // (one exit: with a second one in the middle the compiler builds flags around it)
        read_step<SH, 1>(v, qa, base);
        if (left > 2) {
            list_load(qa, r, lane16, at + 8 * CH);
            if (left == 3) next();
        }
        sums4();
        if (left > 1) {
            read_step<SH, 1>(v, qb, base);
            if (left > 3) {
                list_load(qb, r, lane16, at + 12 * CH);
                if (left == 4) next();
            }
            sums4();
        }
    }
}

// Four gathers of the wavefront: tile rows k[0..3] (per lane group), this lane's four X rows of each.  base is the
// lane's LDS address of row 0 of the W block minus the block's first row times the row size, so that
// address = (row number << SH) + base needs no subtraction.
template <int SH> __device__ __forceinline__ void gather4(float4v (&v)[4], const int4v &k, int base)
{
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = *reinterpret_cast<lds_f4_ptr>((k[t] << SH) + base);
}

// The walk for short slices (low density), where a wavefront's time is the number of instructions it gets through,
// scalar ones and branches included, and the bookkeeping of the walk above costs more than it saves: every step is four
// gathers, whole or not, and the loads are left to the compiler.
// A slice of n entries of a list: lane group g takes entries CH c + 4 g .. + 3 of step c; p points at the lane's
// entries of step 0 and q holds them (loaded by the caller, one slice ahead).  Entries behind the end of the slice
// (up to CH - 1 are loaded beyond it; the index arrays have that much slack) are replaced by k_zero, the row in
// front of the block, which holds zeros.
template <int G, bool NEG>
__device__ __forceinline__ void run_short_slice(float4v &acc, int4v q, const int32_t *__restrict__ p, int n, int base,
                                          int k_zero, int g)
{
    constexpr int CH = Geo<G>::CH, SH = Geo<G>::SH;
    // one loop for whole and partly filled steps: the accumulator is touched in one place only
    for (int c = 0; c < n; c += CH) {
        int4v cur = q;
        if (c + CH < n) q = *reinterpret_cast<const int4v_unaligned *>(p + c + CH);
        if (c + CH > n) {   // the last, partly filled step (wave-uniform)
            const int rem = n - c;
#pragma unroll
            for (int t = 0; t < 4; ++t) cur[t] = (4 * g + t < rem) ? cur[t] : k_zero;
        }
        float4v v[4];
        __builtin_amdgcn_s_setprio(1);   // queueing LDS reads goes before the other wavefronts' additions (about 1 % faster)
        gather4<SH>(v, cur, base);
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if constexpr (NEG) acc -= v[t]; else acc += v[t];
        }
    }
}

// LONG: the walk with hand-placed requests and waits (run_slice), for slices of a few steps; else the plain one.
template <int NCW, int G, bool LONG>
__global__ void __launch_bounds__(NT, 8) k_small(const SmallArgs a)
{
    using geo = Geo<G>;
    constexpr int L = geo::L, RB = geo::RB;
    __shared__ __attribute__((aligned(16))) char lds[RB + STAGE];   // the row of zeros, then the rows of the block
    char *const tile = lds + RB;
    const int M = a.M, N = a.N;
    const int lane = threadIdx.x & 63, g = lane / L, r = lane % L;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    int wg = blockIdx.x;
    if (a.remap) wg = (wg & 7) * a.remap + (wg >> 3);
    const int cg = wg % a.n_colgroups, slice = wg / a.n_colgroups;
    const int c0 = (cg * NW + wave) * NCW;   // < n_pad by construction of the grid
    const int blk0 = min(slice * a.blocks_per_slice, a.n_blocks);
    const int blk1 = min(blk0 + a.blocks_per_slice, a.n_blocks);

    float4v acc[NCW];
#pragma unroll
    for (int j = 0; j < NCW; ++j) acc[j] = float4v{0.f, 0.f, 0.f, 0.f};

    if (blk0 < blk1) {
        const char *xtile = reinterpret_cast<const char *>(a.xt);
        const int piece = threadIdx.x * 16;
        float4v st[LPT];
        auto stage_load = [&](int c) {
#pragma unroll
            for (int i = 0; i < LPT; ++i)
                st[i] = *reinterpret_cast<const float4v *>(xtile + (size_t)c * STAGE + (piece + i * NT * 16));
        };
        auto stage_store = [&]() {
#pragma unroll
            for (int i = 0; i < LPT; ++i) *reinterpret_cast<float4v *>(tile + piece + i * NT * 16) = st[i];
        };
        // slice borders of (block, c0 .. c0+NCW-1): 2 NCW consecutive ints per cut (column j: +1 list, -1 list)
        const const_i32_ptr cuts_base =
            reinterpret_cast<const_i32_ptr>(reinterpret_cast<uintptr_t>(a.cuts)) + (size_t)c0 * 2;
        const size_t cuts_stride = (size_t)a.n_pad * 2;
        int lo[2 * NCW], hi[2 * NCW];
        auto load_cut = [&](int (&dst)[2 * NCW], int blk) {
            const int cut = min(blk * geo::CUTS, a.n_cuts);   // the last block may end early: the end of the lists
#pragma unroll
            for (int i = 0; i < 2 * NCW; ++i) dst[i] = cuts_base[(size_t)cut * cuts_stride + i];
        };

        if (threadIdx.x < RB / 4) reinterpret_cast<float *>(lds)[threadIdx.x] = 0.f;
        load_cut(lo, blk0);
        stage_load(blk0);
        stage_store();
        __syncthreads();
        const int lds0 = (int)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
        const int lane_base = lds0 + RB + r * 16;     // this lane's part of tile row 0
        // exchange the tile (as in the large-M kernel: requests before the barrier, copies behind it)
        auto exchange = [&](int c) {
            stage_load(c);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            stage_store();
            __syncthreads();
        };
        if constexpr (LONG) {
            int nx[2 * NCW];
            load_cut(hi, blk0 + 1);
            // h0: the first entries of the +1 slice about to be walked (or, while a -1 slice is walked, of the next +1
            // slice), h1: the same for the -1 slices.  A slice requests those of the slice after the next one.
            const rsrc_t rp = list_rsrc(a.rip), rn = list_rsrc(a.rin);
            int4v h0, h1;
            load_head<G>(h0, rp, lo[0], hi[0] - lo[0], g);
            load_head<G>(h1, rn, lo[1], hi[1] - lo[1], g);
            for (int c = blk0; c < blk1; ++c) {
                load_cut(nx, c + 2);   // the borders of the next block's slices, for the requests at the end of this block
                const int base = lane_base - c * STAGE;   // tile row 0 is row c * ROWS of W
#pragma unroll
                for (int j = 0; j < NCW; ++j) {
                    // The column's sums are a value of their own while its lists are walked and the array is only touched
                    // here: updated in place inside the loops, the whole array went through copies (and, with four
                    // columns, spills) at every step.
                    float4v sum = acc[j];
                    // the next column's lists, or the first column's in the next block
                    const int p_first = j + 1 < NCW ? lo[2 * j + 2] : hi[0], p_n = (j + 1 < NCW ? hi[2 * j + 2] : nx[0]) - p_first;
                    const int n_first = j + 1 < NCW ? lo[2 * j + 3] : hi[1], n_n = (j + 1 < NCW ? hi[2 * j + 3] : nx[1]) - n_first;
                    loaded<1>(h0);
                    run_slice<G, false>(sum, h0, rp, lo[2 * j], hi[2 * j] - lo[2 * j], base, lane_base - RB, g,
                                        [&]() { load_head<G>(h0, rp, p_first, p_n, g); });
                    loaded<1>(h1);
                    run_slice<G, true>(sum, h1, rn, lo[2 * j + 1], hi[2 * j + 1] - lo[2 * j + 1], base, lane_base - RB, g,
                                       [&]() { load_head<G>(h1, rn, n_first, n_n, g); });
                    acc[j] = sum;
                }
#pragma unroll
                for (int i = 0; i < 2 * NCW; ++i) { lo[i] = hi[i]; hi[i] = nx[i]; }
                if (c + 1 == blk1) break;
                exchange(c + 1);
            }
            // the last two slices' requests (for slices that do not exist) are still in flight: they must have landed
            // before their registers are used for anything else
            loaded<0>(h0);
            loaded<0>(h1);
        } else {
            // first step of a slice: this lane's 4 entries, loaded one slice ahead of their use
            auto first_step = [&](const int32_t *rows, int at) {
                return int4v(*reinterpret_cast<const int4v_unaligned *>(rows + at + 4 * g));
            };
            int4v q = first_step(a.rip, lo[0]);
            for (int c = blk0; c < blk1; ++c) {
                load_cut(hi, c + 1);
                const int base = lane_base - c * STAGE;   // tile row 0 is row c * ROWS of W
                const int k_zero = c * geo::ROWS - 1;
#pragma unroll
                for (int j = 0; j < NCW; ++j) {
                    int4v qn = first_step(a.rin, lo[2 * j + 1]);
                    // The column's sums are a value of their own while its lists are walked and the array is only touched
                    // here: updated in place inside the loops, the whole array went through copies (and, with four
                    // columns, spills) at every step.
                    float4v sum = acc[j];
                    run_short_slice<G, false>(sum, q, a.rip + lo[2 * j] + 4 * g, hi[2 * j] - lo[2 * j], base, k_zero, g);
                    // behind the last column: the first slice of the next block starts where this block's ended
                    q = first_step(a.rip, j + 1 < NCW ? lo[2 * j + 2] : hi[0]);
                    run_short_slice<G, true>(sum, qn, a.rin + lo[2 * j + 1] + 4 * g, hi[2 * j + 1] - lo[2 * j + 1], base, k_zero, g);
                    acc[j] = sum;
                }
#pragma unroll
                for (int i = 0; i < 2 * NCW; ++i) lo[i] = hi[i];
                if (c + 1 == blk1) break;
                exchange(c + 1);
            }
        }
    }

    // partial sums of the lane groups -> totals in every lane (a fixed tree over the groups)
#pragma unroll
    for (int j = 0; j < NCW; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = acc[j][i];
#pragma unroll
            for (int d = L; d < 64; d <<= 1) v += __shfl_xor(v, d, 64);
            acc[j][i] = v;
        }

    if (a.k_slices > 1) {
        // this K slice's partial tile for k_reduce, [column][row]: group 0 stores TM contiguous floats per column
        // (columns PR floats apart; rows TM .. PR - 1, if any, are never looked at)
        constexpr int PR = geo::PR;
        constexpr size_t kTileFloats = (size_t)NW * NCW * PR;
        float *dst = a.partials + ((size_t)cg * a.k_slices + slice) * kTileFloats + (size_t)(wave * NCW) * PR + r * 4;
        if (g == 0) {
#pragma unroll
            for (int j = 0; j < NCW; ++j) __builtin_nontemporal_store(acc[j], reinterpret_cast<float4v *>(dst + (size_t)j * PR));
        }
        return;
    }

    // output: Y = acc + b (bias added once, last), then the optional PReLU; lane group g < 4 stores row 4 r + g
    const int m = 4 * r + g;
    if (g >= 4 || m >= M) return;
    float *yrow = a.Y + (size_t)m * N + c0;
#pragma unroll
    for (int j = 0; j < NCW; ++j) {
        if (c0 + j >= N) continue;
        const float s = g == 0 ? acc[j][0] : g == 1 ? acc[j][1] : g == 2 ? acc[j][2] : acc[j][3];
        const float bias = a.b != nullptr ? a.b[c0 + j] : 0.f;
        yrow[j] = activate(s + bias, a.alpha, a.alpha_stride, c0 + j);
    }
}

template <int NCW, int G, bool LONG>
hipError_t launch(const float *X, const tcsc *t, const float *b, float *Y, int M, int k_slices, const Call &c)
{
    using geo = Geo<G>;
    constexpr int TM = geo::TM;
    const tcsc_layout_t &l = t->layout;
    const DeviceTcsc d = device_view(t);
    const int n_blocks = (l.K + geo::ROWS - 1) / geo::ROWS;
    const int k_pad = n_blocks * geo::ROWS;
    if (M > TM) return hipErrorInvalidValue;
    // workspace: the one tile of X, then whatever is left for the partial sums of the K slices
    const WorkspacePlan wp = plan_workspace(c, (size_t)k_pad * TM * sizeof(float), 1, TM, 0);
    if (wp.slab_rows < TM) return kErrWorkspace;
    const hipStream_t stream = c.stream;
    const Activation &act = c.act;
    hipError_t e = launch_pack(X, wp.xt, M, l.K, k_pad, TM, stream);
    if (e != hipSuccess) return e;

    SmallArgs a;
    a.xt = wp.xt; a.cuts = d.list_cuts; a.rip = d.row_index_pos; a.rin = d.row_index_neg;
    a.b = b; a.alpha = act.alpha; a.alpha_stride = act.alpha_stride; a.Y = Y; a.partials = wp.partials;
    a.M = M; a.N = l.N; a.n_pad = l.n_pad; a.n_cuts = l.n_cuts; a.n_blocks = n_blocks;
    a.n_colgroups = l.n_pad / (NW * NCW);
    if (k_slices > n_blocks) k_slices = n_blocks;
    if (k_slices > kMaxKSlices) k_slices = kMaxKSlices;
    const size_t slice_bytes = (size_t)a.n_colgroups * NW * NCW * geo::PR * sizeof(float);
    if (k_slices > 1 && slice_bytes * k_slices > wp.partial_bytes) k_slices = (int)(wp.partial_bytes / slice_bytes);
    if (k_slices < 1) k_slices = 1;
    a.k_slices = k_slices;
    a.blocks_per_slice = (n_blocks + k_slices - 1) / k_slices;
    const long long grid = (long long)a.n_colgroups * k_slices;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    a.remap = (grid % 8 == 0) ? (int)(grid / 8) : 0;
    if ((e = c.record_before()) != hipSuccess) return e;
    hipLaunchKernelGGL((k_small<NCW, G, LONG>), dim3((unsigned)grid), dim3(NT), 0, stream, a);
    e = hipGetLastError();
    if (e == hipSuccess) e = c.record_after();
    if (e != hipSuccess || k_slices == 1) return e;
    return launch_reduce(NW * NCW, wp.partials, b, act, Y, M, l.N, 1, a.n_colgroups, k_slices, geo::PR, stream);
}

}  // namespace

// M <= 64: one tile of 64 rows, or of 32 / 16 rows with two / four times as many rows of W per block.  K is sliced (at
// block borders) as far as it takes to give every compute unit two workgroups.  Columns per wavefront: 4 (64 per
// workgroup: a block of the tile in the LDS serves twice the columns, half the exchanges per column) when that still
// fills the chip with at most 8 slices of at least 4 blocks each; else 2; a short K (at most four list cuts) is not
// sliced and takes one column per wavefront, which saves the reduction kernel.
hipError_t launch_small(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c)
{
    if (M > 64) return hipErrorInvalidValue;
    const tcsc_layout_t &l = t->layout;
    if (!small_supported(l)) return hipErrorInvalidValue;
    const bool short_k = l.n_cuts <= 4;
    const int G = M <= 16 ? 16 : M <= 32 ? 8 : 4;
    const int slots = 2 * compute_units();
    int ncw = c.cols_per_wave ? (c.cols_per_wave == 1 ? 1 : c.cols_per_wave == 2 ? 2 : 4) : (short_k ? 1 : 2);
    if (c.cols_per_wave == 0 && !short_k) {
        const int block_rows = STAGE / (4 * (256 / G));            // rows of W per block of the tile
        const long long n_blocks = (l.K + block_rows - 1) / block_rows;
        const long long groups4 = l.n_pad / (NW * 4);
        const long long slices4 = groups4 >= slots ? 1 : (slots + groups4 - 1) / groups4;
        if (slices4 <= kMaxKSlices && n_blocks >= 4 * slices4) ncw = 4;
    }
    const long long groups = l.n_pad / (NW * ncw);
    int k_slices = c.k_slices;
    if (k_slices == 0) k_slices = (short_k || groups >= slots) ? 1 : (int)((slots + groups - 1) / groups);
    // Which walk of the lists: by the mean length of a slice (the entries of one list inside one block of rows of W) in
    // steps of the wavefront (4 G entries).  Measured, time of the kernel with the requests placed by hand against the
    // plain walk: 4 steps (M = 64, 32 and 16 at 50 %) 10 %, 11 % and 9 % faster; 2 steps (M = 64, 32 and 16 at 25 %)
    // 3 %, 5 % and 0 % faster; 1 step and less (M = 64 at 12.5 % and 6.25 %) 11 % and 13 % slower.  From 1.5 steps on
    // it is taken.
    const int block_rows = STAGE / (4 * (256 / G));
    const long long n_blocks = (l.K + block_rows - 1) / block_rows;
    const bool long_slices = c.list_walk ? c.list_walk == 2
                                         : (double)(l.nnz_pos + l.nnz_neg) >= 2.0 * (1.5 * 4 * G) * (double)n_blocks * (double)l.N;
    const int shape = G * 8 + ncw;
#define TST_SMALL(NCW_, G_) \
    case G_ * 8 + NCW_: \
        return long_slices ? launch<NCW_, G_, true>(X, t, b, Y, M, k_slices, c) : launch<NCW_, G_, false>(X, t, b, Y, M, k_slices, c)
    switch (shape) {
        TST_SMALL(1, 16);
        TST_SMALL(2, 16);
        TST_SMALL(4, 16);
        TST_SMALL(1, 8);
        TST_SMALL(2, 8);
        TST_SMALL(4, 8);
        TST_SMALL(1, 4);
        TST_SMALL(2, 4);
    default:
        return long_slices ? launch<4, 4, true>(X, t, b, Y, M, k_slices, c) : launch<4, 4, false>(X, t, b, Y, M, k_slices, c);
    }
#undef TST_SMALL
}

// The small-tile kernel addresses a list with 32-bit byte offsets: lists of 2^30 entries or more are not for it (the
// large-M kernel takes any number of rows of X).
bool small_supported(const tcsc_layout_t &l)
{
    return l.nnz_pos + kIndexSlack < (1LL << 30) && l.nnz_neg + kIndexSlack < (1LL << 30);
}

// Bytes of the one tile of X (M <= 64 rows: 64, 32 or 16 rows per tile) over K padded to whole blocks.
size_t small_tile_bytes(int M, int K)
{
    const int TM = M <= 16 ? 16 : M <= 32 ? 32 : 64;
    const int block_rows = STAGE / (4 * TM);
    const long long n_blocks = ((long long)K + block_rows - 1) / block_rows;
    return (size_t)n_blocks * block_rows * TM * sizeof(float);
}

}  // namespace tst
