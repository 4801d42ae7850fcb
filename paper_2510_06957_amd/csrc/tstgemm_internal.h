// Internal declarations shared by the host side and the kernels of libtstgemm.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "tstgemm.h"

namespace tst {

// Geometry of the K-blocked device form (see tcsc_layout_t in tstgemm.h).
constexpr int kKBlock = 64;   // rows of W (entries of an X row) per K-block: one 64-bit row set per list piece
constexpr int kColPad = 64;   // columns are padded to a multiple of this
constexpr int kCutRows = 256; // rows of W per list cut of the small-tile kernel (its K-block)
constexpr int kIndexSlack = 256;  // entries behind each index array that may be read (never used)
constexpr int kChunk5 = 16;       // groups of five rows (bytes) per column and chunk of the value-compression form
// The workspace inside a handle's device buffer: room for 32 MiB of split-K partial sums and 128 MiB of the tiled,
// transposed copy of X, or for one tile of 256 rows over the padded K if that is more.
constexpr size_t kPartialBytes = (size_t)32 << 20;
constexpr size_t kXtMinBytes = (size_t)128 << 20;
inline size_t handle_workspace_bytes(int n_kblocks)
{
    const size_t one = (size_t)256 * n_kblocks * kKBlock * sizeof(float);
    return kPartialBytes + (one > kXtMinBytes ? one : kXtMinBytes);
}

// y = v for v > 0, alpha * v otherwise (alpha == nullptr: y = v).  n: column of Y.
__device__ __forceinline__ float activate(float v, const float *alpha, int alpha_stride, int n)
{
    if (alpha == nullptr) return v;
    return v > 0.f ? v : alpha[(size_t)n * alpha_stride] * v;
}

}  // namespace tst

struct tcsc {
    int K = 0, N = 0;
    std::vector<int32_t> col_start_pos, col_start_neg, row_index_pos, row_index_neg;
    std::vector<int32_t> col_start16_pos, col_start16_neg;   // pointers of the padded 16-bit lists (K <= 65535 only)
    uint32_t forms = TCSC_FORM_ALL;   // device forms the next upload builds (tcsc_select_forms)
    tcsc_layout_t layout{};
    void *dev = nullptr;   // caller's device buffer (borrowed) once uploaded
    bool uploaded = false;
};

namespace tst {

// Device pointers into an uploaded buffer.
struct DeviceTcsc {
    const int32_t *col_start_pos, *col_start_neg, *row_index_pos, *row_index_neg;
    unsigned long long *masks;   // [n_kblocks][n_pad][2]
    int32_t *list_cuts;          // [n_cuts + 1][n_pad][2]
    const int32_t *col_start16_pos, *col_start16_neg;   // the padded 16-bit lists (K <= 65535 only) ...
    uint16_t *row_index16_pos, *row_index16_neg;        // ... pad value K = the row of zeros
    int32_t *signed_index;       // merged lists, -1 entries as ~row
    uint8_t *packed;             // [n_chunks5][n_pad][16] base-3 codes
};

inline DeviceTcsc device_view(const tcsc *t)
{
    char *d = static_cast<char *>(t->dev);
    const tcsc_layout_t &l = t->layout;
    return DeviceTcsc{reinterpret_cast<const int32_t *>(d + l.off_col_start_pos),
                      reinterpret_cast<const int32_t *>(d + l.off_col_start_neg),
                      reinterpret_cast<const int32_t *>(d + l.off_row_index_pos),
                      reinterpret_cast<const int32_t *>(d + l.off_row_index_neg),
                      reinterpret_cast<unsigned long long *>(d + l.off_masks),
                      reinterpret_cast<int32_t *>(d + l.off_list_cuts),
                      reinterpret_cast<const int32_t *>(d + l.off_col_start16_pos),
                      reinterpret_cast<const int32_t *>(d + l.off_col_start16_neg),
                      reinterpret_cast<uint16_t *>(d + l.off_row_index16_pos),
                      reinterpret_cast<uint16_t *>(d + l.off_row_index16_neg),
                      reinterpret_cast<int32_t *>(d + l.off_signed_index),
                      reinterpret_cast<uint8_t *>(d + l.off_packed)};
}

// Optional PReLU behind the bias add: alpha == nullptr means none; alpha_stride 0 = one slope, 1 = one per column.
struct Activation {
    const float *alpha;
    int alpha_stride;
};

// What one call brings besides its operands: stream, activation, scratch memory, launch-shape overrides and the
// optional event pair around the main kernel.  Nothing here outlives the call.
struct Call {
    hipStream_t stream;
    Activation act;
    char *ws;            // scratch (256-byte aligned) or nullptr
    size_t ws_bytes;
    int cols_per_wave, k_slices, slab_tiles;   // 0 = built-in choice
    int list_walk;       // small-tile kernel: 0 = built-in choice, 1 = plain, 2 = requests placed by hand
    bool decode_wide_lists;
    hipEvent_t event_before, event_after;      // both or neither

    hipError_t record_before() const { return event_before ? hipEventRecord(event_before, stream) : hipSuccess; }
    hipError_t record_after() const { return event_after ? hipEventRecord(event_after, stream) : hipSuccess; }
};

// A call whose workspace is absent or too small for the least the path can do: the entry points turn it into
// TSTGEMM_EWORKSPACE.
constexpr hipError_t kErrWorkspace = hipErrorOutOfMemory;

// How a tiled path lays the workspace out: the tiled copy of X for `slab_rows` rows at a time, then the partial sums.
struct WorkspacePlan {
    float *xt;
    float *partials;
    size_t partial_bytes;
    long long slab_rows;   // rows of X per slab, a multiple of the tile height (0: the workspace holds no tile)
};
// tile_bytes: one row tile over the padded K; m_tiles: tiles of the whole call; partial_want: bytes of partial sums the
// launch shape of the whole call in ONE slab would write (0 if it does not slice K).  If everything fits, one slab;
// else the partial sums get min(32 MiB, a quarter of the workspace) and the tiles the rest.
inline WorkspacePlan plan_workspace(const Call &c, size_t tile_bytes, long long m_tiles, int TM, size_t partial_want)
{
    WorkspacePlan p{nullptr, nullptr, 0, 0};
    if (c.ws == nullptr || c.ws_bytes < tile_bytes) return p;
    const size_t xt_all = (size_t)m_tiles * tile_bytes;
    const size_t xt_room = (xt_all + 255) / 256 * 256;
    p.xt = reinterpret_cast<float *>(c.ws);
    if (xt_room + partial_want <= c.ws_bytes) {
        p.partials = reinterpret_cast<float *>(c.ws + xt_room);
        p.partial_bytes = c.ws_bytes - xt_room;
        p.slab_rows = m_tiles * TM;
        return p;
    }
    size_t part = c.ws_bytes / 4 < kPartialBytes ? c.ws_bytes / 4 : kPartialBytes;
    part = part / 256 * 256;
    if (c.ws_bytes - part < tile_bytes) part = (c.ws_bytes - tile_bytes) / 256 * 256;
    const size_t xt_bytes = c.ws_bytes - part;
    long long tiles = (long long)(xt_bytes / tile_bytes);
    if (tiles > m_tiles) tiles = m_tiles;
    p.partials = reinterpret_cast<float *>(c.ws + (c.ws_bytes - part));
    p.partial_bytes = part;
    p.slab_rows = tiles * TM;
    return p;
}
// reblock.hip -- GPU pass: TCSC arrays (already on the device) -> row sets, list cuts, signed lists, base-3 codes.
hipError_t launch_reblock(const tcsc *t, hipStream_t stream);
// tstgemm_side.hip -- X packing pre-pass and split-K reduction, shared by the tiled paths.
constexpr int kMaxKSlices = 8;
int compute_units();
// X (rows x K, row-major) -> xt[tile][k_pad][TM] (TM = 64, 128 or 256 rows per tile, or one tile of 32 or 16; k_pad a
// multiple of 64), zero padded.
hipError_t launch_pack(const float *X, float *xt, int rows, int K, int k_pad, int TM, hipStream_t stream);
// the rule of the tiled paths for how many slices of K fill the chip: as few as give every compute unit two workgroups
inline int slices_to_fill(long long groups, int slots)
{
    if (groups >= slots) return 1;
    const long long s = (slots + groups - 1) / groups;
    return s > kMaxKSlices ? kMaxKSlices : (int)s;
}
// Y = sum of the k_slices partial tiles ([tile][slice][C columns][TM rows], C = 16, 32 or 64) in slice order + b, then act.
hipError_t launch_reduce(int C, const float *partials, const float *b, const Activation &act, float *Y, int M, int N,
                         int m_tiles, int n_colgroups, int k_slices, int TM, hipStream_t stream);
// tstgemm_small.hip -- lane-group gather-add kernel for 8 < M <= 64 (one tile of 64, 32 or 16 rows).
hipError_t launch_small(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c);
bool small_supported(const tcsc_layout_t &l);   // false: the lists are too long for its 32-bit offsets, use launch_large
size_t small_tile_bytes(int M, int K);   // one tile of X for M <= 64 over the padded K
// tstgemm_large.hip -- LDS-tiled gather-add kernel for M > 64.
hipError_t launch_large(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c);
void large_workspace_bytes(int M, int K, int n_pad, size_t *min_bytes, size_t *best_bytes);
// tstgemm_decode.hip -- small-M kernel (M <= 8; X in the LDS, in chunks of K if need be).
bool decode_supported(int M);
hipError_t launch_decode(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c);
// the same kernel on the merged signed lists (inverted index)
hipError_t launch_decode_signed(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c);
// tstgemm_packed.hip -- M <= 8 from the base-3 codes (value compression)
hipError_t launch_packed(const float *X, const tcsc *t, const float *b, float *Y, int M, const Call &c);
size_t packed_partial_bytes(int N);      // the most partial sums launch_packed() writes

}  // namespace tst
