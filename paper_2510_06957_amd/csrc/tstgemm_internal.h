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
constexpr int kIndexSlack = 64;   // entries behind each index array that may be read (never used)
constexpr int kChunk5 = 16;       // groups of five rows (bytes) per column and chunk of the value-compression form
constexpr size_t kPartialBytes = (size_t)32 << 20;       // split-K partial sums: workgroup tiles [tile][slice][column][row] fp32
constexpr size_t kXtMinBytes = (size_t)128 << 20;        // room for the tiled, transposed copy of X (a slab of rows at a time)

// The copy holds whole row tiles of X over all (padded) K: at least one tile of 256 rows must fit.
inline size_t xt_bytes(int n_kblocks)
{
    const size_t one = (size_t)256 * n_kblocks * kKBlock * sizeof(float);
    return one > kXtMinBytes ? one : kXtMinBytes;
}
inline size_t workspace_bytes(int n_kblocks) { return kPartialBytes + xt_bytes(n_kblocks); }

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
    float *partials;     // split-K partial sums
    float *xt;           // xt[tile][k][row]: row tiles of (a slab of) X, transposed, zero padded
    size_t xt_capacity;  // bytes
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
                      reinterpret_cast<uint8_t *>(d + l.off_packed),
                      reinterpret_cast<float *>(d + l.off_workspace),
                      reinterpret_cast<float *>(d + l.off_workspace + kPartialBytes),
                      xt_bytes(l.n_kblocks)};
}

// Optional PReLU behind the bias add: alpha == nullptr means none; alpha_stride 0 = one slope, 1 = one per column.
struct Activation {
    const float *alpha;
    int alpha_stride;
};
// reblock.hip -- GPU pass: TCSC arrays (already on the device) -> row sets, list cuts, signed lists, base-3 codes.
hipError_t launch_reblock(const tcsc *t, hipStream_t stream);
// tstgemm_side.hip -- X packing pre-pass and split-K reduction, shared by the tiled paths.
constexpr int kMaxKSlices = 8;
int compute_units();
// X (rows x K, row-major) -> xt[tile][k_pad][TM] (TM = 64, 128 or 256 rows per tile, or one tile of 32 or 16; k_pad a
// multiple of 64), zero padded.
hipError_t launch_pack(const float *X, float *xt, int rows, int K, int k_pad, int TM, hipStream_t stream);
// Y = sum of the k_slices partial tiles ([tile][slice][C columns][TM rows], C = 16, 32 or 64) in slice order + b, then act.
hipError_t launch_reduce(int C, const float *partials, const float *b, const Activation &act, float *Y, int M, int N,
                         int m_tiles, int n_colgroups, int k_slices, int TM, hipStream_t stream);
// tstgemm_small.hip -- lane-group gather-add kernel for 8 < M <= 64 (one tile of 64, 32 or 16 rows).
hipError_t launch_small(const float *X, const tcsc *t, const float *b, const Activation &act, float *Y, int M,
                        hipStream_t stream);
// tstgemm_large.hip -- LDS-tiled gather-add kernel for M > 64.
hipError_t launch_large(const float *X, const tcsc *t, const float *b, const Activation &act, float *Y, int M,
                        hipStream_t stream);
extern int g_cols_per_wave, g_k_slices, g_slab_tiles;   // tuning overrides, 0 = built-in choice
extern int g_decode_wide_lists;                         // != 0: the small-M kernel reads the 32-bit lists even if 16-bit ones exist
extern hipEvent_t g_event_before, g_event_after;       // recorded around the main kernel of a call when set
// tstgemm_decode.hip -- small-M kernel (M <= 8; X in the LDS, in chunks of K if need be).
bool decode_supported(int M);
hipError_t launch_decode(const float *X, const tcsc *t, const float *b, const Activation &act, float *Y, int M,
                         hipStream_t stream);
// the same kernel on the merged signed lists (inverted index)
hipError_t launch_decode_signed(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream);
// tstgemm_packed.hip -- M <= 8 from the base-3 codes (value compression)
hipError_t launch_packed(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream);

}  // namespace tst
