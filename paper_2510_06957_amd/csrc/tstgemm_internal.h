// Internal declarations shared by the host side and the kernels of libtstgemm.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "tstgemm.h"

namespace tst {

// Geometry of the K-blocked device form (see tcsc_layout_t in tstgemm.h).
constexpr int kKBlock = 64;   // rows of W (entries of an X row) per K-block
constexpr int kChunk = 8;     // index slots per chunk: one 32-byte scalar load
constexpr int kColPad = 64;   // columns are padded to a multiple of this
constexpr int kStreamSlack = 256 + 16;   // zeroed slots behind the stream: the kernel reads it in 1 KiB windows
constexpr int kMaxSplitGroups = 512;                     // workgroups of a split-K launch never exceed this
constexpr size_t kPartialTileBytes = 64 * 256 * 4;       // 64 columns x 256 rows of fp32 partial sums
constexpr size_t kCounterBytes = kMaxSplitGroups * sizeof(int32_t);
constexpr size_t kWorkspaceBytes = kCounterBytes + kMaxSplitGroups * kPartialTileBytes;

inline int pad_chunk(int n) { return (n + kChunk - 1) / kChunk * kChunk; }

}  // namespace tst

struct tcsc {
    int K = 0, N = 0;
    std::vector<int32_t> col_start_pos, col_start_neg, row_index_pos, row_index_neg;
    tcsc_layout_t layout{};
    void *dev = nullptr;   // caller's device buffer (borrowed) once uploaded
    bool uploaded = false;
};

namespace tst {

// Device pointers into an uploaded buffer.
struct DeviceTcsc {
    const int32_t *col_start_pos, *col_start_neg, *row_index_pos, *row_index_neg;
    int32_t *seg_count;
    uint32_t *seg_ptr;
    int32_t *stream;
    int32_t *counters;   // kMaxSplitGroups arrival counters, zero between calls
    float *partials;     // split-K partial sums
};

inline DeviceTcsc device_view(const tcsc *t)
{
    char *d = static_cast<char *>(t->dev);
    const tcsc_layout_t &l = t->layout;
    return DeviceTcsc{reinterpret_cast<const int32_t *>(d + l.off_col_start_pos),
                      reinterpret_cast<const int32_t *>(d + l.off_col_start_neg),
                      reinterpret_cast<const int32_t *>(d + l.off_row_index_pos),
                      reinterpret_cast<const int32_t *>(d + l.off_row_index_neg),
                      reinterpret_cast<int32_t *>(d + l.off_seg_count),
                      reinterpret_cast<uint32_t *>(d + l.off_seg_ptr),
                      reinterpret_cast<int32_t *>(d + l.off_stream),
                      reinterpret_cast<int32_t *>(d + l.off_workspace),
                      reinterpret_cast<float *>(d + l.off_workspace + kCounterBytes)};
}

// reblock.hip -- GPU pass: TCSC arrays (already on the device) -> seg_count, seg_ptr, stream.
hipError_t launch_reblock(const tcsc *t, hipStream_t stream);
// tstgemm_large.hip -- LDS-tiled gather-add kernel for M > 8.
hipError_t launch_large(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream);
extern int g_cols_per_wave, g_k_slices;   // tuning overrides, 0 = built-in choice
// tstgemm_decode.hip -- small-M kernel (M <= 8, whole X resident in the LDS).
bool decode_supported(int M, int K);
hipError_t launch_decode(const float *X, const tcsc *t, const float *b, float *Y, int M, hipStream_t stream);

}  // namespace tst
