// Host side of libtstgemm: handle, TCSC construction and validation (Sec. 2 of the paper), the matrix in the paper's
// two other encodings (Sec. 3), device-buffer layout, upload and the dispatch of the tstgemm*() entry points.
#include <algorithm>
#include <cstring>
#include <new>

#include "tstgemm_internal.h"

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

void compute_layout(tcsc *t)
{
    tcsc_layout_t &l = t->layout;
    l.K = t->K;
    l.N = t->N;
    l.n_pad = (t->N + tst::kColPad - 1) / tst::kColPad * tst::kColPad;
    l.k_block = tst::kKBlock;
    l.n_kblocks = (t->K + tst::kKBlock - 1) / tst::kKBlock;
    l.n_cuts = (t->K + tst::kCutRows - 1) / tst::kCutRows;
    l.nnz_pos = (int64_t)t->row_index_pos.size();
    l.nnz_neg = (int64_t)t->row_index_neg.size();
    uint32_t forms = t->forms;
    if (forms & TCSC_FORM_PACKED) forms |= TCSC_FORM_ROWSETS;   // the codes are built from the row sets
    size_t off = 0;
    // a section of `bytes` bytes if the form is part of the buffer, else nothing at offset 0
    auto place = [&](size_t bytes, bool present = true) {
        if (!present) return (size_t)0;
        size_t o = off;
        off = align_up(off + bytes);
        return o;
    };
    l.off_col_start_pos = place(sizeof(int32_t) * (size_t)(t->N + 1));
    l.off_col_start_neg = place(sizeof(int32_t) * (size_t)(t->N + 1));
    // + slack: the kernels read the lists in groups of up to 64 entries
    l.off_row_index_pos = place(sizeof(int32_t) * (size_t)(l.nnz_pos + tst::kIndexSlack));
    l.off_row_index_neg = place(sizeof(int32_t) * (size_t)(l.nnz_neg + tst::kIndexSlack));
    l.off_masks = place(2 * sizeof(uint64_t) * (size_t)l.n_kblocks * (size_t)l.n_pad, forms & TCSC_FORM_ROWSETS);
    l.off_list_cuts = place(2 * sizeof(int32_t) * (size_t)(l.n_cuts + 1) * (size_t)l.n_pad, forms & TCSC_FORM_CUTS);
    // padded 16-bit lists: every column's list rounded up to 8 entries; the pad value K must fit in 16 bits
    l.has_lists16 = ((forms & TCSC_FORM_LISTS16) && t->K <= 65535) ? 1 : 0;
    l.nnz16_pos = l.nnz16_neg = 0;
    t->col_start16_pos.clear();
    t->col_start16_neg.clear();
    if (l.has_lists16) {
        auto padded = [&](const std::vector<int32_t> &cs, std::vector<int32_t> &cs16) {
            cs16.assign((size_t)t->N + 1, 0);
            int64_t at = 0;
            for (int n = 0; n < t->N; ++n) {
                at += ((int64_t)cs[n + 1] - cs[n] + 7) / 8 * 8;
                if (at > INT32_MAX) return (int64_t)-1;
                cs16[n + 1] = (int32_t)at;
            }
            return at;
        };
        l.nnz16_pos = padded(t->col_start_pos, t->col_start16_pos);
        l.nnz16_neg = padded(t->col_start_neg, t->col_start16_neg);
        if (l.nnz16_pos < 0 || l.nnz16_neg < 0) {   // the padding does not fit 32-bit pointers: go without
            l.has_lists16 = 0;
            l.nnz16_pos = l.nnz16_neg = 0;
            t->col_start16_pos.clear();
            t->col_start16_neg.clear();
        }
    }
    if (!l.has_lists16) forms &= ~TCSC_FORM_LISTS16;
    l.off_col_start16_pos = place(sizeof(int32_t) * (size_t)(t->N + 1), l.has_lists16);
    l.off_col_start16_neg = place(sizeof(int32_t) * (size_t)(t->N + 1), l.has_lists16);
    l.off_row_index16_pos = place(sizeof(uint16_t) * (size_t)(l.nnz16_pos + tst::kIndexSlack), l.has_lists16);
    l.off_row_index16_neg = place(sizeof(uint16_t) * (size_t)(l.nnz16_neg + tst::kIndexSlack), l.has_lists16);
    l.off_signed_index = place(sizeof(int32_t) * (size_t)(l.nnz_pos + l.nnz_neg + tst::kIndexSlack), forms & TCSC_FORM_SIGNED);
    const int groups5 = (t->K + 4) / 5;
    l.n_chunks5 = (groups5 + tst::kChunk5 - 1) / tst::kChunk5;
    l.off_packed = place((size_t)l.n_chunks5 * (size_t)l.n_pad * tst::kChunk5, forms & TCSC_FORM_PACKED);
    l.workspace_bytes = (forms & TCSC_FORM_WORKSPACE) ? tst::handle_workspace_bytes(l.n_kblocks) : 0;
    l.off_workspace = place(l.workspace_bytes, forms & TCSC_FORM_WORKSPACE);
    l.total_bytes = off;
    l.forms = forms;
}

// The padded 16-bit copy of one sign's lists for the small-M kernel (M <= 8, all of X in the LDS): column n's list at
// [cs16[n], cs16[n + 1]), a multiple of 8 entries, pad value K (the row of zeros).  The kernel deals a list to the
// wavefront in rounds of 512 entries: lane l takes the 8 consecutive entries 8 l .. 8 l + 7 of a round and gathers,
// for each of its 8 slots in turn, the row of X in the LDS (16 bytes per plane of four rows of X).  Sixteen consecutive
// lanes gather together, and rows that are equal modulo 16 lie in the same LDS banks: in ascending order (random rows)
// half of the LDS time of M = 8 went into bank conflicts.  The order inside a column's list is free (a sum), so it is
// chosen here: the t-th entry with row = c mod 16 goes to member c of the t-th group of 16 lanes x one slot, which makes
// the sixteen rows of a group different modulo 16; entries of a class that has more members than there are whole
// groups go, in order, to the positions that stayed free, and what is then still free is padding.
void build_lists16(const std::vector<int32_t> &cs, const std::vector<int32_t> &rows, const std::vector<int32_t> &cs16, int N,
                   int K, std::vector<uint16_t> &out)
{
    const uint16_t pad = (uint16_t)K;
    out.assign((size_t)cs16[N] + tst::kIndexSlack, pad);
    std::vector<int32_t> overflow;
    for (int n = 0; n < N; ++n) {
        const int32_t *col = rows.data() + cs[n];
        const int len = cs[n + 1] - cs[n], len16 = cs16[n + 1] - cs16[n];
        uint16_t *dst = out.data() + cs16[n];
        // whole groups: 4 x 8 per whole round of 512, then 8 per 16 whole lanes of the last round
        const int whole_rounds = len16 / 512, last_lanes = (len16 % 512) / 8;
        const int groups = whole_rounds * 32 + (last_lanes / 16) * 8;
        int members[16] = {0};
        overflow.clear();
        for (int i = 0; i < len; ++i) {
            const int c = col[i] & 15, t = members[c]++;
            if (t < groups) {
                const int r = t / 32, j = (t % 32) / 8, e = t % 8;   // group t: round r, lanes 16 j .. 16 j + 15, slot e
                dst[r * 512 + (16 * j + c) * 8 + e] = (uint16_t)col[i];
            } else {
                overflow.push_back(col[i]);
            }
        }
        size_t next = 0;
        for (int p = 0; p < len16 && next < overflow.size(); ++p)
            if (dst[p] == pad) dst[p] = (uint16_t)overflow[next++];
    }
}

// The structural rules of the format: monotone pointers starting at 0, rows inside [0,K),
// strictly ascending inside a column, no row in both lists of a column.
int validate(const int32_t *csp, const int32_t *csn, const int32_t *rip, const int32_t *rin, int K, int N)
{
    if (csp[0] != 0 || csn[0] != 0) return TSTGEMM_EFORMAT;
    for (int n = 0; n < N; ++n)
        if (csp[n + 1] < csp[n] || csn[n + 1] < csn[n]) return TSTGEMM_EFORMAT;
    for (int n = 0; n < N; ++n) {
        for (int32_t i = csp[n]; i < csp[n + 1]; ++i) {
            if (rip[i] < 0 || rip[i] >= K) return TSTGEMM_EFORMAT;
            if (i > csp[n] && rip[i] <= rip[i - 1]) return TSTGEMM_EFORMAT;
        }
        for (int32_t i = csn[n]; i < csn[n + 1]; ++i) {
            if (rin[i] < 0 || rin[i] >= K) return TSTGEMM_EFORMAT;
            if (i > csn[n] && rin[i] <= rin[i - 1]) return TSTGEMM_EFORMAT;
        }
        // both lists ascending: one merge pass finds a row present in both
        int32_t i = csp[n], j = csn[n];
        while (i < csp[n + 1] && j < csn[n + 1]) {
            if (rip[i] == rin[j]) return TSTGEMM_EFORMAT;
            if (rip[i] < rin[j]) ++i; else ++j;
        }
    }
    return TSTGEMM_OK;
}

}  // namespace

extern "C" {

int tcsc_build(const int8_t *W, int K, int N, tcsc_t **out)
{
    if (!W || !out || K < 1 || N < 1) return TSTGEMM_EINVAL;
    *out = nullptr;
    try {
        // pass 1: entries per column and sign (row-major scan, so W is read sequentially)
        std::vector<int64_t> cnt_p((size_t)N + 1, 0), cnt_n((size_t)N + 1, 0);
        for (int k = 0; k < K; ++k) {
            const int8_t *row = W + (size_t)k * N;
            for (int n = 0; n < N; ++n) {
                const int8_t w = row[n];
                if (w == 1) ++cnt_p[n + 1];
                else if (w == -1) ++cnt_n[n + 1];
                else if (w != 0) return TSTGEMM_EFORMAT;
            }
        }
        for (int n = 0; n < N; ++n) { cnt_p[n + 1] += cnt_p[n]; cnt_n[n + 1] += cnt_n[n]; }
        // the inverted-index form numbers the entries of both signs together with 32-bit positions
        if (cnt_p[N] + cnt_n[N] > INT32_MAX) return TSTGEMM_ETOOBIG;
        tcsc *t = new tcsc;
        t->K = K;
        t->N = N;
        t->col_start_pos.assign(cnt_p.begin(), cnt_p.end());
        t->col_start_neg.assign(cnt_n.begin(), cnt_n.end());
        t->row_index_pos.resize((size_t)cnt_p[N]);
        t->row_index_neg.resize((size_t)cnt_n[N]);
        // pass 2: rows visited in ascending order, so every column's list comes out ascending
        std::vector<int32_t> fill_p(t->col_start_pos.begin(), t->col_start_pos.end() - 1);
        std::vector<int32_t> fill_n(t->col_start_neg.begin(), t->col_start_neg.end() - 1);
        for (int k = 0; k < K; ++k) {
            const int8_t *row = W + (size_t)k * N;
            for (int n = 0; n < N; ++n) {
                if (row[n] == 1) t->row_index_pos[(size_t)fill_p[n]++] = k;
                else if (row[n] == -1) t->row_index_neg[(size_t)fill_n[n]++] = k;
            }
        }
        compute_layout(t);
        *out = t;
        return TSTGEMM_OK;
    } catch (const std::bad_alloc &) {
        return TSTGEMM_ENOMEM;
    }
}

int tcsc_from_arrays(const int32_t *csp, const int32_t *csn, const int32_t *rip, const int32_t *rin, int K, int N,
                     tcsc_t **out)
{
    if (!csp || !csn || !out || K < 1 || N < 1) return TSTGEMM_EINVAL;
    *out = nullptr;
    if (csp[0] != 0 || csn[0] != 0) return TSTGEMM_EFORMAT;
    for (int n = 0; n < N; ++n)
        if (csp[n + 1] < csp[n] || csn[n + 1] < csn[n]) return TSTGEMM_EFORMAT;
    if ((csp[N] > 0 && !rip) || (csn[N] > 0 && !rin)) return TSTGEMM_EINVAL;
    if ((int64_t)csp[N] + (int64_t)csn[N] > INT32_MAX) return TSTGEMM_ETOOBIG;
    if (int rc = validate(csp, csn, rip, rin, K, N)) return rc;
    try {
        tcsc *t = new tcsc;
        t->K = K;
        t->N = N;
        t->col_start_pos.assign(csp, csp + N + 1);
        t->col_start_neg.assign(csn, csn + N + 1);
        t->row_index_pos.assign(rip, rip + csp[N]);
        t->row_index_neg.assign(rin, rin + csn[N]);
        compute_layout(t);
        *out = t;
        return TSTGEMM_OK;
    } catch (const std::bad_alloc &) {
        return TSTGEMM_ENOMEM;
    }
}

int tcsc_to_dense(const tcsc_t *t, int8_t *W_out)
{
    if (!t || !W_out) return TSTGEMM_EINVAL;
    std::memset(W_out, 0, (size_t)t->K * t->N);
    for (int n = 0; n < t->N; ++n) {
        for (int32_t i = t->col_start_pos[n]; i < t->col_start_pos[n + 1]; ++i)
            W_out[(size_t)t->row_index_pos[i] * t->N + n] = 1;
        for (int32_t i = t->col_start_neg[n]; i < t->col_start_neg[n + 1]; ++i)
            W_out[(size_t)t->row_index_neg[i] * t->N + n] = -1;
    }
    return TSTGEMM_OK;
}

int tcsc_dims(const tcsc_t *t, int *K, int *N, int64_t *nnz_pos, int64_t *nnz_neg)
{
    if (!t) return TSTGEMM_EINVAL;
    if (K) *K = t->K;
    if (N) *N = t->N;
    if (nnz_pos) *nnz_pos = (int64_t)t->row_index_pos.size();
    if (nnz_neg) *nnz_neg = (int64_t)t->row_index_neg.size();
    return TSTGEMM_OK;
}

int tcsc_arrays(const tcsc_t *t, const int32_t **csp, const int32_t **csn, const int32_t **rip, const int32_t **rin)
{
    if (!t) return TSTGEMM_EINVAL;
    if (csp) *csp = t->col_start_pos.data();
    if (csn) *csn = t->col_start_neg.data();
    if (rip) *rip = t->row_index_pos.data();
    if (rin) *rin = t->row_index_neg.data();
    return TSTGEMM_OK;
}

int tcsc_signed_arrays(const tcsc_t *t, int32_t *col_start, int32_t *index)
{
    if (!t || !col_start || (!index && !(t->row_index_pos.empty() && t->row_index_neg.empty()))) return TSTGEMM_EINVAL;
    int32_t out = 0;
    for (int n = 0; n < t->N; ++n) {
        col_start[n] = out;
        int32_t p = t->col_start_pos[n], q = t->col_start_neg[n];
        const int32_t p1 = t->col_start_pos[n + 1], q1 = t->col_start_neg[n + 1];
        while (p < p1 && q < q1) {
            if (t->row_index_pos[p] < t->row_index_neg[q]) index[out++] = t->row_index_pos[p++];
            else index[out++] = ~t->row_index_neg[q++];
        }
        while (p < p1) index[out++] = t->row_index_pos[p++];
        while (q < q1) index[out++] = ~t->row_index_neg[q++];
    }
    col_start[t->N] = out;
    return TSTGEMM_OK;
}

int tcsc_packed_codes(const tcsc_t *t, uint8_t *codes)
{
    if (!t || !codes) return TSTGEMM_EINVAL;
    static const uint8_t weight[5] = {81, 27, 9, 3, 1};   // value of digit 1 at row j of a group
    const size_t groups = (size_t)(t->K + 4) / 5;
    std::memset(codes, 0, groups * (size_t)t->N);
    for (int n = 0; n < t->N; ++n) {
        uint8_t *col = codes + (size_t)n * groups;
        for (int32_t i = t->col_start_pos[n]; i < t->col_start_pos[n + 1]; ++i)
            col[t->row_index_pos[i] / 5] += weight[t->row_index_pos[i] % 5];
        for (int32_t i = t->col_start_neg[n]; i < t->col_start_neg[n + 1]; ++i)
            col[t->row_index_neg[i] / 5] += 2 * weight[t->row_index_neg[i] % 5];
    }
    return TSTGEMM_OK;
}

int tcsc_device_bytes(const tcsc_t *t, size_t *bytes)
{
    if (!t || !bytes) return TSTGEMM_EINVAL;
    *bytes = t->layout.total_bytes;
    return TSTGEMM_OK;
}

int tcsc_layout(const tcsc_t *t, tcsc_layout_t *out)
{
    if (!t || !out) return TSTGEMM_EINVAL;
    *out = t->layout;
    return TSTGEMM_OK;
}

int tcsc_select_forms(tcsc_t *t, uint32_t forms)
{
    if (!t || (forms & ~TCSC_FORM_ALL)) return TSTGEMM_EINVAL;
    t->forms = forms;
    t->uploaded = false;
    compute_layout(t);
    return TSTGEMM_OK;
}

int tstgemm_workspace_bytes(int M, int K, int N, size_t *min_bytes, size_t *best_bytes)
{
    if (M < 1 || K < 1 || N < 1) return TSTGEMM_EINVAL;
    size_t lo = 0, hi = 0;
    if (M <= 8) {
        hi = tst::packed_partial_bytes(N);
    } else if (M <= 64) {
        // one tile of X, then partial sums of at most 8 K slices of all (padded) columns, 32 or 64 rows each
        lo = tst::small_tile_bytes(M, K);
        const size_t n_pad = ((size_t)N + tst::kColPad - 1) / tst::kColPad * tst::kColPad;
        hi = align_up(lo) + (size_t)tst::kMaxKSlices * n_pad * (M <= 32 ? 32 : 64) * sizeof(float);
        if ((long long)K * N >= (1LL << 30)) {
            // a matrix of this size can have lists too long for the small-tile kernel; then the large-M kernel runs
            size_t lo_large = 0, hi_large = 0;
            tst::large_workspace_bytes(M, K, (int)n_pad, &lo_large, &hi_large);
            lo = lo > lo_large ? lo : lo_large;
            hi = hi > hi_large ? hi : hi_large;
        }
    } else {
        const int n_pad = (N + tst::kColPad - 1) / tst::kColPad * tst::kColPad;
        tst::large_workspace_bytes(M, K, n_pad, &lo, &hi);
    }
    if (min_bytes) *min_bytes = lo;
    if (best_bytes) *best_bytes = hi;
    return TSTGEMM_OK;
}

int tcsc_upload(tcsc_t *t, void *dev_buf, size_t bytes, void *stream)
{
    if (!t || !dev_buf) return TSTGEMM_EINVAL;
    if (reinterpret_cast<uintptr_t>(dev_buf) % kAlign) return TSTGEMM_EINVAL;
    if (bytes < t->layout.total_bytes) return TSTGEMM_ENOMEM;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *d = static_cast<char *>(dev_buf);
    const tcsc_layout_t &l = t->layout;
    t->uploaded = false;
    t->dev = dev_buf;
    auto copy = [&](size_t off, const std::vector<int32_t> &v) {
        if (v.empty()) return hipSuccess;
        return hipMemcpyAsync(d + off, v.data(), v.size() * sizeof(int32_t), hipMemcpyHostToDevice, s);
    };
    if (copy(l.off_col_start_pos, t->col_start_pos) != hipSuccess) return TSTGEMM_EHIP;
    if (copy(l.off_col_start_neg, t->col_start_neg) != hipSuccess) return TSTGEMM_EHIP;
    if (copy(l.off_row_index_pos, t->row_index_pos) != hipSuccess) return TSTGEMM_EHIP;
    if (copy(l.off_row_index_neg, t->row_index_neg) != hipSuccess) return TSTGEMM_EHIP;
    std::vector<uint16_t> lists16_pos, lists16_neg;   // must outlive the copies: freed behind the synchronisation below
    if (l.has_lists16) {
        if (copy(l.off_col_start16_pos, t->col_start16_pos) != hipSuccess) return TSTGEMM_EHIP;
        if (copy(l.off_col_start16_neg, t->col_start16_neg) != hipSuccess) return TSTGEMM_EHIP;
        try {
            build_lists16(t->col_start_pos, t->row_index_pos, t->col_start16_pos, t->N, t->K, lists16_pos);
            build_lists16(t->col_start_neg, t->row_index_neg, t->col_start16_neg, t->N, t->K, lists16_neg);
        } catch (const std::bad_alloc &) {
            return TSTGEMM_ENOMEM;
        }
        if (hipMemcpyAsync(d + l.off_row_index16_pos, lists16_pos.data(), lists16_pos.size() * sizeof(uint16_t),
                           hipMemcpyHostToDevice, s) != hipSuccess ||
            hipMemcpyAsync(d + l.off_row_index16_neg, lists16_neg.data(), lists16_neg.size() * sizeof(uint16_t),
                           hipMemcpyHostToDevice, s) != hipSuccess)
            return TSTGEMM_EHIP;
    }
    // The sources are pageable host memory: wait until the copies have read them.
    if (hipStreamSynchronize(s) != hipSuccess) return TSTGEMM_EHIP;
    if (tst::launch_reblock(t, s) != hipSuccess) return TSTGEMM_EHIP;
    t->uploaded = true;
    return TSTGEMM_OK;
}

}  // extern "C"

namespace {

// One product: checks, the call's context from the options, dispatch on encoding and M.
int run(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, const tstgemm_opts_t &o, void *stream)
{
    if (!X || !t || !Y || M < 1) return TSTGEMM_EINVAL;
    if (K != t->K || N != t->N) return TSTGEMM_EINVAL;
    if (o.encoding < 0 || o.encoding > 2 || (o.encoding != 0 && (M > 8 || o.alpha))) return TSTGEMM_EINVAL;
    if (o.alpha && o.alpha_count != 1 && o.alpha_count != N) return TSTGEMM_EINVAL;
    if (o.cols_per_wave != 0 && o.cols_per_wave != 1 && o.cols_per_wave != 2 && o.cols_per_wave != 4 && o.cols_per_wave != 8)
        return TSTGEMM_EINVAL;
    if (o.k_slices < 0 || o.k_slices > tst::kMaxKSlices || o.slab_tiles < 0) return TSTGEMM_EINVAL;
    if (o.list_walk < 0 || o.list_walk > 2) return TSTGEMM_EINVAL;
    if ((o.event_before == nullptr) != (o.event_after == nullptr)) return TSTGEMM_EINVAL;
    if (o.workspace && reinterpret_cast<uintptr_t>(o.workspace) % kAlign) return TSTGEMM_EINVAL;
    if (!t->uploaded) return TSTGEMM_ENOTUPLOADED;
    const tcsc_layout_t &l = t->layout;

    tst::Call c{};
    c.stream = static_cast<hipStream_t>(stream);
    c.act = tst::Activation{o.alpha, (o.alpha && o.alpha_count != 1) ? 1 : 0};
    if (o.workspace) {
        c.ws = static_cast<char *>(o.workspace);
        c.ws_bytes = o.workspace_bytes;
    } else if (l.forms & TCSC_FORM_WORKSPACE) {
        c.ws = static_cast<char *>(t->dev) + l.off_workspace;
        c.ws_bytes = l.workspace_bytes;
    }
    c.cols_per_wave = o.cols_per_wave;
    c.k_slices = o.k_slices;
    c.slab_tiles = o.slab_tiles;
    c.list_walk = o.list_walk;
    c.decode_wide_lists = o.decode_wide_lists != 0;
    c.event_before = static_cast<hipEvent_t>(o.event_before);
    c.event_after = static_cast<hipEvent_t>(o.event_after);

    hipError_t e;
    if (o.encoding == 1) {
        if (!(l.forms & TCSC_FORM_SIGNED)) return TSTGEMM_ENOFORM;
        e = tst::launch_decode_signed(X, t, b, Y, M, c);
    } else if (o.encoding == 2) {
        if (!(l.forms & TCSC_FORM_PACKED)) return TSTGEMM_ENOFORM;
        e = tst::launch_packed(X, t, b, Y, M, c);
    } else if (tst::decode_supported(M)) {
        e = tst::launch_decode(X, t, b, Y, M, c);
    } else if (M <= 64 && tst::small_supported(l)) {
        if (!(l.forms & TCSC_FORM_CUTS)) return TSTGEMM_ENOFORM;
        e = tst::launch_small(X, t, b, Y, M, c);
    } else {
        if (!(l.forms & TCSC_FORM_ROWSETS)) return TSTGEMM_ENOFORM;
        e = tst::launch_large(X, t, b, Y, M, c);
    }
    return e == hipSuccess ? TSTGEMM_OK : e == tst::kErrWorkspace ? TSTGEMM_EWORKSPACE : TSTGEMM_EHIP;
}

tstgemm_opts_t default_opts()
{
    tstgemm_opts_t o{};
    o.struct_size = sizeof(o);
    return o;
}

}  // namespace

extern "C" {

int tstgemm_ex(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, const tstgemm_opts_t *opts,
               void *stream)
{
    if (opts && opts->struct_size != sizeof(tstgemm_opts_t)) return TSTGEMM_EINVAL;
    return run(X, t, b, Y, M, K, N, opts ? *opts : default_opts(), stream);
}

int tstgemm(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream)
{
    return run(X, t, b, Y, M, K, N, default_opts(), stream);
}

int tstgemm_prelu(const float *X, const tcsc_t *t, const float *b, const float *alpha, int alpha_count, float *Y, int M,
                  int K, int N, void *stream)
{
    if (!alpha || (alpha_count != 1 && alpha_count != N)) return TSTGEMM_EINVAL;
    tstgemm_opts_t o = default_opts();
    o.alpha = alpha;
    o.alpha_count = alpha_count;
    return run(X, t, b, Y, M, K, N, o, stream);
}

int tstgemm_signed(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream)
{
    tstgemm_opts_t o = default_opts();
    o.encoding = 1;
    return run(X, t, b, Y, M, K, N, o, stream);
}

int tstgemm_packed(const float *X, const tcsc_t *t, const float *b, float *Y, int M, int K, int N, void *stream)
{
    tstgemm_opts_t o = default_opts();
    o.encoding = 2;
    return run(X, t, b, Y, M, K, N, o, stream);
}

void tcsc_destroy(tcsc_t *t) { delete t; }

const char *tcsc_strerror(int code)
{
    switch (code) {
    case TSTGEMM_OK: return "ok";
    case TSTGEMM_EINVAL: return "invalid argument (null pointer, non-positive size, or K/N differ from the handle)";
    case TSTGEMM_EFORMAT: return "not a valid ternary matrix / TCSC structure";
    case TSTGEMM_ENOTUPLOADED: return "handle has no device form: call tcsc_upload first";
    case TSTGEMM_EHIP: return "a HIP runtime call failed";
    case TSTGEMM_ENOMEM: return "out of host memory, or device buffer too small";
    case TSTGEMM_ETOOBIG: return "matrix too large for 32-bit TCSC pointers";
    case TSTGEMM_ENOFORM: return "the device form this call reads was not selected when the matrix was uploaded";
    case TSTGEMM_EWORKSPACE: return "no workspace, or one smaller than tstgemm_workspace_bytes() gives as the minimum";
    case TSTGEMM_ESCRATCH: return "tstgemm_noalloc: the call needs more scratch memory than the library's static buffer holds";
    default: return "unknown tstgemm error code";
    }
}

}  // extern "C"
