"""Host-side checks of libtstgemm (no GPU): exported symbols, TCSC construction against the
oracle's, validation of user arrays, error codes, device-layout bookkeeping."""
import ctypes
import pathlib
import re

import numpy as np
import pytest

import oracle
import paper_2510_06957_amd as tg
import synth_inputs as si

ROOT = pathlib.Path(__file__).resolve().parent.parent


def declared_functions():
    names = set()
    for h in (ROOT / "include").glob("*.h"):
        text = re.sub(r"/\*.*?\*/", "", h.read_text(), flags=re.S)
        names |= set(re.findall(r"\b(t(?:csc|stgemm)\w*)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(str(tg.library_path()))
    names = declared_functions()
    assert {"tcsc_build", "tcsc_from_arrays", "tcsc_to_dense", "tcsc_dims", "tcsc_arrays", "tcsc_device_bytes",
            "tcsc_layout", "tcsc_upload", "tstgemm", "tstgemm_prelu", "tcsc_signed_arrays", "tcsc_packed_codes",
            "tstgemm_signed", "tstgemm_packed", "tstgemm_ex", "tstgemm_workspace_bytes", "tcsc_select_forms",
            "tstgemm_probe_lds_read", "tstgemm_probe_stream_read", "tstgemm_probe_tile_copy", "tcsc_destroy",
            "tcsc_strerror"} <= names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/ but not exported"


@pytest.mark.parametrize("K,N,density", [(1, 1, 1.0), (37, 5, 0.5), (513, 65, 0.5), (512, 512, 0.5), (300, 70, 0.0625),
                                         (64, 9, 0.0), (200, 3, 1.0)])
def test_build_matches_oracle_construction(K, N, density):
    W, _, _ = si.make_inputs(1, K, N, density, "uniform", seed=100 + K + N)
    t = tg.tcsc_build(W)
    o = oracle.tcsc_build(W)
    got = tg.tcsc_arrays(t)
    for a, e in zip(got, (o.col_start_pos, o.col_start_neg, o.row_index_pos, o.row_index_neg)):
        assert a.dtype == np.int32 and np.array_equal(a, e)
    assert (t.K, t.N, t.nnz_pos, t.nnz_neg) == (K, N, o.row_index_pos.size, o.row_index_neg.size)
    assert np.array_equal(tg.tcsc_to_dense(t), W)
    t2 = tg.tcsc_from_arrays(*got, K, N)
    assert np.array_equal(tg.tcsc_to_dense(t2), W)


def test_build_rejects_bad_input():
    W = np.zeros((4, 4), np.int8)
    W[1, 2] = 3
    with pytest.raises(tg.TstgemmError) as e:
        tg.tcsc_build(W)
    assert e.value.code == -2
    lib = ctypes.CDLL(str(tg.library_path()))
    out = ctypes.c_void_p()
    assert lib.tcsc_build(None, 4, 4, ctypes.byref(out)) == -1
    z = np.zeros(4, np.int8)
    assert lib.tcsc_build(ctypes.c_void_p(z.ctypes.data), 0, 4, ctypes.byref(out)) == -1
    assert lib.tcsc_build(ctypes.c_void_p(z.ctypes.data), 2, -2, ctypes.byref(out)) == -1


def good_arrays():
    W = np.array([[1, 0, -1], [0, 0, 1], [-1, 0, 1], [1, 0, 0]], np.int8)
    o = oracle.tcsc_build(W)
    return [o.col_start_pos.copy(), o.col_start_neg.copy(), o.row_index_pos.copy(), o.row_index_neg.copy()], 4, 3


@pytest.mark.parametrize("mutation", ["nonmonotone", "start_not_zero", "row_oob", "row_negative", "not_ascending",
                                      "duplicate", "both_lists"])
def test_from_arrays_validation(mutation):
    a, K, N = good_arrays()
    csp, csn, rip, rin = a
    if mutation == "nonmonotone":
        csp[1], csp[2] = 3, 2
    elif mutation == "start_not_zero":
        csn[0] = 1
    elif mutation == "row_oob":
        rip[0] = K
    elif mutation == "row_negative":
        rin[0] = -1
    elif mutation == "not_ascending":
        rip[0], rip[1] = rip[1], rip[0]
    elif mutation == "duplicate":
        rip[1] = rip[0]
    elif mutation == "both_lists":
        rin[0] = rip[0]          # column 0: row 0 would be +1 and -1 at once
    with pytest.raises(tg.TstgemmError) as e:
        tg.tcsc_from_arrays(csp, csn, rip, rin, K, N)
    assert e.value.code == -2


def test_not_uploaded_and_dimension_errors():
    a, K, N = good_arrays()
    t = tg.tcsc_from_arrays(*a, K, N)
    lib = ctypes.CDLL(str(tg.library_path()))
    lib.tstgemm.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 3 + [ctypes.c_void_p]
    fake = ctypes.c_void_p(4096)   # never dereferenced: the call must fail before touching memory
    assert lib.tstgemm(fake, t.handle, None, fake, 2, K, N, None) == -3
    assert lib.tstgemm(fake, t.handle, None, fake, 2, K + 1, N, None) == -1
    assert lib.tstgemm(fake, t.handle, None, fake, 0, K, N, None) == -1
    assert lib.tstgemm(None, t.handle, None, fake, 2, K, N, None) == -1
    # the two small-M variants: the same checks, and M <= 8 only
    for fn in (lib.tstgemm_signed, lib.tstgemm_packed):
        fn.argtypes = lib.tstgemm.argtypes
        assert fn(fake, t.handle, None, fake, 2, K, N, None) == -3
        assert fn(fake, t.handle, None, fake, 9, K, N, None) == -1
        assert fn(fake, t.handle, None, fake, 2, K, N + 1, None) == -1
        assert fn(None, t.handle, None, fake, 2, K, N, None) == -1
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert isinstance(tg.tcsc_strerror(code), str) and tg.tcsc_strerror(code)


def test_layout_bookkeeping():
    W, _, _ = si.make_inputs(1, 513, 65, 0.5, "uniform", seed=5)
    t = tg.tcsc_build(W)
    lay = tg.tcsc_layout(t)
    assert (lay.K, lay.N, lay.k_block) == (513, 65, 64)
    assert lay.n_pad % 64 == 0 and lay.n_pad >= 65 and lay.n_kblocks == -(-513 // 64)
    assert (lay.nnz_pos, lay.nnz_neg) == (int((W == 1).sum()), int((W == -1).sum()))
    assert lay.n_cuts == 3 and lay.n_chunks5 == 7          # 513 rows: 3 cuts of 256, 103 groups of five in 7 chunks of 16
    offs = [lay.off_col_start_pos, lay.off_col_start_neg, lay.off_row_index_pos, lay.off_row_index_neg,
            lay.off_masks, lay.off_list_cuts, lay.off_col_start16_pos, lay.off_col_start16_neg, lay.off_row_index16_pos,
            lay.off_row_index16_neg, lay.off_signed_index, lay.off_packed, lay.off_workspace, lay.total_bytes]
    assert all(o % 256 == 0 for o in offs) and offs == sorted(offs)
    assert lay.total_bytes == tg.tcsc_device_bytes(t)
    assert lay.off_list_cuts - lay.off_masks >= 16 * lay.n_kblocks * lay.n_pad
    # the padded 16-bit lists: every column rounded up to 8 entries
    o = oracle.tcsc_build(W)
    assert lay.has_lists16 == 1
    assert lay.nnz16_pos == int((-(-np.diff(o.col_start_pos) // 8) * 8).sum())
    assert lay.nnz16_neg == int((-(-np.diff(o.col_start_neg) // 8) * 8).sum())
    assert lay.off_col_start16_pos - lay.off_list_cuts >= 8 * (lay.n_cuts + 1) * lay.n_pad
    assert lay.off_row_index16_neg - lay.off_row_index16_pos >= 2 * lay.nnz16_pos
    assert lay.off_signed_index - lay.off_row_index16_neg >= 2 * lay.nnz16_neg
    assert lay.off_packed - lay.off_signed_index >= 4 * (lay.nnz_pos + lay.nnz_neg)
    wide = tg.tcsc_layout(tg.tcsc_build(np.zeros((65536, 1), np.int8)))       # K itself must fit in 16 bits: no copy here
    assert wide.has_lists16 == 0 and wide.nnz16_pos == 0 and wide.off_row_index16_neg == 0
    assert not wide.forms & tg.FORM_LISTS16
    assert lay.off_workspace - lay.off_packed >= 16 * lay.n_chunks5 * lay.n_pad
    assert lay.total_bytes - lay.off_workspace >= lay.workspace_bytes > 0


def test_options_reject_bad_values():
    """tstgemm_ex() checks its options before anything else, so a handle without a device form is enough here (the
    valid combinations then stop at "not uploaded"); X and Y only have to be non-null."""
    lib = tg.binding._load()
    t = tg.tcsc_build(np.zeros((64, 8), np.int8))
    fake = ctypes.c_void_p(256)

    def call(M=100, **fields):
        o = tg.binding.TstgemmOpts()
        o.struct_size = ctypes.sizeof(o)
        for k, v in fields.items():
            setattr(o, k, v)
        return lib.tstgemm_ex(fake, t.handle, None, fake, M, 64, 8, ctypes.byref(o), None)

    assert call() == -3 and lib.tstgemm_ex(fake, t.handle, None, fake, 100, 64, 8, None, None) == -3
    assert call(struct_size=8) == -1
    assert call(cols_per_wave=3) == -1 and call(k_slices=9) == -1 and call(k_slices=-1) == -1 and call(slab_tiles=-1) == -1
    assert call(cols_per_wave=4, k_slices=8, slab_tiles=2) == -3
    assert call(list_walk=3) == -1 and call(list_walk=-1) == -1 and call(list_walk=2) == -3
    assert call(event_before=1) == -1 and call(event_after=1) == -1 and call(event_before=1, event_after=2) == -3
    assert call(encoding=3) == -1 and call(encoding=-1) == -1
    assert call(encoding=1) == -1 and call(M=8, encoding=1) == -3 and call(M=8, encoding=2) == -3   # M <= 8 only
    assert call(M=8, encoding=1, alpha=256, alpha_count=1) == -1                                   # PReLU: TCSC path only
    assert call(alpha=256, alpha_count=3) == -1 and call(alpha=256, alpha_count=8) == -3
    assert call(workspace=100, workspace_bytes=1 << 20) == -1                                      # not 256-byte aligned
    assert call(workspace=512, workspace_bytes=1 << 20) == -3


def test_probes_reject_bad_arguments():
    """The measurement probes check their arguments before they launch anything (no GPU needed for the refusals)."""
    lib = tg.binding._load()
    n = ctypes.c_int64(0)
    fake = ctypes.c_void_p(256)
    assert lib.tstgemm_probe_lds_read(0, ctypes.byref(n), None) == -1
    assert lib.tstgemm_probe_stream_read(None, 1 << 20, None) == -1 and lib.tstgemm_probe_stream_read(fake, 8, None) == -1
    assert lib.tstgemm_probe_tile_copy(None, 1 << 20, 1, ctypes.byref(n), None) == -1
    assert lib.tstgemm_probe_tile_copy(fake, 65535, 1, ctypes.byref(n), None) == -1          # less than one 64 KiB piece
    assert lib.tstgemm_probe_tile_copy(ctypes.c_void_p(260), 1 << 20, 1, ctypes.byref(n), None) == -1   # not 16-byte aligned
    assert lib.tstgemm_probe_tile_copy(fake, 1 << 20, 0, ctypes.byref(n), None) == -1
    assert n.value == 0


def test_selected_forms_shrink_the_device_buffer():
    """A handle only pays for the forms its calls read: the benchmark's smallest configuration with the row sets
    alone (a caller-supplied workspace) needs under 2 MB, where all forms and the built-in workspace take 160 MiB."""
    W, _, _ = si.make_workload("C1")
    t = tg.tcsc_build(W)
    everything = tg.tcsc_device_bytes(t)
    assert tg.tcsc_layout(t).forms == tg.FORM_ALL and everything > 160 << 20
    tg.tcsc_select_forms(t, tg.FORM_ROWSETS)
    lay = tg.tcsc_layout(t)
    assert lay.forms == tg.FORM_ROWSETS and tg.tcsc_device_bytes(t) == lay.total_bytes < 2_000_000
    assert lay.workspace_bytes == 0 and lay.off_list_cuts == 0 and lay.off_signed_index == 0 and lay.off_packed == 0
    assert lay.has_lists16 == 0 and lay.off_masks > lay.off_row_index_neg > lay.off_row_index_pos > 0
    tg.tcsc_select_forms(t, tg.FORM_PACKED)                      # the codes are built from the row sets
    assert tg.tcsc_layout(t).forms == tg.FORM_PACKED | tg.FORM_ROWSETS
    tg.tcsc_select_forms(t, 0)                                   # the TCSC arrays alone (M <= 8 on 32-bit lists)
    assert tg.tcsc_layout(t).forms == 0 and tg.tcsc_device_bytes(t) < everything - (160 << 20)
    with pytest.raises(tg.TstgemmError):
        tg.tcsc_select_forms(t, 64)
    tg.tcsc_select_forms(t, tg.FORM_ALL)
    assert tg.tcsc_device_bytes(t) == everything


def test_workspace_bytes():
    """tstgemm_workspace_bytes: nothing for M <= 8 (but the packed kernel's partial sums), one tile of X as the
    minimum of the tiled paths, all tiles plus the partial sums of the K slices as the best."""
    lo, hi = tg.tstgemm_workspace_bytes(1, 4096, 11008)
    assert lo == 0 and 0 < hi < 16 << 20
    lo, hi = tg.tstgemm_workspace_bytes(64, 16384, 4096)
    assert lo == 64 * 16384 * 4 and lo < hi <= lo + 8 * 4096 * 64 * 4
    assert tg.tstgemm_workspace_bytes(20, 1000, 64)[0] == 32 * 1024 * 4        # tile of 32 rows, K padded to 512-row blocks
    lo, hi = tg.tstgemm_workspace_bytes(256, 4096, 4096)
    assert lo == 256 * 4096 * 4 and hi == lo + 8 * 256 * 4096 * 4               # C2: one tile + 8 K slices of Y
    lo, hi = tg.tstgemm_workspace_bytes(4096, 8192, 8192)
    assert lo == 256 * 8192 * 4 and hi == 16 * lo                               # C5: 16 tiles, K not sliced
    assert tg.tstgemm_workspace_bytes(100, 70, 5)[0] == 128 * 128 * 4           # 128-row tile, K padded to 128
    # a matrix that can hold 2^30 entries per sign may have to go through the large-M kernel for any M > 8 (the
    # small-tile kernel addresses its lists with 32-bit byte offsets): the figures then cover both
    lo, hi = tg.tstgemm_workspace_bytes(64, 65536, 65536)
    lo_l, hi_l = tg.tstgemm_workspace_bytes(128, 65536, 65536)
    assert lo == max(64 * 65536 * 4, lo_l) and hi >= hi_l
    lib = tg.binding._load()
    assert lib.tstgemm_workspace_bytes(0, 1, 1, None, None) == -1 and lib.tstgemm_workspace_bytes(1, 1, 1, None, None) == 0


def test_too_many_entries_for_the_signed_form():
    """The inverted-index form numbers the entries of both signs together with 32-bit positions: arrays whose two
    lists have more than 2^31 - 1 entries together are refused before anything is read."""
    lib = tg.binding._load()
    big = np.array([0, 2 ** 30], np.int32)
    out = ctypes.c_void_p()
    one = np.zeros(1, np.int32)
    rc = lib.tcsc_from_arrays(big.ctypes.data, big.ctypes.data, one.ctypes.data, one.ctypes.data, 2 ** 30, 1,
                              ctypes.byref(out))
    assert rc == -6 and not out.value


@pytest.mark.parametrize("K,N,density", [(1, 1, 1.0), (37, 5, 0.5), (513, 65, 0.5), (64, 9, 1.0), (130, 70, 0.0),
                                         (1000, 33, 0.0625)])
def test_other_encodings_match_the_oracle(K, N, density):
    """The host exporters of the inverted-index and value-compression encodings (Sec. 3) against the oracle's."""
    W, _, _ = si.make_inputs(1, K, N, density, "uniform", seed=150 + K + N)
    t = tg.tcsc_build(W)
    cs, idx = tg.tcsc_signed_arrays(t)
    ocs, oidx = oracle.signed_build(oracle.tcsc_build(W))
    assert np.array_equal(cs, ocs) and np.array_equal(idx, oidx)
    assert np.array_equal(tg.tcsc_packed_codes(t), oracle.pack5(W))
    assert np.array_equal(oracle.unpack5(tg.tcsc_packed_codes(t), K), W)


def test_random_small_matrices_round_trip():
    """Many small random ternary matrices of random shape and density, including empty and full ones: the library's
    builder, its three exporters and from_arrays/to_dense against the oracle's construction and the matrix itself."""
    rng = np.random.default_rng(2025)
    for _ in range(200):
        K, N = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        density = float(rng.choice([0.0, 0.1, 0.5, 0.9, 1.0]))
        u = rng.random((K, N))
        W = np.where(u < density / 2, 1, np.where(u < density, -1, 0)).astype(np.int8)
        t = tg.tcsc_build(W)
        o = oracle.tcsc_build(W)
        arrays = tg.tcsc_arrays(t)
        for a, e in zip(arrays, (o.col_start_pos, o.col_start_neg, o.row_index_pos, o.row_index_neg)):
            assert np.array_equal(a, e)
        assert np.array_equal(tg.tcsc_to_dense(tg.tcsc_from_arrays(*arrays, K, N)), W)
        cs, idx = tg.tcsc_signed_arrays(t)
        assert np.array_equal(oracle.signed_to_dense(cs, idx, K), W)
        assert np.array_equal(oracle.unpack5(tg.tcsc_packed_codes(t), K), W)


def test_header_is_plain_c(tmp_path):
    """include/tstgemm.h must be usable from C: it compiles as C99 with all warnings on, and a C program can call
    the host-side entry points through it (linked against the built library)."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text(r'''
#include <stdio.h>
#include "tstgemm.h"
int main(void)
{
    const int8_t W[6] = {1, 0, -1, 0, 1, -1};   /* K = 2, N = 3 */
    tcsc_t *t = NULL;
    int K = 0, N = 0;
    int64_t p = 0, q = 0;
    size_t bytes = 0;
    uint8_t codes[3];
    if (tcsc_build(W, 2, 3, &t) != TSTGEMM_OK) return 1;
    if (tcsc_dims(t, &K, &N, &p, &q) != TSTGEMM_OK || K != 2 || N != 3 || p != 2 || q != 2) return 2;
    if (tcsc_device_bytes(t, &bytes) != TSTGEMM_OK || bytes == 0) return 3;
    if (tcsc_packed_codes(t, codes) != TSTGEMM_OK) return 4;
    /* column 0 = (1, 0) -> 81; column 1 = (0, 1) -> 27; column 2 = (-1, -1) -> 2*81 + 2*27 = 216 */
    if (codes[0] != 81 || codes[1] != 27 || codes[2] != 216) return 5;
    if (tstgemm(NULL, t, NULL, NULL, 1, 2, 3, NULL) != TSTGEMM_EINVAL) return 6;
    printf("%s\n", tcsc_strerror(TSTGEMM_ENOTUPLOADED));
    tcsc_destroy(t);
    return 0;
}
''')
    exe = tmp_path / "use_header"
    lib = tg.library_path()
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", f"-I{ROOT / 'include'}", str(src), "-o", str(exe),
           str(lib), f"-Wl,-rpath,{lib.parent}", "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr)
    assert "tcsc_upload" in r.stdout
