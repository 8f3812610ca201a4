"""Host-side checks of the C-ABI library: it loads, exports every symbol that
include/sa.h declares, sizes workspaces, and rejects bad arguments with the
documented status codes BEFORE anything is launched (so no GPU is needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sa.h")

SA_OK, SA_INVALID, SA_UNSUPPORTED, SA_WORKSPACE, SA_DEVICE = 0, 1, 2, 3, 4
FAKE = ctypes.c_void_p(0x10000)      # non-null, 256-aligned, never dereferenced on the host


@pytest.fixture(scope="module")
def lib():
    import paper_2406_15486_amd as sa
    return sa.load_library()


@pytest.fixture(scope="module")
def B():
    import paper_2406_15486_amd.binding as b
    return b


def _shape(B, **kw):
    d = dict(batch=1, n_q_heads=4, n_kv_heads=2, seq_len=512, head_dim=128, causal=1, softmax_scale=0.0)
    d.update(kw)
    return B._CShape(*[d[k] for k in ("batch", "n_q_heads", "n_kv_heads", "seq_len", "head_dim", "causal",
                                      "softmax_scale")])


def test_library_exports_every_declared_symbol(lib):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(sa_[a-z_0-9]+)\s*\(", text))
    assert {"sa_sample_scores", "sa_select_strips", "sa_sparse_attn", "sa_dense_attn",
            "sa_workspace_bytes"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in sa.h but not exported"


def test_version_and_status_strings(lib):
    assert lib.sa_version() >= 100
    seen = {lib.sa_status_string(i) for i in range(5)}
    assert len(seen) == 5 and all(seen)
    assert lib.sa_status_string(99)


def test_rows_from_ratio(lib):
    assert lib.sa_rows_from_ratio(1024, 0.05) == 64
    assert lib.sa_rows_from_ratio(8192, 0.05) == 448
    assert lib.sa_rows_from_ratio(131072, 0.05) == 6592
    assert lib.sa_rows_from_ratio(1048576, 0.02) == 20992
    assert lib.sa_rows_from_ratio(40, 0.5) == 40
    assert lib.sa_rows_from_ratio(0, 0.5) == 0 and lib.sa_rows_from_ratio(100, 0.0) == 0


def test_workspace_bytes(lib, B):
    sh = _shape(B)
    sm = B._CSampling(64, 1, 1)
    for op in (0, 2, 3):
        n = lib.sa_workspace_bytes(op, ctypes.byref(sh), ctypes.byref(sm))
        assert n > 0 and n % 256 == 0
    assert lib.sa_workspace_bytes(1, ctypes.byref(sh), None) == 0          # selection needs none
    assert lib.sa_workspace_bytes(7, ctypes.byref(sh), None) == 0          # unknown op
    assert lib.sa_workspace_bytes(3, None, None) == 0
    bad = _shape(B, head_dim=64)
    assert lib.sa_workspace_bytes(3, ctypes.byref(bad), None) == 0
    # grows with the sequence
    big = _shape(B, seq_len=4096)
    assert lib.sa_workspace_bytes(2, ctypes.byref(big), None) > lib.sa_workspace_bytes(2, ctypes.byref(sh), None)


def _dense(lib, sh, ws=FAKE, ws_bytes=1 << 40, q=FAKE, out_dtype=0):
    return lib.sa_dense_attn(ctypes.byref(sh) if sh is not None else None, q, FAKE, FAKE, FAKE, out_dtype, None,
                             ws, ws_bytes, None)


def test_shape_validation(lib, B):
    assert _dense(lib, None) == SA_INVALID
    assert _dense(lib, _shape(B, seq_len=0)) == SA_INVALID
    assert _dense(lib, _shape(B, batch=0)) == SA_INVALID
    assert _dense(lib, _shape(B, n_q_heads=3)) == SA_INVALID               # not a multiple of kv heads
    assert _dense(lib, _shape(B, softmax_scale=-1.0)) == SA_INVALID
    assert _dense(lib, _shape(B, softmax_scale=float("nan"))) == SA_INVALID
    assert _dense(lib, _shape(B, head_dim=64)) == SA_UNSUPPORTED
    assert _dense(lib, _shape(B, causal=0)) == SA_UNSUPPORTED


def test_pointer_and_workspace_validation(lib, B):
    sh = _shape(B)
    assert _dense(lib, sh, q=None) == SA_INVALID
    assert _dense(lib, sh, out_dtype=5) == SA_INVALID
    assert _dense(lib, sh, ws=None) == SA_WORKSPACE
    assert _dense(lib, sh, ws_bytes=16) == SA_WORKSPACE
    assert _dense(lib, sh, ws=ctypes.c_void_p(0x10004)) == SA_WORKSPACE      # misaligned


def test_sampling_validation(lib, B):
    sh = _shape(B)

    def call(sm, col=FAKE):
        return lib.sa_sample_scores(ctypes.byref(sh), ctypes.byref(sm) if sm is not None else None, FAKE, FAKE,
                                    col, FAKE, None, FAKE, 16, None)

    assert call(None) == SA_INVALID
    assert call(B._CSampling(0, 1, 1)) == SA_INVALID
    assert call(B._CSampling(1024, 1, 1)) == SA_INVALID                     # more rows than the sequence
    assert call(B._CSampling(50, 1, 1)) == SA_WORKSPACE                     # any row count is valid; 16 bytes is too small
    assert call(B._CSampling(64, 3, 1)) == SA_WORKSPACE                     # ragged segments (170 + 170 + 172 rows) are valid
    assert call(B._CSampling(171, 3, 1)) == SA_INVALID                      # more rows than a segment of floor(512 / 3) holds
    assert call(B._CSampling(288, 2, 1)) == SA_INVALID                      # more rows than a segment holds
    assert call(B._CSampling(1, 513, 1)) == SA_INVALID                      # more chunks than rows
    assert call(B._CSampling(64, 2, 1)) == SA_WORKSPACE                     # valid; 16 bytes is too small
    assert lib.sa_sample_scores(ctypes.byref(sh), ctypes.byref(B._CSampling(64, 2, 1)), FAKE, FAKE, FAKE, FAKE,
                                FAKE, FAKE, 1 << 40, None) == SA_UNSUPPORTED   # no row_lse output with chunks
    assert call(B._CSampling(64, 1, 100)) == SA_UNSUPPORTED                 # block sizes: 64, 128, 256
    assert call(B._CSampling(64, 1, 0)) == SA_INVALID
    assert call(B._CSampling(64, 1, 128)) == SA_WORKSPACE                   # valid; 16 bytes is too small
    assert call(B._CSampling(64, 1, 1), col=None) == SA_INVALID
    assert call(B._CSampling(64, 1, 1)) == SA_WORKSPACE                     # 16 bytes is too small


def test_sample_scores_least_workspace(lib, B):
    sh = _shape(B, n_q_heads=8, n_kv_heads=2, seq_len=4096)
    sm = B._CSampling(256, 1, 1)
    full = lib.sa_workspace_bytes(0, ctypes.byref(sh), ctypes.byref(sm))
    least = lib.sa_workspace_bytes(5, ctypes.byref(sh), ctypes.byref(sm))
    assert 0 < least <= full // 7 and least % 256 == 0      # one head of eight
    assert lib.sa_workspace_bytes(5, ctypes.byref(sh), ctypes.byref(B._CSampling(0, 1, 1))) == 0
    # a workspace below the least is refused before anything is launched
    assert lib.sa_sample_scores(ctypes.byref(sh), ctypes.byref(sm), FAKE, FAKE, FAKE, FAKE, None, FAKE,
                                least - 256, None) == SA_WORKSPACE


def test_select_and_sparse_validation(lib, B):
    sh = _shape(B)

    def sel(ac, as_, idx=FAKE):
        return lib.sa_select_strips(ctypes.byref(sh), FAKE, FAKE, ctypes.c_float(ac), ctypes.c_float(as_),
                                    idx, FAKE, FAKE, FAKE, None, 0, None)

    assert sel(-0.1, 0.5) == SA_INVALID
    assert sel(1.5, 0.5) == SA_INVALID                                       # thresholds are fractions
    assert sel(0.5, float("inf")) == SA_INVALID
    assert sel(0.5, float("nan")) == SA_INVALID
    assert sel(0.5, 0.5, idx=None) == SA_INVALID

    def sparse(window, cnt=FAKE, ws_bytes=16):
        return lib.sa_sparse_attn(ctypes.byref(sh), FAKE, FAKE, FAKE, FAKE, cnt, FAKE, FAKE, window, FAKE, 0,
                                  None, None, FAKE, ws_bytes, None)

    assert sparse(0) == SA_INVALID                                           # every row must keep its diagonal
    assert sparse(4, cnt=None) == SA_INVALID
    assert sparse(4) == SA_WORKSPACE


def test_block_entry_points_validation(lib, B):
    sh = _shape(B)
    assert lib.sa_block_scores(ctypes.byref(sh), 128, FAKE, FAKE, FAKE, None, None) == SA_INVALID
    assert lib.sa_block_scores(ctypes.byref(sh), 0, FAKE, FAKE, FAKE, FAKE, None) == SA_INVALID
    assert lib.sa_block_scores(ctypes.byref(sh), 96, FAKE, FAKE, FAKE, FAKE, None) == SA_UNSUPPORTED

    def sel(g, ac=0.5):
        return lib.sa_select_blocks(ctypes.byref(sh), g, FAKE, FAKE, ctypes.c_float(ac), ctypes.c_float(0.5),
                                    FAKE, FAKE, FAKE, FAKE, None, 0, None)

    assert sel(0) == SA_INVALID
    assert sel(1) == SA_UNSUPPORTED                                          # per-token: sa_select_strips
    assert sel(32) == SA_UNSUPPORTED
    assert sel(128, ac=-1.0) == SA_INVALID

    def attn(g, window=4, ws_bytes=16, cnt=FAKE):
        return lib.sa_block_sparse_attn(ctypes.byref(sh), g, FAKE, FAKE, FAKE, FAKE, cnt, FAKE, FAKE, window,
                                        FAKE, 0, None, None, FAKE, ws_bytes, None)

    assert attn(-1) == SA_INVALID
    assert attn(1) == SA_UNSUPPORTED
    assert attn(512) == SA_UNSUPPORTED
    assert attn(128, window=0) == SA_INVALID
    assert attn(128, cnt=None) == SA_INVALID
    assert attn(128) == SA_WORKSPACE
    # the block path reads its key blocks in place: no gathered K / V copies in its workspace
    sm = B._CSampling(0, 1, 128)
    nb = lib.sa_workspace_bytes(4, ctypes.byref(sh), ctypes.byref(sm))
    assert 0 < nb < lib.sa_workspace_bytes(2, ctypes.byref(sh), None) // 4 and nb % 256 == 0
    assert lib.sa_workspace_bytes(4, ctypes.byref(sh), None) == 0
    assert lib.sa_workspace_bytes(4, ctypes.byref(sh), ctypes.byref(B._CSampling(0, 1, 100))) == 0
    # sampling at block granularity needs room for the per-token scores as well
    s1 = lib.sa_workspace_bytes(0, ctypes.byref(sh), ctypes.byref(B._CSampling(64, 1, 1)))
    s128 = lib.sa_workspace_bytes(0, ctypes.byref(sh), ctypes.byref(B._CSampling(64, 1, 128)))
    assert s128 >= s1 + 2 * 4 * 512 * 4


def test_chunked_entry_points_validation(lib, B):
    sh = _shape(B)

    def sel(sm, ac=0.5):
        return lib.sa_select_chunked(ctypes.byref(sh), ctypes.byref(sm) if sm is not None else None, FAKE, FAKE,
                                     ctypes.c_float(ac), ctypes.c_float(0.5), FAKE, FAKE, FAKE, FAKE, None, 0, None)

    assert sel(None) == SA_INVALID
    assert sel(B._CSampling(0, 0, 1)) == SA_INVALID
    assert sel(B._CSampling(0, 600, 1)) == SA_INVALID                      # more chunks than rows
    assert sel(B._CSampling(0, 2, 100)) == SA_UNSUPPORTED
    assert sel(B._CSampling(0, 2, 1), ac=-1.0) == SA_INVALID

    def attn(sm, window=4, ws_bytes=16):
        return lib.sa_sparse_attn_chunked(ctypes.byref(sh), ctypes.byref(sm) if sm is not None else None, FAKE, FAKE,
                                          FAKE, FAKE, FAKE, FAKE, FAKE, window, FAKE, 0, None, None, FAKE, ws_bytes,
                                          None)

    assert attn(None) == SA_INVALID
    assert attn(B._CSampling(0, 3, 1)) == SA_WORKSPACE                     # ragged segments are valid
    assert attn(B._CSampling(0, 600, 1)) == SA_INVALID
    assert attn(B._CSampling(0, 2, 1), window=0) == SA_INVALID
    assert attn(B._CSampling(0, 2, 1)) == SA_WORKSPACE
    assert attn(B._CSampling(0, 2, 128)) == SA_WORKSPACE


def test_partitioned_entry_point_validation(lib, B):
    sh = _shape(B, n_q_heads=8, seq_len=4096)
    full = lib.sa_workspace_bytes(2, ctypes.byref(sh), None)

    def need(hpp, segs):
        return lib.sa_partitioned_workspace_bytes(ctypes.byref(sh), ctypes.byref(B._CPartition(hpp, segs)))

    assert need(0, 1) == 0 and need(1, 0) == 0
    assert lib.sa_partitioned_workspace_bytes(ctypes.byref(sh), None) == 0
    assert need(8, 1) == full and need(100, 7) == full            # clamped to the number of heads
    assert need(2, 1) < need(4, 1) < full
    per_head = (need(4, 1) - need(2, 1)) // 2
    assert 4096 * 516 <= per_head <= 4096 * 560                   # gathered K, V^T, index list, bitmaps

    def call(part, ws_bytes=16):
        return lib.sa_sparse_attn_partitioned(ctypes.byref(sh), ctypes.byref(part) if part is not None else None,
                                              FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, FAKE, 0, None, None,
                                              FAKE, ws_bytes, None)

    assert call(None) == SA_INVALID
    assert call(B._CPartition(0, 1)) == SA_INVALID
    assert call(B._CPartition(2, -1)) == SA_INVALID
    assert call(B._CPartition(2, 4)) == SA_WORKSPACE


def test_static_scratch_entry_point_limit(lib, B):
    """sa_dense_attn_static keeps V^T in a 16 MiB static device array: a shape that needs
    more is refused before anything is launched."""
    fits = B._CShape(1, 4, 2, 32768, 128, 1, 0.0)          # 2 * 32768 * 128 * 2 bytes = 16 MiB exactly
    too_big = B._CShape(1, 4, 2, 32769, 128, 1, 0.0)
    assert lib.sa_dense_attn_static(ctypes.byref(too_big), FAKE, FAKE, FAKE, FAKE, 0, None, None) == 5
    assert lib.sa_dense_attn_static(ctypes.byref(fits), FAKE, FAKE, FAKE, None, 0, None, None) == SA_INVALID
    assert lib.sa_dense_attn_static(ctypes.byref(fits), FAKE, FAKE, FAKE, FAKE, 7, None, None) == SA_INVALID
    assert b"static scratch" in lib.sa_status_string(5)


def test_profile_read_before_enable(lib):
    buf = (ctypes.c_float * 4)()
    assert lib.sa_profile_read(99, buf, 4) == -1
    assert lib.sa_profile_read(0, None, 4) == -1
