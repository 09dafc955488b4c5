"""Host-side checks of the C-ABI library (no GPU): it loads, exports every symbol that
include/graft.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "graft.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2605_20104_amd as g
    if not os.path.exists(g.LIB_PATH):
        from paper_2605_20104_amd import build
        build.build()
    return g.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(graft_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    import paper_2605_20104_amd as g
    names = declared_functions()
    assert {"graft_retrieve", "graft_build_tree_mask", "graft_tree_attn", "graft_accept"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None
    assert sorted(g.EXPORTED_SYMBOLS) == names


def test_timing_build_is_the_same_interface_plus_its_own_calls(lib):
    """libgraft_timing.so (the attention kernel with time stamps) exports everything the header
    declares and the calls of the timing tool; the product library has none of those."""
    from paper_2605_20104_amd import build
    if not os.path.exists(build.LIB_TIMING):
        pytest.skip("libgraft_timing.so is not built (python -m paper_2605_20104_amd.build --timing)")
    timing = ctypes.CDLL(build.LIB_TIMING)
    for n in declared_functions():
        assert getattr(timing, n) is not None
    for n in ("graft_attn_stamp_buffer", "graft_attn_stamp_count", "graft_attn_force_plan", "graft_mfma_calibration"):
        assert getattr(timing, n) is not None
        assert not hasattr(lib, n), n
    assert timing.graft_attn_stamp_count() == 24
    timing.graft_mfma_calibration.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int32] * 3 + [ctypes.c_void_p]
    assert timing.graft_mfma_calibration(None, None, None, 1, 256, 1, None) == 1           # GRAFT_ERR_NULL
    one = ctypes.c_void_p(8)                                                                # never dereferenced: the shape is refused first
    assert timing.graft_mfma_calibration(one, one, one, 1, 300, 1, None) == 2              # GRAFT_ERR_SHAPE
    assert timing.graft_mfma_calibration(one, one, one, 0, 256, 1, None) == 2
    # a held plan changes the workspace the same call asks for, and zeros give it back
    args = (1, 64, 40, 8, 128, 2052, 1)
    timing.graft_tree_attn_workspace_bytes.restype = ctypes.c_size_t
    auto = timing.graft_tree_attn_workspace_bytes(*args)
    timing.graft_attn_force_plan(16, 1)
    held = timing.graft_tree_attn_workspace_bytes(*args)
    timing.graft_attn_force_plan(0, 0)
    assert held != auto and timing.graft_tree_attn_workspace_bytes(*args) == auto


def test_header_constants_match_binding():
    import paper_2605_20104_amd as g
    text = open(HEADER).read()
    for name in ("GRAFT_MAX_NODES", "GRAFT_MASK_WORDS", "GRAFT_MAX_CHAINS", "GRAFT_MAX_NGRAM",
                 "GRAFT_PAGE_SIZE", "GRAFT_MAX_SUCCESSORS", "GRAFT_MAX_CHECKPOINTS", "GRAFT_ERR_NULL", "GRAFT_ERR_SHAPE", "GRAFT_ERR_DTYPE",
                 "GRAFT_ERR_WORKSPACE", "GRAFT_ERR_HIP", "GRAFT_STATUS_BAD_LENGTH", "GRAFT_STATUS_BAD_TREE",
                 "GRAFT_STATUS_PATH_OVERFLOW", "GRAFT_F32", "GRAFT_BF16"):
        m = re.search(r"#define\s+%s\s+(\d+)" % name, text)
        assert m and int(m.group(1)) == getattr(g, name), name


def test_version_and_error_state(lib):
    assert lib.graft_version() >= 100
    assert lib.graft_last_hip_error() == 0


P = 0x1000      # a non-NULL placeholder: validation must fail before any pointer is touched


def test_retrieve_validation(lib):
    import paper_2605_20104_amd as g
    f = lib.graft_retrieve
    ok = [P, P, 1, 64, None, None, 0, 2, 4, 2, 4, P, P, P, P, P, P, None]

    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return f(*a)
    assert call(a0=None) == g.GRAFT_ERR_NULL
    assert call(a11=None) == g.GRAFT_ERR_NULL
    assert call(a4=P) == g.GRAFT_ERR_NULL                 # tail without tail_len
    assert call(a2=0) == g.GRAFT_ERR_SHAPE                # B
    assert call(a3=0) == g.GRAFT_ERR_SHAPE                # L_max
    assert call(a7=0) == g.GRAFT_ERR_SHAPE                # n_min < 1
    assert call(a7=5) == g.GRAFT_ERR_SHAPE                # n_min > n_max
    assert call(a8=g.GRAFT_MAX_NGRAM + 1) == g.GRAFT_ERR_SHAPE
    assert call(a9=g.GRAFT_MAX_CHAINS + 1) == g.GRAFT_ERR_SHAPE
    assert call(a9=0) == g.GRAFT_ERR_SHAPE
    assert call(a10=0) == g.GRAFT_ERR_SHAPE


def test_tree_mask_validation(lib):
    import paper_2605_20104_amd as g
    f = lib.graft_build_tree_mask
    assert f(None, P, P, 1, 16, P, P, P, None, 0, 0, P, None) == g.GRAFT_ERR_NULL
    assert f(P, P, P, 1, 16, P, P, P, None, 0, 0, None, None) == g.GRAFT_ERR_NULL
    assert f(P, P, P, 0, 16, P, P, P, None, 0, 0, P, None) == g.GRAFT_ERR_SHAPE
    assert f(P, P, P, 1, g.GRAFT_MAX_NODES + 1, P, P, P, None, 0, 0, P, None) == g.GRAFT_ERR_SHAPE
    assert f(P, P, P, 1, 16, P, P, P, P, 0, 4, P, None) == g.GRAFT_ERR_SHAPE       # paths but no rows
    assert f(P, P, P, 1, 16, P, P, P, P, 4, g.GRAFT_MAX_NODES, P, None) == g.GRAFT_ERR_SHAPE


def test_tree_attn_validation_and_workspace(lib):
    import paper_2605_20104_amd as g
    f = lib.graft_tree_attn
    ws = lib.graft_tree_attn_workspace_bytes
    ok = [P, P, P, 8 * 16 * 128, 128, 16 * 128, P, 130, P, P, P, 1, 40, 32, 8, 128, 16,
          0.088, g.GRAFT_BF16, P, P, 1 << 40, None]

    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return f(*a)
    assert call(a0=None) == g.GRAFT_ERR_NULL
    assert call(a10=None) == g.GRAFT_ERR_NULL
    assert call(a18=7) == g.GRAFT_ERR_DTYPE
    assert call(a15=96) == g.GRAFT_ERR_SHAPE              # D
    assert call(a14=5) == g.GRAFT_ERR_SHAPE               # Hq % Hkv
    assert call(a14=1) == g.GRAFT_ERR_SHAPE               # group of 32 > 16
    assert call(a12=g.GRAFT_MAX_NODES + 1) == g.GRAFT_ERR_SHAPE
    assert call(a16=32) == g.GRAFT_ERR_SHAPE              # page size
    assert call(a4=100) == g.GRAFT_ERR_SHAPE              # token stride < D
    assert call(a4=132) == g.GRAFT_ERR_SHAPE              # token stride not a multiple of 8
    assert call(a17=0.0) == g.GRAFT_ERR_SHAPE             # scale
    assert call(a20=None) == g.GRAFT_ERR_WORKSPACE
    assert call(a21=16) == g.GRAFT_ERR_WORKSPACE
    need = ws(1, 40, 32, 8, 128, 130, g.GRAFT_BF16)
    assert need > 0 and need % 8 == 0
    assert ws(1, 16, 8, 2, 64, 17, g.GRAFT_F32) == 0      # the fp32 path needs no scratch
    assert ws(1, 40, 32, 8, 96, 130, g.GRAFT_BF16) == 0   # unsupported shape -> 0
    # more sequences never need less workspace
    assert ws(4, 96, 32, 8, 128, 4102, g.GRAFT_BF16) >= ws(1, 96, 32, 8, 128, 4102, g.GRAFT_BF16)
    assert ws(64, 16, 8, 8, 128, 40, g.GRAFT_BF16) == 0   # enough (sequence, head) units to fill the chip: one split


def test_accept_validation(lib):
    import paper_2605_20104_amd as g
    f = lib.graft_accept
    ok = [P, P, P, None, 0, P, 1, 16, 8, P, P, P, P, P, None, 0, None]

    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return f(*a)
    assert call(a0=None) == g.GRAFT_ERR_NULL
    assert call(a5=None) == g.GRAFT_ERR_NULL
    assert call(a7=0) == g.GRAFT_ERR_SHAPE
    assert call(a7=g.GRAFT_MAX_NODES + 1) == g.GRAFT_ERR_SHAPE
    assert call(a8=-1) == g.GRAFT_ERR_SHAPE
    assert call(a8=g.GRAFT_MAX_NODES) == g.GRAFT_ERR_SHAPE
    assert call(a3=P, a4=0) == g.GRAFT_ERR_SHAPE          # logits with V = 0
    assert call(a3=P, a4=1000) == g.GRAFT_ERR_WORKSPACE   # logits mode needs the workspace
    assert call(a3=P, a4=1000, a14=P, a15=8) == g.GRAFT_ERR_WORKSPACE
    assert lib.graft_accept_workspace_bytes(1, 16, 1000) == 16 * 16 * 8


def _caller(f, ok):
    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return f(*a)
    return call


def test_matrix_retrieve_validation(lib):
    import paper_2605_20104_amd as g
    call = _caller(lib.graft_matrix_retrieve, [P, 1000, 8, P, P, 80, P, 2, 64, P, P, P, P, None])
    for i in (0, 3, 4, 6, 9, 10, 11, 12):
        assert call(**{"a%d" % i: None}) == g.GRAFT_ERR_NULL
    assert call(a1=0) == g.GRAFT_ERR_SHAPE
    assert call(a2=0) == g.GRAFT_ERR_SHAPE
    assert call(a2=g.GRAFT_MAX_SUCCESSORS + 1) == g.GRAFT_ERR_SHAPE
    assert call(a5=0) == g.GRAFT_ERR_SHAPE
    assert call(a5=g.GRAFT_MAX_NODES + 1) == g.GRAFT_ERR_SHAPE
    assert call(a7=0) == g.GRAFT_ERR_SHAPE
    assert call(a8=g.GRAFT_MAX_NODES + 1) == g.GRAFT_ERR_SHAPE


def test_matrix_update_validation_and_workspace(lib):
    import paper_2605_20104_amd as g
    call = _caller(lib.graft_matrix_update, [P, P, P, 1000, 2, 16, P, 8, P, 0x2000, 1 << 30, None])
    for i in (0, 1, 2, 6, 8):
        assert call(**{"a%d" % i: None}) == g.GRAFT_ERR_NULL
    assert call(a3=0) == g.GRAFT_ERR_SHAPE
    assert call(a7=0) == g.GRAFT_ERR_SHAPE
    assert call(a7=g.GRAFT_MAX_SUCCESSORS + 1) == g.GRAFT_ERR_SHAPE
    assert call(a3=4, a7=8) == g.GRAFT_ERR_SHAPE                  # k > V
    assert call(a4=1024, a5=128) == g.GRAFT_ERR_SHAPE             # B * K_max > 65536
    assert call(a9=None) == g.GRAFT_ERR_WORKSPACE
    assert call(a10=8) == g.GRAFT_ERR_WORKSPACE
    assert call(a9=0x2004) == g.GRAFT_ERR_WORKSPACE               # not 8-byte aligned
    assert lib.graft_matrix_update_workspace_bytes(2, 16, 1000, 8) == 2 * 16 * 16 * 8 * 8
    assert lib.graft_matrix_update_workspace_bytes(2, 16, 1000, 0) == 0


def test_prune_select_validation(lib):
    import paper_2605_20104_amd as g
    call = _caller(lib.graft_prune_select, [P, P, P, P, 2, 64, P, P, P, P, 3, P, P, P, P, P, P, P, None])
    for i in (0, 1, 2, 3, 6, 7, 8, 9, 11, 12, 13, 14, 15, 16, 17):
        assert call(**{"a%d" % i: None}) == g.GRAFT_ERR_NULL
    assert call(a4=0) == g.GRAFT_ERR_SHAPE
    assert call(a5=g.GRAFT_MAX_NODES + 1) == g.GRAFT_ERR_SHAPE
    assert call(a10=-1) == g.GRAFT_ERR_SHAPE
    assert call(a10=g.GRAFT_MAX_CHECKPOINTS + 1) == g.GRAFT_ERR_SHAPE


def test_kv_compact_validation(lib):
    import paper_2605_20104_amd as g
    ok = [P, P, 1 << 20, 4, 8 * 16 * 128, 128, 16 * 128, P, 130, P, P, P, 2, 16, 64, 8, 128, g.GRAFT_BF16, 0x2000, P,
          None]
    call = _caller(lib.graft_kv_compact, ok)
    for i in (0, 1, 7, 9, 10, 11, 18, 19):
        assert call(**{"a%d" % i: None}) == g.GRAFT_ERR_NULL
    assert call(a17=9) == g.GRAFT_ERR_DTYPE
    assert call(a3=0) == g.GRAFT_ERR_SHAPE                        # n_layers
    assert call(a2=0) == g.GRAFT_ERR_SHAPE                        # several layers need a stride
    assert call(a5=100) == g.GRAFT_ERR_SHAPE                      # token stride < D
    assert call(a5=132) == g.GRAFT_ERR_SHAPE                      # 16-byte columns must stay aligned
    assert call(a16=96) == g.GRAFT_ERR_SHAPE                      # D
    assert call(a13=g.GRAFT_MAX_NODES) == g.GRAFT_ERR_SHAPE       # depth_cap
    assert call(a14=0) == g.GRAFT_ERR_SHAPE                       # K_max
    assert call(a0=0x1008) == g.GRAFT_ERR_SHAPE                   # cache base not 16-byte aligned
    assert call(a18=P) == g.GRAFT_ERR_SHAPE                       # new_prefix_len must not be prefix_len itself ...
    assert call(a18=P + 4) == g.GRAFT_ERR_SHAPE                   # ... nor overlap it (B = 2 entries of 4 bytes)
    assert call(a18=P - 4) == g.GRAFT_ERR_SHAPE


def test_accept_noalloc_validation(lib):
    import paper_2605_20104_amd as g
    call = _caller(lib.graft_accept_noalloc, [P, P, P, None, 0, P, 2, 64, 16, P, P, P, P, P, None])
    for i in (0, 1, 2, 5, 9, 10, 11, 12, 13):
        assert call(**{"a%d" % i: None}) == g.GRAFT_ERR_NULL
    assert call(a6=0) == g.GRAFT_ERR_SHAPE
    assert call(a7=g.GRAFT_MAX_NODES + 1) == g.GRAFT_ERR_SHAPE
    assert call(a8=g.GRAFT_MAX_NODES) == g.GRAFT_ERR_SHAPE
    assert call(a3=P, a4=0) == g.GRAFT_ERR_SHAPE                  # logits mode needs a vocabulary
    # more logits rows than the library's own scratch array holds: rejected before anything is launched
    assert call(a3=P, a4=1000, a6=65, a7=128) == g.GRAFT_ERR_WORKSPACE
    m = re.search(r"#define\s+GRAFT_NOALLOC_MAX_ROWS\s+(\d+)", open(HEADER).read())
    assert m and int(m.group(1)) == g.GRAFT_NOALLOC_MAX_ROWS == 8192 and 65 * 128 > 8192


def test_binding_has_no_fallback(monkeypatch):
    import paper_2605_20104_amd as g
    monkeypatch.setattr(g, "_lib", None)
    monkeypatch.setattr(g, "LIB_PATH", "/nonexistent/libgraft.so")
    with pytest.raises(FileNotFoundError):
        g.load_library()
