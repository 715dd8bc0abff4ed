"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments before anything is launched (no GPU needed: no compute call is made)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sste.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2409_09099_amd as pkg
    return pkg.library()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sste_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert {"sste_project_pack", "sste_linear_fwd", "sste_linear_wgrad"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.sste_version() >= 100


def test_no_oracle_or_torch_in_the_library_sources():
    csrc = os.path.join(ROOT, "paper_2409_09099_amd", "csrc")
    for f in os.listdir(csrc):
        text = open(os.path.join(csrc, f)).read()
        assert "oracle" not in text.lower() and "torch" not in text.lower(), f
    for f in ("binding.py", "__init__.py", "build.py"):
        text = open(os.path.join(ROOT, "paper_2409_09099_amd", f)).read()
        assert "import oracle" not in text and "from oracle" not in text, f


def _err(lib):
    return lib.sste_last_error().decode()


def test_project_pack_validation(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)      # never dereferenced: validation fails first
    f = lib.sste_project_pack
    assert f(fake, -1, 8, 8, 1.0, 0, 1.0, fake, fake, None, None) == 2
    assert f(fake, 4, 12, 12, 1.0, 0, 1.0, fake, fake, None, None) == 2 and "multiple of 8" in _err(lib)
    assert f(fake, 4, 64, 8, 1.0, 0, 1.0, fake, fake, None, None) == 2
    assert f(fake, 4, 64, 68, 1.0, 0, 1.0, fake, fake, None, None) == 3
    assert f(fake, 4, 64, 64, 1.0, 7, 1.0, fake, fake, None, None) == 4
    assert f(fake, 4, 64, 64, 0.0, 0, 1.0, fake, fake, None, None) == 5
    assert f(fake, 4, 64, 64, float("inf"), 0, 1.0, fake, fake, None, None) == 5
    assert f(fake, 4, 64, 64, 1.0, 0, 2.0, fake, fake, None, None) == 5
    assert f(fake, 4, 128, 128, 1.0, 1, -1.0, fake, fake, None, None) == 5
    assert f(fake, 4, 16, 16, 1.0, 0, 1.0, fake, fake, None, None) == 7      # whole groups, but not a whole column step
    assert f(fake, 4, 64, 64, 1.0, 1, 1.0, fake, fake, None, None) == 7      # e4m3 values need I % 128 == 0
    assert f(None, 4, 64, 64, 1.0, 0, 1.0, fake, fake, None, None) == 1
    assert f(P(0x1004), 4, 64, 64, 1.0, 0, 1.0, fake, fake, None, None) == 3


def test_linear_fwd_validation(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)
    f = lib.sste_linear_fwd
    assert f(fake, -4, 64, 64, 0, 1.0, fake, fake, 8, 1.0, fake, 8, None) == 2
    assert f(fake, 4, 96, 96, 0, 1.0, fake, fake, 8, 1.0, fake, 8, None) == 7
    assert f(fake, 4, 64, 64, 1, 1.0, fake, fake, 8, 1.0, fake, 8, None) == 7      # e4m3 needs I % 128 == 0
    assert f(fake, 4, 64, 64, 0, 1.0, fake, fake, 12, 1.0, fake, 16, None) == 7
    assert f(fake, 4, 64, 32, 0, 1.0, fake, fake, 8, 1.0, fake, 8, None) == 2
    assert f(fake, 4, 64, 64, 0, 1.0, fake, fake, 8, 1.0, fake, 12, None) == 3
    assert f(fake, 4, 64, 64, 0, -1.0, fake, fake, 8, 1.0, fake, 8, None) == 5
    assert f(None, 4, 64, 64, 0, 1.0, fake, fake, 8, 1.0, fake, 8, None) == 1
    assert f(fake, 4, 64, 64, 3, 1.0, fake, fake, 8, 1.0, fake, 8, None) == 4


def test_linear_wgrad_validation_and_workspace(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)
    f = lib.sste_linear_wgrad
    args = lambda T=128, O=16, I=16, lddy=16, dtype=0, ldx=16, lddw=16, acc=0, ws=None, wsb=0, dy=fake: (
        dy, T, O, lddy, dtype, 1.0, fake, I, ldx, 1.0, 1, 2, fake, lddw, acc, ws, wsb, None)
    assert f(*args(T=102)) == 2          # not whole groups of four tokens
    assert f(*args(T=100)) == 7          # whole groups, but not a multiple of the k-step
    assert f(*args(O=12)) == 7
    assert f(*args(dtype=1, T=128, O=8)) == 7
    assert f(*args(lddy=8)) == 2
    assert f(*args(lddw=18)) == 3
    assert f(*args(acc=2)) == 5
    assert f(*args(dy=None)) == 1
    # a problem that needs split partial sums refuses a missing / small workspace
    need = lib.sste_wgrad_workspace_bytes(8192, 3072, 768, 0)
    assert need >= 2 * 3072 * 768 * 4
    assert f(*args(T=8192, O=3072, I=768, lddy=3072, ldx=768, lddw=768)) == 6
    assert f(*args(T=8192, O=3072, I=768, lddy=3072, ldx=768, lddw=768, ws=fake, wsb=need - 1)) == 6
    assert lib.sste_wgrad_workspace_bytes(512, 256, 1024, 0) == 0
    assert lib.sste_wgrad_workspace_bytes(100, 256, 1024, 0) == 0


def test_other_entry_points_validation(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)
    assert lib.sste_mvue_materialize(fake, 10, 8, 8, 0, 0, 0, fake, fake, None) == 2
    assert lib.sste_mvue_materialize(fake, 16, 8, 8, 0, 0, 0, fake, fake, None) == 7
    assert lib.sste_mvue_materialize(fake, 64, 8, 4, 0, 0, 0, fake, fake, None) == 2
    assert lib.sste_mvue_materialize(None, 64, 8, 8, 0, 0, 0, fake, fake, None) == 1
    assert lib.sste_compute_beta(fake, 4, 16, 16, None, fake, 1 << 20, None) == 1
    assert lib.sste_compute_beta(fake, 4, 16, 16, fake, None, 0, None) == 6
    assert lib.sste_flip_count(fake, fake, 4, 12, fake, None) == 2
    assert lib.sste_flip_count(fake, fake, 4, 16, None, None) == 1


def test_project_pack_batch_prepare(lib):
    """Host-only half of the batch call: validation per item, block counts and the table layout."""
    import struct
    from paper_2409_09099_amd.binding import _PackItem, PACK_TABLE_ITEM_BYTES
    P = ctypes.c_void_p
    prep = lib.sste_project_pack_batch_prepare
    total = ctypes.c_int64(-1)
    items = (_PackItem * 3)(
        _PackItem(0x10000, 0x20000, 0x30000, 40, 128, 136, 1.5, 1.0),       # 3 row blocks x 2 steps = 6 blocks
        _PackItem(None, None, None, 0, 64, 64, 1.0, 1.0),                   # empty item: no blocks
        _PackItem(0x40000, 0x50000, 0x60000, 16, 64, 64, 2.0, 1.0))         # 1 block
    table = ctypes.create_string_buffer(3 * PACK_TABLE_ITEM_BYTES)
    assert prep(ctypes.cast(items, P), 3, 0, ctypes.cast(table, P), ctypes.byref(total)) == 0, _err(lib)
    assert total.value == 7
    rows = [struct.unpack_from("<QQQqqqiffi", table.raw, k * PACK_TABLE_ITEM_BYTES) for k in range(3)]
    # (W, vals, meta, O, ldw_bytes, first_block, steps, beta, val_scale, pad)
    assert rows[0][:7] == (0x10000, 0x20000, 0x30000, 40, 272, 0, 2) and rows[0][7] == 1.5
    assert rows[1][3] == 0 and rows[1][5] == 6
    assert rows[2][:7] == (0x40000, 0x50000, 0x60000, 16, 128, 6, 1)
    # errors name the first offending item
    items[2].I = 96
    assert prep(ctypes.cast(items, P), 3, 0, ctypes.cast(table, P), ctypes.byref(total)) == 7 and "item 2" in _err(lib)
    items[2].I = 64
    items[0].beta = 0.0
    assert prep(ctypes.cast(items, P), 3, 0, ctypes.cast(table, P), ctypes.byref(total)) == 5 and "item 0" in _err(lib)
    items[0].beta = 1.5
    assert prep(ctypes.cast(items, P), 3, 1, ctypes.cast(table, P), ctypes.byref(total)) == 7      # e4m3 needs I % 128 == 0
    assert prep(ctypes.cast(items, P), 3, 9, ctypes.cast(table, P), ctypes.byref(total)) == 4
    assert prep(ctypes.cast(items, P), -1, 0, ctypes.cast(table, P), ctypes.byref(total)) == 2
    assert prep(ctypes.cast(items, P), 3, 0, None, ctypes.byref(total)) == 1
    assert prep(None, 0, 0, None, ctypes.byref(total)) == 0 and total.value == 0
    # launch half: argument checks only (no kernel is enqueued for an empty table)
    launch = lib.sste_project_pack_batch
    assert launch(None, 0, 0, 0, None) == 0
    assert launch(None, 2, 5, 0, None) == 1
    assert launch(P(0x1004), 2, 5, 0, None) == 3
    assert launch(P(0x1000), -2, 5, 0, None) == 2
    assert launch(P(0x1000), 2, 5, 5, None) == 4


def test_linear_dgrad_validation(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)
    f = lib.sste_linear_dgrad
    f.argtypes = [P, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_float, P, P, ctypes.c_int64,
                  ctypes.c_float, P, ctypes.c_int64, P]
    assert f(fake, -4, 64, 64, 0, 1.0, fake, fake, 64, 1.0, fake, 64, None) == 2
    assert f(fake, 4, 64, 64, 1, 1.0, fake, fake, 64, 1.0, fake, 64, None) == 7        # e4m3: I must be a multiple of 128
    assert f(fake, 4, 72, 80, 1, 1.0, fake, fake, 128, 1.0, fake, 128, None) == 7      # e4m3: O must be a multiple of 16
    assert f(fake, 4, 64, 64, 0, 1.0, fake, fake, 96, 1.0, fake, 96, None) == 7        # I must be a multiple of 64
    assert f(fake, 4, 60, 64, 0, 1.0, fake, fake, 64, 1.0, fake, 64, None) == 7        # O must be a multiple of 8
    assert f(fake, 4, 64, 32, 0, 1.0, fake, fake, 64, 1.0, fake, 64, None) == 2        # lddy < O
    assert f(fake, 4, 64, 68, 0, 1.0, fake, fake, 64, 1.0, fake, 64, None) == 3        # lddy breaks the 16-byte row rule
    assert f(fake, 4, 64, 64, 0, 0.0, fake, fake, 64, 1.0, fake, 64, None) == 5
    assert f(fake, 4, 64, 64, 0, 1.0, fake, fake, 64, 1.0, None, 64, None) == 1
    assert f(fake, 4, 64, 64, 5, 1.0, fake, fake, 64, 1.0, fake, 64, None) == 4
    assert f(fake, 4, 64, 64, 2, 1.0, fake, fake, 128, 1.0, fake, 128, None) == 4      # float32 is no gradient format
    assert f(fake, 4, 72, 80, 3, 1.0, fake, fake, 128, 1.0, fake, 128, None) == 7      # e5m2 gradients: sizes as e4m3
    assert f(fake, 0, 64, 64, 3, 1.0, fake, fake, 128, 1.0, None, 128, None) == 0
    assert f(fake, 0, 64, 64, 0, 1.0, fake, fake, 64, 1.0, None, 64, None) == 0         # no tokens: nothing to do


def test_sgd_project_pack_validation(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)
    f = lib.sste_sgd_project_pack
    f.argtypes = [P, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, P, ctypes.c_int64, ctypes.c_float,
                  ctypes.c_float, ctypes.c_int, ctypes.c_float, P, P, P]
    assert f(fake, 1, 16, 64, 64, fake, 64, 0.1, 1.0, 0, 1.0, fake, fake, None) == 4     # W is bf16 or float32 only
    assert f(fake, 0, 16, 64, 68, fake, 64, 0.1, 1.0, 0, 1.0, fake, fake, None) == 3     # bf16 rows: ldw % 8
    assert f(fake, 2, 16, 64, 66, fake, 64, 0.1, 1.0, 0, 1.0, fake, fake, None) == 3     # float32 rows: ldw % 4
    assert f(fake, 0, 16, 64, 64, fake, 32, 0.1, 1.0, 0, 1.0, fake, fake, None) == 2     # ldg < I
    assert f(fake, 0, 16, 64, 64, fake, 66, 0.1, 1.0, 0, 1.0, fake, fake, None) == 3
    assert f(fake, 0, 16, 64, 64, None, 64, 0.1, 1.0, 0, 1.0, fake, fake, None) == 1
    assert f(fake, 0, 16, 64, 64, P(0x1004), 64, 0.1, 1.0, 0, 1.0, fake, fake, None) == 3
    assert f(fake, 0, 16, 64, 64, fake, 64, float("nan"), 1.0, 0, 1.0, fake, fake, None) == 5
    assert f(fake, 0, 16, 64, 64, fake, 64, 0.1, -1.0, 0, 1.0, fake, fake, None) == 5
    assert f(fake, 0, 16, 96, 96, fake, 96, 0.1, 1.0, 0, 1.0, fake, fake, None) == 7
    assert f(None, 2, 0, 64, 64, None, 64, 0.1, 1.0, 0, 1.0, None, None, None) == 0       # empty: nothing to do


def test_sgd_project_pack_batch_prepare(lib):
    class Item(ctypes.Structure):
        _fields_ = [("W", ctypes.c_void_p), ("G", ctypes.c_void_p), ("vals", ctypes.c_void_p), ("meta", ctypes.c_void_p),
                    ("O", ctypes.c_int64), ("I", ctypes.c_int64), ("ldw", ctypes.c_int64), ("ldg", ctypes.c_int64),
                    ("beta", ctypes.c_float), ("val_scale", ctypes.c_float)]

    prep = lib.sste_sgd_project_pack_batch_prepare
    prep.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)]
    items = (Item * 3)(Item(0x1000, 0x2000, 0x3000, 0x4000, 33, 128, 128, 132, 1.5, 1.0),
                       Item(None, None, None, None, 0, 64, 64, 64, 1.0, 1.0),
                       Item(0x5000, 0x6000, 0x7000, 0x8000, 16, 64, 64, 64, 2.0, 1.0))
    table = (ctypes.c_uint8 * (3 * 80))()
    total = ctypes.c_int64(-1)
    assert prep(items, 3, 2, 0, table, ctypes.byref(total)) == 0
    assert total.value == 3 * 2 + 0 + 1
    raw = bytes(table)
    import struct
    W, G, vals, meta, O, ldw_bytes, ldg, first, steps, beta, scale, _ = struct.unpack("<QQQQqqqqiffi", raw[:80])
    assert (W, G, vals, meta, O, ldw_bytes, ldg, first, steps, beta) == (0x1000, 0x2000, 0x3000, 0x4000, 33, 512, 132, 0, 2, 1.5)
    assert struct.unpack("<q", raw[160 + 56:160 + 64])[0] == 6          # first block of the third item
    assert prep(items, 3, 0, 0, table, ctypes.byref(total)) == 0          # bf16 rows: 128 % 8 == 0
    assert struct.unpack("<q", bytes(table)[40:48])[0] == 256
    assert prep(items, 3, 1, 0, table, ctypes.byref(total)) == 4
    items[2].ldg = 66
    assert prep(items, 3, 2, 0, table, ctypes.byref(total)) == 3
    assert b"item 2" in lib.sste_last_error()
    launch = lib.sste_sgd_project_pack_batch
    launch.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p]
    assert launch(None, 1, 4, 0, 0, 0.1, None) == 1
    assert launch(0x1008, 1, 4, 0, 0, 0.1, None) == 3
    assert launch(0x1000, 1, 4, 0, 0, float("inf"), None) == 5
    assert launch(0x1000, 1, 4, 1, 0, 0.1, None) == 4
    assert launch(None, 0, 0, 2, 1, 0.1, None) == 0


def test_problems_beyond_the_32_bit_tile_offsets_are_refused(lib):
    """The kernels address inside a tile with 32-bit offsets; sizes beyond that are refused on the host
    (status 7) before anything is launched."""
    P = ctypes.c_void_p
    fake = P(0x1000)
    i64, f32, ci = ctypes.c_int64, ctypes.c_float, ctypes.c_int
    fwd = lib.sste_linear_fwd
    fwd.argtypes = [P, i64, i64, i64, ci, f32, P, P, i64, f32, P, i64, P]
    assert fwd(fake, 256, 64, 1 << 21, 0, 1.0, fake, fake, 16, 1.0, fake, 16, None) == 7      # a 256-row X tile spans 2^30 bytes
    assert fwd(fake, 256, 1 << 21, 1 << 21, 0, 1.0, fake, fake, 16, 1.0, fake, 16, None) == 7
    dg = lib.sste_linear_dgrad
    dg.argtypes = [P, i64, i64, i64, ci, f32, P, P, i64, f32, P, i64, P]
    assert dg(fake, 256, 64, 1 << 21, 0, 1.0, fake, fake, 64, 1.0, fake, 64, None) == 7
    assert dg(fake, 256, 1 << 16, 1 << 16, 0, 1.0, fake, fake, 1 << 15, 1.0, fake, 1 << 15, None) == 7   # packed weight: 2^31 elements
    wg = lib.sste_linear_wgrad
    wg.argtypes = [P, i64, i64, i64, ci, f32, P, i64, i64, f32, ctypes.c_uint64, ctypes.c_uint64, P, i64, ci, P, ctypes.c_size_t, P]
    assert wg(fake, 1 << 14, 256, 256, 0, 1.0, fake, 256, 1 << 17, 1.0, 0, 0, fake, 256, 0, fake, 1 << 40, None) == 7   # T * ldx * 2 = 2^32


def test_cast_fp8_validation(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)
    f = lib.sste_cast_fp8
    f.argtypes = [P, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_float, P, ctypes.c_int64, P, P]
    assert f(fake, -1, 64, 64, 1, 1.0, fake, 64, None, None) == 2
    assert f(fake, 4, 60, 64, 1, 1.0, fake, 64, None, None) == 2
    assert f(fake, 4, 64, 32, 1, 1.0, fake, 64, None, None) == 2
    assert f(fake, 4, 64, 68, 1, 1.0, fake, 64, None, None) == 3
    assert f(fake, 4, 64, 64, 1, 1.0, fake, 68, None, None) == 3
    assert f(fake, 4, 64, 64, 0, 1.0, fake, 64, None, None) == 4
    assert f(fake, 4, 64, 64, 3, float("inf"), fake, 64, None, None) == 5
    assert f(fake, 4, 64, 64, 3, 1.0, None, 64, None, None) == 1
    assert f(None, 4, 64, 64, 3, 1.0, fake, 64, None, None) == 1
    assert f(fake, 4, 64, 64, 3, 1.0, P(0x1004), 64, None, None) == 3
    assert f(None, 0, 64, 64, 1, 1.0, None, 64, None, None) == 1               # nothing asked for


def test_linear_fwd_ex_validation(lib):
    P = ctypes.c_void_p
    fake = P(0x1000)
    f = lib.sste_linear_fwd_ex
    f.argtypes = [P, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_float, P, P, ctypes.c_int64,
                  ctypes.c_float, P, ctypes.c_int64, ctypes.c_int, ctypes.c_float, P, P]
    ok_args = lambda **kw: [kw.get("X", fake), 4, 128, 128, kw.get("dtype", 1), 1.0, fake, fake, kw.get("O", 16), 1.0, fake, kw.get("ldz", 16),
                            kw.get("z_dtype", 1), kw.get("z_scale", 0.5), kw.get("amax", fake), None]
    assert f(*ok_args(z_dtype=2)) == 4 and "z_dtype" in _err(lib)            # float32 is not an output format
    assert f(*ok_args(z_dtype=3)) == 4                                        # nor is e5m2
    assert f(*ok_args(z_scale=0.0)) == 5
    assert f(*ok_args(z_dtype=0, z_scale=0.5)) == 5 and "z_scale must be 1" in _err(lib)
    assert f(*ok_args(amax=None)) == 1 and "amax_out" in _err(lib)            # an 8-bit output needs its largest magnitude
    assert f(*ok_args(O=8, ldz=8)) == 7                                       # e4m3 rows come in 16-channel pieces
    assert f(*ok_args(ldz=24)) == 3
    assert f(*ok_args(amax=P(0x1002))) == 3
    assert f(*ok_args(X=None)) == 1


def test_amax_history_is_a_sliding_window_maximum(lib):
    from oracle import formats as F

    class H(ctypes.Structure):
        _fields_ = [("window", ctypes.c_float * 64), ("length", ctypes.c_int), ("next", ctypes.c_int)]

    lib.sste_amax_history_init.argtypes = [ctypes.c_void_p, ctypes.c_int]
    lib.sste_amax_history_init.restype = None
    lib.sste_amax_history_push.argtypes = [ctypes.c_void_p, ctypes.c_float, ctypes.c_float]
    lib.sste_amax_history_push.restype = ctypes.c_float
    h = H()
    lib.sste_amax_history_init(ctypes.byref(h), 3)
    seen = []
    for amax in [0.0, 2.0, 7.5, 1.0, 0.5, 0.25, 0.125, 900.0]:
        seen.append(amax)
        got = lib.sste_amax_history_push(ctypes.byref(h), amax, 448.0)
        assert got == float(F.delayed_scale(seen[-3:], "e4m3")), (amax, got)
    assert lib.sste_amax_history_push(ctypes.byref(h), float("nan"), 448.0) == float(F.delayed_scale(seen[-3:], "e4m3"))   # ignored
    assert lib.sste_amax_history_push(ctypes.byref(h), -1.0, 448.0) == float(F.delayed_scale(seen[-3:], "e4m3"))
    lib.sste_amax_history_init(ctypes.byref(h), 1000)                         # clamped to the struct's capacity
    assert h.length == 64
    assert lib.sste_amax_history_push(ctypes.byref(h), 57344.0 * 2, 57344.0) == 2.0
    assert lib.sste_amax_history_push(None, 1.0, 448.0) == 1.0
