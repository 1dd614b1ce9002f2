"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and validates arguments
on the host before anything is launched (no GPU needed: every call here is rejected before a HIP call)."""
import ctypes as ct
import os
import re

import numpy as np

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "maskkv.h")


@pytest.fixture(scope="module")
def mk():
    from paper_2510_09309_amd import binding
    return binding


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(maskkv_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_named_calls():
    names = declared_functions()
    for n in ("maskkv_score", "maskkv_select", "maskkv_compact", "maskkv_attend"):
        assert n in names


def test_library_exports_every_declared_symbol(mk):
    lib = ct.CDLL(mk.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in maskkv.h but not exported"
    assert sorted(mk.SYMBOLS) == declared_functions()
    assert mk.maskkv_version() == 1


def test_bench_library_exports_its_header_and_rejects_bad_probes():
    """libmaskkv_bench.so (measurement probes, stage marks) is a library of its own with a header of its own."""
    from paper_2510_09309_amd import bench_binding as bb
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "maskkv_bench.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(maskkv_bench_[a-z_]+)\s*\(", text)))
    assert names == sorted(bb.SYMBOLS)
    lib = ct.CDLL(bb.LIB_PATH)
    for name in names:
        assert hasattr(lib, name)
    f = ct.c_void_p(0x1000)
    probe = lambda which, iters, src, nbytes, dst_bytes, groups: lib.maskkv_bench_probe(
        ct.c_int(which), ct.c_int32(iters), src, f, ct.c_int64(nbytes), ct.c_int64(dst_bytes), ct.c_int32(groups), None,
        None)
    assert probe(10, 10, None, 0, 1 << 20, 8) == 1             # unknown probe
    assert probe(7, 10, None, 0, 1 << 20, 8) == 1              # split-role probe: operands missing
    assert probe(7, 10, f, 64 * 24 * 16, 8 * 512 * 4 - 4, 8) == 1   # split-role probe: one word per thread of 512
    assert probe(6, 10, None, 0, 1 << 20, 8) == 1              # pipeline probe: operands missing
    assert probe(4, 0, None, 0, 1 << 20, 8) == 1               # no iterations
    assert probe(0, 0, None, 0, 1 << 20, 8) == 1               # no iterations
    assert probe(0, 10, None, 0, 8 * 256 * 4 - 4, 8) == 1      # result buffer too small
    assert probe(2, 0, None, 1024, 1024, 8) == 1               # copy without a source
    assert probe(2, 0, f, 1000, 1024, 8) == 1                  # not a multiple of 16 bytes
    assert probe(2, 0, f, 2048, 1024, 8) == 1                  # copy target too small
    assert probe(3, 0, f, 2048, 1024, 8) == 1                  # read: result buffer too small
    assert probe(5, 10, f, 1024, 1 << 20, 8) == 1              # data-fed matrix probe: operands missing
    lib.maskkv_bench_last_error.restype = ct.c_char_p
    assert b"24 KiB" in lib.maskkv_bench_last_error()


def test_product_library_exports_no_measurement_entry_points(mk):
    lib = ct.CDLL(mk.LIB_PATH)
    for name in ("maskkv_probe", "maskkv_score_profiled", "maskkv_bench_probe", "maskkv_bench_score_marked"):
        assert not hasattr(lib, name), name


def test_strerror(mk):
    lib = mk.raw_library()
    assert lib.maskkv_strerror(0) == b"ok"
    assert b"shape" in lib.maskkv_strerror(2)
    assert b"unknown" in lib.maskkv_strerror(99)


def test_workspace_sizes(mk):
    d = mk.Desc(B=1, H=32, d=128, dtype=mk.MASKKV_BF16, n_resp=256, P_max=32768)
    assert mk.maskkv_score_workspace_bytes(d) > 32 * 256 * 4
    assert mk.maskkv_select_workspace_bytes(d) == 32 * 32768 * 8 + 32 * 8 * 4  # candidates (4096 per chunk) + counts
    assert mk.maskkv_attend_workspace_bytes(d, False) == 0
    assert mk.maskkv_attend_workspace_bytes(d, True) > 0
    grouped = mk.Desc(B=1, H=4, d=128, dtype=mk.MASKKV_BF16, n_resp=256, P_max=32768, q_per_kv=7)
    single = mk.Desc(B=1, H=4, d=128, dtype=mk.MASKKV_BF16, n_resp=256, P_max=32768)
    # 7 query groups per head: row statistics of 7x the voting rows plus the groups' column sums (4 B x P each)
    assert mk.maskkv_score_workspace_bytes(grouped) > mk.maskkv_score_workspace_bytes(single) + 4 * 7 * 32768 * 4
    assert mk.maskkv_select_workspace_bytes(grouped) == mk.maskkv_select_workspace_bytes(single)   # per KV head
    long = mk.Desc(B=2, H=4, d=128, dtype=mk.MASKKV_BF16, n_resp=8, P_max=100000)
    assert mk.maskkv_select_workspace_bytes(long) == 2 * 4 * 25 * 4096 * 8 + 1024   # 800 bytes of counts, padded to 256 B


@pytest.mark.parametrize("kw,status", [
    (dict(d=96), 2), (dict(dtype=7), 3), (dict(B=0), 2), (dict(B=65), 2), (dict(n_resp=0), 1),
    (dict(P_max=-1), 1), (dict(prompt_len=[5000]), 1), (dict(H=0), 2),
    (dict(q_per_kv=-1), 1), (dict(q_per_kv=65), 1), (dict(q_per_kv=64, n_resp=1 << 15), 2),
])
def test_bad_descriptions_are_rejected(mk, kw, status):
    base = dict(B=1, H=4, d=128, dtype=mk.MASKKV_BF16, n_resp=16, P_max=1024)
    base.update(kw)
    with pytest.raises(mk.MaskKVError) as e:
        mk.maskkv_score_workspace_bytes(mk.Desc(**base))
    assert e.value.status == status
    assert mk.raw_library().maskkv_last_error() != b""


def test_bad_call_arguments_are_rejected_before_launch(mk):
    """Fake (never dereferenced) pointers: each call must fail in host validation."""
    lib = mk.raw_library()
    desc = mk.Desc(B=1, H=2, d=64, dtype=mk.MASKKV_F32, n_resp=8, P_max=100).c()
    fake = 0x1000
    good = mk._CTensor(fake, 0, 108 * 64, 64, None)
    misaligned = mk._CTensor(fake + 4, 0, 108 * 64, 64, None)
    short_row = mk._CTensor(fake, 0, 108 * 64, 32, None)
    huge_stride = mk._CTensor(fake, 0, 0, (1 << 24) // 2 + 8, None)   # token stride above 16 MiB in bytes
    null = mk._CTensor(0, 0, 0, 64, None)
    f = ct.c_void_p(fake)
    call_score = lambda q, k, stride, ws, wsn: lib.maskkv_score(
        ct.byref(desc), ct.byref(q), ct.byref(k), ct.c_float(0), f, ct.c_int64(stride), None, ws, ct.c_size_t(wsn), None)
    assert call_score(null, good, 128, f, 1 << 20) == 1
    assert call_score(good, misaligned, 128, f, 1 << 20) == 1
    assert call_score(good, short_row, 128, f, 1 << 20) == 1
    assert call_score(good, huge_stride, 128, f, 1 << 20) == 1
    assert b"16 MiB" in lib.maskkv_last_error()
    assert call_score(good, good, 64, f, 1 << 20) == 1          # score_stride < P_max
    assert call_score(good, good, 128, None, 0) == 4            # no workspace
    assert call_score(good, good, 128, f, 16) == 4              # too small
    assert call_score(good, good, 128, ct.c_void_p(fake + 8), 1 << 20) == 4  # misaligned workspace
    given = lambda lse, stride, ws, wsn: lib.maskkv_score_given_lse(
        ct.byref(desc), ct.byref(good), ct.byref(good), ct.c_float(0), lse, f, ct.c_int64(stride), None, ws,
        ct.c_size_t(wsn), None)
    assert given(None, 128, f, 1 << 20) == 1                    # no row normalisers
    assert b"row_lse" in lib.maskkv_last_error()
    assert given(f, 64, f, 1 << 20) == 1                        # score_stride < P_max
    assert given(f, 128, None, 0) == 4                          # no workspace
    sel = lambda window, mode, cap: lib.maskkv_select(
        ct.byref(desc), f, ct.c_int64(128), ct.c_int(window), ct.c_int(mode), f, None, f, f, ct.c_int64(cap), None,
        ct.c_size_t(0), None)
    assert sel(4, 0, 10) == 1      # even window
    assert sel(0, 0, 10) == 1
    assert sel(65, 0, 10) == 1
    assert sel(7, 3, 10) == 1      # unknown pool mode
    assert sel(7, 0, -1) == 1
    assert lib.maskkv_compact(ct.byref(desc), ct.byref(good), ct.byref(good), f, None, ct.c_int64(4), f, f, None) == 1
    assert lib.maskkv_head_budgets(ct.byref(desc), f, ct.c_int32(10), ct.c_float(1.5), f, None) == 1
    assert lib.maskkv_head_budgets(ct.byref(desc), f, ct.c_int32(-1), ct.c_float(0.1), f, None) == 1
    assert b"alpha" in lib.maskkv_last_error()
    shift = lambda a, b, n, width, dtype, stride, delta: lib.maskkv_value_shift(
        a, b, ct.c_int64(n), ct.c_int32(width), ct.c_int32(dtype), ct.c_int64(stride), ct.c_float(delta), f, f, f, None)
    assert shift(f, None, 10, 64, 0, 64, 0.9) == 1             # NULL input
    assert shift(f, f, 0, 64, 0, 64, 0.9) == 1                 # no tokens
    assert shift(f, f, 10, 60, 0, 64, 0.9) == 1                # width not a multiple of 8
    assert shift(f, f, 10, 64, 0, 32, 0.9) == 1                # row stride below the width
    assert shift(f, f, 10, 64, 1, 68, 0.9) == 1                # bf16 rows of 136 bytes: not 16-byte multiples
    assert shift(f, f, 10, 64, 5, 64, 0.9) == 3                # unknown dtype
    assert shift(f, f, 10, 64, 0, 64, float("nan")) == 1


def test_layer_budgets_host_arithmetic_matches_the_oracle(mk):
    """maskkv_layer_budgets is host-only arithmetic: compare with the oracle on the same float32 importances."""
    from oracle import maskkv_oracle as orc
    rng = np.random.default_rng(11)
    cases = [(32, 32 * 256, 0.4, None), (32, 8192, 0.4, [0, 31]), (12, 1000, 0.25, [0, 1, 11]), (1, 77, 0.4, None),
             (5, 0, 0.4, None), (7, 12345, 1.0, None), (7, 12345, 0.0, [3])]
    for L, k_p, beta, boundary in cases:
        imp = rng.random(L).astype(np.float32) + np.float32(0.01)
        got = mk.maskkv_layer_budgets(imp, k_p, beta, boundary)
        want = orc.layer_budgets(imp.astype(np.float64), k_p, np.float64(np.float32(beta)), boundary)
        assert got == want.tolist(), (L, k_p, beta, boundary)
        assert sum(got) <= k_p
    # the worked case pinned for the oracle (exact binary factors): L=4, k_p=400, beta=0.5, importances 1,2,3,2
    assert mk.maskkv_layer_budgets([1.0, 2.0, 3.0, 2.0], 400, 0.5) == orc.layer_budgets(
        np.array([1.0, 2.0, 3.0, 2.0]), 400, 0.5).tolist()
    with pytest.raises(mk.MaskKVError):
        mk.maskkv_layer_budgets([0.0, 0.0], 10, 0.4)
    with pytest.raises(mk.MaskKVError):
        mk.maskkv_layer_budgets([1.0, 1.0], 10, 0.4, [5])
    lib = mk.raw_library()
    f = ct.c_void_p(0x1000)
    assert lib.maskkv_layer_importance(f, f, ct.c_int64(10), ct.c_int32(100), ct.c_int32(1), ct.c_int64(100), f, f,
                                       ct.c_size_t(1 << 20), None) == 1     # hidden not a multiple of 8
    assert lib.maskkv_layer_importance(f, f, ct.c_int64(10), ct.c_int32(128), ct.c_int32(1), ct.c_int64(128), f, None,
                                       ct.c_size_t(0), None) == 4           # no workspace


def test_select_checks_a_host_copy_of_the_budgets_before_launch(mk):
    """With the optional host copy of the budgets a negative budget is MASKKV_EINVAL and budgets that keep more rows
    than the capacity are MASKKV_ECAPACITY; both before anything is enqueued (the pointers here are fake)."""
    lib = mk.raw_library()
    desc = mk.Desc(B=2, H=2, d=64, dtype=mk.MASKKV_F32, n_resp=8, P_max=100, prompt_len=[100, 40]).c()
    f = ct.c_void_p(0x1000)

    def sel(host, cap):
        arr = (ct.c_int32 * 4)(*host)
        return lib.maskkv_select(ct.byref(desc), f, ct.c_int64(128), ct.c_int(7), ct.c_int(0), f, arr, f, f,
                                 ct.c_int64(cap), None, ct.c_size_t(0), None)
    assert sel([10, -1, 5, 5], 100) == 1
    assert b"negative" in lib.maskkv_last_error()
    assert sel([10, 20, 30, 1000], 99) == 6          # clamped to the prompts: 10 + 20 + 30 + 40 = 100 > 99
    assert b"capacity" in lib.maskkv_last_error()
    assert lib.maskkv_strerror(6) == b"output capacity too small"
    # prompts beyond what the final stage can index, and offsets beyond 31 bits
    big = mk.Desc(B=1, H=2, d=64, dtype=mk.MASKKV_F32, n_resp=8, P_max=(1 << 22) + 1).c()
    assert lib.maskkv_select(ct.byref(big), f, ct.c_int64(1 << 23), ct.c_int(7), ct.c_int(0), f, None, f, f,
                             ct.c_int64(10), f, ct.c_size_t(1 << 40), None) == 2
    wide = mk.Desc(B=64, H=1024, d=64, dtype=mk.MASKKV_F32, n_resp=8, P_max=1 << 20).c()
    assert lib.maskkv_select(ct.byref(wide), f, ct.c_int64(1 << 20), ct.c_int(7), ct.c_int(0), f, None, f, f,
                             ct.c_int64(10), f, ct.c_size_t(1 << 40), None) == 2
