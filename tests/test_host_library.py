"""CPU checks of the C-ABI library: it loads, exports every declared symbol, validates arguments
before touching a device, and its host-side pair sampler agrees with the oracle's."""
import ctypes as C
import os
import re

import pytest

import paper_2605_11222_amd as admmq
from paper_2605_11222_amd import binding
from oracle import admmq_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return admmq.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "admmq.h")).read()
    declared = set(re.findall(r"\b(admmq_[a-z_]+)\s*\(", header))
    assert declared == set(admmq.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    assert lib.admmq_status_string(0) == b"ok"
    assert all(lib.admmq_status_string(c) for c in range(9))


def test_workspace_bytes_monotone(lib):
    a = admmq.workspace_bytes(128, 64, 50)
    b = admmq.workspace_bytes(4096, 4096, 200)
    c = admmq.workspace_bytes(25600, 5120, 300)
    assert 0 < a < b < c
    assert c < 200 * 2 ** 30            # the largest workload fits one 288 GB GPU several times over
    assert admmq.workspace_bytes(0, 4, 4) == 0


def test_pair_sampler_matches_oracle_generator(lib):
    for seed, n in ((0, 2), (7, 128), (2 ** 63 + 5, 4096), (12345, 25600)):
        for r in (0, 3):
            for b in (0, 17, 12799):
                for s in (0, 1, 63):
                    assert admmq.sample_pair(seed, r, b, s, n) == orc.sample_pair(seed, r, b, s, n)


def _ctx(lib):
    h = C.c_void_p()
    assert lib.admmq_create(C.byref(h), -1, None) == 0
    return h


def test_argument_validation_without_a_gpu(lib):
    h = _ctx(lib)
    one = C.c_void_p(256)      # any non-null address: validation must not dereference it
    sched = binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0)
    q = lambda **k: lib.admmq_quantize_layer(
        h, k.get("H", one), k.get("W0", one), k.get("n", 8), k.get("p", 4), k.get("ldw", 4), k.get("bits", 4),
        k.get("g", 0), C.byref(k.get("sched", sched)), k.get("codes", one), one, one, None)
    assert q(H=None) == 1 and q(W0=None) == 1 and q(codes=None) == 1
    assert q(n=0) == 2 and q(p=0) == 2 and q(ldw=3) == 2 and q(g=3) == 2 and q(g=-1) == 2
    assert q(bits=1) == 3 and q(bits=9) == 3
    for bad in (binding._Schedule(0, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0),
                binding._Schedule(10, 0.0, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0),
                binding._Schedule(10, 0.1, 0.9, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0),
                binding._Schedule(10, 0.1, 1.1, -1.0, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0),
                binding._Schedule(10, float("nan"), 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0),
                binding._Schedule(10, 0.1, 1.1, 0.01, 1, -1, 0, 0, -1, 0, 0, 0.8, 0, 0),
                binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, -2, 0, 0, 0.8, 0, 0),
                binding._Schedule(930, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0),       # 0.1 * 1.1^930 > 1e30
                binding._Schedule(10, 1e-31, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0),
                binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0, -1)):      # quiet_stop < 0
        assert q(sched=bad) == 3
    assert q() == 8                       # valid arguments: stops at the missing device
    assert q(sched=binding._Schedule(300, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0)) == 8   # the paper's schedule
    cnt = C.c_uint64(0)
    assert lib.admmq_accumulate_hessian(h, None, 8, one, 0, 4, 8, C.byref(cnt)) == 1
    assert lib.admmq_accumulate_hessian(h, one, 8, one, 0, 4, 7, C.byref(cnt)) == 2
    assert lib.admmq_accumulate_hessian(h, one, 8, one, 5, 4, 8, C.byref(cnt)) == 3
    assert lib.admmq_accumulate_hessian(h, one, 8, one, 0, 0, 8, C.byref(cnt)) == 0 and cnt.value == 0
    assert lib.admmq_accumulate_hessian(h, one, 8, one, 0, 4, 8, C.byref(cnt)) == 8 and cnt.value == 0
    assert lib.admmq_w_update(h, one, one, one, 8, 4, 0.5, one) == 7      # no factorisation yet
    assert lib.admmq_w_update(h, one, one, one, 8, 4, -1.0, one) == 3
    assert lib.admmq_project_dual(h, one, one, 8, 4, one, 4, 3, one, one, 0.5, 0.55, None, one, None) == 2
    assert lib.admmq_project_dual(h, one, one, 8, 4, one, 4, 0, one, one, 0.0, 0.55, None, one, None) == 3
    # the variant that allocates nothing: same validation, a misaligned residual pointer, and the size limit of its
    # fixed scratch array (reciprocals of d and of the scales), all before any device work
    na = lambda **k: lib.admmq_project_dual_noalloc(
        h, k.get("W", one), one, k.get("n", 8), k.get("p", 4), one, 4, k.get("g", 0), one, one, k.get("rho", 0.5),
        0.55, None, one, k.get("res", None))
    assert na(W=None) == 1 and na(g=3) == 2 and na(rho=0.0) == 3 and na(res=C.c_void_p(260)) == 3
    assert na(n=4096, p=4096, g=4) == 6 and na(n=1 << 20, p=(1 << 20) + 64, g=0) == 6
    assert na(n=4096, p=4096, g=0) == 8 and na(n=1 << 20, p=1 << 20, g=0) == 8 and na(n=25600, p=5120, g=128, res=C.c_void_p(264)) == 8
    assert lib.admmq_stream_copy(h, one, None, 64) == 1 and lib.admmq_stream_copy(h, one, one, 24) == 2
    assert lib.admmq_stream_copy(h, C.c_void_p(264), one, 64) == 2 and lib.admmq_stream_copy(h, one, one, 64) == 8
    prm = binding._LsParams(1, 1, 4, 0.01, 0)
    assert lib.admmq_local_search(h, one, one, 1, 4, 4, 4, 0, one, one, one, C.byref(prm), None, None, None) == 2
    assert lib.admmq_set_workspace(h, C.c_void_p(100), 1 << 20) == 6
    lib.admmq_destroy(h)
    assert lib.admmq_create(None, 0, None) == 1


def test_format_argument_validation_without_a_gpu(lib):
    h = _ctx(lib)
    one = 256
    sched = binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0)
    F = binding._Format

    def q(fmt, sched=sched, n=8, stats=None):
        return lib.admmq_quantize_layer_format(h, C.c_void_p(one), C.c_void_p(one), n, 4, 4, C.byref(fmt),
                                               C.byref(sched), C.c_void_p(one), C.c_void_p(one), stats)
    dual = F(binding.FORMAT_DUAL_GRID, 3, 4, one, None, one, one)
    book = F(binding.FORMAT_CODEBOOK, 3, 0, None, one, None, None)
    assert q(dual) == 8 and q(book) == 8                                  # valid: stops at the missing device
    assert q(F(binding.FORMAT_DUAL_GRID, 3, 4, None, None, one, one)) == 1       # a dual grid needs its flags
    assert q(F(binding.FORMAT_DUAL_GRID, 3, 4, one, None, None, one)) == 1
    assert q(F(binding.FORMAT_DUAL_GRID, 3, 3, one, None, one, one)) == 2        # group does not divide n
    assert q(F(binding.FORMAT_DUAL_GRID, 1, 4, one, None, one, one)) == 3
    assert q(F(binding.FORMAT_CODEBOOK, 3, 0, None, None, None, None)) == 1      # a codebook format needs one
    assert q(F(binding.FORMAT_CODEBOOK, 5, 0, None, one, None, None)) == 3       # at most 16 levels
    assert q(F(binding.FORMAT_CODEBOOK, 3, 4, None, one, None, None)) == 3       # levels are per column
    assert q(F(7, 3, 0, None, one, None, None)) == 3
    with_ls = binding._Schedule(10, 0.1, 1.1, 0.01, 1, 2, 0, 0, -1, 0, 0, 0.8, 0, 0)
    with_refresh = binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, 5, 0, 0, 0.8, 0, 0)
    assert q(book, sched=with_ls) == 3 and q(dual, sched=with_refresh) == 3
    assert q(dual, sched=binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0, 2)) == 3    # quiet_stop
    st = binding._Stats()
    flips = (C.c_int64 * 10)()
    st.code_flips = C.cast(flips, C.POINTER(C.c_int64))
    assert q(book, stats=C.byref(st)) == 3
    pd = lambda fmt, rho=0.5: lib.admmq_project_dual_format(
        h, C.c_void_p(one), C.c_void_p(one), 8, 4, C.c_void_p(one), C.byref(fmt), rho, 0.55, None,
        C.c_void_p(one), None, None)
    assert pd(dual) == 8 and pd(book) == 8 and pd(book, rho=0.0) == 3
    assert lib.admmq_grid_init_dual(h, C.c_void_p(one), 8, 4, 4, C.byref(dual)) == 8
    assert lib.admmq_grid_init_dual(h, C.c_void_p(one), 8, 4, 4, C.byref(book)) == 3
    assert lib.admmq_grid_init_dual(h, C.c_void_p(one), 8, 4, 3, C.byref(dual)) == 2
    lib.admmq_destroy(h)


def test_batched_layers_argument_validation_without_a_gpu(lib):
    h = _ctx(lib)
    one = 256
    sched = binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0)
    Lr = binding._Layer

    def q(layers, count=None, sched=sched, n=8, H=one):
        arr = (Lr * max(len(layers), 1))(*layers)
        return lib.admmq_quantize_layers(h, C.c_void_p(H) if H else None, n, arr,
                                         len(layers) if count is None else count, C.byref(sched), None)
    good = Lr(one, 4, 4, 3, 0, one, one, one)
    wide = Lr(one, 6, 8, 4, 4, one, one, one)
    assert q([good]) == 8 and q([good, wide]) == 8                        # valid: stops at the missing device
    assert q([good], count=0) == 2 and q([good], count=65) == 2
    assert q([good], H=0) == 1
    assert q([good, Lr(None, 4, 4, 3, 0, one, one, one)]) == 1            # every matrix needs its weights
    assert q([good, Lr(one, 4, 4, 3, 0, None, one, one)]) == 1            # ... and its outputs
    assert q([good, Lr(one, 4, 3, 3, 0, one, one, one)]) == 2             # ldw < p
    assert q([good, Lr(one, 4, 4, 3, 3, one, one, one)]) == 2             # group does not divide n
    assert q([good, Lr(one, 4, 4, 9, 0, one, one, one)]) == 3
    with_refresh = binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, 5, 0, 0, 0.8, 0, 0)
    assert q([good, wide], sched=with_refresh) == 3                       # the refresh is a per-matrix decision
    with_stop = binding._Schedule(10, 0.1, 1.1, 0.01, 1, 0, 0, 0, -1, 0, 0, 0.8, 0, 0, 3)
    assert q([good, wide], sched=with_stop) == 8                          # stopping early is allowed (joint rule)
    assert lib.admmq_quantize_layers(h, C.c_void_p(one), 8, None, 1, C.byref(sched), None) == 1
    lib.admmq_destroy(h)


def test_fast_products_switch_and_scratch_size(lib):
    """The opt-in split-fp16 products: the switch takes 0 or 1; the extra scratch is reported only for shapes the
    products take (whole 256 x 256 tiles, enough of them times k-slices to fill the chip) and then holds the fp16 pairs of Q, Q^T (4 n^2
    values) and of one n x p operand."""
    h = _ctx(lib)
    assert lib.admmq_set_fast_products(None, 1) == 1
    assert lib.admmq_set_fast_products(h, 2) == 3 and lib.admmq_set_fast_products(h, -1) == 3
    assert lib.admmq_set_fast_products(h, 1) == 0 and lib.admmq_set_fast_products(h, 0) == 0
    fb = lib.admmq_fast_products_bytes
    assert fb(4096, 4096) >= 4 * 4096 * 4096 * 2 + 2 * 4096 * 4096 * 2
    assert fb(4096, 4096) < 4 * 4096 * 4096 * 2 + 2 * 4096 * 4096 * 2 + (1 << 16)
    # 64 tiles: the k axis is cut into four slices, whose partial sums need scratch as well
    assert fb(4096, 1024) >= 4 * 4096 * 4096 * 2 + 2 * 4096 * 1024 * 2 + 4 * 4096 * 1024 * 4
    assert fb(4096, 3328) > 0 and fb(4096, 3072) > 0
    assert fb(512, 512) == 0 and fb(1024, 256) == 0  # too small to fill the chip even in eight slices
    assert fb(4100, 4096) == 0 and fb(4096, 4100) == 0 and fb(0, 4096) == 0
    assert fb(25600, 5120) > fb(12288, 4096) > fb(4096, 4096)
    # 320 tiles: the 256 that fill a launch round go out whole, the other 64 (1024 columns) in four slices
    base = 4 * 4096 * 4096 * 2 + 2 * 4096 * 5120 * 2
    assert base + 4 * 4096 * 1024 * 4 <= fb(4096, 5120) < base + 4 * 4096 * 1024 * 4 + (1 << 16)
    # 2000 tiles (7.8 rounds): nothing to gain from a split, no partial sums
    assert fb(25600, 5120) < 4 * 25600 * 25600 * 2 + 2 * 25600 * 5120 * 2 + (1 << 16)
    lib.admmq_destroy(h)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "library_path", lambda: "/nonexistent/libadmmq.so")
    with pytest.raises(admmq.AdmmqError):
        binding.load_library()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
