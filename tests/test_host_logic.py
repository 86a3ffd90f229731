"""CPU-only checks of the host side: the C-ABI library loads and exports what include/qsl.h declares,
argument errors are caught before any GPU work, the workload generators are deterministic, and
bench.py refuses more than one GPU."""
import ctypes as C
import os
import re
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
from paper_1906_02367_amd import workloads as W  # noqa: E402
from paper_1906_02367_amd.build import LIB_PATH  # noqa: E402


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB_PATH):
        from paper_1906_02367_amd import build
        build.build()
    return C.CDLL(LIB_PATH)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "qsl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qsl_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"qsl_compress", "qsl_error_update", "qsl_aggregate", "qsl_bits_sent", "qsl_create"} <= set(names)
    for name in names:
        assert getattr(lib, name) is not None, name


def test_binding_lists_the_same_entry_points():
    src = open(os.path.join(ROOT, "paper_1906_02367_amd", "binding.py")).read()
    listed = set(re.findall(r'"(qsl_[a-z_]+)"', src))
    assert set(declared_functions()) <= listed


class Config(C.Structure):
    _fields_ = [("d", C.c_uint64), ("num_segments", C.c_uint32), ("seg_offset", C.POINTER(C.c_uint64)),
                ("seg_k", C.POINTER(C.c_uint32)), ("s", C.c_uint32), ("sparsifier", C.c_uint32),
                ("quantizer", C.c_uint32), ("seed", C.c_uint64), ("max_workers", C.c_uint32), ("flags", C.c_uint32)]


def make_cfg(d, off, k, s=16, sp=0, qz=0, R=1):
    off_a = (C.c_uint64 * len(off))(*off)
    k_a = (C.c_uint32 * len(k))(*k)
    cfg = Config(d, len(k), off_a, k_a, s, sp, qz, 1, R, 0)
    cfg._keep = (off_a, k_a)
    return cfg


@pytest.mark.parametrize("kwargs", [
    dict(d=0, off=[0, 0], k=[1]),                      # empty vector
    dict(d=100, off=[0, 100], k=[0]),                  # k = 0
    dict(d=100, off=[0, 100], k=[101]),                # k > d
    dict(d=100, off=[1, 100], k=[5]),                  # offsets do not start at 0
    dict(d=100, off=[0, 60, 50, 100], k=[1, 1, 1]),    # offsets not increasing
    dict(d=100, off=[0, 100], k=[5], s=0),             # no quantisation levels
    dict(d=100, off=[0, 100], k=[5], s=40000),         # too many levels
    dict(d=100, off=[0, 100], k=[5], sp=2),            # unknown sparsifier
    dict(d=100, off=[0, 100], k=[5], qz=7),            # unknown quantiser
    dict(d=100, off=[0, 100], k=[5], R=0),             # no workers
    dict(d=1 << 32, off=[0, 1 << 32], k=[5]),          # d out of range
])
def test_invalid_configurations_are_rejected_before_any_gpu_work(lib, kwargs):
    lib.qsl_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(Config), C.c_void_p]
    lib.qsl_create.restype = C.c_int
    ctx = C.c_void_p()
    cfg = make_cfg(**kwargs)
    assert lib.qsl_create(C.byref(ctx), C.byref(cfg), None) == 1          # QSL_ERR_INVALID_ARG
    assert not ctx.value


@pytest.mark.parametrize("qz,s", [(0, 1), (0, 2), (0, 3), (0, 15), (0, 16), (0, 255), (0, 256), (1, 1), (2, 1), (3, 1), (4, 7)])
def test_index_free_bit_count_of_rand_k(lib, qz, s):
    """Host-only entry point against the oracle's count, and against a message the oracle builds: for the
    quantisers that send all k coordinates, dropping the nnz word and the index field of the transmitted
    format must leave exactly the index-free count."""
    from oracle import oracle as O
    lib.qsl_bits_index_free.argtypes = [C.POINTER(Config), C.POINTER(C.c_uint64)]
    lib.qsl_bits_index_free.restype = C.c_int
    d, off, k = 5_000, [0, 100, 1_124, 5_000], [7, 100, 1]
    bits = C.c_uint64(0)
    cfg = make_cfg(d, off, k, s=s, sp=1, qz=qz)
    assert lib.qsl_bits_index_free(C.byref(cfg), C.byref(bits)) == 0
    op = O.OracleOp(d, off, k, s, O.RANDK, qz, 1)
    assert bits.value == op.bits_index_free()
    if qz in (1, 2, 3):
        v = np.random.default_rng(3).standard_normal(d).astype(np.float32)
        out = op.compress(np.zeros(d, np.float32), v, 0, 0)
        w_idx = 13                                                          # bits of d - 1 = 4999
        assert op.bits_sent(out["msg"]) - 32 - sum(k) * w_idx == bits.value
    cfg = make_cfg(d, off, k, s=s, sp=0, qz=qz)
    assert lib.qsl_bits_index_free(C.byref(cfg), C.byref(bits)) == 5        # QSL_ERR_UNSUPPORTED for Top_k
    assert lib.qsl_bits_index_free(None, C.byref(bits)) == 1


@pytest.mark.parametrize("s", [1, 2, 3, 15, 16, 255, 256])
def test_index_free_qsgd_stream_written_out_and_read_back(lib, s):
    """The index-free count for QSGD, pinned without consulting either formula: the stream is written here, code by
    code, from the oracle's levels and signs (every one of the K chosen coordinates, level 0 included, in the fewest
    whole bits that can tell s + 1 levels apart, then one sign bit), read back with a reader of this test, and
    dequantised as Definition 1's example does (norm * level / s); it must reproduce the values the oracle sent, and
    its length must equal both counts.  A field one bit too narrow cannot hold level s; one bit too wide changes the length."""
    from oracle import oracle as O
    lib.qsl_bits_index_free.argtypes = [C.POINTER(Config), C.POINTER(C.c_uint64)]
    lib.qsl_bits_index_free.restype = C.c_int
    d, off, k = 5_000, [0, 100, 1_124, 5_000], [7, 100, 1]
    op = O.OracleOp(d, off, k, s, O.RANDK, O.QSGD, 7)
    rng = np.random.default_rng(s)
    v = (rng.standard_normal(d) * np.exp(rng.standard_normal(d))).astype(np.float32)
    out = op.compress(np.zeros(d, np.float32), v, 2, 5)
    levels, negs = out["sel_level"].astype(int), out["sel_neg"].astype(int)
    assert levels.max() <= s and (levels == s).any() or s > 3          # a segment with k = 1 always reaches level s
    n_level_bits = 0
    while (1 << n_level_bits) < s + 1:                                  # fewest bits for the s + 1 values 0..s
        n_level_bits += 1
    stream = []                                                         # one bit per list element, first bit first

    def put(value, width):
        assert 0 <= value < (1 << width), "the field cannot hold the value"
        for b in range(width):
            stream.append((value >> b) & 1)

    for scale in out["scales"]:
        put(int(np.float32(scale).view(np.uint32)), 32)
    for lv, ng in zip(levels, negs):
        put(int(lv), n_level_bits)
        put(int(ng), 1)
    # read it back
    pos = 0

    def get(width):
        nonlocal pos
        x = sum(bit << b for b, bit in enumerate(stream[pos:pos + width]))
        pos += width
        return x

    scales = [np.uint32(get(32)).view(np.float32) for _ in k]
    seg_of = np.repeat(np.arange(len(k)), k)
    vals = []
    for j in range(sum(k)):
        lv, ng = get(n_level_bits), get(1)
        mag = np.float32(np.float32(scales[seg_of[j]] * np.float32(lv)) / np.float32(s))
        vals.append(np.float32(0.0) if lv == 0 else (-mag if ng else mag))     # level 0 stands for "nothing sent"
    assert pos == len(stream)
    assert np.array_equal(np.array(vals, dtype=np.float32).view(np.uint32), out["g_val"].view(np.uint32))
    bits = C.c_uint64(0)
    cfg = make_cfg(d, off, k, s=s, sp=1, qz=0)
    assert lib.qsl_bits_index_free(C.byref(cfg), C.byref(bits)) == 0
    assert len(stream) == bits.value == op.bits_index_free()


def test_message_too_long_for_the_word_counters_is_refused(lib):
    """More than 2^32 message words (K above ~2.1e9 with 32-bit indices and fp32 values): refused at qsl_create,
    before any GPU work, instead of truncating the word count."""
    lib.qsl_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(Config), C.c_void_p]
    lib.qsl_create.restype = C.c_int
    ctx = C.c_void_p()
    d = 4_000_000_000
    cfg = make_cfg(d, [0, d], [2_200_000_000], s=1, sp=0, qz=3)
    assert lib.qsl_create(C.byref(ctx), C.byref(cfg), None) == 5          # QSL_ERR_UNSUPPORTED
    assert not ctx.value
    cfg = make_cfg(100, [0, 100], [5])
    cfg.flags = 1 << 9                                                    # an unknown flag
    assert lib.qsl_create(C.byref(ctx), C.byref(cfg), None) == 1


def plan(lib, d, off, k, sp=0, qz=0, flags=0, s=16):
    lib.qsl_plan_paths.argtypes = [C.POINTER(Config), C.POINTER(C.c_uint32)]
    lib.qsl_plan_paths.restype = C.c_int
    cfg = make_cfg(d, off, k, s=s, sp=sp, qz=qz)
    cfg.flags = flags
    out = (C.c_uint32 * len(k))()
    assert lib.qsl_plan_paths(C.byref(cfg), out) == 0
    return list(out)


def test_plan_of_the_selection_paths(lib):
    """The host's per-segment decision (made by the same code in qsl_create), without a GPU."""
    FAST, MULTI, ONE_BLOCK, ALL_KEPT = 0, 1, 3, 4
    # one segment: sparse -> guess; dense -> multi-pass; tiny -> one block; k = size -> nothing to select
    assert plan(lib, 25_557_032, [0, 25_557_032], [25_557]) == [FAST]
    assert plan(lib, 25_557_032, [0, 25_557_032], [2_555_703]) == [MULTI]
    assert plan(lib, 4_096, [0, 4_096], [40]) == [ONE_BLOCK]
    assert plan(lib, 4_097, [0, 4_097], [10]) == [FAST]
    assert plan(lib, 4_097, [0, 4_097], [40]) == [FAST]
    assert plan(lib, 4_097, [0, 4_097], [400]) == [ONE_BLOCK]     # too dense to guess, small enough for one block (up to 40,960)
    assert plan(lib, 40_960, [0, 40_960], [4_000]) == [ONE_BLOCK]
    assert plan(lib, 40_961, [0, 40_961], [4_000]) == [MULTI]
    assert plan(lib, 4_096, [0, 4_096], [4_096]) == [ONE_BLOCK]
    assert plan(lib, 300_000, [0, 300_000], [300_000]) == [ALL_KEPT]
    # the candidates of a chunk must fit its slot (at most 63): 1000 of 65,536 does, 3000 of 100,000 is too dense to guess at all
    assert plan(lib, 65_536, [0, 65_536], [1_000]) == [FAST]
    assert plan(lib, 100_000, [0, 100_000], [3_000]) == [MULTI]
    assert plan(lib, 262_144, [0, 262_144], [1_000]) == [FAST]
    # Rand_k guesses analytically when at most ~14 candidates fall into a chunk
    assert plan(lib, 25_557_032, [0, 25_557_032], [255_570], sp=1) == [FAST]
    assert plan(lib, 25_557_032, [0, 25_557_032], [2_555_703], sp=1) == [MULTI]
    # the testing flags
    assert plan(lib, 25_557_032, [0, 25_557_032], [25_557], flags=1) == [MULTI]
    assert plan(lib, 4_096, [0, 4_096], [40], flags=2) == [MULTI]
    assert plan(lib, 4_096, [0, 4_096], [40], flags=3) == [MULTI]
    assert plan(lib, 30_000, [0, 30_000], [3_000], flags=2) == [MULTI]
    assert plan(lib, 300_000, [0, 300_000], [300_000], flags=1) == [MULTI]
    # the paper's ResNet-50 setting (Section 5.1.1): 119 tensors for one block each (108 of at most 4096 coordinates, 11
    # larger ones that are too dense for guessing), 42 that guess, none left for the multi-pass kernels
    wl = W.config(6)
    paths = plan(lib, wl.d, [int(x) for x in wl.seg_offset], [int(x) for x in wl.seg_k], qz=1, s=1)
    assert (paths.count(ONE_BLOCK), paths.count(MULTI), paths.count(FAST), paths.count(ALL_KEPT)) == (119, 0, 42, 0)
    # invalid descriptions are refused
    cfg = make_cfg(100, [0, 100], [101])
    out = (C.c_uint32 * 1)()
    assert lib.qsl_plan_paths(C.byref(cfg), out) == 1 and lib.qsl_plan_paths(None, out) == 1


def test_null_arguments_and_status_strings(lib):
    lib.qsl_status_string.argtypes = [C.c_int]
    lib.qsl_status_string.restype = C.c_char_p
    assert lib.qsl_status_string(0) == b"ok" and b"non-finite" in lib.qsl_status_string(3)
    lib.qsl_compress.restype = C.c_int
    assert lib.qsl_compress(None, None, None, None, 0, 1, 0, None, None, None, None) == 1
    lib.qsl_msg_capacity_bytes.restype = C.c_size_t
    lib.qsl_msg_capacity_bytes.argtypes = [C.c_void_p]
    assert lib.qsl_msg_capacity_bytes(None) == 0
    lib.qsl_destroy.argtypes = [C.c_void_p]
    assert lib.qsl_destroy(None) == 1


def test_workload_tables():
    for cfg, (R, d, K) in {1: (2, 65_536, 655), 2: (8, 25_557_032, 25_557), 3: (8, 25_557_032, 255_570),
                           5: (4, 1 << 28, 26_844)}.items():
        wl = W.config(cfg)
        assert (wl.R, wl.d, wl.K, wl.L) == (R, d, K, 1)
    wl = W.config(4)
    sizes = np.diff(wl.seg_offset.astype(np.int64))
    assert wl.L == 160 and sizes.sum() == 25_557_032 and sizes.min() >= 64 and sizes.max() <= 2_400_001 * 1.2
    assert np.array_equal(wl.seg_k, (sizes + 999) // 1000)
    a, b = W.config(4), W.config(4)
    assert np.array_equal(a.seg_offset, b.seg_offset)


def test_resnet50_tensor_table_gives_the_total_k_the_paper_prints():
    """Section 5.1.1: k_t = min(d_t, 1000) for each tensor of ResNet-50 gives a total of k = 99,400."""
    sizes = W.resnet50_tensor_sizes()
    assert len(sizes) == 161 and sum(sizes) == 25_557_032
    assert sum(min(n, 1000) for n in sizes) == 99_400
    wl = W.config(6)
    assert wl.L == 161 and wl.K == 99_400 and wl.d == 25_557_032 and wl.R == 8
    assert np.array_equal(np.diff(wl.seg_offset.astype(np.int64)), np.array(sizes))
    assert wl.sparsifier == W.TOPK and wl.quantizer == W.SIGN_L1


def test_host_generators_are_deterministic_and_shaped():
    wl = W.config(2, d=10_000, R=3)
    a = W.delta_all(wl, 4)
    b = W.delta_all(wl, 4)
    assert a.shape == (3, 10_000) and a.dtype == np.float32 and np.array_equal(a, b)
    assert not np.array_equal(a, W.delta_all(wl, 5))
    assert not np.array_equal(a[0], a[1])
    # the component shared by the workers: rows are positively correlated after removing the scale
    sig = W._sigma(wl)
    z = a / sig
    assert np.corrcoef(z[0], z[1])[0, 1] > 0.3
    wl5 = W.config(5, d=20_000, R=1)
    t = W.delta(wl5, 0, 0)
    assert np.isfinite(t).all() and np.abs(t).max() > 20 * np.median(np.abs(t))      # heavy tails


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "ONE GPU" in res.stderr
