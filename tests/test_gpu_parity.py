"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs -- indices, level codes, packed bytes, bit counts and the error memory bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import oracle as O  # noqa: E402
from paper_1906_02367_amd import workloads as W  # noqa: E402

f32 = np.float32


@pytest.fixture(scope="module")
def P():
    import parity_util
    return parity_util


def custom(d, seg_offset, seg_k, s, sparsifier, quantizer, R, name="custom", cfg=2, seed=12345):
    return W.Workload(cfg, name, R, d, np.asarray(seg_offset, dtype=np.uint64), np.asarray(seg_k, dtype=np.uint32), s,
                      sparsifier, quantizer, 1, seed)


# ---------------------------------------------------------------------------------------------
# small shapes: the general (multi-pass) path; several tiles and a ragged tail
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_configs_reduced_size(P, cfg):
    d = {1: 65_536, 2: 70_001, 3: 70_001, 4: 150_000, 5: 99_991}[cfg]
    wl = W.config(cfg, d=d, R=2 if cfg != 1 else None, rounds=4)
    print(f"\n[{wl.name}] d={wl.d} K={wl.K} L={wl.L}", flush=True)
    P.run_parity(wl, 4 if cfg != 1 else 10)


@pytest.mark.parametrize("sparsifier", [W.TOPK, W.RANDK])
@pytest.mark.parametrize("quantizer,s", [(W.QSGD, 15), (W.QSGD, 1), (W.QSGD, 32768), (W.SIGN_L1, 1), (W.SIGN_L2, 1),
                                         (W.FP32, 1), (W.QSGD_SCALED, 4), (W.QSGD_SCALED, 15), (W.SIGN_L3, 1), (W.SIGN_L4, 1)])
def test_operator_grid_small(P, sparsifier, quantizer, s):
    wl = custom(40_003, [0, 40_003], [777], s, sparsifier, quantizer, R=3)
    P.run_parity(wl, 2, worker0=5)


@pytest.mark.parametrize("quantizer,s", [(W.SIGN_L2, 1), (W.FP32, 1), (W.QSGD_SCALED, 2), (W.SIGN_L3, 1), (W.SIGN_L4, 1)])
def test_operator_variants_on_the_fast_path_and_layerwise(P, quantizer, s):
    # the variants next to the hot path: sign scaled by the l2, l3, l4 norm (Lemma 3, m = 2, 3, 4), no quantiser
    # (TopK-SGD), scaled QSGD (Lemma 2)
    wl = custom(1_000_003, [0, 1_000_003], [1000], s, W.TOPK, quantizer, R=2)
    run, op, m_host, _ = P.run_parity(wl, 2, expect_path=0)
    out = torch.zeros(wl.d, dtype=torch.float32, device=run.q.device)
    run.q.aggregate(run.msg, out, 0.5)
    torch.cuda.synchronize()
    want = op.aggregate(run.msg.cpu().numpy(), 0.5)
    assert np.allclose(out.cpu().numpy(), want, rtol=1e-6, atol=1e-30)
    off = [0, 64, 1_000, 40_000, 70_001]
    wl = custom(70_001, off, [3, 10, 400, 30], s, W.RANDK, quantizer, R=2)
    P.run_parity(wl, 2)


def test_not_in_place(P):
    wl = W.config(2, d=50_000, R=2)
    P.run_parity(wl, 3, in_place=False)


# ---------------------------------------------------------------------------------------------
# the single-pass fast path (guess + candidate pool) at sizes that enable it
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,d", [(2, 1_000_003), (3, 600_011), (5, 4_000_037)])
def test_fast_path_mid_size(P, cfg, d):
    wl = W.config(cfg, d=d, R=3, rounds=3)
    print(f"\n[{wl.name}] d={wl.d} K={wl.K}", flush=True)
    P.run_parity(wl, 3, expect_path=0)


def test_fast_and_general_paths_agree_layerwise(P):
    # segments from 64 coordinates to ~1.9 M: a mix of fast and general units in one call
    wl = W.config(4, d=20_000_000, R=2)
    run, op, m_host, paths = P.run_parity(wl, 2)
    assert (paths[0] == 0).any() and (paths[0] == 3).any()
    run, op, m_host, paths = P.run_parity(wl, 1, flags=3)          # every unit through the multi-pass kernels
    assert (paths[0] == 1).all()


def test_failed_guess_falls_back(P):
    # large values exactly where the sample looks -> the guess is far too high -> too few candidates
    d, k, R = 1_000_003, 1000, 2
    wl = custom(d, [0, d], [k], 16, W.TOPK, W.QSGD, R)
    rng = np.random.default_rng(3)
    delta = rng.standard_normal((R, d)).astype(f32)
    n_s = 42.25 * 3.0 / (4.0 * (k / d))                    # the library's sampling plan at alpha = 3
    n_runs = int(np.ceil(n_s / 64.0))
    starts = np.arange(n_runs, dtype=np.int64) * (d // n_runs)          # the library samples runs of 64 at this stride
    pos = (starts[:, None] + np.arange(64)[None, :]).ravel()
    delta[:, pos] *= 1000.0
    run, op, m_host, paths = P.run_parity(wl, 1, deltas=[delta])
    assert np.all(paths[0] == 2), paths
    # ... and the opposite failure: tiny values where the sample looks -> far too many candidates
    delta = rng.standard_normal((R, d)).astype(f32)
    delta[:, pos] *= 1e-6
    run, op, m_host, paths = P.run_parity(wl, 1, deltas=[delta])
    print("paths after a low guess:", paths)


def test_clustered_candidates_use_the_overflow_pool(P):
    # most of the large values sit in a few chunks of 1024 coordinates: their slots cannot hold them,
    # they spill to the overflow pool, and the unit still runs on the single-pass path
    d, k, R = 1_000_003, 1000, 2
    rng = np.random.default_rng(23)
    for sp, qz, s in [(W.TOPK, W.QSGD, 16), (W.TOPK, W.SIGN_L1, 1)]:
        wl = custom(d, [0, d], [k], s, sp, qz, R)
        deltas = []
        for t in range(2):
            delta = rng.standard_normal((R, d)).astype(f32)
            for r in range(R):
                delta[r, 5_000:5_700] *= 50.0                  # 700 coordinates of one chunk-and-a-bit
                delta[r, 777_000:777_040] *= 80.0
                hot = rng.choice(d, 300, replace=False)
                delta[r, hot] *= 30.0
            deltas.append(delta)
        P.run_parity(wl, 2, deltas=deltas, expect_path=0)


# ---------------------------------------------------------------------------------------------
# degenerate inputs
# ---------------------------------------------------------------------------------------------
def _adversarial(d, rng):
    yield "all_equal", np.full(d, 1.5, dtype=f32)
    yield "all_zero", np.zeros(d, dtype=f32)
    yield "signed_zeros", np.where(np.arange(d) % 2 == 0, 0.0, -0.0).astype(f32)
    one = np.full(d, 1e-3, dtype=f32); one[d // 3] = -1e6
    yield "one_dominant", one
    yield "denormals", (rng.integers(-200, 200, d) * 1e-45).astype(f32)
    yield "few_values", rng.integers(-2, 3, d).astype(f32)
    yield "wide_range", (rng.standard_normal(d) * np.exp(8 * rng.standard_normal(d))).astype(f32)


@pytest.mark.parametrize("flags,path", [(0, 3), (2, 1)])      # one-block selection / multi-pass kernels
@pytest.mark.parametrize("quantizer,s", [(W.QSGD, 16), (W.SIGN_L1, 1)])
@pytest.mark.parametrize("k", [1, 37, 4_001])
def test_degenerate_inputs(P, quantizer, s, k, flags, path):
    d = 4_001
    rng = np.random.default_rng(17)
    wl = custom(d, [0, d], [k], s, W.TOPK, quantizer, R=1)
    if k == d and flags == 2:
        path = 4                                     # nothing to select: not a case for the multi-pass kernels
    for name, v in _adversarial(d, rng):
        P.run_parity(wl, 1, deltas=[v[None, :].copy()], flags=flags, expect_path=path)


@pytest.mark.parametrize("d,k", [(40_009, 1), (40_009, 37), (40_009, 200), (12_011, 1), (12_011, 37), (12_011, 60)])
def test_degenerate_inputs_whole_unit_guess(P, k, d):
    # 5 .. 255 chunks: the guess comes from a histogram of the whole unit; inputs with few distinct
    # magnitudes put everything into one bin, overflow the candidate list and must fall back
    rng = np.random.default_rng(23)
    wl = custom(d, [0, d], [k], 16, W.TOPK, W.QSGD, R=1)
    seen = set()
    for name, v in _adversarial(d, rng):
        run, op, m_host, paths = P.run_parity(wl, 1, deltas=[v[None, :].copy()])
        seen.update(paths[0].tolist())
    assert seen == {0, 2}, seen


# sizes around the limit of the one-block selection (4096 coordinates) and of its 16-per-thread layout
@pytest.mark.parametrize("sparsifier", [W.TOPK, W.RANDK])
@pytest.mark.parametrize("d,k", [(4_096, 100), (4_096, 4_096), (4_097, 4_097), (4_097, 3), (4_095, 4_095), (2_063, 1_000),
                                 (16_385, 16_385), (8_209, 4_000), (32_769, 1), (65_537, 655), (17, 16), (15, 15),
                                 (1_025, 1_024), (262_143, 250)])
def test_small_units_one_block_boundaries(P, sparsifier, d, k):
    small = d <= 4_096
    wl = custom(d, [0, d], [k], 7, sparsifier, W.QSGD, R=2)
    P.run_parity(wl, 2, expect_path=3 if small else None)
    wl = custom(d, [0, d], [k], 1, sparsifier, W.SIGN_L1, R=2)
    P.run_parity(wl, 1, flags=3, expect_path=1)                   # the same through the multi-pass kernels
    ties = np.round(np.random.default_rng(d).standard_normal((1, 2, d)) * 2).astype(f32)     # many equal magnitudes
    P.run_parity(wl, 1, deltas=ties, expect_path=3 if small else None)


def test_small_and_large_units_mixed(P):
    # one call with one-block units, multi-pass units and guessed units side by side
    off = [0, 100, 70_000, 70_001, 400_000, 410_000, 1_100_000]
    k = [100, 70, 1, 30_000, 650, 600]
    for sp, qz, s in [(W.TOPK, W.QSGD, 16), (W.RANDK, W.SIGN_L1, 1)]:
        wl = custom(1_100_000, off, k, s, sp, qz, R=3)
        run, op, m_host, paths = P.run_parity(wl, 2)
        assert sorted(set(paths[0].tolist())) == [0, 1, 3], paths[0]


def test_degenerate_inputs_on_fast_sizes(P):
    d, k = 600_000, 500
    rng = np.random.default_rng(19)
    wl = custom(d, [0, d], [k], 4, W.TOPK, W.QSGD, R=1)
    for name, v in _adversarial(d, rng):
        print(name, flush=True)
        P.run_parity(wl, 1, deltas=[v[None, :].copy()])


def test_tiny_segments_and_unaligned_offsets(P):
    off = [0, 64, 65, 130, 1_031, 5_000, 5_003, 40_000, 70_001]
    k = [1, 1, 65, 9, 100, 3, 35, 30_001]
    for sp, qz, s in [(W.TOPK, W.SIGN_L1, 1), (W.TOPK, W.QSGD, 4), (W.RANDK, W.QSGD, 2)]:
        wl = custom(70_001, off, k, s, sp, qz, R=3)
        P.run_parity(wl, 2)


def test_d_equals_one_and_k_equals_d(P):
    wl = custom(1, [0, 1], [1], 16, W.TOPK, W.QSGD, R=2)
    P.run_parity(wl, 2)
    wl = custom(5_000, [0, 5_000], [5_000], 16, W.TOPK, W.QSGD, R=1)      # QSGD on the whole vector
    P.run_parity(wl, 2)
    # the sign of the whole vector (every message lists every coordinate), and the master line on such messages
    wl = custom(20_003, [0, 20_003], [20_003], 1, W.TOPK, W.SIGN_L1, R=3)
    run, op, m_host, _ = P.run_parity(wl, 2)
    x0 = np.random.default_rng(8).standard_normal(wl.d).astype(f32)
    out = torch.from_numpy(x0).to(run.q.device)
    run.q.aggregate(run.msg, out, -1.0 / 3, worker_list=[2, 0], accumulate=True)
    torch.cuda.synchronize()
    msgs = run.msg.cpu().numpy()
    want = op.aggregate(msgs, -1.0 / 3, worker_list=[2, 0], out=x0)
    mag = sum(np.abs(op.decode(msgs[r])[1].astype(np.float64)) for r in (2, 0))
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - want) <= 1e-6 * (mag / 3 + np.abs(want)) + 1e-38)


# k = size of the segment (the error-feedback schemes without sparsification that Section 5 compares with, as
# this operator): no selection at all; ragged sizes around the 4096-coordinate tiles and the 512-block limit
@pytest.mark.parametrize("sparsifier", [W.TOPK, W.RANDK])
@pytest.mark.parametrize("quantizer,s", [(W.QSGD, 15), (W.SIGN_L1, 1), (W.SIGN_L2, 1), (W.FP32, 1), (W.QSGD_SCALED, 3),
                                         (W.SIGN_L3, 1), (W.SIGN_L4, 1)])
def test_every_coordinate_kept(P, sparsifier, quantizer, s):
    for d in (4_097, 300_001, 2_200_003):                        # 2, 74 and 538 tiles (more than the blocks of a unit)
        wl = custom(d, [0, d], [d], s, sparsifier, quantizer, R=2)
        run, op, m_host, _ = P.run_parity(wl, 2, expect_path=4)
        if d == 300_001:
            # the master line on messages that list every coordinate; the third listed row is an empty (all-zero) message
            msgs = torch.cat([run.msg, torch.zeros_like(run.msg[:1])])
            msgs_host = msgs.cpu().numpy()
            x0 = np.random.default_rng(d).standard_normal(d).astype(f32)
            for lst, accumulate in (([1, 0], False), ([0, 2, 1], True)):
                out = torch.from_numpy(x0).to(run.q.device)
                run.q.aggregate(msgs, out, -0.5, worker_list=lst, accumulate=accumulate)
                torch.cuda.synchronize()
                want = op.aggregate(msgs_host, -0.5, worker_list=lst, out=x0.copy() if accumulate else None)
                mag = np.zeros(d)
                for r in lst:
                    i, vv = op.decode(msgs_host[r])
                    mag[i] += np.abs(vv.astype(np.float64))
                got = out.cpu().numpy().astype(np.float64)
                assert np.all(np.abs(got - want) <= 1e-6 * (mag * 0.5 + np.abs(want)) + 1e-38)
            from paper_1906_02367_amd import binding as B
            assert run.q.device_status() == B.OK
    # segments that keep everything beside segments that select, in one call; degenerate values
    off = [0, 5_000, 70_000, 70_001, 400_000, 410_001, 1_100_000]
    k = [5_000, 65_000, 1, 30_000, 10_001, 600]
    wl = custom(1_100_000, off, k, s, sparsifier, quantizer, R=3)
    run, op, m_host, paths = P.run_parity(wl, 2)
    assert paths[0].reshape(3, 6)[0].tolist() == [4, 4, 3, 1, 4, 0], paths[0]
    rng = np.random.default_rng(31)
    d = 50_000
    wl = custom(d, [0, d], [d], s, sparsifier, quantizer, R=1)
    for name, v in _adversarial(d, rng):
        P.run_parity(wl, 1, deltas=[v[None, :].copy()], expect_path=4)
    P.run_parity(wl, 1, flags=1, expect_path=1)                   # the same through the multi-pass kernels


def test_plan_query_agrees_with_what_the_kernels_report(P):
    # the host-only plan (qsl_plan_paths) and the path each unit reports after a call (no guess fails on these inputs)
    from paper_1906_02367_amd import binding as B
    off = [0, 100, 70_000, 70_001, 400_000, 410_001, 1_100_000]
    k = [100, 70, 1, 30_000, 10_001, 600]
    for sp, qz, s, flags in [(W.TOPK, W.QSGD, 16, 0), (W.RANDK, W.SIGN_L1, 1, 0), (W.TOPK, W.SIGN_L1, 1, 2), (W.TOPK, W.FP32, 1, 3)]:
        wl = custom(1_100_000, off, k, s, sp, qz, R=2)
        run, op, m_host, paths = P.run_parity(wl, 1, flags=flags)
        plan = B.plan_paths(wl.d, wl.seg_offset, wl.seg_k, wl.s, wl.sparsifier, wl.quantizer, flags)
        assert paths[0].reshape(2, len(k)).tolist() == [plan.tolist()] * 2, (paths[0], plan)


# ---------------------------------------------------------------------------------------------
# the other entry points
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg", [1, 2, 4])
def test_aggregate_error_update_bits(P, cfg):
    from paper_1906_02367_amd import binding as B
    wl = W.config(cfg, d=80_000, R=4)
    run, op, m_host, _ = P.run_parity(wl, 2)
    q = run.q
    msgs_host = run.msg.cpu().numpy()
    # payload bits
    assert q.bits_sent(run.msg) == [op.bits_sent(msgs_host[r]) for r in range(wl.R)]
    # master line: all workers, then a subset accumulated onto x with scale -1/R
    out = torch.full((wl.d,), 7.0, dtype=torch.float32, device=q.device)
    q.aggregate(run.msg, out, 1.0 / wl.R)
    torch.cuda.synchronize()
    want = op.aggregate(msgs_host, 1.0 / wl.R)
    dense_abs = np.zeros(wl.d)
    for r in range(wl.R):
        i, v = op.decode(msgs_host[r])
        dense_abs[i] += np.abs(v.astype(np.float64))
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - want) <= 1e-6 * dense_abs / wl.R + 1e-38)
    x0 = np.random.default_rng(5).standard_normal(wl.d).astype(f32)
    out = torch.from_numpy(x0).to(q.device)
    q.aggregate(run.msg, out, -1.0 / wl.R, worker_list=[1, 3], accumulate=True)
    torch.cuda.synchronize()
    want = op.aggregate(msgs_host, -1.0 / wl.R, worker_list=[1, 3], out=x0)
    assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - want) <= 1e-6 * (dense_abs / wl.R + np.abs(want)) + 1e-38)
    # stand-alone error update reproduces the fused one bit for bit
    rng = np.random.default_rng(9)
    m0 = rng.standard_normal((wl.R, wl.d)).astype(f32)
    d0 = W.delta_all(wl, 7)
    m_dev, d_dev = torch.from_numpy(m0).to(q.device), torch.from_numpy(d0).to(q.device)
    m_fused = torch.empty_like(m_dev)
    q.compress(m_dev, d_dev, m_fused, 0, 7, run.msg)
    q.error_update(m_dev, d_dev, run.msg)
    torch.cuda.synchronize()
    assert torch.equal(m_dev.view(torch.int32), m_fused.view(torch.int32))
    assert q.device_status() == B.OK


def test_nonfinite_input_is_reported(P):
    from paper_1906_02367_amd import binding as B
    wl = W.config(2, d=100_000, R=2)
    q = B.from_workload(wl)
    m = torch.zeros(2, wl.d, device=q.device)
    delta = torch.randn(2, wl.d, device=q.device)
    delta[1, 77_777] = float("inf")
    q.compress(m, delta, m, 0, 0, q.new_msg(2))
    assert q.device_status() == B.ERR_NONFINITE_INPUT
    assert q.device_status() == B.OK                     # the word is cleared by the query


def test_argument_errors_are_synchronous(P):
    from paper_1906_02367_amd import binding as B
    wl = W.config(2, d=10_000, R=2)
    q = B.from_workload(wl)
    m = torch.zeros(2, wl.d, device=q.device)
    with pytest.raises(B.QslError):
        q.compress(m, m, m, 0, 1 << 62, q.new_msg(2))                   # round out of range
    big = torch.zeros(3, wl.d, device=q.device)
    with pytest.raises(B.QslError):
        q.compress(big, big, big, 0, 0, q.new_msg(3))                   # R > max_workers
    with pytest.raises(B.QslError):
        B.Qsl(100, [0, 100], [101], 16, B.TOPK, B.QSGD, 1, 1)          # k > d
    with pytest.raises(B.QslError):
        q.aggregate(q.new_msg(2), torch.zeros(wl.d, device=q.device), 1.0, worker_list=[0, 0])


def test_results_do_not_depend_on_launch_history(P):
    # same inputs three times, with unrelated calls in between: identical bytes (no stale scratch)
    wl = W.config(2, d=1_000_003, R=2)
    from paper_1906_02367_amd import binding as B
    q = B.from_workload(wl)
    d0 = torch.from_numpy(W.delta_all(wl, 0)).to(q.device)
    d1 = torch.from_numpy(W.delta_all(wl, 1)).to(q.device)
    outs = []
    for rep in range(3):
        m = torch.zeros(2, wl.d, device=q.device)
        msg = q.new_msg(2)
        q.compress(m, d0, m, 0, 0, msg)
        outs.append((m.clone(), msg.clone()))
        junk = torch.zeros(2, wl.d, device=q.device)
        q.compress(junk, d1 * (rep + 1), junk, 0, 5, q.new_msg(2))
    torch.cuda.synchronize()
    for m, msg in outs[1:]:
        assert torch.equal(m.view(torch.int32), outs[0][0].view(torch.int32)) and torch.equal(msg, outs[0][1])


# ---------------------------------------------------------------------------------------------
# Delta = x_t - xhat_{t+1/2} formed on the fly (the synchronisation line of Algorithm 1 as written)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,d,R", [(2, 1_000_003, 3), (3, 600_011, 2), (1, 65_536, 2), (4, 2_000_000, 5), (2, 70_001, 9)])
def test_compress_diff_matches_oracle_and_plain_entry(P, cfg, d, R):
    from paper_1906_02367_amd import binding as B
    wl = W.config(cfg, d=d, R=R)
    op = P.oracle_for(wl)
    q = B.from_workload(wl)
    rng = np.random.default_rng(cfg * 100 + R)
    x = rng.standard_normal(wl.d).astype(f32)
    m_host = (0.3 * W.delta_all(wl, 11)).astype(f32)
    for t in range(2):
        xhat = (x[None, :] - W.delta_all(wl, t)).astype(f32)            # so that x - xhat has the workload's shape
        m_dev, x_dev, xh_dev = (torch.from_numpy(a).to(q.device) for a in (m_host, x, xhat))
        msg, msg2 = q.new_msg(R).fill_(0xCD), q.new_msg(R)
        m_out, m_out2 = torch.empty_like(m_dev), torch.empty_like(m_dev)
        q.compress_diff(m_dev, x_dev, xh_dev, m_out, 3, t, msg)
        q.compress(m_dev, x_dev.unsqueeze(0) - xh_dev, m_out2, 3, t, msg2)
        torch.cuda.synchronize()
        assert q.device_status() == B.OK
        assert torch.equal(msg, msg2) and torch.equal(m_out.view(torch.int32), m_out2.view(torch.int32))
        want = [op.compress_diff(m_host[r], x, xhat[r], 3 + r, t) for r in range(R)]
        got_msg, got_m = msg.cpu().numpy(), m_out.cpu().numpy()
        for r in range(R):
            assert np.array_equal(got_msg[r], want[r]["msg"]), f"round {t} worker {r}: message differs"
            assert np.array_equal(P.bits(got_m[r]), P.bits(want[r]["m_out"])), f"round {t} worker {r}: memory differs"
        m_host = got_m


# ---------------------------------------------------------------------------------------------
# the counter of the random words at the far ends of its fields: round near 2^62, worker ids near
# 2^32, a 64-bit seed with the high bits set (Rand_k uses stream 0, the QSGD rounding stream 1)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d,k", [(9_001, 90), (300_007, 3_000)])
def test_random_word_counter_extremes(P, d, k):
    from paper_1906_02367_amd import binding as B
    seed = (1 << 64) - 59
    wl = custom(d, [0, d], [k], 5, W.RANDK, W.QSGD, R=2, seed=seed)
    op = P.oracle_for(wl)
    q = B.from_workload(wl)
    rng = np.random.default_rng(d)
    m_host = rng.standard_normal((2, d)).astype(f32)
    delta = rng.standard_normal((2, d)).astype(f32)
    for rnd, worker0 in [((1 << 62) - 1, (1 << 32) - 2), ((1 << 32) + 7, 0), ((1 << 61) + (1 << 31), 1 << 31)]:
        m_dev, d_dev = torch.from_numpy(m_host).to(q.device), torch.from_numpy(delta).to(q.device)
        msg = q.new_msg(2)
        q.compress(m_dev, d_dev, m_dev, worker0, rnd, msg)
        torch.cuda.synchronize()
        assert q.device_status() == B.OK
        got_msg, got_m = msg.cpu().numpy(), m_dev.cpu().numpy()
        for r in range(2):
            o = op.compress(m_host[r], delta[r], worker0 + r, rnd)
            assert np.array_equal(got_msg[r], o["msg"]), f"round {rnd} worker {worker0 + r}: message differs"
            assert np.array_equal(P.bits(got_m[r]), P.bits(o["m_out"])), f"round {rnd} worker {worker0 + r}: memory differs"
    with pytest.raises(B.QslError):
        q.compress(m_dev, d_dev, m_dev, 0, 1 << 62, msg)                  # round out of range
    with pytest.raises(B.QslError):
        q.compress(m_dev, d_dev, m_dev, (1 << 32) - 1, 0, msg)            # worker0 + R > 2^32


# ---------------------------------------------------------------------------------------------
# the paper's own per-tensor rule (Section 5.1.1): k_t = min(d_t, 1000) for every tensor -- whole small
# tensors, dense selections in the mid-sized ones, sparse ones in the large
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("quantizer,s", [(W.SIGN_L1, 1), (W.QSGD, 15), (W.SIGN_L3, 1), (W.SIGN_L4, 1)])
def test_per_tensor_rule_k_min_d_1000(P, quantizer, s):
    base = W.config(4, d=6_000_000, R=2)
    sizes = np.diff(base.seg_offset.astype(np.int64))
    k = np.minimum(sizes, 1000).astype(np.uint32)
    wl = W.Workload(4, "cfg4_k_min_d_1000", 2, base.d, base.seg_offset, k, s, W.TOPK, quantizer, 2, base.seed)
    run, op, m_host, paths = P.run_parity(wl, 2)
    assert set(paths[0].tolist()) == {0, 1, 3}, np.bincount(paths[0])


# ---------------------------------------------------------------------------------------------
# dense selections in many mid-sized segments: more multi-pass selection blocks than the GPU holds at once,
# so the blocks of one launch start at different times (a field of the unit state that one launch both read
# and rewrote once showed late blocks the new value here)
# ---------------------------------------------------------------------------------------------
def test_dense_k_in_many_segments_more_blocks_than_fit(P):
    rng = np.random.default_rng(5282)
    d, L, R = 3_328_894, 17, 3
    cuts = np.sort(rng.choice(np.arange(1, d), size=L - 1, replace=False))
    off = np.concatenate([[0], cuts, [d]]).astype(np.uint64)
    sizes = np.diff(off.astype(np.int64))
    k = np.maximum(1, (sizes * rng.uniform(0.05, 1.0, size=L)).astype(np.int64)).astype(np.uint32)
    wl = custom(d, off, k, 1, W.TOPK, W.SIGN_L1, R=R)
    deltas = [(rng.standard_normal((R, d)) * np.exp(2 * rng.standard_normal(d))).astype(f32) for _ in range(3)]
    run, op, m_host, paths = P.run_parity(wl, 3, deltas=deltas, worker0=55)
    assert (paths[0] == 1).sum() >= 30, np.bincount(paths[0])          # most of the 51 units take the multi-pass kernels


def test_side_stream_gives_the_same_bytes(P):
    # the library launches on whatever stream the caller hands it; two contexts on two streams at once
    from paper_1906_02367_amd import binding as B
    wl = W.config(2, d=1_000_003, R=2)
    d0 = torch.from_numpy(W.delta_all(wl, 0)).to("cuda")
    d1 = torch.from_numpy(W.delta_all(wl, 1)).to("cuda")
    qa, qb = B.from_workload(wl), B.from_workload(wl)
    ma, mb = torch.zeros(2, wl.d, device="cuda"), torch.zeros(2, wl.d, device="cuda")
    msga, msgb = qa.new_msg(2), qb.new_msg(2)
    xa, xb = torch.zeros(wl.d, device="cuda"), torch.zeros(wl.d, device="cuda")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    for t, dl in enumerate((d0, d1)):
        qa.compress(ma, dl, ma, 0, t, msga)
        qa.aggregate(msga, xa, -0.5, accumulate=True)
        with torch.cuda.stream(side):
            qb.compress(mb, dl, mb, 0, t, msgb)
            qb.aggregate(msgb, xb, -0.5, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(msga, msgb) and torch.equal(ma.view(torch.int32), mb.view(torch.int32))
    assert torch.equal(xa.view(torch.int32), xb.view(torch.int32))
    assert qa.device_status() == B.OK and qb.device_status() == B.OK


# ---------------------------------------------------------------------------------------------
# the guess carried from call to call: what happens when the next call's values do not look like the last one's
# ---------------------------------------------------------------------------------------------
def test_guess_from_the_previous_call_survives_a_change_of_the_inputs(P):
    """From the second call on a guessing unit takes its threshold guess from the previous call's candidates.  Inputs
    that collapse (v a thousandth of what it was: too few candidates), then grow a millionfold (too many), then
    settle: every round bit for bit the oracle's; the round of a jump runs through the failure path (reported as
    path 2), the round after it is back on the short one."""
    d, k, R = 1_000_003, 1000, 2
    rng = np.random.default_rng(77)
    for qz, s, flags in [(W.QSGD, 16, 0), (W.SIGN_L1, 1, 0), (W.QSGD, 16, 8)]:       # 8: a fresh sample every call
        wl = custom(d, [0, d], [k], s, W.TOPK, qz, R)
        op = P.oracle_for(wl)
        deltas = [rng.standard_normal((R, d)).astype(f32) for _ in range(2)]
        m = np.zeros((R, d), dtype=f32)
        for t in range(2):                                   # the memory after two rounds, from the oracle
            m = np.stack([o["m_out"] for o in P.oracle_round(op, m, deltas[t], t)])
        deltas.append((-m + 1e-3 * rng.standard_normal((R, d))).astype(f32))          # v collapses
        deltas += [(rng.standard_normal((R, d)) * sc).astype(f32) for sc in (1e-3, 1e3, 1e3, 1.0, 1.0)]
        run, op, m_host, paths = P.run_parity(wl, len(deltas), deltas=deltas, flags=flags)
        seen = [sorted(set(p.tolist())) for p in paths]
        print("paths per round:", seen)
        assert seen[0] == [0] and seen[1] == [0]
        if flags == 0:
            assert 2 in seen[2] and 2 in seen[4], seen            # the rounds of the two jumps take the failure path ...
            assert seen[3] == [0] and seen[5] == [0] and seen[7] == [0], seen     # ... and the next ones do not
        else:
            assert all(sset == [0] for sset in seen), seen        # a fresh sample never fails on these inputs


def test_ties_at_the_threshold_beyond_the_short_list(P):
    """Thousands of equal magnitudes exactly at the threshold: the threshold's histogram bin holds more candidates
    than the short list takes, so one block selects the unit from its dense candidate list (ties to the lower
    coordinate)."""
    d, k, R = 1_000_003, 4000, 2
    rng = np.random.default_rng(78)
    wl = custom(d, [0, d], [k], 16, W.TOPK, W.QSGD, R)
    deltas = []
    for t in range(3):
        x = (rng.standard_normal((R, d)) * 0.01).astype(f32)
        for r in range(R):
            big = rng.choice(d, 6000, replace=False)
            x[r, big[:3000]] = (10.0 + rng.random(3000)).astype(f32) * np.sign(rng.standard_normal(3000)).astype(f32)
            x[r, big[3000:]] = f32(5.0) * np.sign(rng.standard_normal(3000)).astype(f32)     # 3000 ties; 1000 of them are kept
        deltas.append(x)
    run, op, m_host, paths = P.run_parity(wl, 3, deltas=deltas)
    print("paths:", [p.tolist() for p in paths])


def test_guess_carried_over_layerwise_and_rand_k(P):
    # several rounds on the segmented and the Rand_k shapes: guesses of many units carried along
    wl = W.config(4, d=6_000_000, R=3)
    P.run_parity(wl, 5)
    wl = W.config(3, d=2_000_003, R=2)
    P.run_parity(wl, 4, expect_path=0)
    wl = W.config(5, d=8_000_003, R=2)
    P.run_parity(wl, 4, expect_path=0)


# ---------------------------------------------------------------------------------------------
# every coordinate kept, index-free messages (the error-feedback schemes without sparsification that Section 5
# compares with, as this operator): two streaming passes
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("sparsifier", [W.TOPK, W.RANDK])
@pytest.mark.parametrize("quantizer,s", [(W.QSGD, 15), (W.QSGD, 1), (W.QSGD, 256), (W.QSGD, 32768), (W.SIGN_L1, 1),
                                         (W.SIGN_L2, 1), (W.FP32, 1), (W.QSGD_SCALED, 3), (W.SIGN_L3, 1), (W.SIGN_L4, 1)])
def test_index_free_format(P, sparsifier, quantizer, s):
    from paper_1906_02367_amd import binding as B
    rng = np.random.default_rng(900 + s + quantizer)
    # one segment, ragged sizes around the 4096-coordinate tiles; many segments, tiny ones inside one tile included
    for d, off in [(1, [0, 1]), (4_095, [0, 4_095]), (300_001, [0, 300_001]),
                   (1_100_003, [0, 5, 70, 4_000, 4_097, 70_001, 400_000, 400_064, 1_100_003])]:
        k = np.diff(np.array(off, dtype=np.int64))
        wl = custom(d, off, k, s, sparsifier, quantizer, R=2)
        run, op, m_host, paths = P.run_parity(wl, 2, dense=True, expect_path=4, worker0=3)
        q = run.q
        msgs = run.msg.cpu().numpy()
        assert q.bits_sent(run.msg) == [op.bits_sent(msgs[r]) for r in range(wl.R)]
        w_code = 32 if quantizer == W.FP32 else 1 + (int(s).bit_length() if quantizer in (W.QSGD, W.QSGD_SCALED) else 0)
        assert q.bits_sent(run.msg)[0] == 32 + 32 * len(k) + d * w_code                    # the closed form
        # the master line and the stand-alone error update on such messages
        x0 = rng.standard_normal(d).astype(f32)
        out = torch.from_numpy(x0).to(q.device)
        q.aggregate(run.msg, out, -0.5, worker_list=[1, 0], accumulate=True)
        torch.cuda.synchronize()
        want = op.aggregate(msgs, -0.5, worker_list=[1, 0], out=x0)
        mag = sum(np.abs(op.decode(msgs[r])[1].astype(np.float64)) for r in (0, 1))
        assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - want) <= 1e-6 * (mag * 0.5 + np.abs(want)) + 1e-38)
        m0 = rng.standard_normal((2, d)).astype(f32)
        dl = rng.standard_normal((2, d)).astype(f32)
        m_dev, d_dev = torch.from_numpy(m0).to(q.device), torch.from_numpy(dl).to(q.device)
        m_fused, m_diff = torch.empty_like(m_dev), torch.empty_like(m_dev)
        msg2 = q.new_msg(2)
        q.compress(m_dev, d_dev, m_fused, 0, 7, run.msg)
        xx = torch.from_numpy(x0).to(q.device)
        q.compress_diff(m_dev, xx, xx.unsqueeze(0) - d_dev, m_diff, 0, 7, msg2)
        q.compress(m_dev, xx.unsqueeze(0) - (xx.unsqueeze(0) - d_dev), m_fused, 0, 7, run.msg)
        q.error_update(m_dev, xx.unsqueeze(0) - (xx.unsqueeze(0) - d_dev), run.msg)
        torch.cuda.synchronize()
        assert torch.equal(m_dev.view(torch.int32), m_fused.view(torch.int32))
        assert torch.equal(msg2, run.msg) and torch.equal(m_diff.view(torch.int32), m_fused.view(torch.int32))
        assert q.device_status() == B.OK
    # degenerate values
    d = 50_000
    wl = custom(d, [0, d], [d], s, sparsifier, quantizer, R=1)
    for name, v in _adversarial(d, rng):
        P.run_parity(wl, 1, deltas=[v[None, :].copy()], dense=True, expect_path=4)
    with pytest.raises(B.QslError):
        B.Qsl(100, [0, 100], [99], 16, B.TOPK, B.QSGD, 1, 1, flags=B.FLAG_DENSE_FORMAT)      # not every coordinate kept


# ---------------------------------------------------------------------------------------------
# the master line with many messages (from 12 on a kernel whose work is linear in the entries takes over)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["long_sign_layerwise", "short_qsgd", "rand_fp32"])
def test_aggregate_many_messages(P, case):
    from paper_1906_02367_amd import binding as B
    rng = np.random.default_rng(len(case))
    if case == "long_sign_layerwise":      # long messages, segments kept whole beside sparse ones (dense runs of entries)
        off = [0, 700, 1_724, 300_000, 301_000, 1_000_003]
        wl = custom(1_000_003, off, [700, 1_024, 9_000, 1_000, 3_000], 1, W.TOPK, W.SIGN_L1, R=8)
    elif case == "short_qsgd":
        wl = custom(300_007, [0, 300_007], [900], 16, W.TOPK, W.QSGD, R=8)
    else:
        wl = custom(70_001, [0, 64, 70_001], [64, 5_000], 1, W.RANDK, W.FP32, R=8)
    q = B.from_workload(wl)
    op = P.oracle_for(wl)
    msg = q.new_msg(64)
    m = torch.zeros(8, wl.d, device=q.device)
    for b in range(8):                                       # 64 messages, eight workers at a time
        delta = torch.from_numpy((rng.standard_normal((8, wl.d)) * np.exp(rng.standard_normal(wl.d))).astype(f32)).to(q.device)
        m.zero_()
        q.compress(m, delta, m, 8 * b, b, msg[8 * b: 8 * b + 8])
    torch.cuda.synchronize()
    msgs = msg.cpu().numpy()
    decoded = [op.decode(msgs[r]) for r in range(64)]
    x0 = rng.standard_normal(wl.d).astype(f32)
    for lst, accumulate in [(list(range(12)), True), ([int(x) for x in rng.permutation(64)[:33]], False), (list(range(63, -1, -1)), True)]:
        out = torch.from_numpy(x0).to(q.device)
        q.aggregate(msg, out, -1.0 / 64, worker_list=lst, accumulate=accumulate)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        # the library's own definition, written out: fp32 additions in list order, one rounding for the scale, one for the accumulate
        acc = np.zeros(wl.d, f32)
        has = np.zeros(wl.d, bool)
        for r in lst:
            i, v = decoded[r]
            acc[i] = np.where(has[i], acc[i] + v, v).astype(f32)
            has[i] = True
        term = (f32(-1.0 / 64) * acc).astype(f32)
        want = x0.copy() if accumulate else np.zeros(wl.d, f32)
        want[has] = (want[has] + term[has]).astype(f32) if accumulate else term[has]
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (case, len(lst))
        # and the oracle's double sum within the tolerance of the aggregate
        ref = op.aggregate(msgs, -1.0 / 64, worker_list=lst, out=x0 if accumulate else None)
        mag = np.zeros(wl.d)
        for r in lst:
            i, v = decoded[r]
            mag[i] += np.abs(v.astype(np.float64))
        assert np.all(np.abs(got.astype(np.float64) - ref) <= 1e-6 * (mag / 64 + np.abs(ref)) + 1e-38)
    assert q.device_status() == B.OK


# ---------------------------------------------------------------------------------------------
# the master line on long messages whose coordinates are shared by all, by about half or by hardly any of the listed
# messages, call after call on one context, with lists that change
# ---------------------------------------------------------------------------------------------
def _aggregate_by_definition(decoded, lst, scale, x0, accumulate, d):
    acc = np.zeros(d, f32)
    has = np.zeros(d, bool)
    for r in lst:
        i, v = decoded[r]
        acc[i] = np.where(has[i], acc[i] + v, v).astype(f32)
        has[i] = True
    term = (f32(scale) * acc).astype(f32)
    want = x0.copy() if accumulate else np.zeros(d, f32)
    want[has] = (want[has] + term[has]).astype(f32) if accumulate else term[has]
    return want


@pytest.mark.parametrize("case", ["sign_layerwise", "qsgd_layerwise", "sign_one_segment"])
def test_aggregate_long_messages_shared_coordinates(P, case):
    from paper_1906_02367_amd import binding as B
    rng = np.random.default_rng(77 + len(case))
    if case == "sign_layerwise":           # segments kept whole (at the same places in every message) beside sparse ones
        off = [0, 700, 1_724, 300_000, 301_000, 1_000_003]
        wl = custom(1_000_003, off, [700, 1_024, 9_000, 1_000, 3_000], 1, W.TOPK, W.SIGN_L1, R=8)
    elif case == "qsgd_layerwise":         # entries drop out: no two messages alike, whole segments included
        off = [0, 700, 1_724, 300_000, 301_000, 1_000_003]
        wl = custom(1_000_003, off, [700, 1_024, 9_000, 1_000, 3_000], 4, W.TOPK, W.QSGD, R=8)
    else:
        wl = custom(2_000_003, [0, 2_000_003], [20_000], 1, W.TOPK, W.SIGN_L1, R=8)
    q = B.from_workload(wl)
    op = P.oracle_for(wl)
    msg = q.new_msg(8)
    # what the workers share decides how many coordinates several messages hold: all, about half, hardly any
    common = (rng.standard_normal(wl.d) * np.exp(rng.standard_normal(wl.d))).astype(f32)
    for share in (1.0, 0.5, 0.0):
        own = (rng.standard_normal((8, wl.d)) * np.exp(rng.standard_normal(wl.d))).astype(f32)
        delta = torch.from_numpy((f32(share) * common[None, :] + f32(1.0 - share) * own).astype(f32)).to(q.device)
        m = torch.zeros(8, wl.d, device=q.device)
        q.compress(m, delta, m, 0, int(share * 10), msg)
        torch.cuda.synchronize()
        msgs = msg.cpu().numpy()
        decoded = [op.decode(msgs[r]) for r in range(8)]
        if share == 0.5:
            both = len(np.intersect1d(decoded[0][0], decoded[1][0]))
            assert 0 < both < len(decoded[0][0])
        x0 = rng.standard_normal(wl.d).astype(f32)
        for lst, accumulate in [(list(range(8)), True), ([5, 2], False), ([7, 0, 3, 6, 1], True), ([4], True),
                                (list(range(7, -1, -1)), False), ([1, 2, 3], True)]:
            out = torch.from_numpy(x0).to(q.device)
            q.aggregate(msg, out, -0.125, worker_list=lst, accumulate=accumulate)
            torch.cuda.synchronize()
            want = _aggregate_by_definition(decoded, lst, -0.125, x0, accumulate, wl.d)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32)), (case, share, lst)
    # a message cut short (here: empty) among full ones: its coordinates are not at the places the others have them
    cut = msg.clone()
    cut[3].zero_()
    torch.cuda.synchronize()
    msgs = cut.cpu().numpy()
    decoded = [op.decode(msgs[r]) if r != 3 else (np.zeros(0, np.int64), np.zeros(0, f32)) for r in range(8)]
    for lst in ([3, 0, 1], [0, 1, 3, 2], list(range(8))):
        out = torch.from_numpy(x0).to(q.device)
        q.aggregate(cut, out, 0.5, worker_list=lst, accumulate=True)
        torch.cuda.synchronize()
        want = _aggregate_by_definition(decoded, lst, 0.5, x0, True, wl.d)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32)), (case, "cut", lst)
    # ... and full lists again afterwards
    msgs = msg.cpu().numpy()
    decoded = [op.decode(msgs[r]) for r in range(8)]
    out = torch.from_numpy(x0).to(q.device)
    q.aggregate(msg, out, 1.0, accumulate=False)
    torch.cuda.synchronize()
    want = _aggregate_by_definition(decoded, list(range(8)), 1.0, x0, False, wl.d)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert q.device_status() == B.OK
