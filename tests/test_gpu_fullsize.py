"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: every
output of every worker compared with the oracle, bit for bit, on device-generated seeded inputs."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_1906_02367_amd import workloads as W  # noqa: E402


@pytest.fixture(scope="module")
def P():
    import parity_util
    return parity_util


@pytest.mark.parametrize("cfg,rounds", [(2, 20), (3, 20), (4, 20), (5, 5), (6, 5), (7, 3), (8, 3)])
def test_full_size_config(P, cfg, rounds):
    wl = W.config(cfg)
    print(f"\n[{wl.name}] R={wl.R} d={wl.d} K={wl.K} L={wl.L}", flush=True)
    run, op, m_host, paths = P.run_parity(wl, rounds, host_deltas=False, dense=wl.dense)
    if cfg in (2, 3, 5):
        assert all((p == 0).all() for p in paths), "the benchmark sizes must run on the single-pass path"
    # master line on the last round's messages
    import torch
    q = run.q
    out = torch.empty(wl.d, dtype=torch.float32, device=q.device)
    q.aggregate(run.msg, out, 1.0 / wl.R)
    torch.cuda.synchronize()
    msgs = run.msg.cpu().numpy()
    want = op.aggregate(msgs, 1.0 / wl.R)
    dense_abs = np.zeros(wl.d)
    for r in range(wl.R):
        i, v = op.decode(msgs[r])
        dense_abs[i] += np.abs(v.astype(np.float64))
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= 1e-6 * dense_abs / wl.R + 1e-38)
    assert q.bits_sent(run.msg) == [op.bits_sent(msgs[r]) for r in range(wl.R)]


@pytest.mark.parametrize("quantizer,s", [(W.QSGD, 15), (W.SIGN_L2, 1)])
def test_index_free_rows_longer_than_the_first_pass_has_blocks(P, quantizer, s):
    """Rows of more than 16384 tiles of 4096 coordinates: a block of the first pass then takes several tiles, and what it
    meets beyond its first unit goes to that unit's counters directly -- three units whose ends lie inside tiles."""
    d = 70_000_003
    off = np.array([0, 33_000_001, 33_002_000, d], dtype=np.uint64)
    k = np.diff(off.astype(np.int64)).astype(np.uint32)
    wl = W.Workload(2, "long_rows_index_free", 1, d, off, k, s, W.TOPK, quantizer, 1, 4321)
    print(f"\n[{wl.name}] R={wl.R} d={wl.d} L={wl.L}", flush=True)
    run, op, m_host, paths = P.run_parity(wl, 2, host_deltas=False, dense=True, expect_path=4)
    msgs = run.msg.cpu().numpy()
    assert run.q.bits_sent(run.msg) == [op.bits_sent(msgs[0])]


@pytest.mark.parametrize("cfg,R", [(4, 1), (6, 2), (6, 1)])
def test_per_tensor_configurations_with_few_workers(P, cfg, R):
    """With few workers the block budget gives the large tensors several blocks: the guessing units then take both
    k_lean_one and the three kernels, side by side on streams of the context's own (and beside k_block_units)."""
    wl = W.config(cfg, R=R)
    print(f"\n[{wl.name}] R={wl.R} d={wl.d} K={wl.K} L={wl.L}", flush=True)
    run, op, m_host, paths = P.run_parity(wl, 4, host_deltas=False)
    assert all((p != 2).all() for p in paths)                       # no guess failed
    msgs = run.msg.cpu().numpy()
    assert run.q.bits_sent(run.msg) == [op.bits_sent(msgs[r]) for r in range(wl.R)]
