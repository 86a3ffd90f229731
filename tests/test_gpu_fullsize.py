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
