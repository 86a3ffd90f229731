"""GPU checks of how a context behaves around the operator itself: stopping and resuming a run from the saved
error memory, a change of stream between two calls, and messages without touching the error memory."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_1906_02367_amd import workloads as W  # noqa: E402


@pytest.fixture(scope="module")
def P():
    import parity_util
    return parity_util


@pytest.mark.parametrize("cfg,d", [(2, 1_000_003), (3, 600_011), (4, 2_000_000)])
def test_resume_from_saved_memory_equals_straight_run(P, cfg, d):
    """The state of the hot path is the error memory and the round counter (the randomness is counter-based):
    10 rounds, the memory copied out and into a fresh context, 10 more -- the same bytes as 20 rounds straight."""
    from paper_1906_02367_amd import binding as B
    wl = W.config(cfg, d=d, R=2)
    dev = torch.device("cuda")
    deltas = [torch.from_numpy(W.delta_all(wl, t)).to(dev) for t in range(20)]

    def run(q, m, x, t0, t1, keep):
        msg = q.new_msg(wl.R)
        for t in range(t0, t1):
            q.compress(m, deltas[t], m, 0, t, msg)
            q.aggregate(msg, x, -1.0 / wl.R, accumulate=True)
            keep.append((msg.clone(), x.clone()))
        torch.cuda.synchronize()
        assert q.device_status() == B.OK

    straight, resumed = [], []
    m_a, x_a = torch.zeros(wl.R, wl.d, device=dev), torch.zeros(wl.d, device=dev)
    run(B.from_workload(wl), m_a, x_a, 0, 20, straight)
    q1 = B.from_workload(wl)
    m_b, x_b = torch.zeros(wl.R, wl.d, device=dev), torch.zeros(wl.d, device=dev)
    run(q1, m_b, x_b, 0, 10, resumed)
    saved_m, saved_x = m_b.cpu().numpy().copy(), x_b.cpu().numpy().copy()     # "checkpoint": the state leaves the device ...
    q1.close()
    del q1, m_b, x_b
    m_c, x_c = torch.from_numpy(saved_m).to(dev), torch.from_numpy(saved_x).to(dev)   # ... and comes back into a fresh context
    run(B.from_workload(wl), m_c, x_c, 10, 20, resumed)
    assert torch.equal(m_a.view(torch.int32), m_c.view(torch.int32))
    for t in range(20):
        assert torch.equal(straight[t][0], resumed[t][0]), f"round {t}: messages differ"
        assert torch.equal(straight[t][1].view(torch.int32), resumed[t][1].view(torch.int32)), f"round {t}: x differs"


def test_calls_on_different_streams_are_ordered(P):
    """compress on stream A, aggregate (and the next compress) on stream B, same context: the library makes the new
    stream wait for the work on the old one, so the bytes equal those of a single-stream run."""
    from paper_1906_02367_amd import binding as B
    wl = W.config(2, d=4_000_037, R=4)
    dev = torch.device("cuda")
    deltas = [torch.from_numpy(W.delta_all(wl, t)).to(dev) for t in range(3)]
    torch.cuda.synchronize()

    def run(streams):
        q = B.from_workload(wl)
        m = torch.zeros(wl.R, wl.d, device=dev)
        msg = q.new_msg(wl.R)
        x = torch.zeros(wl.d, device=dev)
        outs = []
        torch.cuda.synchronize()
        for t in range(3):
            with torch.cuda.stream(streams[(2 * t) % len(streams)]):
                q.compress(m, deltas[t], m, 0, t, msg)
            with torch.cuda.stream(streams[(2 * t + 1) % len(streams)]):
                q.aggregate(msg, x, -0.25, accumulate=True)
                outs.append((msg.clone(), x.clone()))
        torch.cuda.synchronize()
        assert q.device_status() == B.OK
        return m, outs

    one = torch.cuda.current_stream()
    m1, o1 = run([one])
    m2, o2 = run([torch.cuda.Stream(), torch.cuda.Stream()])
    assert torch.equal(m1.view(torch.int32), m2.view(torch.int32))
    for (a, xa), (b, xb) in zip(o1, o2):
        assert torch.equal(a, b) and torch.equal(xa.view(torch.int32), xb.view(torch.int32))


@pytest.mark.parametrize("cfg,d", [(2, 1_000_003), (1, 65_536), (4, 2_000_000)])
def test_messages_without_touching_the_memory(P, cfg, d):
    """m_out = NULL on a context that owns a home for v: the same messages, m unchanged; the stand-alone error
    update then gives the memory of the fused form."""
    from paper_1906_02367_amd import binding as B
    wl = W.config(cfg, d=d, R=2)
    dev = torch.device("cuda")
    q = B.from_workload(wl, flags=B.FLAG_OWN_V)
    q_plain = B.from_workload(wl)
    rng = np.random.default_rng(cfg)
    m0 = (0.3 * rng.standard_normal((wl.R, wl.d))).astype(np.float32)
    delta = torch.from_numpy(W.delta_all(wl, 0)).to(dev)
    m = torch.from_numpy(m0).to(dev)
    msg, msg2 = q.new_msg(wl.R), q_plain.new_msg(wl.R)
    q.compress(m, delta, None, 0, 3, msg)
    m_fused = torch.empty_like(m)
    q_plain.compress(m, delta, m_fused, 0, 3, msg2)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m0.view(np.uint32))          # untouched
    assert torch.equal(msg, msg2)
    q.error_update(m, delta, msg)
    torch.cuda.synchronize()
    assert torch.equal(m.view(torch.int32), m_fused.view(torch.int32))
    with pytest.raises(B.QslError):
        q_plain.compress(m, delta, None, 0, 3, msg2)                                    # no home for v: refused
    assert q.device_status() == B.OK


@pytest.mark.parametrize("cfg,d", [(2, 1_000_003), (3, 600_011), (4, 2_000_000), (6, None)])
def test_same_bytes_whatever_the_launch_shape(P, cfg, d):
    """The operator is applied to each worker's vector on its own (Algorithm 1, worker lines), so how many workers
    one call carries may not show in the result: 6 workers in one call, the same 6 in a context made for 9, and one
    worker per call in a context made for one (other grids, other kernel instances) -- the same bytes, 3 rounds."""
    from paper_1906_02367_amd import binding as B
    wl = W.config(cfg, d=d, R=6)
    dev = torch.device("cuda")
    deltas = [torch.from_numpy(W.delta_all(wl, t)).to(dev) for t in range(3)]
    q6, q9 = B.from_workload(wl), B.from_workload(wl, max_workers=9)
    q1 = [B.from_workload(wl, max_workers=1) for _ in range(wl.R)]      # a context per worker: each carries its own guess
    m6, m9, m1 = (torch.zeros(wl.R, wl.d, device=dev) for _ in range(3))
    for t in range(3):
        msg6, msg9, msg1 = q6.new_msg(wl.R), q9.new_msg(wl.R), q6.new_msg(wl.R)
        q6.compress(m6, deltas[t], m6, 0, t, msg6)
        q9.compress(m9, deltas[t], m9, 0, t, msg9)
        for r in range(wl.R):
            q1[r].compress(m1[r:r + 1], deltas[t][r:r + 1], m1[r:r + 1], r, t, msg1[r:r + 1])
        torch.cuda.synchronize()
        assert torch.equal(msg6, msg9) and torch.equal(msg6, msg1), f"round {t}: messages differ"
        assert torch.equal(m6.view(torch.int32), m9.view(torch.int32)), f"round {t}: memory differs (9-worker context)"
        assert torch.equal(m6.view(torch.int32), m1.view(torch.int32)), f"round {t}: memory differs (one worker per call)"
