"""The master line for callers that cannot allocate (qsl_aggregate_static): through the C ABI, against
qsl_aggregate on a context, on two calls in a row, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_1906_02367_amd import workloads as W  # noqa: E402


def _messages(B, d, k, s, sparsifier, quantizer, R, seed):
    wl = W.Workload(2, "static", R, d, np.array([0, d], dtype=np.uint64), np.array([k], dtype=np.uint32), s, sparsifier,
                    quantizer, 1, seed)
    q = B.from_workload(wl)
    rng = np.random.default_rng(seed)
    delta = torch.from_numpy((rng.standard_normal((R, d)) * np.exp(rng.standard_normal(d))).astype(np.float32)).to(q.device)
    m = torch.zeros(R, d, device=q.device)
    msg = q.new_msg(R)
    q.compress(m, delta, m, 0, 0, msg)
    torch.cuda.synchronize()
    return wl, q, msg


def test_static_aggregate_matches_the_context_entry_point():
    from paper_1906_02367_amd import binding as B
    from oracle import oracle as O
    # first call: long messages (directories in the static array); second: a smaller operator with short messages;
    # third: every coordinate kept (the dense pass)
    cases = [(1_000_003, 8_000, 1, W.TOPK, W.SIGN_L1, 5, [3, 0, 4, 1]),
             (70_001, 700, 16, W.TOPK, W.QSGD, 3, None),
             (20_003, 20_003, 1, W.RANDK, W.SIGN_L2, 2, None)]
    for d, k, s, sp, qz, R, lst in cases:
        wl, q, msg = _messages(B, d, k, s, sp, qz, R, seed=d)
        x0 = np.random.default_rng(1).standard_normal(d).astype(np.float32)
        for accumulate in (False, True):
            want = torch.from_numpy(x0).to(q.device)
            got = torch.from_numpy(x0).to(q.device)
            q.aggregate(msg, want, -1.0 / R, worker_list=lst, accumulate=accumulate)
            B.aggregate_static(d, k, s, sp, qz, msg, got, -1.0 / R, worker_list=lst, accumulate=accumulate)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (d, k, accumulate)
        # and against the oracle's dense sum, at the tolerance of the aggregate
        op = O.OracleOp(d, wl.seg_offset, wl.seg_k, s, sp, qz, wl.seed)
        msgs = msg.cpu().numpy()
        ref = op.aggregate(msgs, -1.0 / R, worker_list=lst, out=x0)
        mag = np.zeros(d)
        for r in (lst if lst is not None else range(R)):
            i, v = op.decode(msgs[r])
            mag[i] += np.abs(v.astype(np.float64))
        assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - ref) <= 1e-6 * (mag / R + np.abs(ref)) + 1e-38)
        assert q.device_status() == B.OK


def test_static_aggregate_refuses_what_does_not_fit():
    from paper_1906_02367_amd import binding as B
    dev = torch.device("cuda")
    out = torch.zeros(16, device=dev)
    msg = torch.zeros(2, 64, dtype=torch.uint8, device=dev)
    lib = B._lib
    off2 = (C.c_uint64 * 3)(0, 8, 16)
    k2 = (C.c_uint32 * 2)(1, 1)
    cfg = B._Config(16, 2, off2, k2, 1, 0, 1, 0, 1, 0)                    # two segments
    stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    assert lib.qsl_aggregate_static(C.byref(cfg), stream, msg.data_ptr(), None, 2, 1.0, 0, out.data_ptr()) == B.ERR_UNSUPPORTED
    d = (1 << 32) - 1                                                        # 65 directories of 4 M words: beyond the array
    off1 = (C.c_uint64 * 2)(0, d)
    k1 = (C.c_uint32 * 1)(100_000)
    cfg = B._Config(d, 1, off1, k1, 1, 0, 1, 0, 1, 0)
    assert lib.qsl_aggregate_static(C.byref(cfg), stream, msg.data_ptr(), None, 64, 1.0, 1, out.data_ptr()) == B.ERR_UNSUPPORTED
    assert lib.qsl_aggregate_static(C.byref(cfg), stream, msg.data_ptr(), None, 65, 1.0, 1, out.data_ptr()) == B.ERR_INVALID_ARG
    assert lib.qsl_aggregate_static(None, stream, msg.data_ptr(), None, 2, 1.0, 1, out.data_ptr()) == B.ERR_INVALID_ARG
