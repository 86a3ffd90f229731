"""Qsparse-local-SGD end to end on a synthetic convex problem, around the C-ABI hot path.

A harness, not part of the hot path: the local SGD steps (Algorithm 1, first worker line) are plain
torch; every synchronisation goes through `qsl_compress` (worker lines of a sync step) and
`qsl_aggregate` (master line) of the library.  The problem is shaped like the paper's convex
experiment (Section 5.2: softmax regression with l2 regularisation, d = 7,850, R = 15 workers,
mini-batch 8, k = 40, learning rate xi / (a + t) with a = d H / k) on a seeded Gaussian mixture that
stands in for MNIST.

`run_sync` is Algorithm 1 (all workers synchronise every H steps); `run_async` is Algorithm 2 (each
worker draws its next interval uniformly from {1..H}; the master adds the messages of the workers
that report, still scaled by 1/R, and sends the model back to those workers only).  Both also track
the virtual sequence of Section 3.4, so that the memory identity  xhat_t - xtilde_t = (1/R) sum_r m_t
can be checked along the run.

    python -m paper_1906_02367_amd.algorithm1        # loss against bits for a few operators
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

from . import binding as B

N_FEATURES, N_CLASSES = 784, 10
D = (N_FEATURES + 1) * N_CLASSES          # 7,850 parameters, as in the paper's convex runs


class SoftmaxProblem:
    """l2-regularised softmax regression on a seeded Gaussian mixture, sharded over R workers."""

    def __init__(self, R=15, n_per_worker=400, seed=0, device="cuda"):
        g = torch.Generator(device="cpu").manual_seed(1906_02367 + seed)
        self.device = torch.device(device)
        self.R, self.n = R, R * n_per_worker
        means = 0.35 * torch.randn(N_CLASSES, N_FEATURES, generator=g)
        y = torch.randint(0, N_CLASSES, (self.n,), generator=g)
        x = means[y] + torch.randn(self.n, N_FEATURES, generator=g)
        x = torch.cat([x, torch.ones(self.n, 1)], dim=1) / math.sqrt(N_FEATURES)
        self.x = x.to(self.device).view(R, n_per_worker, N_FEATURES + 1)        # worker r owns shard r
        self.y = y.to(self.device).view(R, n_per_worker)
        self.lam = 1.0 / self.n
        self.gen = torch.Generator(device=self.device).manual_seed(7 + seed)

    def loss(self, w):
        logits = self.x.reshape(self.n, -1) @ w.view(N_CLASSES, -1).t()
        ce = torch.nn.functional.cross_entropy(logits, self.y.reshape(-1))
        return float(ce + 0.5 * self.lam * (w.double() ** 2).sum())

    def minibatch_grads(self, w_local, b):
        """w_local: [R, D] local parameters; returns the R stochastic gradients [R, D] (one mini-batch each)."""
        R = self.R
        idx = torch.randint(0, self.x.shape[1], (R, b), generator=self.gen, device=self.device)
        xb = torch.gather(self.x, 1, idx.unsqueeze(-1).expand(R, b, N_FEATURES + 1))       # [R, b, F+1]
        yb = torch.gather(self.y, 1, idx)                                                    # [R, b]
        W = w_local.view(R, N_CLASSES, N_FEATURES + 1)
        logits = torch.bmm(xb, W.transpose(1, 2))                                            # [R, b, C]
        p = torch.softmax(logits, dim=2)
        p.scatter_add_(2, yb.unsqueeze(-1), -torch.ones(R, b, 1, device=self.device))
        g = torch.bmm(p.transpose(1, 2), xb) / b                                             # [R, C, F+1]
        return g.reshape(R, D) + self.lam * w_local


@dataclasses.dataclass
class Operator:
    k: int = 40
    s: int = 15                       # 4-bit QSGD of the paper: s = 2^4 - 1
    sparsifier: int = B.TOPK
    quantizer: int = B.QSGD
    seed: int = 1

    def make(self, max_workers, device):
        return B.Qsl(D, [0, D], [self.k], self.s, self.sparsifier, self.quantizer, self.seed, max_workers, device=device)


def _lr(t, H, k, xi):
    return xi / (D * H / k + t)


def run_sync(problem, op: Operator, H=4, T=400, b=8, xi=None, on_sync=None):
    """Algorithm 1.  Returns dict(loss, bits, x, m, identity_err).  `on_sync(t, m_before, delta, msg, m_after,
    x_before, x_after)` is called with device tensors at every synchronisation (the tests hang the oracle there)."""
    dev, R = problem.device, problem.R
    q = op.make(R, dev)
    xi = xi if xi is not None else 0.5 * D * H / op.k
    x = torch.zeros(D, device=dev)                       # the master's model
    xh = torch.zeros(R, D, device=dev)                   # local models xhat^(r)
    m = torch.zeros(R, D, device=dev)                    # error memories
    xt = torch.zeros(D, dtype=torch.float64, device=dev) # virtual sequence (average over workers)
    msg = q.new_msg(R)
    losses, bits, ident, total_bits = [], [], [], 0
    for t in range(T):
        eta = _lr(t, H, op.k, xi)
        g = problem.minibatch_grads(xh, b)
        xh_half = xh - eta * g
        xt -= eta * g.double().mean(0)
        if (t + 1) % H == 0:
            m_before, x_before = (m.clone(), x.clone()) if on_sync else (None, None)
            delta = x.unsqueeze(0) - xh_half if on_sync else None       # only for the observer
            q.compress_diff(m, x, xh_half, m, 0, t, msg)                # g = Q Comp_k(m + x - xhat_half), m updated
            q.aggregate(msg, x, -1.0 / R, accumulate=True)          # x <- x - (1/R) sum_r g^(r)
            total_bits += sum(q.bits_sent(msg))
            if on_sync:
                on_sync(t, m_before, delta, msg, m, x_before, x)
            xh = x.unsqueeze(0).expand(R, D).clone()
        else:
            xh = xh_half
        if (t + 1) % H == 0 or t == T - 1:
            losses.append(problem.loss(x)); bits.append(total_bits)
            lhs = xh.double().mean(0) - xt
            rhs = m.double().mean(0)
            ident.append(float((lhs - rhs).norm() / (rhs.norm() + lhs.norm() + 1e-30)))
    return dict(loss=losses, bits=bits, x=x, m=m, identity_err=max(ident), q=q)


def run_async(problem, op: Operator, H=4, T=400, b=8, xi=None, seed=0, on_sync=None):
    """Algorithm 2: per-worker synchronisation times, subset aggregation scaled by 1/R.
    `on_sync(t, S, m_before, delta, msg, m_after, x_before, x_after)` as in `run_sync`, with the reporting set S."""
    dev, R = problem.device, problem.R
    q = op.make(R, dev)                                  # the master's context (aggregation, bit counts)
    qw = [op.make(1, dev) for _ in range(R)]             # one per worker: each keeps its own worker's threshold guess
    xi = xi if xi is not None else 0.5 * D * H / op.k
    rng = np.random.default_rng(seed)
    next_sync = rng.integers(1, H + 1, size=R)           # worker r synchronises when t + 1 == next_sync[r]
    x = torch.zeros(D, device=dev)
    xr = torch.zeros(R, D, device=dev)                   # the model each worker last received, x^(r)
    xh = torch.zeros(R, D, device=dev)
    m = torch.zeros(R, D, device=dev)
    msg = q.new_msg(R).zero_()                           # rows of workers that have not reported yet read as empty
    losses, bits, total_bits, max_m = [], [], 0, 0.0
    for t in range(T):
        eta = _lr(t, H, op.k, xi)
        xh = xh - eta * problem.minibatch_grads(xh, b)
        S = [r for r in range(R) if next_sync[r] == t + 1]
        if S:
            delta = xr - xh                              # x^(r) - xhat^(r)_{t+1/2}; only the rows in S are used
            m_before, x_before = (m.clone(), x.clone()) if on_sync else (None, None)
            for r in S:                                  # the reporting workers compress, each with its own id
                qw[r].compress(m[r:r + 1], delta[r:r + 1], m[r:r + 1], r, t, msg[r:r + 1])
            q.aggregate(msg, x, -1.0 / R, worker_list=S, accumulate=True)
            total_bits += sum(q.bits_sent(msg)[r] for r in S)
            if on_sync:
                on_sync(t, S, m_before, delta, msg, m, x_before, x)
            for r in S:
                xr[r] = x; xh[r] = x
                next_sync[r] = t + 1 + rng.integers(1, H + 1)
            losses.append(problem.loss(x)); bits.append(total_bits)
            max_m = max(max_m, float(m.norm(dim=1).max()))
    return dict(loss=losses, bits=bits, x=x, m=m, max_memory_norm=max_m, q=q)


def main():
    torch.manual_seed(0)
    prob = SoftmaxProblem()
    print(f"softmax regression, d = {D}, R = {prob.R}, n = {prob.n}; initial loss {prob.loss(torch.zeros(D, device=prob.device)):.4f}")
    rows = [("Top_k fp32 (TopK-SGD), H=1", Operator(quantizer=B.FP32), 1),
            ("SignTop_k, H=1", Operator(quantizer=B.SIGN_L1), 1),
            ("4-bit QTop_k, H=1", Operator(quantizer=B.QSGD, s=15), 1),
            ("scaled 2-bit QTop_k, H=4", Operator(quantizer=B.QSGD_SCALED, s=3), 4),
            ("SignTop_k, H=4", Operator(quantizer=B.SIGN_L1), 4),
            ("SignTop_k, H=8", Operator(quantizer=B.SIGN_L1), 8)]
    print(f"{'scheme':34s} {'final loss':>10s} {'log2(bits)':>11s} {'identity err':>13s}")
    for name, op, H in rows:
        res = run_sync(prob, op, H=H, T=800)
        print(f"{name:34s} {res['loss'][-1]:10.4f} {math.log2(res['bits'][-1]):11.2f} {res['identity_err']:13.2e}")
    res = run_async(prob, Operator(quantizer=B.SIGN_L1), H=4, T=800)
    print(f"{'SignTop_k, asynchronous, H<=4':34s} {res['loss'][-1]:10.4f} {math.log2(res['bits'][-1]):11.2f} {'':>13s}")


if __name__ == "__main__":
    main()
