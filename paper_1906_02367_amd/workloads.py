"""Seeded synthetic workloads: operator parameters and update vectors.

This module holds *no arithmetic of the method* -- only the parameters of the five
benchmark configurations and the generators of their input vectors (the accumulated
local updates Delta that Algorithm 1 feeds to the compression step).  It is the one
module that both the GPU tests/benchmark and the CPU oracle's tests may import.

The vectors stand in for the ResNet-50 update vectors of Section 5.1 of the paper
(d ~ 25.6 M parameters in ~160 tensors, R = 8 workers, k ~ 0.1-1 % of d), which need a
dataset and a training run: heavy-tailed per-coordinate scales, a component shared by
all workers plus independent per-worker noise, and a segment table with tensor sizes
spread log-uniformly over four orders of magnitude.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

BASE_SEED = 190602367
TOPK, RANDK = 0, 1
QSGD, SIGN_L1, SIGN_L2, FP32, QSGD_SCALED, SIGN_L3, SIGN_L4 = 0, 1, 2, 3, 4, 5, 6
RESNET50_D = 25_557_032


@dataclasses.dataclass
class Workload:
    cfg: int                 # 1..5, which benchmark configuration's input distribution this uses
    name: str
    R: int                   # simulated workers
    d: int                   # coordinates per worker
    seg_offset: np.ndarray   # uint64 [L+1]
    seg_k: np.ndarray        # uint32 [L]
    s: int                   # QSGD levels (ignored by the sign quantiser)
    sparsifier: int
    quantizer: int
    rounds: int
    seed: int = BASE_SEED    # seed handed to the operator (Rand_k / QSGD randomness)
    dense: bool = False      # every coordinate kept and index-free messages (the comparison schemes without sparsification)

    @property
    def L(self) -> int:
        return int(self.seg_k.size)

    @property
    def K(self) -> int:
        return int(self.seg_k.sum())


def _rng(cfg, stream, worker=0, rnd=0):
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([BASE_SEED, cfg, stream, worker, rnd])))


def _one_segment(d, k):
    return np.array([0, d], dtype=np.uint64), np.array([k], dtype=np.uint32)


def segment_table(d: int, n_seg: int = 160, lo: float = 64.0, hi: float = 2.4e6, cfg: int = 4):
    """n_seg sizes drawn log-uniform in [lo, hi], rescaled to sum to d (largest remainder, minimum 64)."""
    u = _rng(cfg, 3).uniform(math.log(lo), math.log(hi), size=n_seg)
    raw = np.exp(u)
    min_size = min(64, d // n_seg)
    spare = d - min_size * n_seg
    share = raw / raw.sum() * spare
    sizes = np.floor(share).astype(np.int64)
    rem = spare - int(sizes.sum())
    order = np.argsort(-(share - sizes), kind="stable")
    sizes[order[:rem]] += 1
    sizes += min_size
    assert int(sizes.sum()) == d and sizes.min() >= 1
    off = np.zeros(n_seg + 1, dtype=np.uint64)
    off[1:] = np.cumsum(sizes).astype(np.uint64)
    k = ((sizes + 999) // 1000).astype(np.uint32)      # k_l = ceil(0.001 * size_l)
    return off, k


def resnet50_tensor_sizes() -> list:
    """Sizes of the 161 trainable tensors of ResNet-50 (He et al., 2016; bottleneck blocks 3-4-6-3, 1000
    classes), in layer order: the segment table the paper's ResNet-50 runs compress tensor by tensor
    (Section 5.1.1).  They add up to 25,557,032, and the paper's rule k_t = min(d_t, 1000) gives 99,400
    on them -- the total k that Section 5.1.1 prints."""
    sizes = [64 * 3 * 7 * 7, 64, 64]                                 # stem convolution, its batch-norm scale and shift
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            sizes += [planes * inplanes, planes, planes,             # 1x1 convolution + batch norm
                      planes * planes * 9, planes, planes,           # 3x3
                      4 * planes * planes, 4 * planes, 4 * planes]   # 1x1, widening
            if b == 0:                                               # projection shortcut of the stage's first block
                sizes += [4 * planes * inplanes, 4 * planes, 4 * planes]
            inplanes = 4 * planes
    sizes += [2048 * 1000, 1000]                                     # classifier weight and bias
    return sizes


def config(cfg: int, d: int | None = None, R: int | None = None, rounds: int | None = None) -> Workload:
    """Benchmark configuration `cfg` (1..5; 6 = the paper's own per-tensor rule on ResNet-50's tensor table).
    `d`, `R`, `rounds` shrink it for quick tests; k scales with d."""
    if cfg == 1:
        d0, R0, T0 = 65_536, 2, 10
        dd = d or d0
        off, k = _one_segment(dd, max(1, round(dd * 655 / d0)))
        wl = Workload(1, "cfg1_top1pct_sign", R or R0, dd, off, k, 1, TOPK, SIGN_L1, rounds or T0)
    elif cfg == 2:
        d0, R0, T0 = RESNET50_D, 8, 20
        dd = d or d0
        off, k = _one_segment(dd, max(1, round(dd * 25_557 / d0)))
        wl = Workload(2, "cfg2_top0.1pct_qsgd16", R or R0, dd, off, k, 16, TOPK, QSGD, rounds or T0)
    elif cfg == 3:
        d0, R0, T0 = RESNET50_D, 8, 20
        dd = d or d0
        off, k = _one_segment(dd, max(1, round(dd * 255_570 / d0)))
        wl = Workload(3, "cfg3_rand1pct_qsgd2", R or R0, dd, off, k, 2, RANDK, QSGD, rounds or T0)
    elif cfg == 4:
        d0, R0, T0 = RESNET50_D, 4, 20
        dd = d or d0
        hi = 2.4e6 * dd / d0 if d else 2.4e6
        off, k = segment_table(dd, 160, 64.0, max(hi, 256.0))
        wl = Workload(4, "cfg4_layerwise_top0.1pct_sign", R or R0, dd, off, k, 1, TOPK, SIGN_L1, rounds or T0)
    elif cfg == 5:
        d0, R0, T0 = 1 << 28, 4, 5
        dd = d or d0
        off, k = _one_segment(dd, max(1, round(dd * 26_844 / d0)))
        wl = Workload(5, "cfg5_large_top0.01pct_qsgd256", R or R0, dd, off, k, 256, TOPK, QSGD, rounds or T0)
    elif cfg == 6:
        # the paper's own ResNet-50 setting (Section 5.1.1): every tensor compressed on its own with
        # k_t = min(d_t, 1000), 8 workers, SignTop_k; inputs as for configuration 4 (one scale per tensor)
        if d is not None:
            raise ValueError("configuration 6 has ResNet-50's own tensor table; d cannot be changed")
        sizes = np.array(resnet50_tensor_sizes(), dtype=np.int64)
        off = np.zeros(sizes.size + 1, dtype=np.uint64)
        off[1:] = np.cumsum(sizes).astype(np.uint64)
        k = np.minimum(sizes, 1000).astype(np.uint32)
        wl = Workload(4, "cfg6_resnet50_k_min_d_1000_sign", R or 8, RESNET50_D, off, k, 1, TOPK, SIGN_L1, rounds or 20)
    elif cfg in (7, 8):
        # the comparison schemes of Section 5 without sparsification, as this operator: every coordinate kept (k = d),
        # error feedback, index-free messages; 7: the sign of the whole vector scaled by its l1 norm / d (EF-signSGD),
        # 8: 4-bit QSGD, s = 15 (EF-QSGD).  Inputs as for configuration 2.
        dd = d or RESNET50_D
        off, k = _one_segment(dd, dd)
        wl = Workload(2, "cfg7_ef_sign_dense" if cfg == 7 else "cfg8_ef_qsgd15_dense", R or 2, dd, off, k, 1 if cfg == 7 else 15,
                      TOPK, SIGN_L1 if cfg == 7 else QSGD, rounds or 10, dense=True)
    else:
        raise ValueError("cfg must be 1..8")
    return wl


# ---------------------------------------------------------------------------------------------
# host (numpy) generators: every vector is a pure function of (cfg, worker, round)
# ---------------------------------------------------------------------------------------------
def _sigma(wl: Workload) -> np.ndarray:
    if wl.cfg == 1:
        return np.exp(1.5 * _rng(1, 0).standard_normal(wl.d, dtype=np.float32))
    if wl.cfg in (2, 3):
        return np.exp(2.0 * _rng(2, 0).standard_normal(wl.d, dtype=np.float32))
    if wl.cfg == 4:
        per_seg = np.exp(2.0 * _rng(4, 0).standard_normal(wl.L)).astype(np.float32)
        sizes = np.diff(wl.seg_offset.astype(np.int64))
        return np.repeat(per_seg, sizes)
    if wl.cfg == 5:
        return np.exp(1.0 * _rng(5, 0).standard_normal(wl.d, dtype=np.float32))
    raise ValueError


_sigma_cache: dict = {}


def delta(wl: Workload, rnd: int, worker: int) -> np.ndarray:
    """Delta of one worker at one sync round, float32 [d]."""
    key = (wl.cfg, wl.d, wl.L)
    if key not in _sigma_cache:
        _sigma_cache.clear()
        _sigma_cache[key] = _sigma(wl)
    sig = _sigma_cache[key]
    if wl.cfg in (1, 4):
        z = _rng(wl.cfg, 2, worker, rnd).standard_normal(wl.d, dtype=np.float32)
        return (sig * z).astype(np.float32)
    if wl.cfg in (2, 3):
        g = _rng(2, 1, 0, rnd).standard_normal(wl.d, dtype=np.float32)
        e = _rng(2, 2, worker, rnd).standard_normal(wl.d, dtype=np.float32)
        return (sig * ((g + e) * np.float32(math.sqrt(0.5)))).astype(np.float32)
    if wl.cfg == 5:
        t = _rng(5, 2, worker, rnd).standard_t(3.0, size=wl.d).astype(np.float32)
        return (sig * t).astype(np.float32)
    raise ValueError


def delta_all(wl: Workload, rnd: int) -> np.ndarray:
    """[R, d] float32."""
    return np.stack([delta(wl, rnd, r) for r in range(wl.R)])


# ---------------------------------------------------------------------------------------------
# device (torch) generators for the full-size runs: same distributions, torch's own streams
# ---------------------------------------------------------------------------------------------
class TorchDeltas:
    """Generates Delta[R, d] on a torch device, a pure function of (cfg, round) for a fixed torch build."""

    def __init__(self, wl: Workload, device):
        import torch
        self.torch = torch
        self.wl = wl
        self.device = torch.device(device)
        g = torch.Generator(device=self.device)
        g.manual_seed(BASE_SEED * 1000 + wl.cfg)
        if wl.cfg == 4:
            per_seg = torch.exp(2.0 * torch.randn(wl.L, generator=g, device=self.device))
            sizes = torch.from_numpy(np.diff(wl.seg_offset.astype(np.int64))).to(self.device)
            self.sigma = torch.repeat_interleave(per_seg, sizes)
        else:
            a = {1: 1.5, 2: 2.0, 3: 2.0, 5: 1.0}[wl.cfg]
            self.sigma = torch.exp(a * torch.randn(wl.d, generator=g, device=self.device))

    def __call__(self, rnd: int, out=None):
        torch, wl = self.torch, self.wl
        g = torch.Generator(device=self.device)
        g.manual_seed((BASE_SEED * 1000 + wl.cfg) * 4096 + rnd + 1)
        if out is None:
            out = torch.empty(wl.R, wl.d, dtype=torch.float32, device=self.device)
        for r in range(wl.R):
            row = out[r]
            row.normal_(generator=g)
            if wl.cfg == 5:   # Student-t with 3 degrees of freedom: z / sqrt(chi2_3 / 3)
                chi = torch.zeros_like(row)
                tmp = torch.empty_like(row)
                for _ in range(3):
                    tmp.normal_(generator=g)
                    chi.addcmul_(tmp, tmp)
                row.div_(torch.sqrt(chi / 3.0))
                del chi, tmp
            row.mul_(self.sigma)
        if wl.cfg in (2, 3):
            shared = torch.empty(wl.d, dtype=torch.float32, device=self.device).normal_(generator=g)
            shared.mul_(self.sigma)
            out.add_(shared.unsqueeze(0)).mul_(math.sqrt(0.5))
        return out
