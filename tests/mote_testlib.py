"""Glue shared by the GPU parity tests, the smoke check and the benchmark: turns a seeded
workload (workloads.py) into (a) device tensors + a MoteLayer for the HIP path and (b) the
numpy inputs of the CPU oracle.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import workloads as W


# Routed-expert weights depend on (seed, shape) only, not on the batch: configurations that differ in
# the number of tokens share them.  Small caches keep the full-size tests from drawing and ternarising
# the same 48 matrices again (device: packed words and scales; host: the oracle's ternary matrices).
_GPU_WEIGHTS = {}
_ORACLE_EXPERTS = {}


def _weights_key(cfg, binary):
    return (cfg.seed, cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.sigma_latent, bool(binary))


class GpuProblem:
    """Device side of a workload: weights packed by mote_pack_ternary on the GPU."""

    def __init__(self, cfg: W.MoteConfig, device="cuda:0", latent_source=None, shared_bits=0, binary_experts=False):
        import paper_2506_14435_amd as M
        self.cfg = cfg
        dev = torch.device(device)
        d, f, e = cfg.d_model, cfg.d_ff, cfg.n_experts
        self.x = W.make_x(cfg).to(dev)
        self.w_router = W.make_router(cfg).to(dev)
        bias = W.make_router_bias(cfg)
        self.bias = None if bias is None else bias.to(dev)
        self.shared = tuple(t.to(dev) for t in W.make_shared(cfg))
        words = d * f // 16
        key = _weights_key(cfg, binary_experts) + (str(dev),)
        cached = _GPU_WEIGHTS.get(key) if latent_source is None else None
        if cached is not None:
            self.wt, self.alpha = cached
        else:
            self.wt = [torch.empty(e, words, dtype=torch.int32, device=dev) for _ in range(3)]
            self.alpha = torch.empty(e, 3, dtype=torch.float32, device=dev)
            tmp_alpha = torch.empty(1, dtype=torch.float32, device=dev)
            for ex in range(e):
                for m in range(3):
                    if latent_source is None:
                        lat = W.make_latent(cfg, ex, m).to(dev)
                    else:
                        lat = latent_source(ex, m)
                    M.mote_pack_ternary(lat, packed=self.wt[m][ex], alpha=tmp_alpha, binary=binary_experts)
                    self.alpha[ex, m] = tmp_alpha[0]
                    del lat
            if latent_source is None and e * d * f >= 5e7:       # only the large shapes are worth keeping
                _GPU_WEIGHTS.clear()                              # one large shape at a time
                _GPU_WEIGHTS[key] = (self.wt, self.alpha)
        self.shared_bits = shared_bits
        self.shared_scales = None
        self.shared_bf16 = self.shared
        if shared_bits:          # post-training quantised shared expert: packed by mote_pack_rtn on the GPU
            packed = [M.mote_pack_rtn(t, shared_bits) for t in self.shared]
            self.shared = tuple(p for p, _ in packed)
            self.shared_scales = tuple(s for _, s in packed)
        torch.cuda.synchronize()
        self.layer = M.MoteLayer(self.w_router, *self.shared, *self.wt, self.alpha, cfg.top_k,
                                 router_bias=self.bias, shared_bits=shared_bits, shared_scales=self.shared_scales)


class OracleProblem:
    """Oracle side of the same workload: numpy inputs; experts ternarised lazily by the
    oracle's own Q_w."""

    def __init__(self, cfg: W.MoteConfig, shared_bits=0, binary_experts=False):
        self.cfg = cfg
        self.binary_experts = binary_experts
        self.x = W.bf16_bits(W.make_x(cfg))
        self.w_router = W.bf16_bits(W.make_router(cfg))
        bias = W.make_router_bias(cfg)
        self.bias = None if bias is None else bias.numpy()
        self.shared = tuple(W.bf16_bits(t) for t in W.make_shared(cfg))
        if shared_bits:
            from oracle import mote_oracle as O
            q = [O.rtn_quantize(w, shared_bits) for w in self.shared]
            self.shared = (*q[0], *q[1], *q[2])
        key = _weights_key(cfg, binary_experts)
        if cfg.n_experts * cfg.d_model * cfg.d_ff >= 5e7:
            if key not in _ORACLE_EXPERTS:
                _ORACLE_EXPERTS.clear()                           # one large shape at a time
                _ORACLE_EXPERTS[key] = {}
            self._experts = _ORACLE_EXPERTS[key]
        else:
            self._experts = {}

    def experts(self, e: int):
        from oracle import mote_oracle as O
        if e not in self._experts:
            r = []
            for m in range(3):
                lat = W.make_latent(self.cfg, e, m).numpy()
                t, a = O.binarize(lat) if self.binary_experts else O.ternarize(lat)
                r += [t, a]
            self._experts[e] = tuple(r)
        return self._experts[e]

    def forward(self, tokens=None):
        from oracle import mote_oracle as O
        return O.layer_forward(self.x, self.w_router, self.bias, self.cfg.top_k, self.shared, self.experts,
                               tokens=tokens)

    def block_forward(self, norm, tokens=None):
        from oracle import mote_oracle as O
        return O.block_forward(self.x, norm, self.w_router, self.bias, self.cfg.top_k, self.shared, self.experts,
                               tokens=tokens)


def bits(t: torch.Tensor) -> np.ndarray:
    """Device bf16 tensor -> numpy uint16 bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def error_metrics(out_bf16_bits: np.ndarray, ref_f32: np.ndarray):
    """(max-abs-err, rel-L2) of a bf16 result against the oracle's unrounded fp32 output."""
    got = (out_bf16_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    ref = ref_f32.astype(np.float64)
    max_abs = float(np.abs(got - ref).max())
    rel_l2 = float(np.sqrt(((got - ref) ** 2).sum() / max((ref ** 2).sum(), 1e-300)))
    return max_abs, rel_l2
