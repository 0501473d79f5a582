"""Seeded synthetic inputs for the SVD-factored MLP forward.

This module only *draws* tensors; it contains none of the method's arithmetic
and is the one piece of code that both the GPU tests/bench and the CPU oracle's
tests may share.  Values are drawn in float64, scaled, and rounded ONCE to the
storage type (bf16 round-to-nearest-even through ``torch``; or fp32).  The
rounded values are the inputs of both sides; ``to_f64`` converts them exactly.

The shapes stand in for the LLM MLP layers the paper evaluates (hidden size
2048-7168, intermediate size 8192-18432; paper Sec. 5.1-5.2): no checkpoint or
dataset is used anywhere.

Workloads (``WORKLOADS``):
  linear_fp32   single factored linear layer, fp32, W = Q1 diag(i^-0.7) Q2^T
  mlp_small     d=2048  ffn=8192   r=256            M=128
  decode        d=4096  ffn=14336  r=512            M in {1,4,16}
  prefill       d=4096  ffn=14336  r in {256,512,1024}  M=4096
  wide          d=5120  ffn=27648  r=1024           M=2048, power-law U columns,
                1 % of the entries of X scaled x20
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

BASE_SEED = 20251025

_TENSOR_IDS = {"X": 0, "Ug": 1, "Vg": 2, "Uu": 3, "Vu": 4, "Ud": 5, "Vd": 6, "mask": 7, "G1": 8, "G2": 9}


def _rng(stream: int, name: str) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED, int(stream), _TENSOR_IDS[name]]))


def _store(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    """Round a float64 array once to the storage dtype (RNE)."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).contiguous()


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact conversion of a stored tensor (bf16 / fp32) to numpy float64."""
    return t.detach().cpu().to(torch.float64).numpy()


def _normal(stream: int, name: str, shape, var: float) -> np.ndarray:
    return _rng(stream, name).standard_normal(shape) * np.sqrt(var)


@dataclass
class GatedInputs:
    X: torch.Tensor
    Ug: torch.Tensor
    Vg: torch.Tensor
    Uu: torch.Tensor
    Vu: torch.Tensor
    Ud: torch.Tensor
    Vd: torch.Tensor

    @property
    def dims(self):
        M, d = self.X.shape
        r, ffn = self.Vg.shape
        r_down = self.Ud.shape[1]
        return dict(M=M, d=d, ffn=ffn, r=r, r_down=r_down)

    def factors(self) -> Dict[str, torch.Tensor]:
        return dict(Ug=self.Ug, Vg=self.Vg, Uu=self.Uu, Vu=self.Vu, Ud=self.Ud, Vd=self.Vd)


def make_gated(M: int, d: int, ffn: int, r: int, r_down: Optional[int] = None, *, stream: int = 0,
               dtype: torch.dtype = torch.bfloat16, u_spectrum_exp: Optional[float] = None,
               v_var: Optional[float] = None, outlier_prob: float = 0.0,
               outlier_scale: float = 20.0) -> GatedInputs:
    """Factors ~ N(0, 1/fan_in), X ~ N(0,1).

    ``u_spectrum_exp = a`` scales column i (1-based) of every U by i^-a;
    ``v_var`` overrides the variance of every V (default 1/fan_in = 1/r);
    ``outlier_prob`` multiplies each entry of X by ``outlier_scale`` with that
    probability (element-wise Bernoulli mask).
    """
    r_down = r if r_down is None else r_down

    def u_like(name, rows, cols):
        a = _normal(stream, name, (rows, cols), 1.0 / rows)
        if u_spectrum_exp is not None:
            a = a * (np.arange(1, cols + 1, dtype=np.float64) ** (-u_spectrum_exp))[None, :]
        return _store(a, dtype)

    def v_like(name, rows, cols):
        var = (1.0 / rows) if v_var is None else v_var
        return _store(_normal(stream, name, (rows, cols), var), dtype)

    X = _normal(stream, "X", (M, d), 1.0)
    if outlier_prob > 0.0:
        mask = _rng(stream, "mask").random((M, d)) < outlier_prob
        X = np.where(mask, X * outlier_scale, X)
    return GatedInputs(
        X=_store(X, dtype),
        Ug=u_like("Ug", d, r), Vg=v_like("Vg", r, ffn),
        Uu=u_like("Uu", d, r), Vu=v_like("Vu", r, ffn),
        Ud=u_like("Ud", ffn, r_down), Vd=v_like("Vd", r_down, d),
    )


@dataclass
class LinearInputs:
    X: torch.Tensor      # [M, d]
    U: torch.Tensor      # [d, r]
    V: torch.Tensor      # [r, n]
    W: Optional[np.ndarray] = None   # [d, n] float64, the full-rank matrix before truncation / rounding
    s: Optional[np.ndarray] = None   # singular values of W (float64, descending)


def make_linear_powerlaw(M: int = 32, d: int = 256, n: int = 1024, r: int = 16, *, stream: int = 1,
                         decay: float = 0.7, dtype: torch.dtype = torch.float32) -> LinearInputs:
    """W = Q1 diag(s) Q2^T with s_i = i^-decay, Q1/Q2 orthonormal from sign-fixed reduced QR of
    seeded Gaussians; U = Q1[:, :r] diag(s[:r]), V = Q2[:, :r]^T."""
    k = min(d, n)

    def ortho(name, rows):
        q, rr = np.linalg.qr(_rng(stream, name).standard_normal((rows, k)))
        return q * np.sign(np.diag(rr))[None, :]

    Q1 = ortho("G1", d)
    Q2 = ortho("G2", n)
    s = np.arange(1, k + 1, dtype=np.float64) ** (-decay)
    W = (Q1 * s[None, :]) @ Q2.T
    U = Q1[:, :r] * s[None, :r]
    V = Q2[:, :r].T
    X = _normal(stream, "X", (M, d), 1.0)
    return LinearInputs(X=_store(X, dtype), U=_store(U, dtype), V=_store(V, dtype), W=W, s=s)


def make_linear_gaussian(M: int, d: int, n: int, r: int, *, stream: int = 6, dtype: torch.dtype = torch.bfloat16) -> LinearInputs:
    """Stand-alone factored layer O = (X U) V with Gaussian factors: U ~ N(0, 1/d), V ~ N(0, 1/r), X ~ N(0, 1)
    (so T = X U and O are O(1) per entry).  The shape of the paper's kernel evaluation (Sec. 5.2) is
    d = 8192, r = 4096, n = 16384."""
    return LinearInputs(X=_store(_normal(stream, "X", (M, d), 1.0), dtype), U=_store(_normal(stream, "Ug", (d, r), 1.0 / d), dtype),
                        V=_store(_normal(stream, "Vg", (r, n), 1.0 / r), dtype))


# ----------------------------------------------------------------------------------------------
# Named workloads (the five benchmark configurations).
# ----------------------------------------------------------------------------------------------
WORKLOADS = {
    "mlp_small": dict(d=2048, ffn=8192, r=256, M=128, stream=2),
    "decode": dict(d=4096, ffn=14336, r=512, M=16, stream=3),
    "prefill": dict(d=4096, ffn=14336, r=512, M=4096, stream=4),
    "wide": dict(d=5120, ffn=27648, r=1024, M=2048, stream=5, u_spectrum_exp=0.5, v_var=1.0 / 1024,
                 outlier_prob=0.01),
}


def make_workload(name: str, *, M: Optional[int] = None, r: Optional[int] = None) -> GatedInputs:
    """Inputs of a named gated workload; ``M`` / ``r`` override the defaults (decode: M in {1,4,16};
    prefill: r in {256,512,1024}).  The random stream depends on the workload and on r, not on M:
    a smaller M takes the leading rows of the same X stream only when drawn with the same M."""
    cfg = dict(WORKLOADS[name])
    if M is not None:
        cfg["M"] = M
    if r is not None:
        cfg["r"] = r
        if cfg.get("v_var") is not None:
            cfg["v_var"] = 1.0 / r
    stream = cfg.pop("stream") * 10000 + cfg["r"]
    return make_gated(cfg.pop("M"), cfg.pop("d"), cfg.pop("ffn"), cfg.pop("r"), stream=stream, **cfg)
