"""Work and traffic accounting for factored matmuls (host-side, no GPU).

These are the formulas the benchmark uses to turn a measured time into
TFLOP/s and GB/s.  They follow the paper's own accounting (a multiply-add is
two FLOPs, as in its Table 1) so its printed figures can pin them.
"""
from __future__ import annotations

import math


def xuv_flops(M: int, K: int, r: int, N: int) -> int:
    """FLOPs of O = (X U) V with the intermediate computed once: 2 M r (K + N).
    (numerator of the paper's Eq. 10; Table 1, 'Sequential Matmul')."""
    return 2 * M * r * (K + N)


def xuv_naive_fused_flops(M: int, K: int, r: int, N: int, B_N: int) -> int:
    """FLOPs when (X U) is recomputed for every output column block (paper Alg. 1):
    the first product is repeated ceil(N / B_N) times (Sec. 3.2)."""
    return math.ceil(N / B_N) * 2 * M * K * r + 2 * M * r * N


def xuv_hbm_bytes(M: int, K: int, r: int, N: int, B_M: int, s: int = 2) -> float:
    """HBM traffic model of the paper's fused kernel (denominator of Eq. 10): X read once,
    O written once, U and V re-read for each of the M / B_M row strips."""
    return s * (M * (K + N) + (M / B_M) * r * (K + N))


def xuv_arithmetic_intensity(r: int, B_M: int, s: int = 2) -> float:
    """Paper Eq. 10 in closed form: 2 r / ((1 + r / B_M) s)."""
    return 2.0 * r / ((1.0 + r / B_M) * s)


def peak_sbuf_bytes(B_M: int, B_K: int, B_r: int, B_N: int, r: int, s: int = 2) -> int:
    """Paper Eq. 11: on-chip footprint of the two phases of the fused kernel."""
    return (B_M * r + (B_M + B_r) * max(B_K, B_N)) * s


def block_aligned_rank(k: int, n: int, ratio: float, block_size: int = 128, alpha: float = 0.5) -> int:
    """Paper Eq. 5: rank for a target compression ratio, snapped to a multiple of block_size.
    (At least one block is kept.)"""
    blocks = math.floor(k * n * (1.0 - ratio) / ((k + n) * block_size) + alpha)
    return max(blocks, 1) * block_size


def compression_ratio(k: int, n: int, r: int) -> float:
    """Paper Eq. 4 for one matrix: 1 - r (k + n) / (k n)."""
    return 1.0 - r * (k + n) / (k * n)


def gated_mlp_flops(M: int, d: int, ffn: int, r: int, r_down: int | None = None) -> int:
    """Algorithmic FLOPs of the factored gated MLP: gate + up + down chains (SiLU not counted).
    With r_down = r this is 6 M r (d + ffn)."""
    r_down = r if r_down is None else r_down
    return 2 * xuv_flops(M, d, r, ffn) + xuv_flops(M, ffn, r_down, d)


def gated_mlp_bytes(M: int, d: int, ffn: int, r: int, r_down: int | None = None, s: int = 2) -> int:
    """Compulsory HBM bytes: every factor element once, X once, Y once."""
    r_down = r if r_down is None else r_down
    return s * (2 * r * (d + ffn) + r_down * (d + ffn) + 2 * M * d)


def dense_mlp_flops(M: int, d: int, ffn: int) -> int:
    """FLOPs of the uncompressed gated MLP (three dense matmuls)."""
    return 6 * M * d * ffn


def sqrt_sigma_factors(W, r: int):
    """Rank-r factors of a dense weight W[k, n] with the singular values split evenly between the two sides
    (paper Sec. 3.1, Eq. 6-8): W ~ U V with U = U_r sqrt(S_r) [k, r] and V = sqrt(S_r) V_r^T [r, n].
    Plain truncated SVD of a given matrix (float64 numpy): no whitening, no fine-tuning.  Returns (U, V, s) with s
    all singular values of W, so that the truncation error is known in closed form:
    ||W - U V||_F = sqrt(sum(s[r:]**2))."""
    import numpy as np
    W = np.asarray(W, dtype=np.float64)
    if W.ndim != 2 or not (1 <= r <= min(W.shape)):
        raise ValueError("W must be a matrix and 1 <= r <= min(W.shape)")
    u, s, vt = np.linalg.svd(W, full_matrices=False)
    root = np.sqrt(s[:r])
    return u[:, :r] * root[None, :], root[:, None] * vt[:r, :], s

