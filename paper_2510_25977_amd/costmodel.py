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



# ----------------------------------------------------------------------------------------------
# The MI355X counterpart of the paper's block-size model (Sec. 4.2.2, Eq. 10-11).  On Trainium the block height B_M
# sets the arithmetic intensity against HBM and the SBUF footprint caps it; on a CDNA4 compute unit the tile shape sets
# the operand bytes that must reach the CU per MFMA and the register file caps the tile.
# ----------------------------------------------------------------------------------------------
MFMA_ROWS, MFMA_COLS, MFMA_K = 32, 32, 16          # v_mfma_f32_32x32x16_bf16
MFMA_CLK_PER_SIMD = 32                             # one such MFMA occupies a SIMD's matrix core for 32 clocks
SIMDS_PER_CU = 4
REGISTER_FILE_BYTES_PER_CU = 512 * 1024


def tile_operand_bytes_per_mfma(tile_rows: int, tile_cols: int, s: int = 2) -> float:
    """Operand bytes a workgroup must bring into its CU per MFMA for a tile_rows x tile_cols output tile: one
    contraction block (16) needs (tile_rows + tile_cols) * 16 elements and feeds tile_rows/32 * tile_cols/32 MFMAs.
    256 x 256: 256 B, 128 x 256: 384 B, 128 x 128: 512 B."""
    return (tile_rows + tile_cols) * MFMA_K * s / ((tile_rows // MFMA_ROWS) * (tile_cols // MFMA_COLS))


def tile_operand_rate_at_mfma_peak(tile_rows: int, tile_cols: int, s: int = 2) -> float:
    """Bytes per clock a CU would have to fetch to keep its four matrix cores busy on such a tile
    (256 x 256: 32 B/clk, 128 x 128: 64 B/clk)."""
    return tile_operand_bytes_per_mfma(tile_rows, tile_cols, s) * SIMDS_PER_CU / MFMA_CLK_PER_SIMD


def tile_mfma_fraction(tile_rows: int, tile_cols: int, fetch_bytes_per_clk: float, s: int = 2) -> float:
    """Fraction of the MFMA rate a fetch-bound kernel reaches on such a tile when its CU pulls operands in at the
    given rate (the counterpart of reading Eq. 10 against the machine balance): min(1, rate / rate needed)."""
    return min(1.0, fetch_bytes_per_clk / tile_operand_rate_at_mfma_peak(tile_rows, tile_cols, s))


def tile_accumulator_bytes(tile_rows: int, tile_cols: int) -> int:
    """fp32 accumulators of the tile, spread over the CU's register file (the counterpart of Eq. 11's footprint)."""
    return tile_rows * tile_cols * 4


def tile_fits_register_file(tile_rows: int, tile_cols: int) -> bool:
    """The accumulators of a tile may take at most half of the CU's register file: the eight waves that share the tile
    need the other half for operand fragments, the squashed gate tile (16 bits per accumulator) and addresses.
    256 x 256 fp32 (256 KiB) is the largest square tile that fits; 256 x 512 would fill the file with accumulators."""
    return 2 * tile_accumulator_bytes(tile_rows, tile_cols) <= REGISTER_FILE_BYTES_PER_CU


# What bounds the operand rate of a CU (measured, profiles/): the L1 of a CU keeps at most about 68 requests of 128 B
# outstanding at L2, so by Little's law it pulls at most 68 x 128 B per L2 latency: 35 B/clk when every request hits
# L2 (about 250 clocks), 14 B/clk when every request goes out to the memory-side cache or HBM (about 600 clocks idle,
# 1300 under load) -- which, times 256 CUs, is also the 7 TB/s a plain streaming read reaches on this part.
CU_OUTSTANDING_LINES = 68
LINE_BYTES = 128


def fetch_rate_bound(latency_clk: float, lines: float = CU_OUTSTANDING_LINES) -> float:
    """Bytes per clock a CU can pull in when its requests take latency_clk on average."""
    return lines * LINE_BYTES / latency_clk


def lines_in_flight(fetch_bytes_per_clk: float, latency_clk: float) -> float:
    """Little's law the other way round: lines outstanding at a measured rate and latency."""
    return fetch_bytes_per_clk * latency_clk / LINE_BYTES
