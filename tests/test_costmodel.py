"""Host-side accounting pinned to the figures the paper prints."""
import pytest

from paper_2510_25977_amd import costmodel as cm
from tests.conftest import read_golden


def test_table1_flop_counts():
    for M, K, r, N, B_N, seq, naive in read_golden("paper_table1_flops.txt"):
        M, K, r, N, B_N = map(int, (M, K, r, N, B_N))
        assert round(cm.xuv_flops(M, K, r, N) / 1e9, 2) == seq
        assert round(cm.xuv_naive_fused_flops(M, K, r, N, B_N) / 1e9, 2) == naive
        # the recompute factor of Sec. 3.2: ceil(8192 / 512) = 16, a 4x increase in FLOPs
        assert cm.xuv_naive_fused_flops(M, K, r, N, B_N) / cm.xuv_flops(M, K, r, N) == pytest.approx(4.0)


def test_table3_arithmetic_intensity_eq10():
    M, K, N = 4096, 7168, 18432
    for B_M, r, s, printed in read_golden("paper_table3_intensity.txt"):
        B_M, r, s = int(B_M), int(r), int(s)
        ai = cm.xuv_arithmetic_intensity(r, B_M, s)
        assert abs(ai - printed) <= 0.035          # the paper truncates / rounds to two decimals
        # closed form == ratio of the two models
        assert ai == pytest.approx(cm.xuv_flops(M, K, r, N) / cm.xuv_hbm_bytes(M, K, r, N, B_M, s))


def test_eq11_is_max_of_two_phases():
    B_M, B_K, B_r, B_N, r = 1024, 512, 128, 256, 4096
    p1 = (B_M * r + B_M * B_K + B_K * B_r) * 2
    p2 = (B_M * r + B_r * B_N + B_M * B_N) * 2
    # the paper's closed form bounds both phases from above
    assert cm.peak_sbuf_bytes(B_M, B_K, B_r, B_N, r) >= max(p1, p2)
    assert cm.peak_sbuf_bytes(B_M, B_K, B_r, B_N, r) == (B_M * r + (B_M + B_r) * max(B_K, B_N)) * 2


def test_rank_rule_eq5():
    # k n (1-ratio) / ((k+n) block) = 2048*8192*0.8/(10240*128) = 10.24 -> floor(10.74) = 10 blocks
    assert cm.block_aligned_rank(2048, 8192, 0.2, 128) == 1280
    # 4096*14336*0.95/(18432*128) = 23.64 -> floor(24.14) = 24 blocks
    assert cm.block_aligned_rank(4096, 14336, 0.05, 128) == 3072
    assert cm.block_aligned_rank(64, 64, 0.99, 128) == 128          # never zero blocks
    r = cm.block_aligned_rank(4096, 14336, 0.05, 128)
    assert abs(cm.compression_ratio(4096, 14336, r) - 0.05) < 0.02


def test_gated_mlp_totals():
    M, d, ffn, r = 4096, 4096, 14336, 512
    assert cm.gated_mlp_flops(M, d, ffn, r) == 6 * M * r * (d + ffn)
    assert cm.gated_mlp_bytes(M, d, ffn, r) == 2 * (3 * r * (d + ffn) + 2 * M * d)
    assert cm.dense_mlp_flops(M, d, ffn) == 6 * M * d * ffn
    assert cm.gated_mlp_flops(16, d, ffn, r, r_down=256) == 2 * 2 * 16 * r * (d + ffn) + 2 * 16 * 256 * (d + ffn)


def test_sqrt_sigma_factors_truncation_error_and_balance():
    """Factoriser of Eq. 6-8 on a synthetic matrix: Eckart-Young residual, equal column / row norms of the two
    factors (each carries sqrt(s_i)), and the oracle's factored product equals X W_r."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(7)
    W = rng.standard_normal((48, 80)) @ np.diag(np.arange(1, 81, dtype=np.float64) ** -0.8)
    r = 16
    U, V, s = cm.sqrt_sigma_factors(W, r)
    assert U.shape == (48, r) and V.shape == (r, 80)
    assert np.isclose(np.linalg.norm(W - U @ V), np.sqrt(np.sum(s[r:] ** 2)), rtol=1e-10)
    assert np.allclose(np.linalg.norm(U, axis=0), np.sqrt(s[:r]), rtol=1e-10)
    assert np.allclose(np.linalg.norm(V, axis=1), np.sqrt(s[:r]), rtol=1e-10)
    X = rng.standard_normal((5, 48))
    assert np.allclose(oracle.linear(X, U, V), X @ (U @ V), rtol=1e-10, atol=1e-12)
    r_rule = cm.block_aligned_rank(48, 80, 0.5, block_size=8)
    U2, V2, _ = cm.sqrt_sigma_factors(W, r_rule)
    assert cm.compression_ratio(48, 80, r_rule) <= 0.55 and U2.shape[1] == r_rule



def test_tile_model_of_the_compute_unit():
    """The tile-shape model behind the kernels' block sizes (counterpart of the paper's Eq. 10-11 on a CDNA4 CU),
    checked against the figures the design quotes and against rocprofv3 measurements of the default workload
    (profiles/prefill_r512_pmc_traffic_mfma.txt): MFMA-busy fraction 0.31 for the 128 x 128 first stage and 0.53-0.54
    for the 256 x 256 gate/up kernel at the operand rates measured there."""
    assert cm.tile_operand_bytes_per_mfma(256, 256) == 256
    assert cm.tile_operand_bytes_per_mfma(128, 256) == 384
    assert cm.tile_operand_bytes_per_mfma(128, 128) == 512
    assert cm.tile_operand_rate_at_mfma_peak(256, 256) == 32
    assert cm.tile_operand_rate_at_mfma_peak(128, 128) == 64
    # measured: k_s1 pulls ~20 B/clk per CU (4.325e6 requests x 128 B over 256 CUs x 1.06e5 clk) and is 0.308 MFMA-busy
    assert abs(cm.tile_mfma_fraction(128, 128, 20.0) - 0.31) < 0.01
    # measured: k_gate_up pulls 17-18 B/clk and is 0.53-0.54 MFMA-busy
    assert 0.52 < cm.tile_mfma_fraction(256, 256, 17.5) < 0.56
    assert cm.tile_mfma_fraction(256, 256, 44.0) == 1.0          # the copy rate from L2 alone would not bound it
    # register file: 256 x 256 is the largest tile with two waves per SIMD; the paper's SBUF limit in this chip's terms
    assert cm.tile_fits_register_file(256, 256) and not cm.tile_fits_register_file(256, 512)
    assert cm.tile_accumulator_bytes(256, 256) == 256 * 1024
