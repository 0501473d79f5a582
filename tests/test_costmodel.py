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



def _derived_rows():
    """(profile, kernel, {figure: value}) of every 'derived per kernel' line under profiles/ (rocprofv3 counters of
    bench.py runs, summarised by paper_2510_25977_amd.profsum)."""
    import re
    from pathlib import Path
    rows = []
    for f in sorted((Path(__file__).resolve().parent.parent / "profiles").glob("*_all_kernels.txt")):
        block = f.read_text().split("derived per kernel", 1)[1].split("raw counters", 1)[0]
        for line in block.splitlines()[1:]:
            m = re.match(r"\s+(k_\w+)\s+(.*)", line)
            if not m:
                continue
            figs = {k: float(v) for k, v in re.findall(r"(\w+)\s+([0-9.]+)", m.group(2))}
            rows.append((f.name, m.group(1), figs))
    return rows


def test_tile_model_of_the_compute_unit_against_the_profiles():
    """The tile-shape model behind the kernels' block sizes (counterpart of the paper's Eq. 10-11 on a CDNA4 CU): a
    tile needs (rows + cols) x 32 operand bytes per contraction block of 16 and feeds rows x cols / 1024 MFMAs of 32
    clocks on four matrix cores, so a kernel that pulls `fetch` bytes per clock into its CU can keep the matrix cores
    busy for the fraction fetch / (bytes per MFMA / 8).  Checked against two INDEPENDENT sets of counters of the
    committed profiles: fetch comes from the L1's request counter (TCP_TCC_READ_REQ x 128 B over the active clocks),
    the busy fraction from the sequencer (SQ_VALU_MFMA_BUSY_CYCLES)."""
    assert cm.tile_operand_bytes_per_mfma(256, 256) == 256
    assert cm.tile_operand_bytes_per_mfma(128, 256) == 384
    assert cm.tile_operand_bytes_per_mfma(128, 128) == 512
    assert cm.tile_operand_rate_at_mfma_peak(256, 256) == 32
    assert cm.tile_operand_rate_at_mfma_peak(128, 128) == 64
    assert cm.tile_mfma_fraction(256, 256, 44.0) == 1.0
    # register file: 256 x 256 is the largest tile with two waves per SIMD; the paper's SBUF limit in this chip's terms
    assert cm.tile_fits_register_file(256, 256) and not cm.tile_fits_register_file(256, 512)
    assert cm.tile_accumulator_bytes(256, 256) == 256 * 1024
    tile = {"k_s1": (128, 128), "k_gate_up": (256, 256), "k_down1": (256, 256), "k_out": (256, 256)}
    checked = 0
    for prof, kernel, f in _derived_rows():
        if kernel not in tile or not prof.startswith(("prefill", "wide")):
            continue
        predicted = cm.tile_mfma_fraction(*tile[kernel], f["fetch"])
        # the fused gate/up kernel also spends matrix-core-idle time on the SiLU burst, so it sits a little below
        assert abs(predicted - f["mfma_busy"]) <= 0.07, (prof, kernel, predicted, f)
        checked += 1
    assert checked >= 15
    # what bounds `fetch`: lines of 128 B a CU has outstanding at L2 (Little's law on the same counters).  The kernels
    # that wait for operands sit at 58 - 69 in every profile but one (84), nothing is ever above that: fetch is about
    # 68 x 128 B / latency
    for prof, kernel, f in _derived_rows():
        if "in_flight" in f:
            assert f["in_flight"] <= 90.0, (prof, kernel, f)
            assert abs(f["in_flight"] - cm.lines_in_flight(f["fetch"], f["latency"])) <= 0.6
    assert cm.fetch_rate_bound(latency_clk=250.0) > 32 > cm.fetch_rate_bound(latency_clk=300.0)   # 256 x 256 tiles need 32 B/clk
    assert 13.0 < cm.fetch_rate_bound(latency_clk=600.0) < 15.0    # all 256 CUs at HBM latency: ~7 TB/s at 2.1 GHz
