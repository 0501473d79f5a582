"""The roof microbenchmarks of the library run and order the way the benchmark's reading of them assumes: the matrix
cores are slower on operands with many live bits than on zeros (power-limited clock), and a product cannot beat the
rate measured on operands like its own."""
import time

import pytest
import torch

from paper_2510_25977_amd import binding as B

pytestmark = pytest.mark.gpu


def mfma_tflops(mode, iters=4000):
    dev = torch.device("cuda:0")
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    s = torch.cuda.current_stream().cuda_stream
    best = 0.0
    for _ in range(6):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        B.svdmlp_roof_mfma_operands(iters, mode, sink.data_ptr(), cus, s)
        b.record()
        b.synchronize()
        best = max(best, cus * 8 * 4 * iters * 32768 / (a.elapsed_time(b) * 1e-3) / 1e12)
    assert int(sink.abs().sum().item()) == 0
    return best


def test_mfma_roof_depends_on_operand_values():
    zero = mfma_tflops(B.ROOF_OPERANDS_ZERO)
    const = mfma_tflops(B.ROOF_OPERANDS_CONSTANT)
    rnd = mfma_tflops(B.ROOF_OPERANDS_RANDOM)
    # published dense bf16 peak 2.5 PFLOP/s; nothing measured may exceed it by more than timer noise
    assert 500.0 < rnd <= const * 1.03 and const <= zero * 1.03 and zero < 2600.0, (zero, const, rnd)
    # the point of the third mode: real data runs visibly below the zero-operand rate
    assert rnd < 0.9 * zero, (zero, rnd)


def test_tile_skeleton_without_copies_reaches_the_matrix_cores_rate():
    """Barriers and LDS reads of the two-phase tile skeleton cost next to nothing: on zeros it runs at the published
    peak, on random operands within a fifth of the rate the register-operand loop reaches on random operands (measured:
    1755 against 1900 TFLOP/s; the LDS reads draw power too)."""
    dev = torch.device("cuda:0")
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    s = torch.cuda.current_stream().cuda_stream
    steps = 2000
    rate = {}
    for mode in (B.ROOF_OPERANDS_ZERO, B.ROOF_OPERANDS_RANDOM):
        best = 0.0
        for _ in range(6):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            B.svdmlp_roof_pingpong(steps, mode, sink.data_ptr(), cus, s)
            b.record()
            b.synchronize()
            best = max(best, cus * 8 * 16 * steps * 32768 / (a.elapsed_time(b) * 1e-3) / 1e12)
        rate[mode] = best
    assert int(sink.abs().sum().item()) == 0
    assert rate[B.ROOF_OPERANDS_ZERO] > 0.9 * mfma_tflops(B.ROOF_OPERANDS_ZERO), rate
    assert rate[B.ROOF_OPERANDS_RANDOM] > 0.8 * mfma_tflops(B.ROOF_OPERANDS_RANDOM), rate
    assert rate[B.ROOF_OPERANDS_RANDOM] < 0.9 * rate[B.ROOF_OPERANDS_ZERO], rate


def test_roof_entry_points_check_their_arguments():
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    for bad in (dict(iters=0, operands=1), dict(iters=10, operands=3), dict(iters=10, operands=-1)):
        with pytest.raises(B.SvdMlpError) as e:
            B.svdmlp_roof_mfma_operands(bad["iters"], bad["operands"], sink.data_ptr(), 4)
        assert e.value.status == B.SVDMLP_INVALID_ARGUMENT
        with pytest.raises(B.SvdMlpError) as e:
            B.svdmlp_roof_pingpong(bad["iters"], bad["operands"], sink.data_ptr(), 4)
        assert e.value.status == B.SVDMLP_INVALID_ARGUMENT
