"""Pins for the fp64 CPU oracle: every check here is fixed by mathematics or by numpy's own float64
routines, never by the oracle itself or by the GPU path."""
import math

import numpy as np
import pytest

import oracle
from paper_2510_25977_amd import synth
from tests.conftest import read_golden


def relmax(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


def np_silu(x):
    return x / (1.0 + np.exp(-x))


def np_dense_mlp(X, Ug, Vg, Uu, Vu, Ud, Vd):
    """Dense evaluation with the factor products formed first (different association order)."""
    Wg, Wu, Wd = Ug @ Vg, Uu @ Vu, Ud @ Vd
    return (np_silu(X @ Wg) * (X @ Wu)) @ Wd


# ------------------------------------------------------------------ full-rank exactness
def test_full_rank_exact_svd_reproduces_XW():
    rng = np.random.default_rng(7)
    W = rng.standard_normal((48, 80))
    X = rng.standard_normal((9, 48))
    Uf, s, Vt = np.linalg.svd(W, full_matrices=False)
    O = oracle.linear(X, Uf * s[None, :], Vt)
    assert relmax(O, X @ W) <= 1e-10


@pytest.mark.parametrize("r", [256])
def test_full_rank_constructed_factors_reproduce_XW(r):
    li = synth.make_linear_powerlaw(r=r, dtype=np_dtype_to_torch("float64"))
    X, U, V = synth.to_f64(li.X), synth.to_f64(li.U), synth.to_f64(li.V)
    assert relmax(oracle.linear(X, U, V), X @ li.W) <= 1e-10


def np_dtype_to_torch(name):
    import torch
    return getattr(torch, name)


# ------------------------------------------------------------------ Eckart-Young
def test_eckart_young_residual_matches_closed_form():
    (n_sv, decay, r, resid, total), = read_golden("eckart_young_powerlaw.txt")
    li = synth.make_linear_powerlaw(M=4, r=int(r), decay=decay, dtype=np_dtype_to_torch("float64"))
    assert li.s.shape[0] == int(n_sv)
    U, V = synth.to_f64(li.U), synth.to_f64(li.V)
    d = U.shape[0]
    W_r = oracle.linear(np.eye(d), U, V)          # the oracle applied to the identity yields U_r V_r
    assert abs(np.linalg.norm(li.W - W_r) - resid) <= 1e-10 * resid
    assert abs(np.linalg.norm(li.W) - total) <= 1e-10 * total
    # cross-check the stored closed form against the formula itself
    s = np.arange(1, int(n_sv) + 1, dtype=np.float64) ** (-decay)
    assert abs(math.sqrt((s[int(r):] ** 2).sum()) - resid) <= 1e-14


def test_truncation_obeys_operator_norm_bound():
    li = synth.make_linear_powerlaw(M=32, r=16, dtype=np_dtype_to_torch("float64"))
    X, U, V = synth.to_f64(li.X), synth.to_f64(li.U), synth.to_f64(li.V)
    E = X @ li.W - oracle.linear(X, U, V)
    bound = li.s[16] * np.linalg.norm(X, axis=1)
    assert np.all(np.linalg.norm(E, axis=1) <= bound * (1 + 1e-9))


# ------------------------------------------------------------------ brute force, tiny integers
def test_tiny_integer_case_matches_dense_form():
    X = np.array([[1, -2, 0, 3], [0, 1, 1, -1], [2, 0, -1, 1]], dtype=np.float64)
    Ug = np.array([[1, 0], [0, 1], [1, 1], [-1, 2]], dtype=np.float64)
    Uu = np.array([[0, 1], [2, -1], [1, 0], [1, 1]], dtype=np.float64)
    Vg = np.array([[1, 0, -1, 2, 0], [0, 1, 1, -1, 3]], dtype=np.float64) / 4
    Vu = np.array([[2, 1, 0, -1, 1], [1, -1, 2, 0, 1]], dtype=np.float64) / 4
    Ud = np.array([[1, -1], [0, 2], [1, 1], [-2, 0], [1, 3]], dtype=np.float64) / 2
    Vd = np.array([[1, 0, 2, -1], [0, 1, -1, 3]], dtype=np.float64)
    Z = oracle.gated(X, Ug, Vg, Uu, Vu, Ud, Vd)
    assert Z.shape == (3, 4)
    assert relmax(Z, np_dense_mlp(X, Ug, Vg, Uu, Vu, Ud, Vd)) <= 1e-12
    # one entry by hand: row 0.  Tg = X0 Ug = [1-0+0-3, 0-2+0+6] = [-2, 4]
    Tg0 = X[0] @ Ug
    assert np.array_equal(Tg0, np.array([-2.0, 4.0]))
    G0 = (Tg0 @ Vg)                       # [-2/4, 4/4, (2+4)/4, (-4-4)/4, 12/4]
    assert np.allclose(G0, [-0.5, 1.0, 1.5, -2.0, 3.0], atol=0, rtol=0)
    _, H = oracle.gated(X, Ug, Vg, Uu, Vu, Ud, Vd, return_H=True)
    P0 = (X[0] @ Uu) @ Vu
    expect_H0 = np.array([g / (1 + math.exp(-g)) * p for g, p in zip(G0, P0)])
    assert relmax(H[0], expect_H0) <= 1e-15


# ------------------------------------------------------------------ special cases
def _rand_gated(seed, M=5, d=12, ffn=20, r=6, r2=4):
    rng = np.random.default_rng(seed)
    return dict(X=rng.standard_normal((M, d)), Ug=rng.standard_normal((d, r)), Vg=rng.standard_normal((r, ffn)),
                Uu=rng.standard_normal((d, r)), Vu=rng.standard_normal((r, ffn)),
                Ud=rng.standard_normal((ffn, r2)), Vd=rng.standard_normal((r2, d)))


def test_zero_gate_factor_gives_exact_zero():
    a = _rand_gated(1)
    a["Vg"][:] = 0.0
    assert np.all(oracle.gated(**a) == 0.0)


def test_zero_input_gives_exact_zero():
    a = _rand_gated(2)
    a["X"][:] = 0.0
    assert np.all(oracle.gated(**a) == 0.0)


def test_identity_factors_reduce_to_silu_times_x():
    n = 7
    I = np.eye(n)
    X = np.random.default_rng(3).standard_normal((4, n))
    Z = oracle.gated(X, I, I, I, I, I, I)
    assert relmax(Z, np_silu(X) * X) <= 1e-15


def test_gate_and_up_are_not_interchangeable_and_silu_is_on_gate():
    # gate = identity, up broadcasts x_0: Z = SiLU(X) * x_0 (down = identity); with the roles swapped it would be X * SiLU(x_0).
    n = 5
    I = np.eye(n)
    X = np.random.default_rng(4).standard_normal((3, n))
    Uu = np.zeros((n, n)); Uu[0, 0] = 1.0      # Tu = [x_0, 0, ..., 0]
    Vu = np.zeros((n, n)); Vu[0, :] = 1.0      # P[m, :] = x_0 for every column
    Z = oracle.gated(X, I, I, Uu, Vu, I, I)
    assert relmax(Z, np_silu(X) * X[:, :1]) <= 1e-15


def test_large_positive_gate_is_linear_and_large_negative_vanishes():
    a = _rand_gated(5)
    a["Vg"] = np.abs(a["Vg"]) + 1.0
    a["Ug"] = np.abs(a["Ug"]) + 1.0
    a["X"] = np.abs(a["X"]) * 40 + 40       # G is huge and positive: SiLU(G) -> G
    G = (a["X"] @ a["Ug"]) @ a["Vg"]
    P = (a["X"] @ a["Uu"]) @ a["Vu"]
    assert relmax(oracle.gated(**a), ((G * P) @ a["Ud"]) @ a["Vd"]) <= 1e-12
    a["Vg"] = -a["Vg"]                       # hugely negative gate: H -> 0
    Z = oracle.gated(**a)
    assert np.max(np.abs(Z)) <= 1e-100


def test_linear_in_up_branch_and_in_down_factors():
    a = _rand_gated(6)
    Z = oracle.gated(**a)
    b = dict(a); b["Uu"] = a["Uu"] * 4.0     # power of two: exact scaling
    assert np.array_equal(oracle.gated(**b), Z * 4.0)
    c = dict(a); c["Vd"] = a["Vd"] * 0.5
    assert np.array_equal(oracle.gated(**c), Z * 0.5)


def test_rows_are_independent():
    a = _rand_gated(8, M=6)
    Z = oracle.gated(**a)
    b = dict(a); b["X"] = a["X"][[4, 1]]
    assert np.array_equal(oracle.gated(**b), Z[[4, 1]])


def test_non_square_shapes_catch_transposed_operands():
    # all five extents distinct, so a transposed or mis-strided operand cannot go unnoticed
    a = _rand_gated(9, M=3, d=11, ffn=17, r=5, r2=7)
    assert relmax(oracle.gated(**a), np_dense_mlp(**a)) <= 1e-12
    X, U, V = a["X"], a["Ug"], a["Vg"]
    assert relmax(oracle.linear(X, U, V), X @ U @ V) <= 1e-13


# ------------------------------------------------------------------ numpy float64 chain, mid-size random inputs
@pytest.mark.parametrize("M,d,ffn,r,r2", [(33, 256, 640, 64, 64), (7, 384, 512, 96, 32)])
def test_matches_numpy_chain_on_bf16_valued_inputs(M, d, ffn, r, r2):
    gi = synth.make_gated(M, d, ffn, r, r2, stream=77)
    a = {k: synth.to_f64(v) for k, v in dict(X=gi.X, **gi.factors()).items()}
    H_np = np_silu((a["X"] @ a["Ug"]) @ a["Vg"]) * ((a["X"] @ a["Uu"]) @ a["Vu"])
    Z_np = (H_np @ a["Ud"]) @ a["Vd"]
    Z, H = oracle.gated(**a, return_H=True)
    assert relmax(H, H_np) <= 1e-11
    assert relmax(Z, Z_np) <= 1e-11


# ------------------------------------------------------------------ SiLU values
def test_silu_values_and_identities():
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) <= 1e-16
    for x in (0.3, 1.7, 5.0, 20.0):
        assert abs(oracle.silu(x) - oracle.silu(-x) - x) <= 1e-15 * max(1.0, x)   # x s(x) + x s(-x) = x
        assert oracle.silu(x) > 0 > oracle.silu(-x)
    # minimum of SiLU is about -0.27846 at x ~ -1.27846
    assert abs(oracle.silu(-1.2784645427610738) + 0.2784645427610738) <= 1e-12


def test_argument_validation():
    a = _rand_gated(10)
    with pytest.raises(ValueError):
        oracle.gated(a["X"], a["Ug"], a["Vg"], a["Uu"][:, :-1], a["Vu"], a["Ud"], a["Vd"])
    with pytest.raises(ValueError):
        oracle.linear(a["X"], a["Ug"], a["Vg"][:-1])
    assert oracle.threads() >= 1
