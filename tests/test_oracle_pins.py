"""Pins of the fp64 CPU oracle to facts fixed by the paper's equations and by
mathematics, none of which re-run the oracle's own formula: hand-evaluated
tiny cases with textbook sigmoid values, SiLU identities through an
independent library routine (tanh), zero cases, linearity, row independence,
d_ff-permutation and d_ff-split invariances (the tensor-parallel algebra of
Appendix A.1), agreement with an independent dgemm (numpy ``@``) on the
mathematical shapes, and exact bf16 widening.  Each is chosen so that a
dropped term, a wrong sign or index, or a transposed operand fails it.
"""
import math

import numpy as np
import pytest

import dfk_inputs as di
from oracle import oracle

SIG1 = 0.7310585786300049   # Sigmoid(1), textbook value
SIG2 = 0.8807970779778823   # Sigmoid(2), textbook value


def f32(a):
    return np.asarray(a, dtype=np.float32)


# ---------------------------------------------------------------- SiLU pins

def test_silu_zero_and_textbook_values():
    assert oracle.silu(0.0) == 0.0
    assert oracle.silu(1.0) == pytest.approx(SIG1, rel=1e-15)
    assert oracle.silu(2.0) == pytest.approx(2 * SIG2, rel=1e-15)
    assert oracle.silu(-1.0) == pytest.approx(-(1.0 - SIG1), rel=1e-14)


def test_silu_odd_part_identity():
    # Sigmoid(x) + Sigmoid(-x) = 1  =>  SiLU(x) - SiLU(-x) = x
    for x in np.linspace(-30, 30, 241):
        assert oracle.silu(x) - oracle.silu(-x) == pytest.approx(x, abs=1e-13)


def test_silu_matches_tanh_form():
    # Sigmoid(x) = (1 + tanh(x/2)) / 2, through the C library's tanh
    for x in np.linspace(-20, 20, 401):
        assert oracle.silu(x) == pytest.approx(0.5 * x * (1.0 + math.tanh(0.5 * x)),
                                               rel=1e-12, abs=1e-15)


def test_silu_asymptotes_and_extremes():
    assert oracle.silu(40.0) == pytest.approx(40.0, rel=1e-15)
    assert oracle.silu(800.0) == 800.0
    lo = oracle.silu(-800.0)          # exp overflows to +inf; limit is 0 from below
    assert lo == 0.0 and math.copysign(1.0, lo) == -1.0
    assert -1e-15 < oracle.silu(-40.0) < 0.0


def test_silu_single_minimum():
    xs = np.linspace(-6, 2, 800001)
    ys = np.array([oracle.silu(x) for x in xs[::400]])
    # coarse scan then refine around the coarse minimiser
    i = int(np.argmin(ys))
    fine = np.linspace(xs[::400][i - 1], xs[::400][i + 1], 4001)
    fy = np.array([oracle.silu(x) for x in fine])
    xm, ym = fine[int(np.argmin(fy))], float(fy.min())
    assert xm == pytest.approx(-1.278, abs=2e-3)
    assert ym == pytest.approx(-0.278, abs=1e-3)
    # stationarity: Sigmoid(x)(1 + x(1 - Sigmoid(x))) = 0  <=>  SiLU(x*) = 1 + x*
    assert ym == pytest.approx(1.0 + xm, abs=1e-5)
    assert np.all(np.diff(fy[: int(np.argmin(fy))]) <= 0) and np.all(np.diff(fy[int(np.argmin(fy)):]) >= 0)


# ------------------------------------------------- hand-evaluated tiny cases

def test_tiny_2x2_by_hand():
    # x=(1,2); gate columns e1,e2 -> g=(1,2); up columns (1,1),(1,-1) -> u=(3,-1)
    X = f32([[1, 2]])
    Wg = f32([[1, 0], [0, 1]])          # stored [d_ff, d_model]: row j = column j of W_gate
    Wu = f32([[1, 1], [1, -1]])
    Wd = f32([[1, 2], [3, 4]])          # [d_ff, d_model]
    a2 = [3 * SIG1, -1 * 2 * SIG2]
    want = [a2[0] * 1 + a2[1] * 3, a2[0] * 2 + a2[1] * 4]
    Y = oracle.swiglu_mlp(X, Wg, Wu, Wd)
    np.testing.assert_allclose(Y, [want], rtol=1e-14)
    G, U, A2 = oracle.gate_up_silu(X, Wg, Wu)
    np.testing.assert_array_equal(G, [[1, 2]])
    np.testing.assert_array_equal(U, [[3, -1]])
    np.testing.assert_allclose(A2, [a2], rtol=1e-15)


def test_tiny_nonsquare_by_hand_catches_transposes():
    # M=2, d_model=3, d_ff=2: every operand is non-square, so a transposed
    # read of any of them changes the answer or the shape.
    X = f32([[1, 0, 2], [0, -1, 1]])
    Wg = f32([[1, 1, 0], [0, 2, 1]])     # gate column 0 = (1,1,0), column 1 = (0,2,1)
    Wu = f32([[2, 0, 1], [1, 1, 1]])
    Wd = f32([[1, -1, 2], [0, 3, 1]])
    # row 0: g=(1,2) u=(4,3); row 1: g=(-1,-1) u=(1,0)
    sil = {1: SIG1, 2: 2 * SIG2, -1: -(1 - SIG1)}
    a2 = [[4 * sil[1], 3 * sil[2]], [1 * sil[-1], 0.0]]
    wd = [[1.0, -1.0, 2.0], [0.0, 3.0, 1.0]]
    want = [[a2[r][0] * wd[0][n] + a2[r][1] * wd[1][n] for n in range(3)] for r in range(2)]
    Y = oracle.swiglu_mlp(X, Wg, Wu, Wd)
    np.testing.assert_allclose(Y, want, rtol=1e-14, atol=1e-16)
    G, U, _ = oracle.gate_up_silu(X, Wg, Wu)
    np.testing.assert_array_equal(G, [[1, 2], [-1, -1]])
    np.testing.assert_array_equal(U, [[4, 3], [1, 0]])


def test_rank_one_closed_form():
    # d_ff = 1: Y = SiLU(x.w_g) (x.w_u) w_d
    rng = np.random.default_rng(5)
    x, wg, wu, wd = (rng.standard_normal(7).astype(np.float32) for _ in range(4))
    g = float(np.dot(x.astype(np.float64), wg.astype(np.float64)))
    u = float(np.dot(x.astype(np.float64), wu.astype(np.float64)))
    want = 0.5 * g * (1 + math.tanh(0.5 * g)) * u * wd.astype(np.float64)
    Y = oracle.swiglu_mlp(x[None], wg[None], wu[None], wd[None])
    np.testing.assert_allclose(Y[0], want, rtol=1e-12)


# --------------------------------------------------- structural invariants

def _rand(M=3, d=24, ff=40, seed=11, dtype="fp32"):
    return di.mlp_inputs(M, d, ff, seed=seed, dtype=dtype)


def test_zero_cases_are_exact():
    t = _rand()
    z = lambda a: np.zeros_like(a)
    assert not np.any(oracle.swiglu_mlp(z(t["X"]), t["Wg"], t["Wu"], t["Wd"]))
    assert not np.any(oracle.swiglu_mlp(t["X"], z(t["Wg"]), t["Wu"], t["Wd"]))
    assert not np.any(oracle.swiglu_mlp(t["X"], t["Wg"], z(t["Wu"]), t["Wd"]))
    assert not np.any(oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], z(t["Wd"])))
    assert np.any(oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"]))


def test_linear_in_wdown_and_wup_not_in_x_or_wgate():
    t = _rand(seed=21)
    t2 = _rand(seed=22)
    a, b = 2.0, -0.5   # exactly representable scalings keep fp32 inputs exact
    y = lambda X, Wg, Wu, Wd: oracle.swiglu_mlp(f32(X), f32(Wg), f32(Wu), f32(Wd))
    base1, base2 = y(t["X"], t["Wg"], t["Wu"], t["Wd"]), y(t["X"], t["Wg"], t["Wu"], t2["Wd"])
    # general linear combination: quantise both W_down to multiples of 2^-10 so
    # that a*W1 + b*W2 is exactly representable in fp32
    q = lambda w: (np.round(w.astype(np.float64) * 1024.0) / 1024.0).astype(np.float32)
    W1, W2 = q(t["Wd"]), q(t2["Wd"])
    comb = a * W1.astype(np.float64) + b * W2.astype(np.float64)
    assert np.array_equal(comb.astype(np.float32).astype(np.float64), comb)
    np.testing.assert_allclose(
        y(t["X"], t["Wg"], t["Wu"], comb.astype(np.float32)),
        a * y(t["X"], t["Wg"], t["Wu"], W1) + b * y(t["X"], t["Wg"], t["Wu"], W2),
        rtol=1e-11, atol=1e-13)
    # scaling alone is always exact in fp32 for powers of two
    np.testing.assert_allclose(y(t["X"], t["Wg"], t["Wu"], a * t["Wd"]), a * base1, rtol=1e-14)
    np.testing.assert_allclose(y(t["X"], t["Wg"], a * t["Wu"], t["Wd"]), a * base1, rtol=1e-14)
    # additivity in W_up with disjoint supports (exact in fp32)
    Wu_a, Wu_b = t["Wu"].copy(), t["Wu"].copy()
    Wu_a[:, ::2] = 0
    Wu_b[:, 1::2] = 0
    np.testing.assert_allclose(y(t["X"], t["Wg"], Wu_a, t["Wd"]) + y(t["X"], t["Wg"], Wu_b, t["Wd"]),
                               base1, rtol=1e-11, atol=1e-13)
    # additivity in W_down with disjoint supports
    Wd_a, Wd_b = t["Wd"].copy(), t["Wd"].copy()
    Wd_a[::2] = 0
    Wd_b[1::2] = 0
    np.testing.assert_allclose(y(t["X"], t["Wg"], t["Wu"], Wd_a) + y(t["X"], t["Wg"], t["Wu"], Wd_b),
                               base1, rtol=1e-11, atol=1e-13)
    # negative controls: the block is NOT linear in X or in W_gate
    assert not np.allclose(y(a * t["X"], t["Wg"], t["Wu"], t["Wd"]), a * base1, rtol=1e-3)
    assert not np.allclose(y(t["X"], a * t["Wg"], t["Wu"], t["Wd"]), a * base1, rtol=1e-3)


def test_rows_are_independent():
    t = _rand(M=5, seed=31)
    full = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    perm = np.array([3, 0, 4, 1, 2])
    np.testing.assert_array_equal(oracle.swiglu_mlp(t["X"][perm], t["Wg"], t["Wu"], t["Wd"]), full[perm])
    for m in range(5):
        np.testing.assert_array_equal(
            oracle.swiglu_mlp(t["X"][m:m + 1], t["Wg"], t["Wu"], t["Wd"])[0], full[m])


def test_dff_permutation_invariance():
    t = _rand(seed=41)
    perm = np.random.default_rng(0).permutation(t["Wg"].shape[0])
    a = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    b = oracle.swiglu_mlp(t["X"], t["Wg"][perm], t["Wu"][perm], t["Wd"][perm])
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    # permuting only two of the three breaks it
    c = oracle.swiglu_mlp(t["X"], t["Wg"][perm], t["Wu"][perm], t["Wd"])
    assert not np.allclose(a, c, rtol=1e-3)


def test_dff_split_identity():
    # Appendix A.1: W_gate, W_up split by d_ff columns, W_down by d_ff rows;
    # the shards' outputs sum to the unsharded output.
    t = _rand(ff=45, seed=51)
    full = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])
    for bounds in ([0, 45], [0, 7, 45], [0, 1, 16, 17, 45], [0, 11, 22, 33, 45]):
        tot = np.zeros_like(full)
        for lo, hi in zip(bounds[:-1], bounds[1:]):
            tot += oracle.swiglu_mlp(t["X"], t["Wg"][lo:hi], t["Wu"][lo:hi], t["Wd"][lo:hi])
        np.testing.assert_allclose(tot, full, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_against_independent_dgemm_on_math_shapes(dtype):
    # Mathematical shapes: W_gate, W_up in R^{d_model x d_ff}, W_down in
    # R^{d_ff x d_model}; numpy's dgemm is an independent contraction.
    t = di.mlp_inputs(4, 96, 136, seed=61, dtype=dtype)
    X = di.as_f64(t["X"])
    Wgate_math = di.as_f64(t["Wg"]).T      # [d_model, d_ff]
    Wup_math = di.as_f64(t["Wu"]).T
    Wdown_math = di.as_f64(t["Wd"])        # [d_ff, d_model]
    assert Wgate_math.shape == (96, 136) and Wdown_math.shape == (136, 96)
    A_gate = X @ Wgate_math
    A_1 = X @ Wup_math
    A_2 = A_1 * (0.5 * A_gate * (1.0 + np.tanh(0.5 * A_gate)))
    Yn = A_2 @ Wdown_math
    G, U, A2 = oracle.gate_up_silu(t["X"], t["Wg"], t["Wu"])
    np.testing.assert_allclose(G, A_gate, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(U, A_1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(A2, A_2, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"]), Yn,
                               rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(oracle.down(A2, t["Wd"]), Yn, rtol=1e-11, atol=1e-13)


def test_thread_count_does_not_change_a_bit():
    t = di.mlp_inputs(3, 64, 100, seed=71)
    ref = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"], nthreads=1)
    for n in (2, 3, 8, 200):
        np.testing.assert_array_equal(oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"], nthreads=n), ref)


def test_bf16_widening_is_exact():
    # 1.0, -2.0, 0.5, smallest subnormal bf16, +inf is excluded (non-finite)
    bits = np.array([[0x3F80, 0xC000, 0x3F00, 0x0001]], np.uint16)
    want = np.array([1.0, -2.0, 0.5, 2.0 ** -133])
    eye = np.zeros((4, 4), np.uint16)
    for i in range(4):
        eye[i, i] = 0x3F80
    G, U, _ = oracle.gate_up_silu(bits, eye, eye)
    np.testing.assert_array_equal(G[0], want)
    np.testing.assert_array_equal(U[0], want)
    # bf16 and fp32 inputs holding the same values give the same result bit for bit
    t = di.mlp_inputs(2, 32, 48, seed=81, dtype="bf16")
    t32 = {k: di.bf16_bits_to_f32(v) for k, v in t.items()}
    np.testing.assert_array_equal(oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"]),
                                  oracle.swiglu_mlp(t32["X"], t32["Wg"], t32["Wu"], t32["Wd"]))


def test_fp16_widening_is_exact_for_every_finite_pattern():
    # Stage two with A_2 = [[1]] returns the row of W_down widened to fp64: all 63488 finite
    # IEEE half patterns (zeros, subnormals, normals, both signs) against numpy's own conversion,
    # by hand for a few, and through the fp32 route.
    bits = np.arange(65536, dtype=np.uint16)
    finite = bits[(bits & 0x7C00) != 0x7C00]
    row = finite.view(np.float16).reshape(1, -1)
    got = oracle.down(np.ones((1, 1)), row)[0]
    np.testing.assert_array_equal(got, row[0].astype(np.float64))
    hand = np.array([[0x3C00, 0xC000, 0x0001, 0x03FF, 0x0400, 0x7BFF, 0x8000, 0xFBFF]], np.uint16).view(np.float16)
    want = np.array([1.0, -2.0, 2.0 ** -24, 1023 * 2.0 ** -24, 2.0 ** -14, 65504.0, 0.0, -65504.0])
    got = oracle.down(np.ones((1, 1)), hand)[0]
    np.testing.assert_array_equal(got, want)
    t = di.mlp_inputs(2, 32, 48, seed=83, dtype="fp16")
    t32 = {k: v.astype(np.float32) for k, v in t.items()}
    np.testing.assert_array_equal(oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"]),
                                  oracle.swiglu_mlp(t32["X"], t32["Wg"], t32["Wu"], t32["Wd"]))


def test_rejects_mixed_types_and_bad_shapes():
    t = di.mlp_inputs(1, 16, 24, seed=1)
    with pytest.raises(TypeError):
        oracle.swiglu_mlp(t["X"], di.bf16_bits_to_f32(t["Wg"]), t["Wu"], t["Wd"])
    with pytest.raises(ValueError):
        oracle.swiglu_mlp(t["X"], t["Wg"].T.copy(), t["Wu"], t["Wd"])


def test_golden_tiny_config_is_reproduced():
    # stored by tests/golden/make_golden.py (oracle only); guards against drift
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "c1_tiny_y.txt")
    want = np.array([float.fromhex(l) for l in open(path) if not l.startswith("#")])
    t = di.mlp_inputs(1, 512, 1536, seed=0, dtype="bf16")
    got = oracle.swiglu_mlp(t["X"], t["Wg"], t["Wu"], t["Wd"])[0]
    assert want.shape == (512,)
    np.testing.assert_array_equal(got, want)
    assert 0.1 < np.abs(want).max() < 10.0     # well-scaled for the max-normalised metric


# ---- the decoder-layer form around the block: H + MLP(RMSNorm(H; w, eps)) ----

def test_rmsnorm_by_hand_and_closed_forms():
    # 3-4-5: mean square 12.5
    h = np.array([[3.0, 4.0]], np.float32)
    np.testing.assert_allclose(oracle.rmsnorm(h), [[3 / math.sqrt(12.5), 4 / math.sqrt(12.5)]], rtol=1e-15)
    # a constant row normalises to its sign times w; eps shifts the denominator
    c = np.full((1, 8), -2.5, np.float32)
    w = np.arange(1, 9, dtype=np.float32)
    np.testing.assert_allclose(oracle.rmsnorm(c, w), [-w.astype(np.float64)], rtol=1e-15)
    np.testing.assert_allclose(oracle.rmsnorm(c, w, eps=6.25), [-w.astype(np.float64) * 2.5 / math.sqrt(12.5)], rtol=1e-15)
    # zero row stays zero with eps > 0
    np.testing.assert_array_equal(oracle.rmsnorm(np.zeros((2, 4), np.float32), None, eps=1e-6), np.zeros((2, 4)))


def test_rmsnorm_invariants_and_numpy_route():
    t = di.mlp_inputs(5, 96, 8, seed=91, dtype="fp32")
    H = t["X"]
    w = di.tensor(92, (96,), 1.0, "fp32")
    N = oracle.rmsnorm(H, w)
    H64, w64 = H.astype(np.float64), w.astype(np.float64)
    np.testing.assert_allclose(N, H64 * w64 / np.sqrt((H64 ** 2).mean(axis=1, keepdims=True)), rtol=1e-13)
    # unit mean square before the weight; invariance under a positive power-of-two scaling of H
    np.testing.assert_allclose(((N / w64) ** 2).mean(axis=1), np.ones(5), rtol=1e-13)
    np.testing.assert_allclose(oracle.rmsnorm(H * np.float32(4.0), w), N, rtol=1e-14)
    np.testing.assert_allclose(oracle.rmsnorm(-H, w), -N, rtol=1e-15)
    # rows are independent; w = None is w = 1
    np.testing.assert_array_equal(oracle.rmsnorm(H[2:3], w), N[2:3])
    np.testing.assert_array_equal(oracle.rmsnorm(H, None), oracle.rmsnorm(H, np.ones(96, np.float32)))
    # 16-bit inputs are widened exactly
    for dt in ("bf16", "fp16"):
        Hb, wb = di.tensor(93, (3, 40), 1.0, dt), di.tensor(94, (40,), 1.0, dt)
        np.testing.assert_array_equal(oracle.rmsnorm(Hb, wb, 1e-5),
                                      oracle.rmsnorm(di.as_f64(Hb).astype(np.float32), di.as_f64(wb).astype(np.float32), 1e-5))


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_mlp_block_is_residual_plus_block_of_normalised_input(dtype):
    t = di.mlp_inputs(3, 64, 72, seed=95, dtype=dtype)
    w = di.tensor(96, (64,), 1.0, dtype)
    eps = 1e-5
    got = oracle.mlp_block(t["X"], w, eps, t["Wg"], t["Wu"], t["Wd"])
    # composed by hand from the pinned pieces, through numpy's dgemm
    H = di.as_f64(t["X"])
    N = H * di.as_f64(w) / np.sqrt((H ** 2).mean(axis=1, keepdims=True) + eps)
    G, U = N @ di.as_f64(t["Wg"]).T, N @ di.as_f64(t["Wu"]).T
    want = H + (U * G / (1.0 + np.exp(-G))) @ di.as_f64(t["Wd"])
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)
    # W_down = 0: the residual alone, exactly; w = 1, huge H: the block sees unit-scale input
    zero = np.zeros_like(t["Wd"])
    np.testing.assert_array_equal(oracle.mlp_block(t["X"], w, eps, t["Wg"], t["Wu"], zero), H)
    # the normalised input is scale-free: H and 2H differ in the output only by the residual
    if dtype == "fp32":
        a = oracle.mlp_block(t["X"], w, 0.0, t["Wg"], t["Wu"], t["Wd"]) - H
        b = oracle.mlp_block(t["X"] * np.float32(2), w, 0.0, t["Wg"], t["Wu"], t["Wd"]) - 2 * H
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
    # thread count does not change a bit
    np.testing.assert_array_equal(oracle.mlp_block(t["X"], w, eps, t["Wg"], t["Wu"], t["Wd"], nthreads=1),
                                  oracle.mlp_block(t["X"], w, eps, t["Wg"], t["Wu"], t["Wd"], nthreads=5))
