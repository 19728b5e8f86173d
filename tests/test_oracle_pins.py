"""Pins for the fp64 oracle: each test derives its expected value by a route that
does not call the oracle function under test (exact rational scalar orbits, SVD
closed form, pure-Python brute force, symmetries, the singular-value band,
Lemma 1), so a dropped term, a wrong sign, a swapped coefficient or a transposed
operand in the oracle fails at least one of them.  CPU only."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import muon_oracle as orc

A_, B_, C_ = 3.4445, -4.7750, 2.0315


# ----------------------------------------------------------------------------------------------
# independent helpers (no oracle calls)
# ----------------------------------------------------------------------------------------------
def quintic(x, a=A_, b=B_, c=C_):
    return a * x + b * x ** 3 + c * x ** 5


def quintic_n(x, n, a=A_, b=B_, c=C_):
    for _ in range(n):
        x = quintic(x, a, b, c)
    return x


def svd_closed_form(M, n, a=A_, b=B_, c=C_):
    """U f^n(S/||M||_F) V^T: Eq. 2 acts on singular values only (section 2.1, SVD remark)."""
    U, S, Vt = np.linalg.svd(np.asarray(M, dtype=np.float64), full_matrices=False)
    S = S / math.sqrt(float(np.sum(S * S)))
    return (U * quintic_n(S, n, a, b, c)) @ Vt


def load_orbits(golden_dir):
    rows = {}
    with open(os.path.join(golden_dir, "scalar_orbits.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            rows[parts[0]] = [float(p) for p in parts[1:]]
    return rows


def py_matmul(X, Y):
    """Pure-Python triple loop on lists of lists."""
    n, k, m = len(X), len(Y), len(Y[0])
    return [[sum(X[i][t] * Y[t][j] for t in range(k)) for j in range(m)] for i in range(n)]


def py_transpose(X):
    return [list(r) for r in zip(*X)]


def py_muon_step(W, G, M, lr, wd, mu, N, a, b, c, rs, nesterov):
    """The whole step with Python floats and loops, following Eq. 1-4 term by term."""
    R, Cc = len(W), len(W[0])
    Mt = [[mu * M[i][j] + G[i][j] for j in range(Cc)] for i in range(R)]
    U = [[(mu * Mt[i][j] + G[i][j]) if nesterov else Mt[i][j] for j in range(Cc)] for i in range(R)]
    nrm = math.sqrt(sum(u * u for row in U for u in row))
    X = [[u / nrm for u in row] for row in U]
    for _ in range(N):
        XXt = py_matmul(X, py_transpose(X))
        T1 = py_matmul(XXt, X)
        T2 = py_matmul(py_matmul(XXt, XXt), X)
        X = [[a * X[i][j] + b * T1[i][j] + c * T2[i][j] for j in range(Cc)] for i in range(R)]
    s = rs * math.sqrt(max(R, Cc))
    Wn = [[W[i][j] - lr * (s * X[i][j] + wd * W[i][j]) for j in range(Cc)] for i in range(R)]
    return Wn, Mt, X


# ----------------------------------------------------------------------------------------------
# scalar facts about the quintic
# ----------------------------------------------------------------------------------------------
def test_golden_orbits_match_exact_rational_arithmetic(golden_dir):
    a, b, c = Fraction(34445, 10000), Fraction(-4775, 1000), Fraction(20315, 10000)
    for key, vals in load_orbits(golden_dir).items():
        x = Fraction(key)
        for v in vals:
            x = a * x + b * x ** 3 + c * x ** 5
            assert abs(float(x) - v) < 2e-15


def test_coefficients_are_the_papers():
    assert (orc.NS_A, orc.NS_B, orc.NS_C) == (3.4445, -4.7750, 2.0315)
    assert orc.DEFAULT_MU == 0.95 and orc.DEFAULT_NS_STEPS == 5 and orc.DEFAULT_RMS_SCALE == 0.2


def test_quintic_fixed_points_near_one():
    # nonzero fixed points solve c x^4 + b x^2 + (a - 1) = 0
    disc = math.sqrt(B_ * B_ - 4 * C_ * (A_ - 1))
    roots = sorted(math.sqrt((-B_ + s * disc) / (2 * C_)) for s in (-1, 1))
    assert roots == pytest.approx([0.86803, 1.26373], abs=1e-5)
    for r in roots:
        assert quintic(r) == pytest.approx(r, abs=1e-12)


# ----------------------------------------------------------------------------------------------
# newton_schulz against scalar orbits / hand-worked small cases
# ----------------------------------------------------------------------------------------------
def test_diag_3_4_follows_the_scalar_orbits(golden_dir):
    orb = load_orbits(golden_dir)
    for k in range(1, 6):
        O = orc.newton_schulz(np.diag([3.0, 4.0]), steps=k)
        expect = np.diag([orb["3/5"][k - 1], orb["4/5"][k - 1]])
        assert np.max(np.abs(O - expect)) < 1e-13


def test_rank_one_all_ones(golden_dir):
    orb = load_orbits(golden_dir)
    O = orc.newton_schulz(np.ones((2, 2)))
    assert np.max(np.abs(O - orb["1"][4] / 2)) < 1e-13


def test_row_vector_3_4(golden_dir):
    orb = load_orbits(golden_dir)
    O = orc.newton_schulz(np.array([[3.0, 4.0]]))
    assert np.max(np.abs(O - orb["1"][4] * np.array([[0.6, 0.8]]))) < 1e-13
    Ot = orc.newton_schulz(np.array([[3.0], [4.0]]))
    assert np.max(np.abs(Ot - orb["1"][4] * np.array([[0.6], [0.8]]))) < 1e-13


def test_rotation_is_scaled_by_orbit_of_inv_sqrt2():
    th = 0.7
    R = np.array([[math.cos(th), -math.sin(th)], [math.sin(th), math.cos(th)]])
    O = orc.newton_schulz(R)
    assert np.max(np.abs(O - quintic_n(1 / math.sqrt(2), 5) * R)) < 1e-13
    assert quintic_n(1 / math.sqrt(2), 5) == pytest.approx(1.108111115683, abs=1e-11)


def test_upper_triangular_2x2_hand_case():
    # M = [[2,1],[0,1]]: singular values and vectors in closed form.
    M = np.array([[2.0, 1.0], [0.0, 1.0]])
    O = orc.newton_schulz(M)
    expect = np.array([[0.741926967907, 0.172057278921], [-0.397812410065, 0.967682099052]])
    assert np.max(np.abs(O - expect)) < 1e-11
    assert np.max(np.abs(O - svd_closed_form(M, 5))) < 1e-12


@pytest.mark.parametrize("shape", [(3, 5), (5, 3), (8, 8), (16, 64), (64, 16), (1, 7), (7, 1)])
@pytest.mark.parametrize("steps", [0, 1, 2, 5, 10])
def test_svd_closed_form(shape, steps):
    rng = np.random.default_rng(hash((shape, steps)) % 2 ** 32)
    M = rng.standard_normal(shape)
    O = orc.newton_schulz(M, steps=steps)
    assert np.max(np.abs(O - svd_closed_form(M, steps))) < 1e-10


def test_svd_closed_form_other_coefficients():
    rng = np.random.default_rng(5)
    M = rng.standard_normal((6, 9))
    for abc in [(1.5, -0.5, 0.0), (2.0, -1.5, 0.5), (1.0, 0.0, 0.0), (0.0, 0.0, 1.0), (0.0, 1.0, 0.0)]:
        O = orc.newton_schulz(M, steps=3, a=abc[0], b=abc[1], c=abc[2])
        assert np.max(np.abs(O - svd_closed_form(M, 3, *abc))) < 1e-11


def test_iterate_runs_the_formula_on_any_shape_without_transposing():
    # orient=False applies Eq. 2 as printed to a tall matrix; the oriented route must agree
    rng = np.random.default_rng(11)
    M = rng.standard_normal((40, 12))
    assert np.max(np.abs(orc.newton_schulz(M, orient=True) - orc.newton_schulz(M, orient=False))) < 1e-12
    assert np.max(np.abs(orc.newton_schulz(M, orient=False) - svd_closed_form(M, 5))) < 1e-11


def test_ten_steps_is_five_steps_twice_without_renormalising():
    rng = np.random.default_rng(3)
    X0 = orc.frobenius_normalize(rng.standard_normal((10, 20)))
    X5 = orc.newton_schulz_iterate(X0, 5)
    assert np.array_equal(orc.newton_schulz_iterate(X5, 5), orc.newton_schulz_iterate(X0, 10))
    assert np.max(np.abs(orc.newton_schulz_iterate(X0, 10) - svd_closed_form(X0, 10))) < 1e-11


# ----------------------------------------------------------------------------------------------
# invariants
# ----------------------------------------------------------------------------------------------
def test_singular_value_band_after_five_steps():
    # f maps [0, 1.2024] into itself; local max f(0.55453) = 1.202368605, local min f(1.05014) = 0.681831462
    xs = np.linspace(0.0, 1.2024, 200001)
    assert quintic(xs).max() == pytest.approx(1.202368605, abs=2e-9)
    inner = xs[(xs > 0.9) & (xs < 1.2)]
    assert quintic(inner).min() == pytest.approx(0.681831462, abs=2e-9)
    rng = np.random.default_rng(0)
    G = rng.standard_normal((128, 256))
    s0 = np.linalg.svd(orc.frobenius_normalize(G), compute_uv=False)
    assert s0.min() > 0.0015 and s0.max() <= 1.0
    s5 = np.linalg.svd(orc.newton_schulz(G), compute_uv=False)
    assert s5.min() >= 0.68183 - 1e-6 and s5.max() <= 1.20237 + 1e-6
    s10 = np.linalg.svd(orc.newton_schulz(G, steps=10), compute_uv=False)
    assert s10.min() >= 0.68183 - 1e-6 and s10.max() <= 1.20237 + 1e-6


@pytest.mark.parametrize("shape", [(128, 256), (256, 128), (64, 64)])
def test_lemma1_update_rms(shape):
    # ||O||_F^2 = sum sigma_i^2, so RMS(O) sqrt(max(A,B)) = sqrt(mean sigma_i^2) lies in the band,
    # and equals 1 for the exact polar factor (Lemma 1, section 2.2 and appendix A).
    rng = np.random.default_rng(1)
    G = rng.standard_normal(shape)
    O = orc.newton_schulz(G)
    r = orc.update_rms(O) * math.sqrt(max(shape))
    assert 0.68 <= r <= 1.21
    U, _, Vt = np.linalg.svd(G, full_matrices=False)
    assert orc.update_rms(U @ Vt) * math.sqrt(max(shape)) == pytest.approx(1.0, abs=1e-12)
    assert orc.update_rms(O) == pytest.approx(math.sqrt(float(np.mean(O ** 2))), rel=1e-15)


def test_symmetries():
    rng = np.random.default_rng(2)
    M = rng.standard_normal((7, 11))
    O = orc.newton_schulz(M)
    assert np.max(np.abs(orc.newton_schulz(37.5 * M) - O)) < 1e-12          # scale invariance
    assert np.max(np.abs(orc.newton_schulz(-M) + O)) < 1e-14                # odd
    assert np.max(np.abs(orc.newton_schulz(M.T) - O.T)) < 1e-12             # transpose
    Q, _ = np.linalg.qr(rng.standard_normal((7, 7)))
    R, _ = np.linalg.qr(rng.standard_normal((11, 11)))
    assert np.max(np.abs(orc.newton_schulz(Q @ M @ R) - Q @ O @ R)) < 1e-12  # orthogonal equivariance


def test_orthonormal_rows_are_scaled_only():
    rng = np.random.default_rng(4)
    Q, _ = np.linalg.qr(rng.standard_normal((12, 5)))
    M = Q.T  # 5x12, orthonormal rows; every singular value of M/||M||_F is 1/sqrt(5)
    O = orc.newton_schulz(M)
    assert np.max(np.abs(O - quintic_n(1 / math.sqrt(5), 5) * M)) < 1e-12


def test_more_steps_tighten_towards_the_band_not_to_one():
    rng = np.random.default_rng(6)
    G = rng.standard_normal((32, 32))
    for N in (5, 10):
        s = np.linalg.svd(orc.newton_schulz(G, steps=N), compute_uv=False)
        # 32x32 Gaussian has tiny singular values; they only grow (monotone region) or sit in the band
        assert s.max() <= 1.20237 + 1e-6
    s5 = np.linalg.svd(orc.newton_schulz(G, steps=5), compute_uv=False).min()
    s10 = np.linalg.svd(orc.newton_schulz(G, steps=10), compute_uv=False).min()
    assert s10 >= min(s5, 0.68183 - 1e-6)


# ----------------------------------------------------------------------------------------------
# degenerate settings
# ----------------------------------------------------------------------------------------------
def test_zero_steps_and_identity_coefficients_give_normalised_input():
    rng = np.random.default_rng(7)
    U = rng.standard_normal((4, 6))
    expect = U / math.sqrt(sum(float(u) ** 2 for u in U.ravel()))
    assert np.max(np.abs(orc.newton_schulz(U, steps=0) - expect)) < 1e-15
    assert np.max(np.abs(orc.newton_schulz(U, steps=5, a=1.0, b=0.0, c=0.0) - expect)) < 1e-15


def test_eps_and_zero_input():
    Z = np.zeros((3, 4))
    assert np.array_equal(orc.newton_schulz(Z, eps=1e-7), Z)
    U = np.array([[3.0, 4.0]])
    assert np.allclose(orc.frobenius_normalize(U, eps=5.0), U / 10.0, rtol=0, atol=1e-16)
    W = np.array([[1.0, -2.0], [3.0, 4.0]])
    Wn, Mn, On = orc.muon_step(W, np.zeros((2, 2)), np.zeros((2, 2)), lr=0.02, weight_decay=0.1, eps=1e-7)
    assert np.allclose(Wn, W * (1 - 0.02 * 0.1), rtol=0, atol=2e-15)
    assert np.array_equal(Mn, np.zeros((2, 2))) and np.array_equal(On, np.zeros((2, 2)))


def test_elementwise_stages_brute_force():
    rng = np.random.default_rng(8)
    W, G, M = (rng.standard_normal((5, 3)) for _ in range(3))
    Mt = orc.momentum_update(M, G, 0.95)
    Un = orc.ns_input(Mt, G, 0.95, True)
    Up = orc.ns_input(Mt, G, 0.95, False)
    O = rng.standard_normal((5, 3))
    Wn = orc.apply_update(W, O, 0.02, 0.1, 0.2)
    for i in range(5):
        for j in range(3):
            assert Mt[i, j] == 0.95 * M[i, j] + G[i, j]
            assert Un[i, j] == 0.95 * Mt[i, j] + G[i, j]
            assert Up[i, j] == Mt[i, j]
            # decay multiplies W_{t-1} and is not scaled by 0.2 sqrt(max(A,B)); max(5,3) = 5
            assert Wn[i, j] == pytest.approx(W[i, j] - 0.02 * (0.2 * math.sqrt(5.0) * O[i, j] + 0.1 * W[i, j]), rel=1e-15)
    assert np.array_equal(orc.momentum_update(M, G, 0.0), G)


def test_apply_update_degenerate_hyperparameters():
    rng = np.random.default_rng(9)
    W, O = rng.standard_normal((4, 9)), rng.standard_normal((4, 9))
    assert np.array_equal(orc.apply_update(W, O, 0.0, 0.1), W)
    assert np.array_equal(orc.apply_update(W, O, 0.3, 0.0, rms_scale=0.0), W)
    # sqrt(max(A,B)) uses the larger side whichever it is
    d = orc.apply_update(np.zeros((4, 9)), np.ones((4, 9)), 1.0, 0.0)
    dt = orc.apply_update(np.zeros((9, 4)), np.ones((9, 4)), 1.0, 0.0)
    assert np.allclose(d, -0.2 * 3.0) and np.allclose(dt, -0.2 * 3.0)


def test_update_scaling_variants():
    """Eq. 5-7 of section 3.1.  Update Norm makes the RMS of the applied update exactly rms_scale; Baseline equals
    Adjusted LR when max(A, B) = H and differs from it by sqrt(max(A, B) / H) otherwise."""
    rng = np.random.default_rng(14)
    W = rng.standard_normal((6, 24))
    O = rng.standard_normal((6, 24)) * 0.3
    zero = np.zeros_like(W)
    # Update Norm: with lambda = 0, lr = 1 the weight change is the scaled update itself
    d = orc.apply_update(zero, O, 1.0, 0.0, 0.2, "update_norm")
    assert math.sqrt(float(np.mean(d ** 2))) == pytest.approx(0.2, rel=1e-14)
    assert np.max(np.abs(d + 0.2 * O / math.sqrt(float(np.mean(O ** 2))))) < 1e-15
    assert np.array_equal(orc.apply_update(W, zero, 0.5, 0.0, 0.2, "update_norm"), W)        # O = 0: no update, no NaN
    # scale invariance of Update Norm in O
    assert np.max(np.abs(orc.apply_update(W, 7.0 * O, 0.1, 0.01, 0.2, "update_norm") -
                         orc.apply_update(W, O, 0.1, 0.01, 0.2, "update_norm"))) < 1e-14
    # Baseline vs Adjusted LR
    adj = orc.apply_update(zero, O, 1.0, 0.0, 0.2, "adjusted_lr")
    assert np.max(np.abs(orc.apply_update(zero, O, 1.0, 0.0, 0.2, "baseline", hidden_size=24) - adj)) < 1e-15
    base6 = orc.apply_update(zero, O, 1.0, 0.0, 0.2, "baseline", hidden_size=6)
    assert np.max(np.abs(base6 * 2.0 - adj)) < 1e-14                                         # sqrt(24 / 6) = 2
    for i in range(6):
        for j in range(24):
            assert base6[i, j] == pytest.approx(-(0.2 * math.sqrt(6.0) * O[i, j]), rel=1e-15)
    # weight decay is untouched by the mode
    for mode, h in (("adjusted_lr", None), ("baseline", 9.0), ("update_norm", None)):
        assert np.max(np.abs(orc.apply_update(W, zero, 0.5, 0.1, 0.2, mode, h) - W * (1 - 0.05))) < 1e-15
    with pytest.raises(ValueError):
        orc.update_factor(O, (6, 24), 0.2, "nope")
    # for the exact polar factor all three coincide when H = max(A, B) (Lemma 1: RMS = 1/sqrt(max(A, B)))
    U, _, Vt = np.linalg.svd(rng.standard_normal((6, 24)), full_matrices=False)
    P = U @ Vt
    a = orc.apply_update(zero, P, 1.0, 0.0, 0.2, "adjusted_lr")
    assert np.max(np.abs(orc.apply_update(zero, P, 1.0, 0.0, 0.2, "update_norm") - a)) < 1e-14


# ----------------------------------------------------------------------------------------------
# whole step
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("nesterov", [False, True])
@pytest.mark.parametrize("shape", [(3, 4), (4, 3), (2, 2)])
def test_whole_step_against_pure_python_loops(shape, nesterov):
    rng = np.random.default_rng(10)
    W, G, M = (rng.standard_normal(shape) for _ in range(3))
    Wn, Mn, On = orc.muon_step(W, G, M, lr=0.02, weight_decay=0.1, mu=0.95, nesterov=nesterov)
    pw, pm, po = py_muon_step(W.tolist(), G.tolist(), M.tolist(), 0.02, 0.1, 0.95, 5, A_, B_, C_, 0.2, nesterov)
    assert np.max(np.abs(Mn - np.array(pm))) < 1e-15
    assert np.max(np.abs(On - np.array(po))) < 1e-11
    assert np.max(np.abs(Wn - np.array(pw))) < 1e-12


def test_two_step_example_separates_plain_and_nesterov(golden_dir):
    orb = load_orbits(golden_dir)
    W0 = np.array([[1.0, 2.0], [3.0, 4.0]])
    G1 = np.diag([3.0, 4.0])
    G2 = np.array([[1.0, -2.0], [0.5, 1.0]])
    hp = dict(lr=0.02, weight_decay=0.1, mu=0.95)
    sc = 0.2 * math.sqrt(2.0)
    # step 1: M0 = 0, so U is diag(3,4) times 1 (plain) or 1.95 (Nesterov); NS is scale invariant
    O1 = np.diag([orb["3/5"][4], orb["4/5"][4]])
    W1_expect = W0 - 0.02 * (sc * O1 + 0.1 * W0)
    outs = {}
    for nest in (False, True):
        W1, M1, _ = orc.muon_step(W0, G1, np.zeros((2, 2)), nesterov=nest, **hp)
        assert np.max(np.abs(W1 - W1_expect)) < 1e-13
        assert np.array_equal(M1, G1)
        W2, M2, O2 = orc.muon_step(W1, G2, M1, nesterov=nest, **hp)
        assert np.max(np.abs(M2 - np.array([[3.85, -2.0], [0.5, 4.8]]))) < 1e-15
        U = 0.95 * M2 + G2 if nest else M2
        O2_expect = svd_closed_form(U, 5)
        assert np.max(np.abs(O2 - O2_expect)) < 1e-12
        assert np.max(np.abs(W2 - (W1_expect - 0.02 * (sc * O2_expect + 0.1 * W1_expect)))) < 1e-12
        outs[nest] = O2
    assert np.max(np.abs(outs[True] - outs[False])) > 0.1
    assert np.max(np.abs(W1_expect - np.array([[0.993910794874, 1.996], [2.994, 3.985668826493]]))) < 1e-11
    assert np.max(np.abs(outs[False] - np.array([[0.748606320510, -0.435503704403],
                                                  [0.065029846068, 0.983239764122]]))) < 1e-11
    assert np.max(np.abs(outs[True] - np.array([[0.731293973732, -0.403739392268],
                                                 [0.308164396922, 0.760783352638]]))) < 1e-11


def test_inputs_are_widened_exactly_and_not_modified():
    rng = np.random.default_rng(12)
    W = rng.standard_normal((4, 6)).astype(np.float32)
    G = rng.standard_normal((4, 6)).astype(np.float32)
    M = rng.standard_normal((4, 6)).astype(np.float32)
    keep = (W.copy(), G.copy(), M.copy())
    a = orc.muon_step(W, G, M, lr=0.02, weight_decay=0.1)
    b = orc.muon_step(W.astype(np.float64), G.astype(np.float64), M.astype(np.float64), lr=0.02, weight_decay=0.1)
    for x, y in zip(a, b):
        assert x.dtype == np.float64 and np.array_equal(x, y)
    for x, y in zip((W, G, M), keep):
        assert np.array_equal(x, y)


# ----------------------------------------------------------------------------------------------
# the pins have teeth: a planted mistake in a copy of the oracle's iteration fails them
# ----------------------------------------------------------------------------------------------
def _mutants():
    def drop_c(X, a, b, c):
        G = X @ X.T
        return a * X + b * (G @ X)

    def wrong_sign(X, a, b, c):
        G = X @ X.T
        return a * X - b * (G @ X) + c * ((G @ G) @ X)

    def swapped_bc(X, a, b, c):
        G = X @ X.T
        return a * X + c * (G @ X) + b * ((G @ G) @ X)

    def cube_not_square(X, a, b, c):
        G = X @ X.T
        return a * X + b * (G @ X) + c * ((G @ G @ G) @ X)

    return {"drop_c": drop_c, "wrong_sign": wrong_sign, "swapped_bc": swapped_bc, "cube": cube_not_square}


@pytest.mark.parametrize("name", ["drop_c", "wrong_sign", "swapped_bc", "cube"])
def test_planted_mistakes_are_caught_by_the_closed_form(name):
    step = _mutants()[name]
    rng = np.random.default_rng(13)
    M = rng.standard_normal((5, 8))
    X = M / np.linalg.norm(M)
    for _ in range(5):
        X = step(X, A_, B_, C_)
    assert np.max(np.abs(X - svd_closed_form(M, 5))) > 1e-3


# ----------------------------------------------------------------------------------------------
# per-iteration coefficient schedule (extension of Eq. 2: iteration k uses its own triple)
# ----------------------------------------------------------------------------------------------
POLISH = (15.0 / 8.0, -10.0 / 8.0, 3.0 / 8.0)     # textbook order-5 Newton-Schulz polynomial (fixed point exactly 1)
MIXED_SCHEDULE = [(A_, B_, C_), (A_, B_, C_), (A_, B_, C_), POLISH, POLISH]


def svd_closed_form_schedule(M, schedule):
    U, S, Vt = np.linalg.svd(np.asarray(M, dtype=np.float64), full_matrices=False)
    S = S / math.sqrt(float(np.sum(S * S)))
    for a, b, c in schedule:
        S = quintic(S, a, b, c)
    return (U * S) @ Vt


@pytest.mark.parametrize("shape", [(5, 8), (8, 5), (7, 7), (1, 6)])
def test_schedule_matches_composed_scalar_polynomials(shape):
    rng = np.random.default_rng(31)
    M = rng.standard_normal(shape)
    O = orc.newton_schulz(M, steps=len(MIXED_SCHEDULE), schedule=MIXED_SCHEDULE)
    assert np.max(np.abs(O - svd_closed_form_schedule(M, MIXED_SCHEDULE))) < 1e-11
    # the order of the triples matters, and the closed form sees it
    rev = MIXED_SCHEDULE[::-1]
    O_rev = orc.newton_schulz(M, steps=len(rev), schedule=rev)
    assert np.max(np.abs(O_rev - svd_closed_form_schedule(M, rev))) < 1e-11
    assert np.max(np.abs(O_rev - O)) > 1e-4


def test_constant_schedule_is_the_plain_iteration():
    rng = np.random.default_rng(32)
    M = rng.standard_normal((6, 10))
    plain = orc.newton_schulz(M, steps=4)
    assert np.array_equal(orc.newton_schulz(M, steps=4, schedule=[(A_, B_, C_)] * 4), plain)


def test_schedule_position_k_is_used_by_iteration_k():
    """Identity triples (1, 0, 0) everywhere except position j: the result is ONE real step, whichever j."""
    rng = np.random.default_rng(33)
    M = rng.standard_normal((4, 7))
    one = orc.newton_schulz(M, steps=1)
    for j in range(4):
        sched = [(1.0, 0.0, 0.0)] * 4
        sched[j] = (A_, B_, C_)
        assert np.max(np.abs(orc.newton_schulz(M, steps=4, schedule=sched) - one)) < 1e-14
    # two different real steps do not commute with each other's position
    s01 = [(A_, B_, C_), POLISH]
    assert np.max(np.abs(orc.newton_schulz(M, steps=2, schedule=s01) - svd_closed_form_schedule(M, s01))) < 1e-12


def test_polishing_steps_pull_singular_values_to_one():
    """After the paper's five steps the singular values sit in [0.68, 1.21]; the textbook polynomial maps that band
    monotonically towards 1 (p(1) = 1, p'(1) = 0), so a few appended polishing steps give a near-orthogonal O."""
    rng = np.random.default_rng(34)
    M = rng.standard_normal((16, 24))
    sched = [(A_, B_, C_)] * 5 + [POLISH] * 4
    O = orc.newton_schulz(M, steps=len(sched), schedule=sched)
    sv = np.linalg.svd(O, compute_uv=False)
    assert np.max(np.abs(sv - 1.0)) < 1e-6
    assert np.max(np.abs(O @ O.T - np.eye(16))) < 1e-5


def test_schedule_of_wrong_length_is_rejected():
    with pytest.raises(ValueError):
        orc.newton_schulz(np.ones((2, 3)), steps=3, schedule=[(A_, B_, C_)] * 2)


def test_whole_step_with_schedule_uses_it():
    rng = np.random.default_rng(35)
    W, G, M0 = rng.standard_normal((3, 5, 9)) * np.array([0.02, 1e-3, 1e-3])[:, None, None]
    Wt, Mt, O = orc.muon_step(W, G, M0, lr=0.02, weight_decay=0.1, ns_steps=len(MIXED_SCHEDULE), schedule=MIXED_SCHEDULE)
    U = 0.95 * Mt + G
    assert np.max(np.abs(O - svd_closed_form_schedule(U, MIXED_SCHEDULE))) < 1e-11
    assert np.max(np.abs(Wt - (W - 0.02 * (0.2 * math.sqrt(9) * O + 0.1 * W)))) < 1e-15
