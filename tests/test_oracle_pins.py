"""Pins for the CPU oracle: each routine is checked against something other than
itself -- a hand-derived worked example, closed forms, invariants of the
equations, numpy/LAPACK routines on the special cases they cover, and brute
force on tiny inputs.  No GPU needed.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _problem(r, d, n, seed, w_std=0.05):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((r, d)) * w_std).astype(np.float32)
    X = np.maximum(rng.standard_normal((d, n)), 0).astype(np.float32)
    return W, X


def _golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = np.array([float(x) for x in v])
    return out


# ---------------------------------------------------------------- Hessian
def test_hessian_hand_case():
    # X = [[1,2],[3,4]]: X X^T = [[5,11],[11,25]], times 2/N with N = 2.
    X = np.array([[1, 2], [3, 4]], dtype=np.float32)
    assert np.array_equal(oracle.hessian(X), np.array([[5.0, 11.0], [11.0, 25.0]]))


def test_hessian_matches_blas_and_is_symmetric():
    _, X = _problem(1, 37, 301, 1)
    H = oracle.hessian(X)
    Xd = X.astype(np.float64)
    ref = 2.0 * (Xd @ Xd.T) / X.shape[1]
    assert np.allclose(H, ref, rtol=1e-13, atol=0)
    assert np.array_equal(H, H.T)


def test_hessian_is_the_hessian_of_the_layer_objective():
    # second difference of E(w) = (1/N)|wX - w0X|^2 along e_a, e_b equals H_ab
    _, X = _problem(1, 5, 40, 2)
    H = oracle.hessian(X)
    Xd = X.astype(np.float64)
    E = lambda w: np.sum((w @ Xd) ** 2) / X.shape[1]
    eye = np.eye(5)
    for a, b in [(0, 0), (1, 3), (4, 2)]:
        fd = (E(eye[a] + eye[b]) - E(eye[a]) - E(eye[b]) + E(0 * eye[a]))
        assert np.isclose(fd, H[a, b], rtol=1e-12)


def test_damp_closed_form():
    H = np.diag([1.0, 2.0, 6.0]) + 0.1
    Hd, lam = oracle.damp(H, 0.01, 0.25)
    assert np.isclose(lam, 0.01 * (1.1 + 2.1 + 6.1) / 3 + 0.25, rtol=1e-15)
    assert np.allclose(Hd - H, lam * np.eye(3), rtol=0, atol=1e-15)


# ---------------------------------------------------------------- inverse
def test_spd_inverse_identity_and_lapack():
    _, X = _problem(1, 48, 96, 3)
    Hd, _ = oracle.damp(oracle.hessian(X), 0.01)
    Hinv = oracle.spd_inverse(Hd)
    assert np.allclose(Hd @ Hinv, np.eye(48), atol=1e-10)
    assert np.allclose(Hinv, np.linalg.inv(Hd), rtol=1e-9, atol=1e-12)
    assert np.array_equal(Hinv, Hinv.T)


def test_spd_inverse_2x2_closed_form():
    Hinv = oracle.spd_inverse(np.array([[2.0, 1.0], [1.0, 2.0]]))
    assert np.allclose(Hinv, np.array([[2.0, -1.0], [-1.0, 2.0]]) / 3.0, rtol=1e-15)


def test_spd_inverse_rejects_non_pd():
    _, X = _problem(1, 16, 8, 4)            # N < d: singular without damping
    with pytest.raises(oracle.OracleError) as e:
        oracle.spd_inverse(oracle.hessian(X))
    assert e.value.code == oracle.ENOTPD
    with pytest.raises(oracle.OracleError):
        oracle.spd_inverse(np.array([[1.0, 2.0], [2.0, 1.0]]))


# ---------------------------------------------------------------- grid
def test_grid_hand_cases():
    W = np.array([[-1.0, 0.5, 2.0, 0.0],      # lo -1 hi 2, maxq 3 -> scale 1 zero 1
                  [0.25, 0.5, 1.5, 1.0],      # all positive: range widened to [0, 1.5]
                  [-3.0, -1.0, -2.0, -0.5],   # all negative: [-3, 0]
                  [0.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    s, z = oracle.grid(W, 2, 0)
    assert np.allclose(s[:, 0], [1.0, 0.5, 1.0, 1.0], rtol=1e-15)
    assert np.array_equal(z[:, 0], [1.0, 0.0, 3.0, 0.0])


def test_grid_groups_use_original_columns():
    W = np.array([[-1.0, 2.0, -4.0, 8.0]], dtype=np.float32)
    s, z = oracle.grid(W, 4, 2)
    assert s.shape == (1, 2)
    assert np.allclose(s[0], [3.0 / 15, 12.0 / 15], rtol=1e-15)
    assert np.array_equal(z[0], [5.0, 5.0])


def test_row_extremes_get_end_codes_and_rtn_error_bound():
    W, X = _problem(7, 24, 64, 5)
    # diagonal H: no compensation -> plain round-to-nearest on the grid
    H = np.diag(np.linspace(1.0, 3.0, 24))
    res = oracle.quantize_layer(W, H=H, bits=3, damp_rel=0.0)
    s = res.scales[:, :1]
    assert np.all(np.abs(res.Q - W) <= s / 2 * (1 + 1e-12))
    lo = np.minimum(W.min(1), 0)
    hi = np.maximum(W.max(1), 0)
    for i in range(7):
        if W[i].min() <= 0:
            assert res.codes[i, np.argmin(W[i])] == 0
        assert res.codes[i, np.argmax(W[i])] == 7
        assert res.codes[i].min() >= 0 and res.codes[i].max() <= 7
    # and it equals the textbook affine quantizer evaluated independently in numpy
    Wd = W.astype(np.float64)
    sc = (hi - lo)[:, None] / 7
    zp = np.rint(-lo[:, None] / sc)
    ref_codes = np.clip(np.rint(Wd / sc) + zp, 0, 7)
    assert np.array_equal(res.codes, ref_codes.astype(np.int64))
    assert np.allclose(res.Q, sc * (ref_codes - zp), rtol=1e-15)


def test_diagonal_h_result_is_independent_of_order():
    W, _ = _problem(5, 12, 1, 6)
    H = np.diag(np.linspace(0.5, 2.0, 12))
    a = oracle.quantize_layer(W, H=H, bits=4, damp_rel=0.0, order_mode=oracle.ORDER_NATURAL)
    b = oracle.quantize_layer(W, H=H, bits=4, damp_rel=0.0, order_mode=oracle.ORDER_SENSI_DESC)
    assert np.array_equal(a.codes, b.codes)


# ---------------------------------------------------------------- sensitivity, order
def test_sensitivity_hand_case():
    # one row [0.3, 0.7], 2 bits: scale 7/30, quant -> [7/30, 0.7]; Hinv diag [2/3, 2/3]
    W = np.array([[0.3, 0.7]], dtype=np.float32)
    s, z = oracle.grid(W, 2, 0)
    S = oracle.sensitivity(W, np.array([2 / 3, 2 / 3]), 2, 0, s, z)
    assert np.allclose(S, [(1 / 15) ** 2 / (4 / 3), 0.0], rtol=1e-6, atol=1e-14)


def test_sensitivity_sums_rows_and_divides_by_own_column_diag():
    W, X = _problem(9, 10, 50, 7)
    s, z = oracle.grid(W, 4, 0)
    hd = np.linspace(0.5, 5.0, 10)
    S = oracle.sensitivity(W, hd, 4, 0, s, z)
    Wd = W.astype(np.float64)
    q = s * (np.clip(np.rint(Wd / s) + z, 0, 15) - z)
    assert np.allclose(S, ((q - Wd) ** 2).sum(0) / (2 * hd), rtol=1e-13)


def test_order_is_stable_descending():
    S = np.array([1.0, 3.0, 2.0, 3.0, 0.5, 2.0])
    assert list(oracle.order(S)) == [1, 3, 2, 5, 0, 4]
    rng = np.random.default_rng(8)
    S = rng.random(200)
    assert np.array_equal(oracle.order(S), np.argsort(-S, kind="stable"))


# ---------------------------------------------------------------- worked example (golden file)
def test_worked_example_d2():
    g = _golden("d2_worked_example.txt")
    W = np.array([[0.3, 0.7]], dtype=np.float32)
    H = np.array([[2.0, 1.0], [1.0, 2.0]])
    full = oracle.quantize_layer(W, H=H, bits=2, damp_rel=0.0, order_mode=oracle.ORDER_NATURAL)
    assert np.allclose(full.scales[0, 0], g["scale"][0], rtol=1e-7)
    assert full.zeros[0, 0] == g["zero"][0]
    assert np.array_equal(full.codes[0], g["codes"].astype(np.int64))
    assert np.allclose(full.Q[0], g["q"], rtol=1e-7)
    assert np.isclose(full.loss, g["loss"][0], rtol=1e-6)
    one = oracle.quantize_layer(W, H=H, bits=2, damp_rel=0.0, order_mode=oracle.ORDER_NATURAL, steps=1)
    assert np.isclose(one.W_work[0, 1], g["w1_after_step0"][0], rtol=1e-7)
    assert np.isclose(one.Hinv_work[1, 1], g["hinv11_after_step0"][0], rtol=1e-14)


def test_d2_closed_form_compensation():
    # quantizing a first moves b by (w_a - q_a) H_ab / H_bb  (minimiser of the 2-variable quadratic)
    rng = np.random.default_rng(9)
    for _ in range(5):
        A = rng.standard_normal((2, 2))
        H = A @ A.T + 0.5 * np.eye(2)
        W = rng.standard_normal((3, 2)).astype(np.float32)
        res = oracle.quantize_layer(W, H=H, bits=3, damp_rel=0.0, order_mode=oracle.ORDER_NATURAL, steps=1)
        Wd = W.astype(np.float64)
        expect = Wd[:, 1] + (Wd[:, 0] - res.Q[:, 0]) * H[0, 1] / H[1, 1]
        assert np.allclose(res.W_work[:, 1], expect, rtol=1e-12)


# ---------------------------------------------------------------- Eq. 12: the shared inverse
@pytest.mark.parametrize("mode", [oracle.ORDER_NATURAL, oracle.ORDER_SENSI_DESC])
def test_eliminated_hinv_is_inverse_of_remaining_block(mode):
    W, X = _problem(6, 14, 40, 10)
    for t in [0, 1, 5, 13]:
        res = oracle.quantize_layer(W, X=X, bits=4, order_mode=mode, steps=t)
        rem = np.array(sorted(set(range(14)) - set(res.perm[:t].tolist())))
        direct = np.linalg.inv(res.H_damped[np.ix_(rem, rem)])
        assert np.allclose(res.Hinv_work[np.ix_(rem, rem)], direct, rtol=1e-9, atol=1e-12)
        gone = res.perm[:t]
        assert np.all(res.Hinv_work[gone, :] == 0) and np.all(res.Hinv_work[:, gone] == 0)


def test_pivot_rows_are_the_cholesky_factor_of_permuted_hinv():
    # rows used by successive eliminations = diag(U) * U with Hinv[perm][:,perm] = U^T U (LAPACK potrf)
    W, X = _problem(4, 10, 30, 11)
    full = oracle.quantize_layer(W, X=X, bits=4)
    p = full.perm
    U = np.linalg.cholesky(full.Hinv[np.ix_(p, p)]).T
    for t in range(10):
        snap = oracle.quantize_layer(W, X=X, bits=4, steps=t)
        row = snap.Hinv_work[p[t], p[t:]]
        assert np.allclose(row, U[t, t] * U[t, t:], rtol=1e-9, atol=1e-13)


# ---------------------------------------------------------------- Eq. 9 / 11: compensation
@pytest.mark.parametrize("group", [0, 4])
def test_compensated_weights_solve_the_constrained_least_squares(group):
    r, d, n = 5, 12, 60
    W, X = _problem(r, d, n, 12)
    for t in [1, 4, 11]:
        res = oracle.quantize_layer(W, X=X, bits=3, group=group, steps=t)
        done = res.perm[:t]
        rem = np.array([j for j in range(d) if j not in set(done.tolist())])
        Hd = res.H_damped
        Wd = W.astype(np.float64)
        # minimise (w - w0) Hd (w - w0)^T with w[done] = q[done]
        delta_done = res.Q[:, done] - Wd[:, done]
        expect = Wd[:, rem] - delta_done @ Hd[np.ix_(done, rem)] @ np.linalg.inv(Hd[np.ix_(rem, rem)])
        assert np.allclose(res.W_work[:, rem], expect, rtol=1e-8, atol=1e-12)
        # same thing as an ordinary least-squares fit of the layer output (+ the damping rows)
        A = np.vstack([np.sqrt(2.0 / n) * X.astype(np.float64).T, np.sqrt(res.lam) * np.eye(d)])
        for i in range(r):
            target = A @ Wd[i] - A[:, done] @ res.Q[i, done]
            sol, *_ = np.linalg.lstsq(A[:, rem], target, rcond=None)
            assert np.allclose(res.W_work[i, rem], sol, rtol=1e-7, atol=1e-10)


def test_greedy_step_is_the_constrained_minimiser_tiny():
    # d = 5: after one step, no other change of the free weights has a lower 1/2 dw^T H dw
    W, X = _problem(1, 5, 30, 13)
    res = oracle.quantize_layer(W, X=X, bits=2, steps=1)
    j = res.perm[0]
    Hd = res.H_damped
    w0 = W[0].astype(np.float64)
    dw = res.W_work[0] - w0
    dw[j] = res.Q[0, j] - w0[j]
    best = 0.5 * dw @ Hd @ dw
    free = [k for k in range(5) if k != j]
    for step in [1e-2, 1e-4]:
        for signs in itertools.product([-1, 0, 1], repeat=4):
            trial = dw.copy()
            trial[free] += step * np.array(signs)
            assert 0.5 * trial @ Hd @ trial >= best * (1 - 1e-12)
    # and the loss the oracle books for the step is that minimum (Eq. 10)
    assert np.isclose(res.loss, best, rtol=1e-10)


# ---------------------------------------------------------------- loss identities
@pytest.mark.parametrize("bits,group", [(4, 0), (3, 8), (8, 0)])
def test_loss_telescopes_to_half_trace_and_to_output_error(bits, group):
    r, d, n = 8, 16, 80
    W, X = _problem(r, d, n, 14)
    res = oracle.quantize_layer(W, X=X, bits=bits, group=group)
    dW = W.astype(np.float64) - res.Q
    half_trace = 0.5 * np.trace(dW @ res.H_damped @ dW.T)
    assert np.isclose(res.loss, half_trace, rtol=1e-9)
    out_err = np.sum((dW @ X.astype(np.float64)) ** 2) / n
    assert np.isclose(res.loss, out_err + 0.5 * res.lam * np.sum(dW ** 2), rtol=1e-9)
    # the oracle's own evaluators agree with the numpy expressions
    assert np.isclose(oracle.loss_eval(W, res.Q, res.H_damped), half_trace, rtol=1e-12)
    assert np.isclose(oracle.output_error(W, res.Q, X), out_err, rtol=1e-12)


def test_high_bit_limit_q_equals_w():
    W, X = _problem(6, 20, 100, 15)
    for bits in [24, 30]:
        res = oracle.quantize_layer(W, X=X, bits=bits)
        rng_ = (np.maximum(W.max(1), 0) - np.minimum(W.min(1), 0)).astype(np.float64)
        assert np.max(np.abs(res.Q - W) / rng_[:, None]) < 2.0 ** (-bits + 1)
        assert res.loss < 1e-10


# ---------------------------------------------------------------- ordering symmetries
def test_permutation_equivariance():
    W, X = _problem(5, 11, 50, 16)
    rng = np.random.default_rng(17)
    P = rng.permutation(11).astype(np.int32)
    H = oracle.hessian(X)
    a = oracle.quantize_layer(W, H=H, bits=4, order_mode=oracle.ORDER_CUSTOM, perm=P)
    Wp = np.ascontiguousarray(W[:, P])
    Hp = np.ascontiguousarray(H[np.ix_(P, P)])
    b = oracle.quantize_layer(Wp, H=Hp, bits=4, order_mode=oracle.ORDER_NATURAL)
    assert np.array_equal(a.codes[:, P], b.codes)
    assert np.allclose(a.Q[:, P], b.Q, rtol=1e-12)
    assert np.isclose(a.loss, b.loss, rtol=1e-10)


def test_scaling_h_changes_only_the_loss():
    W, X = _problem(5, 11, 50, 18)
    H = oracle.hessian(X)
    a = oracle.quantize_layer(W, H=H, bits=4)
    b = oracle.quantize_layer(W, H=8.0 * H, bits=4)      # power of two: exact
    assert np.array_equal(a.perm, b.perm)
    assert np.array_equal(a.codes, b.codes)
    assert np.isclose(b.loss, 8.0 * a.loss, rtol=1e-12)


def test_sensi_order_puts_most_sensitive_column_first():
    W, X = _problem(5, 11, 50, 19)
    res = oracle.quantize_layer(W, X=X, bits=4)
    assert res.perm[0] == np.argmax(res.S)
    assert np.all(np.diff(res.S[res.perm]) <= 0)


def test_column_loop_rejects_bad_perm():
    W, X = _problem(2, 4, 10, 20)
    with pytest.raises(oracle.OracleError):
        oracle.quantize_layer(W, X=X, bits=4, order_mode=oracle.ORDER_CUSTOM,
                              perm=np.array([0, 1, 1, 2], dtype=np.int32))


# ---------------------------------------------------------------- other sort keys (Section 4.1, Table 3)
def test_column_keys_against_numpy():
    W, X = _problem(9, 13, 60, 21)
    s, z = oracle.grid(W, 3, 0)
    hd = np.linspace(0.5, 4.0, 13)
    Wd = W.astype(np.float64)
    q = s * (np.clip(np.rint(Wd / s) + z, 0, 7) - z)
    err = ((q - Wd) ** 2).sum(0)
    assert np.allclose(oracle.column_key(W, hd, 3, 0, s, z, oracle.KEY_ERR), err, rtol=1e-13)
    assert np.allclose(oracle.column_key(W, hd, 3, 0, s, z, oracle.KEY_W), (Wd ** 2).sum(0), rtol=1e-13)
    assert np.allclose(oracle.column_key(W, hd, 3, 0, s, z, oracle.KEY_SENSI), err / (2 * hd), rtol=1e-13)


def test_order_directions_are_stable():
    S = np.array([1.0, 3.0, 2.0, 3.0, 0.5, 2.0])
    assert list(oracle.order(S, ascending=True)) == [4, 0, 2, 5, 1, 3]
    assert list(oracle.order(S, ascending=False)) == [1, 3, 2, 5, 0, 4]
    rng = np.random.default_rng(22)
    S = rng.integers(0, 5, 300).astype(np.float64)          # many ties
    assert np.array_equal(oracle.order(S, True), np.argsort(S, kind="stable"))
    assert np.array_equal(oracle.order(S, False), np.argsort(-S, kind="stable"))


@pytest.mark.parametrize("mode", [oracle.ORDER_ERR_DESC, oracle.ORDER_W_DESC, oracle.ORDER_SENSI_ASC,
                                  oracle.ORDER_ERR_ASC, oracle.ORDER_W_ASC])
def test_every_order_is_the_custom_order_of_its_own_permutation(mode):
    W, X = _problem(6, 15, 70, 23)
    H = oracle.hessian(X)
    a = oracle.quantize_layer(W, H=H, bits=4, order_mode=mode)
    kind, asc = oracle._ORDER_KEYS[mode]
    key = oracle.column_key(W, np.diag(a.Hinv).copy(), 4, 0, a.scales, a.zeros, kind)
    expect = np.argsort(key if asc else -key, kind="stable").astype(np.int32)
    assert np.array_equal(a.perm, expect)
    b = oracle.quantize_layer(W, H=H, bits=4, order_mode=oracle.ORDER_CUSTOM, perm=expect)
    assert np.array_equal(a.codes, b.codes) and np.isclose(a.loss, b.loss, rtol=1e-12)
    # the loss identity holds for any order
    dW = W.astype(np.float64) - a.Q
    assert np.isclose(a.loss, 0.5 * np.trace(dW @ a.H_damped @ dW.T), rtol=1e-9)


# ---------------------------------------------------------------- dynamic order (Section 5: sorting repeated per column)
def test_dynamic_order_is_the_custom_order_of_its_own_permutation():
    W, X = _problem(7, 14, 80, 24)
    a = oracle.quantize_layer(W, X=X, bits=3, order_mode=oracle.ORDER_SENSI_DYNAMIC)
    assert sorted(a.perm) == list(range(14))
    b = oracle.quantize_layer(W, X=X, bits=3, order_mode=oracle.ORDER_CUSTOM, perm=a.perm)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.Q, b.Q) and a.loss == b.loss
    # first choice = largest initial score = first column of the static order
    assert a.perm[0] == oracle.quantize_layer(W, X=X, bits=3).perm[0]


@pytest.mark.parametrize("group", [0, 3])
def test_dynamic_order_takes_the_column_with_the_largest_loss_term(group):
    """Eq. 10 is the loss a column incurs when it is quantized now.  At every step, processing any
    other remaining column next would add a smaller (or equal) term to the loss: checked through the
    loss accumulated by the static loop run on each alternative order (an independent route to the
    same number: the loop's own (w - q)^2 / (2 Hinv_tt), not the score routine)."""
    d = 6
    W, X = _problem(5, d, 40, 25)
    H = oracle.hessian(X)
    a = oracle.quantize_layer(W, H=H, bits=3, group=group, order_mode=oracle.ORDER_SENSI_DYNAMIC)
    for t in range(d):
        done = list(a.perm[:t])
        before = oracle.quantize_layer(W, H=H, bits=3, group=group, order_mode=oracle.ORDER_CUSTOM,
                                       perm=a.perm, steps=t).loss if t else 0.0
        gains = {}
        for cand in range(d):
            if cand in done:
                continue
            rest = [k for k in range(d) if k not in done and k != cand]
            p = np.array(done + [cand] + rest, dtype=np.int32)
            gains[cand] = oracle.quantize_layer(W, H=H, bits=3, group=group, order_mode=oracle.ORDER_CUSTOM,
                                                perm=p, steps=t + 1).loss - before
        best = max(gains.values())
        assert gains[int(a.perm[t])] >= best * (1 - 1e-9)
        # and the choice is strict here (no ties in this problem), so it is the unique argmax
        assert int(a.perm[t]) == max(gains, key=gains.get)


def test_dynamic_order_equals_static_order_without_compensation():
    # X with orthogonal rows: H diagonal, no compensation, the diagonal of Hinv never changes,
    # so the scores of the remaining columns never change either.
    rng = np.random.default_rng(26)
    d = 9
    Qm, _ = np.linalg.qr(rng.standard_normal((32, d)))
    X = (Qm.T * np.linspace(1.0, 3.0, d)[:, None]).astype(np.float32)
    W = (rng.standard_normal((6, d)) * 0.1).astype(np.float32)
    H = np.diag(np.diag(oracle.hessian(X)))            # exactly diagonal
    a = oracle.quantize_layer(W, H=H, bits=4, order_mode=oracle.ORDER_SENSI_DYNAMIC)
    b = oracle.quantize_layer(W, H=H, bits=4, order_mode=oracle.ORDER_SENSI_DESC)
    assert np.array_equal(a.perm, b.perm) and np.array_equal(a.codes, b.codes)


def test_dynamic_order_breaks_ties_by_index_and_honours_steps():
    # two identical columns with identical statistics: the smaller index goes first
    rng = np.random.default_rng(27)
    W = (rng.standard_normal((4, 5)) * 0.1).astype(np.float32)
    W[:, 3] = W[:, 1]
    H = np.eye(5) * 2.0
    a = oracle.quantize_layer(W, H=H, bits=2, damp_rel=0.0, order_mode=oracle.ORDER_SENSI_DYNAMIC)
    assert list(a.perm).index(1) + 1 == list(a.perm).index(3)
    part = oracle.quantize_layer(W, H=H, bits=2, damp_rel=0.0, order_mode=oracle.ORDER_SENSI_DYNAMIC, steps=2)
    assert np.array_equal(part.perm[:2], a.perm[:2])
    assert sorted(part.perm) == list(range(5)) and list(part.perm[2:]) == sorted(part.perm[2:])
    assert np.all(part.Q[:, part.perm[2:]] == 0.0)


# ---------------------------------------------------------------- per-row OBQ baseline (Section 4.2, first paragraphs)
def test_obq_row_is_the_shared_loop_on_that_row_with_the_rows_own_order():
    """Rows never interact, so OBQ on row i must equal the (pinned) shared-inverse loop run on the
    single row i with the order OBQ chose for it: same codes, same values, same loss."""
    W, X = _problem(5, 12, 70, 31)
    base = oracle.quantize_layer(W, X=X, bits=3, group=4)
    o = oracle.obq_rows(W, base.Hinv, 3, 4, base.scales, base.zeros)
    for i in range(5):
        assert sorted(o.order[i]) == list(range(12))
        one = oracle.column_loop(W[i:i + 1], base.Hinv, o.order[i], 3, 4, base.scales[i:i + 1], base.zeros[i:i + 1])
        assert np.array_equal(o.codes[i], one.codes[0])
        assert np.array_equal(o.Q[i], one.Q[0])
        assert np.isclose(o.lossrow[i], one.loss, rtol=1e-13)
    # the loss identity holds per row whatever the order
    dW = W.astype(np.float64) - o.Q
    assert np.allclose(o.lossrow, 0.5 * np.einsum("ij,jk,ik->i", dW, base.H_damped, dW), rtol=1e-9)


def test_obq_takes_the_weight_with_the_smallest_loss_term():
    d = 6
    W, X = _problem(2, d, 40, 32)
    base = oracle.quantize_layer(W, X=X, bits=3)
    o = oracle.obq_rows(W, base.Hinv, 3, 0, base.scales, base.zeros)
    i = 1
    for t in range(d):
        done = list(o.order[i][:t])
        before = oracle.column_loop(W[i:i + 1], base.Hinv, o.order[i], 3, 0, base.scales[i:i + 1],
                                    base.zeros[i:i + 1], steps=t).loss if t else 0.0
        gains = {}
        for cand in range(d):
            if cand in done:
                continue
            rest = [k for k in range(d) if k not in done and k != cand]
            p = np.array(done + [cand] + rest, dtype=np.int32)
            gains[cand] = oracle.column_loop(W[i:i + 1], base.Hinv, p, 3, 0, base.scales[i:i + 1],
                                             base.zeros[i:i + 1], steps=t + 1).loss - before
        assert int(o.order[i][t]) == min(gains, key=gains.get)


def test_obq_row_range_and_diagonal_case():
    rng = np.random.default_rng(33)
    W = (rng.standard_normal((4, 7)) * 0.1).astype(np.float32)
    H = np.diag(np.linspace(1.0, 2.0, 7))
    base = oracle.quantize_layer(W, H=H, bits=4, damp_rel=0.0)
    part = oracle.obq_rows(W, base.Hinv, 4, 0, base.scales, base.zeros, rows=(1, 3))
    full = oracle.obq_rows(W, base.Hinv, 4, 0, base.scales, base.zeros)
    assert np.array_equal(part.codes[1:3], full.codes[1:3]) and np.all(part.codes[[0, 3]] == 0)
    # diagonal H: no compensation, every order gives plain round-to-nearest
    assert np.array_equal(full.codes, base.codes)
