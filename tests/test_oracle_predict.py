"""Pins for the oracle's query predictor (Sec. 4.2, Eq. 2-5; Alg. 1 steps 1-6).

The paper prints no worked example, so the pins are closed forms and invariants that
follow from the equations, plus numpy.linalg.solve as a library special case.
"""
import numpy as np
import pytest
import torch

import oracle


def bf(x):
    return torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)


def f64(t):
    return t.to(torch.float64).numpy()


def softmax(x):
    e = np.exp(x - np.max(x))
    return e / e.sum()


def run(q_win, q_cur, eps, beta=1.0, weights=False):
    """q_win [W, D], q_cur [D] (array-likes) -> q_hat [D] fp32 numpy (and weights [W, W])."""
    qw = bf(q_win)[None, None]
    qc = bf(q_cur)[None, None]
    if weights:
        qh, w = oracle.predict_query(qw, qc, eps, beta, return_weights=True)
        return qh[0, 0].numpy(), w[0, 0].numpy()
    return oracle.predict_query(qw, qc, eps, beta)[0, 0].numpy()


def test_window_one_returns_current_query():
    # k = 1 has a single softmax weight equal to 1, applied to Q_t (Eq. 4 with i = 1).
    rng = np.random.default_rng(0)
    D = 128
    cur = rng.standard_normal(D)
    prev = rng.standard_normal((1, D))
    for eps in (1e-4, 1e-2, 10.0):
        for beta in (1.0, -1.0):
            got = run(prev, cur, eps, beta)
            assert np.array_equal(got, bf(cur).float().numpy())


@pytest.mark.parametrize("beta", [1.0, -1.0])
def test_orthogonal_window_closed_form(beta):
    # R_i = alpha_i e_i (i = 1 newest), T = sum_i gamma_i e_i  =>  the Gram matrix is
    # diagonal and omega_i = alpha_i gamma_i / (alpha_i^2 + eps) for every window size.
    W, D, eps = 4, 8, 0.5
    alpha = np.array([2.0, 1.0, -1.5, 0.5])
    gamma = np.array([1.0, -0.5, 2.0, 0.25])
    q_win = np.zeros((W, D))
    for i in range(1, W + 1):
        q_win[W - i, i - 1] = alpha[i - 1]          # oldest first in memory
    T = np.zeros(D)
    T[:W] = gamma
    T[W] = 3.0                                       # a component only Q_t has
    omega = alpha * gamma / (alpha ** 2 + eps)
    # expected prediction: (1/W) sum_k sum_{i<=k} softmax(beta*omega_{1..k})_i * Q_{t+1-i}
    shifted = [T] + [q_win[W - i] for i in range(1, W)]       # Q_t, Q_{t-1}, ..., Q_{t-W+1}
    exp = np.zeros(D)
    wexp = np.zeros((W, W))
    for k in range(1, W + 1):
        w = softmax(beta * omega[:k])
        wexp[k - 1, :k] = w
        for i in range(k):
            exp += w[i] * shifted[i]
    exp /= W
    got, wts = run(q_win, T, eps, beta, weights=True)
    np.testing.assert_allclose(wts, wexp, rtol=0, atol=1e-14)
    np.testing.assert_allclose(got, exp.astype(np.float32), rtol=1e-7, atol=0)
    # the oldest predecessor Q_{t-W} (direction e_W) never enters the shifted window
    assert got[W - 1] == np.float32(exp[W - 1])
    a1 = np.mean([wexp[k, 0] for k in range(W)])
    assert abs(got[W] - 3.0 * a1) < 1e-6            # Q_t's own component carries weight a_1


def test_ridge_solve_matches_numpy():
    rng = np.random.default_rng(1)
    for k, D, eps in [(1, 16, 0.1), (5, 32, 1e-3), (16, 128, 1e-2), (16, 8, 0.3)]:
        R = rng.standard_normal((k, D))
        T = rng.standard_normal(D)
        om = oracle.ridge_weights(R, T, eps)
        ref = np.linalg.solve(R @ R.T + eps * np.eye(k), R @ T)
        np.testing.assert_allclose(om, ref, rtol=1e-9, atol=1e-12)
        # normal equations hold
        res = (R @ R.T + eps * np.eye(k)) @ om - R @ T
        assert np.max(np.abs(res)) < 1e-9 * max(1.0, np.max(np.abs(R @ T)))
        # and it minimises the ridge objective: the gradient of ||R^T w - T||^2 + eps||w||^2 vanishes
        grad = 2 * R @ (R.T @ om - T) + 2 * eps * om
        assert np.max(np.abs(grad)) < 1e-8 * max(1.0, np.max(np.abs(R @ T)))


def test_weights_follow_window_size_subproblems():
    # w^{(k)} must come from the k newest predecessors only.
    rng = np.random.default_rng(2)
    W, D, eps = 6, 32, 0.05
    q_win = f64(bf(rng.standard_normal((W, D))))
    cur = f64(bf(rng.standard_normal(D)))
    _, wts = run(q_win, cur, eps, weights=True)
    for k in range(1, W + 1):
        R = np.stack([q_win[W - i] for i in range(1, k + 1)])
        om = np.linalg.solve(R @ R.T + eps * np.eye(k), R @ cur)
        np.testing.assert_allclose(wts[k - 1, :k], softmax(om), rtol=1e-9, atol=1e-13)
        assert np.all(wts[k - 1, k:] == 0)


def test_constant_sequence_is_fixed_point():
    rng = np.random.default_rng(3)
    v = bf(rng.standard_normal(128)).float().numpy()
    for W in (2, 7, 16):
        for eps in (1e-3, 1.0):
            got = run(np.tile(v, (W, 1)), v, eps)
            np.testing.assert_allclose(got, v, rtol=3e-7, atol=0)


def test_convex_combination_of_shifted_window():
    rng = np.random.default_rng(4)
    W, D = 16, 128
    q_win = bf(rng.standard_normal((W, D))).float().numpy()
    cur = bf(rng.standard_normal(D)).float().numpy()
    got, wts = run(q_win, cur, 1e-2, weights=True)
    assert np.all(wts >= 0)
    np.testing.assert_allclose(wts.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    shifted = np.vstack([cur[None], q_win[::-1][: W - 1]])    # Q_t, Q_{t-1}, ...
    assert np.all(got <= shifted.max(axis=0) + 1e-6)
    assert np.all(got >= shifted.min(axis=0) - 1e-6)
    a = wts.sum(axis=0) / W                                    # a_i = (1/W) sum_{k>=i} w^{(k)}_i
    np.testing.assert_allclose(got, (a[:, None] * shifted).sum(axis=0), rtol=1e-6, atol=1e-6)


def test_scaling_covariance():
    # queries * c and eps * c^2 leave omega unchanged and scale the prediction by c.
    rng = np.random.default_rng(5)
    W, D = 8, 64
    q_win = bf(rng.standard_normal((W, D))).float().numpy()
    cur = bf(rng.standard_normal(D)).float().numpy()
    a, wa = run(q_win, cur, 0.02, weights=True)
    b, wb = run(4.0 * q_win, 4.0 * cur, 0.32, weights=True)   # c = 4 is exact in bf16
    np.testing.assert_allclose(wb, wa, rtol=0, atol=1e-12)
    np.testing.assert_allclose(b, 4.0 * a, rtol=2e-7, atol=0)


def test_large_eps_limit_running_means():
    # eps -> inf: omega -> 0, uniform weights, q_hat = (1/W) sum_k mean(S_1..S_k).
    rng = np.random.default_rng(6)
    W, D = 5, 16
    q_win = bf(rng.standard_normal((W, D))).float().numpy().astype(np.float64)
    cur = bf(rng.standard_normal(D)).float().numpy().astype(np.float64)
    shifted = np.vstack([cur[None], q_win[::-1][: W - 1]])
    exp = np.mean([shifted[:k].mean(axis=0) for k in range(1, W + 1)], axis=0)
    got = run(q_win, cur, 1e12)
    np.testing.assert_allclose(got, exp, rtol=1e-6, atol=1e-7)


def test_batch_and_head_layout():
    # every (b, h) is an independent problem laid out [B, Hq, W, D]
    rng = np.random.default_rng(7)
    B, H, W, D = 2, 3, 4, 16
    qw = bf(rng.standard_normal((B, H, W, D)))
    qc = bf(rng.standard_normal((B, H, D)))
    full = oracle.predict_query(qw, qc, 0.1).numpy()
    for b in range(B):
        for h in range(H):
            one = oracle.predict_query(qw[b:b + 1, h:h + 1].contiguous(), qc[b:b + 1, h:h + 1].contiguous(), 0.1)
            assert np.array_equal(full[b, h], one[0, 0].numpy())


def test_rejects_bad_arguments():
    qw = bf(np.zeros((1, 1, 2, 4)))
    qc = bf(np.zeros((1, 1, 4)))
    with pytest.raises(RuntimeError):
        oracle.predict_query(qw, qc, 0.0)


# ---- single-solve variant (Alg. 1 steps 3-5: one ridge solve, truncate and renormalise per window size) ----
def run_single(q_win, q_cur, eps, beta=1.0):
    qh, w = oracle.predict_query(bf(q_win)[None, None], bf(q_cur)[None, None], eps, beta, return_weights=True,
                                 single_solve=True)
    return qh[0, 0].numpy(), w[0, 0].numpy()


@pytest.mark.parametrize("beta", [1.0, -1.0])
def test_single_solve_weights_are_truncated_softmax_of_one_numpy_solve(beta):
    rng = np.random.default_rng(11)
    W, D, eps = 7, 32, 0.05
    q_win = f64(bf(rng.standard_normal((W, D))))
    cur = f64(bf(rng.standard_normal(D)))
    got, wts = run_single(q_win, cur, eps, beta)
    R = np.stack([q_win[W - i] for i in range(1, W + 1)])                 # newest predecessor first
    om = np.linalg.solve(R @ R.T + eps * np.eye(W), R @ cur)              # ONE solve, all W predecessors
    shifted = np.vstack([cur[None], R[: W - 1]])                          # Q_t, Q_{t-1}, ..., Q_{t-W+1}
    exp = np.zeros(D)
    for k in range(1, W + 1):
        w = softmax(beta * om[:k])                                        # truncate to the k newest, renormalise
        np.testing.assert_allclose(wts[k - 1, :k], w, rtol=1e-9, atol=1e-13)
        assert np.all(wts[k - 1, k:] == 0)
        exp += w @ shifted[:k]
    np.testing.assert_allclose(got, (exp / W).astype(np.float32), rtol=1e-6, atol=1e-7)
    # the last row (k = W) is what the per-window-size procedure also gets; shorter windows differ in general
    _, wts_sub = run(q_win, cur, eps, beta, weights=True)
    np.testing.assert_allclose(wts[W - 1], wts_sub[W - 1], rtol=1e-9, atol=1e-13)
    assert np.max(np.abs(wts[2] - wts_sub[2])) > 1e-6


def test_single_solve_special_cases():
    rng = np.random.default_rng(12)
    # W = 1: the only weight is 1 and sits on Q_t
    cur = rng.standard_normal(128)
    got, _ = run_single(rng.standard_normal((1, 128)), cur, 0.1)
    assert np.array_equal(got, bf(cur).float().numpy())
    # constant sequence: fixed point
    v = bf(rng.standard_normal(128)).float().numpy()
    got, _ = run_single(np.tile(v, (9, 1)), v, 0.01)
    np.testing.assert_allclose(got, v, rtol=3e-7, atol=0)
    # orthogonal window: the Gram matrix is diagonal, so sub-problems and truncation coincide and the
    # single solve reproduces the per-window-size prediction exactly
    W, D, eps = 4, 8, 0.5
    alpha = np.array([2.0, 1.0, -1.5, 0.5])
    q_win = np.zeros((W, D))
    for i in range(1, W + 1):
        q_win[W - i, i - 1] = alpha[i - 1]
    T = np.zeros(D)
    T[:W] = [1.0, -0.5, 2.0, 0.25]
    T[W] = 3.0
    a, wa = run_single(q_win, T, eps)
    b, wb = run(q_win, T, eps, weights=True)
    np.testing.assert_allclose(wa, wb, rtol=0, atol=1e-14)
    np.testing.assert_allclose(a, b, rtol=1e-7, atol=0)
