"""Pins of the oracle's two comparison updates (DCD-PSGD, CHOCO-SGD) -- CPU only.

The DeepSqueeze paper (arXiv:1907.07346) gives no update rule for the methods it compares itself with.  Its
section "Why DeepSqueeze is better" prints unrolled forms of X_t (X_0 = 0) and states two things about them:

  (a) with no compression error every method is the paper's D-PSGD, X_t = -gamma sum_s G_s W_eff^{t-s};
  (b) the compression error Delta_s of a step reaches X_t through powers of W_eff alone (DCD-PSGD), through
      (W_eff - I) times such powers (CHOCO-SGD), through (W_eff - I)^2 times such powers (DeepSqueeze), which is
      what the three norm bounds at the end of that section compare.

The oracle's rules (`step_dcd`, `step_choco` in oracle/ds_oracle.cpp) are the simplest per-worker rules with these
two properties.  The tests below fix them by (a), by their one-step matrix forms with a NON-symmetric W (a
transposed operand fails), by C[.] being the already pinned operator applied to the quantity the rule names, by the
node-average behaviour, and by the unrolled forms over T = 6 steps in double.  The unrolled forms that follow from
the rules differ from the printed ones in the exponent of W_eff, a stray factor eta and (DCD-PSGD) the last term of
the sum; the tests also show that the printed variants do not satisfy (b)'s own recursion for the same errors.
Against the cited papers themselves the rules are parity unpinned: neither paper is available here.

Arrays are n x N (one row per worker), so the paper's right-multiplication by W is a left-multiplication here.
"""
import numpy as np
import pytest

import oracle
from oracle import (ALGO_CHOCO_SGD, ALGO_DCD_PSGD, ALGO_DEEPSQUEEZE, KIND_IDENTITY, KIND_QUANT_MAXABS, KIND_SIGN_MEANABS,
                    KIND_TOPK, OracleState)
from test_oracle_pins import COMPRESSORS, metropolis_matrix

mp = np.linalg.matrix_power
ALGOS = [ALGO_DCD_PSGD, ALGO_CHOCO_SGD]


def nonsymmetric_W(n, r):
    P = np.eye(n)[r.permutation(n)]
    W = 0.5 * np.eye(n) + 0.3 * P + 0.2 * np.roll(np.eye(n), 1, axis=1)
    assert not np.allclose(W, W.T)
    np.testing.assert_allclose(W.sum(0), 1), np.testing.assert_allclose(W.sum(1), 1)
    return W


def apply_operator(v, comp, n, N, seed, t):
    """C[v] from the DeepSqueeze step, whose operators the other pin file fixes: with x = 0, g = 0 and delta = v
    line 5 of Algorithm 1 forms exactly v, and the step returns C[v]."""
    st = OracleState(n=n, N=N, W=np.eye(n), gamma=0.0, eta=0.0, dtype=np.float64, seed=seed, t=t,
                     delta=np.array(v, dtype=np.float64), **comp)
    cv, msg = oracle.step(st, np.zeros((n, N)))
    return cv, msg


# ----------------------------------------------------------------------------- (a): no compression error = D-PSGD

@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("n,eta", [(5, 0.5), (8, 0.3)])
def test_without_compression_error_every_method_is_dpsgd(algo, n, eta):
    N, T, gamma = 7, 6, 0.3
    W = metropolis_matrix(n, 4, seed=n)
    r = np.random.default_rng(1)
    gs = [r.standard_normal((n, N)) for _ in range(T)]
    st = OracleState(n=n, N=N, W=W, kind=KIND_IDENTITY, gamma=gamma, eta=eta, dtype=np.float64, algo=algo)
    ds = OracleState(n=n, N=N, W=W, kind=KIND_IDENTITY, gamma=gamma, eta=eta, dtype=np.float64, algo=ALGO_DEEPSQUEEZE)
    for g in gs:
        oracle.step(st, g)
        oracle.step(ds, g)
    Weff = (1 - eta) * np.eye(n) + eta * W
    X = np.zeros((n, N))
    for s, g in enumerate(gs):
        X += -gamma * mp(Weff, T - s) @ g
    np.testing.assert_allclose(st.x, X, rtol=0, atol=1e-13)
    np.testing.assert_allclose(st.x, ds.x, rtol=0, atol=1e-13)      # and equal to Algorithm 1 with C = identity


# ----------------------------------------------------------------------------- one step, matrix form

@pytest.mark.parametrize("comp", COMPRESSORS)
def test_dcd_one_step_matrix_form(comp):
    # Z = W_eff (X - gamma G) - X,   X+ = X + C[Z]   =>   X+ = W_eff (X - gamma G) - (Z - C[Z])
    n, N, gamma, eta = 6, 45, 0.2, 0.4
    r = np.random.default_rng(3)
    W = nonsymmetric_W(n, r)
    x0, junk, g = r.standard_normal((3, n, N))
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, dtype=np.float64, seed=11, t=4, x=x0.copy(), delta=junk.copy(),
                     algo=ALGO_DCD_PSGD, **comp)
    cv, msg = oracle.step(st, g)
    Weff = (1 - eta) * np.eye(n) + eta * W
    Z = Weff @ (x0 - gamma * g) - x0
    want_cv, want_msg = apply_operator(Z, comp, n, N, seed=11, t=4)
    np.testing.assert_allclose(cv, want_cv, rtol=0, atol=1e-14)     # the operator sees the move, nothing else
    assert np.array_equal(msg, want_msg)                            # and the message is the packed C[Z]
    np.testing.assert_array_equal(st.x, x0 + cv)
    np.testing.assert_array_equal(st.delta, junk)                   # no second state array
    assert st.t == 5


@pytest.mark.parametrize("comp", COMPRESSORS)
def test_choco_one_step_matrix_form_and_node_average(comp):
    # Q = C[(X - gamma G) - Xhat],  Xhat+ = Xhat + Q,  X+ = (X - gamma G) + eta (W - I) Xhat+
    # rewritten: X+ = W_eff (X - gamma G) - (W_eff - I) Delta,  Delta = (X - gamma G) - Xhat+
    n, N, gamma, eta = 6, 45, 0.2, 0.4
    r = np.random.default_rng(4)
    W = nonsymmetric_W(n, r)
    x0, h0, g = r.standard_normal((3, n, N))
    h0 = x0 + 0.1 * h0
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, dtype=np.float64, seed=12, t=2, x=x0.copy(), delta=h0.copy(),
                     algo=ALGO_CHOCO_SGD, **comp)
    q, msg = oracle.step(st, g)
    xh = x0 - gamma * g
    want_q, want_msg = apply_operator(xh - h0, comp, n, N, seed=12, t=2)
    np.testing.assert_allclose(q, want_q, rtol=0, atol=1e-14)
    assert np.array_equal(msg, want_msg)
    np.testing.assert_array_equal(st.delta, h0 + q)                 # the public copy moves by what was sent
    I = np.eye(n)
    np.testing.assert_allclose(st.x, xh + eta * (W - I) @ st.delta, rtol=0, atol=1e-14)
    Weff = (1 - eta) * I + eta * W
    Delta = xh - st.delta
    np.testing.assert_allclose(st.x, Weff @ xh - (Weff - I) @ Delta, rtol=0, atol=1e-13)
    # columns of W - I sum to zero: the node average moves by -gamma * mean gradient whatever was lost
    np.testing.assert_allclose(st.x.mean(0), x0.mean(0) - gamma * g.mean(0), rtol=0, atol=1e-14)


@pytest.mark.parametrize("comp", COMPRESSORS[:4])
def test_dcd_node_average_drifts_by_the_mean_error(comp):
    # X+ = W_eff (X - gamma G) - Delta: the average loses mean_i Delta_i at every step (what (b) calls the error
    # reaching X undamped); Algorithm 1 and CHOCO-SGD keep the average exact.
    n, N, gamma, eta = 7, 64, 0.1, 0.5
    W = metropolis_matrix(n, 5, seed=11)
    r = np.random.default_rng(5)
    x0, g = r.standard_normal((2, n, N))
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, dtype=np.float64, x=x0.copy(), algo=ALGO_DCD_PSGD, **comp)
    cv, _ = oracle.step(st, g, want_msg=False)
    Weff = (1 - eta) * np.eye(n) + eta * W
    Delta = (Weff @ (x0 - gamma * g) - x0) - cv
    assert np.abs(Delta.mean(0)).max() > 1e-4
    np.testing.assert_allclose(st.x.mean(0), x0.mean(0) - gamma * g.mean(0) - Delta.mean(0), rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- unrolled forms, T = 6, double

def _free_run(algo, comp, n, N, W, gamma, eta, gs):
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, dtype=np.float64, seed=5, algo=algo, **comp)
    I = np.eye(n)
    Weff = (1 - eta) * I + eta * W
    deltas = []
    for t, g in enumerate(gs):
        x_before, hat_before = st.x.copy(), st.delta.copy()
        cv, _ = oracle.step(st, g, want_msg=False)
        xh = x_before - gamma * g
        if algo == ALGO_DCD_PSGD:
            operand = Weff @ xh - x_before
        else:
            operand = xh - hat_before
        # the error of this step is the already pinned operator's error on the operand the rule names
        want_cv, _ = apply_operator(operand, comp, n, N, seed=5, t=t)
        np.testing.assert_allclose(cv, want_cv, rtol=0, atol=1e-13)
        deltas.append(operand - want_cv)
    return st, deltas


@pytest.mark.parametrize("comp", COMPRESSORS[:4])
def test_dcd_unrolled_form(comp):
    # X_T = -gamma sum_{s<T} W_eff^{T-s} G_s - sum_{s<T} W_eff^{T-1-s} Delta_s     (X_0 = 0)
    n, N, gamma, eta, T = 5, 32, 0.25, 0.5, 6
    W = oracle.ring_matrix(n)
    gs = np.random.default_rng(6).standard_normal((T, n, N))
    st, deltas = _free_run(ALGO_DCD_PSGD, comp, n, N, W, gamma, eta, gs)
    Weff = (1 - eta) * np.eye(n) + eta * W
    X = np.zeros((n, N))
    for s in range(T):
        X += -gamma * mp(Weff, T - s) @ gs[s] - mp(Weff, T - 1 - s) @ deltas[s]
    np.testing.assert_allclose(st.x, X, rtol=0, atol=1e-12)
    # the printed variant (eta W_eff^{T-s} Delta_s, s <= T-2) is not the unrolling of any rule whose step-s error
    # is Delta_s: it misses the error of the last step altogether
    printed = np.zeros((n, N))
    for s in range(T):
        printed += -gamma * mp(Weff, T - s) @ gs[s]
    for s in range(T - 1):
        printed -= eta * mp(Weff, T - s) @ deltas[s]
    assert np.abs(printed - st.x).max() > 1e-3


@pytest.mark.parametrize("comp", COMPRESSORS[:4])
def test_choco_unrolled_form(comp):
    # X_T = -gamma sum_{s<T} W_eff^{T-s} G_s - sum_{s<T} W_eff^{T-1-s} (W_eff - I) Delta_s     (X_0 = Xhat_0 = 0)
    n, N, gamma, eta, T = 5, 32, 0.25, 0.5, 6
    W = oracle.ring_matrix(n)
    gs = np.random.default_rng(7).standard_normal((T, n, N))
    st, deltas = _free_run(ALGO_CHOCO_SGD, comp, n, N, W, gamma, eta, gs)
    I = np.eye(n)
    Weff = (1 - eta) * I + eta * W
    X = np.zeros((n, N))
    for s in range(T):
        X += -gamma * mp(Weff, T - s) @ gs[s] - mp(Weff, T - 1 - s) @ (Weff - I) @ deltas[s]
    np.testing.assert_allclose(st.x, X, rtol=0, atol=1e-12)
    printed = np.zeros((n, N))
    for s in range(T):
        printed += -gamma * mp(Weff, T - s) @ gs[s] - eta * mp(Weff, T - s) @ (Weff - I) @ deltas[s]
    assert np.abs(printed - st.x).max() > 1e-3


def test_choco_copy_error_is_the_operator_error():
    # after a step, (X - gamma G) - Xhat+ equals d - C[d] for d = (X - gamma G) - Xhat
    n, N, gamma, eta = 4, 64, 0.3, 0.4
    r = np.random.default_rng(8)
    x0, h0, g = r.standard_normal((3, n, N))
    comp = COMPRESSORS[0]
    st = OracleState(n=n, N=N, W=oracle.ring_matrix(n), gamma=gamma, eta=eta, dtype=np.float64, x=x0.copy(), delta=h0.copy(),
                     algo=ALGO_CHOCO_SGD, **comp)
    q, _ = oracle.step(st, g, want_msg=False)
    d = (x0 - gamma * g) - h0
    np.testing.assert_allclose((x0 - gamma * g) - st.delta, d - q, rtol=0, atol=1e-15)


# ----------------------------------------------------------------------------- (b): how far one step's error reaches

@pytest.mark.parametrize("eta", [0.25, 0.5])
def test_error_damping_order_of_the_three_methods(eta):
    # ||(W_eff - I)^2 D|| <= eta (1 - lambda_n) ||(W_eff - I) D|| <= (eta (1 - lambda_n))^2 ||D||  for symmetric
    # doubly stochastic W ("Why DeepSqueeze is better", the three bounds), and one step's error enters each
    # method's X with exactly that factor: perturb the operand's error and look at X+.
    n, N = 8, 40
    W = oracle.ring_matrix(n)
    I = np.eye(n)
    E = eta * (W - I)
    lam_n = np.linalg.eigvalsh(W).min()
    c = eta * (1 - lam_n)
    D = np.random.default_rng(9).standard_normal((n, N))
    fro = lambda A: np.linalg.norm(A, "fro")
    assert fro(E @ E @ D) <= c * fro(E @ D) * (1 + 1e-12) <= c * c * fro(D) * (1 + 1e-12)
    assert c <= 1.0 + 1e-12

    def x_after(algo, loss):
        """One step from X = 0 with gradients chosen so that the operand is V; top-k drops `loss` (supported on
        the entries it does not keep), everything else equal."""
        comp = dict(kind=KIND_TOPK, k=N // 2)
        st = OracleState(n=n, N=N, W=W, gamma=1.0, eta=eta, dtype=np.float64, algo=algo, **comp)
        big = np.zeros((n, N)); big[:, :N // 2] = 10.0 + np.arange(N // 2)       # always kept
        small = np.zeros((n, N)); small[:, N // 2:] = loss[:, N // 2:]           # always dropped
        if algo == ALGO_DCD_PSGD:        # operand = W_eff (-G): choose G = -W_eff^{-1} (big + small)
            G = -np.linalg.solve((1 - eta) * I + eta * W, big + small)
        else:                            # operand = -G for CHOCO-SGD and (delta = 0) for Algorithm 1
            G = -(big + small)
        oracle.step(st, G, want_msg=False)
        return st.x, G

    loss = np.zeros((n, N)); loss[:, N // 2:] = 0.01 * D[:, N // 2:]
    zero = np.zeros((n, N))
    Weff = I + E
    # DCD-PSGD: X+ = W_eff(-G) - Delta
    xa, Ga = x_after(ALGO_DCD_PSGD, loss)
    np.testing.assert_allclose(xa, Weff @ (-Ga) - loss, rtol=0, atol=1e-12)
    # CHOCO-SGD: X+ = W_eff(-G) - (W_eff - I) Delta
    xb, Gb = x_after(ALGO_CHOCO_SGD, loss)
    np.testing.assert_allclose(xb, Weff @ (-Gb) - E @ loss, rtol=0, atol=1e-12)
    # Algorithm 1, first step (Delta_{-1} = 0): X+ = W_eff(-G) - (W_eff - I) Delta as well; the second factor
    # (W_eff - I) appears from the next step on, when the carried error is sent again (pinned by
    # test_unrolled_closed_form in the other pin file)
    xc, Gc = x_after(ALGO_DEEPSQUEEZE, loss)
    np.testing.assert_allclose(xc, Weff @ (-Gc) - E @ loss, rtol=0, atol=1e-12)
    assert fro(E @ loss) < fro(loss)


# ----------------------------------------------------------------------------- float vs double, all-cores build

@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("comp", [COMPRESSORS[2], COMPRESSORS[3]])
def test_comparison_fp32_and_fp64_runs_agree(algo, comp):
    n, N, T = 6, 80, 5
    W = oracle.ring_matrix(n)
    gs = np.random.default_rng(13).standard_normal((T, n, N)).astype(np.float32)
    a = OracleState(n=n, N=N, W=W, gamma=0.1, eta=0.3, algo=algo, **comp)
    b = OracleState(n=n, N=N, W=W, gamma=float(np.float32(0.1)), eta=float(np.float32(0.3)), dtype=np.float64, algo=algo, **comp)
    for g in gs:
        oracle.step(a, g, want_msg=False)
        oracle.step(b, g.astype(np.float64), want_msg=False)
    np.testing.assert_allclose(a.x, b.x, rtol=0, atol=2e-5)
    np.testing.assert_allclose(a.delta, b.delta, rtol=0, atol=2e-5)


@pytest.mark.parametrize("algo", ALGOS)
def test_comparison_all_cores_build_gives_the_same_bits(algo):
    n, N = 6, 3000
    for kind, kw in ((KIND_QUANT_MAXABS, dict(bits=2, block=256)), (KIND_SIGN_MEANABS, dict(block=128)), (KIND_TOPK, dict(k=37))):
        outs = []
        for all_cores in (False, True):
            st = OracleState(n=n, N=N, W=oracle.ring_matrix(n), kind=kind, gamma=0.1, eta=0.4, seed=3, algo=algo, **kw)
            r = np.random.default_rng(5)
            msgs = [oracle.step(st, r.standard_normal((n, N)).astype(np.float32), all_cores=all_cores) for _ in range(3)]
            outs.append((st.x, st.delta, msgs))
        a, b_ = outs
        assert a[0].tobytes() == b_[0].tobytes() and a[1].tobytes() == b_[1].tobytes()
        for (cv0, m0), (cv1, m1) in zip(a[2], b_[2]):
            assert cv0.tobytes() == cv1.tobytes() and np.array_equal(m0, m1)


def test_comparison_steps_reject_an_unknown_rule():
    st = OracleState(n=3, N=8, W=oracle.ring_matrix(3), kind=KIND_IDENTITY, gamma=0.1, eta=0.4, algo=7)
    with pytest.raises(RuntimeError):
        oracle.step(st, np.zeros((3, 8), np.float32))
