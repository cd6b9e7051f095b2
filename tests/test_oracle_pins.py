"""Pins of the CPU oracle against what the paper and plain mathematics fix.

None of these tests touches the GPU library.  Each one is chosen so that a
plausible mistake in `oracle/ds_oracle.cpp` (dropped term, wrong sign or index,
transposed W, wrong bit position, biased rounding) makes it fail.

Citations are to the DeepSqueeze paper (arXiv:1907.07346): Algorithm 1, the
section "Mathematical formulation" (matrix form, W_eff form), the section "Why
DeepSqueeze is better" (closed forms), Assumption 1, and the supplement's
node-average recursion.  The paper's matrices are N x n with W acting on the
right; arrays here are n x N (one row per worker), so W acts on the left.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import (KIND_IDENTITY, KIND_QUANT_MAXABS, KIND_SIGN_MEANABS, KIND_TOPK, KIND_QUANT_L2NORM, KIND_RAND_SPARSE, KIND_GSPAR,
                    OracleState)


# ----------------------------------------------------------------------------- helpers

def metropolis_matrix(n, extra_edges, seed):
    """Symmetric doubly stochastic W of a connected random graph (ring + chords), varying degree."""
    r = np.random.default_rng(seed)
    A = np.zeros((n, n), dtype=bool)
    for i in range(n):
        A[i, (i + 1) % n] = A[(i + 1) % n, i] = True
    for _ in range(extra_edges):
        i, j = r.integers(0, n, 2)
        if i != j:
            A[i, j] = A[j, i] = True
    deg = A.sum(1)
    W = np.zeros((n, n))
    for i in range(n):
        for j in range(n):
            if A[i, j]:
                W[i, j] = 1.0 / (1 + max(deg[i], deg[j]))
    for i in range(n):
        W[i, i] = 1.0 - W[i].sum()
    return W


def run(st, gs, **kw):
    out = []
    for g in gs:
        out.append(oracle.step(st, g, **kw))
    return out


def unpack_codes(words, bits, m):
    """Independent decoder of the packed code words (little-endian bit order inside a word)."""
    codes = np.zeros(m, dtype=np.int64)
    per = 32 // bits
    for e in range(m):
        codes[e] = (int(words[e // per]) >> (bits * (e % per))) & ((1 << bits) - 1)
    return codes


def split_block_message(msg, N, block, bits):
    """Yield (scale, words, m) per block of one worker's message."""
    off = 0
    for j0 in range(0, N, block):
        m = min(block, N - j0)
        nw = (m * bits + 31) // 32
        s = np.frombuffer(msg[off:off + 4].tobytes(), dtype=np.float32)[0]
        w = np.frombuffer(msg[off + 4:off + 4 + 4 * nw].tobytes(), dtype=np.uint32)
        off += 4 + 4 * nw
        yield s, w, m
    assert off == len(msg)


# ----------------------------------------------------------------------------- Philox

def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) if l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        w = [int(h, 16) for h in r]
        assert list(oracle.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def test_rounding_word_is_addressed_by_seed_step_worker_element():
    # element j uses word j mod 4 of the block whose counter is (j // 4, i, t, 'QUNT'), key = seed halves
    seed = 0x0123456789ABCDEF
    for (t, i, j) in [(0, 0, 0), (3, 2, 5), (7, 1, 1023), (2 ** 32 + 5, 9, 4 * 77 + 3)]:
        blk = oracle.philox4x32_10([j // 4, i, t & 0xFFFFFFFF, 0x51554E54], [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.rounding_word(seed, t, i, j) == int(blk[j % 4])
    # distinct addresses give distinct streams
    ws = {oracle.rounding_word(1, t, i, j) for t in range(4) for i in range(4) for j in range(16)}
    assert len(ws) == 4 * 4 * 16


def test_rounding_words_look_uniform():
    w = np.array([oracle.rounding_word(5, 1, 0, j) for j in range(1 << 14)], dtype=np.uint64)
    bits = ((w[:, None] >> np.arange(32, dtype=np.uint64)) & 1).mean(0)
    assert np.all(np.abs(bits - 0.5) < 5 * 0.5 / np.sqrt(len(w)))
    hist = np.bincount((w >> 28).astype(np.int64), minlength=16)
    chi2 = ((hist - len(w) / 16) ** 2 / (len(w) / 16)).sum()
    assert chi2 < 45.0        # 15 dof, p ~ 1e-4


# ----------------------------------------------------------------------------- P1: identity = D-PSGD

@pytest.mark.parametrize("n,eta", [(5, 0.5), (8, 0.3)])
def test_identity_reduces_to_dpsgd_closed_form(n, eta):
    # X_t = -gamma sum_s G_s W_eff^{t-s}, W_eff = (1-eta) I + eta W   ("Why DeepSqueeze is better", D-PSGD)
    N, T, gamma = 7, 5, 0.3
    W = metropolis_matrix(n, 4, seed=n)
    r = np.random.default_rng(1)
    gs = [r.standard_normal((n, N)) for _ in range(T)]
    st = OracleState(n=n, N=N, W=W, kind=KIND_IDENTITY, gamma=gamma, eta=eta, dtype=np.float64)
    run(st, gs)
    Weff = (1 - eta) * np.eye(n) + eta * W
    X = np.zeros((n, N))
    for s, g in enumerate(gs):
        X += -gamma * np.linalg.matrix_power(Weff, T - s) @ g
    np.testing.assert_allclose(st.x, X, rtol=0, atol=1e-13)
    np.testing.assert_array_equal(st.delta, 0.0)


def test_time_varying_graph_product_form():
    # with a different symmetric doubly stochastic W_t at every step and no compression,
    # X_T = -gamma sum_s W_eff,T-1 ... W_eff,s G_s  (the D-PSGD closed form with a product instead of a power)
    n, N, T, gamma, eta = 6, 9, 4, 0.2, 0.4
    r = np.random.default_rng(21)
    Ws = [metropolis_matrix(n, 3 + t, seed=30 + t) for t in range(T)]
    gs = [r.standard_normal((n, N)) for _ in range(T)]
    st = OracleState(n=n, N=N, W=Ws[0], kind=KIND_IDENTITY, gamma=gamma, eta=eta, dtype=np.float64)
    for t in range(T):
        st.set_W(Ws[t])
        oracle.step(st, gs[t], want_msg=False)
    X = np.zeros((n, N))
    for s_ in range(T):
        term = gs[s_]
        for t in range(s_, T):
            term = ((1 - eta) * np.eye(n) + eta * Ws[t]) @ term
        X += -gamma * term
    np.testing.assert_allclose(st.x, X, rtol=0, atol=1e-13)
    # and with compression the node average still moves by -gamma * mean gradient at every step
    st = OracleState(n=n, N=N, W=Ws[0], gamma=gamma, eta=eta, dtype=np.float64, **COMPRESSORS[0])
    for t in range(T):
        before = st.x.mean(0).copy()
        st.set_W(Ws[t])
        oracle.step(st, gs[t], want_msg=False)
        np.testing.assert_allclose(st.x.mean(0), before - gamma * gs[t].mean(0), rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- P2/P3/P4: one-step identities

COMPRESSORS = [
    dict(kind=KIND_QUANT_MAXABS, bits=4, block=16),
    dict(kind=KIND_QUANT_MAXABS, bits=2, block=32),
    dict(kind=KIND_SIGN_MEANABS, block=8),
    dict(kind=KIND_TOPK, k=5),
    dict(kind=KIND_QUANT_L2NORM, bits=2),
    dict(kind=KIND_QUANT_L2NORM, bits=4),
    dict(kind=KIND_RAND_SPARSE, k=20),
    dict(kind=KIND_GSPAR, k=15),
]


@pytest.mark.parametrize("comp", COMPRESSORS)
def test_one_step_matches_matrix_form_with_nonsymmetric_W(comp):
    # Algorithm 1 line 9 is x_i += eta sum_j (W_ij - I_ij) C_j, i.e. X+ = (X - gamma G) + eta (W - I) C.
    # A non-symmetric doubly stochastic W exposes a transposed operand.
    n, N, gamma, eta = 6, 45, 0.2, 0.4
    r = np.random.default_rng(3)
    P = np.eye(n)[r.permutation(n)]
    W = 0.5 * np.eye(n) + 0.3 * P + 0.2 * np.roll(np.eye(n), 1, axis=1)
    assert not np.allclose(W, W.T)
    np.testing.assert_allclose(W.sum(0), 1), np.testing.assert_allclose(W.sum(1), 1)
    x0, d0, g = r.standard_normal((3, n, N))
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, dtype=np.float64, x=x0.copy(), delta=d0.copy(), **comp)
    cv, _ = oracle.step(st, g, want_msg=False)
    V = x0 - gamma * g + d0
    np.testing.assert_allclose(st.delta + cv, V, rtol=0, atol=1e-15)                     # line 6
    np.testing.assert_allclose(st.x, x0 - gamma * g + eta * (W - np.eye(n)) @ cv, rtol=0, atol=1e-14)


@pytest.mark.parametrize("comp", COMPRESSORS)
def test_weff_form_and_node_average(comp):
    # X+ = W_eff (X - gamma G) + (W_eff - I)(Delta_old - Delta_new)   (matrix form rewritten with W_eff)
    # and mean_i x_i moves by exactly -gamma * mean_i g_i              (supplement, node-average recursion)
    n, N, gamma, eta = 7, 64, 0.1, 0.5
    W = metropolis_matrix(n, 5, seed=11)
    r = np.random.default_rng(4)
    x0, d0, g = r.standard_normal((3, n, N))
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, dtype=np.float64, x=x0.copy(), delta=d0.copy(), **comp)
    oracle.step(st, g, want_msg=False)
    Weff = (1 - eta) * np.eye(n) + eta * W
    rhs = Weff @ (x0 - gamma * g) + (Weff - np.eye(n)) @ (d0 - st.delta)
    np.testing.assert_allclose(st.x, rhs, rtol=0, atol=1e-13)
    np.testing.assert_allclose(st.x.mean(0), x0.mean(0) - gamma * g.mean(0), rtol=0, atol=1e-14)


@pytest.mark.parametrize("comp", COMPRESSORS)
def test_node_average_in_fp32_over_many_steps(comp):
    n, N, gamma, eta, T = 8, 96, 0.1, 0.4, 20
    W = oracle.ring_matrix(n)
    r = np.random.default_rng(5)
    gs = r.standard_normal((T, n, N)).astype(np.float32)
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, seed=3, **comp)
    run(st, gs, want_cv=False, want_msg=False)
    expect = -np.float64(np.float32(gamma)) * gs.astype(np.float64).mean(1).sum(0)
    np.testing.assert_allclose(st.x.astype(np.float64).mean(0), expect, rtol=0, atol=2e-5)


# ----------------------------------------------------------------------------- P5: closed form over several steps

@pytest.mark.parametrize("comp", COMPRESSORS[:3])
def test_unrolled_closed_form(comp):
    # X_t = -gamma sum_{s<t} W_eff^{t-s} G_s - (W_eff - I) Delta_{t-1}
    #       - sum_{s<=t-2} W_eff^{t-2-s} (W_eff - I)^2 Delta_s            (X_0 = 0, Delta_{-1} = 0)
    # This is the unrolled update of "Why DeepSqueeze is better"; the printed versions disagree with each
    # other in the signs / eta factors, this one follows from the W_eff form by induction.
    n, N, gamma, eta, T = 5, 32, 0.25, 0.5, 6
    W = oracle.ring_matrix(n)
    r = np.random.default_rng(6)
    gs = r.standard_normal((T, n, N))
    st = OracleState(n=n, N=N, W=W, gamma=gamma, eta=eta, dtype=np.float64, **comp)
    deltas = []
    for g in gs:
        oracle.step(st, g, want_msg=False)
        deltas.append(st.delta.copy())
    I = np.eye(n)
    Weff = (1 - eta) * I + eta * W
    mp = np.linalg.matrix_power
    X = np.zeros((n, N))
    for s in range(T):
        X += -gamma * mp(Weff, T - s) @ gs[s]
    X -= (Weff - I) @ deltas[T - 1]
    for s in range(T - 1):
        X -= mp(Weff, T - 2 - s) @ mp(Weff - I, 2) @ deltas[s]
    np.testing.assert_allclose(st.x, X, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- P6: hand-expanded example

def _parse_alg1_example(path):
    steps, cur = [], None
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        key, rest = line.split(None, 1)
        if key == "t":
            cur = {}
            steps.append(cur)
            continue
        cur[key] = np.array([[float(Fraction(tok)) for tok in row.split()] for row in rest.split("|")])
    return steps


@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-15), (np.float32, 5e-7)])
def test_hand_expanded_sign_example(golden_dir, dtype, tol):
    steps = _parse_alg1_example(os.path.join(golden_dir, "alg1_sign_ring3.txt"))
    st = OracleState(n=3, N=2, W=oracle.ring_matrix(3), kind=KIND_SIGN_MEANABS, block=2, gamma=1.0, eta=0.5,
                     dtype=dtype)
    for rec in steps:
        cv, msg = oracle.step(st, rec["g"].astype(dtype))
        np.testing.assert_allclose(cv, rec["c"], rtol=tol, atol=0)
        np.testing.assert_allclose(st.delta, rec["d"], rtol=0, atol=4 * tol)
        np.testing.assert_allclose(st.x, rec["x"], rtol=0, atol=4 * tol)
        # message: per worker [scale][1 word]; bit e set <=> element e negative (sign(+0) = +)
        m = msg.reshape(3, 8)
        for i in range(3):
            s = np.frombuffer(m[i, :4].tobytes(), np.float32)[0]
            w = int(np.frombuffer(m[i, 4:].tobytes(), np.uint32)[0])
            assert abs(s - rec["s"][i, 0]) <= 5e-7 * 4    # the message carries the scale in fp32
            assert w == sum(1 << e for e in range(2) if rec["v"][i, e] < 0)


def test_hand_expanded_example_matches_rational_brute_force(golden_dir):
    # the stored example itself, re-derived with exact rationals in matrix form
    steps = _parse_alg1_example(os.path.join(golden_dir, "alg1_sign_ring3.txt"))
    n, N, gam, eta = 3, 2, Fraction(1), Fraction(1, 2)
    W = [[Fraction(1, 3)] * 3 for _ in range(3)]
    X = [[Fraction(0)] * N for _ in range(n)]
    D = [[Fraction(0)] * N for _ in range(n)]
    for rec in steps:
        G = [[Fraction(int(v)) for v in row] for row in rec["g"]]
        V = [[X[i][j] - gam * G[i][j] + D[i][j] for j in range(N)] for i in range(n)]
        S = [sum(abs(v) for v in V[i]) / N for i in range(n)]
        C = [[S[i] if V[i][j] >= 0 else -S[i] for j in range(N)] for i in range(n)]
        D = [[V[i][j] - C[i][j] for j in range(N)] for i in range(n)]
        X = [[X[i][j] - gam * G[i][j] + eta * sum((W[i][k] - (i == k)) * C[k][j] for k in range(n))
              for j in range(N)] for i in range(n)]
        np.testing.assert_allclose(np.array(X, dtype=float), rec["x"], atol=1e-15)
        np.testing.assert_allclose(np.array(D, dtype=float), rec["d"], atol=1e-15)


def test_window_step_equals_the_columns_of_the_wide_step():
    # the windowed entry point (used to check very long vectors piecewise) against the plain one
    n, N, B = 5, 64 * 9 + 13, 64
    W = oracle.ring_matrix(n)
    r = np.random.default_rng(31)
    x0, d0, g = (r.standard_normal((3, n, N)) * 0.3).astype(np.float32)
    for comp in (dict(kind=KIND_QUANT_MAXABS, bits=4, block=B), dict(kind=KIND_SIGN_MEANABS, block=B),
                 dict(kind=KIND_IDENTITY)):
        wide = OracleState(n=n, N=N, W=W, gamma=0.1, eta=0.4, seed=7, t=5, x=x0.copy(), delta=d0.copy(), **comp)
        oracle.step(wide, g, want_cv=False)
        for c0, c1 in ((0, 3 * B), (4 * B, 7 * B), (8 * B, N)):
            win = OracleState(n=n, N=c1 - c0, W=W, gamma=0.1, eta=0.4, seed=7, t=5,
                              x=x0[:, c0:c1].copy(), delta=d0[:, c0:c1].copy(), **comp)
            oracle.step_window(win, g[:, c0:c1], c0)
            np.testing.assert_array_equal(win.x, wide.x[:, c0:c1])
            np.testing.assert_array_equal(win.delta, wide.delta[:, c0:c1])
    # a window that starts elsewhere draws other rounding words
    a = OracleState(n=n, N=B, W=W, gamma=0.1, eta=0.4, seed=7, x=x0[:, :B].copy(), kind=KIND_QUANT_MAXABS, bits=2, block=B)
    b_ = OracleState(n=n, N=B, W=W, gamma=0.1, eta=0.4, seed=7, x=x0[:, :B].copy(), kind=KIND_QUANT_MAXABS, bits=2, block=B)
    assert not np.array_equal(oracle.step_window(a, g[:, :B], 0), oracle.step_window(b_, g[:, :B], B))


# ----------------------------------------------------------------------------- the experiments' compressor

def l2norm_state(v, bits, dtype=np.float32, n=1):
    v = np.asarray(v, dtype=dtype).reshape(n, -1)
    W = np.ones((1, 1)) if n == 1 else np.eye(n)
    return OracleState(n=n, N=v.shape[1], W=W, kind=KIND_QUANT_L2NORM, bits=bits, gamma=0.0, eta=0.5,
                       dtype=dtype, x=v.copy())


def test_l2norm_worked_example(golden_dir):
    rec = {l.split()[0]: l.split()[1:] for l in open(os.path.join(golden_dir, "l2norm_2bit_micro.txt"))
           if l[0] != "#"}
    v = np.array([float(t) for t in rec["v"]], dtype=np.float32)
    y = np.array([int(t) for t in rec["y"]])
    nrm = np.float32(np.sqrt(float(rec["sum_v2"][0])))
    unit = np.float32(float(nrm) / np.sqrt(float(rec["sum_y2"][0])))
    st = l2norm_state(v, 2)
    cv, msg = oracle.step(st, np.zeros((1, 8), np.float32))
    assert msg[:4].tobytes() == nrm.tobytes()
    assert np.frombuffer(msg[4:8].tobytes(), np.uint32)[0] == int(rec["word"][0], 16) and len(msg) == 8
    assert list(unpack_codes(np.frombuffer(msg[4:8].tobytes(), np.uint32), 2, 8)) == [int(t) for t in rec["q"]]
    np.testing.assert_array_equal(cv[0], y.astype(np.float32) * unit)
    np.testing.assert_array_equal(st.delta[0], v - y.astype(np.float32) * unit)
    np.testing.assert_array_equal(st.x[0], v)                   # W = [1]: nothing is mixed in


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_l2norm_receiver_restores_the_euclidean_norm(bits, dtype):
    # the property the paper states: the decoded tensor has the Euclidean norm of the original one
    r = np.random.default_rng(21)
    n, N, L = 3, 1000 + 37, (1 << bits) - 1
    v = (r.standard_normal((n, N)) * np.array([[1e-3], [1.0], [50.0]])).astype(dtype)
    st = l2norm_state(v, bits, dtype=dtype, n=n)
    cv, msg = oracle.step(st, np.zeros_like(v), want_msg=(dtype == np.float32))
    tol = 2e-7 if dtype == np.float32 else 1e-14
    exact = np.sqrt((v.astype(np.float64) ** 2).sum(1))
    np.testing.assert_allclose(np.sqrt((cv.astype(np.float64) ** 2).sum(1)), exact, rtol=tol)
    # C[v] is a positive multiple of a vector of odd integers in [-L, L] ...
    unit = np.abs(cv).min(1, keepdims=True)                     # |y| = 1 occurs in every row of this input
    y = cv / unit
    assert np.all(np.abs(y - np.rint(y)) < 1e-5) and np.all(np.rint(np.abs(y)) % 2 == 1) and np.abs(y).max() <= L + 1e-5
    # ... namely the nearest odd integer to L v / max|v| (no randomness: two runs agree, and the seed is irrelevant)
    target = L * v.astype(np.float64) / np.abs(v).max(1, keepdims=True)
    assert np.all(np.abs(np.rint(y) - target) <= 1.0 + 1e-5)
    st2 = l2norm_state(v, bits, dtype=dtype, n=n)
    st2.seed = 1234
    cv2, _ = oracle.step(st2, np.zeros_like(v), want_msg=False)
    np.testing.assert_array_equal(cv, cv2)
    if dtype == np.float32:
        # the message alone gives back C[v]: the receiver knows only the codes and the norm
        row = 4 + 4 * ((N * bits + 31) // 32)
        assert len(msg) == n * row
        for i in range(n):
            m = msg[i * row:(i + 1) * row]
            sent = np.frombuffer(m[:4].tobytes(), np.float32)[0]
            assert abs(float(sent) - exact[i]) <= 1e-7 * exact[i]
            q = unpack_codes(np.frombuffer(m[4:].tobytes(), np.uint32), bits, N)
            yy = 2 * q - L
            dec = yy.astype(np.float32) * np.float32(float(sent) / np.sqrt(float((yy * yy).sum())))
            np.testing.assert_array_equal(dec, cv[i])
            # padding bits of the last word are zero
            last = int(np.frombuffer(m[-4:].tobytes(), np.uint32)[0])
            used = (N * bits) % 32
            assert used == 0 or last >> used == 0


def test_l2norm_rounds_to_the_nearest_level_ties_to_even():
    # brute force in exact rational arithmetic; with s = max|v| = L the map is t = v/2 + L/2, exact in
    # floating point for multiples of 1/4, and every even integer v is a real tie (t = q + 1/2)
    for bits in (2, 4):
        L = (1 << bits) - 1
        ks = np.arange(-4 * L, 4 * L + 1)
        v = ks / 4.0
        st = l2norm_state(v, bits, dtype=np.float64)
        cv, _ = oracle.step(st, np.zeros((1, v.size)), want_msg=False)
        unit = np.abs(cv).min()
        got = np.rint(cv[0] / unit).astype(int)
        ties = 0
        for k, yk in zip(ks, got):
            t = (Fraction(int(k), 4 * L) + 1) * Fraction(L, 2)  # (v/s + 1) L / 2
            lo = t.numerator // t.denominator
            fr = t - lo
            ties += fr == Fraction(1, 2)
            q = lo + (1 if fr > Fraction(1, 2) or (fr == Fraction(1, 2) and lo % 2 == 1) else 0)
            assert yk == 2 * q - L, (bits, k, yk, q)
        assert ties == L                                        # t = 1/2, 3/2, ..., L - 1/2


@pytest.mark.parametrize("bits,bound", [(2, 0.5), (4, 0.05)])
def test_l2norm_satisfies_the_signal_to_noise_assumption(bits, bound):
    # Assumption 1.6: |C[v] - v|^2 <= alpha^2 |v|^2 with alpha < 1.  On Gaussian vectors the operator
    # behaves like a scaled sign for 2 bits (alpha^2 = 2 (1 - sqrt(2/pi)) ~ 0.40) and like a fine grid for 4.
    r = np.random.default_rng(22)
    v = r.standard_normal((4, 1 << 14))
    st = l2norm_state(v, bits, dtype=np.float64, n=4)
    cv, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
    alpha2 = ((cv - v) ** 2).sum(1) / (v ** 2).sum(1)
    assert np.all(alpha2 < bound), alpha2
    if bits == 2:
        assert np.all(alpha2 > 0.3)


def test_l2norm_zero_vector_and_single_element():
    st = l2norm_state(np.zeros(10), 4)
    cv, msg = oracle.step(st, np.zeros((1, 10), np.float32))
    assert np.all(cv == 0) and np.all(st.delta == 0) and np.all(msg == 0)
    st = l2norm_state([-2.5], 2)                                 # one element: C[v] = v exactly
    cv, msg = oracle.step(st, np.zeros((1, 1), np.float32))
    assert cv[0, 0] == np.float32(-2.5) and st.delta[0, 0] == 0 and msg[4] == 0


def test_sum_of_squares_is_the_adjacent_pairs_tree_in_double():
    A = 2.0 ** 27                                               # A^2 = 2^54, where doubles are 4 apart
    # tree: (A^2+1) -> A^2, (1+1) three times, A^2+2 -> tie -> A^2, 2+2, A^2+4 exact; left to right stays at A^2
    assert oracle.sum_squares_tree([A, 1, 1, 1, 1, 1, 1, 1]) == 2.0 ** 54 + 4
    # five elements are padded to eight: (A^2+1), (1+1), (1+0), (0+0) -> A^2+2 -> A^2, 1 -> A^2
    assert oracle.sum_squares_tree([A, 1, 1, 1, 1]) == 2.0 ** 54
    assert oracle.sum_squares_tree([1, 1, 1, 1, A]) == 2.0 ** 54 + 4
    r = np.random.default_rng(23)
    v = r.standard_normal(3001).astype(np.float32)
    import math
    exact = math.fsum(float(t) * float(t) for t in v)
    assert abs(oracle.sum_squares_tree(v) - exact) <= 1e-13 * exact
    assert oracle.sum_squares_tree(np.zeros(0, np.float32)) == 0.0


# ----------------------------------------------------------------------------- random sparsification

def test_rand_sparse_mask_rule_message_and_residual():
    n, N, k, seed = 4, 3001, 500, 9
    r = np.random.default_rng(41)
    v = r.standard_normal((n, N)).astype(np.float32)
    st = OracleState(n=n, N=N, W=np.eye(n), kind=KIND_RAND_SPARSE, k=k, gamma=0.0, eta=0.5, seed=seed, t=6, x=v.copy())
    cv, msg = oracle.step(st, np.zeros_like(v))
    T = (k << 24) // N
    SPAR = int.from_bytes(b"SPAR", "big")
    cap = k + 8 * 23 + 64                                       # ceil(sqrt(500)) = 23
    assert oracle.rand_sparse_capacity(N, k) == cap and len(msg) == n * (4 + 4 * cap)
    for i in range(n):
        # the mask: top 24 bits of the element's own Philox word (stream 'SPAR') below floor(k 2^24 / N)
        words = [oracle.philox4x32_10([j // 4, i, 6, SPAR], [seed, 0])[j % 4] for j in range(N)]
        keep = np.array([(int(wd) >> 8) < T for wd in words])
        assert [oracle.keep_word(seed, 6, i, j) for j in (0, 1, 5, N - 1)] == [int(words[j]) for j in (0, 1, 5, N - 1)]
        np.testing.assert_array_equal(cv[i], np.where(keep, v[i], np.float32(0)))
        np.testing.assert_array_equal(st.delta[i], np.where(keep, np.float32(0), v[i]))
        row = msg[i * (4 + 4 * cap):(i + 1) * (4 + 4 * cap)]
        count = int(np.frombuffer(row[:4].tobytes(), np.uint32)[0])
        vals = np.frombuffer(row[4:].tobytes(), np.float32)
        assert count == keep.sum()
        np.testing.assert_array_equal(vals[:count], v[i][keep])                 # ascending index
        assert np.all(row[4 + 4 * count:] == 0)
    # the keep stream is not the rounding stream
    assert oracle.keep_word(seed, 6, 0, 0) != oracle.rounding_word(seed, 6, 0, 0)
    assert oracle.rand_sparse_capacity(50, 40) == 50            # never more than N


def test_rand_sparse_threshold_is_strict():
    # keep iff (word >> 8) < T, T = floor(k 2^24 / N): with N = 4096, T = 4096 k; find an element whose 24 bits
    # ARE a multiple of 4096 and give it exactly that T: it must be dropped (an off-by-one T would keep it)
    N, found = 4096, 0
    for seed in range(60):
        tops = np.array([oracle.keep_word(seed, 0, 0, j) >> 8 for j in range(N)])
        hits = np.nonzero((tops % 4096 == 0) & (tops >= 4096))[0]
        if hits.size == 0:
            continue
        j = int(hits[0])
        k = int(tops[j]) // 4096
        v = np.arange(1, N + 1, dtype=np.float32)[None, :]
        st = OracleState(n=1, N=N, W=np.ones((1, 1)), kind=KIND_RAND_SPARSE, k=k, gamma=0.0, eta=0.5, seed=seed, x=v.copy())
        cv, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
        assert cv[0, j] == 0 and st.delta[0, j] == v[0, j]
        np.testing.assert_array_equal(cv[0] != 0, tops < 4096 * k)
        found += 1
        if found == 3:
            break
    assert found == 3


def test_rand_sparse_rate_independence_and_signal_to_noise():
    # keep rate = floor(k 2^24 / N) / 2^24 within 5 sigma; masks of different workers and steps are unrelated;
    # |C[v] - v|^2 / |v|^2 averages to 1 - p: the alpha^2 of Assumption 1.6
    n, N, k = 3, 200_000, 20_000
    p = ((k << 24) // N) / 2.0 ** 24
    r = np.random.default_rng(42)
    v = r.standard_normal((n, N)).astype(np.float64)
    st = OracleState(n=n, N=N, W=np.eye(n), kind=KIND_RAND_SPARSE, k=k, gamma=0.0, eta=0.5, seed=1, dtype=np.float64, x=v.copy())
    cv1, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
    st.x[:], st.delta[:] = v, 0.0
    cv2, _ = oracle.step(st, np.zeros_like(v), want_msg=False)                  # next step: another mask
    m1, m2 = cv1 != 0, cv2 != 0
    sd = np.sqrt(p * (1 - p) / N)
    assert np.all(np.abs(m1.mean(1) - p) < 5 * sd) and np.all(np.abs(m2.mean(1) - p) < 5 * sd)
    for a, b_ in ((m1[0], m1[1]), (m1[0], m2[0]), (m1[2], m2[1])):
        both = (a & b_).mean()
        assert abs(both - p * p) < 5 * np.sqrt(p * p * (1 - p * p) / N)
    # neighbours inside a Philox group of four are unrelated too
    assert abs((m1[0][0::4] & m1[0][1::4]).mean() - p * p) < 5 * np.sqrt(p * p / (N / 4))
    alpha2 = ((cv1 - v) ** 2).sum(1) / (v ** 2).sum(1)
    assert np.all(np.abs(alpha2 - (1 - p)) < 0.01)
    np.testing.assert_array_equal(cv1[m1], v[m1])                               # kept values are exact, no rescaling


def test_rand_sparse_keeping_everything_is_dpsgd():
    n, N = 5, 257
    W = oracle.ring_matrix(n)
    r = np.random.default_rng(43)
    gs = r.standard_normal((4, n, N)).astype(np.float32)
    a = OracleState(n=n, N=N, W=W, kind=KIND_RAND_SPARSE, k=N, gamma=0.1, eta=0.4)
    b_ = OracleState(n=n, N=N, W=W, kind=KIND_IDENTITY, gamma=0.1, eta=0.4)
    for g in gs:
        oracle.step(a, g, want_msg=False), oracle.step(b_, g, want_msg=False)
    np.testing.assert_array_equal(a.x, b_.x)
    assert np.all(a.delta == 0)


# ----------------------------------------------------------------------------- GSpar (magnitude-proportional sparsifier)

def test_gspar_mask_rule_message_and_residual():
    # keep iff u < p, u = (word >> 8) / 2^24 from the stream 'GSPR', p = fp32(lambda) * |v| in fp32,
    # lambda = k / sum |v|; the message lists the kept (column, value) pairs in ascending column order
    n, N, k, seed = 4, 3001, 500, 9
    r = np.random.default_rng(51)
    v = (r.standard_normal((n, N)) * np.exp(r.standard_normal((n, N)))).astype(np.float32)      # heavy-ish tails
    st = OracleState(n=n, N=N, W=np.eye(n), kind=KIND_GSPAR, k=k, gamma=0.0, eta=0.5, seed=seed, t=6, x=v.copy())
    cv, msg = oracle.step(st, np.zeros_like(v))
    GSPR = int.from_bytes(b"GSPR", "big")
    cap = k + 8 * 23 + 64
    assert len(msg) == n * (8 + 8 * cap)
    for i in range(n):
        words = np.array([oracle.philox4x32_10([j // 4, i, 6, GSPR], [seed, 0])[j % 4] for j in range(N)], dtype=np.uint64)
        assert [oracle.gspar_word(seed, 6, i, j) for j in (0, 1, 5, N - 1)] == [int(words[j]) for j in (0, 1, 5, N - 1)]
        lam = np.float32(k / np.abs(v[i].astype(np.float64)).sum())          # the tree sum differs from this one in the last bits at most
        assert abs(float(lam) - k / oracle.sum_abs_tree(v[i])) <= 1e-7 * float(lam)
        lam = np.float32(k / oracle.sum_abs_tree(v[i]))
        p = lam * np.abs(v[i])                                               # fp32 product
        assert p.dtype == np.float32
        u = ((words >> np.uint64(8)).astype(np.float64) / 2.0 ** 24).astype(np.float32)     # exact in fp32
        keep = u < p
        assert 0.5 * k < keep.sum() < 1.5 * k
        np.testing.assert_array_equal(cv[i], np.where(keep, v[i], np.float32(0)))
        np.testing.assert_array_equal(st.delta[i], np.where(keep, np.float32(0), v[i]))
        row = msg[i * (8 + 8 * cap):(i + 1) * (8 + 8 * cap)]
        head = np.frombuffer(row[:8].tobytes(), np.uint32)
        assert head[0] == keep.sum() and head[1] == 0
        pairs = np.frombuffer(row[8:].tobytes(), np.uint32).reshape(cap, 2)
        np.testing.assert_array_equal(pairs[:head[0], 0], np.nonzero(keep)[0])
        np.testing.assert_array_equal(pairs[:head[0], 1].view(np.float32), v[i][keep])
        assert np.all(pairs[head[0]:] == 0)
    assert oracle.gspar_word(seed, 6, 0, 0) not in (oracle.keep_word(seed, 6, 0, 0), oracle.rounding_word(seed, 6, 0, 0))


def test_gspar_sum_of_magnitudes_is_the_adjacent_pairs_tree_in_double():
    # an input where the balanced tree and a left-to-right sum give different doubles
    v = np.array([1.0, -2.0 ** -53, 2.0 ** -53, -2.0 ** -53, 2.0 ** -60], dtype=np.float32)
    tree = ((1.0 + 2.0 ** -53) + (2.0 ** -53 + 2.0 ** -53)) + ((2.0 ** -60 + 0.0) + (0.0 + 0.0))
    seq = 0.0
    for a in np.abs(v.astype(np.float64)):
        seq += a
    assert tree == 1.0 + 2.0 ** -52 and seq == 1.0
    assert oracle.sum_abs_tree(v) == tree
    big = np.random.default_rng(52).standard_normal(100_003).astype(np.float32)
    assert abs(oracle.sum_abs_tree(big) - np.abs(big.astype(np.float64)).sum()) < 1e-9 * np.abs(big).sum()
    assert oracle.sum_abs_tree(np.zeros(7, np.float32)) == 0.0


def test_gspar_threshold_is_strict_and_uses_24_bits():
    # keep iff u < p with u the top 24 bits of the word.  Four elements whose magnitudes sum to exactly 16 make
    # lambda = k / 16 = 1/8 exact for k = 2; element 0 gets |v| = 8 u_0, so p_0 = u_0 exactly: it must be dropped
    # (u <= p would keep it; so would a u built from 23 bits, since u_0's lowest bit is set).  Element 1 gets the
    # next fp32 above 8 u_1 and must be kept.
    found = 0
    for seed in range(200):
        w0, w1 = oracle.gspar_word(seed, 0, 0, 0) >> 8, oracle.gspar_word(seed, 0, 0, 1) >> 8
        if not (w0 & 1) or not (2 ** 21 < w0 < 2 ** 23) or not (2 ** 21 < w1 < 2 ** 23):
            continue
        a0 = np.float32(8.0 * w0 / 2.0 ** 24)
        a1 = np.nextafter(np.float32(8.0 * w1 / 2.0 ** 24), np.float32(16))
        rest = 16.0 - float(a0) - float(a1)                     # exact in double; split into two fp32
        lo = rest % 2.0 ** -19
        hi = rest - lo
        v = np.array([[a0, -a1, hi, lo]], dtype=np.float32)
        assert float(v[0, 2]) == hi and float(v[0, 3]) == lo and oracle.sum_abs_tree(v[0]) == 16.0
        st = OracleState(n=1, N=4, W=np.ones((1, 1)), kind=KIND_GSPAR, k=2, gamma=0.0, eta=0.5, seed=seed, x=v.copy())
        cv, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
        assert cv[0, 0] == 0 and cv[0, 1] == -a1
        found += 1
        if found == 3:
            break
    assert found == 3


def test_gspar_probabilities_rate_and_signal_to_noise():
    # over many steps (fresh masks) the keep frequency of an element is min(1, lambda |v_j|); the expected count is
    # k when nothing is cut off; E|C[v] - v|^2 = sum v_j^2 (1 - p_j) < |v|^2: Assumption 1.6 with alpha < 1
    N, k, T = 2000, 300, 400
    r = np.random.default_rng(53)
    v = r.standard_normal((1, N))
    lam = k / np.abs(v[0]).sum()
    p = np.minimum(1.0, lam * np.abs(v[0]))
    assert p.max() < 1.0 and abs(p.sum() - k) < 1e-9 * k
    freq = np.zeros(N)
    err = 0.0
    st = OracleState(n=1, N=N, W=np.ones((1, 1)), kind=KIND_GSPAR, k=k, gamma=0.0, eta=0.5, seed=4, dtype=np.float64, x=v.copy())
    counts = []
    for t in range(T):
        st.x[:], st.delta[:] = v, 0.0
        cv, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
        kept = cv[0] != 0
        np.testing.assert_array_equal(cv[0][kept], v[0][kept])             # kept values are exact, no rescaling
        freq += kept
        counts.append(kept.sum())
        err += ((cv[0] - v[0]) ** 2).sum()
    sd = np.sqrt(p * (1 - p) / T)
    assert np.all(np.abs(freq / T - p) < 5 * sd + 1e-12)
    assert abs(np.mean(counts) - k) < 5 * np.sqrt((p * (1 - p)).sum() / T)
    want = (v[0] ** 2 * (1 - p)).sum()
    assert abs(err / T - want) < 0.02 * want and want < (v[0] ** 2).sum()
    # larger magnitudes are kept more often: the operator is not the uniform mask of the random sparsifier
    order = np.argsort(np.abs(v[0]))
    assert freq[order[-200:]].mean() > 3 * freq[order[:200]].mean()


def test_gspar_cut_off_probabilities_zero_vector_and_k_equal_N():
    # one dominant element: lambda |v_j| >= 1, so it is kept at every step and the expected count stays below k
    N, k = 512, 64
    v = np.full((1, N), 1e-3, dtype=np.float32)
    v[0, 77] = 50.0
    for t in range(20):
        st = OracleState(n=1, N=N, W=np.ones((1, 1)), kind=KIND_GSPAR, k=k, gamma=0.0, eta=0.5, seed=2, t=t, x=v.copy())
        cv, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
        assert cv[0, 77] == np.float32(50.0)
        assert (cv[0] != 0).sum() < k
    # all-zero vector: nothing is kept, the message is an empty list
    st = OracleState(n=1, N=N, W=np.ones((1, 1)), kind=KIND_GSPAR, k=k, gamma=0.0, eta=0.5)
    cv, msg = oracle.step(st, np.zeros((1, N), np.float32))
    assert not cv.any() and not msg.any()
    # k = N on a constant-magnitude vector: every p_j = 1 up to rounding of lambda; u < 1 always, so all are kept
    v = np.where(np.random.default_rng(54).random((1, 64)) < 0.5, -2.0, 2.0).astype(np.float32)
    st = OracleState(n=1, N=64, W=np.ones((1, 1)), kind=KIND_GSPAR, k=64, gamma=0.0, eta=0.5, x=v.copy())
    cv, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
    np.testing.assert_array_equal(cv, v)


# ----------------------------------------------------------------------------- P7: quantiser

def test_quantiser_worked_example(golden_dir):
    rec = {l.split()[0]: l.split()[1:] for l in open(os.path.join(golden_dir, "quant_2bit_micro.txt"))
           if l[0] != "#"}
    v = np.array([[float(t) for t in rec["v"]]], dtype=np.float32)
    seen = set()
    for seed in range(40):
        st = OracleState(n=1, N=4, W=np.ones((1, 1)), kind=KIND_QUANT_MAXABS, bits=2, block=1024,
                         gamma=0.0, eta=0.5, seed=seed, x=v.copy())
        cv, msg = oracle.step(st, np.zeros((1, 4), np.float32))
        u = (oracle.rounding_word(seed, 0, 0, 2) >> 8) / 2.0 ** 24
        case = "up" if u < 0.75 else "down"
        seen.add(case)
        r = rec[case]
        codes = [int(c) for c in r[1:5]]
        c = [float(c) for c in r[6:10]]
        d = [float(c) for c in r[11:15]]
        assert msg.tobytes()[:4] == np.float32(float(rec["scale"][0])).tobytes()
        assert msg[4] == int(r[16], 16) and list(msg[5:8]) == [0, 0, 0]
        assert list(unpack_codes(np.frombuffer(msg[4:8].tobytes(), np.uint32), 2, 4)) == codes
        np.testing.assert_array_equal(cv[0], np.array(c, np.float32))
        np.testing.assert_array_equal(st.delta[0], np.array(d, np.float32))
        # W = [1]: W - I = 0, so x moves by -gamma g only
        np.testing.assert_array_equal(st.x, v)
    assert seen == {"up", "down"}


@pytest.mark.parametrize("bits,block", [(4, 512), (2, 1024), (8, 256)])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_quantiser_is_unbiased_bounded_and_on_grid(bits, block, dtype):
    # every block holds the same pattern, so position e sees `reps` independent roundings of one value
    reps, L = 2048, (1 << bits) - 1
    r = np.random.default_rng(7)
    pat = r.uniform(-1, 1, block)
    pat[0], pat[1], pat[2] = 1.0, -1.0, 0.0               # scale exactly 1
    v = np.tile(pat, reps)[None, :].astype(dtype)
    st = OracleState(n=1, N=block * reps, W=np.ones((1, 1)), kind=KIND_QUANT_MAXABS, bits=bits, block=block,
                     gamma=0.0, eta=0.5, seed=9, dtype=dtype, x=v.copy())
    cv, msg = oracle.step(st, np.zeros_like(v), want_msg=(dtype == np.float32))
    c = cv.reshape(reps, block).astype(np.float64)
    step_sz = 2.0 / L
    grid = (2 * np.arange(L + 1) - L) / L
    lvl = (c + 1.0) * (L / 2.0)                                                    # on the grid: an integer level
    assert np.all(np.abs(lvl - np.rint(lvl)) < 1e-4) and lvl.min() > -1e-4 and lvl.max() < L + 1e-4
    assert np.all(np.abs(c - pat) <= step_sz * (1 + 1e-6))                        # error bound
    assert np.all(c[:, 0] == 1.0) and np.all(c[:, 1] == -1.0)                     # extremes exact
    sem = step_sz / 2 / np.sqrt(reps)
    assert np.all(np.abs(c.mean(0) - v[0, :block].astype(np.float64)) < 5 * sem)  # E[C[v]] = v
    # both neighbours of an off-grid value do occur, and draws of the 4 elements of one group differ
    assert len(np.unique(c[:, 2])) == 2
    up = c > pat
    assert 0.2 < np.mean(up[:, 4] != up[:, 5]) < 0.8
    if dtype == np.float32:
        # the packed words decode (independently) to the same values
        dec = []
        for s, w, m in split_block_message(msg, block * reps, block, bits):
            assert s == np.float32(1.0)
            q = unpack_codes(w, bits, m)
            dec.append((2 * q - L) * (np.float32(1.0) / np.float32(L)))
        np.testing.assert_array_equal(np.concatenate(dec).astype(np.float32), cv[0])


def test_quantiser_ragged_tail_and_zero_block():
    bits, block, N = 4, 64, 64 * 3 + 10
    r = np.random.default_rng(8)
    v = r.standard_normal((2, N)).astype(np.float32)
    v[1, 64:128] = 0.0                                      # an all-zero block
    st = OracleState(n=2, N=N, W=np.eye(2), kind=KIND_QUANT_MAXABS, bits=bits, block=block, gamma=0.0, eta=0.5,
                     x=v.copy())
    cv, msg = oracle.step(st, np.zeros_like(v))
    assert len(msg) == 2 * (3 * (4 + 32) + 4 + 8)           # tail: 10 codes -> 2 words
    per = len(msg) // 2
    for i in range(2):
        j0 = 0
        for s, w, m in split_block_message(msg[i * per:(i + 1) * per], N, block, bits):
            assert s == np.abs(v[i, j0:j0 + m]).max()
            q = unpack_codes(w, bits, m)
            if s == 0:
                assert np.all(q == 0) and np.all(cv[i, j0:j0 + m] == 0)
            if m < block:                                   # padding codes of the tail word are zero
                assert int(w[-1]) >> (bits * (m % 8)) == 0
            np.testing.assert_array_equal(((2 * q - 15) * (s / np.float32(15))).astype(np.float32),
                                          cv[i, j0:j0 + m])
            j0 += m
    np.testing.assert_array_equal(st.delta, v - cv)


# ----------------------------------------------------------------------------- sign compressor

@pytest.mark.parametrize("N,block", [(256 * 3 + 40, 256), (100, 8), (5, 16)])
def test_sign_scale_is_block_mean_and_contracts(N, block):
    r = np.random.default_rng(9)
    v = r.standard_normal((1, N))
    v[0, 3] = 0.0
    st = OracleState(n=1, N=N, W=np.ones((1, 1)), kind=KIND_SIGN_MEANABS, block=block, gamma=0.0, eta=0.5,
                     dtype=np.float64, x=v.copy())
    cv, _ = oracle.step(st, np.zeros_like(v), want_msg=False)
    for j0 in range(0, N, block):
        blk = v[0, j0:j0 + block]
        s = np.abs(blk).mean()                               # mean over the real elements of a ragged tail
        np.testing.assert_allclose(cv[0, j0:j0 + block], np.where(np.signbit(blk), -s, s), rtol=1e-14)
        # Assumption 1.6 holds deterministically: |v - C|^2 = |v|^2 - m s^2 <= (1 - 1/m) |v|^2
        err = ((blk - cv[0, j0:j0 + block]) ** 2).sum()
        assert err <= (1 - 1.0 / len(blk)) * (blk ** 2).sum() + 1e-12


def test_sign_of_negative_zero_is_negative():
    # the code is the IEEE sign bit: -0.0 is sent as "negative" and decodes to -scale
    v = np.array([[1.0, -0.0, 0.0, -3.0]], dtype=np.float32)
    # (v = (x - gamma g) + delta keeps the sign of a zero only if delta's zero has it too: -0 + +0 = +0)
    d = np.array([[0.0, -0.0, 0.0, 0.0]], dtype=np.float32)
    st = OracleState(n=1, N=4, W=np.ones((1, 1)), kind=KIND_SIGN_MEANABS, block=4, gamma=0.0, eta=0.5, x=v.copy(), delta=d)
    cv, msg = oracle.step(st, np.zeros_like(v))
    np.testing.assert_array_equal(cv[0], np.float32([1.0, -1.0, 1.0, -1.0]))
    assert np.frombuffer(msg[4:8].tobytes(), np.uint32)[0] == 0b1010 and np.frombuffer(msg[:4].tobytes(), np.float32)[0] == 1.0


def test_sign_fp32_sum_is_the_pairwise_tree():
    # fp32 sums depend on the order; the oracle's must be the balanced pairwise tree over the padded block
    block, N = 256, 256 + 40
    r = np.random.default_rng(10)
    v = (r.standard_normal((1, N)) * 10 ** r.uniform(-3, 3, (1, N))).astype(np.float32)
    st = OracleState(n=1, N=N, W=np.ones((1, 1)), kind=KIND_SIGN_MEANABS, block=block, gamma=0.0, eta=0.5,
                     x=v.copy())
    _, msg = oracle.step(st, np.zeros_like(v))
    got = [s for s, _, _ in split_block_message(msg, N, block, 1)]

    def tree(a):
        return a[0] if len(a) == 1 else np.float32(tree(a[:len(a) // 2]) + tree(a[len(a) // 2:]))
    for b, j0 in enumerate(range(0, N, block)):
        a = np.zeros(block, np.float32)
        m = min(block, N - j0)
        a[:m] = np.abs(v[0, j0:j0 + m])
        assert got[b] == np.float32(tree(a) / np.float32(m))
    sequential = np.float32(0)
    for val in np.abs(v[0, :block]):
        sequential = np.float32(sequential + val)
    assert sequential / np.float32(block) != got[0]          # the test can tell the orders apart


# ----------------------------------------------------------------------------- P8: top-k

def brute_force_topk(v, k):
    order = sorted(range(len(v)), key=lambda j: (-abs(float(v[j])), j))
    return sorted(order[:k])


@pytest.mark.parametrize("case", ["random", "all_equal", "plus_minus_pairs", "ties_at_threshold", "k_eq_N"])
def test_topk_matches_full_sort(case):
    N, k = 1000, 37
    r = np.random.default_rng(12)
    if case == "random":
        v = r.standard_normal(N)
    elif case == "all_equal":
        v = np.full(N, -2.5)
    elif case == "plus_minus_pairs":
        a = r.standard_normal(N // 2)
        v = np.concatenate([a, -a])[r.permutation(N)]
    elif case == "ties_at_threshold":
        v = r.integers(-6, 7, N).astype(np.float64)
    else:
        v, k = r.standard_normal(N), N
    v = v.astype(np.float32)[None, :]
    st = OracleState(n=1, N=N, W=np.ones((1, 1)), kind=KIND_TOPK, k=k, gamma=0.0, eta=0.5, x=v.copy())
    cv, msg = oracle.step(st, np.zeros_like(v))
    keep = brute_force_topk(v[0], k)
    pairs = np.frombuffer(msg.tobytes(), dtype=np.dtype([("j", "<u4"), ("v", "<f4")]))
    assert list(pairs["j"]) == keep                          # ascending index, ties to the lower index
    np.testing.assert_array_equal(pairs["v"], v[0, keep])
    expect = np.zeros(N, np.float32)
    expect[keep] = v[0, keep]
    np.testing.assert_array_equal(cv[0], expect)
    np.testing.assert_array_equal(st.delta[0], v[0] - expect)
    if case == "all_equal":
        assert keep == list(range(k))
    # Assumption 1.6 with alpha^2 = 1 - k/N
    assert ((v[0] - cv[0]) ** 2).sum() <= (1 - k / N) * (v[0] ** 2).sum() * (1 + 1e-6)


# ----------------------------------------------------------------------------- float vs double, messages, misc

@pytest.mark.parametrize("comp", [COMPRESSORS[2], COMPRESSORS[3]])
def test_fp32_and_fp64_runs_agree_for_deterministic_compressors(comp):
    n, N, T = 6, 80, 5
    W = oracle.ring_matrix(n)
    r = np.random.default_rng(13)
    gs = r.standard_normal((T, n, N)).astype(np.float32)
    a = OracleState(n=n, N=N, W=W, gamma=0.1, eta=0.3, **comp)
    b = OracleState(n=n, N=N, W=W, gamma=float(np.float32(0.1)), eta=float(np.float32(0.3)), dtype=np.float64, **comp)
    for g in gs:
        oracle.step(a, g, want_msg=False)
        oracle.step(b, g.astype(np.float64), want_msg=False)
    np.testing.assert_allclose(a.x, b.x, rtol=0, atol=2e-5)
    np.testing.assert_allclose(a.delta, b.delta, rtol=0, atol=2e-5)


def test_identity_message_is_v_and_step_counter_advances():
    n, N = 3, 9
    r = np.random.default_rng(14)
    x0, d0, g = r.standard_normal((3, n, N)).astype(np.float32)
    st = OracleState(n=n, N=N, W=oracle.ring_matrix(n), kind=KIND_IDENTITY, gamma=0.5, eta=0.5,
                     x=x0.copy(), delta=d0.copy())
    cv, msg = oracle.step(st, g)
    assert st.t == 1
    np.testing.assert_array_equal(np.frombuffer(msg.tobytes(), np.float32).reshape(n, N), cv)
    np.testing.assert_array_equal(st.delta, 0)


def test_stochastic_rounding_depends_on_step_and_seed_only_through_the_counter():
    # same (seed, t) -> same codes (restartable); another t or seed -> other codes
    n, N = 2, 256
    r = np.random.default_rng(15)
    x0 = r.standard_normal((n, N)).astype(np.float32)
    g = np.zeros((n, N), np.float32)

    def codes(seed, t):
        st = OracleState(n=n, N=N, W=np.eye(n), kind=KIND_QUANT_MAXABS, bits=4, block=64, gamma=0.0, eta=0.5,
                         seed=seed, t=t, x=x0.copy())
        return oracle.step(st, g)[1]
    assert np.array_equal(codes(1, 5), codes(1, 5))
    assert not np.array_equal(codes(1, 5), codes(1, 6))
    assert not np.array_equal(codes(1, 5), codes(2, 5))


def test_ring_and_torus_matrices():
    for n in (3, 8, 16):
        W = oracle.ring_matrix(n)
        np.testing.assert_allclose(W, W.T)
        np.testing.assert_allclose(W.sum(1), 1)
        ev = np.sort(np.linalg.eigvalsh(W))
        np.testing.assert_allclose(ev, np.sort(1 / 3 + 2 / 3 * np.cos(2 * np.pi * np.arange(n) / n)), atol=1e-12)
    W = oracle.torus_matrix(8, 8)
    np.testing.assert_allclose(W, W.T)
    np.testing.assert_allclose(W.sum(1), 1)
    assert np.all((W > 0).sum(1) == 5)
    k = np.arange(8)
    ev = (1 + 2 * np.cos(2 * np.pi * k[:, None] / 8) + 2 * np.cos(2 * np.pi * k[None, :] / 8)) / 5
    np.testing.assert_allclose(np.sort(np.linalg.eigvalsh(W)), np.sort(ev.ravel()), atol=1e-12)
    # eta <= 1/2 keeps W_eff positive semi-definite (used by the paper's proof of Theorem 1)
    assert np.linalg.eigvalsh(0.5 * np.eye(64) + 0.5 * W).min() > -1e-12


def test_diagnostics_definitions():
    n, N = 5, 40
    r = np.random.default_rng(22)
    W = metropolis_matrix(n, 3, seed=2)
    st = OracleState(n=n, N=N, W=W, gamma=0.1, eta=0.4, dtype=np.float64, x=r.standard_normal((n, N)),
                     delta=r.standard_normal((n, N)), **COMPRESSORS[2])
    d = oracle.diagnostics(st)
    X, D = st.x, st.delta
    # ||X(I - A_n)||_F^2 = ||X||_F^2 - n |mean|^2 ; ||Delta (W_eff - I)||_F^2 with W_eff = (1-eta) I + eta W
    np.testing.assert_allclose(d["consensus_sq"], (X ** 2).sum() - n * (X.mean(0) ** 2).sum(), rtol=1e-12)
    Weff = 0.6 * np.eye(n) + 0.4 * W
    np.testing.assert_allclose(d["delta_mixed_sq"], np.linalg.norm((Weff - np.eye(n)) @ D, "fro") ** 2, rtol=1e-12)
    np.testing.assert_allclose(d["delta_sq"], np.linalg.norm(D, "fro") ** 2, rtol=1e-12)
    # complete-graph averaging with eta = 1 and no compression reaches consensus in one step, with nothing carried over
    st = OracleState(n=n, N=N, W=np.full((n, n), 1.0 / n), kind=KIND_IDENTITY, gamma=0.0, eta=1.0, dtype=np.float64,
                     x=r.standard_normal((n, N)))
    oracle.step(st, np.zeros((n, N)), want_msg=False)
    d = oracle.diagnostics(st)
    assert d["consensus_sq"] < 1e-25 and d["delta_sq"] == 0.0 and d["delta_mixed_sq"] == 0.0


def test_all_cores_build_gives_the_same_bits():
    """The library built with -fopenmp (workers side by side, used only by the benchmark's baseline leg) and the
    sequential one are the same program: every output equal bit for bit, for every operator."""
    rng = np.random.default_rng(77)
    n, N = 6, 3000
    for kind, kw in ((oracle.KIND_QUANT_MAXABS, dict(bits=2, block=256)), (oracle.KIND_SIGN_MEANABS, dict(block=128)),
                     (oracle.KIND_TOPK, dict(k=37)), (oracle.KIND_QUANT_L2NORM, dict(bits=4)),
                     (oracle.KIND_RAND_SPARSE, dict(k=300)), (oracle.KIND_GSPAR, dict(k=300)), (oracle.KIND_IDENTITY, {})):
        outs = []
        for all_cores in (False, True):
            st = oracle.OracleState(n=n, N=N, W=oracle.ring_matrix(n), kind=kind, gamma=0.1, eta=0.4, seed=3, **kw)
            r = np.random.default_rng(5)
            msgs = []
            for t in range(3):
                g = r.standard_normal((n, N)).astype(np.float32)
                cv, msg = oracle.step(st, g, all_cores=all_cores)
                msgs.append((cv, msg))
            outs.append((st.x, st.delta, msgs))
        a, b_ = outs
        assert np.array_equal(a[0].view(np.uint32), b_[0].view(np.uint32))
        assert np.array_equal(a[1].view(np.uint32), b_[1].view(np.uint32))
        for (cv0, m0), (cv1, m1) in zip(a[2], b_[2]):
            assert np.array_equal(cv0.view(np.uint32), cv1.view(np.uint32)) and np.array_equal(m0, m1)
    assert oracle.threads() == 1 and oracle.threads(all_cores=True) >= 1
