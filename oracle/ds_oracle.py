"""ctypes front end of the CPU oracle (``ds_oracle.cpp``) -- test infrastructure.

The arithmetic of the method lives in the C++ file; this module only builds it
with g++, marshals numpy arrays, and offers the small dense helpers (mixing
matrices of a ring and of a 2-D torus, CSR conversion) that tests need to state
the paper's matrix identities.  Nothing here is used by the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

KIND_IDENTITY = 0      # C[v] = v: DeepSqueeze reduces to D-PSGD (paper, "Consistence with D-PSGD")
KIND_QUANT_MAXABS = 1  # stochastic b-bit block quantisation, max-abs scale
KIND_SIGN_MEANABS = 2  # sign bit + block mean-abs scale
KIND_TOPK = 3          # k largest magnitudes of the whole vector
KIND_QUANT_L2NORM = 4  # b-bit codes over the whole vector + its Euclidean norm (the paper's experiments)
KIND_RAND_SPARSE = 5   # every element kept with probability k/N, no rescaling
KIND_GSPAR = 6         # element j kept with probability min(1, k |v_j| / sum |v|), no rescaling; (column, value) pairs

ALGO_DEEPSQUEEZE = 0   # Algorithm 1
ALGO_DCD_PSGD = 1      # compressed difference of the model update ("Why DeepSqueeze is better", DCD-PSGD item)
ALGO_CHOCO_SGD = 2     # compressed difference to a public copy, gossip on the copies (same section, CHOCO-SGD item)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ds_oracle.cpp")
_LIB = os.path.join(_HERE, "libds_oracle.so")
_LIB_OMP = os.path.join(_HERE, "libds_oracle_omp.so")     # same source with -fopenmp: the benchmark's all-cores baseline
_lib = None
_lib_omp = None


def build_oracle(force: bool = False, omp: bool = False) -> str:
    """Compile the oracle with g++ (contraction off, no fast-math). Returns the .so path.

    omp=True builds the second library, in which the loops over workers run on all host cores."""
    out = _LIB_OMP if omp else _LIB
    stale = (not os.path.exists(out)) or os.path.getmtime(out) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               *(["-fopenmp"] if omp else []), _SRC, "-o", out]
        subprocess.run(cmd, check=True)
    return out


def threads(all_cores: bool = False) -> int:
    """Threads a step runs on: 1, or what OpenMP gives the all-cores library."""
    return int(_load(all_cores).dso_threads())


def _load(omp: bool = False):
    global _lib, _lib_omp
    if omp and _lib_omp is not None:
        return _lib_omp
    if not omp and _lib is not None:
        return _lib
    lib = ctypes.CDLL(build_oracle(omp=omp))
    u64, i32, u32 = ctypes.c_uint64, ctypes.c_int, ctypes.c_uint32
    vp = ctypes.c_void_p
    for name, real in (("dso_step_f32", ctypes.c_float), ("dso_step_f64", ctypes.c_double)):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [i32, u64, vp, vp, vp, i32, i32, u64, u64, real, real, u64, u64,
                       vp, vp, vp, vp, vp, u64, ctypes.POINTER(u64)]
    for name, real in (("dso_compare_step_f32", ctypes.c_float), ("dso_compare_step_f64", ctypes.c_double)):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [i32, i32, u64, vp, vp, vp, i32, i32, u64, u64, real, real, u64, u64,
                       vp, vp, vp, vp, vp, u64, ctypes.POINTER(u64)]
    lib.dso_step_window_f32.restype = ctypes.c_int
    lib.dso_step_window_f32.argtypes = [i32, u64, u64, vp, vp, vp, i32, i32, u64, ctypes.c_float, ctypes.c_float,
                                        u64, u64, vp, vp, vp, vp, u64, ctypes.POINTER(u64)]
    lib.dso_philox4x32_10.restype = None
    lib.dso_philox4x32_10.argtypes = [vp, vp, vp]
    lib.dso_rounding_word.restype = u32
    lib.dso_rounding_word.argtypes = [u64, u64, u32, u64]
    lib.dso_keep_word.restype = u32
    lib.dso_keep_word.argtypes = [u64, u64, u32, u64]
    lib.dso_gspar_word.restype = u32
    lib.dso_gspar_word.argtypes = [u64, u64, u32, u64]
    lib.dso_sum_abs_tree_f32.restype = ctypes.c_double
    lib.dso_sum_abs_tree_f32.argtypes = [vp, u64]
    lib.dso_rand_sparse_capacity.restype = u64
    lib.dso_rand_sparse_capacity.argtypes = [u64, u64]
    lib.dso_sum_squares_tree_f32.restype = ctypes.c_double
    lib.dso_sum_squares_tree_f32.argtypes = [vp, u64]
    lib.dso_threads.restype = ctypes.c_int
    lib.dso_threads.argtypes = []
    if omp:
        _lib_omp = lib
    else:
        _lib = lib
    return lib


def philox4x32_10(counter, key):
    """Philox4x32-10 block function: 4 counter words, 2 key words -> 4 output words."""
    lib = _load()
    c = np.asarray(counter, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    lib.dso_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def rounding_word(seed: int, t: int, i: int, j: int) -> int:
    """The 32-bit word that decides the stochastic rounding of element (i, j) at step t."""
    return int(_load().dso_rounding_word(seed, t, i, j))


def keep_word(seed: int, t: int, i: int, j: int) -> int:
    """The 32-bit word that decides whether the random sparsifier keeps element (i, j) at step t."""
    return int(_load().dso_keep_word(seed, t, i, j))


def gspar_word(seed: int, t: int, i: int, j: int) -> int:
    """The 32-bit word that decides whether the magnitude-proportional sparsifier keeps element (i, j) at step t."""
    return int(_load().dso_gspar_word(seed, t, i, j))


def sum_abs_tree(v) -> float:
    """Sum of |v| of a float32 vector in float64, balanced adjacent-pairs tree over the zero-padded vector."""
    a = np.ascontiguousarray(v, dtype=np.float32)
    return float(_load().dso_sum_abs_tree_f32(a.ctypes.data, a.size))


def rand_sparse_capacity(N: int, k: int) -> int:
    """Values a worker's random-sparsification message has room for: min(N, k + 8 ceil(sqrt k) + 64)."""
    return int(_load().dso_rand_sparse_capacity(N, k))


def sum_squares_tree(v) -> float:
    """Sum of squares of a float32 vector in float64, balanced adjacent-pairs tree over the zero-padded vector."""
    a = np.ascontiguousarray(v, dtype=np.float32)
    return float(_load().dso_sum_squares_tree_f32(a.ctypes.data, a.size))


# --- dense helpers for the tests' matrix identities --------------------------------------------

def ring_matrix(n: int) -> np.ndarray:
    """W of a ring: 1/3 on the diagonal and on the two cyclic neighbours (float64)."""
    assert n >= 3
    W = np.zeros((n, n))
    for i in range(n):
        for j in (i - 1, i, i + 1):
            W[i, j % n] = 1.0 / 3.0
    return W


def torus_matrix(rows: int, cols: int) -> np.ndarray:
    """W of a rows x cols 2-D torus (node id = r*cols + c): 1/5 on self and the 4 neighbours."""
    assert rows >= 3 and cols >= 3
    n = rows * cols
    W = np.zeros((n, n))
    for r in range(rows):
        for c in range(cols):
            i = r * cols + c
            for rr, cc in ((r, c), (r - 1, c), (r + 1, c), (r, c - 1), (r, c + 1)):
                W[i, (rr % rows) * cols + (cc % cols)] = 0.2
    return W


def dense_to_csr(W: np.ndarray):
    """CSR (rowptr, col, val) of W with ascending columns; the diagonal is always stored."""
    n = W.shape[0]
    rowptr, col, val = [0], [], []
    for i in range(n):
        for j in range(n):
            if W[i, j] != 0.0 or i == j:
                col.append(j)
                val.append(W[i, j])
        rowptr.append(len(col))
    return (np.asarray(rowptr, dtype=np.int32), np.asarray(col, dtype=np.int32),
            np.asarray(val, dtype=np.float64))


def message_bytes(kind: int, n: int, N: int, bits: int = 0, block: int = 0, k: int = 0) -> int:
    """Size of one step's packed messages for all n workers."""
    if kind == KIND_IDENTITY:
        return n * N * 4
    if kind == KIND_TOPK:
        return n * k * 8
    if kind == KIND_QUANT_L2NORM:
        return n * (4 + 4 * ((N * bits + 31) // 32))
    if kind == KIND_RAND_SPARSE:
        return n * (4 + 4 * rand_sparse_capacity(N, k))
    if kind == KIND_GSPAR:
        return n * (8 + 8 * rand_sparse_capacity(N, k))
    b = bits if kind == KIND_QUANT_MAXABS else 1
    full, tail = divmod(N, block)
    per_row = full * (4 + 4 * ((block * b + 31) // 32))
    if tail:
        per_row += 4 + 4 * ((tail * b + 31) // 32)
    return n * per_row


@dataclass
class OracleState:
    """x, delta (n x N), the step counter and the fixed parameters of a run.

    algo selects the update rule; for ALGO_CHOCO_SGD `delta` holds the workers' public copies xhat, for
    ALGO_DCD_PSGD it is not used."""
    n: int
    N: int
    W: np.ndarray                      # dense n x n, float64
    kind: int
    gamma: float
    eta: float
    bits: int = 0
    block: int = 0
    k: int = 0
    seed: int = 0
    dtype: type = np.float32
    t: int = 0
    algo: int = ALGO_DEEPSQUEEZE
    x: np.ndarray = field(default=None, repr=False)
    delta: np.ndarray = field(default=None, repr=False)

    def __post_init__(self):
        if self.x is None:             # Algorithm 1, line 1 and Assumption 1.4: start from zero
            self.x = np.zeros((self.n, self.N), dtype=self.dtype)
        if self.delta is None:
            self.delta = np.zeros((self.n, self.N), dtype=self.dtype)
        self._csr = dense_to_csr(np.asarray(self.W, dtype=np.float64))

    def set_W(self, W: np.ndarray):
        """Use another mixing matrix from the next step on (time-varying graph)."""
        self.W = W
        self._csr = dense_to_csr(np.asarray(W, dtype=np.float64))


def diagnostics(st: OracleState) -> dict:
    """The quantities the paper's analysis tracks, from their definitions in float64 (rows = workers):
    consensus_sq   = ||X (I - A_n)||_F^2 = sum_i |x_i - mean_i x_i|^2     (supplement, proof of Lemma 1)
    delta_sq       = ||Delta||_F^2
    delta_mixed_sq = ||Delta (W_eff - I)||_F^2, W_eff - I = eta (W - I)    (section "Why DeepSqueeze is better")
    """
    X = st.x.astype(np.float64)
    D = st.delta.astype(np.float64)
    if st.dtype == np.float32:      # the coefficients an fp32 run mixes with: W and W - I rounded to fp32
        A = (np.asarray(st.W, dtype=np.float32) - np.eye(st.n, dtype=np.float32)).astype(np.float64)
        eta = float(np.float32(st.eta))
    else:
        A = np.asarray(st.W, dtype=np.float64) - np.eye(st.n)
        eta = float(st.eta)
    mixed = eta * A @ D
    return {"consensus_sq": float(((X - X.mean(0)) ** 2).sum()), "delta_sq": float((D ** 2).sum()),
            "delta_mixed_sq": float((mixed ** 2).sum())}


def step_window(st: OracleState, g: np.ndarray, col0: int):
    """One fp32 step on the columns [col0, col0 + st.N) of a wider problem (per-block operators and identity
    only; col0 a multiple of the block size).  `st` holds the window's x and delta.  Returns the window's message."""
    lib = _load()
    assert st.dtype == np.float32
    g = np.ascontiguousarray(g, dtype=np.float32)
    assert g.shape == (st.n, st.N)
    rowptr, col, val = st._csr
    wval = np.ascontiguousarray(val, dtype=np.float32)
    cap = message_bytes(st.kind, st.n, st.N, st.bits, st.block, st.k)
    msg = np.zeros(cap, dtype=np.uint8)
    used = ctypes.c_uint64(0)
    rc = lib.dso_step_window_f32(st.n, st.N, col0, rowptr.ctypes.data, col.ctypes.data, wval.ctypes.data,
                                 st.kind, st.bits, st.block, st.gamma, st.eta, st.seed, st.t,
                                 st.x.ctypes.data, st.delta.ctypes.data, g.ctypes.data,
                                 msg.ctypes.data, cap, ctypes.byref(used))
    if rc != 0:
        raise RuntimeError(f"oracle window step failed with code {rc}")
    st.t += 1
    assert used.value == cap
    return msg


def step(st: OracleState, g: np.ndarray, want_cv: bool = True, want_msg: bool = True, all_cores: bool = False):
    """Advance `st` by one iteration with gradients g (n x N). Returns (C[v], message bytes).

    all_cores=True runs the same code from the library built with -fopenmp (workers side by side)."""
    lib = _load(all_cores)
    dt = np.dtype(st.dtype)
    assert dt in (np.dtype(np.float32), np.dtype(np.float64))
    g = np.ascontiguousarray(g, dtype=dt)
    assert g.shape == (st.n, st.N)
    assert st.x.dtype == dt and st.delta.dtype == dt and st.x.flags.c_contiguous and st.delta.flags.c_contiguous
    rowptr, col, val = st._csr
    wval = np.ascontiguousarray(val, dtype=dt)     # fp32 run: W rounded once to fp32
    cv = np.empty((st.n, st.N), dtype=dt) if want_cv else None
    cap = message_bytes(st.kind, st.n, st.N, st.bits, st.block, st.k) if want_msg else 0
    msg = np.zeros(cap, dtype=np.uint8) if want_msg else None
    used = ctypes.c_uint64(0)
    f32 = dt == np.dtype(np.float32)
    if st.algo == ALGO_DEEPSQUEEZE:
        fn = lib.dso_step_f32 if f32 else lib.dso_step_f64
    else:
        compare = lib.dso_compare_step_f32 if f32 else lib.dso_compare_step_f64
        fn = lambda *a: compare(st.algo, *a)
    rc = fn(st.n, st.N, rowptr.ctypes.data, col.ctypes.data, wval.ctypes.data,
            st.kind, st.bits, st.block, st.k, st.gamma, st.eta, st.seed, st.t,
            st.x.ctypes.data, st.delta.ctypes.data, g.ctypes.data,
            cv.ctypes.data if want_cv else None,
            msg.ctypes.data if want_msg else None, cap, ctypes.byref(used))
    if rc != 0:
        raise RuntimeError(f"oracle step failed with code {rc}")
    st.t += 1
    if want_msg:
        assert used.value == cap, (used.value, cap)
    return cv, msg
