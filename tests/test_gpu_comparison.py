"""GPU parity of the two comparison updates (DS_ALGO_DCD_PSGD, DS_ALGO_CHOCO_SGD) against the CPU oracle.

Same bar as for Algorithm 1 (tests/test_gpu_parity.py): packed messages bit for bit; x and the second state array
(the public copies xhat of CHOCO-SGD; untouched by DCD-PSGD) within 1e-6 relative per element per step and 1e-5
relative L2 after a run.  The kernels reproduce the oracle's fp32 expression order, so the tests also insist on
zero elements differing bitwise.
"""
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from paper_1907_07346_amd import binding as b
from paper_1907_07346_amd import workloads as wl
from test_gpu_parity import (_full_size_free_run, assert_close, free_run, lock_step, oracle_state, say, small, upload)

pytestmark = pytest.mark.gpu

ALGOS = [(wl.ALGO_DCD_PSGD, "dcd"), (wl.ALGO_CHOCO_SGD, "choco")]


def with_algo(w, algo, tag):
    return replace(w, algo=algo, name=f"{tag}_{w.name}")


SHAPES = [
    small(wl.KIND_QUANT_MAXABS, 8, 512 * 5 + 37, bits=4, block=512),
    small(wl.KIND_QUANT_MAXABS, 16, 1024 * 3 + 74, bits=2, block=1024),             # 2 rows per wave
    small(wl.KIND_QUANT_MAXABS, 3, 256 * 4, bits=4, block=256),
    small(wl.KIND_QUANT_MAXABS, 5, 100, bits=2, block=256),                         # one ragged block
    small(wl.KIND_QUANT_MAXABS, 20, 1024 * 2 + 1, bits=4, block=1024),
    small(wl.KIND_QUANT_MAXABS, 64, 512 * 3 + 300, bits=4, block=512, topo=wl.TOPO_TORUS2D, torus=(8, 8)),   # 128 KB of LDS
    small(wl.KIND_QUANT_MAXABS, 70, 512 * 2 + 5, bits=2, block=512),                # looped rows (re-read x, g)
    small(wl.KIND_QUANT_MAXABS, 12, 2048 * 2 + 2000, bits=4, block=2048),
    small(wl.KIND_QUANT_MAXABS, 15, 512 * 4 + 4, bits=2, block=512, topo=wl.TOPO_TORUS2D, torus=(3, 5)),
    small(wl.KIND_QUANT_MAXABS, 150, 256 + 5, bits=4, block=256),                   # 150 KB of LDS, looped
    small(wl.KIND_SIGN_MEANABS, 8, 256 * 7 + 40, block=256),
    small(wl.KIND_SIGN_MEANABS, 16, 1024 * 2 + 999, block=1024),
    small(wl.KIND_SIGN_MEANABS, 3, 2, block=256),
    small(wl.KIND_SIGN_MEANABS, 33, 512 * 3 + 1, block=512),
    small(wl.KIND_SIGN_MEANABS, 9, 2048 + 7, block=2048, topo=wl.TOPO_TORUS2D, torus=(3, 3)),
    small(wl.KIND_QUANT_MAXABS, 3, 1, bits=4, block=256),                           # a single parameter per worker
    small(wl.KIND_SIGN_MEANABS, 4, 1, block=512),
    small(wl.KIND_QUANT_MAXABS, 8, 64 * 37 + 5, bits=4, block=64),                  # blocks narrower than a sweep
    small(wl.KIND_QUANT_MAXABS, 16, 128 * 19 + 77, bits=2, block=128),
    small(wl.KIND_QUANT_MAXABS, 20, 128 * 9, bits=4, block=128, topo=wl.TOPO_TORUS2D, torus=(4, 5)),
    small(wl.KIND_SIGN_MEANABS, 8, 64 * 41 + 33, block=64),
    small(wl.KIND_SIGN_MEANABS, 33, 128 * 7 + 1, block=128),
    small(wl.KIND_QUANT_MAXABS, 8, 512 * 5 + 37, bits=8, block=512),                # 8-bit codes
    small(wl.KIND_QUANT_MAXABS, 16, 64 * 31 + 9, bits=8, block=64, topo=wl.TOPO_TORUS2D, torus=(4, 4)),
    small(wl.KIND_QUANT_MAXABS, 5, 2048 * 2 + 100, bits=8, block=2048),
]
CASES = [with_algo(w, algo, tag) for algo, tag in ALGOS for w in SHAPES]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_comparison_lock_step_small_shapes(w):
    say("case", w.name)
    lock_step(w, steps=3)


@pytest.mark.parametrize("algo,tag", ALGOS)
def test_comparison_every_launch_shape(algo, tag):
    """Every candidate launch shape of the comparison kernels that fits the configuration gives the same bits."""
    seen = 0
    all_names = set()
    for base in (small(wl.KIND_QUANT_MAXABS, 8, 256 * 9 + 11, bits=2, block=256),
                 small(wl.KIND_QUANT_MAXABS, 16, 512 * 5 + 3, bits=4, block=512),
                 small(wl.KIND_SIGN_MEANABS, 30, 1024 * 2 + 77, block=1024),
                 # more tiles than workgroups fit on the device at once: the shapes that walk over tiles and
                 # request the next one ahead (DCD-PSGD) take several tiles per workgroup, and a ragged one
                 small(wl.KIND_QUANT_MAXABS, 16, 512 * 2100 + 3, bits=4, block=512),
                 small(wl.KIND_QUANT_MAXABS, 40, 256 * 2600 + 9, bits=2, block=256)):
        w = with_algo(base, algo, tag)
        names = set()
        for i in range(24):
            ds = b.DeepSqueeze.from_workload(w, plan=dict(tile_plan=i))
            name = ds.ds_plan_name()
            ds.ds_destroy()
            if name in names:          # an index past the last candidate leaves the choice automatic
                break
            names.add(name)
            say("case", w.name, "plan", i, name)
            assert name.startswith(tag + "/")
            lock_step(w, steps=2, plan=dict(tile_plan=i))
        assert names
        seen += len(names)
        all_names |= names
    assert seen >= 5
    if algo == wl.ALGO_DCD_PSGD:
        assert any("/ahead/" in nm for nm in all_names) and any("in-turn" in nm for nm in all_names)


@pytest.mark.parametrize("algo,tag", ALGOS)
def test_comparison_general_graph_and_pitches(algo, tag):
    n = 10
    r = np.random.default_rng(3)
    A = np.zeros((n, n), bool)
    for i in range(n):
        A[i, (i + 1) % n] = A[(i + 1) % n, i] = True
    for _ in range(6):
        i, j = r.integers(0, n, 2)
        if i != j:
            A[i, j] = A[j, i] = True
    deg = A.sum(1)
    W = np.zeros((n, n))
    for i in range(n):
        for j in range(n):
            if A[i, j]:
                W[i, j] = 1.0 / (1 + max(deg[i], deg[j]))
        W[i, i] = 1.0 - W[i].sum()
    rp, co, va = oracle.dense_to_csr(W)
    for base in (small(wl.KIND_QUANT_MAXABS, n, 512 * 3 + 9, bits=4, block=512), small(wl.KIND_SIGN_MEANABS, n, 777, block=256)):
        w = with_algo(base, algo, tag)
        say("case", w.name, "csr")
        lock_step(w, steps=2, W=W, csr=(rp, co, va.astype(np.float32)))
    # a gradient pitch wider than N, and a pinned state pitch
    w = with_algo(small(wl.KIND_QUANT_MAXABS, 8, 512 * 2 + 100, bits=2, block=512), algo, tag)
    lock_step(w, steps=2, pitch=512 * 3 + 64)
    lock_step(w, steps=2, plan=dict(pitch_skew=0))


@pytest.mark.parametrize("w", [with_algo(w, algo, tag) for algo, tag in ALGOS for w in (
        small(wl.KIND_QUANT_MAXABS, 8, 40_003, bits=4, block=512, grad="quadratic", gamma=0.2),
        small(wl.KIND_QUANT_MAXABS, 16, 30_001, bits=2, block=1024, grad="student_t3"),
        small(wl.KIND_SIGN_MEANABS, 9, 20_011, block=256, topo=wl.TOPO_TORUS2D, torus=(3, 3), grad="quadratic", gamma=0.2))],
        ids=lambda w: w.name)
def test_comparison_free_runs(w):
    """Thirty iterations from zero on both sides with nothing rewritten in between."""
    say("case", w.name)
    nbits = free_run(w, steps=30)
    say(w.name, "free run: state elements differing bitwise:", nbits)
    assert nbits == 0


@pytest.mark.parametrize("algo,tag", ALGOS)
def test_comparison_restart_and_determinism(algo, tag):
    """read_state at step 3, write_state into a fresh handle: the continuation is bit-identical; the step counter
    selects the rounding words as in Algorithm 1's kernel."""
    w = with_algo(small(wl.KIND_QUANT_MAXABS, 8, 512 * 7 + 5, bits=2, block=512), algo, tag)
    gs = [upload(wl.gradient(w, t)) for t in range(6)]
    a = b.DeepSqueeze.from_workload(w)
    for t in range(3):
        a.ds_step(gs[t])
    x3, h3 = a.ds_read_state()
    c = b.DeepSqueeze.from_workload(w)
    c.ds_write_state(x3, h3, 3)
    for t in range(3, 6):
        a.ds_step(gs[t])
        c.ds_step(gs[t])
        assert np.array_equal(a.ds_read_messages(), c.ds_read_messages())
    xa, ha = a.ds_read_state()
    xc, hc = c.ds_read_state()
    assert xa.tobytes() == xc.tobytes() and ha.tobytes() == hc.tobytes()
    assert a.ds_step_count() == c.ds_step_count() == 6
    a.ds_destroy()
    c.ds_destroy()


def test_comparison_refusals():
    """What the comparison kernels do not serve is refused with a reason, at validation already where possible."""
    cfg, _ = b.make_config(8, 1000, wl.TOPO_RING, wl.KIND_TOPK, 0.1, 0.4, k=10, algo=wl.ALGO_CHOCO_SGD)
    st, why = b.ds_validate_config(cfg)
    assert st == b.DS_EINVAL and "CHOCO" in why
    cfg, _ = b.make_config(8, 1000, wl.TOPO_RING, wl.KIND_QUANT_MAXABS, 0.1, 0.4, bits=4, block=512, algo=5)
    st, why = b.ds_validate_config(cfg)
    assert st == b.DS_EINVAL and "algo" in why
    # 200 rows of 512-column tiles are 400 KB of fp32: more than LDS holds
    cfg, keep = b.make_config(200, 4096, wl.TOPO_RING, wl.KIND_QUANT_MAXABS, 0.1, 0.4, bits=4, block=512, algo=wl.ALGO_DCD_PSGD)
    with pytest.raises(b.DsqError) as e:
        b.DeepSqueeze(cfg, keep)
    assert "LDS" in str(e.value)
    # the entry point without allocations serves Algorithm 1 only
    cfg, _ = b.make_config(8, 4096, wl.TOPO_RING, wl.KIND_QUANT_MAXABS, 0.1, 0.4, bits=4, block=512, algo=wl.ALGO_CHOCO_SGD)
    x = torch.zeros((8, 4096), device="cuda")
    d = torch.zeros((8, 4096), device="cuda")
    g = torch.zeros((8, 4096), device="cuda")
    msg = torch.zeros(b.ds_message_bytes(cfg), dtype=torch.uint8, device="cuda")
    with pytest.raises(b.DsqError) as e:
        b.ds_step_static(cfg, x, d, g, msg, 0)
    assert "Algorithm 1" in str(e.value)


@pytest.mark.parametrize("algo,tag", ALGOS)
@pytest.mark.parametrize("idx", [1, 3])
def test_comparison_full_size_two_free_steps(algo, tag, idx):
    """The comparison updates at the sizes of configurations 1 (ring of 16, 2-bit, 11.17 M columns) and 3 (8 x 8
    torus, 4-bit, 4.19 M columns): two iterations in a row, messages after each, the whole state at the end."""
    w = with_algo(wl.configs()[idx], algo, tag)
    _full_size_free_run(w, idx, steps=2)
