"""ds_step_static (one step on caller-owned arrays, nothing allocated, scratch in a static device array)
against ds_step on a handle: bit for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_1907_07346_amd import binding as b
from paper_1907_07346_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _case(n, N, topo, torus, kind, bits, block, seed, t):
    w = wl.Config(f"static_n{n}_N{N}_k{kind}", n=n, N=N, topo=topo, torus=torus, kind=kind, gamma=0.1, eta=0.4, steps=1,
                  grad="normal", grad_scale=0.5, bits=bits, block=block, seed=seed)
    x0, d0 = wl.random_state(w, seed=seed + 100)
    g = wl.gradient(w, t)
    return w, x0, d0, g, t


def _by_handle(w, x0, d0, g, t):
    ds = b.DeepSqueeze.from_workload(w)
    ds.ds_write_state(x0, d0, t)
    pitch = (w.N + 3) // 4 * 4
    gd = torch.zeros((w.n, pitch), dtype=torch.float32, device="cuda")
    gd[:, :w.N] = torch.from_numpy(g).cuda()
    ds.ds_step(gd)
    x, d = ds.ds_read_state()
    m = ds.ds_read_messages()
    ds.ds_destroy()
    return x, d, m


def _static(w, x0, d0, g, t):
    cfg, _ = b.config_from_workload(w)
    ld = (w.N + 4095) // 4096 * 4096 + 2560
    x = torch.zeros((w.n, ld), dtype=torch.float32, device="cuda")
    d = torch.zeros((w.n, ld), dtype=torch.float32, device="cuda")
    gd = torch.zeros((w.n, ld), dtype=torch.float32, device="cuda")
    x[:, :w.N] = torch.from_numpy(x0).cuda()
    d[:, :w.N] = torch.from_numpy(d0).cuda()
    gd[:, :w.N] = torch.from_numpy(g).cuda()
    msg = torch.full((b.ds_message_bytes(cfg),), 0xAB, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    b.ds_step_static(cfg, x, d, gd, msg, t)
    torch.cuda.synchronize()
    assert float(x[:, w.N:].abs().max()) == 0.0 and float(d[:, w.N:].abs().max()) == 0.0, "padding columns touched"
    return x[:, :w.N].cpu().numpy(), d[:, :w.N].cpu().numpy(), msg.cpu().numpy()


def test_static_step_equals_handle_step_twice_second_smaller():
    cases = [
        _case(64, 512 * 37 + 100, wl.TOPO_TORUS2D, (8, 8), wl.KIND_QUANT_MAXABS, 4, 512, seed=3, t=7),    # the larger input first
        _case(5, 1024 * 3 + 74, wl.TOPO_RING, (0, 0), wl.KIND_QUANT_MAXABS, 2, 1024, seed=4, t=2),        # then a smaller one
        _case(8, 256 * 11 + 40, wl.TOPO_RING, (0, 0), wl.KIND_SIGN_MEANABS, 0, 256, seed=5, t=0),
        _case(3, 700, wl.TOPO_RING, (0, 0), wl.KIND_IDENTITY, 0, 0, seed=6, t=1),
    ]
    for w, x0, d0, g, t in cases:
        print("case", w.name, flush=True)
        want = _by_handle(w, x0, d0, g, t)
        got = _static(w, x0, d0, g, t)
        assert np.array_equal(got[2], want[2]), f"{w.name}: messages differ"
        assert np.array_equal(got[0].view(np.uint32), want[0].view(np.uint32)), f"{w.name}: x differs"
        assert np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32)), f"{w.name}: delta differs"


def test_static_step_rejects_what_its_scratch_cannot_hold():
    x = torch.zeros((4, 4096 + 2560), dtype=torch.float32, device="cuda")
    msg = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")

    def attempt(**kw):
        args = dict(n=4, N=4000, topo=wl.TOPO_RING, kind=wl.KIND_QUANT_MAXABS, gamma=0.1, eta=0.4, bits=4, block=512)
        args.update(kw)
        cfg, keep = b.make_config(args.pop("n"), args.pop("N"), args.pop("topo"), args.pop("kind"), args.pop("gamma"),
                                  args.pop("eta"), **args)
        with pytest.raises(b.DsqError) as e:
            b.ds_step_static(cfg, x, x, x, msg, 0)
        assert e.value.status == b.DS_EINVAL
        return str(e.value)

    assert "1024" in attempt(n=1025, N=16)
    assert "serves" in attempt(kind=wl.KIND_TOPK, k=40)
    assert "serves" in attempt(kind=wl.KIND_RAND_SPARSE, k=40)
    rp, co, va = np.array([0, 1, 2, 3, 4], np.int32), np.arange(4, dtype=np.int32), np.ones(4, np.float32)
    assert "RING" in attempt(topo=wl.TOPO_CSR, W_csr=(rp, co, va))
    assert "ld" in attempt(N=7000)                                     # the arrays' pitch is too small for N
