"""Free run of DeepSqueeze (and of the update rules it is compared with) on a synthetic quadratic, entirely on the GPU.

n workers on a ring minimise  f(x) = 1/n sum_i 1/2 |x - c_i|^2  (minimiser: the mean of the c_i) from noisy
gradients g_i = (x_i - c_i) + sigma xi.  The gradients are drawn on the device by ds_workload_gradient from the
library's own state buffer (borrowed through ds_state_ptrs), so nothing crosses PCIe between steps, and the
run is reproducible bit for bit (the generator has a host twin, detgen.py); ds_diagnostics gives the
consensus distance and the carried compression error.  This illustrates the behaviour the paper's Theorem 1
describes (convergence under compression thanks to the error compensation); it is not the paper's experiment,
whose data and model are not available here.

    python -m paper_1907_07346_amd.demo_quadratic [--steps 300] [--N 65536] [--workers 8] [--eta-sweep]

--eta-sweep adds, per compressor, the averaging rate eta swept from 0.05 to 1 next to the rate Theorem 1 allows,
min(1/2, (alpha^(-2/3) - 1) / 4), with alpha measured on the run itself as |v - C[v]| / |v| (Assumption 1.6's
constant; the last step's value).
"""
from __future__ import annotations

import argparse

import torch

from . import binding as b
from . import detgen
from . import workloads as wl


class _Borrowed:
    def __init__(self, ptr, shape):
        self.__cuda_array_interface__ = {"shape": shape, "typestr": "<f4", "data": (ptr, False), "version": 2,
                                         "strides": None}


def run(kind, n, N, steps, gamma, eta, sigma, report, algo=wl.ALGO_DEEPSQUEEZE, want_alpha=False, **comp):
    cfg, keep = b.make_config(n, N, wl.TOPO_RING, kind, gamma, eta, seed=1, algo=algo, **comp)
    ds = b.DeepSqueeze(cfg, keep)
    c = torch.from_numpy(detgen.centres(n, N, seed=1)).cuda()
    opt = c.mean(0)
    f_opt = float(0.5 * ((opt - c) ** 2).sum(1).mean())
    xp, dp, ld = ds.ds_state_ptrs()
    g = torch.zeros((n, ld), device="cuda")
    rows = []
    alpha = float("nan")
    for t in range(steps + 1):
        if t in report:
            ds.ds_state_ptrs()                                  # completes a deferred tail, if the path has one
            x = torch.as_tensor(_Borrowed(xp, (n, ld)), device="cuda")[:, :N]
            xbar = x.mean(0)
            gap = float(0.5 * ((xbar - c) ** 2).sum(1).mean()) - f_opt
            d = ds.ds_diagnostics()
            rows.append((t, gap / N, d["consensus_sq"] / (n * N), d["delta_sq"] / (n * N)))
        if t == steps:
            break
        ds.ds_state_ptrs()
        b.ds_workload_gradient("quadratic", n, N, sigma, 1, t, g, xp, ld)
        if want_alpha and t == steps - 1:                       # v of Algorithm 1, line 5, formed here for the ratio only
            x = torch.as_tensor(_Borrowed(xp, (n, ld)), device="cuda")[:, :N]
            d = torch.as_tensor(_Borrowed(dp, (n, ld)), device="cuda")[:, :N]
            v_norm = float((x.double() - gamma * g[:, :N].double() + d.double()).norm())
        ds.ds_step(g)
        if want_alpha and t == steps - 1:
            ds.ds_state_ptrs()
            d = torch.as_tensor(_Borrowed(dp, (n, ld)), device="cuda")[:, :N]
            alpha = float(d.double().norm()) / v_norm if v_norm > 0 else 0.0
    bytes_per_step = ds.ds_diagnostics()["message_bytes"]
    ds.ds_destroy()
    if want_alpha:
        return rows, bytes_per_step, alpha
    return rows, bytes_per_step


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--N", type=int, default=65536)
    ap.add_argument("--workers", type=int, default=8)
    ap.add_argument("--gamma", type=float, default=0.1)
    ap.add_argument("--sigma", type=float, default=0.1)
    ap.add_argument("--eta-sweep", action="store_true")
    args = ap.parse_args()
    n, N = args.workers, args.N
    report = sorted({0, args.steps // 10, args.steps // 3, args.steps})
    cases = [
        ("identity (D-PSGD)", wl.KIND_IDENTITY, 0.5, {}),
        ("4-bit blocks of 512", wl.KIND_QUANT_MAXABS, 0.5, dict(bits=4, block=512)),
        ("2-bit blocks of 64", wl.KIND_QUANT_MAXABS, 0.3, dict(bits=2, block=64)),
        ("2-bit blocks of 1024", wl.KIND_QUANT_MAXABS, 0.3, dict(bits=2, block=1024)),
        ("sign, blocks of 256", wl.KIND_SIGN_MEANABS, 0.2, dict(block=256)),
        ("top 1 %", wl.KIND_TOPK, 0.2, dict(k=max(1, N // 100))),
        ("random 10 %", wl.KIND_RAND_SPARSE, 0.2, dict(k=max(1, N // 10))),
        ("GSpar 10 %", wl.KIND_GSPAR, 0.2, dict(k=max(1, N // 10))),
        ("4 bits + norm (paper)", wl.KIND_QUANT_L2NORM, 0.5, dict(bits=4)),
        ("2 bits + norm (paper)", wl.KIND_QUANT_L2NORM, 0.3, dict(bits=2)),
    ]
    print(f"{n} workers on a ring, N = {N}, gamma = {args.gamma}, sigma = {args.sigma}; per parameter: "
          f"f(mean x) - f*, consensus distance, carried error")
    for name, kind, eta, comp in cases:
        rows, nbytes = run(kind, n, N, args.steps, args.gamma, eta, args.sigma, report, **comp)
        ratio = n * N * 4 / nbytes
        line = "  ".join(f"t={t}: {gap:.2e} {cons:.2e} {dsq:.2e}" for t, gap, cons, dsq in rows)
        print(f"{name:24s} eta={eta:.1f} msg {ratio:6.1f}x smaller | {line}", flush=True)
    # The update rules side by side under the same compressor and rates (the setting of the paper's convergence
    # figure: the same bits for every method).  Third column: the carried error for DeepSqueeze, the squared
    # norm of the public copies for CHOCO-SGD, nothing for DCD-PSGD (it has no second state array).
    rules = [("DeepSqueeze", wl.ALGO_DEEPSQUEEZE), ("CHOCO-SGD", wl.ALGO_CHOCO_SGD), ("DCD-PSGD", wl.ALGO_DCD_PSGD)]
    for cname, kind, eta, comp in (("4-bit blocks of 512", wl.KIND_QUANT_MAXABS, 0.4, dict(bits=4, block=512)),
                                   ("2-bit blocks of 512", wl.KIND_QUANT_MAXABS, 0.4, dict(bits=2, block=512)),
                                   ("sign, blocks of 256", wl.KIND_SIGN_MEANABS, 0.4, dict(block=256))):
        print(f"update rules under {cname}, eta = {eta}:")
        rows, _ = run(wl.KIND_IDENTITY, n, N, args.steps, args.gamma, eta, args.sigma, report)
        print(f"  {'D-PSGD (no compression)':24s} | " + "  ".join(f"t={t}: {gap:.2e} {cons:.2e}" for t, gap, cons, _ in rows), flush=True)
        for rname, algo in rules:
            rows, _ = run(kind, n, N, args.steps, args.gamma, eta, args.sigma, report, algo=algo, **comp)
            line = "  ".join(f"t={t}: {gap:.2e} {cons:.2e} {dsq:.2e}" for t, gap, cons, dsq in rows)
            print(f"  {rname:24s} | {line}", flush=True)
    if args.eta_sweep:
        eta_sweep(args, cases)


def eta_sweep(args, cases):
    """Consensus distance and carried error at the end of the run for a range of averaging rates, next to the
    rate Theorem 1 allows for the compressor's measured alpha."""
    n, N = args.workers, args.N
    etas = (0.05, 0.1, 0.2, 0.4, 0.6, 0.8, 1.0)
    print(f"averaging rate sweep, {args.steps} steps; per parameter at the end: consensus distance / carried error "
          f"(inf or nan: diverged)")
    for name, kind, _, comp in cases:
        cells, alpha = [], float("nan")
        for eta in etas:
            rows, _, a = run(kind, n, N, args.steps, args.gamma, eta, args.sigma, [args.steps], want_alpha=True, **comp)
            _, _, cons, dsq = rows[-1]
            cells.append(f"eta={eta:g}: {cons:.2e}/{dsq:.2e}")
            if eta == 0.2:
                alpha = a
        bound = 0.5 if not alpha > 0 else min(0.5, (alpha ** (-2.0 / 3.0) - 1.0) / 4.0)
        print(f"{name:24s} alpha={alpha:.3f} Theorem 1: eta <= {bound:.3f} | " + "  ".join(cells), flush=True)


if __name__ == "__main__":
    main()
