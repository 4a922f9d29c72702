"""Time line of the tuned product kernel's work items, from a profiling build of the library.

The kernel template in ``csrc/gemm_mfma_kernel.h`` takes time stamps (shader clock and the 100 MHz
clock) at the boundaries of a workgroup's items when compiled with ``-DCUBE3D_PROFILE``: kernel start,
two K-tiles in, third K-tile done, K loop done, next item's first loads issued, epilogue issued, first
fragments read, and so on per item.  Build that variant beside the product and run one product of a
benchmark configuration through it:

    CUBE3D_OUT=libcube3d_profile.so CUBE3D_EXTRA_FLAGS=-DCUBE3D_PROFILE python3 -m paper_2105_14450_amd.build
    python3 -m paper_2105_14450_amd.item_timeline --config config4 --product fwd --dist normal

The stamps go to a device buffer whose address the profiling build reads from the environment
(``CUBE3D_PROF_PTR``); the product's own library never does.  Operands are drawn on the device
(this is a timing tool, not a parity check).
"""
import argparse
import os
import sys

CONFIGS = {"config2": (4, 8192, 2048, 8192, False), "config4": (4, 32768, 8192, 32768, False),
           "config5": (8, 16384, 12288, 49152, True), "config3_mlp_up": (4, 8192, 2048, 8192, False),
           "config3_mlp_down": (4, 8192, 8192, 2048, False)}
LABELS_FIRST = ["kernel start", "two K-tiles in (first loads landed)", "third K-tile done"]
LABELS_ITEM = ["K loop done (taken about one K-tile early)", "next item's first loads issued", "epilogue issued",
               "first fragments of the next item read", "two K-tiles in", "third K-tile done (waited for the stores)"]
# the map-addressed kernels (--cube) take no stamps inside the K loop
LABELS_ITEM_CUBE = ["K loop done (taken about one K-tile early)", "next item's first loads issued", "epilogue issued",
                    "first fragments of the next item read"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="config4", choices=sorted(CONFIGS))
    ap.add_argument("--product", default="fwd", choices=["fwd", "dx", "dw"])
    ap.add_argument("--dist", default="normal", choices=["normal", "zeros"])
    ap.add_argument("--cube", action="store_true",
                    help="the product over the whole q^3 cube, shards read and written in place (map-addressed kernels; "
                         "forward with bias) instead of one rank's share")
    ap.add_argument("--lib", default="libcube3d_profile.so", help="file name of the profiling build inside the package")
    args = ap.parse_args()

    import numpy as np
    import torch

    from . import binding as c3
    c3.LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), args.lib)
    c3.load()
    q, M, K, N, fp8 = CONFIGS[args.config]
    Mb, Kb, Nb = M // q, K // q, N // q
    zeros = args.dist == "zeros"
    if fp8:
        mk = (lambda *s: torch.zeros(*s, device="cuda", dtype=torch.uint8)) if zeros else \
            (lambda *s: torch.randint(0, 256, s, device="cuda", dtype=torch.uint8) & 0x77)
        X, W, G = mk(Mb, Kb), mk(Kb, Nb), mk(Mb, Nb)
        d = c3.make_desc(q, M, K, N, in_dtype=c3.FP8_E4M3, out_dtype=c3.BF16, scale_x=0.01, scale_w=0.001, scale_dy=0.01)
    else:
        mk = (lambda *s: torch.zeros(*s, device="cuda", dtype=torch.bfloat16)) if zeros else \
            (lambda *s: torch.randn(*s, device="cuda").to(torch.bfloat16))
        X, W, G = mk(Mb, Kb), (mk(Kb, Nb) * 0.02).to(torch.bfloat16), mk(Mb, Nb)
        d = c3.make_desc(q, M, K, N, in_dtype=c3.BF16, out_dtype=c3.BF16)
    P, Q, R = (torch.empty(s, device="cuda", dtype=torch.bfloat16) for s in ((Mb, Nb), (Mb, Kb), (Kb, Nb)))
    r = (1, 2, 3)
    fn = {"fwd": lambda: c3.cube3d_linear_fwd(d, r, X, W, P), "dx": lambda: c3.cube3d_linear_bwd_dx(d, r, G, W, Q),
          "dw": lambda: c3.cube3d_linear_bwd_dw(d, r, X, G, R)}[args.product]
    if args.cube:
        if fp8:
            ap.error("--cube: bf16 configurations only")
        n, Ms, Ns = q ** 3, M // q ** 2, N // q ** 2
        d = c3.make_desc(q, M, K, N, in_dtype=c3.BF16, out_dtype=c3.F32, shard_dtype=c3.BF16,
                         in_axis=c3.AXIS_Z if args.config == "config3_mlp_down" else c3.AXIS_Y)
        xs, ws, gs = mk(n, Ms, Kb), (mk(n, Kb, Ns) * 0.02).to(torch.bfloat16), mk(n, Ms, Nb)
        bias = torch.zeros(n, Ns, device="cuda") if zeros else torch.randn(n, Ns, device="cuda")
        ys, dxs, dws = (torch.empty(sh, device="cuda", dtype=torch.bfloat16) for sh in ((n, Ms, Nb), (n, Ms, Kb), (n, Kb, Ns)))
        fn = {"fwd": lambda: c3.virtual_cube_linear_fwd(d, xs, ws, bias, ys),
              "dx": lambda: c3.virtual_cube_linear_bwd_dx(d, gs, ws, dxs),
              "dw": lambda: c3.virtual_cube_linear_bwd_dw(d, xs, gs, dws)}[args.product]
    prof = torch.zeros(1024 * 64, dtype=torch.int64, device="cuda")
    for _ in range(30):
        fn()
    torch.cuda.synchronize()
    os.environ["CUBE3D_PROF_PTR"] = str(prof.data_ptr())
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    del os.environ["CUBE3D_PROF_PTR"]
    a = prof.cpu().numpy().reshape(1024, 32, 2)
    a = a[a[:, 0, 0] > 0]
    if a.shape[0] == 0:
        print("no stamps: is %s a -DCUBE3D_PROFILE build?" % args.lib, file=sys.stderr)
        return 1
    clk, rt = a[:, :, 0].astype(np.float64), a[:, :, 1].astype(np.float64)
    counts = (clk > 0).sum(axis=1)
    n = int(counts.min())          # workgroups with more items have more stamps: the common prefix is shown
    t0 = rt[:, 0].min()
    print("%s %s%s, operands %s: %d workgroups, %d to %d stamps each (the first %d shown)" % (
        args.config, args.product, " over the whole cube in place" if args.cube else "", args.dist, a.shape[0], n,
        int(counts.max()), n))
    print("| stamp | what | shader cycles since the previous stamp (median) | us since the first stamp of the launch: median (min .. max over workgroups) |")
    print("|---|---|---|---|")
    for i in range(n):
        if args.cube:
            label = LABELS_FIRST[0] if i == 0 else LABELS_ITEM_CUBE[(i - 1) % 4]
        else:
            label = LABELS_FIRST[i] if i < 3 else LABELS_ITEM[(i - 3) % 6]
        dc = np.median(clk[:, i] - clk[:, i - 1]) if i else 0
        us = (rt[:, i] - t0) / 100.0
        print("| %d | %s | %.0f | %.2f (%.2f .. %.2f) |" % (i, label, dc, np.median(us), us.min(), us.max()))
    tot = clk[:, n - 1] - clk[:, 0]
    dur = np.median(rt[:, n - 1] - rt[:, 0])
    print("first to last stamp of a workgroup: median %.0f cycles in %.2f us = %.3f GHz" % (np.median(tot), dur / 100.0,
                                                                                         np.median(tot) / (dur * 10.0)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
