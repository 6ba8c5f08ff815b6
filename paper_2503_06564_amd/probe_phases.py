"""Phase and clock probe of the tiled int8 product (two workgroups per compute unit).

A build of the library with -DTRDQ_PROBE_PHASES makes every workgroup of qgemm8_tiled_kernel record
the constant-rate timer and the shader cycle counter at entry, after its first operands have landed,
after its k-loop and at its end, plus the die and compute unit it ran on; the records land in the
buffer that otherwise receives the integer sums.  This script prints, per shape: the span from the
first entry to the last exit, the mean length of the three phases, the shader clock during the
k-loop (cycle counter / timer) per die, and the k-loop's length in cycles against the number of
cycles its matrix instructions need (16 per instruction; the two workgroups of a compute unit
share the four matrix pipes).

    python -m paper_2503_06564_amd.probe_phases --build     # on the build machine (hipcc only)
    python -m paper_2503_06564_amd.probe_phases             # on the GPU
"""
import argparse
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
PROBE_LIB = os.path.join(HERE, "libtrdq_probe.so")
SHAPES = [(4096, 1152, 3456), (4096, 1152, 4608), (4096, 4608, 4608), (16384, 1152, 4608)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true", help="compile the probe library and exit")
    args = ap.parse_args()
    if args.build:
        from . import build
        print(build.build(extra=["-DTRDQ_PROBE_PHASES"], lib=PROBE_LIB, obj_dir=build.OBJ_DIR + "_probe"))
        return 0
    if not os.path.exists(PROBE_LIB):
        sys.exit(f"{PROBE_LIB} is missing: run this module with --build first")
    import numpy as np
    import torch
    from . import trdq
    trdq.LIB_PATH = PROBE_LIB
    dev = torch.device("cuda:0")
    for (M, K, N) in SHAPES:
        g = torch.Generator(device="cpu").manual_seed(0)
        W = (torch.randn((K, N), generator=g) * 0.02).to(dev)
        d = torch.ones(K, device=dev)
        w = trdq.prepare_weights(W, d, wbits=8)
        X = torch.randn((M, K), generator=g).to(torch.bfloat16).to(dev)
        Xt = torch.empty((trdq.xq_tiled_nbytes(M, K),), dtype=torch.int8, device=dev)
        sx = torch.empty((M,), dtype=torch.float32, device=dev)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        trdq.rotate_quant_tiled(X, d, Xt, sx)
        rec = torch.zeros((M, N), dtype=torch.int32, device=dev)
        for _ in range(6):              # the last launch is the one read back
            rec.zero_()
            trdq.qgemm_tiled(w, Xt, sx, Y, acc_debug=rec)
            torch.cuda.synchronize()
        o = rec.cpu().numpy().reshape(-1).view(np.uint64).reshape(-1, 16)
        o = o[o[:, 11] == 1]
        t = o[:, 0:4].astype(np.float64) * 10.0         # ns (100 MHz timer)
        c = o[:, 4:8].astype(np.float64)
        xcc = (o[:, 9] & 0xF).astype(int)
        t0 = t[:, 0].min()
        us = lambda a: a / 1e3
        kl_t, kl_c = t[:, 2] - t[:, 1], c[:, 2] - c[:, 1]
        tall = o[:, 10] == 256
        # matrix instructions of one workgroup: K / 64 steps x 9 x (rows / 64) per wave, 16 cycles each; a
        # compute unit's pipes carry both of its workgroups
        steps = K // 64
        need = steps * 9 * 16 * (np.where(tall, 4, 2)).astype(np.float64)
        print(f"M={M} K={K} N={N}: {len(o)} workgroups ({int(tall.sum())} of 256 tokens), first entry -> last exit {us(t[:, 3].max() - t0):.2f} us, "
              f"entries within {us(t[:, 0].max() - t0):.2f} us")
        print(f"   mean phases: operands in {us(t[:, 1] - t[:, 0]).mean():.2f} us, k-loop {us(kl_t).mean():.2f} us "
              f"(min {us(kl_t).min():.2f}, max {us(kl_t).max():.2f}), epilogue {us(t[:, 3] - t[:, 2]).mean():.2f} us")
        print(f"   k-loop: {kl_c.mean():.0f} cycles per workgroup; its own matrix instructions need {need.mean():.0f}, "
              f"those of the two workgroups of a compute unit {2 * need.mean():.0f}")
        for x in sorted(set(xcc)):
            m = xcc == x
            print(f"   die {x}: {int(m.sum()):4d} workgroups, k-loop {us(kl_t[m]).mean():6.2f} us, shader clock {kl_c[m].sum() / kl_t[m].sum():.3f} GHz")
        sys.stdout.flush()
        w.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
