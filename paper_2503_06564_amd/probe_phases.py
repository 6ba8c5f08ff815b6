"""Phase and clock probe of the tiled products.

A build of the library with -DTRDQ_PROBE_PHASES makes every workgroup of the tiled product kernels
(qgemm8_tiled_kernel, qgemm8_tiled_ksplit_kernel, qgemm4_tiled_kernel) record the constant-rate timer
and the shader cycle counter at entry, after its first operands have landed, after its k-loop and at
its end, plus the die and compute unit it ran on; the records land in the buffer that otherwise
receives the integer sums.  This script prints, per shape: the span from the first entry to the last
exit, the mean length of the three phases, the shader clock during the k-loop (cycle counter /
timer) per die, and the k-loop's length in cycles against the number of cycles its matrix
instructions need (16 per instruction on the SIMD's one matrix pipe; with two workgroups per compute
unit a pipe carries a wave of each).

    python -m paper_2503_06564_amd.probe_phases --build     # on the build machine (hipcc only)
    python -m paper_2503_06564_amd.probe_phases             # on the GPU
"""
import argparse
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
PROBE_LIB = os.path.join(HERE, "libtrdq_probe.so")
# (weight bits, tokens, K, N): the four layers of a DiT-XL/2 block at 4096 tokens, one long-K and one many-round
# int8 case, and the int4 kernel
CASES = [(8, 4096, 1152, 3456), (8, 4096, 1152, 1152), (8, 4096, 1152, 4608), (8, 4096, 4608, 1152),
         (8, 4096, 4608, 4608), (8, 16384, 1152, 4608), (4, 4096, 1152, 4608), (4, 16384, 1152, 4608)]
KERNEL = {1: "qgemm8_tiled_kernel", 2: "qgemm8_tiled_ksplit_kernel", 4: "qgemm4_tiled_kernel"}


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
    for (wbits, M, K, N) in CASES:
        g = torch.Generator(device="cpu").manual_seed(0)
        W = (torch.randn((K, N), generator=g) * 0.02).to(dev)
        d = torch.ones(K, device=dev)
        w = trdq.prepare_weights(W, d, wbits=wbits)
        X = torch.randn((M, K), generator=g).to(torch.bfloat16).to(dev)
        Xt = torch.empty((trdq.xq_tiled_nbytes(M, K),), dtype=torch.int8, device=dev)
        sx = torch.empty((M,), dtype=torch.float32, device=dev)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        trdq.rotate_quant_tiled(X, d, Xt, sx)
        rec = torch.zeros((K // 128 if wbits == 4 else 1, M, N), dtype=torch.int32, device=dev)
        for _ in range(6):              # the last launch is the one read back
            rec.zero_()
            trdq.qgemm_tiled(w, Xt, sx, Y, acc_debug=rec)
            torch.cuda.synchronize()
        o = rec.cpu().numpy().reshape(-1).view(np.uint64)[: (M // 128) * (N // 128) * 16 * 2].reshape(-1, 16)
        o = o[np.isin(o[:, 11], (1, 2, 4)) & (o[:, 0] != 0)]
        kind = int(o[0, 11])
        t = o[:, 0:4].astype(np.float64) * 10.0         # ns (100 MHz timer)
        c = o[:, 4:8].astype(np.float64)
        xcc = (o[:, 9] & 0xF).astype(int)
        t0 = t[:, 0].min()
        us = lambda a: a / 1e3
        kl_t, kl_c = t[:, 2] - t[:, 1], c[:, 2] - c[:, 1]
        steps = K // 64
        if kind == 1:       # a wave: 9 x (rows / 64) matrix instructions per k-step; two workgroups share a pipe
            own = steps * 9 * 16 * np.where(o[:, 10] == 256, 4, 2).astype(np.float64)
            need = f"its own matrix instructions need {own.mean():.0f}, those of the two workgroups of a compute unit {2 * own.mean():.0f}"
        elif kind == 2:     # a wave: half of the k-steps, 36 matrix instructions each, alone on its pipe
            need = f"its matrix instructions need {steps // 2 * 36 * 16}"
        else:               # a wave: 16 matrix instructions per k-step; per scale group 176 vector instructions of 4 cycles
            need = (f"its own matrix instructions need {steps * 16 * 16}, those of two workgroups {2 * steps * 16 * 16}, "
                    f"the vector instructions of two workgroups {2 * (steps // 2) * 176 * 4}")
        print(f"W{wbits} M={M} K={K} N={N} ({KERNEL[kind]}): {len(o)} workgroups, first entry -> last exit "
              f"{us(t[:, 3].max() - t0):.2f} us, entries within {us(t[:, 0].max() - t0):.2f} us")
        print(f"   mean phases: operands in {us(t[:, 1] - t[:, 0]).mean():.2f} us, k-loop {us(kl_t).mean():.2f} us "
              f"(min {us(kl_t).min():.2f}, max {us(kl_t).max():.2f}), after the loop {us(t[:, 3] - t[:, 2]).mean():.2f} us")
        print(f"   k-loop: {kl_c.mean():.0f} cycles per workgroup; {need}")
        clocks = [kl_c[xcc == x].sum() / kl_t[xcc == x].sum() for x in sorted(set(xcc))]
        print("   shader clock in the k-loop per die (GHz): " + " ".join(f"{v:.3f}" for v in clocks))
        sys.stdout.flush()
        w.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
