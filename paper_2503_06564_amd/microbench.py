"""Timings of the entry points outside bench.py's step (one MI355X, synthetic inputs):

    python -m paper_2503_06564_amd.microbench fused      # trdq_linear_fused against the unfused pair, 16..4096 tokens
    python -m paper_2503_06564_amd.microbench dense      # dense-block rotate+quantise passes against the Hadamard ones
    python -m paper_2503_06564_amd.microbench greedy     # greedy construction of the rotation blocks (Eq. 6-7)
    python -m paper_2503_06564_amd.microbench cosine     # Eq. 11 on attention-sized tensors
    python -m paper_2503_06564_amd.microbench peaks      # the chip's own ceilings: int8 matrix issue, streaming 2 B in / 1 B out
    python -m paper_2503_06564_amd.microbench all

Back-to-back launches between two events on the launch stream, cycling through a few input sets;
one line of JSON per measurement.  Inputs are N(0, 1) activations and seeded orthogonal blocks; the
figures do not depend on the values."""
import argparse
import json
import time

import numpy as np
import torch

from . import trdq, workloads as wl


def _timeit(fn, iters=50, warm=5):
    st = torch.cuda.current_stream()
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for i in range(iters):
        fn(i)
    e1.record(st)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters          # microseconds


def _timeit_graph(fn, per_graph=32, replays=8):
    """The same, with the launches replayed from a captured graph: for kernels of a few microseconds
    the interpreter cannot issue launches as fast as the device retires them."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for i in range(4):
            fn(i)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for i in range(per_graph):
            fn(i)
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (per_graph * replays)


def _out(**kw):
    print(json.dumps(kw), flush=True)


def fused(dev):
    for kind in ("proj", "qkv"):
        K, N = wl.LAYER_SHAPES[kind]
        for M in (16, 128, 256, 512, 1024, 2048, 4096):
            R = 4
            g = torch.Generator(device="cpu").manual_seed(0)
            Xs = [torch.randn((M, K), generator=g).to(torch.bfloat16).to(dev) for _ in range(R)]
            d = torch.ones(K, device=dev) * 1.25
            Xq = torch.empty((M, K), dtype=torch.int8, device=dev)
            sx = torch.empty((M,), device=dev)
            Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            W = torch.randn((K, N), generator=g).to(dev) * 0.02
            bias = torch.zeros(N, device=dev)
            ws = [trdq.prepare_weights(W, d, wbits=8) for _ in range(R)]
            fu = [trdq.bind_linear_fused(Xs[i], d, ws[i], Y, bias=bias) for i in range(R)]
            rq = [trdq.bind_rotate_quant(Xs[i], d, Xq, sx, warm=ws[i]) for i in range(R)]
            gm = [trdq.bind_qgemm(ws[i], Xq, sx, Y, bias=bias) for i in range(R)]

            def pair(i):
                rq[i % R]()
                gm[i % R]()
            _out(what="linear_fused vs rotate_quant+qgemm", layer=kind, tokens=M,
                 fused_us=round(_timeit(lambda i: fu[i % R](), 200, 10), 2), pair_us=round(_timeit(pair, 200, 10), 2))


def dense(dev):
    for M in (4096, 32768):
        for K in (1152, 4608):
            R = 4
            Xs = [torch.randn((M, K), device=dev).to(torch.bfloat16) for _ in range(R)]
            d = torch.ones(K, device=dev) * 1.25
            R1 = torch.from_numpy(wl.orthogonal_uniform_first_row(1, K // 128).astype(np.float32)).to(dev)
            rot1 = trdq.Rotation(R1, d)
            perm = torch.randperm(K, device=dev).to(torch.int32)
            Xq = torch.empty((M, K), dtype=torch.int8, device=dev)
            sx = torch.empty((M,), device=dev)
            row = dict(what="rotate+quantise passes", tokens=M, K=K,
                       hadamard_us=round(_timeit(lambda i: trdq.rotate_quant(Xs[i % R], d, Xq, sx)), 1),
                       dense_us=round(_timeit(lambda i: trdq.rotate_quant_dense(Xs[i % R], rot1, Xq, sx)), 1),
                       hadamard_rpr_us=round(_timeit(lambda i: trdq.rotate_quant_rpr(Xs[i % R], d, perm, Xq, sx)), 1))
            R2 = torch.from_numpy(wl.orthogonal_uniform_first_row(2, K // 128).astype(np.float32)).to(dev)
            rot2 = trdq.Rotation(R2)
            row["dense_rpr_us"] = round(_timeit(lambda i: trdq.rotate_quant_dense_rpr(Xs[i % R], rot1, perm, rot2, Xq, sx),
                                                20 if M * K > (1 << 26) else 50), 1)
            nbytes = trdq.rotate_quant_dense_rpr_ws_nbytes(M, K)
            if nbytes:
                ws = torch.empty((nbytes,), dtype=torch.uint8, device=dev)
                row["dense_rpr_ws_us"] = round(_timeit(
                    lambda i: trdq.rotate_quant_dense_rpr_ws(Xs[i % R], rot1, perm, rot2, Xq, sx, ws)), 1)
                row["workspace_MB"] = round(nbytes / 1e6, 1)
            _out(**row)


def greedy(dev):
    for Mc, K, steps in ((4096, 1152, 64), (4096, 4608, 64), (1024, 1152, 256)):
        X = torch.randn((Mc, K), device=dev).to(torch.bfloat16)
        d = torch.ones(K, device=dev)
        Q = torch.from_numpy(wl.orthogonal_uniform_first_row(1, steps)).to(dev)
        Rout = torch.zeros((K // 128, 128, 128), device=dev)
        trdq.greedy_rotation(X, d, Q, Rout)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n = trdq.greedy_rotation(X, d, Q, Rout)
        torch.cuda.synchronize()
        t = time.perf_counter() - t0
        _out(what="greedy_rotation (Eq. 6-7)", calibration_tokens=Mc, K=K, steps=steps, ms=round(t * 1e3, 2),
             us_per_step=round(t / steps * 1e6, 1), chosen_steps=n.tolist())


def cosine(dev):
    for n, L in ((1, 4096 * 1152), (28, 4096 * 1152), (16, 256 * 1152)):
        R = 2
        As = [torch.randn((n, L), device=dev).to(torch.bfloat16) for _ in range(R)]
        Bs = [torch.randn((n, L), device=dev).to(torch.bfloat16) for _ in range(R)]
        ws = torch.zeros(3 * n, dtype=torch.float64, device=dev)
        out = torch.zeros(n, device=dev)
        t = _timeit(lambda i: trdq.cosine_similarity(As[i % R], Bs[i % R], ws, out), 20, 3)
        _out(what="cosine_similarity (Eq. 11)", segments=n, elements=L, us=round(t, 1), tb_per_s=round(4 * n * L / t / 1e6, 2))


def measure_peaks(dev, quick=False, emit=None, stream_sizes=None):
    """What the chip delivers on the two bounding operations alone: int8 matrix instructions issued
    from registers by every SIMD (TOP/s), and a pass that reads two bytes and writes one per element
    (GB/s) at the rotate-and-quantise sizes.  `quick`: one launch shape for the matrix yardstick; `stream_sizes`: (tokens, K) pairs.
    `emit`, if given, receives one record per measurement."""
    emit = emit or (lambda **kw: None)
    res = {}
    best = 0.0
    shapes = ((1024, 4),) if quick else ((256, 4), (256, 8), (512, 4), (1024, 4))
    iters = 20000
    for wgs, waves in shapes:
        sink = torch.zeros(wgs * waves * 64, dtype=torch.int32, device=dev)
        ops = [0]

        def run(i):
            ops[0] = trdq.peak_mfma_i8(sink, wgs, waves, iters)
        t = _timeit(run, 5, 2)
        tops = ops[0] / t / 1e6
        if int(sink.min()) != 32 * 64 * iters or int(sink.max()) != 32 * 64 * iters:
            raise RuntimeError("matrix-issue yardstick: wrong accumulator sum")
        emit(what="peak int8 matrix issue (registers only)", workgroups=wgs, waves=waves, us=round(t, 1),
             tops=round(tops, 1))
        best = max(best, tops)
    res["mfma_i8_tops"] = best
    # the same loop on pseudo-random operand bytes: the clock the chip holds while its matrix pipes
    # work on data that toggles, which is what a product of quantised codes runs at
    best_data = 0.0
    for wgs, waves in shapes:
        sink = torch.zeros(wgs * waves * 64, dtype=torch.int32, device=dev)
        ops = [0]

        def run_data(i):
            ops[0] = trdq.peak_mfma_i8(sink, wgs, waves, iters, random_data=True)
        t = _timeit(run_data, 5, 2)
        tops = ops[0] / t / 1e6
        emit(what="peak int8 matrix issue (registers only, random operand bytes)", workgroups=wgs, waves=waves,
             us=round(t, 1), tops=round(tops, 1))
        best_data = max(best_data, tops)
    res["mfma_i8_data_tops"] = best_data
    res["stream_gbs"] = {}
    sizes = stream_sizes or ((4096, 1152), (4096, 4608), (32768, 1152), (32768, 4608))
    for M, K in sizes:
        R = 2 if M * K > (1 << 26) else 4
        src = [torch.randint(0, 1 << 15, (M, K), dtype=torch.int16, device=dev) for _ in range(R)]
        dst = [torch.empty((M, K), dtype=torch.int8, device=dev) for _ in range(R)]
        big = M * K > (1 << 26)
        t = min(_timeit(lambda i: trdq.peak_stream(src[i % R], dst[i % R]), 20 if big else 100, 5),
                _timeit_graph(lambda i: trdq.peak_stream(src[i % R], dst[i % R]), 8 if big else 32, 4 if big else 8))
        gbs = 3.0 * M * K / t / 1e3
        emit(what="peak stream (2 B read + 1 B written per element)", tokens=M, K=K, us=round(t, 2), gb_per_s=round(gbs, 0))
        res["stream_gbs"][f"{M}x{K}"] = gbs
        res.setdefault("stream_us", {})[f"{M}x{K}"] = t
    return res


def peaks(dev):
    measure_peaks(dev, emit=_out)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["fused", "dense", "greedy", "cosine", "peaks", "all"])
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("microbench needs the GPU")
    trdq.lib()
    dev = torch.device("cuda:0")
    for name, fn in (("fused", fused), ("dense", dense), ("greedy", greedy), ("cosine", cosine), ("peaks", peaks)):
        if a.what in (name, "all"):
            fn(dev)


if __name__ == "__main__":
    main()
