#!/usr/bin/env python3
"""Benchmark of the MDBF forward product on one MI355X.

Workload (N=1): the LLaMA-7B attention projection as a decode GEMV -- m=n=4096, k=2656, l=16,
one fp16 token, about 1.5 bits/weight.  One "step" is one pass of the whole hot path (pack is
offline; scale-in, binary product 1, envelope accumulate + re-scale, binary product 2, envelope
accumulate) over one batch of `copies` INDEPENDENT layers of that shape, each with its own
signs, envelopes and activation vector, resident in HBM.  The batch exceeds 1 GB, several times
the 256 MB last-level cache, so every step streams its weights from HBM.  The batch is issued
through mdbf_forward_batch (per factor one scale-in launch and one product launch).  Also
reported, never as `value`: the product kernel timed by itself (the roofline object), the same
layers issued as one mdbf_forward call each from a HIP graph, one layer re-run hot in cache, the
latency of a single call, a 16-token call on an MLP projection, the 2048-token prefill call, and a plan
of 96 MLP projections with 1 and with 16 tokens.

Prints ONE JSON line (fields: see the README).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBS = 8000.0

# the arithmetic of the one-token product kernels (inputs, envelopes and outputs are fp16 either way)
DTYPE_OF_KERNEL = {
    "stage_mx_kernel": "fp4 signs x fp6 limbs (3 per activation, power-of-two scale per 32: block-floating, "
                       "~13 bits of the block maximum), f32 accumulate; f16 in/out",
    "stage_fast_kernel": "f16 x f16, f32 accumulate",
}

M, N, K, L = 4096, 4096, 2656, 16


def algorithmic_bytes(m, n, k, l, T=1, ebytes=2, xbytes=2, ybytes=2):
    """Bytes one forward call must move: packed signs + envelope factors + x + y."""
    signs = (m + n) * k // 8
    env = ebytes * l * (m + n + 2 * k)
    return signs + env + T * (xbytes * n + ybytes * m)


def make_device_layers(torch, mb, copies, seed):
    """`copies` independent layers generated on the device from one seed: i.i.d. sign bits,
    envelopes |N(0,1)|*0.02 + 1e-3 (fp16), activations N(0,1) (fp16)."""
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    layers, Xs, Ys = [], [], []
    nb_sa = mb.mdbf_packed_bytes(M, K)
    nb_sb = mb.mdbf_packed_bytes(K, N)

    def env(rows):
        return (torch.randn((rows, L), generator=g, device="cuda:0").abs() * 0.02 + 1e-3).half()

    for _ in range(copies):
        sa = torch.randint(-2 ** 31, 2 ** 31 - 1, (nb_sa // 4,), dtype=torch.int32, generator=g, device="cuda:0")
        sb = torch.randint(-2 ** 31, 2 ** 31 - 1, (nb_sb // 4,), dtype=torch.int32, generator=g, device="cuda:0")
        layers.append(mb.DeviceLayer(M, N, K, L, sa.view(torch.uint8), sb.view(torch.uint8),
                                     env(M), env(K), env(K), env(N)))
        Xs.append(torch.randn((1, N), generator=g, device="cuda:0").half())
        Ys.append(torch.zeros((1, M), dtype=torch.float16, device="cuda:0"))
    return layers, Xs, Ys


def preheat(torch, fn, min_ms=150.0):
    """Run fn() back to back for at least min_ms of GPU time: the shader clock needs some 50 ms of sustained
    load to settle, whatever the counted warm-up says.  Returns the milliseconds spent."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total, batch = 0.0, 8
    while total < min_ms:
        e0.record()
        for _ in range(batch):
            fn()
        e1.record()
        torch.cuda.synchronize()
        dt = e0.elapsed_time(e1)
        total += dt
        # aim at batches of about 30 ms so that the check costs little idle time
        batch = max(batch, min(4096, int(batch * 30.0 / max(dt, 1e-3))))
    return total


def oracle_check(torch, mb, layer, X, Y):
    """Download one layer (logical signs through mdbf_unpack) and compare with the CPU oracle."""
    from oracle import mdbf_oracle as orc
    M, N, K = layer.m, layer.n, layer.k
    SA = mb.mdbf_unpack(layer.SA_packed, M, K).cpu().numpy()
    SB = mb.mdbf_unpack(layer.SB_packed, K, N).cpu().numpy()
    args = (SA, SB, layer.A.float().cpu().numpy(), layer.Q.float().cpu().numpy(),
            layer.G.float().cpu().numpy(), layer.B.float().cpu().numpy())
    ref = orc.forward_factored(*args, X.float().cpu().numpy())
    return orc.max_rel_error(Y.float().cpu().numpy(), ref), args


def cpu_baseline(args, X, budget_s=8.0):
    """The oracle's factored forward, as it stands (numpy fp64; its matrix products run in the BLAS numpy is
    linked with), on the host: once with all the threads that BLAS takes and once limited to one."""
    from oracle import mdbf_oracle as orc
    from threadpoolctl import threadpool_info, threadpool_limits
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    Xh = X.float().cpu().numpy()

    def timed(budget, max_calls):
        orc.forward_factored(*args, Xh)
        t0 = time.perf_counter()
        calls = 0
        while True:
            orc.forward_factored(*args, Xh)
            calls += 1
            if time.perf_counter() - t0 > budget or calls >= max_calls:
                break
        return (time.perf_counter() - t0) / calls, calls

    dt, calls = timed(budget_s, 200)
    with threadpool_limits(limits=1):
        dt1, calls1 = timed(budget_s, 60)
    nbytes = algorithmic_bytes(M, N, K, L)
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": int(cores),
            "kind": "oracle", "ms_per_call": dt * 1e3,
            "one_core": {"value": nbytes / dt1 / 1e9, "unit": "GB/s", "cores": 1, "ms_per_call": dt1 * 1e3,
                         "calls": calls1},
            "implementation": "numpy fp64, factored order (H1-H5), sign matrices as int8 converted per call; "
                              "threads are the BLAS pool's, not OpenMP loops over rows",
            "sample": "%d forward calls of the numpy fp64 oracle (factored order) on one 4096x4096 k=2656 l=16 layer"
                      % calls}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the shader clock takes some 50 ms of sustained load to settle; every timed loop below is preceded by a
    # time-based preheat, so that a few dozen steps (0.3 ms each) measure the same state as a few thousand
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--preheat-ms", type=float, default=150.0,
                    help="GPU time of untimed load before the counted warm-up (clock settling)")
    ap.add_argument("--copies", type=int, default=336, help="independent layers per step (336 x 3.17 MB > 1 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the graph / hot / latency side measurements")
    ap.add_argument("--fp16-staged", action="store_true",
                    help="headline plan on the fp16-staged kernel (MDBF_FLAG_FP16_STAGED) instead of the block-scaled one")
    ap.add_argument("--quick", action="store_true",
                    help="side measurements with a twentieth of their repetitions (for runs under hardware counters, "
                         "where every dispatch is serialised)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy, the known-size reference for the HBM traffic counters")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (--gpus 1); the forward product of one layer "
              "is a single-GPU kernel and no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_24545_amd import binding as mb
    mb.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if a.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        dst = torch.empty_like(src)
        torch.bitwise_xor(src, 85, out=dst)   # an elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    layers, Xs, Ys = make_device_layers(torch, mb, a.copies, seed=2)
    plan = mb.BatchPlan(layers, Xs, Ys, fp16_staged=a.fp16_staged)
    bytes_call = algorithmic_bytes(M, N, K, L)
    bytes_step = bytes_call * a.copies

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- the timed region: K steps of the batched path, after a time-based preheat and the W counted steps
    preheat_ms = preheat(torch, plan.run, a.preheat_ms)
    for _ in range(a.warmup):
        plan.run()
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    for _ in range(a.steps):
        plan.run()
    e1.record()
    torch.cuda.synchronize()
    ms_total = e0.elapsed_time(e1)
    ms_step = ms_total / a.steps
    gbs = bytes_step / ms_step / 1e6

    err, host_args = oracle_check(torch, mb, layers[0], Xs[0], Ys[0])
    err_last, _ = oracle_check(torch, mb, layers[-1], Xs[-1], Ys[-1])

    # ---- roofline of the dominant kernel: the product kernel (one launch per factor, two per step), timed
    #      by itself over the same number of steps; the scale-in results of the last full step stay valid
    part_steps = a.steps if a.quick else max(a.steps, 200)
    e0, e1 = ev(), ev()
    preheat(torch, lambda: plan.run_part(3, 2), a.preheat_ms)
    e0.record()
    for _ in range(part_steps):
        plan.run_part(3, 2)
    e1.record()
    torch.cuda.synchronize()
    avg_launch_ms = e0.elapsed_time(e1) / (2 * part_steps)
    preheat(torch, lambda: plan.run_part(3, 1), a.preheat_ms)
    e0.record()
    for _ in range(part_steps):
        plan.run_part(3, 1)
    e1.record()
    torch.cuda.synchronize()
    # scale-in launches per step: two, or one when the first factor's product launch writes the second factor's
    # activation records itself (three launches per step)
    n_si = max(plan.launches() - 2, 1)
    avg_scale_in_ms = e0.elapsed_time(e1) / (n_si * part_steps)
    traffic = None   # HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE runs
    tpath = os.path.join(ROOT, "profiles", "traffic_attn_decode.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            rec = json.load(f)
        if rec["kernel"].startswith(plan.kernel(1)):     # the record is of the block-scaled kernel
            traffic = rec["hbm_bytes_per_layer_per_launch"] * a.copies
    # the share of a layer's algorithmic bytes that the product kernel itself moves, averaged over its two
    # launches per step: the packed signs of the factor, the envelope factor on its output side (G resp. A)
    # and y; the other envelope factor (B resp. Q) and x are read by the scale-in kernel
    q_in_product = 2 * L * K if n_si == 1 else 0     # the envelope factor Q: read by whoever builds the z records
    product_bytes_layer = ((M + N) * K // 8 + 2 * L * (K + M) + 2 * M + q_in_product) / 2
    scale_in_bytes_layer = (2 * L * (N + K) + 2 * N - q_in_product) / n_si
    assert 2 * product_bytes_layer + n_si * scale_in_bytes_layer == algorithmic_bytes(M, N, K, L)
    bytes_launch = product_bytes_layer * a.copies
    roof = {"bound": "hbm", "kernel": plan.kernel(1), "launches_timed": 2 * part_steps,
            "launches_per_step": plan.launches(), "achieved": bytes_launch / avg_launch_ms / 1e6,
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": traffic,
            "avg_launch_us": avg_launch_ms * 1e3, "algorithmic_bytes_per_launch": bytes_launch,
            "scale_in_avg_launch_us": avg_scale_in_ms * 1e3,
            "scale_in_algorithmic_bytes_per_launch": scale_in_bytes_layer * a.copies}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # the read bandwidth a plain kernel reaches on this device (non-temporal 16-byte loads over 1 GiB, 2
    # workgroups of 256 lanes per compute unit, four loads in flight per lane: the best of a sweep): the
    # practical ceiling next to the nominal peak
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    sink = torch.zeros(2048, dtype=torch.int32, device="cuda:0")
    for _ in range(5):
        mb.mdbf_stream_read(buf, sink)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(50):
        mb.mdbf_stream_read(buf, sink)
    e1.record()
    torch.cuda.synchronize()
    roof["stream_read_GBps"] = 50 * buf.numel() / e0.elapsed_time(e1) / 1e6
    roof["frac_of_stream_read"] = roof["achieved"] / roof["stream_read_GBps"]
    del buf, sink

    extras = {}
    if not a.no_extras:
        # (1) one mdbf_forward call per layer, replayed from a HIP graph
        ws = [torch.empty(mb.mdbf_workspace_bytes(l.desc("f16", "f16"), 1), dtype=torch.uint8, device="cuda:0")
              for l in layers]
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            for i in range(min(4, a.copies)):
                mb.mdbf_forward(layers[i], Xs[i], y_dtype="f16", Y=Ys[i], workspace=ws[i])
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            for i in range(a.copies):
                mb.mdbf_forward(layers[i], Xs[i], y_dtype="f16", Y=Ys[i], workspace=ws[i])
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        reps = 5
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        us_call = e0.elapsed_time(e1) * 1e3 / (reps * a.copies)
        extras["per_call_graph"] = {"us_per_call": us_call, "GB/s": bytes_call / us_call / 1e3}
        # (1b) the same calls captured on four streams: the layers are independent, so the graph may have
        #      parallel branches and the device runs several calls' launches side by side
        side = [torch.cuda.Stream() for _ in range(3)]
        g4 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g4, stream=s):
            for st in side:
                st.wait_stream(s)
            branches = [s] + side
            for i in range(a.copies):
                mb.mdbf_forward(layers[i], Xs[i], y_dtype="f16", Y=Ys[i], workspace=ws[i], stream=branches[i % 4])
            for st in side:
                s.wait_stream(st)
        g4.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            g4.replay()
        e1.record()
        torch.cuda.synchronize()
        us4 = e0.elapsed_time(e1) * 1e3 / (reps * a.copies)
        err4, _ = oracle_check(torch, mb, layers[2], Xs[2], Ys[2])
        extras["per_call_graph_4_branches"] = {"us_per_call": us4, "GB/s": bytes_call / us4 / 1e3,
                                               "max_rel_err_vs_oracle": err4}
        del g4
        # (2) the same layer again and again (cache resident) through the batched entry point
        hot = mb.BatchPlan([layers[0]] * 64, [Xs[0]] * 64, [Ys[0]] * 64)
        preheat(torch, hot.run, a.preheat_ms)
        e0.record()
        for _ in range(100):
            hot.run()
        e1.record()
        torch.cuda.synchronize()
        extras["hot_in_cache"] = {"GB/s": 64 * bytes_call * 100 / e0.elapsed_time(e1) / 1e6}
        # (3) latency of one isolated call (two launches: each factor's contraction split across workgroups),
        #     stream-ordered
        e0.record()
        for _ in range(200):
            mb.mdbf_forward(layers[1], Xs[1], y_dtype="f16", Y=Ys[1], workspace=ws[1])
        e1.record()
        torch.cuda.synchronize()
        extras["single_call_stream"] = {"us_per_call": e0.elapsed_time(e1) * 1e3 / 200}
        del ws, g, hot
        # (4) 16 tokens through one MLP projection (11008 x 4096, k = 4096) and (5) the 2048-token prefill
        #     call on the attention shape: reconstruct-order kernel, bound by the fp16 matrix cores
        from paper_2512_24545_amd import synth

        def time_call(m, n, k, T, reps):
            Lh = synth.make_layer(m, n, k, L, seed=11)
            dl = mb.DeviceLayer.from_host(Lh)
            X = torch.randn((T, n), device="cuda:0").half()
            Y = torch.empty((T, m), dtype=torch.float32, device="cuda:0")
            wsb = torch.empty(mb.mdbf_workspace_bytes(dl.desc("f16", "f32"), T), dtype=torch.uint8, device="cuda:0")
            preheat(torch, lambda: mb.mdbf_forward(dl, X, y_dtype="f32", Y=Y, workspace=wsb), a.preheat_ms)
            e0.record()
            for _ in range(reps):
                mb.mdbf_forward(dl, X, y_dtype="f32", Y=Y, workspace=wsb)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            issued = 2.0 * (m + n) * k * (T + L)      # reconstruct order: (l + T) multiply-adds per sign entry
            return {"ms_per_call": ms, "tokens_per_s": T / ms * 1e3,
                    "dense_equivalent_TFLOPs": 2.0 * m * n * T / ms / 1e9,
                    "issued_TFLOPs": issued / ms / 1e9,
                    "roofline": {"bound": "mfma", "kernel": "stage_gemm_kernel", "achieved": issued / ms / 1e9,
                                 "peak": 2500.0, "unit": "TFLOP/s", "frac": issued / ms / 1e9 / 2500.0,
                                 "flops_per_call": issued}}

        q = 20 if a.quick else 1
        extras["decode_T16_mlp_gate"] = time_call(11008, 4096, 4096, 16, 300 // q)
        extras["prefill_T2048_attn"] = time_call(M, N, K, 2048, 300 // q)
        # matrix-core busy share of the prefill kernels, from the committed counter run (profiles/)
        cpath = os.path.join(ROOT, "profiles", "counters_prefill.json")
        if os.path.exists(cpath):
            with open(cpath) as f:
                extras["prefill_T2048_attn"]["roofline"]["mfma_busy_frac_counter"] = json.load(f)["mfma_busy_frac"]

        # (6) the MLP projections as they are meant to be issued: 96 independent layers (32 x gate, up, down;
        #     11008 x 4096 and 4096 x 11008, k = 4096, 0.82 GB) in one plan, with 1 and with 16 tokens each
        from paper_2512_24545_amd import workloads

        def time_mlp_plan(T, reps):
            gen = torch.Generator(device="cuda:0")
            gen.manual_seed(33)
            pl, px, py, nbytes = [], [], [], 0
            for _ in range(32):
                for (m, n) in ((11008, 4096), (11008, 4096), (4096, 11008)):
                    pl.append(workloads._device_layer(torch, gen, m, n, 4096, L))
                    px.append(torch.randn((T, n), generator=gen, device="cuda:0").half())
                    py.append(torch.zeros((T, m), dtype=torch.float16, device="cuda:0"))
                    nbytes += algorithmic_bytes(m, n, 4096, L, T)
            plan_mlp = mb.BatchPlan(pl, px, py)
            preheat(torch, plan_mlp.run, a.preheat_ms)
            e0.record()
            for _ in range(reps):
                plan_mlp.run()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            # one gate-shaped and one down-shaped layer of the plan against the oracle
            errs = [oracle_check(torch, mb, pl[i], px[i], py[i])[0] for i in (0, len(pl) - 1)]
            return {"layers": len(pl), "tokens": T, "kernel": plan_mlp.kernel(1), "ms_per_pass": ms,
                    "us_per_layer": ms * 1e3 / len(pl), "GB/s": nbytes / ms / 1e6,
                    "pct_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS * 100.0, "max_rel_err_vs_oracle": max(errs)}

        extras["mlp_plan_T1"] = time_mlp_plan(1, 300 // q)
        extras["mlp_plan_T16"] = time_mlp_plan(16, 150 // q)

        # (7) the quantizer's projection on the GPU: MSVID_16 of a 4096 x 2656 factor (the shape of U for the
        #     attention projections), 8 passes; checked on a 512 x 384 matrix by Theorem 1's closed form (error of
        #     the projection = tail of |Z|'s spectrum, from numpy's SVD)
        def time_msvid(rows, cols, l, iters, reps):
            gen = torch.Generator(device="cuda:0")
            gen.manual_seed(77)
            Z = torch.randn((rows, cols), generator=gen, device="cuda:0")
            b = mb.mdbf_msvid_block(l)
            X0 = torch.randn((cols, b), generator=gen, device="cuda:0")
            need = mb.C.c_size_t(0)
            mb.lib().mdbf_msvid_workspace_bytes(rows, cols, l, mb.C.byref(need))
            wsb = torch.empty(need.value, dtype=torch.uint8, device="cuda:0")
            fn = lambda: mb.mdbf_msvid(Z, l, X0, iters=iters, workspace=wsb)
            preheat(torch, fn, min(a.preheat_ms, 50.0))
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            # Z is read once per product (2 per pass + 1 for the Rayleigh-Ritz step) and once, with a transposed
            # copy and the int8 mask written, at the start
            nbytes = (2 * iters + 1 + 2) * rows * cols * 4 + rows * cols
            Zs = synth.normal_block(512, 384, 5).astype(np.float64)
            S, A, Q, sg = mb.mdbf_msvid(torch.from_numpy(Zs.astype(np.float32)).cuda(), l,
                                        torch.from_numpy(synth.normal_block(384, b, 6)).cuda(), iters=iters)
            torch.cuda.synchronize()
            sig = np.linalg.svd(np.abs(Zs), compute_uv=False)
            err = np.linalg.norm(Zs - S.cpu().numpy() * (A.cpu().numpy().astype(np.float64) @ Q.cpu().numpy().astype(np.float64).T))
            return {"rows": rows, "cols": cols, "l": l, "passes": iters, "ms_per_call": ms,
                    "error_over_optimum_512x384": float(err / np.sqrt((sig[l:] ** 2).sum())),
                    "mask_exact_512x384": bool((S.cpu().numpy() == np.where(Zs < 0, -1, 1)).all()),
                    "roofline": {"bound": "hbm", "kernel": "abs_t_mul_kernel", "achieved": nbytes / ms / 1e6,
                                 "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": nbytes / ms / 1e6 / HBM_PEAK_GBS,
                                 "algorithmic_bytes_per_call": nbytes}}

        extras["msvid_4096x2656_l16"] = time_msvid(4096, 2656, 16, 8, 100 // q)

        # (8) the decoder stack at 1.5 bits per weight (224 matrices of the LLaMA-7B shapes, one plan) with 1 and
        #     8 tokens per matrix, and the toy configuration (256 x 256, k = 128, l = 4, fp32: latency only)
        import types
        stack = {}
        for T in (1, 8):
            r = workloads.run_stack(torch, types.SimpleNamespace(budget="1.5", tokens=T, warmup=30 // q + 1,
                                                                 passes=100 // q))
            stack[T] = r
        toy, toyX = synth.config_toy()
        tdl = mb.DeviceLayer.from_host(toy)
        tX = torch.from_numpy(toyX).cuda()
        tY = mb.mdbf_forward(tdl, tX, y_dtype="f32")
        torch.cuda.synchronize()
        toy_err, _ = oracle_check(torch, mb, tdl, tX, tY)
        e0.record()
        for _ in range(200 // q):
            mb.mdbf_forward(tdl, tX, y_dtype="f32", Y=tY)
        e1.record()
        torch.cuda.synchronize()
        toy_us = e0.elapsed_time(e1) * 1e3 / (200 // q)

        # ---- one typed record per benchmark configuration (the figures above, with their roof)
        def hbm_roof(gbs_):
            return {"bound": "hbm", "peak": HBM_PEAK_GBS, "unit": "GB/s", "achieved": gbs_, "frac": gbs_ / HBM_PEAK_GBS}
        pre = extras["prefill_T2048_attn"]
        t16 = extras["decode_T16_mlp_gate"]
        extras["records"] = [
            {"config": 1, "workload": "toy 256x256 k=128 l=4 T=1, fp32 in/out, one mdbf_forward call", "us_per_call": toy_us,
             "max_rel_err_vs_oracle": toy_err, "roofline": None, "note": "launch-bound: 22 KB of operands"},
            {"config": 2, "workload": "attn decode 4096x4096 k=2656 l=16 T=1, %d layers per plan" % a.copies,
             "kernel": plan.kernel(1), "ms_per_pass": ms_step, "roofline": hbm_roof(gbs),
             "max_rel_err_vs_oracle": max(err, err_last)},
            {"config": 2, "workload": "the same layer, one mdbf_forward call (two launches)", "kernel": "stage_mx_split_kernel",
             "us_per_call": extras["single_call_stream"]["us_per_call"],
             "roofline": hbm_roof(bytes_call / extras["single_call_stream"]["us_per_call"] / 1e3)},
            {"config": 3, "workload": "MLP projections 11008x4096 / 4096x11008 k=4096 l=16 T=1, 96 layers per plan",
             "kernel": extras["mlp_plan_T1"]["kernel"], "ms_per_pass": extras["mlp_plan_T1"]["ms_per_pass"],
             "roofline": hbm_roof(extras["mlp_plan_T1"]["GB/s"]),
             "max_rel_err_vs_oracle": extras["mlp_plan_T1"]["max_rel_err_vs_oracle"]},
            {"config": 3, "workload": "the same with T=16", "kernel": extras["mlp_plan_T16"]["kernel"],
             "ms_per_pass": extras["mlp_plan_T16"]["ms_per_pass"], "roofline": hbm_roof(extras["mlp_plan_T16"]["GB/s"]),
             "max_rel_err_vs_oracle": extras["mlp_plan_T16"]["max_rel_err_vs_oracle"],
             "note": "the binding roof at 16 tokens is the matrix cores (l-expanded or reconstruct order), not HBM"},
            {"config": 3, "workload": "gate projection 11008x4096 k=4096 T=16, one mdbf_forward call",
             "kernel": "stage_gemm_split_kernel", "ms_per_call": t16["ms_per_call"], "roofline": t16["roofline"]},
            {"config": 4, "workload": "prefill 4096x4096 k=2656 l=16 T=2048, one mdbf_forward call",
             "kernel": "stage_gemm_kernel", "ms_per_call": pre["ms_per_call"], "tokens_per_s": pre["tokens_per_s"],
             "dense_equivalent_TFLOPs": pre["dense_equivalent_TFLOPs"], "roofline": pre["roofline"]},
            {"config": 5, "workload": "decoder stack 1.5 bpw, 224 matrices per plan, T=1", "ms_per_pass": stack[1]["ms_per_pass"],
             "roofline": hbm_roof(stack[1]["GB/s"])},
            {"config": 5, "workload": "decoder stack 1.5 bpw, 224 matrices per plan, T=8", "ms_per_pass": stack[8]["ms_per_pass"],
             "roofline": hbm_roof(stack[8]["GB/s"]),
             "note": "matrix-core bound (reconstruct-order kernel); HBM fraction for comparison only"},
        ]

    out = {
        "metric": "MDBF decode GEMV HBM GB/s (% peak) + prefill TFLOP/s, LLaMA-7B shapes",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_OF_KERNEL.get(plan.kernel(1), "f16"), "data": "synthetic",
        "config": {"workload": "attn_decode 4096x4096 k=2656 l=16 T=1 (1.503 bpw), %d independent layers per step "
                               "via mdbf_forward_batch" % a.copies,
                   "copies": a.copies, "algorithmic_bytes_per_call": bytes_call,
                   "bytes_per_step": bytes_step},
        "pct_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS,
        "us_per_layer": ms_step * 1e3 / a.copies,
        "max_rel_err_vs_oracle": max(err, err_last),
        "preheat_ms": preheat_ms,
        "roofline": roof,
    }
    out.update(extras)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host_args, Xs[0])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
