"""Run one of the named synthetic workloads on cuda:0 and print its time per pass.

    python3 -m paper_2512_24545_amd.workloads stack   --budget 1.5 --tokens 8 --passes 300 --warmup 100
    python3 -m paper_2512_24545_amd.workloads prefill --tokens 2048 --x-dtype f16 --passes 200 --warmup 300

`stack`: the 32-layer decoder stack (224 independent products per pass: q, k, v, o, gate, up, down per
layer, LLaMA-7B shapes at the given bit budget), `--tokens` activations per matrix, issued as one plan
through mdbf_forward_batch.  `prefill`: one 4096 x 4096, k = 2656, l = 16 layer with `--tokens` tokens
through mdbf_forward.  Layers are drawn on the device (random packed sign words, envelopes
|N(0,1)| * 0.02 + 1e-3 in fp16, activations N(0,1)).  With few passes and no warm-up this is the program to
put under a profiler; bench.py remains the benchmark.
"""
import argparse
import json
import sys

from . import binding as mb
from . import synth


def _device_layer(torch, g, m, n, k, l):
    def words(nbytes):
        w = torch.randint(-2 ** 31, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, generator=g, device="cuda:0")
        return w.view(torch.uint8)

    def env(rows):
        return (torch.randn((rows, l), generator=g, device="cuda:0").abs() * 0.02 + 1e-3).half()

    return mb.DeviceLayer(m, n, k, l, words(mb.mdbf_packed_bytes(m, k)), words(mb.mdbf_packed_bytes(k, n)),
                          env(m), env(k), env(k), env(n))


def _time(torch, fn, warmup, passes):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(passes):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / passes


def run_stack(torch, args):
    g = torch.Generator(device="cuda:0")
    g.manual_seed(5)
    T = args.tokens
    specs = [synth.stack_matrix_spec(args.budget, 0, mat) for mat in range(7)]
    layers, Xs, Ys, nbytes = [], [], [], 0
    for _ in range(32):
        for sp in specs:
            m, n, k, l = sp["m"], sp["n"], sp["k"], sp["l"]
            layers.append(_device_layer(torch, g, m, n, k, l))
            Xs.append(torch.randn((T, n), generator=g, device="cuda:0").half())
            Ys.append(torch.zeros((T, m), dtype=torch.float16, device="cuda:0"))
            nbytes += (m + n) * k // 8 + 2 * l * (m + n + 2 * k) + T * 2 * (m + n)
    plan = mb.BatchPlan(layers, Xs, Ys)
    ms = _time(torch, plan.run, args.warmup, args.passes)
    return {"workload": "stack", "budget_bpw": args.budget, "matrices": len(layers), "tokens": T,
            "ms_per_pass": ms, "algorithmic_MB": nbytes / 1e6, "GB/s": nbytes / ms / 1e6,
            "pct_hbm_peak": nbytes / ms / 1e6 / 80.0}


def run_prefill(torch, args):
    m, n, k, l, T = 4096, 4096, 2656, 16, args.tokens
    g = torch.Generator(device="cuda:0")
    g.manual_seed(4)
    dl = _device_layer(torch, g, m, n, k, l)
    xdt = {"f16": torch.float16, "bf16": torch.bfloat16}[args.x_dtype]
    X = torch.randn((T, n), generator=g, device="cuda:0").to(xdt)
    Y = torch.empty((T, m), dtype=torch.float32, device="cuda:0")
    d = dl.desc(args.x_dtype, "f32")
    ws = torch.empty(mb.mdbf_workspace_bytes(d, T), dtype=torch.uint8, device="cuda:0")
    ms = _time(torch, lambda: mb.mdbf_forward(dl, X, y_dtype="f32", Y=Y, workspace=ws), args.warmup, args.passes)
    return {"workload": "prefill", "tokens": T, "x_dtype": args.x_dtype, "ms_per_call": ms,
            "tokens_per_s": T / ms * 1e3, "dense_equivalent_TFLOPs": 2.0 * m * n * T / ms / 1e9,
            "issued_TFLOPs": 2.0 * (m + n) * k * (T + l) / ms / 1e9}


def main(argv=None):
    ap = argparse.ArgumentParser(prog="python3 -m paper_2512_24545_amd.workloads")
    ap.add_argument("workload", choices=["stack", "prefill"])
    ap.add_argument("--budget", default="1.5", choices=["1.0", "1.5", "2.0"])
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--x-dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--passes", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=100)
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        sys.exit("this program needs a GPU")
    mb.lib()
    if args.tokens is None:
        args.tokens = 8 if args.workload == "stack" else 2048
    out = run_stack(torch, args) if args.workload == "stack" else run_prefill(torch, args)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
