#!/usr/bin/env python3
"""Benchmark of the fused QCMD/QRDA adagrad step on one MI355X.

Default workload ("largest"): d = 2^30 fp32 parameters, M = 64 workers whose gradients are
generated on the device (Laplace(0,1e-3), 95 % exact zeros), quantized bucket by bucket (4096)
and kept only as packed 2-bit codes + scales; steps alternate QCMD (tracking z) and QRDA on
shared state.  The generator and the quantizer run before the timed region (the quantizer's
own rate is reported separately); a timed step is one fused unpack+average+accumulate+update
pass over all d coordinates.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build is single-GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak

# HBM bytes per launch from rocprofv3 --pmc runs of this same command (FETCH_SIZE, WRITE_SIZE,
# each scaled by what the counter reads for a plain elementwise kernel of known size: FETCH_SIZE
# reads half the true KiB on this chip, WRITE_SIZE the true KiB).  NOT measured in this run: the
# figures are copied from the profile summary named beside them and are reported together with
# that file's name; null for workloads that were not profiled.
TRAFFIC_SOURCE = "profiles/step_kernel_largest_traffic.txt"
PROFILED_TRAFFIC_BYTES = {
    ("largest", "qcmd_z"): 30.60e9 + 12.885e9,
    ("largest", "qrda"): 26.31e9 + 12.885e9,
}

WORKLOADS = {
    # name: d, M, bucket, generator, lambda, bytes/coord as {kernel: B}
    "largest": dict(d=1 << 30, M=64, bucket=4096, gen="laplace", lam=1e-6,
                    schedule="alternate"),
    "opt_qcmd": dict(d=10 ** 8, M=8, bucket=4096, gen="student", lam=1e-5, schedule="qcmd"),
    "opt_qrda": dict(d=250_000_000, M=32, bucket=4096, gen="gauss", lam=1e-5, schedule="qrda"),
    # the paper's literal setting: one threshold/scale per message and q_t = Q(SynQ_t) with one scale
    "opt_qcmd_global": dict(d=10 ** 8, M=8, bucket=0, gen="student", lam=1e-5, schedule="qcmd",
                            requant="global"),
    "mid": dict(d=1 << 26, M=64, bucket=4096, gen="laplace", lam=1e-6, schedule="alternate"),
    # whole Algorithm-1 steps (local gradients -> quantize+pack -> fused QCMD step) on the
    # synthetic stand-ins for the paper's linear-model experiments
    "tiny_train": dict(train="dense", d=1000, n=4096, M=4, B=64, bucket=0, lam=1e-3),
    "sparse_train": dict(train="csr", d=1 << 20, n=1 << 16, M=16, B=256, bucket=4096, lam=1e-4),
    # worker/server side of the sparse encoding: indicator -> Q(S(g, I)) -> decode
    "select": dict(select=True, d=1 << 28, M=8, bucket=4096),
    # the same with the paper's own message: one scale, d indicator bits, one stream of 2k code bits
    "select_one_scale": dict(select=True, d=1 << 28, M=8, bucket=0),
    "select_bucket_256": dict(select=True, d=1 << 28, M=8, bucket=256),
    # stochastic (TernGrad/Philox) quantizer against the threshold quantizer on the same input
    "stochastic": dict(stoch=True, d=1 << 28, M=4, bucket=4096),
    # a convolutional net's parameter list in one flat vector, each tensor quantized on its own
    "multi_tensor": dict(segments=True, M=8),
    "small": dict(d=1 << 22, M=64, bucket=4096, gen="laplace", lam=1e-6, schedule="alternate"),
}


def algorithmic_bytes_per_coord(kind, M):
    """Bytes the method itself must move per coordinate and step: 2-bit codes of M workers
    plus the fp32 state each kernel reads and writes (scales add 4*M/4096, ignored)."""
    return {"qcmd": 16 + M / 4, "qcmd_z": 24 + M / 4, "qrda": 20 + M / 4}[kind]


def train_bench(args, wl, qa, synth, torch, np, dev):
    """K full steps of Algorithm 1 (minus indicator/selection): M local gradients, one batched
    quantize+pack, one fused QCMD step.  Row ids of all steps are uploaded before timing."""
    d, M, B, bucket, lam, n = wl["d"], wl["M"], wl["B"], wl["bucket"], wl["lam"], wl["n"]
    eta, delta = 0.1, 1e-8
    csr = wl["train"] == "csr"
    prob = synth.csr_problem(n=n, d=d, M=M, seed=1) if csr else synth.dense_problem(n=n, d=d, M=M, seed=0)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    if csr:
        A, indptr, indices = up(prob.vals), up(prob.indptr), up(prob.indices)
    else:
        A, indptr, indices = up(prob.A), None, None
    y = up(prob.y)
    L = qa.Layout.make(d, M, bucket)
    gs = ((d + 3) // 4) * 4
    x, G, z = (torch.zeros(d, dtype=torch.float32, device=dev) for _ in range(3))
    g = torch.zeros((M, gs), dtype=torch.float32, device=dev)
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=dev)
    scales = torch.zeros((M, L.scale_stride), dtype=torch.float32, device=dev)
    ws = lambda op: torch.empty(max(qa.qa_workspace_bytes(L, op), 256), dtype=torch.uint8, device=dev)
    ws_g = ws(qa.QA_OP_GRAD_CSR if csr else qa.QA_OP_GRAD_DENSE)
    ws_q, ws_s = ws(qa.QA_OP_QUANTIZE), ws(qa.QA_OP_STEP)
    total = args.warmup + args.steps
    rows = up(np.stack([synth.minibatch_rows(n, M, B, t, 1) for t in range(1, total + 1)]))
    fmt = qa.QA_CSR if csr else qa.QA_DENSE

    def step(t):
        qa.qa_local_grad_batched(fmt, A, indptr, indices, n, d, y, rows[t], B, M, x, g, gs, None, ws_g)
        qa.qa_quantize_pack(L, g, gs, codes, scales, None, 0, ws_q)
        qa.qa_step_qcmd(L, codes, scales, x, G, None, eta, lam, delta, qa.QA_REQUANT_NONE, ws_s)

    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()
    graph = None
    if args.graph:
        # the K timed steps as ONE HIP graph (every call only enqueues kernels): one launch
        keep = [v.clone() for v in (x, G, z)]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for t in range(args.warmup, total):
                step(t)
        for v, k in zip((x, G, z), keep):       # capture does not run the steps; start from the
            v.copy_(k)                          # state after the warm-up all the same
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for t in range(args.warmup, total):
            step(t)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    out = {"metric": "full Algorithm-1 step (M local gradients + quantize+pack + fused QCMD): coordinates/s",
           "value": d * args.steps / wall, "unit": "coordinates/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{args.workload}: d={d}, n={n}, M={M}, B={B}, bucket={bucket}, "
                                  f"{wl['train']} rows", "launches_per_step": (4 if csr else 2) + 2,
                      "hip_graph": bool(args.graph)},
           "nnz_x_after": int((x != 0).sum().item())}
    print(json.dumps(out))


def select_bench(args, wl, qa, synth, torch, np, dev):
    """Indicator, selected quantize+pack and decode for M workers; each kernel timed alone."""
    d, M, bucket = wl["d"], wl["M"], wl["bucket"]
    eta, lam, delta = 0.1, 1e-4, 1e-8
    L = qa.Layout.make(d, M, bucket)
    nb, NW = L.n_buckets, (d + 31) // 32
    g = torch.empty((M, d), dtype=torch.float32, device=dev)
    for m in range(M):
        synth.grad_laplace_sparse(d, m, 1, device=dev, out=g[m])
    gen = torch.Generator(device=dev); gen.manual_seed(5)
    x = torch.randn(d, generator=gen, device=dev) * (torch.rand(d, generator=gen, device=dev) < 0.02)
    G = torch.rand(d, generator=gen, device=dev) * 1e-6
    z = torch.zeros(d, dtype=torch.float32, device=dev)
    ind = torch.zeros((M, NW), dtype=torch.int32, device=dev)
    sel = torch.zeros((M, L.code_stride), dtype=torch.int32, device=dev)
    dense = torch.zeros((M, L.code_stride), dtype=torch.int32, device=dev)
    cnt = torch.zeros((M, nb), dtype=torch.int32, device=dev)
    sc = torch.zeros((M, nb), dtype=torch.float32, device=dev)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    def wsp(op):
        n = qa.qa_workspace_bytes(L, op)
        return torch.empty(n, dtype=torch.uint8, device=dev) if n else None

    ws_sel, ws_step = wsp(qa.QA_OP_SELECT), wsp(qa.QA_OP_STEP_SELECTED)
    t_ind = timed(lambda: qa.qa_indicator(L, qa.QA_METHOD_QCMD, g, d, x, G, z, 1, eta, lam, delta, ind, NW))
    t_q = timed(lambda: qa.qa_quantize_pack_selected(L, g, d, ind, NW, sel, cnt, sc, None, ws_sel))
    t_dec = timed(lambda: qa.qa_decode_selected(L, ind, NW, sel, dense, ws_sel))
    again = torch.zeros((M, L.code_stride), dtype=torch.int32, device=dev)
    cnt2 = torch.zeros((M, nb), dtype=torch.int32, device=dev)
    t_selc = timed(lambda: qa.qa_select_codes(L, dense, ind, NW, again, cnt2, ws_sel))   # the pull direction's S
    # the server's update: dense step on the decoded codes vs the step that reads the sparse
    # messages directly (state copies so that both start from the same x, G, z each time)
    xs, Gs, zs = x.clone(), G.clone(), z.clone()
    t_step_dense = timed(lambda: qa.qa_step_qcmd(L, dense, sc, xs, Gs, zs, eta, lam, delta,
                                                 qa.QA_REQUANT_NONE, None))
    xs.copy_(x); Gs.copy_(G); zs.copy_(z)
    t_step_sparse = timed(lambda: qa.qa_step_qcmd_selected(L, ind, NW, sel, sc, xs, Gs, zs, eta, lam,
                                                           delta, qa.QA_REQUANT_NONE, ws_step))
    k = int(cnt.sum().item())
    frac = k / (M * d)
    by = {"indicator": (4 * M + 8 + M / 8) * d, "quantize_selected": M * d * (4 + 1 / 8) + k / 4,
          "decode": M * d * (1 / 8 + 1 / 4) + k / 4, "select_codes": M * d * (1 / 8 + 1 / 4) + k / 4}
    by["step_qcmd_dense_codes"] = d * (M / 4 + 24)
    by["step_qcmd_selected"] = d * (M / 8 + 24) + k / 4
    ms = {"indicator": t_ind, "quantize_selected": t_q, "decode": t_dec, "select_codes": t_selc,
          "step_qcmd_dense_codes": t_step_dense, "step_qcmd_selected": t_step_sparse}
    out = {"metric": "sparse encoding kernels: worker-coordinates/s (indicator + Q(S(g,I)) + decode)",
           "value": M * d / ((t_ind + t_q + t_dec) * 1e-3), "unit": "worker-coordinates/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_ind + t_q + t_dec,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": f"{args.workload}: d={d}, M={M}, bucket={bucket}, selected fraction {frac:.4f}"},
           "kernels": {n: {"ms": ms[n], "algorithmic_GBps": by[n] / (ms[n] * 1e-3) / 1e9,
                           "frac_of_peak": by[n] / (ms[n] * 1e-3) / 1e9 / HBM_PEAK_GBPS} for n in ms},
           "message_bits_vs_dense": (M * (32 * nb + d) + 2 * k) / (M * (32 * nb + 2 * d))}
    print(json.dumps(out))


def stochastic_bench(args, wl, qa, synth, torch, np, dev):
    d, M, bucket = wl["d"], wl["M"], wl["bucket"]
    L = qa.Layout.make(d, M, bucket)
    g = torch.empty((M, d), dtype=torch.float32, device=dev)
    for m in range(M):
        synth.grad_gaussian_biased(d, m, 1, device=dev, out=g[m])
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=dev)
    scales = torch.zeros((M, L.scale_stride), dtype=torch.float32, device=dev)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    t_s = timed(lambda: qa.qa_quantize_pack_stochastic(L, g, d, codes, scales, 7, 1))
    t_t = timed(lambda: qa.qa_quantize_pack(L, g, d, codes, scales, None, 0, None))
    th = torch.zeros((M, L.scale_stride), dtype=torch.float32, device=dev)
    t_e = timed(lambda: qa.qa_quantize_pack(L, g, d, codes, scales, th, qa.QA_THRESH_EXACT, None))
    gb = 4.25 * M * d / 1e9
    out = {"metric": "stochastic ternary quantize+pack: worker-coordinates/s",
           "value": M * d / (t_s * 1e-3), "unit": "worker-coordinates/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_s, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"stochastic: d={d}, M={M}, bucket={bucket}, dense Gaussian gradients"},
           "kernels": {"stochastic": {"ms": t_s, "algorithmic_GBps": gb / (t_s * 1e-3),
                                      "frac_of_peak": gb / (t_s * 1e-3) / HBM_PEAK_GBPS},
                       "threshold": {"ms": t_t, "algorithmic_GBps": gb / (t_t * 1e-3),
                                     "frac_of_peak": gb / (t_t * 1e-3) / HBM_PEAK_GBPS},
                       # ranking per 4096-bucket + threshold quantizer: reads g twice
                       "exact_threshold": {"ms": t_e, "algorithmic_GBps": (gb + 4 * M * d / 1e9) / (t_e * 1e-3)}}}
    print(json.dumps(out))


def conv_net_tensor_list():
    """Synthetic parameter list with the length mix of an AlexNet-style CIFAR classifier with
    batch normalisation before every layer (5 conv + 3 fully connected layers: a few tensors of
    10^5..10^7.6 weights, many of 10^1..10^3.6 biases and normalisation parameters)."""
    lengths = []
    cin = 3
    for k, cout in ((11, 96), (5, 256), (3, 384), (3, 384), (3, 256)):
        lengths += [cin, cin, k * k * cin * cout, cout]          # bn scale, bn shift, kernel, bias
        cin = cout
    fin = 256 * 6 * 6
    for fout in (4096, 4096, 10):
        lengths += [fin, fin, fin * fout, fout]
        fin = fout
    begin, pos = [], 0
    for n in lengths:
        begin.append(pos)
        pos = (pos + n + 15) // 16 * 16
    return begin, lengths, pos


def segments_bench(args, wl, qa, synth, torch, np, dev):
    M = wl["M"]
    begin, length, d = conv_net_tensor_list()
    nseg = len(begin)
    L = qa.Layout.make(d, M, 0, 0.75, None, nseg)
    table = torch.zeros(qa.qa_segment_plan_bytes(d, nseg), dtype=torch.uint8, device=dev)
    plan = qa.qa_segment_plan_init(d, begin, length, table)
    g = torch.empty((M, d), dtype=torch.float32, device=dev)
    for m in range(M):
        synth.grad_gaussian_biased(d, m, 1, device=dev, out=g[m])
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=dev)
    scales = torch.zeros((M, nseg), dtype=torch.float32, device=dev)
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    G = torch.zeros(d, dtype=torch.float32, device=dev)
    z = torch.zeros(d, dtype=torch.float32, device=dev)
    wq = torch.empty(qa.qa_segment_workspace_bytes(plan, M, qa.QA_OP_QUANTIZE), dtype=torch.uint8, device=dev)
    wst = torch.empty(qa.qa_segment_workspace_bytes(plan, M, qa.QA_OP_STEP), dtype=torch.uint8, device=dev)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    covered = float(sum(length))
    t_q = timed(lambda: qa.qa_quantize_pack_segments(L, plan, g, d, codes, scales, None, wq))
    t_s = timed(lambda: qa.qa_step_qcmd_segments(L, plan, codes, scales, x, G, z, 0.1, 1e-5, 1e-8, 0, None))
    t_r = timed(lambda: qa.qa_step_qrda_segments(L, plan, codes, scales, x, G, z, 3, 0.1, 1e-5, 1e-8,
                                                 qa.QA_REQUANT_BUCKET, wst))
    by_q = 8.25 * M * covered            # gradient read twice (two passes), codes written once
    by_s = (24 + M / 4) * covered
    by_r = (4 + M / 4 + 8.25 + 20 + 0.25) * covered   # average out, quantize it, update from it
    total = t_q + t_s
    out = {"metric": "tensor-list step (quantize+pack of M gradients + fused QCMD step): coordinates/s",
           "value": covered / (total * 1e-3), "unit": "coordinates/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": total, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"multi_tensor: {nseg} tensors, {int(covered)} parameters "
                                  f"(lengths {min(length)}..{max(length)}), M={M}, {plan.n_pieces} pieces"},
           "kernels": {"quantize_pack_segments": {"ms": t_q, "algorithmic_GBps": by_q / (t_q * 1e-3) / 1e9},
                       "step_qcmd_segments": {"ms": t_s, "algorithmic_GBps": by_s / (t_s * 1e-3) / 1e9},
                       "step_qrda_segments_requant": {"ms": t_r, "algorithmic_GBps": by_r / (t_r * 1e-3) / 1e9}}}
    print(json.dumps(out))


DEVICE_STATE = None


def device_state():
    """Clocks, performance level and power cap of the first AMD GPU as sysfs shows them (plain
    file reads: no child process), or None where those files are not visible."""
    import glob
    try:
        for dev_dir in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
            if not os.path.exists(os.path.join(dev_dir, "pp_dpm_sclk")):
                continue

            def read(rel):
                try:
                    with open(os.path.join(dev_dir, rel)) as f:
                        return f.read().strip()
                except OSError:
                    return None

            def current(rel):                    # the level marked with '*'
                txt = read(rel)
                if not txt:
                    return None
                cur = [ln for ln in txt.splitlines() if ln.rstrip().endswith("*")]
                return (cur[0] if cur else txt.splitlines()[-1]).replace("*", "").strip()

            out = {"sclk": current("pp_dpm_sclk"), "mclk": current("pp_dpm_mclk"),
                   "fclk": current("pp_dpm_fclk"),
                   "performance_level": read("power_dpm_force_performance_level")}
            caps = glob.glob(os.path.join(dev_dir, "hwmon", "hwmon*", "power1_cap"))
            if caps:
                with open(caps[0]) as f:
                    out["power_cap_W"] = int(f.read().strip()) / 1e6
            out = {k: v for k, v in out.items() if v is not None}
            return dict(out, read="sysfs, before the run, GPU idle") if out else None
    except Exception:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="largest", choices=sorted(WORKLOADS))
    ap.add_argument("--code-pad-words", type=int, default=None,
                    help="extra 32-bit words between workers' code streams (default: every "
                         "worker's stream starts on a 1 KiB boundary, 3 KiB (mod 16 KiB) after "
                         "the previous one: with a power-of-two distance the M streams of a tile "
                         "meet in the same memory channels, measured 1-6 %% slower)")
    ap.add_argument("--state-placement", choices=("spread", "block"), default=None,
                    help="x, G, z as rows chosen by a short probe among five allocations lying "
                         "about 44 GiB apart plus the three rows of a contiguous block (spread: "
                         "the default from d = 2^26 on), or simply as one contiguous [3][d] block "
                         "(block).  The record carries the probe's table and, for spread, the "
                         "step times of a fresh block measured after the timed steps")
    ap.add_argument("--placement-probe", choices=("all", "first"), default="all",
                    help="spread placement: time every combination of three candidate rows and take the "
                         "fastest (default), or stop at the first that reaches the rate of a plain copy")
    ap.add_argument("--placement-rows", default=None,
                    help="with spread placement: take these three of the eight candidate rows as "
                         "x, G, z (e.g. 0,1,4) instead of probing, and skip the block's measurement: "
                         "for profiler runs, whose per-kernel statistics count every launch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="tiny_train / sparse_train: replay the timed steps from one HIP graph")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (workers and server are slices of "
              "one GPU's memory); --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    global DEVICE_STATE
    DEVICE_STATE = device_state()          # before this process touches the GPU

    import numpy as np
    import torch

    import paper_2208_05631_amd as qa
    from paper_2208_05631_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = WORKLOADS[args.workload]
    if "train" in wl:
        return train_bench(args, wl, qa, synth, torch, np, dev)
    if "select" in wl:
        return select_bench(args, wl, qa, synth, torch, np, dev)
    if "stoch" in wl:
        return stochastic_bench(args, wl, qa, synth, torch, np, dev)
    if "segments" in wl:
        return segments_bench(args, wl, qa, synth, torch, np, dev)
    d, M, bucket, lam = wl["d"], wl["M"], wl["bucket"], wl["lam"]
    eta, delta = 0.1, 1e-8
    W = (d + 15) // 16
    if args.code_pad_words is None:
        args.code_pad_words = qa.Layout.spaced_code_stride(d) - W
    L = qa.Layout.make(d, M, bucket, code_stride=W + args.code_pad_words)
    gen = {"laplace": synth.grad_laplace_sparse, "student": synth.grad_student_t_sparse,
           "gauss": synth.grad_gaussian_biased}[wl["gen"]]

    # ---- state first (the resident arrays are allocated once, before any temporary) ----
    # One [3][row] block, rows a multiple of 64 KiB apart: the step time depends on how x, G and z
    # lie relative to each other (measured in one process: +4 % when G and z are shifted by 4 KiB
    # and 8 KiB against x), and three separate allocations leave that to the allocator.
    row = (d + 16383) // 16384 * 16384
    if args.state_placement is None:
        args.state_placement = "spread" if d >= (1 << 26) else "block"
    placement = {"mode": args.state_placement}
    if args.state_placement == "spread":
        # Five candidate rows far apart in device memory; which three serve as x, G, z is decided
        # by a probe once the messages exist (below), before the warm-up.
        from paper_2208_05631_amd import placement as qa_placement
        cand, spacer = qa_placement.spread_rows(5, row, dev)
        # ... and a contiguous block's three rows: in some processes those are the fast ones
        cand_block = torch.zeros((3, row), dtype=torch.float32, device=dev)
        cand += [cand_block[0], cand_block[1], cand_block[2]]
        placement.update(candidates="rows 0-4: separate allocations %.0f GiB apart; rows 5-7: one "
                                    "contiguous [3][d] block" % (spacer / 2**30))
        state = None
        x, G, z = cand[0][:d], cand[1][:d], cand[2][:d]
    else:
        state = torch.zeros((3, row), dtype=torch.float32, device=dev)
        x, G, z = state[0, :d], state[1, :d], state[2, :d]

    # ---- inputs: generate each worker's gradient on the device, quantize, keep only codes ----
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=dev)
    scales = torch.zeros((M, L.scale_stride), dtype=torch.float32, device=dev)
    L1 = qa.Layout.make(d, 1, bucket, code_stride=L.code_stride, scale_stride=L.scale_stride)
    gbuf = torch.empty(d, dtype=torch.float32, device=dev)
    nq = qa.qa_workspace_bytes(L1, qa.QA_OP_QUANTIZE)
    wsq = torch.empty(nq, dtype=torch.uint8, device=dev) if nq else None
    requant = {"none": qa.QA_REQUANT_NONE, "global": qa.QA_REQUANT_GLOBAL}[wl.get("requant", "none")]
    ns = qa.qa_workspace_bytes(L, qa.QA_OP_STEP) if requant else 0
    wss = torch.empty(ns, dtype=torch.uint8, device=dev) if ns else None
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    q_ms = []
    for m in range(M):
        gen(d, m, 1, device=dev, out=gbuf)
        ev0.record()
        qa.qa_quantize_pack(L1, gbuf, d, codes[m], scales[m], None, 0, wsq)
        ev1.record()
        torch.cuda.synchronize()
        q_ms.append(ev0.elapsed_time(ev1))
    del gbuf          # stays in torch's cache: returning 4 GiB to the driver here stalls the queue
    quant_ms = float(np.median(q_ms[1:] if M > 1 else q_ms))
    # all M gradients in one call, when they fit beside everything else (same codes and scales come out)
    quant_all_ms = None
    if M > 1 and M * d * 4 <= (16 << 30) and d % 4 == 0:
        gall = torch.empty((M, d), dtype=torch.float32, device=dev)
        for m in range(M):
            gen(d, m, 1, device=dev, out=gall[m])
        nqa = qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE)
        wsa = torch.empty(nqa, dtype=torch.uint8, device=dev) if nqa else None
        qa.qa_quantize_pack(L, gall, d, codes, scales, None, 0, wsa)
        ev0.record()
        for _ in range(3):
            qa.qa_quantize_pack(L, gall, d, codes, scales, None, 0, wsa)
        ev1.record()
        torch.cuda.synchronize()
        quant_all_ms = ev0.elapsed_time(ev1) / 3
        del gall, wsa
    qbytes = 4.25 if 0 < bucket <= 4096 else 8.25      # larger buckets read the gradient twice

    def kind_of(t):
        if wl["schedule"] == "alternate":
            return "qcmd_z" if t % 2 == 1 else "qrda"
        return wl["schedule"]

    def step(t):
        k = kind_of(t)
        if k == "qrda":
            qa.qa_step_qrda(L, codes, scales, x, G, z, t, eta, lam, delta, requant, wss)
        else:
            qa.qa_step_qcmd(L, codes, scales, x, G, z if k == "qcmd_z" else None, eta, lam, delta,
                            requant, wss)
        return k

    def probe_ms(rx, rG, rz, n=4):
        # n steps of the timed schedule on these rows (after one untimed step)
        nonlocal x, G, z
        x, G, z = rx[:d], rG[:d], rz[:d]
        step(1)
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        for s_ in range(n):
            step(2 + s_)
        p1.record()
        torch.cuda.synchronize()
        return p0.elapsed_time(p1) / n

    if args.state_placement == "spread":
        if args.placement_rows:
            best = tuple(int(v) for v in args.placement_rows.split(","))
            assert len(best) == 3 and len(set(best)) == 3 and all(0 <= v < len(cand) for v in best)
            placement.update(chosen=list(best), probe_ms_per_step=None)
        else:
            # All 56 combinations are timed (four steps each, under two seconds in all) and the
            # fastest is taken; with --placement-probe first the search stops at the first one
            # that is good enough = the step's bytes at 101 % of the rate a plain copy reaches
            # in this process (combinations in index order, separate rows first).
            pa = torch.empty(min(d, 1 << 30), dtype=torch.float32, device=dev).fill_(1.0)
            pb = torch.empty_like(pa)
            for _ in range(2):
                torch.mul(pa, 1.0, out=pb)
            p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            p0.record()
            for _ in range(5):
                torch.mul(pa, 1.0, out=pb)
            p1.record()
            torch.cuda.synchronize()
            copy_rate = 8.0 * pa.numel() * 5 / (p0.elapsed_time(p1) * 1e-3)          # bytes/s
            del pa, pb
            sched = [kind_of(2 + s_) for s_ in range(4)]
            step_bytes = sum(algorithmic_bytes_per_coord(k_, M) for k_ in sched) / len(sched) * d
            target_ms = step_bytes / (1.01 * copy_rate) * 1e3
            best, table = qa_placement.choose_rows(
                cand, 3, probe_ms, good_enough_ms=target_ms if args.placement_probe == "first" else None)
            placement.update(chosen=list(best), probe=args.placement_probe,
                             good_enough_ms=round(target_ms, 3), tried=len(table),
                             probe_ms_per_step={str(c): round(v, 3) for c, v in table.items()})
        placement["row_ptrs"] = [hex(r.data_ptr()) for r in cand]
        keep = [cand[i] for i in best]
        del cand, cand_block
        for r in keep:
            r.zero_()                                     # the probe stepped on them
        x, G, z = keep[0][:d], keep[1][:d], keep[2][:d]
        torch.cuda.empty_cache()

    t = 0
    for _ in range(args.warmup):
        t += 1
        step(t)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, inputs resident in HBM ----
    events = []
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        t += 1
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()                      # the kernels run on torch's current stream
        k = step(t)
        e1.record()
        events.append((k, e0, e1))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin

    per_kind = {}
    for k, e0, e1 in events:
        per_kind.setdefault(k, []).append(e0.elapsed_time(e1))
    kernels = {}
    for k, ms in per_kind.items():
        avg = float(np.mean(ms))
        bpc = algorithmic_bytes_per_coord(k, M)
        if requant:      # separate passes: average out (M/4 + 4; also leaves the quantizer's tile
            # sums), quantize it (4.25: one pass over it), update from its codes (0.25 + state)
            bpc = (M / 4 + 4) + 4.25 + (bpc - M / 4 + 0.25)
        kernels[k] = {"avg_ms": avg, "median_ms": float(np.median(ms)), "min_ms": float(np.min(ms)),
                      "max_ms": float(np.max(ms)), "launches": len(ms), "bytes_per_coord": bpc,
                      "achieved_GBps": bpc * d / (avg * 1e-3) / 1e9,
                      "frac": bpc * d / (avg * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    dominant = max(kernels, key=lambda k: kernels[k]["avg_ms"] * kernels[k]["launches"])
    dk = kernels[dominant]
    nnz_x = int((x != 0).sum().item())

    def timed_launches(fn, n):
        fn()                                                  # one untimed launch first
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        for _ in range(n):
            fn()
        a1.record()
        torch.cuda.synchronize()
        return a0.elapsed_time(a1) / n

    def entry(avg, n, bpc):
        gbps = bpc * d / (avg * 1e-3) / 1e9
        return {"avg_ms": avg, "launches": n, "bytes_per_coord": bpc, "achieved_GBps": gbps,
                "frac": gbps / HBM_PEAK_GBPS}

    # Other calls on the same resident messages, after the K timed steps and not part of them,
    # each with as many launches as a kernel of the timed schedule got.
    also = {}
    n_also = max(3, args.steps // 2)
    if wl["schedule"] == "alternate":
        # plain QCMD: z not tracked, 16 + M/4 B per coordinate (equation QCMD as printed)
        avg = timed_launches(lambda: qa.qa_step_qcmd(L, codes, scales, x, G, None, eta, lam, delta,
                                                     qa.QA_REQUANT_NONE, None), n_also)
        also["qcmd"] = entry(avg, n_also, algorithmic_bytes_per_coord("qcmd", M))
        # row a4 alone: the average written out as fp32 (M/4 B of codes in, 4 B out per coordinate)
        gbar = torch.empty(d, dtype=torch.float32, device=dev)
        avg = timed_launches(lambda: qa.qa_aggregate_unpack(L, codes, scales, gbar), n_also)
        also["aggregate_unpack"] = entry(avg, n_also, M / 4 + 4)
        del gbar          # stays in torch's cache (see the note on the gradient buffer above)
        # the paper's double quantization at bucket granularity, formed inside the same kernel
        if 0 < bucket <= 4096:
            rq = qa.QA_REQUANT_BUCKET
            avg = timed_launches(lambda: qa.qa_step_qcmd(L, codes, scales, x, G, z, eta, lam, delta, rq,
                                                         None), n_also)
            also["qcmd_z_requant_bucket"] = entry(avg, n_also, algorithmic_bytes_per_coord("qcmd_z", M))
            # the server's call alone: messages in, q_t = Q(SynQ_t) out as a one-worker message
            qc = torch.zeros((1, L.code_stride), dtype=torch.int32, device=dev)
            qs = torch.zeros((1, L.scale_stride), dtype=torch.float32, device=dev)
            avg = timed_launches(lambda: qa.qa_aggregate_quantize(L, codes, scales, rq, qc, qs, None, None),
                                 n_also)
            also["aggregate_quantize_bucket"] = entry(avg, n_also, M / 4 + 0.25)
            del qc, qs

    # ---- the same schedule with x, G, z as one contiguous block, for the record ----
    if args.state_placement == "spread" and wl["schedule"] == "alternate" and not args.placement_rows:
        blk = torch.zeros((3, row), dtype=torch.float32, device=dev)
        kx, kG, kz = x, G, z
        x, G, z = blk[0, :d], blk[1, :d], blk[2, :d]
        placement["block_ms"] = {
            "qcmd_z": timed_launches(lambda: step(1), n_also),
            "qrda": timed_launches(lambda: step(2), n_also)}
        x, G, z = kx, kG, kz
        del blk

    # ---- what this machine's memory system gives a plain copy: fp32 elementwise kernel with 128-bit
    # accesses (torch's), min(d, 2^30) elements, 8 B moved per element ----
    n_copy = min(d, 1 << 30)
    src = torch.empty(n_copy, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty(n_copy, dtype=torch.float32, device=dev)
    copy_ms = timed_launches(lambda: torch.mul(src, 1.0, out=dst), 10)
    copy_gbps = 8.0 * n_copy / (copy_ms * 1e-3) / 1e9
    del src, dst

    out = {
        "metric": "fused QCMD/QRDA step: coordinates/s and achieved HBM GB/s (% peak), 1 MI355X",
        "value": d * args.steps / wall,
        "unit": "coordinates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: d={d}, M={M}, bucket={bucket}, "
                               f"{wl['gen']} gradients as packed 2-bit codes, schedule={wl['schedule']}, "
                               f"requant={wl.get('requant', 'none')}", "d": d, "M": M, "bucket": bucket,
                   "code_pad_words": args.code_pad_words,
                   "messages": "one set of M quantized gradients, generated and quantized before the "
                               "timed region, is re-used by every step (the step time depends on "
                               "the values by about 2 %)",
                   "state_placement": ("x, G, z: three of eight candidate rows (five separate allocations "
                                       "about 44 GiB apart, three rows of one block), chosen by a probe of "
                                       "four steps per combination before the warm-up (state_placement in "
                                       "this record has the table and a contiguous block's times)"
                                       if args.state_placement == "spread" else
                                       "x, G, z: one contiguous [3][d] block")},
        "roofline": {"bound": "hbm", "kernel": f"step_lut_kernel[{dominant}]",
                     "achieved": dk["achieved_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": dk["achieved_GBps"] / HBM_PEAK_GBPS,
                     "algorithmic_bytes": dk["bytes_per_coord"] * d,
                     "traffic": PROFILED_TRAFFIC_BYTES.get((args.workload, dominant)),
                     "traffic_source": (TRAFFIC_SOURCE + " (rocprofv3 --pmc runs of this command; "
                                        "not measured in this run)"
                                        if (args.workload, dominant) in PROFILED_TRAFFIC_BYTES else None),
                     "copy_GBps": copy_gbps, "frac_of_copy": dk["achieved_GBps"] / copy_gbps,
                     "copy_kernel": f"torch.mul(src, 1.0, out=dst), {n_copy} fp32, 8 B per element, "
                                    f"{copy_ms:.3f} ms"},
        "kernels": kernels,
        "kernels_outside_timed_steps": also,
        "quantize_pack": {"ms_per_worker": quant_ms, "worker_coords_per_s": d / (quant_ms * 1e-3),
                          "achieved_GBps": qbytes * d / (quant_ms * 1e-3) / 1e9,
                          "frac": qbytes * d / (quant_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                          "all_workers_one_call_ms": quant_all_ms,
                          "all_workers_one_call_GBps": (qbytes * d * M / (quant_all_ms * 1e-3) / 1e9
                                                        if quant_all_ms else None)},
        # rows a2-a8 together for this configuration: M quantize+pack launches (measured above, one
        # worker's fp32 gradient at a time: M of them do not fit beside the state) + the fused step
        "quantize_plus_step": {"ms_per_step": M * quant_ms + wall * 1e3 / args.steps,
                               "coordinates_per_s": d / ((M * quant_ms + wall * 1e3 / args.steps) * 1e-3),
                               "algorithmic_bytes_per_coord": M * qbytes + sum(
                                   v["bytes_per_coord"] * v["launches"] for v in kernels.values()) / args.steps},
        "nnz_x_after": nnz_x,
        "device": torch.cuda.get_device_name(0),
        "device_state": DEVICE_STATE,
        # where the big blocks lie: the step time depends on their placement in device memory
        "buffers": {"state": hex(x.data_ptr()), "codes": hex(codes.data_ptr())},
        # how x, G, z were placed in device memory (see paper_2208_05631_amd/placement.py)
        "state_placement": placement,
    }

    # ---- CPU baseline: the oracle as it stands, one host thread pinned to one core, on a
    # bounded sample: the first ds coordinates of the same messages ----
    if not args.no_cpu_baseline:
        import oracle
        ds = min(d, 1 << 22)
        Ws, nbs = ds // 16, (ds // bucket if bucket else 1)
        c_s = codes[:, :Ws].cpu().numpy().view(np.uint32).copy()
        s_s = scales[:, :nbs].cpu().numpy().copy()
        ox, oG, oz = (np.zeros(ds, np.float32) for _ in range(3))
        n_cpu = 30                                # about 15 s of one host core
        oracle.lib()
        allowed = sorted(os.sched_getaffinity(0))
        core = allowed[len(allowed) // 2]
        os.sched_setaffinity(0, {core})
        try:
            c0 = time.perf_counter()
            for tt in range(1, n_cpu + 1):
                if kind_of(tt) == "qrda":
                    oracle.step_qrda(c_s, s_s, ds, bucket, ox, oG, oz, tt, eta, lam, delta)
                else:
                    oracle.step_qcmd(c_s, s_s, ds, bucket, ox, oG, oz if kind_of(tt) == "qcmd_z" else None,
                                     eta, lam, delta, requant)
            cpu_s = time.perf_counter() - c0
        finally:
            os.sched_setaffinity(0, set(allowed))
        model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                for line in f:
                    if line.startswith("model name"):
                        model = line.split(":", 1)[1].strip()
                        break
        except OSError:
            pass
        out["cpu_baseline"] = {"value": ds * n_cpu / cpu_s, "unit": "coordinates/s", "cores": 1,
                               "kind": "oracle", "cpu_model": model, "nproc": os.cpu_count(),
                               "cpus_allowed": len(allowed), "pinned_to_core": core,
                               "sample": f"first {ds} coordinates (all {M} workers), {n_cpu} steps of "
                                         f"the timed schedule, {cpu_s:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
