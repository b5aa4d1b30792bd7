"""Benchmark of the NAtS-L hybrid-attention forward on one MI355X.

One step = one pass of the whole hot path (mask scan + K/V compaction, linear branch,
softmax branch over the compacted keys, merge) over one batch of seeded synthetic input
already resident in HBM.  Workload: B=2, H=16, L=8192, d=128, C=64, bf16, 5% softmax tokens.
Prints one JSON line: whole-job tokens/s (tokens = B*L), the roofline of the dominant kernel
(HIP-event timing of each kernel inside the timed region) and the CPU oracle timed on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK = {"hbm": (8000.0, "GB/s"), "mfma": (2500.0, "TFLOP/s"), "alu_f32": (157.3, "TFLOP/s")}

# the launches that together are the linear branch's segmented scan (recurrence, output and merge)
SEG_SCAN = ("gdn_seg_pass1", "gdn_seg_fix", "gdn_seg_pass2")


def kernel_work(name, cfg, sum_cnt):
    """Algorithmic work of one forward call that falls to each kernel -> (bound, amount).

    bytes for HBM-bound kernels, FLOP for the kernels whose work is dense products (priced against the
    bf16/fp16 matrix-core peak whatever the time they take is really spent on).  Only what the method needs is
    counted: work a kernel repeats to run segments of the recurrence side by side is not."""
    BH, L, d, C = cfg.B * cfg.H, cfg.L, cfg.d, cfg.C
    n_tok = BH * L
    esz = 2 if cfg.dtype == "bf16" else 4
    if name == "scan_compact":      # mask in, cnt + idx out, gathered K/V rows in and out
        n_soft = int(round(cfg.p_softmax * n_tok))
        return "hbm", n_tok * (1 + 4) + n_soft * (4 + 4 * d * esz)
    if name == "gdn_recurrent":     # per row-token: decay d, S.k 2d, rank-1 2d, S.q 2d (fp32 VALU)
        return "alu_f32", n_tok * d * (7 * d)
    if name == "softmax_fp32":      # QK^T and PV: 4 d FLOP per visible (query, key) pair (fp32 VALU)
        return "alu_f32", 4 * d * sum_cnt
    if name == "gdn_chunk_inv":     # K K^T and Q K^T (2 x 2 C d per token) and the triangular solve (C^2 / 3)
        return "mfma", n_tok * (4 * C * d + C * C / 3.0)
    if name == "gdn_seg_scan":      # K S0^T, Q S0^T, U^T K (3 x 2 d^2) and T (.), P U and the W-type product (3 x 2 C d)
        return "mfma", n_tok * (6 * d * d + 6 * C * d)
    if name == "flash_softmax":
        return "mfma", 4 * d * sum_cnt
    return None


def profile_cell(fname, kernel, column):
    """Cell (as text) of the row `kernel` under the header `column` in a committed rocprofv3 summary table."""
    try:
        header = None
        for line in open(os.path.join(ROOT, "profiles", fname)):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) < 3:
                continue
            if header is None and column in cells:
                header = cells
            elif header is not None and cells[1] == kernel:
                return cells[header.index(column)]
    except (OSError, ValueError):
        pass
    return None


def measured_traffic_bytes(kernel):
    """HBM bytes per forward call of `kernel` from the committed rocprofv3 --pmc summary (None if absent)."""
    c = profile_cell("fwd_cfg2_headline_bf16_hbm_traffic.md", kernel, "total MB")
    return float(c) * 1e6 if c else None


def measured_mfma_busy(kernel):
    """Share of the busy CU cycles in which a matrix instruction was executing, from the committed counter summary."""
    c = profile_cell("fwd_cfg2_headline_bf16_mfma_lds_counters.md", kernel, "MFMA utilisation")
    try:
        return float(c.split("%")[0]) / 100.0
    except (AttributeError, ValueError):
        return None


def preheat_chip(ms, kind="mfma"):
    """Keeps the chip busy for about `ms` with work that is no part of the path, so that what follows starts at
    operating clocks (see the note where the forward's steps are timed).  Returns the milliseconds it took."""
    import torch

    from paper_2602_03681_amd import binding as nb
    if ms <= 0:
        return 0.0
    dev = torch.device("cuda:0")
    if kind in ("copy", "mix"):
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
    scratch = torch.empty(4096, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    p0 = time.perf_counter()
    while (time.perf_counter() - p0) * 1e3 < ms:
        if kind in ("copy", "mix"):
            for _ in range(20):
                dst.copy_(src)
        if kind in ("mfma", "mix"):
            nb.probe_mfma(4000, scratch)
        torch.cuda.synchronize()
    return (time.perf_counter() - p0) * 1e3


def measure_decode(steps, warmup, split=True, preheat_ms=200.0):
    """Decode workload (B=64, H=16, d=128, bf16, cache length U{64..2048}): HBM-bound streaming of the
    fp32 state (read + write) and the live cache rows, one call per token.  split: the step runs on a caller
    workspace as many blocks of equal size (two launches) instead of one block per (batch, head)."""
    import numpy as np
    import torch

    import paper_2602_03681_amd as nats
    from paper_2602_03681_amd import binding as nb
    from nats_inputs import CONFIGS, make_decode_inputs

    cfg = CONFIGS["cfg4_decode_bf16"]
    steps = max(steps, 1)
    x = make_decode_inputs(cfg, steps=steps + warmup)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    g = {}
    for k, v in x.items():
        if isinstance(v, np.ndarray):
            t = torch.from_numpy(v).to(dev)
            g[k] = t.to(torch.bfloat16) if k in ("q", "k", "v", "k_cache", "v_cache") else t
    o = torch.empty((cfg.B, cfg.H, cfg.d), dtype=torch.bfloat16, device=dev)
    ws = None
    if split:
        ws = torch.empty(nb.decode_workspace_bytes(cfg.B, cfg.H, cfg.d, g["k_cache"].shape[2], nb.NATS_BF16),
                         dtype=torch.uint8, device=dev)

    def step(i):
        nats.hybrid_attn_decode(g["state"], g["k_cache"], g["v_cache"], g["cache_len"], g["q"][i], g["k"][i],
                                g["v"][i], g["alpha"][i], g["beta"][i], g["mask"][i], out=o, workspace=ws)

    preheat_chip(preheat_ms)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    len0 = g["cache_len"].sum().item()
    nb.profile_begin(4 * steps)
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern = nb.profile_end()
    len1 = g["cache_len"].sum().item()
    ms = (t1 - t0) * 1e3 / steps
    bh, d = cfg.B * cfg.H, cfg.d
    bytes_per_step = bh * 8 * d * d + 0.5 * (len0 + len1) * 4 * d      # state r+w (fp32) + live K,V rows (bf16)
    kernel_ms = sum(k["total_ms"] for k in kern.values()) / steps        # all launches of a step
    achieved = bytes_per_step / (kernel_ms * 1e-3) / 1e9
    return {"metric": "hybrid_attn_decode_tokens_per_s", "value": round(cfg.B / (ms * 1e-3), 1), "unit": "tokens/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "cfg4_decode_bf16: B=64 H=16 d=128, cache length U{64..2048}, one token per step"
                                   + (", step as equal blocks on a caller workspace" if split else "")},
            "kernels_ms": {k: round(v["total_ms"] / steps, 4) for k, v in kern.items()},
            "roofline": {"kernel": "+".join(kern) if kern else "decode", "bound": "hbm", "achieved": round(achieved, 1),
                         "peak": 8000.0, "unit": "GB/s", "frac": round(achieved / 8000.0, 4), "traffic": None,
                         "algorithmic_bytes": int(bytes_per_step), "avg_kernel_ms": round(kernel_ms, 4)},
            "cpu_baseline": None}


def bench_decode(args):
    out = measure_decode(args.steps, args.warmup, split=not args.decode_one_block, preheat_ms=args.preheat_ms)
    print(json.dumps(out))


def bench_backward(args):
    print(json.dumps(measure_backward(args.steps, args.warmup, args.routing, args.backward_by_tokens, args.combine_mode,
                                      preheat_ms=args.preheat_ms)))


def measure_backward(steps_in, warmup_in, routing_name="token", by_tokens=False, combine_mode=0, preheat_ms=200.0):
    """Backward pass on workload 2's shapes (bf16 tensors, fp32 gradients): a step is one nats_hybrid_attn_bwd call.
    The linear branch's adjoint runs by chunks on fp32 matrix instructions (operands per chunk, states forwards,
    state gradients backwards, then every chunk's gradients); the softmax branch's products run on fp16 / bf16 matrix
    instructions with two-term fp16 weights.  Roofline: fp32 matrix peak for the chunk kernels, counted per chunk of
    64 tokens with triangular products at 10 of 16 tiles.  combine_mode 1, 2: the backward through the merge of Eq. 21
    (its single-normalisation ablation), which widens the tensors and runs the fp32 kernels."""
    import torch

    import paper_2602_03681_amd as nats
    from paper_2602_03681_amd import binding as nb
    from nats_inputs import CONFIGS, make_config_inputs, make_grad_output

    cfg = CONFIGS["cfg2_headline_bf16"]
    x = make_config_inputs(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    g = {k: torch.from_numpy(v).to(dev) for k, v in x.items()}
    Q, K, V = (g[k].to(torch.bfloat16) for k in ("Q", "K", "V"))
    dO = torch.from_numpy(make_grad_output(cfg.B, cfg.H, cfg.L, cfg.d, "bf16", seed=cfg.seed + 1)).to(dev).to(torch.bfloat16)
    import ctypes
    math = nb.NATS_MATH_FP32 if by_tokens else nb.NATS_MATH_AUTO
    routing = nb.NATS_ROUTE_CHUNK if routing_name == "chunk" else nb.NATS_ROUTE_TOKEN
    if routing == nb.NATS_ROUTE_CHUNK:   # same shapes and softmax share, one routing decision per chunk of 64 tokens
        from nats_inputs import make_chunk_mask
        mask_c = make_chunk_mask(cfg.B, cfg.H, cfg.L // cfg.C, cfg.p_softmax, cfg.seed + 1)
        mask_c[:, :, 0] = 1
        g["mask"] = torch.from_numpy(mask_c).to(dev)
    prm = nb.make_fwd_params(cfg.B, cfg.H, cfg.L, cfg.d, cfg.C, nb.NATS_BF16, math=math, routing=routing,
                             combine_mode=combine_mode)
    ws = torch.empty(int(nb.load_library().nats_hybrid_attn_bwd_workspace_bytes(ctypes.byref(prm))), dtype=torch.uint8,
                     device=dev)

    def step():
        return nats.hybrid_attn_bwd(Q, K, V, g["alpha"], g["beta"], g["mask"], dO, workspace=ws, math=math, routing=routing,
                                    combine_mode=combine_mode)

    steps = max(1, min(steps_in, 20))
    preheat_chip(preheat_ms)
    for _ in range(max(1, min(warmup_in, 3))):
        step()
    torch.cuda.synchronize()
    nb.profile_begin(32 * steps)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    kern = nb.profile_end(32)
    n_tok = cfg.B * cfg.H * cfg.L
    n_chunks, d = n_tok // 64, cfg.d
    tri = 10.0 / 16.0   # tiles of a 64 x 64 triangular operand that are multiplied
    sq, st = 2.0 * 64 * d * d, 2.0 * 64 * 64 * d   # a [64 x d] . [d x d] product, a [64 x 64] . [64 x d] one
    flops = {   # per chunk
        "gdn_bwd_prep": 2 * tri * st,                       # K K^T, Q K^T
        "gdn_chunk_states": 2 * sq + 2 * tri * st,          # K S^T, the state update; T and At products
        "gdn_chunk_state_grads": 3 * sq + 2 * tri * st,     # K dS^T, two state updates; P^T and T^T products
        "gdn_chunk_grads": 3 * sq + 4 * tri * st + st,      # dO' S0, dR S0, U dS1; dP, dAt, (dP.G) K, (dP.G)^T Q; symmetric . K
        "gdn_chunk_out": sq + tri * st,                     # Q S0^T, P U (the branch's rows for the merge's adjoint)
        # token by token: about 25 d_k flops per state row and token (re-run of the chunk, then the adjoint)
        "gdn_recurrent_bwd": 25.0 * 64 * d * d,
    }
    dom = max(kern, key=lambda k: kern[k]["total_ms"])
    roofs = {}
    for k, f in flops.items():
        if k in kern:
            ach = f * n_chunks / (kern[k]["avg_ms"] * 1e-3) / 1e12
            roofs[k] = {"bound": "alu" if k == "gdn_recurrent_bwd" else "mfma", "achieved": round(ach, 3), "peak": 157.3,
                        "unit": "TFLOP/s", "frac": round(ach / 157.3, 5), "avg_kernel_ms": round(kern[k]["avg_ms"], 4)}
    lead = max(roofs, key=lambda k: roofs[k]["avg_kernel_ms"])
    out = {"metric": "hybrid_attn_bwd_tokens_per_s", "value": round(cfg.B * cfg.L / (ms * 1e-3), 1), "unit": "tokens/s",
           "n_gpus": 1, "steps": steps, "warmup": warmup_in, "ms_per_step": round(ms, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "backward of cfg2_headline_bf16" + (", routing per chunk" if routing_name == "chunk" else "")
                                  + " (bf16 tensors, fp32 gradients; linear branch "
                                  + ("token by token in fp32" if by_tokens else "by chunks on fp32 MFMA")
                                  + (", softmax-branch products on MFMA with two-term fp16 weights)" if combine_mode == 0 else
                                     f", through the merge combine_mode {combine_mode}: tensors widened, fp32 kernels)")},
           "kernels_ms": {k: round(v["avg_ms"], 4) for k, v in kern.items()}, "dominant": dom,
           "roofline": dict(kernel=lead, traffic=None, **roofs[lead]), "kernel_rooflines": roofs,
           "cpu_baseline": None}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
    ap.add_argument("--preheat-kind", choices=("copy", "mfma", "mix"), default="mfma",
                    help="what keeps the chip busy: device copies, the matrix-instruction probe, or both in turn")
    ap.add_argument("--preheat-ms", type=float, default=200.0,
                    help="keep the chip busy with work that is no part of the path for about this long before the "
                         "warm-up steps, so that they start at operating clocks (0: off)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain 256 MiB device copy: the known-size dispatch against which "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a captured HIP graph (extra key graph_replay_ms_per_step)")
    ap.add_argument("--probes", action="store_true",
                    help="also time an MFMA-issue probe and a 256 MiB copy and report them as measured_peaks")
    ap.add_argument("--routing", choices=("token", "chunk"), default="token",
                    help="granularity of the routing mask: per token (default, the headline workload) or per chunk")
    ap.add_argument("--gdn-segments", type=int, default=0,
                    help="segments per (batch, head) of the linear branch's recurrence (0: the library's choice)")
    ap.add_argument("--decode", action="store_true", help="measure the decode workload instead of the forward")
    ap.add_argument("--decode-one-block", action="store_true",
                    help="with --decode: one block per (batch, head), no workspace (the step's other form)")
    ap.add_argument("--no-decode-line", action="store_true",
                    help="leave the short decode measurement out of the forward's JSON line")
    ap.add_argument("--no-backward-line", action="store_true",
                    help="leave the short backward measurement out of the forward's JSON line")
    ap.add_argument("--backward", action="store_true", help="measure the backward pass instead")
    ap.add_argument("--combine-mode", type=int, default=0, choices=[0, 1, 2],
                    help="--backward only: the merge the backward runs through (0 plain sum, 1 Eq. 21, 2 one normalisation)")
    ap.add_argument("--backward-by-tokens", action="store_true",
                    help="with --backward: the linear branch's adjoint token by token (math = NATS_MATH_FP32)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")

    if args.decode:
        return bench_decode(args)
    if args.backward:
        return bench_backward(args)

    import numpy as np
    import torch

    import paper_2602_03681_amd as nats
    from paper_2602_03681_amd import binding as nb
    from nats_inputs import CONFIGS, make_config_inputs

    cfg = CONFIGS["cfg2_headline_bf16"]
    x = make_config_inputs(cfg)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    g = {k: torch.from_numpy(v).to(dev) for k, v in x.items()}
    Q, K, V = (g[k].to(torch.bfloat16) for k in ("Q", "K", "V"))
    alpha, beta, mask = g["alpha"], g["beta"], g["mask"]
    routing = nb.NATS_ROUTE_CHUNK if args.routing == "chunk" else nb.NATS_ROUTE_TOKEN
    if routing == nb.NATS_ROUTE_CHUNK:
        # same shapes and softmax share, one routing decision per chunk of 64 tokens (Section 4.1 as stated)
        from nats_inputs import make_chunk_mask
        mask_c = make_chunk_mask(cfg.B, cfg.H, cfg.L // cfg.C, cfg.p_softmax, cfg.seed + 1)
        mask_c[:, :, 0] = 1
        x["mask"] = mask_c
        mask = torch.from_numpy(mask_c).to(dev)
        tok = np.repeat(mask_c, cfg.C, axis=-1).astype(np.int64)
        before = np.cumsum(tok, axis=-1) - tok * (np.arange(cfg.L) % cfg.C + 1)      # rows of earlier chunks
        sum_cnt = int((before + np.arange(cfg.L) % cfg.C + 1).sum())                # + own chunk, causally
    else:
        sum_cnt = int(np.cumsum(x["mask"] != 0, axis=-1, dtype=np.int64).sum())
    params = nb.make_fwd_params(cfg.B, cfg.H, cfg.L, cfg.d, cfg.C, nb.NATS_BF16, routing=routing,
                                gdn_segments=args.gdn_segments)
    ws = torch.empty(nb.fwd_workspace_bytes(params), dtype=torch.uint8, device=dev)
    O = torch.empty_like(Q)

    def step():
        nats.hybrid_attn_fwd(Q, K, V, alpha, beta, mask, cfg.C, routing=routing, out=O, workspace=ws,
                             gdn_segments=args.gdn_segments)

    preheat_ms = 0.0
    if args.preheat_ms > 0:
        # A GPU that has been idle (a fresh box, the seconds of input generation above) runs its first tens of
        # milliseconds of work below its operating clocks: measured here, 20 steps after 5 warm-up steps take 0.27 ms
        # each from idle and 0.238 ms after 200 ms of any matrix-core load, the same as after 200 or 1000 warm-up steps
        # of the path itself.  So before the warm-up steps the chip is kept busy for about preheat_ms with work that is
        # no part of the path (the matrix-instruction probe of nats_measure.h, a chip-filling loop of independent MFMA;
        # or device copies, which bring the clocks up only part of the way: 0.249 ms), and the W + K steps run at the
        # clocks a running service sees.  The line reports "preheat_ms" and "preheat_kind"; --preheat-ms 0 turns it off.
        preheat_ms = preheat_chip(args.preheat_ms, args.preheat_kind)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if not args.no_kernel_events:
        nb.profile_begin(64 * args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernels = {} if args.no_kernel_events else nb.profile_end()
    graph_ms = None
    if args.graph:
        # the same step replayed from a HIP graph (launch gaps removed); reported beside the eager figure
        gs = torch.cuda.Stream()
        gs.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(gs):
            with torch.cuda.graph(graph, stream=gs):
                step()
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - g0) * 1e3 / args.steps
    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
    measured_peaks = None
    if args.probes:
        scratch = torch.empty(4096, dtype=torch.float32, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        nb.probe_mfma(2000, scratch)
        torch.cuda.synchronize()
        e0.record()
        flop = nb.probe_mfma(20000, scratch)
        e1.record()
        torch.cuda.synchronize()
        mfma_tflops = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 10 * 2 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        measured_peaks = {"mfma_f16_16x16x32_TFLOPs": round(mfma_tflops, 1), "copy_256MiB_GBs": round(copy_gbs, 1)}
        del src, dst
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens = cfg.B * cfg.L
    value = tokens / (ms_per_step * 1e-3)

    # per step: time and algorithmic work of each kernel; the two passes and the fix-up of the segmented scan count
    # as one kernel (its average duration is the sum of the three launches' averages)
    per_step = {}
    for name, k in kernels.items():
        key = "gdn_seg_scan" if name in SEG_SCAN else name
        per_step[key] = per_step.get(key, 0.0) + k["total_ms"] / args.steps
    n_tok = cfg.B * cfg.H * cfg.L
    compulsory = 4 * n_tok * cfg.d * 2 + 8 * n_tok + n_tok      # Q, K, V in, O out; alpha, beta; mask
    kernel_rooflines = {}
    for name, ms in per_step.items():
        work = kernel_work(name, cfg, sum_cnt)
        if work is None:
            continue
        bound, amount = work
        peak, unit = PEAK[bound]
        ach = amount / (ms * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
        kernel_rooflines[name] = {"bound": {"hbm": "hbm", "mfma": "mfma", "alu_f32": "alu"}[bound],
                                  "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
                                  "work": amount, "ms_per_step": round(ms, 4),
                                  "traffic": measured_traffic_bytes(name), "mfma_busy": measured_mfma_busy(name)}
    roofline = None
    if per_step:
        dom = max(per_step, key=per_step.get)
        if dom in kernel_rooflines:
            r = kernel_rooflines[dom]
            roofline = {"kernel": dom, "bound": r["bound"], "achieved": r["achieved"], "peak": r["peak"],
                        "unit": r["unit"], "frac": r["frac"], "traffic": r["traffic"],
                        "avg_kernel_ms": r["ms_per_step"], "mfma_busy": r["mfma_busy"],
                        "launches": [n for n in SEG_SCAN if n in kernels] if dom == "gdn_seg_scan" else [dom]}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import c_oracle
        heads = 16      # all heads of batch 0, all L tokens: each (b,h) is an independent unit and takes one thread
        xs = {k: np.ascontiguousarray(v[:1, :heads]) for k, v in x.items()}
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 20:
            c0 = time.perf_counter()
            c_oracle.fwd(**xs, want=(), chunk_routing=cfg.C if args.routing == "chunk" else 0)
            t_cpu += time.perf_counter() - c0
            reps += 1
        head_tok_per_s = reps * heads * cfg.L / t_cpu
        cpu_baseline = {"value": round(head_tok_per_s / cfg.H, 1), "unit": "tokens/s",
                        "cores": min(c_oracle.threads(), heads), "kind": "oracle",
                        "sample": f"{heads} of {cfg.B * cfg.H} (batch, head) pairs, all {cfg.L} tokens, "
                                  f"{reps} repetitions; rate scaled by 1/H to whole tokens"}

    out = {"metric": "hybrid_attn_fwd_tokens_per_s", "value": round(value, 1), "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": "cfg2_headline_bf16: B=2 H=16 L=8192 d=128 C=64 bf16, mask~Bernoulli(0.05)"
                                  + (" per chunk of 64 tokens (routing per chunk)" if args.routing == "chunk" else ""),
                      "global_batch": cfg.B, "seq_len": cfg.L, "heads": cfg.H, "d_head": cfg.d,
                      "parallelism": "single GPU"},
           "kernels_ms": {k: round(v["total_ms"] / args.steps, 4) for k, v in kernels.items()},
           "kernel_launches_per_step": {k: v["launches"] // args.steps for k, v in kernels.items()},
           "roofline": roofline, "kernel_rooflines": kernel_rooflines, "cpu_baseline": cpu_baseline}
    if not args.no_decode_line:
        # the decode workload beside the headline figure (30 steps after 5): tokens/s and its HBM roofline
        del Q, K, V, O, ws
        torch.cuda.empty_cache()
        dec = measure_decode(30, 5, preheat_ms=args.preheat_ms)
        out["decode"] = {k: dec[k] for k in ("metric", "value", "unit", "ms_per_step", "config", "kernels_ms", "roofline")}
    if not args.no_backward_line:
        # ... and the backward pass on the headline shapes (10 calls after 2)
        torch.cuda.empty_cache()
        bw = measure_backward(10, 2, args.routing, preheat_ms=args.preheat_ms)
        out["backward"] = {k: bw[k] for k in ("metric", "value", "unit", "ms_per_step", "config", "kernels_ms", "roofline")}
    if measured_peaks is not None:
        out["measured_peaks"] = measured_peaks
    if graph_ms is not None:
        out["graph_replay_ms_per_step"] = round(graph_ms, 4)
    flop_total = 4.0 * cfg.d * sum_cnt + (10.0 * cfg.C * cfg.d + 6.0 * cfg.d ** 2 + cfg.C ** 2 / 3.0) * cfg.B * cfg.H * cfg.L
    out["algorithmic_TFLOPs"] = round(flop_total / (ms_per_step * 1e-3) / 1e12, 2)
    out["preheat_ms"] = round(preheat_ms, 1)
    out["preheat_kind"] = args.preheat_kind if preheat_ms > 0 else None
    out["mfma_frac_whole_forward"] = round(flop_total / (ms_per_step * 1e-3) / 1e12 / PEAK["mfma"][0], 4)
    tr = [measured_traffic_bytes(k) for k in per_step]
    measured = sum(tr) if tr and all(t is not None for t in tr) else None
    out["hbm_bytes"] = {"compulsory": compulsory, "measured": measured}
    # HBM rate of the whole step: the bytes the counters saw per call (committed summary) over this run's step time,
    # against the published 8 TB/s
    if measured is not None:
        gbps = measured / (ms_per_step * 1e-3) / 1e9
        out["hbm_GBps"] = {"achieved": round(gbps, 1), "peak": PEAK["hbm"][0], "frac": round(gbps / PEAK["hbm"][0], 4)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
