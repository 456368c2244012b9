#!/usr/bin/env python3
"""Benchmark of the MI355X NMT training step.

One "step" is one weight update of Transformer-big in fp16 with dynamic loss scaling over the 16
sub-batches (at most 3584 tokens each) of configuration 4.  Two launch configurations of the same
update are timed over the same number of steps and reported side by side:
  * `value` / `ms_per_step`: the sentences of all 16 sub-batches packed into ONE forward + backward
    pass (same sentences, dropout masks and sums; gradients summed in fp32 inside the weight-gradient
    products), one accumulate call, overflow check + Adam -- the form a 288 GB GPU allows;
  * `strict_order`: the method's literal loop, 16 x (forward + loss, backward, accumulate) over the
    padded sub-batches one by one, then overflow check + Adam.
Inputs are synthetic (seeded length / token distributions standing in for the paper's WMT
sub-batches) and resident in HBM before the timed region starts.  Prints ONE JSON line: the
headline fields, `roofline` (the GEMM products of the timed step, from HIP events around each),
`whole_update`, `strict_order`, `phases_ms_per_update`, `hbm_kernels`, `fp32_comparison`, `cpu_baseline`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload big_accum|big|big40k|base]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0      # MI355X dense fp16 MFMA peak (published)
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E peak (published)

WORKLOAD_DESC = {
    "big_accum": ("big", 16, "Transformer-big (6+6, d=1024, F=4096, 16 heads, V=32768), the 16 sub-batches of <=3584 tokens of one update"),
    "big": ("big", 1, "Transformer-big, one sub-batch of <=3584 tokens per update"),
    "big40k": ("big40k", 4, "Transformer-big with V=40000, 4 sub-batches of <=5120 tokens per update"),
    "base": ("base", 1, "Transformer-base (6+6, d=512), one sub-batch of <=3584 tokens per update"),
}


def model_flops(model, B, S, T):
    """Algorithmic FLOPs of one sub-batch's forward + backward (3x forward; padded positions count,
    causal self-attention counts half a square; recomputation is not counted)."""
    d, F, V, Le, Ld = model["d_model"], model["d_ff"], model["vocab"], model["enc_layers"], model["dec_layers"]
    Ns, Nt = B * S, B * T
    enc = Le * (Ns * (8 * d * d + 4 * d * F) + 4 * B * S * S * d)
    dec = Ld * (Nt * (12 * d * d + 4 * d * F) + Ns * 4 * d * d + 2 * B * T * T * d + 4 * B * T * S * d)
    return 3 * (enc + dec + 2 * Nt * d * V)


def model_flops_packed(model, src_lens, tgt_lens):
    """The same count over the real (non-pad) positions of every sentence."""
    d, F, V, Le, Ld = model["d_model"], model["d_ff"], model["vocab"], model["enc_layers"], model["dec_layers"]
    ls, lt = src_lens.astype(float), tgt_lens.astype(float)
    enc = Le * (ls * (8 * d * d + 4 * d * F) + 4 * ls * ls * d)
    dec = Ld * (lt * (12 * d * d + 4 * d * F) + ls * 4 * d * d + 2 * lt * lt * d + 4 * lt * ls * d)
    return float((3 * (enc + dec + 2 * lt * d * V)).sum())


def gemm_shapes(model, Ns, Nt):
    """(M, N, K, a_t, b_t, count, epilogue) of every GEMM of one forward + backward pass over Ns source and
    Nt target positions.  epilogue: what the step's kernel does besides the product, because it decides
    which kernel form runs: "bias" / "bias_relu" (forward), "none", "add" (an input gradient that adds the
    gradient arriving over the residual branch, or the encoder-output gradient of the previous layer),
    "relu_mask" (the input gradient through the ReLU)."""
    d, F, V, Le, Ld = model["d_model"], model["d_ff"], model["vocab"], model["enc_layers"], model["dec_layers"]
    out = []

    def linear(N, n_in, n_out, count, fwd="bias", dgrad="add"):
        out.append((N, n_out, n_in, 0, 0, count, fwd))              # y = x W^T + b
        out.append((N, n_in, n_out, 0, 1, count, dgrad))            # dx = dy W
        out.append((n_out, n_in, N, 1, 1, count, "none"))           # dW = dy^T x

    for N, L in ((Ns, Le), (Nt, Ld)):
        linear(N, d, 3 * d, L)                                      # q, k, v
        linear(N, d, d, L, dgrad="none")                            # attention output projection
        linear(N, d, F, L, fwd="bias_relu")                         # feed-forward, first layer
        linear(N, F, d, L, dgrad="relu_mask")                       # feed-forward, second layer
    linear(Nt, d, d, Ld)                                            # cross-attention queries
    linear(Nt, d, d, Ld, dgrad="none")                              # cross-attention output projection
    linear(Ns, d, 2 * d, Ld)                                        # cross-attention keys and values
    linear(Nt, d, V, 1, fwd="none", dgrad="none")                   # vocabulary projection
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="big_accum", choices=sorted(WORKLOAD_DESC))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pipes", type=int, default=1, help="forward/backward passes kept in flight on separate streams")
    ap.add_argument("--group", type=int, default=16, help="sub-batches stacked into one forward/backward pass")
    ap.add_argument("--padded", action="store_true", help="keep the sub-batches' padding rows (default: sentences packed back to back)")
    ap.add_argument("--no-legs", action="store_true", help="skip the per-phase / per-kernel legs (timed region only)")
    ap.add_argument("--leg", default="all", choices=["all", "strict"], help="strict: only the one-by-one order (16 x forward/backward/"
                    "accumulate, four in flight), e.g. under a profiler; prints that leg's record")
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE", help="profiling aid: a launch-form switch of nmt_tuning "
                    "set for the whole run (e.g. gemm_persist=0); none changes a result bit")
    ap.add_argument("--one-stream", action="store_true", help="profiling aid: weight-gradient kernels on the caller's stream, so that a kernel "
                    "trace shows every kernel running alone")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives or sharding); use --gpus 1")

    import numpy as np
    import torch

    import nmt_inputs as I
    import paper_1806_00187_amd as A
    from paper_1806_00187_amd.session import Session, Trainer

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    A.load()
    if args.one_stream:
        A.nmt_tuning("one_stream", 1)
    for item in args.tune:
        name, _, value = item.partition("=")
        A.nmt_tuning(name, int(value))
    model_name, k_micro, desc = WORKLOAD_DESC[args.workload]
    model = I.MODELS[model_name]
    log = lambda *a: print(*a, file=sys.stderr, flush=True)

    t0 = time.time()
    weights = I.init_weights(seed=0, **model)
    batches = I.workload_batches(args.workload, which="random", count=k_micro, n_sentences=50_000)
    shapes = [(b["src"].shape[0], b["src"].shape[1], b["tgt_in"].shape[1]) for b in batches]
    ntoks = [int((b["tgt_out"] != I.PAD).sum()) for b in batches]
    log(f"[bench] inputs ready in {time.time() - t0:.1f}s; sub-batch shapes (B,S,T): {shapes}")
    if args.leg == "strict":
        print(json.dumps({"strict_order": strict_leg(model, weights, batches, ntoks, shapes, args.steps, Session, Trainer, torch, log)}))
        return
    group = max(1, min(args.group, k_micro))
    n_pass = -(-k_micro // group)
    sess = Session(model, weights, max_sentences=max(s[0] for s in shapes), max_len=256, n_pipes=max(1, min(args.pipes, n_pass)))
    dbatches = [sess.to_device(b) for b in batches]
    packed = not args.padded
    src_lens = np.concatenate([(b["src"] != I.PAD).sum(1) for b in batches])
    tgt_lens = np.concatenate([(b["tgt_out"] != I.PAD).sum(1) for b in batches])
    if packed:
        dbatches = sess.pack(batches, size=group)      # the same sentences without the padding rows, still resident in HBM
        for g in dbatches:
            sess._reserve_bytes(A.nmt_workspace_bytes_packed(sess.ctx, g["packed"].shape[0], g["n_src"], g["n_tgt"]))
    elif group > 1:
        dbatches = Session.group(dbatches, group)      # ids of a group's sub-batches back to back, still resident in HBM
        for g in dbatches:
            sess.reserve(g["segs"])
    else:
        for b, s, t in shapes:
            sess.reserve(b, s, t)
    pass_rows = [(sum(b * s for b, s, _ in shapes[i:i + group]), sum(b * t for b, _, t in shapes[i:i + group])) for i in range(0, k_micro, group)]
    if packed:
        pass_rows = [(g["n_src"], g["n_tgt"]) for g in dbatches]
    tr = Trainer(sess, peak_lr=1e-3, warmup=4000, init_scale=128.0)
    if sess.n_pipes > 1:    # several passes in flight: the streams that overlap best, by measurement
        sess.choose_streams(dbatches, loss_scale=16.0, tries=6, log=log)

    # warm-up: also lets the dynamic loss scale settle (an overflowing update is skipped and halves it)
    skipped = 0
    for _ in range(max(args.warmup, 0)):
        _, _, flag = tr.step(dbatches, n_tok=sum(ntoks))
        skipped += flag
    while True:     # make sure the timed region runs full (non-skipped) updates
        _, _, flag = tr.step(dbatches, n_tok=sum(ntoks))
        if not flag:
            break
        skipped += 1
    log(f"[bench] warm-up done, loss scale {tr.scale}, skipped {skipped} overflowing updates")

    stream = torch.cuda.current_stream()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    ev0.record(stream)
    flags = []
    for _ in range(args.steps):
        loss, ntok, flag = tr.step(dbatches, n_tok=sum(ntoks))
        flags.append(flag)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    tokens_per_step = sum(ntoks)
    value = tokens_per_step / (ms_per_step * 1e-3)
    flops_step = model_flops_packed(model, src_lens, tgt_lens) if packed else sum(model_flops(model, *s) for s in shapes)
    achieved_tflops = flops_step / (ms_per_step * 1e-3) / 1e12
    log(f"[bench] {ms_per_step:.2f} ms/update, {value:,.0f} target tok/s, {achieved_tflops:.1f} TFLOP/s, loss/token {loss / ntok:.3f}")

    how = (f"all {k_micro} sub-batches packed into {n_pass} forward+backward pass(es) (no padding rows), accumulate x{n_pass}, overflow check, Adam"
           if packed else f"{k_micro} padded sub-batches in groups of {group} per pass")
    result = {
        "metric": "target tokens/sec/GPU (train step, Transformer-big fp16)" if model_name != "base" else "target tokens/sec/GPU (train step)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "value_is": how,
        "config": {"workload": f"{args.workload}: {desc}; timed as: {how}", "micro_batches_per_update": k_micro,
                   "target_tokens_per_update": tokens_per_step, "padded_shapes_BST": shapes, "loss_scale": tr.scale,
                   "overflow_updates_in_timed_region": int(sum(flags)), "sub_batches_per_pass": group, "passes_in_flight": sess.n_pipes,
                   "rows": "packed (no padding rows)" if packed else "padded", "source_positions_per_update": int(sum(r[0] for r in pass_rows)),
                   "target_positions_per_update": int(sum(r[1] for r in pass_rows)), "wall_ms_per_step": wall * 1e3 / args.steps},
        "roofline": None,
        "whole_update": {"bound": "mfma", "kernel": "every launch of the timed region", "achieved": achieved_tflops,
                         "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s", "frac": achieved_tflops / PEAK_FP16_TFLOPS,
                         "algorithmic_flops_per_update": flops_step},
        "paper_context": {"tokens_per_s_per_gpu": 24400, "hardware": "V100, inside an 8-GPU job incl. all-reduce (Table 1, cumul)"},
    }

    if not args.no_legs:
        result["phases_ms_per_update"] = phase_leg(sess, tr, dbatches, ntoks, torch)
        result["roofline"] = gemm_event_leg(sess, tr, dbatches, ntoks, A, torch, log,
                                            read_profile_traffic() if (args.workload == "big_accum" and packed and group == 16) else None)
        result["roofline"]["by_shape"] = gemm_leg(model, pass_rows, A, torch, log)
        result["hbm_kernels"] = hbm_leg(sess, torch)
        result["fp32_comparison"] = fp32_leg(model, pass_rows, result["roofline"]["ms_per_update"], A, torch, log)
    if result["roofline"] is None:      # --no-legs: only the end-to-end rate is known
        result["roofline"] = dict(result["whole_update"], traffic=None)
    scale = tr.scale
    sess.close()
    del sess, tr, dbatches
    # after the session above is gone: its second stream, while it exists, takes a place on the process's hardware
    # queues, and the four pipes of the one-by-one order then overlap less (134-137 ms instead of 107)
    if not args.no_legs and (packed or group > 1):
        result["strict_order"] = strict_leg(model, weights, batches, ntoks, shapes, args.steps, Session, Trainer, torch, log)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(model, weights, batches[:2], tokens_per_step, scale, log)
    # key order of the printed line: headline, roofline, the one-by-one order, then the other legs
    order = ["strict_order", "phases_ms_per_update", "hbm_kernels", "fp32_comparison", "cpu_baseline"]
    result = {**{k: v for k, v in result.items() if k not in order}, **{k: result[k] for k in order if k in result}}
    print(json.dumps(result))


def _timed(torch, fn, reps):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    st = torch.cuda.current_stream()
    fn()
    torch.cuda.synchronize()
    e0.record(st)
    for _ in range(reps):
        fn()
    e1.record(st)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def strict_leg(model, weights, batches, ntoks, shapes, steps, Session, Trainer, torch, log):
    """The same update in the method's literal order ("Training with Larger Batches"): the 16 padded sub-batches one by
    one (forward + loss, backward, accumulate each; four in flight on separate streams, accumulation chained in
    sub-batch order), then overflow check + Adam.  Timed over the same number of steps as the headline; the time
    of each of the five calls summed over one update comes from a serial (one sub-batch in flight) pass."""
    import paper_1806_00187_amd as A
    sess = Session(model, weights, max_sentences=max(b["src"].shape[0] for b in batches), max_len=256, n_pipes=min(4, len(batches)))
    dbs = [sess.to_device(b) for b in batches]
    for b in batches:
        sess.reserve(b["src"].shape[0], b["src"].shape[1], b["tgt_in"].shape[1])
    tr = Trainer(sess, peak_lr=1e-3, warmup=4000, init_scale=128.0)
    # which hardware queues the runtime has put the four streams on decides how well the pipes overlap (107 to 141 ms
    # measured for the same work): the session tries a few sets of streams on the forward/backward part of an update
    chosen_ms = sess.choose_streams(dbs, loss_scale=32.0, tries=6, log=log)
    # (with several pipes the session keeps each pipe's weight gradients on the pipe's own stream and lets every
    #  product take large tiles as if it had a quarter of the chip: four products run side by side)
    for _ in range(12):                                  # settle the loss scale
        if not tr.step(dbs, n_tok=sum(ntoks))[2]:
            break
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(torch.cuda.current_stream())
    flags = [tr.step(dbs, n_tok=sum(ntoks))[2] for _ in range(steps)]
    e1.record(torch.cuda.current_stream())
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    sess.close()
    # per-call times of the 16-call path (serial, so that the events of one call do not cover another's kernels)
    serial = Session(model, weights, max_sentences=max(b["src"].shape[0] for b in batches), max_len=256)
    sdbs = [serial.to_device(b) for b in batches]
    str_ = Trainer(serial, peak_lr=1e-3, warmup=4000, init_scale=tr.scale)
    str_.step(sdbs, n_tok=sum(ntoks))
    phases = phase_leg(serial, str_, sdbs, ntoks, torch)
    serial.close()
    flops = sum(model_flops(model, *s_) for s_ in shapes)
    tflops = flops / (ms * 1e-3) / 1e12
    log(f"[bench] strict order (16 padded sub-batches one by one, 4 in flight): {ms:.2f} ms/update, {tflops:.1f} TFLOP/s, loss scale {tr.scale}")
    return {"what": "16 x (forward+loss, backward, accumulate) over the padded sub-batches one by one (4 in flight), then overflow check + Adam",
            "ms_per_step": ms, "value": sum(ntoks) / (ms * 1e-3), "unit": "tokens/s", "steps": steps, "loss_scale": tr.scale,
            "overflow_updates": int(sum(flags)), "achieved_tflops": tflops, "frac_of_fp16_peak": tflops / PEAK_FP16_TFLOPS,
            "streams": "the fastest of 6 sets of 4 streams on the forward/backward part of one update (the runtime's placement of streams "
                       "on hardware queues decides how well the pipes overlap: 107-141 ms measured for the same work)",
            "forward_backward_ms_on_the_chosen_streams": chosen_ms,
            "phases_ms_per_update_serial": phases}


def phase_leg(sess, tr, dbatches, ntoks, torch):
    """Time of each C-ABI call summed over one update (HIP events on the launch stream)."""
    st = torch.cuda.current_stream()
    names = ["forward_loss", "backward", "accumulate", "check_overflow", "adam_step"]
    acc = dict.fromkeys(names, 0.0)
    events = []

    def mark():
        e = torch.cuda.Event(enable_timing=True)
        e.record(st)
        events.append(e)

    torch.cuda.synchronize()
    for j, db in enumerate(dbatches):
        mark(); sess.forward_loss(db, tr.scale, tr.t, j)
        mark(); sess.backward()
        mark(); sess.accumulate(j == 0)
    mark(); sess.check_overflow(1.0 / (tr.scale * sum(ntoks)))
    mark(); sess.adam_step(tr.lr(), tr.t)
    mark()
    torch.cuda.synchronize()
    seq = ["forward_loss", "backward", "accumulate"] * len(dbatches) + ["check_overflow", "adam_step"]
    for i, name in enumerate(seq):
        acc[name] += events[i].elapsed_time(events[i + 1])
    return acc


PROFILE_TRAFFIC = os.path.join(ROOT, "profiles", "bench_big_accum_gemm_hbm_traffic.txt")


def read_profile_traffic():
    """HBM-side bytes per GEMM product of the default workload from the committed rocprofv3 --pmc summary (FETCH_SIZE /
    WRITE_SIZE calibrated against kernels of known size): its line "per-product-bytes: moved=<n> algorithmic=<n>"."""
    try:
        import re
        m = re.search(r"per-product-bytes:\s*moved=([0-9.e+]+)\s+algorithmic=([0-9.e+]+)", open(PROFILE_TRAFFIC).read())
        return {"bytes_per_launch": float(m.group(1)), "algorithmic_bytes_per_launch": float(m.group(2)),
                "source": "profiles/bench_big_accum_gemm_hbm_traffic.txt"}
    except Exception:
        return None


def gemm_event_leg(sess, tr, dbatches, ntoks, A, torch, log, traffic, updates=3):
    """The dominant kernel measured in the step itself: the timed update is run `updates` more times with a pair of
    HIP events around every GEMM product on the stream it is launched on (weight-gradient products on the caller's
    stream as well, so that every duration is that of a product running alone); algorithmic FLOPs 2 M N K of all
    products / the sum of their durations."""
    A.nmt_tuning("one_stream", 1)
    A.nmt_tuning("gemm_timing", 1)
    try:
        A.nmt_gemm_timing()
        for _ in range(updates):
            for j, db in enumerate(dbatches):
                sess.forward_loss(db, tr.scale, tr.t, j)
                sess.backward()
                sess.accumulate(j == 0)
        ms, n, flops = A.nmt_gemm_timing()
    finally:
        A.nmt_tuning("defaults")
    achieved = flops / ms / 1e9
    log(f"[bench] GEMM products in the step (HIP events, one stream): {achieved:.1f} TFLOP/s over {n // updates} products per update, "
        f"{ms / updates:.2f} ms per update")
    return {"bound": "mfma", "kernel": "gemm_kernel / gemm_persistent_kernel (every GEMM product of the timed update, incl. split-k reduction)",
            "achieved": achieved, "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP16_TFLOPS, "traffic": traffic,
            "how": f"HIP events around every product on its launch stream, {updates} updates of the timed step with the backward pass on one stream",
            "launches_per_update": n // updates, "avg_launch_us": ms * 1e3 / n, "ms_per_update": ms / updates,
            "algorithmic_flops_per_launch": flops / n}


def gemm_leg(model, pass_rows, A, torch, log):
    """Every distinct GEMM shape of the update timed alone through nmt_op_gemm on random operands (HIP events, 10
    launches each): which shapes are fast and which are slow."""
    agg = {}
    for s in pass_rows:
        for (M, N, K, a_t, b_t, count, epi) in gemm_shapes(model, *s):
            key = (M, N, K, a_t, b_t, epi)
            agg[key] = agg.get(key, 0) + count
    tot_flops = tot_ms = 0.0
    n_launch = 0
    worst, best = None, None
    per_kind = {}
    cache = {}
    partial = torch.empty(16 << 20, dtype=torch.float32, device="cuda")   # the step's partial-sum scratch size
    warm = torch.randn(8192, 8192, device="cuda", dtype=torch.float16)   # the first shape is not timed on a chip at rest
    _timed(torch, lambda: A.nmt_op_gemm(warm, 0, 8192, warm, 0, 8192, warm.new_empty(8192, 8192), 8192, 8192, 8192, 8192), 20)
    del warm
    for (M, N, K, a_t, b_t, epi), count in agg.items():
        rows_a, cols_a = (K, M) if a_t else (M, K)
        rows_b, cols_b = (K, N) if b_t else (N, K)
        bufs = cache.get((rows_a, cols_a, rows_b, cols_b, M, N))
        if bufs is None:
            bufs = (torch.randn(rows_a, cols_a, device="cuda", dtype=torch.float16),
                    torch.randn(rows_b, cols_b, device="cuda", dtype=torch.float16) * 0.03,
                    torch.empty(M, N, device="cuda", dtype=torch.float16))
            cache = {(rows_a, cols_a, rows_b, cols_b, M, N): bufs}
        a, b, c = bufs
        if a_t and b_t:   # weight gradient: as in the step, the library may cut the contraction into pieces (fp32 partial sums)
            ms = _timed(torch, lambda: A.nmt_op_gemm_splitk(a, a_t, cols_a, b, b_t, cols_b, c, N, M, N, K, partial, 0), 10)
        else:             # with the epilogue the step uses for this product
            bias = torch.zeros(N, device="cuda", dtype=torch.float16) if epi.startswith("bias") else None
            other = torch.randn(M, N, device="cuda", dtype=torch.float16) if epi in ("add", "relu_mask") else None
            ms = _timed(torch, lambda: A.nmt_op_gemm(a, a_t, cols_a, b, b_t, cols_b, c, N, M, N, K, bias, epi == "bias_relu", None,
                                                      other if epi == "add" else None, other if epi == "relu_mask" else None), 10)
            del other
        fl = 2.0 * M * N * K
        tot_flops += fl * count
        tot_ms += ms * count
        n_launch += count
        kind = {(0, 0): "forward", (0, 1): "dgrad", (1, 1): "wgrad"}[(a_t, b_t)]
        pk = per_kind.setdefault(kind, [0.0, 0.0])
        pk[0] += fl * count
        pk[1] += ms * count
        rate = fl / ms / 1e9
        if worst is None or rate < worst[0]:
            worst = (rate, [M, N, K, kind])
        if best is None or rate > best[0]:
            best = (rate, [M, N, K, kind])
    achieved = tot_flops / tot_ms / 1e9
    log(f"[bench] GEMM leg: {achieved:.1f} TFLOP/s over {n_launch} launches, {tot_ms:.2f} ms per update; worst {worst}, best {best}")
    return {"what": "each distinct shape timed alone on random operands", "achieved": achieved, "frac": achieved / PEAK_FP16_TFLOPS,
            "launches_per_update": n_launch, "avg_launch_us": tot_ms * 1e3 / n_launch, "ms_per_update": tot_ms,
            "by_kind_tflops": {k: v[0] / v[1] / 1e9 for k, v in per_kind.items()}, "worst_tflops": worst, "best_tflops": best}


PEAK_FP32_MATRIX_TFLOPS = 157.3   # MI355X dense fp32 matrix peak (published)


def fp32_leg(model, pass_rows, fp16_gemm_ms, A, torch, log):
    """What the paper measures first ("Half-Precision Training"; Table 1, "Our reimplementation" against "16-bit"): the
    same work in fp32.  Every GEMM shape of the update through the benchmark-only fp32 product (fp32 matrix
    instructions, fp32 operands and result), timed alone; set against the fp16 products of the timed step."""
    agg = {}
    for s_ in pass_rows:
        for (M, N, K, a_t, b_t, count, _) in gemm_shapes(model, *s_):
            agg[(M, N, K, a_t, b_t)] = agg.get((M, N, K, a_t, b_t), 0) + count
    tot_ms = tot_fl = 0.0
    for (M, N, K, a_t, b_t), count in agg.items():
        ra, ca = (K, M) if a_t else (M, K)
        rb, cb = (K, N) if b_t else (N, K)
        ca4, cb4 = (ca + 3) // 4 * 4, (cb + 3) // 4 * 4
        a = torch.randn(ra, ca4, device="cuda", dtype=torch.float32)
        b = torch.randn(rb, cb4, device="cuda", dtype=torch.float32) * 0.03
        # a weight gradient (small result, contraction over all positions) is cut along k as in the fp16 step
        tiles = -(-M // 128) * -(-N // 128)
        splits = max(1, min(64, 1024 // tiles, K // 512)) if (a_t and b_t) else 1
        c = torch.empty(splits * M, N, device="cuda", dtype=torch.float32)
        ms = _timed(torch, lambda: A.nmt_op_gemm_f32(a, a_t, ca4, b, b_t, cb4, c, N, M, N, K, splits), 2)
        tot_ms += ms * count
        tot_fl += 2.0 * M * N * K * count
        del a, b, c
    tflops = tot_fl / tot_ms / 1e9
    log(f"[bench] fp32 comparison: the update's GEMMs in fp32 take {tot_ms:.1f} ms ({tflops:.1f} TFLOP/s) against {fp16_gemm_ms:.1f} ms in fp16: "
        f"{tot_ms / fp16_gemm_ms:.1f}x")
    return {"what": "every GEMM product of the update with fp32 operands on the fp32 matrix instructions (benchmark-only kernel), each shape timed alone",
            "gemm_ms_per_update_fp32": tot_ms, "achieved": tflops, "peak": PEAK_FP32_MATRIX_TFLOPS, "unit": "TFLOP/s",
            "frac": tflops / PEAK_FP32_MATRIX_TFLOPS, "gemm_ms_per_update_fp16": fp16_gemm_ms,
            "fp16_speedup_on_the_gemms": tot_ms / fp16_gemm_ms,
            "paper": "2.9x shorter training with 16-bit at equal settings on 8 x V100 (Table 1, 'Our reimplementation' vs '16-bit')"}


def hbm_leg(sess, torch):
    """Achieved GB/s of the HBM-bound update kernels: algorithmic bytes per parameter
    (accumulate 2+4+4, overflow check 4 read, Adam 16 read + 14 written) x P / duration."""
    P = sess.P
    out = {}
    for name, fn, bpp in (("accumulate", lambda: sess.accumulate(False), 10), ("check_overflow", lambda: sess.check_overflow(1.0), 4),
                          ("adam_step", None, 30)):
        if fn is None:
            sess.flag.zero_()
            fn = lambda: sess.adam_step(0.0, 1)          # lr 0: full traffic, weights unchanged
        ms = _timed(torch, fn, 5)
        gbs = bpp * P / (ms * 1e-3) / 1e9
        out[name] = {"ms": ms, "bytes_per_param": bpp, "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    return out


def cpu_baseline(model, weights, sample, tokens_per_update, loss_scale, log):
    """The fp64 numpy oracle timed on the host cores: forward + backward + fp16 rounding + accumulate on two whole
    sub-batches of the update, and overflow check + Adam over all parameters once; scaled to a whole update by
    target tokens."""
    import numpy as np
    import nmt_inputs as I
    from oracle import nmt_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    cfg = O.Config(model["enc_layers"], model["dec_layers"], model["d_model"], model["n_heads"], model["d_ff"], model["vocab"],
                   dropout=model["dropout"])
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    acc, ntok, t_micro = None, 0, 0.0
    for j, mb in enumerate(sample):
        t0 = time.perf_counter()
        loss, n, cache = O.forward_loss(P16, cfg, mb["src"], mb["tgt_in"], mb["tgt_out"], step=1, micro=j)
        g = O.to_fp16_storage(O.backward(P16, cfg, cache, loss_scale))
        acc = O.accumulate(acc, g, j == 0)
        t_micro += time.perf_counter() - t0
        ntok += n
        del cache, g
    t0 = time.perf_counter()
    flag, un = O.check_overflow(acc, 1.0 / (loss_scale * ntok))
    m = {k: np.zeros_like(v) for k, v in P16.items()}
    v = {k: np.zeros_like(val) for k, val in P16.items()}
    O.adam_step(P16, m, v, un, 1e-3, 0.9, 0.98, 1e-8, 1, flag)
    t_update = time.perf_counter() - t0
    total = t_micro / ntok * tokens_per_update + t_update
    val = tokens_per_update / total
    shapes = [(b["src"].shape[0], b["src"].shape[1], b["tgt_in"].shape[1]) for b in sample]
    log(f"[bench] oracle: {t_micro:.1f}s for {ntok} tokens in {len(sample)} sub-batches, {t_update:.1f}s for overflow check + Adam (flag {flag}); "
        f"{val:.1f} tok/s on {cores} threads")
    return {"value": val, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"fp64 numpy oracle: forward+backward+fp16 rounding+accumulate on {len(sample)} whole sub-batches of the update, (B,S,T)={shapes}, "
                      f"{ntok} target tokens ({t_micro:.1f} s), overflow check + Adam over all parameters once ({t_update:.1f} s), scaled to one update "
                      f"of {tokens_per_update} tokens"}


if __name__ == "__main__":
    main()
