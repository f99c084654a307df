#!/usr/bin/env python3
"""Benchmark of the DPPO loss hot path (forward + backward over the full vocabulary) on ONE
MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--in-place]
                  [--diagnostics] [--mask-rule dppo|ratio_clip|none] [--eps-low E] [--eps-high E] [--ratio-cap C]

A step is one pass of the whole path (log-softmax statistics, gathers, divergence, mask,
loss, gradient over all V logits) over one synthetic batch that is already resident in HBM.
Prints ONE JSON line.  The default workload is the Qwen3-vocabulary Binary-TV configuration
(T = 32768 tokens, V = 151936), the one the headline metric is quoted on.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E peak
DEFAULT_WORKLOAD = "c3_qwen3_binary_tv"
DOMINANT_KERNEL = {"resident": "dppo_resident_kernel", "resident_long": "dppo_resident_long_kernel", "resident_multi": "dppo_resident_multi_kernel",
                   "streaming": "dppo_streaming_kernel",
                   "fullvocab": "dppo_fullvocab_kernel", "fullvocab_resident": "dppo_fullvocab_resident_kernel"}


def kernel_source_hash(path: str) -> str:
    """Hash of the device code behind one kernel path (its kernel file and the shared device
    helpers): stored HBM-traffic counters hold only for it."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2602_04879_amd", "csrc")
    files = ["dppo_common.hpp", f"dppo_{path}.hip"] + (["dppo_resident_parts.hpp"] if path.startswith("resident") else [])
    for fn in files:
        h.update(open(os.path.join(src, fn), "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(workload: str, path: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None when there is
    none for this workload / kernel path or the kernels have changed since it was taken."""
    fn = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(fn):
        return None
    try:
        rec = json.load(open(fn)).get(f"{workload}:{path}")
    except Exception:
        return None
    if not rec or rec.get("kernel_source_hash") != kernel_source_hash(path):
        return None
    return rec.get("bytes_per_launch")


def algorithmic_bytes_per_token(V: int, K: int, full: bool = False, backward: bool = True) -> int:
    """What the method itself must move per token, forward + backward: the bf16 logits row read
    once (and, for the exact full-vocabulary variants, the rollout policy's bf16 row read once),
    the bf16 gradient row written once, and the per-token side inputs/outputs."""
    side_in = 4 + 4 + 4 + 8 * K          # sampled id, mu log-prob, advantage, top-K ids + log-probs
    side_out = 4 + 4 + 1                 # divergence, per-token loss, mask
    return 2 * V + (2 * V if full else 0) + (2 * V if backward else 0) + side_in + side_out


def host_threads() -> int:
    """Hardware threads this process may use: its CPU affinity, capped by the share the
    environment grants (OMP_NUM_THREADS)."""
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    try:
        n = min(n, max(1, int(os.environ.get("OMP_NUM_THREADS", n))))
    except ValueError:
        pass
    return max(1, n)


def _oracle_rows(batch, sl, backward):
    """Run the oracle, as it stands, on one block of rows (host arrays made outside the timing)."""
    from oracle import dppo_oracle as O
    V = batch["V"]
    z = batch["logits"][sl, :V].float().cpu().numpy()
    ids = batch["sampled_ids"][sl].cpu().numpy()
    lmu = batch["mu_logp"][sl].cpu().numpy()
    adv = batch["advantages"][sl].cpu().numpy()
    tk_i = batch["mu_topk_ids"][sl].cpu().numpy() if batch["mu_topk_ids"] is not None else None
    tk_l = batch["mu_topk_logp"][sl].cpu().numpy() if batch["mu_topk_logp"] is not None else None
    y = batch["mu_logits"][sl, :V].float().cpu().numpy() if batch.get("mu_logits") is not None else None
    return lambda: O.dppo_loss(z, ids, lmu, adv, batch["delta"], batch["variant"], batch["loss_scale"], tk_i, tk_l,
                               want_grad=backward, mu_logits=y)


def cpu_baseline(batch, budget_s: float, chunk_rows: int = 64, backward: bool = True) -> dict:
    """Time the float64 oracle, as it stands, on leading rows of the same batch, twice: on one
    thread, and on all hardware threads (blocks of rows handed to a thread pool; numpy releases
    the interpreter lock inside its array operations).  Each leg spends about budget_s / 2 seconds
    of wall time.  `value` / `cores` are the all-threads leg."""
    from concurrent.futures import ThreadPoolExecutor
    T = batch["T"]
    nthreads = host_threads()
    kind = "fwd+bwd" if backward else "fwd"
    # leg 1: one thread
    done, wall = 0, 0.0
    while done < T and wall < budget_s / 2:
        sl = slice(done, min(T, done + chunk_rows))
        fn = _oracle_rows(batch, sl, backward)
        t0 = time.perf_counter()
        fn()
        wall += time.perf_counter() - t0
        done += sl.stop - sl.start
    one = {"value": done / wall, "rows": done, "seconds": wall}
    # leg 2: all threads, rounds of one block per thread
    done2, wall2, cpu2 = 0, 0.0, 0.0
    start = done
    with ThreadPoolExecutor(max_workers=nthreads) as ex:
        while wall2 < budget_s / 2:
            blocks = []
            for _ in range(nthreads):
                r0 = (start + done2 + len(blocks) * chunk_rows) % max(T - chunk_rows, 1)
                blocks.append(_oracle_rows(batch, slice(r0, min(T, r0 + chunk_rows)), backward))
            t0, c0 = time.perf_counter(), time.process_time()
            list(ex.map(lambda f: f(), blocks))
            wall2 += time.perf_counter() - t0
            cpu2 += time.process_time() - c0
            done2 += sum(min(T, chunk_rows) for _ in blocks)
    return {"value": done2 / wall2, "unit": "tokens/s", "cores": nthreads, "kind": "oracle",
            "sample": f"{done2} rows of the same batch (blocks of {chunk_rows} rows, wrapping around) over {nthreads} threads, {kind}, float64 numpy, "
                      f"{wall2:.1f} s wall, {cpu2:.1f} s of CPU time; one thread: first {one['rows']} rows in {one['seconds']:.1f} s",
            "one_thread": {"value": one["value"], "unit": "tokens/s", "cores": 1},
            "host_threads": nthreads, "nproc": os.cpu_count()}


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix-core peak


def bench_lmhead(args, w, dev) -> int:
    """The path from the final hidden states: one step = logits chunk by chunk on the matrix cores,
    the loss kernel in place on each chunk, and the gradients of the hidden states and of the
    lm_head weight."""
    import torch
    from paper_2602_04879_amd import binding as B
    from paper_2602_04879_amd import workloads as W
    batch = W.make_lmhead_batch(w, w.d_model, dev, rows_per_step=2048)
    T, V, d = batch["T"], batch["V"], batch["d"]
    out = B.alloc_outputs(T, dev)
    fwd = args.forward_only
    flags = B.FLAG_FORCE_STREAMING if args.force_streaming else 0
    grad_hidden = None if fwd else torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    grad_weight = None if fwd else torch.empty((V, d), dtype=torch.float32, device=dev)
    fused = fwd and not args.force_streaming
    ws_bytes = B.lmhead_fwd_workspace_bytes(T, V, batch["K"], args.chunk_rows) if fused else B.lmhead_workspace_bytes(T, V, args.chunk_rows)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        return B.run_lmhead(batch, backward=not fwd, chunk_rows=args.chunk_rows, out=out, grad_hidden=grad_hidden, grad_weight=grad_weight,
                            workspace=ws, stream=stream, flags=flags)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / args.steps
    # What the matrix cores sustain under the board's power limit: a loop of nothing but products
    # on every compute unit, both instruction shapes, the last of four ~15 ms launches each.
    ceilings = {}
    probe_out = torch.empty(4096 * 256, dtype=torch.float32, device=dev)
    for shape, key in ((16, "mfma_16x16x32_TFLOPs"), (32, "mfma_32x32x16_TFLOPs")):
        for _ in range(4):
            ev0.record(stream)
            fl = B.probe_mfma(shape, 30000 if shape == 16 else 60000, probe_out, stream=stream)
            ev1.record(stream)
            torch.cuda.synchronize()
        ceilings[key] = fl / (ev0.elapsed_time(ev1) * 1e-3) / 1e12
    # the three products (logits, gradient of the hidden states, gradient of the weight): 2 T V d flops each;
    # forward only: the first one
    flops = (2.0 if fwd else 6.0) * T * V * d
    achieved = flops / (ms * 1e-3) / 1e12
    chunk = args.chunk_rows if args.chunk_rows > 0 else 8192
    rec = {
        "metric": "dppo_lmhead_loss_fwd_tokens_per_s" if fwd else "dppo_lmhead_loss_fwd_bwd_tokens_per_s", "value": T / (ms * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "V": V, "d": d, "K": batch["K"], "variant": int(batch["variant"]),
                   "delta": batch["delta"], "chunk_rows": chunk, "kernel_path": B.last_path(),
                   "outputs": "loss, per-token" if fwd else "loss, per-token, grad_hidden bf16, grad_weight fp32",
                   "workspace_bytes": ws_bytes, "logits_bytes_resident": 0 if fused else min(chunk, T) * V * 2,
                   "logits_bytes_if_materialised": T * V * 2},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "kernel": "dppo_gemm_nt_kernel",
                     "algorithmic_flops_per_step": flops, "ceilings": ceilings,
                     "frac_of_product_only_loop": achieved / ceilings["mfma_16x16x32_TFLOPs"]},
        "loss": float(out["loss"].item()), "masked_tokens": int((out["mask"] == 0).sum().item()),
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline_lmhead(batch, args.cpu_seconds, backward=not fwd)
    print(json.dumps(rec), flush=True)
    return 0


def cpu_baseline_lmhead(batch, budget_s: float, chunk_rows: int = 16, backward: bool = True) -> dict:
    """Time the float64 oracle of the hidden-state path on leading rows of the same batch."""
    from oracle import dppo_oracle as O
    T = batch["T"]
    Wd = batch["weight"].float().cpu().numpy()
    done, wall, cpu = 0, 0.0, 0.0
    while done < T and wall < budget_s:
        sl = slice(done, min(T, done + chunk_rows))
        h = batch["hidden"][sl].float().cpu().numpy()
        tk_i = batch["mu_topk_ids"][sl].cpu().numpy() if batch["mu_topk_ids"] is not None else None
        tk_l = batch["mu_topk_logp"][sl].cpu().numpy() if batch["mu_topk_logp"] is not None else None
        t0, c0 = time.perf_counter(), time.process_time()
        O.lmhead_dppo_loss(h, Wd, batch["sampled_ids"][sl].cpu().numpy(), batch["mu_logp"][sl].cpu().numpy(),
                           batch["advantages"][sl].cpu().numpy(), batch["delta"], batch["variant"], batch["loss_scale"], tk_i, tk_l,
                           want_grad=backward)
        wall += time.perf_counter() - t0
        cpu += time.process_time() - c0
        done += sl.stop - sl.start
    return {"value": done / wall, "unit": "tokens/s", "cores": max(1, round(cpu / wall)), "kind": "oracle",
            "sample": f"first {done} of {T} rows of the same batch, logits + {'fwd+bwd + hidden-state and weight gradients' if backward else 'fwd'}, float64 numpy, {wall:.1f} s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--diagnostics", action="store_true", help="also write the per-token diagnostics [T, 8] (entropy, |pi - mu|, covered mass, ...)")
    ap.add_argument("--mask-rule", choices=["dppo", "ratio_clip", "none"], default="dppo",
                    help="dppo: divergence mask (default); ratio_clip: PPO / GRPO(-ClipHigher) with --eps-low/--eps-high; none: PG-IS, CISPO / PG-TIS")
    ap.add_argument("--eps-low", type=float, default=0.2)
    ap.add_argument("--eps-high", type=float, default=0.28)
    ap.add_argument("--ratio-cap", type=float, default=0.0, help="C of the unified gradient form (0: no cap)")
    ap.add_argument("--relax-alpha", type=float, default=0.0, help="with --mask-rule ratio_clip: rollout probability below which the clip is relaxed (Sec. 6)")
    ap.add_argument("--relax-sides", type=int, default=3, help="1: upper threshold, 2: lower, 3: both")
    ap.add_argument("--anchor", action="store_true", help="anchor the mask to a recomputed policy (mu_logp plus N(0, 0.3^2) noise): MiniRL with --mask-rule ratio_clip, the decoupled DPPO otherwise")
    ap.add_argument("--in-place", action="store_true", help="write the gradient over the logits (the boundary allows it); the logits are restored, untimed, before every step")
    ap.add_argument("--force-streaming", action="store_true", help="time the general two-pass kernel")
    ap.add_argument("--static-rows", action="store_true", help="rows fixed by the workgroup index instead of handed out at run time")
    ap.add_argument("--ld", type=int, default=0, help="row pitch of logits / gradient in elements (0: V)")
    ap.add_argument("--forward-only", action="store_true", help="time dppo_loss_fwd (no gradient) instead of forward+backward")
    ap.add_argument("--chunk-rows", type=int, default=0, help="tokens per chunk of the hidden-state workloads (0: library default)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures ONE GPU: the path is data-parallel over tokens with no exchange "
              "but one scalar; run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2602_04879_amd import binding as B
    from paper_2602_04879_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = W.WORKLOADS[args.workload]
    if w.d_model:
        return bench_lmhead(args, w, dev)
    batch = W.make_batch(w, dev, rows_per_step=2048, ld=(args.ld or None))
    T, V, K = batch["T"], batch["V"], batch["K"]
    chunk = w.chunk_rows or T
    flags = (B.FLAG_FORCE_STREAMING if args.force_streaming else 0) | (B.FLAG_STATIC_ROWS if args.static_rows else 0)

    # caller-side buffers, allocated once: gradient (separate from the logits so that every
    # step sees the same input), per-token outputs, one loss scalar per T-chunk
    in_place = args.in_place and not args.forward_only
    pristine = batch["logits"].clone() if in_place else None
    grad = batch["logits"] if in_place else torch.empty_like(batch["logits"])
    out = B.alloc_outputs(T, dev, want_diagnostics=args.diagnostics)
    rule = {"mask_rule": {"dppo": B.MASK_DIVERGENCE, "ratio_clip": B.MASK_RATIO_CLIP, "none": B.MASK_NONE}[args.mask_rule],
            "eps_low": args.eps_low, "eps_high": args.eps_high, "ratio_cap": args.ratio_cap,
            "relax_alpha": args.relax_alpha, "relax_sides": args.relax_sides if args.relax_alpha > 0 else 0}
    # A small working set would otherwise be served by the 256 MB Infinity Cache step after step:
    # consecutive steps then rotate among enough copies of (logits, gradient) to make 4 GiB.
    per_step_bytes = 2 * batch["logits"].numel() * 2
    nrot = 1 if (in_place or batch.get("mu_logits") is not None) else max(1, min(128, -(-(4 << 30) // per_step_bytes)))
    copies = [(batch["logits"], grad)] + [(batch["logits"].clone(), torch.empty_like(grad)) for _ in range(nrot - 1)]

    anchor = None
    if args.anchor:
        gen = torch.Generator(device=dev).manual_seed(w.seed + 77)
        anchor = torch.minimum(batch["mu_logp"] + 0.3 * torch.randn(T, generator=gen, device=dev), torch.zeros_like(batch["mu_logp"]))

    def make_calls(logits_c, grad_c):
        cs = []
        for c0 in range(0, T, chunk):
            c1 = min(T, c0 + chunk)
            o = dict(out)
            o["loss"] = torch.empty(1, dtype=torch.float32, device=dev)
            for k in ("loss_tok", "divergence", "mask") + (("diagnostics",) if args.diagnostics else ()):
                o[k] = out[k][c0:c1]
            sl = slice(c0, c1)
            a = B.make_args(logits_c[sl], batch["sampled_ids"][sl], batch["mu_logp"][sl], batch["advantages"][sl],
                            batch["delta"], batch["variant"], batch["loss_scale"], o,
                            batch["mu_topk_ids"][sl] if K else None, batch["mu_topk_logp"][sl] if K else None,
                            V=V, flags=flags, grad_logits=grad_c[sl],
                            mu_logits=batch["mu_logits"][sl] if batch.get("mu_logits") is not None else None,
                            anchor_logp=anchor[sl] if anchor is not None else None, **rule)
            a.ld = batch["ld"]
            cs.append((a, o))
        return cs
    call_sets = [make_calls(lc, gc) for lc, gc in copies]
    calls = call_sets[0]

    stream = torch.cuda.current_stream()

    run = B.dppo_loss_fwd if args.forward_only else B.dppo_loss_fwd_bwd
    step_no = [0]

    def step():
        for a, _ in call_sets[step_no[0] % nrot]:
            run(a, stream)
        step_no[0] += 1

    # One HIP event pair per step, on the stream the kernels are launched on; the step time reported
    # is the MEDIAN over the steps.  In place, every step overwrites its input, so the logits are
    # restored (untimed) before each one.
    def timed(n):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for e0, e1 in evs:
            if in_place:
                batch["logits"].copy_(pristine)
            e0.record(stream)
            step()
            e1.record(stream)
        torch.cuda.synchronize()
        return sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    timed(args.warmup)
    torch.cuda.synchronize()
    t_wall = time.perf_counter()
    times = timed(args.steps)
    t_wall = time.perf_counter() - t_wall
    ms_per_step = times[len(times) // 2] if len(times) % 2 else 0.5 * (times[len(times) // 2 - 1] + times[len(times) // 2])
    ms_mean = sum(times) / len(times)
    if in_place:
        batch["logits"].copy_(pristine)
    path = B.last_path()

    # the device's streaming ceilings on THESE buffers (the rate depends on the footprint), measured
    # with the library's plain copy kernels (grid-stride, and one workgroup per row like the loss
    # kernels) and its read kernel
    ceilings = {}
    nbytes = batch["logits"].numel() * 2
    if nbytes % 16 == 0 and nbytes >= (1 << 28):
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        flat = lambda t: t.view(-1).view(torch.uint8)
        # (source, destination) pairs: the same rotating copies the timed steps used
        pairs = [(pristine, grad)] if in_place else copies
        probes = [("copy", lambda s_, d_: B.probe_copy(flat(d_), flat(s_), stream), 2 * nbytes),
                  ("read", lambda s_, d_: B.probe_read(flat(s_), sink, stream), nbytes)]
        if (V * 2) % 16 == 0 and (batch["ld"] * 2) % 16 == 0:
            probes.append(("copy_rows", lambda s_, d_: B.probe_copy_rows(d_[:, :V], s_[:, :V], stream), 2 * T * V * 2))
            if V * 2 <= 512 * 38 * 16:
                # the loss kernel's own memory pattern with none of its arithmetic
                probes.append(("copy_resident", lambda s_, d_: B.probe_copy_resident(d_[:, :V], s_[:, :V], stream), 2 * T * V * 2))
        for name, fn, moved in probes:
            fn(*pairs[0])
            torch.cuda.synchronize()
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = max(5, int(2e10 // moved))      # about 20 GB moved per probe, whatever the buffers' size
            c0.record(stream)
            for i in range(reps):
                fn(*pairs[i % len(pairs)])
            c1.record(stream)
            torch.cuda.synchronize()
            ceilings[name + "_GBs"] = moved / (c0.elapsed_time(c1) / reps * 1e-3) / 1e9

    launches = len(calls)
    alg_bytes_launch = algorithmic_bytes_per_token(V, K, batch.get("mu_logits") is not None, not args.forward_only) * (T // launches)
    # a launch of the dominant kernel plus its share of the step's small change (the ~5 us loss
    # reduction and the gaps between launches): a little MORE than the kernel's own duration
    step_ms_per_launch = ms_per_step / launches
    achieved = alg_bytes_launch / (step_ms_per_launch * 1e-3) / 1e9
    loss = sum(float(o["loss"].item()) for _, o in calls)

    rec = {
        "metric": "dppo_loss_fwd_tokens_per_s" if args.forward_only else "dppo_loss_fwd_bwd_tokens_per_s",
        "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_stat": "median of one HIP event pair per step", "ms_per_step_mean": ms_mean,
        "ms_per_step_min": times[0], "ms_per_step_max": times[-1], "timed_region_wall_s": t_wall,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "T": T, "V": V, "K": K, "variant": int(batch["variant"]),
                   "recipe": {"logit_std": w.logit_std, "zipf_s": w.zipf_s, "rollout_noise_std": w.noise_std,
                              "drift_frac": w.drift_frac, "drift_std": w.drift_std, "advantages": w.adv, "group": w.group,
                              "seed": w.seed,
                              "note": "drift: this share of the tokens has the trainer's sampled-token logit moved by "
                                      "N(0, drift_std^2) after the rollout, so that a few tokens are masked; not part of "
                                      "the configuration string this workload stands for, byte-neutral"},
                   "delta": batch["delta"], "logits_dtype": "bf16", "ld": batch["ld"], "launches_per_step": launches,
                   "kernel_path": path, "buffer_sets": nrot, "rows": "fixed by workgroup index" if args.static_rows else "library default", "mask_rule": args.mask_rule, "mask_anchor": "recomputed policy (synthetic)" if args.anchor else "rollout policy", "ratio_cap": args.ratio_cap, "diagnostics": args.diagnostics, "grad": "none (forward only)" if args.forward_only else "in place over the logits" if in_place else "separate buffer"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None if (args.forward_only or in_place or args.diagnostics or args.anchor) else stored_traffic(args.workload, path),
                     "kernel": DOMINANT_KERNEL.get(path, path), "algorithmic_bytes_per_launch": alg_bytes_launch,
                     "step_ms_per_launch": step_ms_per_launch, "device_ceilings": ceilings,
                     "frac_of_copy_ceiling": (achieved / ceilings["copy_GBs"]) if ceilings else None,
                     "frac_of_resident_copy": (achieved / ceilings["copy_resident_GBs"]) if ceilings.get("copy_resident_GBs") else None},
        "loss": loss, "masked_tokens": int((out["mask"] == 0).sum().item()),
    }
    if rec["roofline"]["traffic"]:
        # what the counters say went over the HBM interface per second of this run's kernel time
        rec["roofline"]["traffic_GBs"] = rec["roofline"]["traffic"] / (step_ms_per_launch * 1e-3) / 1e9
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(batch, args.cpu_seconds, backward=not args.forward_only)
    print(json.dumps(rec), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
