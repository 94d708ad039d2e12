"""Benchmark of the whole policy step (prefill + K-1 decode steps + selection) on one MI355X.

Prints ONE JSON line: actions/sec of the policy step on the 7B-shaped workload C3 (bf16, batch 64,
256 patches + 34 instruction tokens, 7 greedy action tokens), with the roofline of the dominant
kernel (the prefill gate/up GEMM, timed with HIP events on the launch stream) and the fp64 oracle
timed on the host cores for a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def model_numbers(wl, cu_seq):
    s = wl.shape
    d, f, L = s.d_model, s.d_ffn, s.n_layers
    S = np.diff(cu_seq).astype(np.int64)
    T = int(S.sum())
    P = s.n_matrix_params
    es = 2 if s.dtype == "bf16" else 4
    prefill_flops = 2 * P * T + L * int((2 * S * S * d).sum()) + 2 * s.n_action_bins * d * wl.batch
    kv_pos_bytes = 2 * d * L * es                      # K and V of one position, all layers
    decode_bytes = []
    for k in range(1, wl.n_tokens):                    # step k reads ctx = S + k positions (incl. the new one)
        decode_bytes.append(P * es + int((S + k).sum()) * kv_pos_bytes + wl.batch * kv_pos_bytes)
    return dict(T=T, P=P, prefill_flops=prefill_flops, decode_bytes=decode_bytes,
                gateup_flops=2 * T * 2 * f * d, qkv_flops=2 * T * 3 * d * d, o_flops=2 * T * d * d,
                down_flops=2 * T * d * f)


def measured_traffic(kernel: str, workload: str):
    """HBM-side bytes per launch (fetch + write) from the committed rocprofv3 --pmc summary
    profiles/pmc_traffic_<workload>.md, or None if the summary or the kernel's row is missing."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_{workload}.md")
    if not os.path.exists(path):
        return None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0] == kernel:
            try:
                return (float(cells[2]) + float(cells[3])) * 1e6
            except ValueError:
                return None
    return None


def cpu_baseline(wl, weights, obs, gum):
    """The oracle as it stands ("cached" mode, proved equal to full recompute by the tests) on two whole
    sequences of the batch (the first and the last), all layers, all K tokens."""
    from threadpoolctl import threadpool_info
    from oracle import vla_oracle as O
    rows = [0, wl.batch - 1]
    pol = O.OraclePolicy(wl.shape, weights)
    pes = [obs["patch_emb"][obs["cu_patch"][b]:obs["cu_patch"][b + 1]] for b in rows]
    ids = [obs["instr_ids"][obs["cu_instr"][b]:obs["cu_instr"][b + 1]] for b in rows]
    temp = wl.temperature if wl.sampling == "gumbel" else 0.0
    t0 = time.perf_counter()
    pol.policy_step(pes, ids, wl.n_tokens, temperature=temp, gumbel=None if gum is None else gum[rows], mode="cached")
    dt = time.perf_counter() - t0
    cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    return {"value": len(rows) * (wl.n_tokens / wl.action_dim) / dt, "unit": "actions/s", "cores": int(cores),
            "kind": "oracle",
            "sample": f"{len(rows)} of {wl.batch} sequences (first and last), all {wl.shape.n_layers} layers, "
                      f"{wl.n_tokens} tokens each: {dt:.1f} s; sequences are independent, so the rate is per sequence"}


def weight_update_leg(pol, weights, step, torch):
    """In-place update of every tensor from device-resident sources (what a broadcast leaves on the inference
    GPU), enqueued on a second stream: device time with the policy idle, and host-observed latency from the drain
    signal to the new version being live when a policy step was enqueued just before.  Same weights are written
    back, so the benchmark's state is unchanged.  Outside the timed region of `value`."""
    dev_w = {n: pol.to_device(t) for n, t in weights.items()}
    nbytes = sum(t.numel() * t.element_size() for t in dev_w.values())
    side = torch.cuda.Stream(device=pol.device)
    torch.cuda.synchronize()
    res = {}
    idle, busy = [], []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pol.drain_begin()
        pol.update_begin(side)
        e0.record(side)
        pol.update_tensors(dev_w, side)
        pol.update_commit(side)
        e1.record(side)
        side.synchronize()
        idle.append(e0.elapsed_time(e1))
    for _ in range(3):
        step()                                   # a whole policy step is in flight when the drain signal comes
        t0 = time.perf_counter()
        pol.drain_begin()
        pol.update_begin(side)
        pol.update_tensors(dev_w, side)
        pol.update_commit(side)
        side.synchronize()
        busy.append((time.perf_counter() - t0) * 1e3)
    torch.cuda.synchronize()
    res["tensors"] = len(dev_w)
    res["source_bytes"] = nbytes
    res["device_ms_idle"] = min(idle)
    res["gbs_read_plus_write"] = 2 * nbytes / (min(idle) * 1e-3) / 1e9
    res["drain_to_live_ms_with_step_in_flight"] = min(busy)
    res["version"] = pol.state()[1]
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--batch", type=int, default=0, help="override the batch (0 = the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prof-mask", type=lambda v: int(v, 0), default=0x3ffff)
    ap.add_argument("--no-weight-update", action="store_true",
                    help="skip the (untimed, reported under detail) in-place weight update measurement")
    ap.add_argument("--precision", choices=["high", "fast"], default="high",
                    help="arithmetic of the 16-bit path: high = two-term operands in the leading layers (meets the "
                         "stated tolerances at 32 layers; the headline), fast = single-term operands everywhere")
    ap.add_argument("--two-term-layers", type=int, default=0,
                    help="--precision high: number of leading layers with two-term operands (0 = the library's "
                         "default, 4)")
    ap.add_argument("--no-other-mode", action="store_true", help="skip the short run of the other precision mode")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the policy shards by "
              "sequence with full weight replicas and no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2603_18464_amd as P
    from paper_2603_18464_amd import VlaPolicy

    wl = W.get_workload(args.workload)
    if args.batch:
        wl = wl.scaled(batch=args.batch)
    t0 = time.perf_counter()
    weights = W.make_weights(wl.shape, wl.seed, threads=16)
    obs = W.make_observations(wl)
    gum = W.make_gumbel(wl) if wl.sampling == "gumbel" else None
    cu_seq = obs["cu_patch"] + obs["cu_instr"]
    nums = model_numbers(wl, cu_seq)
    from paper_2603_18464_amd.binding import VLA_PREC_FAST, VLA_PREC_HIGH
    prec = VLA_PREC_HIGH if args.precision == "high" else VLA_PREC_FAST
    pol = VlaPolicy(wl.shape, wl.batch, wl.max_seq, nums["T"] + wl.batch * (wl.n_tokens - 1), value_max_steps=64,
                    precision=prec, two_term_layers=args.two_term_layers)
    pol.load_weights(weights)
    pol.load_value_head(W.make_value_weights(wl.shape, wl.seed, 64))
    if args.no_weight_update and args.no_other_mode and args.no_cpu_baseline:
        weights = None
    pe = pol.to_device(obs["patch_emb"])
    ids = torch.from_numpy(obs["instr_ids"]).to(pol.device)
    gdev = None if gum is None else torch.from_numpy(gum).to(pol.device)
    temp = wl.temperature if wl.sampling == "gumbel" else 0.0
    out = None
    print(f"# inputs ready in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)

    def step():
        nonlocal out
        out = pol.policy_step(pe, obs["cu_patch"], ids, obs["cu_instr"], wl.n_tokens, temperature=temp,
                              gumbel=gdev, action_dim=wl.action_dim, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    actions_per_s = wl.batch * (wl.n_tokens / wl.action_dim) / (dt / args.steps)

    # per-kernel-family durations with HIP events on the launch stream, over the same number of steps
    P.vla_prof_enable(pol.ctx, args.prof_mask)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    fam = {}
    for i in range(P.vla_prof_count()):
        name, n, ms = P.vla_prof_read(pol.ctx, i)
        if n:
            fam[name] = {"launches": n, "avg_ms": ms / n, "total_ms_per_step": ms / args.steps}
    P.vla_prof_enable(pol.ctx, 0)

    # roofline of the dominant kernel: the prefill GEMM family that takes the most time per step.  `achieved` counts
    # algorithmic flops only (2 * T * N * K of the layer's matrix).  The GEMMs of two-term layers (the first 4 of the
    # default mode) are a template instantiation and a family of their own (`*_two_prefill`): they also run a low-term
    # pass on the 8-bit matrix instructions (half the cycles of the main pass), which is time spent for accuracy and
    # is not counted as work.
    per_launch = {"gemm_qkv_prefill": nums["qkv_flops"], "gemm_o_prefill": nums["o_flops"],
                  "gemm_gateup_prefill": nums["gateup_flops"], "gemm_down_prefill": nums["down_flops"]}
    kernel_names = {"gemm_qkv_prefill": "gemm_f16_pipe_kernel<4,2,EpiQkv,%s> (prefill QKV GEMM)",
                    "gemm_o_prefill": "gemm_f16_pipe_kernel<2,2,EpiResid,%s> (prefill output projection)",
                    "gemm_gateup_prefill": "gemm_f16_pipe_kernel<2,2,EpiSwiglu,%s> (prefill gate/up GEMM)",
                    "gemm_down_prefill": "gemm_f16_pipe_kernel<2,2,EpiResid,%s> (prefill down projection)"}
    for k in list(per_launch):
        k2 = k.replace("_prefill", "_two_prefill")
        per_launch[k2] = per_launch[k]
        kernel_names[k2] = kernel_names[k] % "true" + ", two-term layers: with the 8-bit low-term pass"
        kernel_names[k] = kernel_names[k] % "false"
    roofline = None
    present = [k for k in per_launch if k in fam]
    if present:
        dom = max(present, key=lambda k: fam[k]["total_ms_per_step"])
        g = fam[dom]
        ach = per_launch[dom] / (g["avg_ms"] * 1e-3) / 1e12
        traffic = measured_traffic(dom, wl.name)
        roofline = {"bound": "mfma", "kernel": kernel_names[dom], "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "avg_launch_ms": g["avg_ms"],
                    "flops_per_launch": per_launch[dom], "traffic": traffic,
                    "traffic_from": None if traffic is None else
                    f"profiles/pmc_traffic_{wl.name}.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                    "committed; not re-measured by this run)"}
    extra = {}
    pre_ms = sum(v["total_ms_per_step"] for k, v in fam.items() if k.endswith("_prefill"))
    gemm_pre_ms = sum(v["total_ms_per_step"] for k, v in fam.items() if k.startswith("gemm") and k.endswith("_prefill"))
    dec_ms = sum(v["total_ms_per_step"] for k, v in fam.items() if k.endswith("_decode"))
    if gemm_pre_ms:
        # flops actually executed by the tiled prefill GEMMs (the last layer's output projection and feed-forward
        # run only on the rows that feed the head, in their own family "prefill_tail")
        done = sum(per_launch[k] * fam[k]["launches"] / args.steps for k in per_launch if k in fam)
        extra["prefill_gemm_tflops"] = done / (gemm_pre_ms * 1e-3) / 1e12
        extra["prefill_gemm_frac_of_mfma_peak"] = extra["prefill_gemm_tflops"] / PEAK_BF16_TFLOPS
        extra["prefill_gemm_tflops_by_family"] = {k: per_launch[k] / (fam[k]["avg_ms"] * 1e-3) / 1e12 for k in present}
    if dec_ms and nums["decode_bytes"]:
        gbs = sum(nums["decode_bytes"]) / (dec_ms * 1e-3) / 1e9
        extra["decode_gbs"] = gbs
        extra["decode_frac_of_hbm_peak"] = gbs / PEAK_HBM_GBS
        extra["decode_ms_per_token_step"] = dec_ms / max(1, wl.n_tokens - 1)
    if wl.shape.dtype == "bf16":
        # what this device sustains with nothing in the way, next to the vendor peaks the fractions are quoted on
        mf, sr = P.vla_probe(pol.ctx, 0, pol._stream()), P.vla_probe(pol.ctx, 1, pol._stream())
        extra["ceilings"] = {"mfma_only_tflops": mf, "stream_read_gbs": sr}
        if roofline:
            roofline["frac_of_measured_mfma_loop"] = roofline["achieved"] / mf
        if "decode_gbs" in extra:
            extra["decode_frac_of_measured_stream_read"] = extra["decode_gbs"] / sr
    extra["action_tokens_per_s"] = wl.batch * wl.n_tokens / (dt / args.steps)
    extra["prefill_kernels_ms"] = pre_ms
    extra["families"] = fam
    # the one-pass (placeholder-fed) variant of the step on the same batch: reported, not the headline value
    pout = None
    ph = wl.shape.vocab - wl.shape.n_action_bins

    def pstep():
        nonlocal pout
        pout = pol.policy_step_parallel(pe, obs["cu_patch"], ids, obs["cu_instr"], wl.n_tokens, ph, temperature=temp,
                                        gumbel=gdev, action_dim=wl.action_dim, out=pout)
    pstep()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        pstep()
    torch.cuda.synchronize()
    pdt = (time.perf_counter() - t0) / args.steps
    extra["parallel_decoding"] = {"ms_per_step": pdt * 1e3,
                                  "actions_per_s": wl.batch * (wl.n_tokens / wl.action_dim) / pdt}
    # the same step with the value head on the rollout path (v_t of the trajectory), reported only
    vout = None
    step_t = torch.arange(wl.batch, dtype=torch.int32, device=pol.device) % 64

    def vstep():
        nonlocal vout
        vout = pol.policy_step(pe, obs["cu_patch"], ids, obs["cu_instr"], wl.n_tokens, temperature=temp, gumbel=gdev,
                               action_dim=wl.action_dim, out=vout, step_t=step_t)
    vstep()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        vstep()
    torch.cuda.synchronize()
    extra["with_value_head_ms_per_step"] = (time.perf_counter() - t0) / args.steps * 1e3
    if not args.no_weight_update:
        extra["weight_update"] = weight_update_leg(pol, weights, step, torch)

    line = {
        "metric": "actions/sec of the batched VLA policy step (prefill + action-token decode + log-probs)",
        "value": actions_per_s, "unit": "actions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if wl.shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: 7B Llama-shaped VLA backbone" if wl.shape.n_layers == 32 else wl.name,
                   "n_layers": wl.shape.n_layers, "d_model": wl.shape.d_model, "batch": wl.batch,
                   "prefix_tokens": nums["T"], "action_tokens": wl.n_tokens, "sampling": wl.sampling,
                   "precision": args.precision if wl.shape.dtype == "bf16" else "f32",
                   "weights": ("bf16 at the boundary, re-encoded exactly as f16*2^8 for the matrix cores; f32 "
                               "accumulation; activations and KV cache " +
                               (f"as two terms (f16 + an 8-bit or f16 low term) in the first "
                                f"{min(args.two_term_layers or 4, wl.shape.n_layers)} layers, one f16 term after "
                                "them: meets the stated tolerances at 32 layers"
                                if args.precision == "high" else "as one f16 term (fast mode)"))
                   if wl.shape.dtype == "bf16" else "f32"},
        "roofline": roofline, "detail": extra,
    }
    pol.close()
    del pol
    torch.cuda.empty_cache()
    if wl.shape.dtype == "bf16" and not args.no_other_mode:
        # the other arithmetic mode of the 16-bit path on the same batch: reported, never the headline value
        other = VLA_PREC_FAST if prec == VLA_PREC_HIGH else VLA_PREC_HIGH
        if weights is None:
            weights = W.make_weights(wl.shape, wl.seed, threads=16)
        pol2 = VlaPolicy(wl.shape, wl.batch, wl.max_seq, nums["T"] + wl.batch * (wl.n_tokens - 1), precision=other)
        pol2.load_weights(weights)
        pe2 = pol2.to_device(obs["patch_emb"])
        out2 = None
        for i in range(args.warmup + args.steps):
            if i == args.warmup:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            out2 = pol2.policy_step(pe2, obs["cu_patch"], ids, obs["cu_instr"], wl.n_tokens, temperature=temp,
                                    gumbel=gdev, action_dim=wl.action_dim, out=out2)
        torch.cuda.synchronize()
        dt2 = (time.perf_counter() - t0) / args.steps
        extra["other_precision_mode"] = {
            "precision": ("fast (single-term operands)" if other == VLA_PREC_FAST
                          else "high (two-term operands in the first 4 layers)"),
            "ms_per_step": dt2 * 1e3, "actions_per_s": wl.batch * (wl.n_tokens / wl.action_dim) / dt2,
            "note": "the fast mode misses the stated logit / log-prob tolerances at 32 layers (tests/parity.py)"}
        pol2.close()
    if not args.no_cpu_baseline:
        if weights is None:
            weights = W.make_weights(wl.shape, wl.seed, threads=16)
        line["cpu_baseline"] = cpu_baseline(wl, weights, obs, gum)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
