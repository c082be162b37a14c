#!/usr/bin/env python3
"""Throughput of the OBRS hot path on one MI355X.

A step is one pass of the whole hot path (row stage + batch stage, `jp_obrs_forward`) over one
batch of seeded synthetic logits that are already resident in HBM.  The workload is the
Qwen3-1.7B-shaped rollout batch (T=8192 tokens, V=151936, bf16 logits, k=64, lambda=1).

Prints one JSON line: tokens/s for the whole path, the HBM roofline of the dominant kernel (the
row kernel, timed with HIP events on the launch stream) and the float64 CPU oracle timed on a
bounded sample of the same batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "OBRS tokens/sec at V=151936 bf16 on 1 MI355X; achieved HBM GB/s vs peak"
HBM_PEAK_GBS = 8000.0

KERNEL_SOURCES = ("paper_2602_06107_amd/csrc/jp_row_kernel.hip", "paper_2602_06107_amd/csrc/jp_device_utils.h")
# of the header shared by all kernels only the row kernel's own part counts: its argument struct and
# the row record (from "struct RowArgs" up to "struct ZExactArgs")
KERNEL_ARGS_HEADER = ("paper_2602_06107_amd/csrc/jp_obrs_internal.h", b"struct RowArgs", b"struct ZExactArgs")


def kernel_source_digest() -> str:
    """sha256 over the sources of the row kernel: a traffic record only counts for the code it was taken on."""
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    rel, first, last = KERNEL_ARGS_HEADER
    with open(os.path.join(ROOT, rel), "rb") as f:
        text = f.read()
    h.update(text[text.index(first):text.index(last)])
    return h.hexdigest()[:16]


def measured_traffic(T: int, V: int, k: int):
    """HBM bytes per row-kernel launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs whose
    summaries are committed under profiles/ (a line `traffic_record: {json}` in the summary, KiB per
    dispatch and the factors a plain copy of known size gave in the same run).  Returns
    (bytes or None, where it came from / why not): None when no record covers this workload or the
    kernel sources have changed since the record was taken."""
    import glob
    digest = kernel_source_digest()
    stale = None
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        with open(path) as f:
            for line in f:
                if not line.startswith("traffic_record:"):
                    continue
                rec = json.loads(line[len("traffic_record:"):])
                if (rec.get("kernel"), rec.get("T"), rec.get("V"), rec.get("k")) != ("row_kernel", T, V, k):
                    continue
                if rec.get("kernel_source_sha256") != digest:
                    stale = "record in profiles/%s was taken on other kernel sources (%s, now %s)" % (
                        os.path.basename(path), rec.get("kernel_source_sha256"), digest)
                    continue
                nbytes = int(rec["fetch_kib"] * 1024 * rec["fetch_factor"] + rec["write_kib"] * 1024 * rec["write_factor"])
                return nbytes, "profiles/" + os.path.basename(path)
    return None, stale or "no traffic record for this workload under profiles/"


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def algorithmic_bytes_per_token(V: int, k: int, esz: int) -> int:
    """Bytes the row stage must move per token: both logit rows once, the sampled id and the
    uniform, the seven per-token results (a, mask, log q, log p, log-ratio, Z_approx, |V_k|) and
    the two top-k id lists."""
    reads = 2 * V * esz + 4 + 4
    writes = 4 + 1 + 4 + 4 + 4 + 4 + 4 + 2 * k * 4
    return reads + writes


MFMA_BF16_PEAK_TFLOPS = 2500.0


def bench_lm_head(args, torch, obrs, wl, dev):
    """Context figure for the fused lm_head form (T=16384, d=2048/4096, V=151936, k=64): a step is
    one jp_obrs_forward_lmhead call; the roofline is the dense bf16 MFMA peak against the flops of
    the two projections over the whole call (transposes and row kernels included)."""
    T = args.tokens if args.tokens > 0 else 16384
    w = wl.lm_head(T=T, device=dev, k=args.k if args.k > 0 else 64).with_params(lam=args.lam)
    V, da, dp = w.V, w.H_actor.shape[1], w.H_policy.shape[1]
    nbytes = obrs.jp_obrs_lmhead_workspace_bytes(T, V, da, dp, w.k, args.vocab_chunk)
    buf = obrs.alloc_buffers(T, V, w.k, obrs.JP_F32, 0, dev, workspace_bytes=nbytes)

    one_wave = args.flags & obrs.JP_FLAG_ONE_WAVE_PER_ROW          # the only --flags bit this workload takes
    Wa, Wp, lm_flags = w.W_actor, w.W_policy, one_wave
    if args.w_vocab_major:
        Wa, Wp, lm_flags = w.W_actor.t().contiguous(), w.W_policy.t().contiguous(), obrs.JP_FLAG_W_VOCAB_MAJOR | one_wave

    def step():
        obrs.jp_obrs_forward_lmhead(w.H_actor, Wa, w.H_policy, Wp, w.sampled_ids,
                                    w.uniforms, None, w.lam, w.k, w.c1, w.c2, lm_flags, buf, args.vocab_chunk)

    stored = args.stored != "none"
    if stored:
        # --stored: one head only (jp_obrs_forward_lmhead_stored).  The stored actor side is what
        # the two-head form itself finds on the same inputs: its top-k(q) ids and log-probabilities.
        full = obrs.alloc_buffers(T, V, w.k, obrs.JP_F32, obrs.JP_FLAG_TOPK_LOGPROBS, dev, workspace_bytes=nbytes)
        obrs.jp_obrs_forward_lmhead(w.H_actor, Wa, w.H_policy, Wp, w.sampled_ids, w.uniforms, None, w.lam, w.k,
                                    w.c1, w.c2, lm_flags | obrs.JP_FLAG_TOPK_LOGPROBS, full, args.vocab_chunk)
        torch.cuda.synchronize()
        s_ids, s_lq, s_lqx = full.topk_actor.clone(), full.topk_actor_logq.clone(), full.logq.clone()
        del full, buf
        rule = {"drop": obrs.JP_TAIL_DROP, "kth": obrs.JP_TAIL_KTH, "rest": obrs.JP_TAIL_REST}[args.stored]
        nbytes = obrs.jp_obrs_lmhead_stored_workspace_bytes(T, V, dp, w.k, args.vocab_chunk)
        buf = obrs.alloc_buffers(T, V, w.k, obrs.JP_F32, 0, dev, workspace_bytes=nbytes,
                                 want=["accept_prob", "mask", "logq", "logp", "logratio", "z_approx", "w_obrs",
                                       "rho", "union_size", "topk_policy", "stats"])

        def step():
            obrs.jp_obrs_forward_lmhead_stored(w.H_policy, Wp, s_ids, s_lq, s_lqx, w.sampled_ids, w.uniforms, None,
                                               w.lam, w.k, w.c1, w.c2, lm_flags, rule, buf, args.vocab_chunk)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    st = buf.stats()
    flops = 2.0 * T * V * (dp if stored else da + dp)
    tflops = flops * args.steps / wall / 1e12
    print(json.dumps({
        "metric": "OBRS tokens/sec, fused lm_head form%s (context, not the headline metric)"
                  % (", stored actor side (%s)" % args.stored if stored else ""),
        "value": T * args.steps / wall, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16 x bf16 -> f32", "data": "synthetic",
        "config": {"workload": "lm_head: T=%d, d_actor=%d, d_policy=%d, V=%d, k=%d, lambda=%g, chunk=%s, W as %s"
                               % (T, da, dp, V, w.k, w.lam, args.vocab_chunk or "library default (4096 at this T)" if T > 6144 or args.vocab_chunk else "library default (from T)",
                                  "[V, d]" if args.w_vocab_major else "[d, V]"),
                   "kappa": st.kappa, "alpha_hat": st.alpha_hat},
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "kernel": "whole call (gemm_tn_kernel dominates)", "flops": flops},
        "cpu_baseline": None}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200,
                    help="timed steps (the legs that time single kernels with events use at most 20 launches)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", choices=["rollout", "training", "long", "lm_head"], default="rollout",
                    help="rollout (T=8192, k=64) is the configuration the metric is quoted on; the "
                         "others are for context")
    ap.add_argument("--tokens", type=int, default=0, help="override T of the workload")
    ap.add_argument("--k", type=int, default=0, help="override k of the workload")
    ap.add_argument("--lam", type=float, default=1.0)
    ap.add_argument("--flags", type=int, default=0,
                    help="JP_FLAG_* bits for the timed calls (default 0: the hot path as quoted; "
                         "8 adds the per-token distillation KL to the same sweep)")
    ap.add_argument("--vocab-chunk", type=int, default=0, help="lm_head workload: columns per chunk")
    ap.add_argument("--w-vocab-major", action="store_true",
                    help="lm_head workload: hand the weights over as [V, d] (no transpose inside the call)")
    ap.add_argument("--calibrate-copy", type=int, default=0,
                    help="also run this many plain elementwise passes (bf16 negate) over the actor tensor: "
                         "a kernel of known HBM traffic that scales rocprofv3 FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--grad", choices=["none", "bf16", "f32"], default="none",
                    help="also time jp_obrs_distill_grad (gradient of the distillation term w.r.t. the "
                         "actor logits, written in this dtype) and report it as \"distill_grad\"")
    ap.add_argument("--stored", choices=["none", "drop", "kth", "rest"], default="none",
                    help="also time jp_obrs_forward_stored (actor side as TopK_inf ids + log-probabilities, "
                         "only the policy tensor is swept) with this rule and report it as \"stored_actor\"; "
                         "with --workload lm_head: time jp_obrs_forward_lmhead_stored instead of the two-head form")
    ap.add_argument("--token-logprob", action="store_true",
                    help="also time jp_obrs_token_logprob (log-probability of the sampled token under one "
                         "more logit tensor, one sweep) and report it as \"token_logprob\"")
    ap.add_argument("--budget", type=float, default=0.0,
                    help="also time jp_obrs_lambda_for_budget (per-row lambda that meets this acceptance "
                         "budget) and the one-lambda-per-batch variant, and report them as \"lambda_for_budget\"")
    ap.add_argument("--cpu-rows", type=int, default=4096,
                    help="rows of the batch the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--cpu-rows-single", type=int, default=256,
                    help="rows the CPU oracle is timed on with ONE thread, for a per-core figure (0 = skip)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; the hot path has no collectives and "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_06107_amd import obrs
    from paper_2602_06107_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload == "lm_head":
        return bench_lm_head(args, torch, obrs, wl, dev)
    make = {"rollout": wl.rollout, "training": wl.training, "long": wl.long_response}[args.workload]
    w = make(dev, T=args.tokens) if args.tokens > 0 else make(dev)
    w = w.with_params(lam=args.lam, k=args.k if args.k > 0 else w.k)
    T, V = w.T, w.V
    esz = w.actor.element_size()
    buf = obrs.alloc_buffers(T, V, w.k, obrs.JP_BF16, args.flags, dev)
    torch.cuda.synchronize()

    def step():
        obrs.jp_obrs_forward(w.actor, w.policy, w.sampled_ids, w.uniforms, None, w.lam, w.k, w.c1,
                             w.c2, args.flags, buf)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = T * args.steps / wall
    st = buf.stats()

    # ---- dominant kernel: the row kernel alone, HIP events on the launch stream -----------------
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(min(args.steps, 20))]
    for a, b in evs:
        a.record()
        obrs.jp_obrs_rows(w.actor, w.policy, w.sampled_ids, w.uniforms, w.lam, w.k, args.flags & ~1, buf)
        b.record()
    torch.cuda.synchronize()
    row_ms = sorted(a.elapsed_time(b) for a, b in evs)
    row_ms_avg = sum(row_ms) / len(row_ms)
    algo_bytes = algorithmic_bytes_per_token(V, w.k, esz) * T
    achieved = algo_bytes / (row_ms_avg * 1e-3) / 1e9
    traffic, traffic_source = measured_traffic(T, V, w.k)

    # the attainable read-only ceiling of this machine, from code in the tree: the one-tensor sweep
    # of jp_obrs_token_logprob (log-sum-exp + one gather, nothing else), timed the same way
    lp_tmp = torch.empty(T, dtype=torch.float32, device=dev)
    cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 20) + 1)]
    for a, b in cev:
        a.record()
        obrs.jp_obrs_token_logprob(w.policy, w.sampled_ids, lp_tmp)
        b.record()
    torch.cuda.synchronize()
    c_ms = sorted(a.elapsed_time(b) for a, b in cev[1:])
    c_avg = sum(c_ms) / len(c_ms)
    ceiling = {"kernel": "token_logprob_kernel<bf16> (one tensor, read only)", "kernel_ms_avg": c_avg,
               "achieved": T * (V * esz + 8) / (c_avg * 1e-3) / 1e9, "unit": "GB/s"}

    # JP_FLAG_EXACT_Z: what the second sweep costs and how much of Z the top-k estimate holds
    exact_info = None
    if args.flags & 1:
        xev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 20) + 1)]
        for a, b in xev:
            a.record()
            obrs.jp_obrs_rows(w.actor, w.policy, w.sampled_ids, w.uniforms, w.lam, w.k, args.flags, buf)
            b.record()
        torch.cuda.synchronize()
        x_ms = sorted(a.elapsed_time(b) for a, b in xev[1:])
        x_avg = sum(x_ms) / len(x_ms)
        ratio = (buf.z_approx.double() / buf.z_exact.double())
        exact_info = {"rows_plus_exact_z_ms_avg": x_avg, "exact_z_extra_ms": x_avg - row_ms_avg,
                      "z_approx_over_z_exact_mean": float(ratio.mean()), "z_approx_over_z_exact_min": float(ratio.min()),
                      "mean_z_exact": st.mean_z_exact, "mean_z_approx": st.mean_z_approx, "k": w.k}

    grad_info = None
    if args.grad != "none":
        gdt = torch.bfloat16 if args.grad == "bf16" else torch.float32
        grad = torch.empty((T, V), dtype=gdt, device=dev)
        gev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(min(args.steps, 20) + 1)]
        for a, b in gev:
            a.record()
            obrs.jp_obrs_distill_grad(w.actor, w.policy, None, 1.0 / T, grad, buf)
            b.record()
        torch.cuda.synchronize()
        g_ms = sorted(a.elapsed_time(b) for a, b in gev[1:])
        g_avg = sum(g_ms) / len(g_ms)
        g_bytes = T * (V * (2 * esz + grad.element_size()) + 8 + 8 + 1)   # two rows in, one row out, LSEs, row status
        grad_info = {"kernel": "distill_grad_kernel<bf16,%s>" % args.grad, "kernel_ms_avg": g_avg,
                     "kernel_ms_min": g_ms[0], "algorithmic_bytes": g_bytes, "bound": "hbm",
                     "achieved": g_bytes / (g_avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": g_bytes / (g_avg * 1e-3) / 1e9 / HBM_PEAK_GBS, "tokens_per_s": T / (g_avg * 1e-3)}
        del grad

    stored_info = None
    if args.stored != "none":
        rule = {"drop": obrs.JP_TAIL_DROP, "kth": obrs.JP_TAIL_KTH, "rest": obrs.JP_TAIL_REST}[args.stored]
        # the rollout phase's record of the actor, taken here from the two-tensor path's own outputs
        fb = obrs.alloc_buffers(T, V, w.k, obrs.JP_BF16, obrs.JP_FLAG_TOPK_LOGPROBS, dev)
        obrs.jp_obrs_forward(w.actor, w.policy, w.sampled_ids, w.uniforms, None, w.lam, w.k, w.c1, w.c2,
                             obrs.JP_FLAG_TOPK_LOGPROBS, fb)
        torch.cuda.synchronize()
        s_ids, s_lq, s_lqx = fb.topk_actor, fb.topk_actor_logq, fb.logq
        sb = obrs.alloc_buffers(T, V, w.k, obrs.JP_BF16, 0, dev)
        sev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(min(args.steps, 20) + 1)]
        for a, b in sev:
            a.record()
            obrs.jp_obrs_forward_stored(w.policy, s_ids, s_lq, s_lqx, w.sampled_ids, w.uniforms, None, w.lam,
                                        w.k, w.c1, w.c2, 0, rule, sb)
            b.record()
        torch.cuda.synchronize()
        s_ms = sorted(a.elapsed_time(b) for a, b in sev[1:])
        s_avg = sum(s_ms) / len(s_ms)
        # one logit row, the stored list (ids + log-probs) and log q(x) in; per-token results and one id list out
        s_bytes = T * (V * esz + w.k * 8 + 4 + 8 + 25 + w.k * 4)
        sst = sb.stats()
        stored_info = {"call": "jp_obrs_forward_stored (row stage + batch stage), rule " + args.stored,
                       "ms_avg": s_avg, "ms_min": s_ms[0], "tokens_per_s": T / (s_avg * 1e-3),
                       "algorithmic_bytes": s_bytes, "bound": "hbm", "achieved": s_bytes / (s_avg * 1e-3) / 1e9,
                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": s_bytes / (s_avg * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "kappa": sst.kappa, "mean_z_approx": sst.mean_z_approx}
        del fb, sb

    logprob_info = None
    if args.token_logprob:
        lp_out = torch.empty(T, dtype=torch.float32, device=dev)
        lev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(min(args.steps, 20) + 1)]
        for a, b in lev:
            a.record()
            obrs.jp_obrs_token_logprob(w.policy, w.sampled_ids, lp_out)
            b.record()
        torch.cuda.synchronize()
        l_ms = sorted(a.elapsed_time(b) for a, b in lev[1:])
        l_avg = sum(l_ms) / len(l_ms)
        l_bytes = T * (V * esz + 4 + 4)
        logprob_info = {"kernel": "token_logprob_kernel<bf16>", "kernel_ms_avg": l_avg, "kernel_ms_min": l_ms[0],
                        "algorithmic_bytes": l_bytes, "bound": "hbm", "achieved": l_bytes / (l_avg * 1e-3) / 1e9,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": l_bytes / (l_avg * 1e-3) / 1e9 / HBM_PEAK_GBS}

    budget_info = None
    if args.budget > 0:
        lam_out = torch.empty(T, dtype=torch.float32, device=dev)
        bev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(min(args.steps, 5) + 1)]
        for a, b in bev:
            a.record()
            obrs.jp_obrs_lambda_for_budget(w.actor, w.policy, args.budget, buf, out=lam_out)
            b.record()
        torch.cuda.synchronize()
        b_ms = sorted(a.elapsed_time(b) for a, b in bev[1:])
        b_avg = sum(b_ms) / len(b_ms)
        # two sweeps of both rows is what the search needs on this recipe (one approximate, one exact);
        # a row that needs more moves more bytes than it is credited with here
        b_bytes = 2 * T * 2 * V * esz
        budget_info = {"kernel": "budget_kernel<bf16>", "abar": args.budget, "kernel_ms_avg": b_avg,
                       "kernel_ms_min": b_ms[0], "sweeps_credited": 2, "algorithmic_bytes": b_bytes, "bound": "hbm",
                       "achieved": b_bytes / (b_avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": b_bytes / (b_avg * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "mean_lambda": float(lam_out.double().mean())}
        one = torch.empty(1, dtype=torch.float32, device=dev)
        b_scratch = torch.empty(obrs._lib.jp_obrs_budget_scratch_bytes(), dtype=torch.uint8, device=dev)
        for a, b in bev:
            a.record()
            obrs.jp_obrs_lambda_for_budget_batch(w.actor, w.policy, args.budget, buf, out=one, scratch=b_scratch)
            b.record()
        torch.cuda.synchronize()
        bb_ms = sorted(a.elapsed_time(b) for a, b in bev[1:])
        budget_info["batch"] = {"call_ms_avg": sum(bb_ms) / len(bb_ms), "call_ms_min": bb_ms[0], "lambda": float(one.item())}

    if args.calibrate_copy > 0:
        scratch = torch.empty_like(w.actor)
        for _ in range(args.calibrate_copy):
            torch.neg(w.actor, out=scratch)      # elementwise kernel: reads and writes T*V*2 bytes
        torch.cuda.synchronize()
        del scratch

    # ---- CPU oracle on a bounded sample of the same batch ---------------------------------------
    cpu = None
    if args.cpu_rows > 0:
        from oracle import obrs_oracle as orc
        n = min(args.cpu_rows, T)
        a_np = wl.logits_to_numpy(w.actor[:n])
        p_np = wl.logits_to_numpy(w.policy[:n])
        x_np = w.sampled_ids[:n].cpu().numpy()
        u_np = w.uniforms[:n].cpu().numpy()
        orc.lib()
        c0 = time.perf_counter()
        R = orc.rows(a_np, p_np, x_np, u_np, w.lam, w.k)
        orc.batch(R.out, R.out["mask"], w.lam, w.c1, w.c2)
        cw = time.perf_counter() - c0
        cpu = {"value": n / cw, "unit": "tokens/s", "cores": int(R.threads), "kind": "oracle",
               "cpu_model": cpu_model(),
               "sample": f"first {n} of {T} rows of the same batch, float64 C oracle, "
                         f"{cw:.1f} s wall"}
        n1 = min(args.cpu_rows_single, n)
        if n1 > 0:
            c0 = time.perf_counter()
            R1 = orc.rows(a_np[:n1], p_np[:n1], x_np[:n1], u_np[:n1], w.lam, w.k, n_threads=1)
            c1 = time.perf_counter() - c0
            cpu["single_thread"] = {"value": n1 / c1, "unit": "tokens/s", "cores": int(R1.threads),
                                    "sample": f"first {n1} rows, one thread, {c1:.1f} s wall"}

    line = {
        "metric": METRIC,
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: T=%d, V=%d, bf16 logits, k=%d, lambda=%g, c1=c2=3"
                               % (w.name, T, V, w.k, w.lam),
                   "logits_dtype": "bf16", "T": T, "V": V, "k": w.k, "lambda": w.lam, "flags": args.flags,
                   "kappa": st.kappa, "alpha_hat": st.alpha_hat},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "traffic_over_algorithmic": (traffic / algo_bytes) if traffic else None,
                     "read_only_ceiling": ceiling,
                     "kernel": "row_kernel<bf16,key32,%d>" % (64 if w.k <= 64 else 128 if w.k <= 128 else 256), "kernel_ms_avg": row_ms_avg,
                     "kernel_ms_min": row_ms[0], "algorithmic_bytes": algo_bytes},
        "cpu_baseline": cpu,
    }
    if exact_info is not None:
        line["exact_z"] = exact_info
    if grad_info is not None:
        line["distill_grad"] = grad_info
    if stored_info is not None:
        line["stored_actor"] = stored_info
    if logprob_info is not None:
        line["token_logprob"] = logprob_info
    if budget_info is not None:
        line["lambda_for_budget"] = budget_info
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
