#!/usr/bin/env python3
"""Throughput of the batched verification step on one MI355X.

One step = sled_verify_batch + sled_accept + sled_kv_append (commit) over one ragged batch of
synthetic requests, inputs resident in HBM.  Workload: Llama-3-8B-shaped decoder (bf16, random
init), 16 requests, contexts uniform in [512, 2048], k uniform in [2, 8], greedy acceptance.

Prints one JSON line: verified draft tokens/s (whole job), p50 step latency, the HBM roofline of
the dominant kernel (the weight-streaming projection GEMM) and the CPU oracle timed on a bounded
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# L2 fetch + write-back bytes per projection launch: a STORED counter figure, not read in this run (FETCH_SIZE and
# WRITE_SIZE of rocprofv3 need runs of their own; each is scaled by what the counter reads for a 1 GiB copy;
# profiles/verify_step_llama8b_b16_hbm_traffic.txt gives the commands and the table).  Taken with gemm_bf16_kernel as
# it stands in csrc/gemm.hip (retaken after every change to that file's kernel code, last after K slices became
# uneven: 149.9 MB each time); to be reset to None whenever that kernel changes.
MEASURED_TRAFFIC = {"llama8b_b16": 149.9e6}
TRAFFIC_NOTE = "stored rocprofv3 FETCH_SIZE+WRITE_SIZE figure for gemm_bf16_kernel (profiles/verify_step_llama8b_b16_hbm_traffic.txt), not measured in this run"
CPU_SAMPLE_REQUESTS, CPU_SAMPLE_LAYERS = 16, 24   # the oracle's bounded sample (about 10-20 s of CPU work)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--workload", default="llama8b_b16", choices=["llama8b_b16", "llama8b_hetero64", "llama70b_b32", "tiny_bf16", "accept_only"],
                    help="llama8b_b16 is the headline configuration; hetero64 uses sampling acceptance over "
                         "full-vocabulary draft probabilities, the others greedy; accept_only times sled_accept "
                         "alone (256 requests x 8 drafts, vocabulary 128256, sampling) on given logits")
    ap.add_argument("--sigma", type=float, default=1.0,
                    help="accept_only: standard deviation of the noise between draft and target logits (the other "
                         "two of 0.25, 1, 4 are reported in the breakdown)")
    ap.add_argument("--q-top", type=int, default=64,
                    help="accept_only: also time sled_accept_sparse with the draft distributions cut to this many entries (0 = skip)")
    ap.add_argument("--weights", default="bf16", choices=["bf16", "fp8", "fp4"],
                    help="fp8: the same shapes with FP8 E4M3 projection weights and per-row scales; fp4: FP4 E2M1 codes with a power-of-two scale per 32 inputs (sled_model_set_weight_bits)")
    ap.add_argument("--batch-invariant", action="store_true",
                    help="time the step with sled_model_set_batch_invariant on (results independent of the batch to the last bit)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--contiguous-pages", action="store_true",
                    help="give every request a run of consecutive physical pages instead of scattering them (for comparison)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a 1 GiB device-to-device copy three times before the steps, so that a counter run "
                         "(FETCH_SIZE / WRITE_SIZE) holds a kernel of known traffic to scale the counters by")
    ap.add_argument("--profile-steps", type=int, default=5, help="steps of the event-instrumented region")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2506_09397_amd import sled, synth
    from paper_2506_09397_amd.runtime import Verifier

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    sled.lib()  # fails loudly if libsled.so has not been built
    torch.cuda.set_device(0)
    if args.workload == "accept_only":
        print(json.dumps(bench_accept(args)))
        return

    if args.workload == "llama8b_b16":
        shape, kind = synth.SHAPES["llama8b"], "b16"
    elif args.workload == "llama8b_hetero64":
        shape, kind = synth.SHAPES["llama8b"], "hetero64"
    elif args.workload == "llama70b_b32":
        shape, kind = synth.SHAPES["llama70b"], "b32"
    else:
        shape, kind = synth.SHAPES["tiny_bf16"], "b16"
    batch = synth.draw_batch(kind, shape.vocab, seed=args.seed)
    B, T, n_drafts = batch.B, batch.T, int(sum(batch.k))
    total_steps = args.warmup + args.steps + args.profile_steps + 2
    ctx_budget = sum(batch.ctx_len) + B * (shape.k_max + 1) * (total_steps + 1)
    n_pages = ctx_budget // 16 + 2 * B + 8
    w8 = args.weights != "bf16"
    wcls = {"bf16": synth.SynthWeights, "fp8": synth.SynthWeightsW8, "fp4": synth.SynthWeightsW4}[args.weights]
    weights = wcls(shape, seed=args.seed, device="cuda")
    v = Verifier(shape, weights, n_pages, B, B, ctx_budget, batch_invariant=args.batch_invariant)
    reqs = [v.open() for _ in range(B)]
    KV = []
    for i in range(B):
        KV.append(synth.context_kv(shape, batch.ctx_len[i], seed=args.seed, req=i, device="cuda"))
    # physical pages scattered over the pool (see Verifier.append_contexts_scattered)
    v.append_contexts_scattered(reqs, KV, seed=args.seed + 11, contiguous=args.contiguous_pages)
    KV = [kv if i < CPU_SAMPLE_REQUESTS else None for i, kv in enumerate(KV)]
    tokens = torch.from_numpy(batch.tokens).cuda()
    torch.cuda.synchronize()

    sampling = kind == "hetero64"
    if sampling:
        # draft probabilities softmax(target-shaped logits + N(0,1) noise) over the full vocabulary, uniforms
        q = synth.draft_probs(n_drafts, shape.vocab, 1.0, seed=args.seed + 3, device="cuda", base_std=1.28)
        u_acc = synth.uniforms(n_drafts, seed=args.seed + 4, device="cuda")
        u_smp = synth.uniforms(B, seed=args.seed + 5, device="cuda")

    def step():
        logits = v.verify(reqs, batch.k, tokens)
        if sampling:
            a, t = v.accept(sled.SAMPLE, batch.k, logits, tokens, q, u_acc, u_smp)
        else:
            a, t = v.accept(sled.GREEDY, batch.k, logits, tokens)
        v.commit(reqs, a)

    if args.copy_calibration:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for s in range(args.steps):
        step()
        ev[s + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    lat = sorted(ev[s].elapsed_time(ev[s + 1]) for s in range(args.steps))
    p50, p90 = lat[len(lat) // 2], lat[min(len(lat) - 1, int(len(lat) * 0.9))]
    value = n_drafts * args.steps / (t1 - t0)
    emitted = int(v.accept_len[:B].sum().item()) + B   # accepted drafts + one correction/bonus token each, last step

    # context actually held after the timed region (greedy on random tokens accepts ~0 drafts, so it
    # grew by about one token per step); used for the algorithmic K/V bytes
    lens = v.lengths(reqs)
    kv_bytes = sum(lens) * shape.kv_bytes_per_token()
    weight_bytes = int(shape.streamed_params() * {"bf16": 32, "fp8": 16, "fp4": 8.5}[args.weights] / 16)   # fp4: codes + a scale byte per 32
    logits_bytes = T * shape.vocab * 4

    # event-instrumented region: per-class kernel time on the stream the kernels run on
    sled.sled_profile_enable(v.model, True)
    for _ in range(args.profile_steps):
        step()
    ms, n = sled.sled_profile_read(v.model)
    sled.sled_profile_enable(v.model, False)
    psteps = max(args.profile_steps, 1)
    proj_ms = max(ms[sled.PROF_PROJ] / psteps, 1e-9)
    proj_launches = n[sled.PROF_PROJ] // psteps
    achieved = weight_bytes / (proj_ms * 1e-3) / 1e9
    roofline = {
        "bound": "hbm", "kernel": "gemm_bf16_kernel (projection GEMMs, weight stream)",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": (traffic := None if (w8 or args.batch_invariant) else MEASURED_TRAFFIC.get(args.workload)),
        "traffic_source": TRAFFIC_NOTE if traffic is not None else None,
        "launches_per_step": proj_launches, "avg_launch_us": round(proj_ms * 1e3 / max(proj_launches, 1), 2),
        "bytes_per_launch": round(weight_bytes / max(proj_launches, 1)),
    }
    step_bytes = weight_bytes + kv_bytes + logits_bytes
    copy_gbs = copy_bandwidth_gbs()
    breakdown = {
        "verify_launches_per_step": sum(n) // psteps,
        "proj_ms": round(proj_ms, 4), "attn_ms": round(ms[sled.PROF_ATTN] / psteps, 4),
        "rows_ms": round(ms[sled.PROF_ROWS] / psteps, 4),
        "attn_GBps": round(kv_bytes / max(ms[sled.PROF_ATTN] / psteps, 1e-9) / 1e6, 1),
        "step_bytes": step_bytes, "step_hbm_frac": round(step_bytes / (p50 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "copy_GBps": round(copy_gbs, 1), "step_frac_of_copy": round(step_bytes / (p50 * 1e-3) / 1e9 / copy_gbs, 4),
        "emitted_tokens_per_s": round(emitted / (p50 * 1e-3), 1),
    }

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, weights, batch, KV, args)

    out = {
        "metric": "verified draft tokens/sec per batched verify step", "value": round(value, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "p50_ms": round(p50, 4), "p90_ms": round(p90, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": {"bf16": "bf16", "fp8": "bf16 (fp8 e4m3 weights)", "fp4": "bf16 (mxfp4 weights)"}[args.weights], "data": "synthetic",
        "config": {"workload": f"{args.workload}: {shape.n_layers} layers d={shape.d_model} Hq/Hkv={shape.n_q_heads}/"
                               f"{shape.n_kv_heads} F={shape.d_ffn} V={shape.vocab}, B={B}, T={T} packed rows, "
                               f"{n_drafts} draft tokens, {sum(lens)} context tokens, {'sampling' if sampling else 'greedy'} acceptance, "
                               f"seed {args.seed}" + (", batch-invariant mode" if args.batch_invariant else "") + {"bf16": "", "fp8": ", FP8 E4M3 weights", "fp4": ", MXFP4 weights"}[args.weights]},
        "roofline": roofline, "breakdown": breakdown, "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    v.destroy()


def copy_bandwidth_gbs():
    """Bytes moved per second (read + write) by a 1 GiB device-to-device copy on this GPU."""
    import torch
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def bench_accept(args):
    """sled_accept alone: 256 requests x (8 drafts + 1 bonus row) x vocabulary 128256, target logits N(0, 2), draft
    logits = target + sigma * N(0, 1), drafts drawn from q, speculative-sampling acceptance (Eq. 1)."""
    import numpy as np
    import torch
    from paper_2506_09397_amd import sled, synth
    vocab, k = 128256, [8] * 256
    B, T, nd = len(k), sum(k) + len(k), sum(k)
    ws = sled.workspace(sled.sled_accept_workspace_bytes(B, T, vocab))
    a = torch.zeros(B, dtype=torch.int32, device="cuda")
    t = torch.zeros(B, dtype=torch.int32, device="cuda")
    row_bytes = vocab * 4
    per_sigma = {}
    main = None
    sigmas = [args.sigma] + [x for x in (0.25, 1.0, 4.0) if x != args.sigma]
    cpu = None
    for sg in sigmas:
        case = synth.accept_case(k, vocab, sg, seed=args.seed + int(sg * 100), device="cuda")

        def step():
            sled.sled_accept(sled.SAMPLE, k, vocab, 1.0, case.logits, case.tokens, case.q, case.u_acc, case.u_smp, a, t, ws)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        t0 = time.perf_counter()
        ev[0].record()
        for s in range(args.steps):
            step()
            ev[s + 1].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        lat = sorted(ev[s].elapsed_time(ev[s + 1]) for s in range(args.steps))
        p50, p90 = lat[len(lat) // 2], lat[min(len(lat) - 1, int(len(lat) * 0.9))]
        acc = a.cpu().numpy()
        # least the rule has to touch: rows 0..a_i of each request, and the draft distribution of the rejected draft
        min_bytes = int(sum((int(x) + 1) + (1 if x < ki else 0) for x, ki in zip(acc, k))) * row_bytes
        scan_bytes = T * row_bytes + int(sum(1 for x, ki in zip(acc, k) if x < ki)) * row_bytes * 2 + \
            int(sum(1 for x, ki in zip(acc, k) if x >= ki)) * row_bytes
        rec = {"ms_per_step": round((t1 - t0) * 1e3 / args.steps, 4), "p50_ms": round(p50, 4), "p90_ms": round(p90, 4),
               "mean_accept_len": round(float(acc.mean()), 3), "verified_draft_tokens_per_s": round(nd / (p50 * 1e-3), 1),
               "min_bytes": min_bytes, "min_bytes_GBps": round(min_bytes / (p50 * 1e-3) / 1e9, 1),
               "touched_bytes": scan_bytes, "touched_GBps": round(scan_bytes / (p50 * 1e-3) / 1e9, 1)}
        if args.q_top > 0:
            # the same logits and drafts with the draft distributions cut to their top entries, through the sparse entry point
            top = torch.topk(case.q, args.q_top, dim=1)
            q_ids = top.indices.int().contiguous()
            q_probs = (top.values / top.values.sum(dim=1, keepdim=True)).float().contiguous()

            def step_sparse():
                sled.sled_accept_sparse(k, vocab, 1.0, case.logits, case.tokens, q_ids, q_probs, case.u_acc, case.u_smp, a, t, ws)

            for _ in range(args.warmup):
                step_sparse()
            torch.cuda.synchronize()
            ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
            ev2[0].record()
            for s in range(args.steps):
                step_sparse()
                ev2[s + 1].record()
            torch.cuda.synchronize()
            lat2 = sorted(ev2[s].elapsed_time(ev2[s + 1]) for s in range(args.steps))
            rec[f"sparse_top{args.q_top}_p50_ms"] = round(lat2[len(lat2) // 2], 4)
            rec[f"sparse_top{args.q_top}_mean_accept_len"] = round(float(a.float().mean().item()), 3)
            del top, q_ids, q_probs
        per_sigma[str(sg)] = rec
        if main is None:
            main = dict(rec, wall=(t1 - t0))
            if not args.no_cpu_baseline:
                cpu = cpu_baseline_accept(case, k, vocab)
        del case
        torch.cuda.empty_cache()
    copy_gbs = copy_bandwidth_gbs()
    achieved = main["touched_GBps"]
    return {
        "metric": "verified draft tokens/sec, acceptance step alone", "value": round(nd * args.steps / main["wall"], 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main["ms_per_step"],
        "p50_ms": main["p50_ms"], "p90_ms": main["p90_ms"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32 logits, f64 sums", "data": "synthetic",
        "config": {"workload": f"accept_only: B={B}, k=8 (+1 bonus row), V={vocab}, T={T} logits rows, sampling, "
                               f"sigma={args.sigma}, seed {args.seed}"},
        "roofline": {"bound": "hbm", "kernel": "sled_accept: accept_row_stats (scan of all logits rows) + accept_finish (decision, inverse-CDF draw)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None, "bytes_per_launch": main["touched_bytes"],
                     "frac_on_min_bytes": round(main["min_bytes_GBps"] / HBM_PEAK_GBS, 4),
                     "copy_GBps": round(copy_gbs, 1), "frac_of_copy": round(achieved / copy_gbs, 4)},
        "breakdown": per_sigma, "cpu_baseline": cpu,
    }


def cpu_baseline_accept(case, k, vocab, n_req=16):
    """The oracle's acceptance on the first n_req requests of the case."""
    import numpy as np
    from oracle import sled_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    kk = k[:n_req]
    T, nd = sum(kk) + n_req, sum(kk)
    logits = case.logits[:T].cpu().numpy().astype(np.float64)
    tokens = case.tokens[:T].cpu().numpy()
    q = case.q[:nd].cpu().numpy().astype(np.float64)
    u_acc = case.u_acc[:nd].cpu().numpy().astype(np.float64)
    u_smp = case.u_smp[:n_req].cpu().numpy().astype(np.float64)
    t0 = time.perf_counter()
    reps = 0
    while time.perf_counter() - t0 < 10.0:
        O.accept_batch("sample", kk, logits, tokens, q, u_acc, u_smp)
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return {"value": round(nd / dt, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n_req} of {len(k)} requests ({T} logits rows), {reps} repetitions, {dt:.3f} s each"}


def cpu_baseline(shape, weights, batch, KV, args):
    """The oracle as it stands, on a bounded sample: the first CPU_SAMPLE_REQUESTS requests of the batch
    through the first CPU_SAMPLE_LAYERS layers plus final norm, LM head and acceptance; layer time is
    scaled to the full depth and request time to the full batch by rows."""
    import numpy as np
    from oracle import sled_oracle as O
    from oracle.harness import oracle_model
    from paper_2506_09397_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    n_req = min(CPU_SAMPLE_REQUESTS, batch.B)
    # the oracle widens the sampled layers to float64: keep that under about 45 GB of host memory
    n_lay = max(1, min(CPU_SAMPLE_LAYERS, shape.n_layers, int(45e9 // (shape.layer_params() * 8))))
    om = oracle_model(shape, weights, n_layers=n_lay)
    offs = batch.row_offsets()
    reqs = []
    for i in range(n_req):
        K, V = KV[i]
        reqs.append({"tokens": batch.tokens[offs[i]: offs[i + 1]], "K": synth.as_f64(K[:n_lay]), "V": synth.as_f64(V[:n_lay])})
    om.weights.embed(); om.weights.final()
    for l in range(n_lay):
        om.weights.layer(l)          # widen to float64 outside the timed part
    rows = sum(len(r["tokens"]) for r in reqs)
    t0 = time.perf_counter()
    res = O.verify_batch(om, reqs)
    t_all = time.perf_counter() - t0
    # time of the head alone, to scale only the layer part with depth
    om0 = oracle_model(shape, weights, n_layers=0)
    om0.weights._c = om.weights._c
    reqs0 = [{"tokens": r["tokens"], "K": r["K"][:0], "V": r["V"][:0]} for r in reqs]
    t0 = time.perf_counter()
    O.verify_batch(om0, reqs0)
    t_head = time.perf_counter() - t0
    t0 = time.perf_counter()
    logits = np.concatenate([r["logits"] for r in res], axis=0).astype(np.float32).astype(np.float64)
    O.accept_batch("greedy", batch.k[:n_req], logits, batch.tokens[: offs[n_req]])
    t_acc = time.perf_counter() - t0
    t_layers = max(t_all - t_head, 0.0)
    est = (t_layers * shape.n_layers / n_lay + t_head + t_acc) * batch.T / rows
    return {"value": round(sum(batch.k) / est, 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n_req} of {batch.B} requests ({rows} of {batch.T} rows), first {n_lay} of {shape.n_layers} "
                      f"layers + LM head + greedy acceptance, {t_all + t_acc:.1f} s measured, scaled by depth and rows "
                      f"to {est:.1f} s per step"}


if __name__ == "__main__":
    main()
