"""Measurement sweeps around the batched verify step (one MI355X, synthetic inputs, through the C ABI).

    python bench_sweeps.py batch     # step latency vs batch size and speculative length
    python bench_sweeps.py rows [llama70b] [sizes]   # projection time vs number of packed rows (MFMA regime)
    python bench_sweeps.py prefill   # prompt ingest (sled_prefill): prompt length x rows per slice
    python bench_sweeps.py weights   # verify step with bf16, FP8 and FP4 weights, by rows

`batch` is the one-GPU analogue of the paper's throughput-versus-batch-size curve (Sec. 4.1) and of its
study of the speculative length (Sec. 4.2): Llama-3-8B shape, contexts uniform in [512, 2048], every request
with the same k.  `rows` packs many short requests (16 context tokens, k = 8) so that attention is
negligible and reads the time of the projection kernels from the library's timing hooks:
useful FLOP = 2 * rows * streamed parameters.
"""
from __future__ import annotations

import sys
import time

import numpy as np
import torch

import os

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from paper_2506_09397_amd import sled, synth  # noqa: E402
from paper_2506_09397_amd.runtime import Verifier  # noqa: E402

MFMA_PEAK_BF16 = 2.5e15


def _time_steps(v, reqs, k, tokens, steps=8, warmup=2, profile=False):
    def step():
        logits = v.verify(reqs, k, tokens)
        a, t = v.accept(sled.GREEDY, k, logits, tokens)
        v.commit(reqs, a)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for s in range(steps):
        step()
        ev[s + 1].record()
    torch.cuda.synchronize()
    lat = sorted(ev[s].elapsed_time(ev[s + 1]) for s in range(steps))
    out = {"p50_ms": lat[len(lat) // 2]}
    if profile:
        sled.sled_profile_enable(v.model, True)
        for _ in range(3):
            step()
        ms, n = sled.sled_profile_read(v.model)
        sled.sled_profile_enable(v.model, False)
        out["proj_ms"] = ms[sled.PROF_PROJ] / 3
        out["attn_ms"] = ms[sled.PROF_ATTN] / 3
    return out


def batch_sweep(seed=0):
    shape = synth.SHAPES["llama8b"]
    weights = synth.SynthWeights(shape, seed=seed, device="cuda")
    rng = np.random.default_rng(seed)
    ctx_all = rng.integers(512, 2049, size=64).tolist()
    print(f"{'B':>3s} {'k':>2s} {'T':>4s} {'ctx tokens':>10s} {'p50 ms':>8s} {'verified draft tok/s':>21s} {'HBM frac':>9s}")
    for B in (1, 2, 4, 8, 16, 32, 64):
        ctx = ctx_all[:B]
        budget = sum(ctx) + B * 9 * 16
        v = Verifier(shape, weights, budget // 16 + 2 * B + 8, B, B, budget)
        reqs = [v.open() for _ in range(B)]
        for i in range(B):
            K, V = synth.context_kv(shape, ctx[i], seed=seed, req=i, device="cuda")
            v.append_context([reqs[i]], [K], [V])
        for k1 in (2, 4, 8):
            k = [k1] * B
            T = B * (k1 + 1)
            tokens = torch.from_numpy(rng.integers(0, shape.vocab, size=T).astype(np.int32)).cuda()
            r = _time_steps(v, reqs, k, tokens)
            lens = v.lengths(reqs)
            step_bytes = shape.streamed_params() * 2 + sum(lens) * shape.kv_bytes_per_token() + T * shape.vocab * 4
            print(f"{B:3d} {k1:2d} {T:4d} {sum(lens):10d} {r['p50_ms']:8.3f} {B * k1 / (r['p50_ms'] * 1e-3):21.0f} "
                  f"{step_bytes / (r['p50_ms'] * 1e-3) / 8e12:9.3f}")
        v.destroy()


def rows_sweep(seed=0, sizes=(128, 256, 512, 1024, 2048, 4096), kind="llama8b"):
    shape = synth.SHAPES[kind]
    weights = synth.SynthWeights(shape, seed=seed, device="cuda")
    rng = np.random.default_rng(seed)
    flop_per_row = 2.0 * shape.streamed_params()
    print(f"{'rows':>5s} {'p50 ms':>8s} {'proj ms':>8s} {'useful TFLOP/s':>15s} {'of bf16 MFMA peak':>18s} {'weight GB/s':>12s}")
    for T in sizes:
        B = (T + 8) // 9
        k = [8] * B
        k[-1] = T - 9 * (B - 1) - 1
        if k[-1] < 0:
            B -= 1
            k = [8] * B
        T_real = sum(k) + B
        ctx = [16] * B
        budget = sum(ctx) + B * 9 * 16
        v = Verifier(shape, weights, budget // 16 + 2 * B + 8, B, B, budget)
        reqs = [v.open() for _ in range(B)]
        K, V = synth.context_kv(shape, 16, seed=seed, req=0, device="cuda")
        for i in range(B):
            v.append_context([reqs[i]], [K], [V])
        tokens = torch.from_numpy(rng.integers(0, shape.vocab, size=T_real).astype(np.int32)).cuda()
        r = _time_steps(v, reqs, k, tokens, steps=4, warmup=1, profile=True)
        tf = flop_per_row * T_real / (r["proj_ms"] * 1e-3)
        print(f"{T_real:5d} {r['p50_ms']:8.3f} {r['proj_ms']:8.3f} {tf / 1e12:15.1f} {tf / MFMA_PEAK_BF16:18.3f} "
              f"{shape.streamed_params() * 2 / (r['proj_ms'] * 1e-3) / 1e9:12.0f}")
        v.destroy()


def prefill_sweep(seed=0):
    """Prompt ingest through sled_prefill, Llama-3-8B shape: prompt length x rows per slice."""
    shape = synth.SHAPES["llama8b"]
    weights = synth.SynthWeights(shape, seed=seed, device="cuda")
    rng = np.random.default_rng(seed)
    per = shape.k_max + 1
    print(f"{'prompt':>7s} {'rows/slice':>11s} {'ms':>9s} {'tokens/s':>10s} {'useful TFLOP/s':>15s} {'of bf16 MFMA peak':>18s}")
    for blocks in (14, 56, 112, 224):
        for n in (1024, 4096):
            budget = n + 64
            v = Verifier(shape, weights, budget // 16 + 8, 1, blocks, budget)
            r = v.open()
            toks = torch.from_numpy(rng.integers(0, shape.vocab, size=n).astype(np.int32)).cuda()
            v.prefill(r, toks[:per])                      # warm-up of the kernels, then a fresh session
            v.close_request(r)
            r = v.open()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            v.prefill(r, toks)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            # projections: 2 x streamed parameters per token (the LM head runs for one row only);
            # attention: QK^T and PV over the causal triangle, 2 x 2 x d_model x n^2 / 2 per layer
            flop = 2.0 * (shape.streamed_params() - shape.vocab * shape.d_model) * n + \
                2.0 * shape.n_layers * shape.n_q_heads * shape.head_dim * float(n) * n
            print(f"{n:7d} {blocks * per:11d} {dt * 1e3:9.2f} {n / dt:10.0f} {flop / dt / 1e12:15.1f} {flop / dt / MFMA_PEAK_BF16:18.3f}",
                  flush=True)
            v.destroy()


def weights_sweep(seed=0):
    """The verify step with bf16, 8-bit (FP8 E4M3 + per-row scale) and 4-bit (FP4 E2M1 + block scale) weights, Llama-3-8B shape,
    1024 context tokens per request: where halving the weight stream pays (few packed rows) and
    where the projections are no longer bound by it (a hundred rows)."""
    shape = synth.SHAPES["llama8b"]
    cases = ((1, 4), (4, 4), (8, 3), (16, 5), (16, 7))
    res = {}
    for name, cls in (("bf16", synth.SynthWeights), ("fp8", synth.SynthWeightsW8), ("fp4", synth.SynthWeightsW4)):
        weights = cls(shape, seed=seed, device="cuda")
        K, V = synth.context_kv(shape, 1024, seed=seed, req=0, device="cuda")
        for B, k1 in cases:
            budget = B * 1024 + B * 9 * 40
            v = Verifier(shape, weights, budget // 16 + 2 * B + 8, B, B, budget)
            reqs = [v.open() for _ in range(B)]
            for r in reqs:
                v.append_context([r], [K], [V])
            tokens = torch.randint(0, shape.vocab, (B * (k1 + 1),), dtype=torch.int32, device="cuda")
            res[name, B, k1] = _time_steps(v, reqs, [k1] * B, tokens, steps=12, warmup=3, profile=True)
            v.destroy()
        del weights
    print(f"{'B':>3s} {'k':>2s} {'rows':>5s} | step ms: {'bf16':>7s} {'fp8':>7s} {'fp4':>7s} | projections ms: {'bf16':>7s} {'fp8':>7s} {'fp4':>7s} | "
          f"step vs bf16: {'fp8':>6s} {'fp4':>6s}")
    for B, k1 in cases:
        a, b, c = res["bf16", B, k1], res["fp8", B, k1], res["fp4", B, k1]
        print(f"{B:3d} {k1:2d} {B * (k1 + 1):5d} |          {a['p50_ms']:7.3f} {b['p50_ms']:7.3f} {c['p50_ms']:7.3f} |                 "
              f"{a['proj_ms']:7.3f} {b['proj_ms']:7.3f} {c['proj_ms']:7.3f} |               {b['p50_ms'] / a['p50_ms']:6.3f} {c['p50_ms'] / a['p50_ms']:6.3f}")


if __name__ == "__main__":
    which = sys.argv[1] if len(sys.argv) > 1 else ""
    if which not in ("batch", "rows", "prefill", "weights"):
        print(__doc__)
        sys.exit(0 if which in ("-h", "--help") else 2)
    sled.lib()
    torch.cuda.set_device(0)
    if which == "batch":
        batch_sweep()
    elif which == "rows":
        # optional shape name and list of row counts, e.g. `rows 1024` for a counter run over one size, `rows llama70b`
        args = sys.argv[2:]
        kind = args.pop(0) if args and args[0] in synth.SHAPES else "llama8b"
        rows_sweep(sizes=tuple(int(a) for a in args) or (128, 256, 512, 1024, 2048, 4096), kind=kind)
    elif which == "prefill":
        prefill_sweep()
    else:
        weights_sweep()
