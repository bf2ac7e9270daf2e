"""Shared pieces of the GPU parity tests: run the HIP library through its C ABI and the CPU oracle
on the same seeded inputs and compare."""
from __future__ import annotations

import numpy as np
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import sled, synth
from paper_2506_09397_amd.runtime import Verifier
from helpers import oracle_model, oracle_requests  # noqa: F401

# Decisions whose oracle margin is below these bounds may legitimately differ by the ~1e-15 relative round-off of
# float64 sums taken in different orders (an accept test whose two sides agree to four digits is decided with a
# float64 normaliser in the library too; the inverse-CDF draw always is); everything else must match bit for bit.
MARGIN_ACC = 1e-11
MARGIN_CDF = 1e-11
MARGIN_ARGMAX = 0.0


def run_accept_gpu(mode, case: synth.AcceptCase, vocab: int, temperature: float = 1.0):
    B, T = len(case.k), sum(case.k) + len(case.k)
    ws = sled.workspace(sled.sled_accept_workspace_bytes(B, T, vocab))
    a = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    t = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    sled.sled_accept(mode, case.k, vocab, temperature, case.logits, case.tokens,
                     case.q if mode == sled.SAMPLE else None, case.u_acc if mode == sled.SAMPLE else None,
                     case.u_smp if mode == sled.SAMPLE else None, a, t, ws)
    torch.cuda.synchronize()
    return a.cpu().numpy(), t.cpu().numpy()


def oracle_accept(mode, case: synth.AcceptCase, temperature: float = 1.0):
    name = "greedy" if mode == sled.GREEDY else "sample"
    temperature = float(np.float32(temperature))    # the C entry point takes a float32: both sides divide by that number
    return O.accept_batch(name, case.k, synth.as_f64(case.logits), case.tokens.cpu().numpy(),
                          synth.as_f64(case.q) if mode == sled.SAMPLE else None,
                          synth.as_f64(case.u_acc) if mode == sled.SAMPLE else None,
                          synth.as_f64(case.u_smp) if mode == sled.SAMPLE else None, temperature)


def compare_accept(mode, k, got_a, got_t, want, label=""):
    """Bit-exact on every decision with a safe margin; counts the others and checks they are valid."""
    n_sub = 0
    for i, w in enumerate(want):
        if mode == sled.GREEDY:
            safe = w["margin"] > MARGIN_ARGMAX
        else:
            safe = w["margin_acc"] > MARGIN_ACC and w["margin_cdf"] > MARGIN_CDF
        if safe:
            assert (int(got_a[i]), int(got_t[i])) == (w["accept_len"], w["out_token"]), \
                f"{label} request {i}: gpu ({got_a[i]}, {got_t[i]}) oracle ({w['accept_len']}, {w['out_token']})"
        else:
            n_sub += 1
            assert 0 <= got_a[i] <= k[i]
    return n_sub


def build_verifier(shape: synth.ModelShape, weights_seed: int, n_pages: int, max_requests: int, B_max: int,
                   ctx_tokens_max: int, gain_jitter: float = 0.0, std: float = 0.02):
    """Weights are drawn on the GPU; the same object (same seed, same device) later feeds the oracle."""
    w = synth.SynthWeights(shape, seed=weights_seed, device="cuda", std=std, gain_jitter=gain_jitter)
    v = Verifier(shape, w, n_pages, max_requests, B_max, ctx_tokens_max)
    return v, w
