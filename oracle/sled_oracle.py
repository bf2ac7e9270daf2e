"""CPU oracle for the server-side batched verification step of SLED (arXiv 2506.09397).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
library is checked against.  It shares no code with the HIP path, is never imported
by the product package, and must not be used to produce product results.

What it computes, per verification request (Sec. 3.2: a request is the device's
context plus its draft tokens; the answer is the rejected position and a corrective
token):

  1. the target model's logits for the request's k+1 query tokens
     [pending, draft_1 .. draft_k], all scored by a single forward pass (Sec. 3.1)
     on top of the request's cached context K/V -- forward_rows() / verify_batch();
  2. the acceptance decision of Eq. 1 (Sec. 3.1): accept draft x with probability
     min(1, p_target(x) / p_draft(x)), on failure resample from the normalised
     positive part of p_target - p_draft -- accept_sample(); and its deterministic
     counterpart, exact match against the target's argmax chain -- accept_greedy().

Requests are processed one at a time; there is no padding, packing, paging, tiling,
or online softmax here (Sec. 3.4's padded batch is result-identical to this because
padded positions are masked out).  All arithmetic is float64.  numpy's matmul,
exp, cumsum and argmax serve as library steps.

The target model is a LLaMA-family decoder (Sec. 4): pre-norm, RMSNorm, rotary
position embedding with the half-split pairing (i, i + D/2) used by the public
LLaMA implementations, grouped-query attention (query head h reads kv head
h // group), SwiGLU MLP, no biases, untied LM head.

Storage option (round_points).  All sums, the softmax, the residual stream and the
logits are float64 in every mode.
  "exact"     rounds nothing (weights and given context K/V are bf16 values already).
  "kv_bf16"   the definition for a model whose K/V cache is bf16 (what parity of a
              SLED_BF16 model is judged against): exact arithmetic, except that K and V
              of the new tokens are rounded to bf16 (nearest, ties to even) when they
              enter the cache -- the cache of such a model holds bf16 numbers, so every
              later key/value read sees the rounded value.  Nothing else is rounded.
Storage-contract studies, NOT used for parity ("parity unpinned" for these three; they
exist to measure what an activation format would cost, see tests/test_oracle_forward.py
for the bound that ties them to "kv_bf16"):
  "bf16x2"    as "kv_bf16", and every other activation between operators (normalised
              activations, q, softmax numerators, attention output, SwiGLU product) kept as a
              PAIR of bf16 numbers hi + lo (about 16 significant bits)
  "bf16"      ... as a single bf16 number
  "fp16"      ... as a single IEEE half (11 significant bits)

Pins (tests/test_oracle_*.py, no GPU): Hugging Face's LlamaForCausalLM in float64
for the forward; closed forms, brute force over the uniforms, chi-square
distribution preservation and invariants for acceptance; greedy verify loop equals
plain autoregressive decoding.  Whole-step values on the 8B/70B-shaped random models
have no external reference: "parity unpinned" beyond those properties.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

LOG2E = 1.4426950408889634


# --------------------------------------------------------------------------- rounding
def bf16_round(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (ties to even) of each element, returned as float64."""
    x32 = np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))
    u = x32.reshape(-1).view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = u.astype(np.uint32).view(np.float32).astype(np.float64)
    return out.reshape(x32.shape)


def bf16x2_round(x: np.ndarray) -> np.ndarray:
    """Value kept as a pair of bfloat16 numbers hi + lo: hi = bf16(x), lo = bf16(x - hi)."""
    hi = bf16_round(x)
    return hi + bf16_round(np.asarray(x, dtype=np.float64) - hi)


def fp16_round(x: np.ndarray) -> np.ndarray:
    """Nearest IEEE half of each element, returned as float64 (study mode only)."""
    return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


STUDY_MODES = ("bf16x2", "bf16", "fp16")


def _rounder(round_points: str, cached: bool = False):
    """Storage rounding of an activation.  `cached` marks K and V of the new tokens, which enter a
    bf16 cache as single bf16 numbers in every mode but "exact"; the other activations are rounded
    only by the storage-contract study modes."""
    if round_points == "exact":
        return lambda a: a
    if cached:
        return bf16_round
    if round_points == "kv_bf16":
        return lambda a: a
    if round_points == "bf16":
        return bf16_round
    if round_points == "bf16x2":
        return bf16x2_round
    if round_points == "fp16":
        return fp16_round
    raise ValueError(round_points)


# --------------------------------------------------------------------------- operators
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * gain / sqrt(mean(x^2) + eps) along the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding of x[n, H, D] at integer positions[n].

    Pair (i, i + D/2), i < D/2, is rotated by the angle pos * theta**(-2i/D)."""
    D = x.shape[-1]
    half = D // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def attention_rows(q: np.ndarray, K: np.ndarray, V: np.ndarray, n_ctx: int, group: int,
                   round_points: str = "exact") -> np.ndarray:
    """Attention of n query rows that sit at positions n_ctx .. n_ctx+n-1.

    q[n, Hq, D]; K, V[n_ctx + n, Hkv, D] (context keys first, then the n new keys).
    Row j attends to keys 0 .. n_ctx + j: the whole context and the new keys up to
    itself.  Scores are scaled by 1/sqrt(D).  Returns [n, Hq, D].

    Storage-contract study modes only: the softmax numerators that multiply V are stored
    rounded.  They are taken relative to a power of two, p = 2^(t - M) with t the score in
    log2 units and M the smallest whole number >= max t, because only then is their rounding
    independent of the reference (scaling by 2^n commutes with rounding).  The denominator
    sums the unrounded numerators."""
    n, Hq, D = q.shape
    out = np.empty_like(q)
    scale = 1.0 / math.sqrt(D)
    for h in range(Hq):
        g = h // group
        for j in range(n):
            m = n_ctx + j + 1
            s = (K[:m, g, :] @ q[j, h, :]) * scale
            if round_points not in STUDY_MODES:
                p = np.exp(s - s.max())
                out[j, h, :] = (p @ V[:m, g, :]) / p.sum()
            else:
                t = s * LOG2E
                p = np.exp2(t - math.ceil(t.max()))
                out[j, h, :] = (_rounder(round_points)(p) @ V[:m, g, :]) / p.sum()
    return out


# --------------------------------------------------------------------------- forward
class OracleModel:
    """Float64 view of a model: shape constants plus accessors returning numpy arrays.

    `weights` is any object with embed() -> [V,d], layer(l) -> dict(wq,wk,wv,wo,wg,wu,wd,
    g_attn,g_mlp) and final() -> dict(g_final, lm_head); linear weights are
    [out_features, in_features].  Layers are fetched one at a time so a large model
    never has to be resident in float64."""

    def __init__(self, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
                 rope_theta, rms_eps, weights, round_points="exact"):
        self.n_layers, self.d_model = n_layers, d_model
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.d_ffn, self.vocab = d_ffn, vocab
        self.rope_theta, self.rms_eps = rope_theta, rms_eps
        self.weights = weights
        self.round_points = round_points
        self.group = n_q_heads // n_kv_heads


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 numbers at the magnitude of x (8 significant bits); that of the smallest normal for x = 0."""
    a = np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)
    return np.ldexp(1.0, np.floor(np.log2(a)).astype(np.int64) - 7)


def layer_rows(model: OracleModel, W: Dict[str, np.ndarray], h: np.ndarray, positions: np.ndarray,
               K_ctx: np.ndarray, V_ctx: np.ndarray, stored: Optional[Tuple[np.ndarray, np.ndarray]] = None,
               audit: Optional[dict] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One decoder layer for the n rows of one request.

    h[n, d] residual stream in; K_ctx, V_ctx[n_ctx, Hkv, D] this layer's cached context
    (K already rotated).  Returns (h_out, k_new[n,Hkv,D] rotated, v_new[n,Hkv,D]).

    stored = (k, v)[n, Hkv, D], bf16 numbers: what a cache under test holds for the new rows.  Rounding to the cache
    is a decision a floating-point value takes, and a value that lies within round-off of the midpoint of two bf16
    numbers may go either way; a single such flip is a whole bf16 step and, twenty layers on, moves logits by more
    than any tolerance.  With `stored` the decision is taken as the cache under test took it: the layer attends to
    the stored numbers, and `audit` records how good they are as roundings of the exactly computed values:
    "max_excess" = the largest |stored - exact| - half a bf16 step at exact, in units of the root mean square of the
    element's head vector (0 or less: a correct rounding of the exact value itself; e: a correct rounding of a value
    within e * rms of it), and "flips" = how many differ from the oracle's own rounding, of "elements" -- for the
    caller to bound."""
    R, RC = _rounder(model.round_points), _rounder(model.round_points, cached=True)
    n = h.shape[0]
    Hq, Hkv, D = model.n_q_heads, model.n_kv_heads, model.head_dim
    x = R(rmsnorm(h, W["g_attn"], model.rms_eps))
    q = (x @ W["wq"].T).reshape(n, Hq, D)
    k = (x @ W["wk"].T).reshape(n, Hkv, D)
    v = (x @ W["wv"].T).reshape(n, Hkv, D)
    q = R(rope(q, positions, model.rope_theta))
    k = rope(k, positions, model.rope_theta)
    if stored is None:
        k, v = RC(k), RC(v)
    else:
        for name, exact, given in (("k", k, stored[0]), ("v", v, stored[1])):
            given = np.asarray(given, dtype=np.float64)
            if audit is not None:
                rms = np.sqrt((exact * exact).mean(axis=-1, keepdims=True))
                excess = (np.abs(given - exact) - 0.5 * bf16_ulp(exact)) / np.maximum(rms, 1e-300)
                audit["max_excess"] = max(audit.get("max_excess", -math.inf), float(excess.max()))
                audit["flips"] = audit.get("flips", 0) + int((given != bf16_round(exact)).sum())
                audit["elements"] = audit.get("elements", 0) + given.size
        k, v = np.asarray(stored[0], dtype=np.float64), np.asarray(stored[1], dtype=np.float64)
    K_all = np.concatenate([K_ctx, k], axis=0)
    V_all = np.concatenate([V_ctx, v], axis=0)
    o = R(attention_rows(q, K_all, V_all, K_ctx.shape[0], model.group, model.round_points)).reshape(n, Hq * D)
    h = h + o @ W["wo"].T
    x = R(rmsnorm(h, W["g_mlp"], model.rms_eps))
    a = R(silu(x @ W["wg"].T) * (x @ W["wu"].T))
    h = h + a @ W["wd"].T
    return h, k, v


def verify_batch(model: OracleModel, requests: Sequence[dict], progress=None) -> List[dict]:
    """Score every request's tokens on top of its own cached context.

    requests[i] = {"tokens": int[n_i] = [pending, draft_1..draft_k],
                   "K": [n_layers, L_i, Hkv, D], "V": same}   (L_i may be 0);
                  optionally "K_stored", "V_stored": [n_layers, n_i, Hkv, D], the bf16 numbers a cache under test
                  holds for the new rows (see layer_rows); the result then carries "audit".
    The n_i tokens sit at positions L_i .. L_i + n_i - 1.  Logits row j is the target
    distribution of the token that follows tokens[j].
    Returns per request {"logits": [n_i, V], "K_new": [n_layers, n_i, Hkv, D], "V_new": same}.
    Requests never interact: the loop over requests is the definition of the batch.
    progress(l), if given, is called after layer l (long runs report where they are; no effect on any value)."""
    E = model.weights.embed()
    hs, pos = [], []
    for r in requests:
        toks = np.asarray(r["tokens"], dtype=np.int64)
        L = r["K"].shape[1]
        hs.append(E[toks].astype(np.float64))
        pos.append(np.arange(L, L + len(toks)))
    del E
    Knew = [np.empty((model.n_layers, len(r["tokens"]), model.n_kv_heads, model.head_dim)) for r in requests]
    Vnew = [np.empty_like(a) for a in Knew]
    audits = [{} if "K_stored" in r else None for r in requests]
    for l in range(model.n_layers):
        W = model.weights.layer(l)
        for i, r in enumerate(requests):
            st = (r["K_stored"][l], r["V_stored"][l]) if audits[i] is not None else None
            hs[i], Knew[i][l], Vnew[i][l] = layer_rows(model, W, hs[i], pos[i], r["K"][l], r["V"][l], st, audits[i])
        del W
        if progress is not None:
            progress(l)
    F = model.weights.final()
    R = _rounder(model.round_points)
    out = []
    for i in range(len(requests)):
        x = R(rmsnorm(hs[i], F["g_final"], model.rms_eps))
        out.append({"logits": x @ F["lm_head"].T, "K_new": Knew[i], "V_new": Vnew[i]})
        if audits[i] is not None:
            out[-1]["audit"] = audits[i]
    return out


def empty_kv(model: OracleModel) -> Tuple[np.ndarray, np.ndarray]:
    z = np.zeros((model.n_layers, 0, model.n_kv_heads, model.head_dim))
    return z, z.copy()


def prefill(model: OracleModel, tokens: Sequence[int]) -> dict:
    """Textbook causal forward over a whole sequence with no cache: logits for every
    position and the K/V a cache would hold afterwards."""
    K0, V0 = empty_kv(model)
    r = verify_batch(model, [{"tokens": tokens, "K": K0, "V": V0}])[0]
    return {"logits": r["logits"], "K": r["K_new"], "V": r["V_new"]}


# --------------------------------------------------------------------------- acceptance
def softmax64(z: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    t = np.asarray(z, dtype=np.float64) / float(temperature)
    e = np.exp(t - t.max())
    return e / e.sum()


def argmax_lowest(z: np.ndarray) -> Tuple[int, float]:
    """Index of the largest entry, lowest index on ties; also the gap to the runner-up."""
    z = np.asarray(z, dtype=np.float64)
    best = int(np.argmax(z))  # numpy returns the first maximal index
    if z.size > 1:
        rest = np.delete(z, best)
        gap = float(z[best] - rest.max())
    else:
        gap = math.inf
    return best, gap


def inverse_cdf(w: np.ndarray, u: float) -> Tuple[int, float]:
    """Smallest index v whose inclusive prefix sum exceeds u * sum(w), scanning indices in
    ascending order; if round-off leaves none, the last index with positive weight.
    Also returns the distance from u*sum(w) to the nearest boundary of the chosen cell,
    relative to sum(w)."""
    C = np.cumsum(w)
    S = float(C[-1])
    target = float(u) * S
    hit = np.nonzero(C > target)[0]
    if hit.size:
        v = int(hit[0])
    else:
        v = int(np.nonzero(w > 0)[0][-1])
    lo = float(C[v - 1]) if v > 0 else 0.0
    margin = min(abs(target - lo), abs(float(C[v]) - target)) / S if S > 0 else 0.0
    return v, margin


def accept_greedy(logits: np.ndarray, drafts: Sequence[int]) -> dict:
    """Deterministic verification of one request.

    logits[k+1, V]; row j-1 judges draft j (1-based).  The accepted length is the number
    of leading drafts equal to the argmax of their judging row; the emitted token is the
    argmax of the first row whose draft failed, or of the last row when all passed."""
    k = len(drafts)
    a, gaps = 0, []
    for j in range(k):
        t, gap = argmax_lowest(logits[j])
        gaps.append(gap)
        if int(drafts[j]) != t:
            return {"accept_len": j, "out_token": t, "margin": min(gaps)}
        a = j + 1
    t, gap = argmax_lowest(logits[k])
    gaps.append(gap)
    return {"accept_len": a, "out_token": t, "margin": min(gaps)}


def accept_sample(logits: np.ndarray, drafts: Sequence[int], q: np.ndarray, u_acc: Sequence[float],
                  u_smp: float, temperature: float = 1.0) -> dict:
    """Speculative-sampling verification of one request (Eq. 1, Sec. 3.1).

    logits[k+1, V]; q[k, V] draft probabilities; draft j (0-based) is judged by row j:
    with p = softmax(logits[j] / temperature) it is accepted iff u_acc[j] * q[j, d] <= p[d],
    i.e. with probability min(1, p(d)/q(d)).  At the first rejection the emitted token is
    drawn by inverse CDF with u_smp from max(0, p - q[j]) normalised (from p itself if that
    residual has no mass); if nothing is rejected a bonus token is drawn from row k.
    A draft id outside [0, V) has target probability 0 and is rejected where it stands.
    margin_acc: smallest |u q - p| / p over the tests taken; margin_cdf: see inverse_cdf."""
    k = len(drafts)
    V = logits.shape[1]
    margin_acc = math.inf
    for j in range(k):
        p = softmax64(logits[j], temperature)
        d = int(drafts[j])
        inside = 0 <= d < V
        if inside:
            lhs = float(u_acc[j]) * float(q[j, d])
            pd = float(p[d])
            margin_acc = min(margin_acc, abs(lhs - pd) / max(pd, 1e-300))
        if not inside or not (lhs <= pd):
            r = np.maximum(0.0, p - np.asarray(q[j], dtype=np.float64))
            if r.sum() <= 0.0:
                r = p
            v, mc = inverse_cdf(r, u_smp)
            return {"accept_len": j, "out_token": v, "margin_acc": margin_acc, "margin_cdf": mc}
    p = softmax64(logits[k], temperature)
    v, mc = inverse_cdf(p, u_smp)
    return {"accept_len": k, "out_token": v, "margin_acc": margin_acc, "margin_cdf": mc}


def accept_batch(mode: str, k: Sequence[int], logits: np.ndarray, tokens: np.ndarray,
                 q: Optional[np.ndarray] = None, u_acc: Optional[np.ndarray] = None,
                 u_smp: Optional[np.ndarray] = None, temperature: float = 1.0) -> List[dict]:
    """Acceptance for a packed batch: logits[T, V] and tokens[T] hold k_i+1 rows per request in
    request order; q[sum k, V] and u_acc[sum k] hold one row per draft in the same order."""
    out, row, dr = [], 0, 0
    for i, ki in enumerate(k):
        lg = logits[row: row + ki + 1]
        drafts = tokens[row + 1: row + 1 + ki]
        if mode == "greedy":
            out.append(accept_greedy(lg, drafts))
        elif mode == "sample":
            out.append(accept_sample(lg, drafts, q[dr: dr + ki], u_acc[dr: dr + ki], u_smp[i], temperature))
        else:
            raise ValueError(mode)
        row += ki + 1
        dr += ki
    return out


def row_confidence(logits: np.ndarray, temperature: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """Confidence score of every row (Eq. 2 compares it with the threshold c_th): the probability that
    softmax(logits / temperature) gives its most likely token, and that token (lowest id among ties)."""
    conf = np.empty(logits.shape[0], dtype=np.float64)
    top = np.empty(logits.shape[0], dtype=np.int64)
    for r in range(logits.shape[0]):
        p = softmax64(logits[r], temperature)
        top[r], _ = argmax_lowest(logits[r])
        conf[r] = p[top[r]]
    return conf, top


# --------------------------------------------------------------------------- decoding loops
def decode_greedy(model: OracleModel, prompt: Sequence[int], n_new: int) -> List[int]:
    """Plain autoregressive greedy decoding with a cache: one token per forward."""
    pf = prefill(model, prompt[:-1]) if len(prompt) > 1 else None
    K, V = (pf["K"], pf["V"]) if pf else empty_kv(model)
    pending, out = int(prompt[-1]), []
    for _ in range(n_new):
        r = verify_batch(model, [{"tokens": [pending], "K": K, "V": V}])[0]
        t, _ = argmax_lowest(r["logits"][0])
        K = np.concatenate([K, r["K_new"]], axis=1)
        V = np.concatenate([V, r["V_new"]], axis=1)
        out.append(t)
        pending = t
    return out


def speculative_greedy(model: OracleModel, prompt: Sequence[int], n_new: int, drafter) -> Tuple[List[int], List[int]]:
    """Draft -> verify -> commit loop (Sec. 3.2) with deterministic verification.

    drafter(history) -> list of draft tokens (any length >= 0).  After each verification the
    pending token and the accepted drafts enter the cache and the emitted token becomes the
    next pending token.  Returns (generated tokens, accepted lengths per round)."""
    pf = prefill(model, prompt[:-1]) if len(prompt) > 1 else None
    K, V = (pf["K"], pf["V"]) if pf else empty_kv(model)
    pending, out, acc = int(prompt[-1]), [], []
    hist = list(prompt)
    while len(out) < n_new:
        drafts = [int(t) for t in drafter(hist)]
        r = verify_batch(model, [{"tokens": [pending] + drafts, "K": K, "V": V}])[0]
        res = accept_greedy(r["logits"], drafts)
        a = res["accept_len"]
        K = np.concatenate([K, r["K_new"][:, : a + 1]], axis=1)
        V = np.concatenate([V, r["V_new"][:, : a + 1]], axis=1)
        new = drafts[:a] + [res["out_token"]]
        out += new
        hist += new
        acc.append(a)
        pending = res["out_token"]
    return out[:n_new], acc
