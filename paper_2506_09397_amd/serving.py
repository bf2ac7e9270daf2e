"""Serving loop around the verification step: request queue, static batch planner and the
multi-round draft -> verify -> accept -> commit cycle of many devices (Sec. 3.2, Sec. 3.4), plus an
event-driven simulation of Poisson device traffic (Sec. 4) that reports a whole-system token
generation rate.

Host-side orchestration only: every number that reaches a device comes out of sled_verify_batch,
sled_accept and sled_kv_append.  The pieces:

  Server          one model + K/V pool on one GPU.  `submit` queues a verification request
                  (device id, round number, pending token, draft tokens); `run_batch` takes up to
                  `batch_size` queued requests in arrival order (static batching, Sec. 3.4; the ragged
                  pack replaces the paper's padding), runs the three calls and returns one response
                  per request: (accepted length, correction or bonus token).  A device whose answer
                  got lost re-sends its round (Sec. 3.3, the device-side timer): the server recognises
                  the round number and answers from its record instead of verifying twice, so the
                  committed context never runs ahead of what the device knows.
  ReplayDrafter   stands in for a device's draft model: it knows the target's greedy continuation
                  of its prompt (computed beforehand, one token per step, through the same server)
                  and corrupts each draft token with probability 1 - beta, which sets the acceptance
                  rate.  Whatever it drafts, the text the device ends up with is the target's own
                  greedy text: verification is lossless (Sec. 3.1).  (It equals the precomputed
                  continuation token for token unless two logits tie to within the round-off that
                  separates two batchings of the same request; the tiny-model tests demand equality.)
  SamplingDrafter stands in for a device that drafts by sampling: every draft comes with the distribution it was
                  drawn from (dense, or its top entries as (id, probability) pairs), which is what the server's
                  sampling mode (Eq. 1, seeded uniforms per device and round) verifies against.
  simulate        devices draft for an exponentially distributed time (mean k x per-token draft
                  time), queue at the server, wait for the batch to fill, get their answer after the
                  measured GPU time of the step; virtual clock, real GPU work.

    python -m paper_2506_09397_amd.serving --shape llama8b --devices 32 --batch 16 --k 6 --beta 0.8 --tokens 64
"""
from __future__ import annotations

import argparse
import collections
import dataclasses
import heapq
import json
import time
from typing import Deque, Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import sled, synth
from .runtime import Verifier


@dataclasses.dataclass
class Pending:
    device: int
    round_no: int
    pending_token: int
    drafts: List[int]
    # speculative sampling only: the distributions the drafts were drawn from, one row per draft -- dense
    # float32 [k, vocab], or sparse as (token ids int32 [k, m], probabilities float32 [k, m]); on the GPU
    q: Optional[object] = None


@dataclasses.dataclass
class Response:
    device: int
    round_no: int
    accept_len: int
    out_token: int
    replayed: bool = False   # answered from the record of an earlier, lost answer


class Server:
    """Queue + static batch planner + the verification step for a set of devices."""

    def __init__(self, verifier: Verifier, batch_size: int, device: str = "cuda", mode: str = "greedy",
                 temperature: float = 1.0, seed: int = 0):
        """mode "greedy": exact match against the target's argmax chain.  mode "sample": speculative sampling
        (Eq. 1): every request carries the distributions its drafts were drawn from, and the uniforms of a round
        are a function of (seed, device, round number) alone, so an answer does not depend on how the round
        was batched and a retried round draws the same numbers."""
        assert mode in ("greedy", "sample")
        self.v = verifier
        self.batch_size = batch_size
        self.device = device        # where the packed token ids of a step are put
        self.mode = mode
        self.temperature = float(temperature)
        self.seed = int(seed)
        self.observer = None        # called with everything a step consumed and produced (tests, tracing)
        self.queue: Deque[Pending] = collections.deque()
        self.req_of: Dict[int, int] = {}              # device -> request id in the pool
        self.last: Dict[int, Response] = {}           # device -> answer of its latest verified round
        self.steps = 0
        self.rows = 0
        self.drafts_seen = 0

    # ---- sessions ---------------------------------------------------------------------------
    def open(self, device: int, K: Optional[torch.Tensor] = None, V: Optional[torch.Tensor] = None,
             prompt: Optional[Sequence[int]] = None) -> None:
        """Start a session with the context the device already has (everything before its pending token): either
        its K/V ([layers, tokens, kv heads, head dim], model dtype, on the GPU), or the prompt tokens themselves,
        which then run through the target model into the cache (sled_prefill)."""
        assert device not in self.req_of
        r = self.v.open()
        self.req_of[device] = r
        if K is not None and K.shape[1] > 0:
            self.v.append_context([r], [K], [V])
        if prompt is not None and len(prompt) > 0:
            self.v.prefill(r, torch.tensor([int(t) for t in prompt], dtype=torch.int32, device=self.device), want_logits=False)

    def close(self, device: int) -> None:
        self.v.close_request(self.req_of.pop(device))
        self.last.pop(device, None)
        self.queue = collections.deque(p for p in self.queue if p.device != device)

    # ---- requests ---------------------------------------------------------------------------
    def submit(self, device: int, round_no: int, pending_token: int, drafts: Sequence[int], q=None) -> Optional[Response]:
        """Queue a verification request.  A round the server has already verified (the device did not get the
        answer and sent it again, possibly with more drafts) is answered at once from the record.  In sampling
        mode q holds the draft distributions (see Pending)."""
        last = self.last.get(device)
        if last is not None and round_no <= last.round_no:
            if round_no < last.round_no:
                raise ValueError(f"device {device}: round {round_no} is older than the last answered round {last.round_no}")
            return dataclasses.replace(last, replayed=True)
        if len(drafts) > self.v.shape.k_max:
            drafts = drafts[: self.v.shape.k_max]   # the rest is drafted again next round
        if self.mode == "sample":
            if len(drafts) and q is None:
                raise ValueError("sampling mode: a request with drafts needs their distributions q")
            if q is not None:
                q = tuple(x[: len(drafts)] for x in q) if isinstance(q, tuple) else q[: len(drafts)]
        self.queue.append(Pending(device, round_no, int(pending_token), [int(d) for d in drafts], q if self.mode == "sample" else None))
        return None

    def round_uniforms(self, device: int, round_no: int, k: int) -> Tuple[np.ndarray, float]:
        """The uniforms of one round: k for the accept tests, one for the resample / bonus draw (float32 values)."""
        u = np.random.default_rng([self.seed, int(device), int(round_no)]).random(k + 1, dtype=np.float32)
        return u[:k], float(u[k])

    def ready(self) -> bool:
        return len(self.queue) >= self.batch_size

    def run_batch(self, allow_partial: bool = False) -> List[Response]:
        """One verification step over the oldest `batch_size` queued requests (fewer only if allow_partial)."""
        if not self.queue or (len(self.queue) < self.batch_size and not allow_partial):
            return []
        batch: List[Pending] = []
        seen = set()
        rest: Deque[Pending] = collections.deque()
        while self.queue and len(batch) < self.batch_size:
            p = self.queue.popleft()
            if p.device in seen:      # one row block per request and step: a second request of a device waits
                rest.append(p)
                continue
            seen.add(p.device)
            batch.append(p)
        self.queue.extendleft(reversed(rest))
        reqs = [self.req_of[p.device] for p in batch]
        k = [len(p.drafts) for p in batch]
        toks: List[int] = []
        for p in batch:
            toks += [p.pending_token] + p.drafts
        tokens = torch.tensor(toks, dtype=torch.int32, device=self.device)
        logits = self.v.verify(reqs, k, tokens)
        extra = {}
        if self.mode == "greedy":
            a, t = self.v.accept(sled.GREEDY, k, logits, tokens)
        else:
            us = [self.round_uniforms(p.device, p.round_no, len(p.drafts)) for p in batch]
            u_acc = torch.from_numpy(np.concatenate([u for u, _ in us]).astype(np.float32)).to(self.device)
            u_smp = torch.tensor([x for _, x in us], dtype=torch.float32, device=self.device)
            qs = [p.q for p in batch if len(p.drafts)]
            sparse = bool(qs) and isinstance(qs[0], tuple)
            assert all(isinstance(x, tuple) == sparse for x in qs), "one step takes dense or sparse draft distributions, not both"
            B = len(batch)
            if sparse:
                m = max(int(ids.shape[1]) for ids, _ in qs)
                pad = lambda x, fill: torch.nn.functional.pad(x, (0, m - x.shape[1]), value=fill)   # id -1 / probability 0: padding
                q_ids = torch.cat([pad(ids.to(torch.int32), -1) for ids, _ in qs]).contiguous()
                q_probs = torch.cat([pad(pr.to(torch.float32), 0.0) for _, pr in qs]).contiguous()
                sled.sled_accept_sparse(k, self.v.shape.vocab, self.temperature, logits, tokens, q_ids, q_probs, u_acc, u_smp,
                                        self.v.accept_len[:B], self.v.out_token[:B], self.v.acc_ws)
                a, t = self.v.accept_len[:B], self.v.out_token[:B]
                extra = {"q_ids": q_ids, "q_probs": q_probs}
            else:
                q = torch.cat(qs).contiguous() if qs else None
                a, t = self.v.accept(sled.SAMPLE, k, logits, tokens, q, u_acc, u_smp, temperature=self.temperature)
                extra = {"q": q}
            extra.update({"u_acc": u_acc, "u_smp": u_smp})
        self.v.commit(reqs, a)
        if self.observer is not None:
            self.observer(dict(batch=batch, k=k, tokens=tokens, logits=logits, accept_len=a, out_token=t, **extra))
        a_h, t_h = a.cpu().tolist(), t.cpu().tolist()     # the answers leave the GPU here
        # (the pool reserves pages for every staged row only until the exact lengths, which follow the commit back
        # to the host on their own, are picked up by its next call: nothing here waits for them)
        out = []
        for p, ai, ti in zip(batch, a_h, t_h):
            r = Response(p.device, p.round_no, int(ai), int(ti))
            self.last[p.device] = r
            out.append(r)
        self.steps += 1
        self.rows += len(toks)
        self.drafts_seen += sum(k)
        return out


class ReplayDrafter:
    """Draft tokens for a device whose target continuation is known: token j of a draft is the true next token
    with probability beta (as long as all earlier ones were), anything else afterwards."""

    def __init__(self, truth: Sequence[int], vocab: int, beta: float, seed: int):
        self.truth = list(truth)
        self.vocab = vocab
        self.beta = beta
        self.rng = np.random.default_rng(seed)

    def draft(self, n_done: int, k: int) -> List[int]:
        out: List[int] = []
        good = True
        for j in range(k):
            pos = n_done + j
            good = good and pos < len(self.truth) and self.rng.random() < self.beta
            if good:
                out.append(self.truth[pos])
            else:
                wrong = int(self.rng.integers(0, self.vocab))
                if pos < len(self.truth) and wrong == self.truth[pos]:
                    wrong = (wrong + 1) % self.vocab
                out.append(wrong)
        return out


class SamplingDrafter:
    """Stands in for a device that drafts by sampling: draft j of a round is drawn from a distribution
    q_j = softmax(noise-perturbed seeded logits) that depends on (device seed, number of tokens so far, j) only --
    not a language model, but all Eq. 1 asks of a drafter: each draft comes with the distribution it was drawn from.
    top > 0 keeps the `top` most likely tokens, renormalised, and hands q over sparsely as (ids, probabilities)."""

    truth = None

    def __init__(self, vocab: int, seed: int, device: str = "cuda", sharpness: float = 2.0, top: int = 0):
        self.vocab, self.seed, self.device, self.sharpness, self.top = vocab, seed, device, sharpness, top

    def draft_with_q(self, n_done: int, k: int):
        if k == 0:
            return [], None
        g = torch.Generator(device=self.device)
        g.manual_seed((self.seed * 1_000_003 + n_done * 101 + 7) % (2**31 - 1))
        z = self.sharpness * torch.randn(k, self.vocab, generator=g, device=self.device, dtype=torch.float32)
        q = torch.softmax(z, dim=-1)
        if self.top > 0:
            top = torch.topk(q, self.top, dim=1)
            probs = (top.values / top.values.sum(dim=1, keepdim=True)).float()
            pick = torch.multinomial(probs, 1, generator=g).squeeze(1)
            ids = top.indices.to(torch.int32)
            drafts = ids[torch.arange(k, device=self.device), pick]
            return [int(x) for x in drafts.cpu()], (ids.contiguous(), probs.contiguous())
        drafts = torch.multinomial(q, 1, generator=g).squeeze(1)
        return [int(x) for x in drafts.cpu()], q


def greedy_continuations(server: Server, devices: Sequence[int], first_tokens: Sequence[int], n_new: int) -> List[List[int]]:
    """The target's own continuation of every device's context, one token per step (k = 0 requests), all
    devices batched; the sessions are left where they started (closed and to be re-opened by the caller)."""
    out: List[List[int]] = [[] for _ in devices]
    pend = list(first_tokens)
    saved = server.batch_size
    server.batch_size = len(devices)
    for step in range(n_new):
        for i, d in enumerate(devices):
            server.submit(d, step, pend[i], [])
        for r in server.run_batch():
            i = devices.index(r.device)
            out[i].append(r.out_token)
            pend[i] = r.out_token
    server.batch_size = saved
    return out


def simulate(server: Server, drafters: Dict[int, ReplayDrafter], first_tokens: Dict[int, int], n_new: int, k: int,
             draft_ms_per_token: float, seed: int = 0, lose_every: int = 0) -> dict:
    """Event-driven run of all devices until each has n_new tokens.  Device cycle: draft (exponential time with
    mean k x draft_ms_per_token, the Poisson request model of Sec. 4), send, wait for the batch and the step, apply
    the answer.  The server starts a step when `batch_size` requests wait (or when fewer devices than that are
    still running).  `lose_every` > 0 drops every n-th answer on its way back; the device then sends the round
    again.  Returns the generated texts and the whole-system token rate on the virtual clock."""
    rng = np.random.default_rng(seed)
    texts: Dict[int, List[int]] = {d: [] for d in drafters}
    pend = dict(first_tokens)
    rounds = {d: 0 for d in drafters}
    events: List[Tuple[float, int, int]] = []     # (time, tie-breaker, device): device finishes drafting
    tie = 0
    for d in drafters:
        heapq.heappush(events, (rng.exponential(k * draft_ms_per_token), tie, d))
        tie += 1
    now = 0.0
    gpu_ms = 0.0
    answers = 0
    sent: Dict[int, Pending] = {}
    active = set(drafters)
    left_path = set()

    def send(d: int, t: float) -> None:
        nonlocal tie
        kk = min(k, max(0, n_new - len(texts[d]) - 1))
        if hasattr(drafters[d], "draft_with_q"):
            drafts, q = drafters[d].draft_with_q(len(texts[d]), kk)
        else:
            drafts, q = drafters[d].draft(len(texts[d]), kk), None
        sent[d] = Pending(d, rounds[d], pend[d], drafts, q)
        r = server.submit(d, rounds[d], pend[d], drafts, q)
        assert r is None

    def apply(r: Response, t: float) -> None:
        nonlocal tie
        d = r.device
        p = sent.pop(d)
        texts[d] += p.drafts[: r.accept_len] + [r.out_token]
        pend[d] = r.out_token
        rounds[d] += 1
        if drafters[d].truth is not None and texts[d] != drafters[d].truth[: len(texts[d])]:
            # the target took another path than the one the drafter replays (see main): the session ends here,
            # since a drafter that is always wrong would only add one-token rounds to the tail of the run
            left_path.add(d)
            active.discard(d)
        elif len(texts[d]) >= n_new:
            texts[d] = texts[d][:n_new]
            active.discard(d)
        else:
            heapq.heappush(events, (t + rng.exponential(k * draft_ms_per_token), tie, d))
            tie += 1

    while active:
        # deliver drafting completions up to the point where a batch can start
        while events and (not server.ready() and not (len(server.queue) >= len(active))):
            t, _, d = heapq.heappop(events)
            now = max(now, t)
            send(d, now)
        assert server.queue, "every running device is either drafting or queued"
        on_gpu = server.device != "cpu"
        if on_gpu:
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        resp = server.run_batch(allow_partial=True)
        if on_gpu:
            torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) * 1e3
        gpu_ms += dt
        now += dt
        for r in resp:
            answers += 1
            if lose_every and answers % lose_every == 0:
                # the answer is lost; the device's timer fires and it sends the same round again
                again = server.submit(r.device, r.round_no, sent[r.device].pending_token, sent[r.device].drafts, sent[r.device].q)
                assert again is not None and again.replayed and (again.accept_len, again.out_token) == (r.accept_len, r.out_token)
                r = again
            apply(r, now)
    total = sum(len(x) for x in texts.values())
    return {"texts": texts, "virtual_ms": now, "gpu_ms": gpu_ms, "steps": server.steps, "tokens": total,
            "tokens_per_s": total / (now * 1e-3), "tokens_per_gpu_s": total / (gpu_ms * 1e-3),
            "mean_rows_per_step": server.rows / max(server.steps, 1),
            "accepted_per_draft": (total - sum(rounds.values())) / max(server.drafts_seen, 1),
            "devices_off_replayed_path": len(left_path)}


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shape", default="llama8b", choices=sorted(synth.SHAPES))
    ap.add_argument("--layers", type=int, default=0, help="use only this many layers of the shape (0 = all)")
    ap.add_argument("--devices", type=int, default=32)
    ap.add_argument("--batch", type=int, default=16, help="static batch size of the planner")
    ap.add_argument("--k", type=int, default=6, help="draft tokens per request")
    ap.add_argument("--beta", type=float, default=0.8, help="probability that a draft token is the target's")
    ap.add_argument("--tokens", type=int, default=64, help="tokens to generate per device")
    ap.add_argument("--context", type=int, default=1024, help="mean context length (uniform in [c/2, 3c/2])")
    ap.add_argument("--draft-ms", type=float, default=10.0, help="device time per draft token")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--batch-invariant", action="store_true",
                    help="make a request's logits independent of its batch to the last bit (sled_model_set_batch_invariant)")
    ap.add_argument("--weights", default="bf16", choices=["bf16", "fp8", "fp4"],
                    help="projection weight format of the target (sled_model_set_weight_bits)")
    ap.add_argument("--sweep", action="store_true", help="run batch sizes 4..32 x k in {2, 4, 8} instead of --batch/--k")
    args = ap.parse_args()
    sled.lib()
    torch.cuda.set_device(0)
    shape = synth.SHAPES[args.shape]
    if args.layers:
        shape = synth.scaled_shape(shape, n_layers=args.layers)
    rng = np.random.default_rng(args.seed)
    ctx = rng.integers(args.context // 2, args.context * 3 // 2 + 1, size=args.devices).tolist()
    budget = sum(ctx) + args.devices * (2 * args.tokens + 4 * (shape.k_max + 1))
    weights = {"bf16": synth.SynthWeights, "fp8": synth.SynthWeightsW8, "fp4": synth.SynthWeightsW4}[args.weights](
        shape, seed=args.seed, device="cuda")
    v = Verifier(shape, weights, budget // 16 + 3 * args.devices + 8, args.devices, args.devices, budget,
                 batch_invariant=args.batch_invariant)
    server = Server(v, args.batch)
    devs = list(range(args.devices))
    first = [int(x) for x in rng.integers(0, shape.vocab, size=args.devices)]
    KV = [synth.context_kv(shape, ctx[d], seed=args.seed, req=d, device="cuda") for d in devs]
    for d in devs:
        server.open(d, *KV[d])
    truth = greedy_continuations(server, devs, first, args.tokens)
    configs = [(args.batch, args.k)]
    if args.sweep:
        configs = [(b, k) for b in (4, 8, 16, 32) if b <= args.devices for k in (2, 4, 8) if k <= shape.k_max]
    ok = True
    for batch, k in configs:
        for d in devs:                      # back to the start of every session
            server.close(d)
        server.steps = server.rows = server.drafts_seen = 0
        server.batch_size = batch
        for d in devs:
            server.open(d, *KV[d])
        drafters = {d: ReplayDrafter(truth[d], shape.vocab, args.beta, seed=args.seed * 1000 + d) for d in devs}
        res = simulate(server, drafters, dict(zip(devs, first)), args.tokens, min(k, shape.k_max), args.draft_ms, seed=args.seed)
        ok = ok and res["devices_off_replayed_path"] == 0
        res.pop("texts")
        res.update({"shape": args.shape, "layers": shape.n_layers, "devices": args.devices, "batch": batch, "k": k,
                    "beta": args.beta, "draft_ms_per_token": args.draft_ms, "mean_context": int(np.mean(ctx)), "batch_invariant": args.batch_invariant})
        print(json.dumps({k_: (round(x, 3) if isinstance(x, float) else x) for k_, x in res.items()}), flush=True)
    v.destroy()
    if not ok:
        # Not an error at full model size: the continuation was computed in other batches than the ones the
        # simulation forms, the order of the float32 sums in attention depends on how a batch splits the pages
        # over workgroups, and a K/V value next to a bf16 rounding boundary can then land on its other side;
        # where the two best logits are closer than that, the argmax differs and the text takes another path
        # from there on (the drafter keeps proposing the old one, so that device's acceptance drops).
        print("note: some devices left the precomputed continuation and were stopped there (near-ties of the two best logits)")


if __name__ == "__main__":
    main()
