"""Convenience wrapper around the C entry points for tests and the benchmark: owns the handles,
the scratch and the output buffers of one model on one GPU.  Buffers and argument marshalling
only -- every step of the path runs inside libsled's kernels."""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import sled
from .synth import ModelShape


class Verifier:
    def __init__(self, shape: ModelShape, weights, n_pages: int, max_requests: int, B_max: int,
                 ctx_tokens_max: int, batch_invariant: bool = False):
        self.shape = shape
        self.model = sled.sled_model_create(shape)
        if batch_invariant:
            sled.sled_model_set_batch_invariant(self.model, True)   # before the workspace is sized
        sled.load_weights(self.model, weights)
        self.pool = sled.sled_kvpool_create(self.model, n_pages, max_requests)
        self.T_max = B_max * (shape.k_max + 1)
        self.B_max = B_max
        self.ws = sled.workspace(sled.sled_verify_workspace_bytes(self.model, B_max, self.T_max, ctx_tokens_max))
        self.acc_ws = sled.workspace(sled.sled_accept_workspace_bytes(B_max, self.T_max, shape.vocab))
        self.logits = torch.empty(self.T_max, shape.vocab, dtype=torch.float32, device="cuda")
        self.accept_len = torch.zeros(B_max, dtype=torch.int32, device="cuda")
        self.out_token = torch.zeros(B_max, dtype=torch.int32, device="cuda")

    def open(self) -> int:
        return sled.sled_kvpool_open(self.pool)

    def close_request(self, req: int) -> None:
        sled.sled_kvpool_close(self.pool, req)

    def append_context(self, reqs: Sequence[int], K: Sequence[torch.Tensor], V: Sequence[torch.Tensor]) -> None:
        """K[i], V[i]: [n_layers, n_tokens_i, n_kv_heads, head_dim] in the model dtype, on the GPU."""
        n = [int(k.shape[1]) for k in K]
        sled.sled_kv_append(self.pool, reqs, n, [k.contiguous() for k in K], [v.contiguous() for v in V])

    def append_contexts_scattered(self, reqs: Sequence[int], KV: Sequence, seed: int = 0, contiguous: bool = False) -> None:
        """Uploads the contexts KV[i] = (K, V) of all `reqs` one page (16 tokens) at a time in a seeded random
        interleaving of the requests.  The pool hands out free pages in ascending order, so this scatters every
        request's physical pages over the pool, as on a server whose sessions grow side by side.
        contiguous=True uploads request after request instead (each on a run of consecutive pages)."""
        import numpy as np
        rng = np.random.default_rng(seed)
        n_tok = [int(kv[0].shape[1]) for kv in KV]
        left = np.array([(n + 15) // 16 for n in n_tok])
        done = np.zeros(len(reqs), dtype=np.int64)
        while left.sum() > 0:
            i = int(np.argmax(left > 0)) if contiguous else int(rng.choice(len(reqs), p=left / left.sum()))
            a, b = int(done[i]) * 16, min((int(done[i]) + 1) * 16, n_tok[i])
            self.append_context([reqs[i]], [KV[i][0][:, a:b]], [KV[i][1][:, a:b]])
            done[i] += 1
            left[i] -= 1

    def verify(self, reqs: Sequence[int], k: Sequence[int], tokens: torch.Tensor) -> torch.Tensor:
        T = int(sum(k)) + len(k)
        out = self.logits[:T]
        sled.sled_verify_batch(self.model, self.pool, reqs, k, tokens, out, self.ws)
        return out

    def prefill(self, req: int, tokens: torch.Tensor, want_logits: bool = True) -> Optional[torch.Tensor]:
        """Run a prompt (int32 ids on the GPU) into the request's cache; returns the last token's logits [vocab]."""
        out = self.logits[0] if want_logits else None
        sled.sled_prefill(self.model, self.pool, req, tokens, out, self.ws)
        return out

    def accept(self, mode: int, k: Sequence[int], logits: torch.Tensor, tokens: torch.Tensor,
               draft_q: Optional[torch.Tensor] = None, u_acc: Optional[torch.Tensor] = None,
               u_smp: Optional[torch.Tensor] = None, temperature: float = 1.0):
        B = len(k)
        sled.sled_accept(mode, k, self.shape.vocab, temperature, logits, tokens, draft_q, u_acc, u_smp,
                         self.accept_len[:B], self.out_token[:B], self.acc_ws)
        return self.accept_len[:B], self.out_token[:B]

    def commit(self, reqs: Sequence[int], accept_len: torch.Tensor) -> None:
        sled.sled_kv_append(self.pool, reqs, accept_len=accept_len)

    def read_kv(self, req: int, first_token: int, n_tokens: int):
        """K and V of positions first_token .. first_token + n_tokens - 1 as stored, each [n_layers, n_tokens, n_kv_heads, head_dim]."""
        s = self.shape
        K = torch.empty(s.n_layers, n_tokens, s.n_kv_heads, s.head_dim, dtype=s.torch_dtype, device="cuda")
        V = torch.empty_like(K)
        sled.sled_kv_read(self.pool, req, first_token, n_tokens, K, V)
        return K, V

    def lengths(self, reqs: Sequence[int]) -> List[int]:
        return sled.sled_kvpool_lengths(self.pool, reqs)

    def destroy(self) -> None:
        torch.cuda.synchronize()
        sled.sled_kvpool_destroy(self.pool)
        sled.sled_model_destroy(self.model)
        self.pool = self.model = None
