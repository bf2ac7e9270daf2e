"""The pins must catch plausible mistakes: each case below plants one mistake in the oracle (on the
CPU, by swapping a function of the module for a wrong version) and demands that at least one of the
pin tests then fails.  A mistake that survives means the pins do not really hold the oracle."""
import math

import numpy as np
import pytest

from oracle import sled_oracle as O

import test_oracle_accept as TA
import test_oracle_forward as TF


# ---------------------------------------------------------------- wrong versions, forward pass
def rope_wrong_sign(x, positions, theta):
    D = x.shape[-1]
    half = D // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c + x2 * s, x2 * c - x1 * s], axis=-1)      # rotates the other way


def rope_adjacent_pairs(x, positions, theta):
    D = x.shape[-1]
    half = D // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    out = np.empty_like(x)
    x1, x2 = x[..., 0::2], x[..., 1::2]                                     # pairs (2i, 2i+1) instead of (i, i+D/2)
    out[..., 0::2] = x1 * c - x2 * s
    out[..., 1::2] = x2 * c + x1 * s
    return out


def rope_wrong_frequency(x, positions, theta):
    D = x.shape[-1]
    half = D // 2
    inv_freq = theta ** (-1.0 * np.arange(half, dtype=np.float64) / D)      # exponent i/D instead of 2i/D
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def rmsnorm_no_eps(x, g, eps):
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True)) * g            # eps dropped


def rmsnorm_subtract_mean(x, g, eps):
    xc = x - x.mean(axis=-1, keepdims=True)                                 # LayerNorm instead of RMSNorm
    return xc / np.sqrt((xc * xc).mean(axis=-1, keepdims=True) + eps) * g


def silu_as_sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))                                         # the factor z dropped


def _attention_variant(scale_of, key_count_of, head_map):
    def attention_rows(q, K, V, n_ctx, group, round_points="exact"):
        n, Hq, D = q.shape
        out = np.empty_like(q)
        for h in range(Hq):
            g = head_map(h, group, K.shape[1])
            for j in range(n):
                m = key_count_of(n_ctx, j, n)
                s = (K[:m, g, :] @ q[j, h, :]) * scale_of(D)
                p = np.exp(s - s.max())
                out[j, h, :] = (p @ V[:m, g, :]) / p.sum()
        return out
    return attention_rows


ok_scale = lambda D: 1.0 / math.sqrt(D)
ok_keys = lambda n_ctx, j, n: n_ctx + j + 1
ok_head = lambda h, group, Hkv: h // group
attn_unscaled = _attention_variant(lambda D: 1.0, ok_keys, ok_head)
attn_off_by_one = _attention_variant(ok_scale, lambda n_ctx, j, n: max(1, n_ctx + j), ok_head)   # a row does not see itself
attn_no_causal = _attention_variant(ok_scale, lambda n_ctx, j, n: n_ctx + n, ok_head)            # rows see later drafts
attn_head_interleaved = _attention_variant(ok_scale, ok_keys, lambda h, group, Hkv: h % Hkv)     # wrong GQA mapping

for _n in ("attn_unscaled", "attn_off_by_one", "attn_no_causal", "attn_head_interleaved"):
    globals()[_n].__name__ = _n

def _layer_rows_variant(round_q, round_v, round_before_attention):
    """layer_rows of the bf16-cache definition with the cache rounding misplaced."""
    def layer_rows(model, W, h, positions, K_ctx, V_ctx, stored=None, audit=None):
        cache_round = O.bf16_round if model.round_points != "exact" else (lambda a: a)
        n = h.shape[0]
        Hq, Hkv, D = model.n_q_heads, model.n_kv_heads, model.head_dim
        x = O.rmsnorm(h, W["g_attn"], model.rms_eps)
        q = O.rope((x @ W["wq"].T).reshape(n, Hq, D), positions, model.rope_theta)
        k = O.rope((x @ W["wk"].T).reshape(n, Hkv, D), positions, model.rope_theta)
        v = (x @ W["wv"].T).reshape(n, Hkv, D)
        if round_q:
            q = cache_round(q)
        k_st, v_st = cache_round(k), (cache_round(v) if round_v else v)
        k_at, v_at = (k_st, v_st) if round_before_attention else (k, v)
        o = O.attention_rows(q, np.concatenate([K_ctx, k_at]), np.concatenate([V_ctx, v_at]), K_ctx.shape[0], model.group,
                             model.round_points).reshape(n, Hq * D)
        h = h + o @ W["wo"].T
        x = O.rmsnorm(h, W["g_mlp"], model.rms_eps)
        h = h + (O.silu(x @ W["wg"].T) * (x @ W["wu"].T)) @ W["wd"].T
        return h, k_st, v_st
    return layer_rows


cache_round_after_attention = _layer_rows_variant(False, True, False)   # rows of one pass see unrounded new keys
cache_forgets_v = _layer_rows_variant(False, False, True)               # V enters the cache unrounded
cache_rounds_q_too = _layer_rows_variant(True, True, True)              # q rounded although it is never cached
for _n in ("cache_round_after_attention", "cache_forgets_v", "cache_rounds_q_too"):
    globals()[_n].__name__ = _n

FORWARD_PINS = [
    lambda: TF.test_prefill_matches_hf_llama(TF.SMALL),
    TF.test_cached_verify_matches_hf_llama_with_cache,
    TF.test_single_forward_equals_step_by_step,
    TF.test_causality_and_batch_independence,
    TF.test_attention_rows_matches_torch_sdpa,
    TF.test_attention_single_query_textbook,
    TF.test_rope_closed_forms,
    TF.test_rmsnorm_and_silu_closed_forms,
    TF.test_kv_bf16_rounds_what_enters_the_cache_and_nothing_else,
]


FORWARD_MUTANTS = [
    ("rope", rope_wrong_sign), ("rope", rope_adjacent_pairs), ("rope", rope_wrong_frequency),
    ("rmsnorm", rmsnorm_no_eps), ("rmsnorm", rmsnorm_subtract_mean), ("silu", silu_as_sigmoid),
    ("attention_rows", attn_unscaled), ("attention_rows", attn_off_by_one), ("attention_rows", attn_no_causal),
    ("attention_rows", attn_head_interleaved),
    ("layer_rows", cache_round_after_attention), ("layer_rows", cache_forgets_v), ("layer_rows", cache_rounds_q_too),
]


# ---------------------------------------------------------------- wrong versions, acceptance
def _accept_sample_variant(accept_test, residual_of, bonus_row):
    def accept_sample(logits, drafts, q, u_acc, u_smp, temperature=1.0):
        k = len(drafts)
        margin_acc = math.inf
        for j in range(k):
            p = O.softmax64(logits[j], temperature)
            d = int(drafts[j])
            margin_acc = min(margin_acc, abs(float(u_acc[j]) * float(q[j, d]) - float(p[d])) / max(float(p[d]), 1e-300))
            if not accept_test(float(u_acc[j]), float(q[j, d]), float(p[d])):
                r = residual_of(p, np.asarray(q[j], dtype=np.float64))
                if r.sum() <= 0.0:
                    r = p
                v, mc = O.inverse_cdf(r, u_smp)
                return {"accept_len": j, "out_token": v, "margin_acc": margin_acc, "margin_cdf": mc}
        p = O.softmax64(logits[bonus_row(k)], temperature)
        v, mc = O.inverse_cdf(p, u_smp)
        return {"accept_len": k, "out_token": v, "margin_acc": margin_acc, "margin_cdf": mc}
    return accept_sample


ok_test = lambda u, qd, pd: u * qd <= pd
ok_resid = lambda p, q: np.maximum(0.0, p - q)
acc_inverted_ratio = _accept_sample_variant(lambda u, qd, pd: u * pd <= qd, ok_resid, lambda k: k)   # q/p instead of p/q
acc_resample_from_p = _accept_sample_variant(ok_test, lambda p, q: p, lambda k: k)                    # residual forgotten
acc_abs_residual = _accept_sample_variant(ok_test, lambda p, q: np.abs(p - q), lambda k: k)           # |p - q| instead of (p - q)+
acc_bonus_wrong_row = _accept_sample_variant(ok_test, ok_resid, lambda k: max(k - 1, 0))              # bonus from the last judging row


def accept_greedy_no_stop(logits, drafts):
    """Counts matches anywhere instead of the leading run."""
    k = len(drafts)
    tops = [O.argmax_lowest(logits[j]) for j in range(k + 1)]
    a = sum(int(drafts[j]) == tops[j][0] for j in range(k))
    return {"accept_len": a, "out_token": tops[a][0], "margin": min(g for _, g in tops)}


def argmax_highest(row):
    row = np.asarray(row)
    best = row.max()
    idx = int(np.nonzero(row == best)[0][-1])                                # ties to the highest id
    rest = np.delete(row, idx)
    return idx, float(best - rest.max()) if rest.size else math.inf


def inverse_cdf_exclusive(w, u):
    w = np.asarray(w, dtype=np.float64)
    C = np.cumsum(w) - w                                                     # exclusive prefix sums
    S = float(w.sum())
    hit = np.nonzero(C > float(u) * S)[0]
    v = int(hit[0]) if hit.size else int(np.nonzero(w > 0)[0][-1])
    return v, 1.0


for _n in ("acc_inverted_ratio", "acc_resample_from_p", "acc_abs_residual", "acc_bonus_wrong_row"):
    globals()[_n].__name__ = _n

ACCEPT_PINS = [
    lambda: [TA.test_golden_eq1_examples(c) for c in TA._golden_cases()],
    TA.test_exhaustive_grid_against_rational_enumeration,
    TA.test_sampling_preserves_target_distribution_chi_square,
    TA.test_expected_accept_length_closed_form,
    TA.test_sampling_invariants,
    TA.test_inverse_cdf_cells,
    TA.test_greedy_rules,
]

ACCEPT_MUTANTS = [
    ("accept_sample", acc_inverted_ratio), ("accept_sample", acc_resample_from_p), ("accept_sample", acc_abs_residual),
    ("accept_sample", acc_bonus_wrong_row), ("accept_greedy", accept_greedy_no_stop), ("argmax_lowest", argmax_highest),
    ("inverse_cdf", inverse_cdf_exclusive),
]


def _some_pin_fails(pins):
    for pin in pins:
        try:
            pin()
        except AssertionError:
            return True          # only a failed comparison counts: a crash would prove nothing about the pins
    return False


def test_pins_pass_on_the_unmodified_oracle():
    assert not _some_pin_fails(FORWARD_PINS[1:3] + ACCEPT_PINS[:2])


@pytest.mark.parametrize("name,wrong", FORWARD_MUTANTS, ids=[f"{n}:{f.__name__}" for n, f in FORWARD_MUTANTS])
def test_forward_pins_catch(monkeypatch, name, wrong):
    monkeypatch.setattr(O, name, wrong)
    assert _some_pin_fails(FORWARD_PINS), f"no pin noticed {wrong.__name__}"


@pytest.mark.parametrize("name,wrong", ACCEPT_MUTANTS, ids=[f"{n}:{f.__name__}" for n, f in ACCEPT_MUTANTS])
def test_acceptance_pins_catch(monkeypatch, name, wrong):
    monkeypatch.setattr(O, name, wrong)
    assert _some_pin_fails(ACCEPT_PINS), f"no pin noticed {wrong.__name__}"
