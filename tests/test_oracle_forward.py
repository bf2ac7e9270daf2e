"""Pins for the oracle's forward pass (CPU only).

The oracle is checked against things other than itself:
  * Hugging Face's LlamaForCausalLM in float64 (an independent implementation of the
    LLaMA-family decoder named in Sec. 4) -- catches a wrong rotary pairing, a dropped
    gain, a transposed weight, a wrong GQA head mapping, a wrong attention scale;
  * torch's scaled_dot_product_attention for the ragged verify attention;
  * torch's own float32 -> bfloat16 conversion for the rounding helper;
  * closed forms of rotary embedding, RMSNorm and SiLU;
  * the properties Sec. 3.1 fixes: one forward over all drafts equals scoring them one
    step at a time; a cached forward equals a cache-free recompute; causality.
"""
import math

import numpy as np
import pytest
import torch

from oracle import sled_oracle as O
from paper_2506_09397_amd import synth
from helpers import oracle_model, oracle_requests

SMALL = synth.ModelShape(n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=64,
                         vocab=64, dtype="f32", rope_theta=10000.0)
SMALL_MHA = synth.ModelShape(n_layers=3, d_model=48, n_q_heads=3, n_kv_heads=3, head_dim=16, d_ffn=80,
                             vocab=50, dtype="f32", rope_theta=500000.0)


def _hf_model(shape, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                      num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                      rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta, max_position_embeddings=512,
                      tie_word_embeddings=False, attention_bias=False, mlp_bias=False,
                      attn_implementation="eager")
    m = LlamaForCausalLM(cfg).to(torch.float64).eval()
    sd = {"model.embed_tokens.weight": w.embed(), "model.norm.weight": w.tensor("g_final"),
          "lm_head.weight": w.tensor("lm_head")}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj",
             "g_attn": "input_layernorm", "g_mlp": "post_attention_layernorm"}
    for l in range(shape.n_layers):
        for k, v in w.layer(l).items():
            sd[f"model.layers.{l}.{names[k]}.weight"] = v
    missing = m.load_state_dict({k: v.to(torch.float64) for k, v in sd.items()}, strict=True)
    return m


@pytest.mark.parametrize("shape", [SMALL, SMALL_MHA])
def test_prefill_matches_hf_llama(shape):
    w = synth.SynthWeights(shape, seed=3, std=0.2, gain_jitter=0.2)
    om = oracle_model(shape, w)
    toks = synth.context_tokens(23, shape.vocab, seed=1)
    ours = O.prefill(om, toks)["logits"]
    hf = _hf_model(shape, w)
    with torch.no_grad():
        ref = hf(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    assert ours.shape == ref.shape
    # the library evaluates rotary angles and softmax in float32 even for a float64 model
    assert np.abs(ours - ref).max() < 2e-5 * max(1.0, np.abs(ref).max())


def test_cached_verify_matches_hf_llama_with_cache():
    """k+1 query rows on top of a cache == the last k+1 rows of the full-sequence forward."""
    shape = SMALL
    w = synth.SynthWeights(shape, seed=5, std=0.2, gain_jitter=0.2)
    om = oracle_model(shape, w)
    toks = synth.context_tokens(19 + 5, shape.vocab, seed=2)
    pf = O.prefill(om, toks[:19])
    r = O.verify_batch(om, [{"tokens": toks[19:], "K": pf["K"], "V": pf["V"]}])[0]
    hf = _hf_model(shape, w)
    with torch.no_grad():
        ref = hf(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    assert np.abs(r["logits"] - ref[19:]).max() < 2e-5 * max(1.0, np.abs(ref).max())


def test_single_forward_equals_step_by_step():
    """Sec. 3.1: the target scores all drafts in one forward; row j must equal the one-row
    forward after committing drafts 1..j."""
    shape = SMALL
    w = synth.SynthWeights(shape, seed=7, std=0.2)
    om = oracle_model(shape, w)
    ctx = synth.context_tokens(11, shape.vocab, seed=3)
    pf = O.prefill(om, ctx)
    toks = synth.context_tokens(6, shape.vocab, seed=4)
    all_at_once = O.verify_batch(om, [{"tokens": toks, "K": pf["K"], "V": pf["V"]}])[0]
    K, V = pf["K"], pf["V"]
    for j, t in enumerate(toks):
        r = O.verify_batch(om, [{"tokens": [t], "K": K, "V": V}])[0]
        assert np.abs(r["logits"][0] - all_at_once["logits"][j]).max() < 1e-11
        assert np.abs(r["K_new"][:, 0] - all_at_once["K_new"][:, j]).max() < 1e-12
        K = np.concatenate([K, r["K_new"]], axis=1)
        V = np.concatenate([V, r["V_new"]], axis=1)


def test_causality_and_batch_independence():
    shape = SMALL
    w = synth.SynthWeights(shape, seed=9, std=0.2)
    om = oracle_model(shape, w)
    pf = O.prefill(om, synth.context_tokens(9, shape.vocab, seed=5))
    toks = synth.context_tokens(5, shape.vocab, seed=6)
    base = O.verify_batch(om, [{"tokens": toks, "K": pf["K"], "V": pf["V"]}])[0]["logits"]
    for j in range(1, 5):
        t2 = toks.copy()
        t2[j] = (t2[j] + 1) % shape.vocab
        other = {"tokens": toks[:3], "K": pf["K"][:, :4], "V": pf["V"][:, :4]}
        got = O.verify_batch(om, [other, {"tokens": t2, "K": pf["K"], "V": pf["V"]}])[1]["logits"]
        assert np.array_equal(got[:j], base[:j])          # rows before the change: unchanged
        assert np.abs(got[j] - base[j]).max() > 1e-6      # the changed row: changed


def test_attention_rows_matches_torch_sdpa():
    rng = np.random.default_rng(0)
    for (n_ctx, n, Hq, Hkv, D) in [(0, 3, 2, 2, 8), (5, 1, 1, 1, 4), (17, 9, 8, 2, 16), (33, 5, 8, 1, 8)]:
        q = rng.standard_normal((n, Hq, D))
        K = rng.standard_normal((n_ctx + n, Hkv, D))
        V = rng.standard_normal((n_ctx + n, Hkv, D))
        G = Hq // Hkv
        ours = O.attention_rows(q, K, V, n_ctx, G)
        tq = torch.from_numpy(q).permute(1, 0, 2)[None]
        tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
        tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
        mask = torch.zeros(n, n_ctx + n, dtype=torch.bool)
        for j in range(n):
            mask[j, : n_ctx + j + 1] = True
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)[0]
        assert np.abs(ours - ref.permute(1, 0, 2).numpy()).max() < 1e-12


def test_attention_single_query_textbook():
    """n = 1, one head: softmax(K q / sqrt(D)) V written out by hand."""
    K = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])[:, None, :]
    V = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])[:, None, :]
    q = np.array([[[2.0, 0.0]]])
    s = np.array([2.0, 0.0, 2.0]) / math.sqrt(2.0)
    p = np.exp(s) / np.exp(s).sum()
    want = p @ V[:, 0, :]
    got = O.attention_rows(q, K, V, 2, 1)[0, 0]
    assert np.allclose(got, want, atol=1e-15)


def test_rope_closed_forms():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 3, 8))
    # position 0 is the identity
    assert np.array_equal(O.rope(x, np.zeros(4), 10000.0), x)
    # D = 2, theta irrelevant (exponent 0): plain rotation by `pos` radians of the pair (x0, x1)
    v = np.array([[[1.0, 0.0]]])
    out = O.rope(v, np.array([0.5]), 123.0)[0, 0]
    assert np.allclose(out, [math.cos(0.5), math.sin(0.5)], atol=1e-15)
    # frequencies: pair i of D=4 turns by pos * theta^(-2i/4)
    v = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    out = O.rope(v, np.array([3.0]), 100.0)[0, 0]
    assert np.allclose(out, [math.cos(3.0), math.cos(0.3), math.sin(3.0), math.sin(0.3)], atol=1e-15)
    # norm preserving per pair; relative-position property <R_a q, R_b k> = <q, R_{b-a} k>
    y = O.rope(x, np.array([3, 7, 11, 200]), 10000.0)
    assert np.allclose(x[..., :4] ** 2 + x[..., 4:] ** 2, y[..., :4] ** 2 + y[..., 4:] ** 2)
    qv, kv = rng.standard_normal((1, 1, 8)), rng.standard_normal((1, 1, 8))
    lhs = (O.rope(qv, np.array([5]), 1e4) * O.rope(kv, np.array([12]), 1e4)).sum()
    rhs = (qv * O.rope(kv, np.array([7]), 1e4)).sum()
    assert abs(lhs - rhs) < 1e-12


def test_rmsnorm_and_silu_closed_forms():
    x = np.array([[3.0, 4.0]])
    g = np.array([2.0, 0.5])
    want = x / math.sqrt((9 + 16) / 2 + 1e-5) * g
    assert np.allclose(O.rmsnorm(x, g, 1e-5), want, atol=1e-15)
    # scale invariance when eps -> 0
    assert np.allclose(O.rmsnorm(5 * x, g, 0.0), O.rmsnorm(x, g, 0.0))
    z = np.array([-2.0, 0.0, 1.5])
    assert np.allclose(O.silu(z), z * (1 / (1 + np.exp(-z))))
    assert O.silu(np.array([0.0]))[0] == 0.0


def test_bf16_round_matches_torch_conversion():
    g = torch.Generator().manual_seed(0)
    x = torch.randn(20000, generator=g, dtype=torch.float32) * 3
    # exact ties and edge values
    edge = torch.tensor([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 65280.0, 1e-30, 3.140625])
    x = torch.cat([x, edge])
    want = x.to(torch.bfloat16).to(torch.float64).numpy()
    got = O.bf16_round(x.to(torch.float64).numpy())
    assert np.array_equal(got, want)
    assert O.bf16_round(np.zeros((2, 3))).shape == (2, 3)


def test_round_points_only_touch_storage_tensors():
    """The study modes change results by about their precision and no more; exact mode is untouched; the parity
    definition for bf16 models ("kv_bf16") is the default and differs from "exact" by the cache rounding alone."""
    shape = synth.scaled_shape(SMALL, dtype="bf16")
    w = synth.SynthWeights(shape, seed=11, std=0.2)
    toks = synth.context_tokens(12, shape.vocab, seed=8)
    a = O.prefill(oracle_model(shape, w, "exact"), toks)["logits"]
    b = O.prefill(oracle_model(shape, w, "bf16"), toks)["logits"]
    c = O.prefill(oracle_model(shape, w, "bf16x2"), toks)["logits"]
    kv = O.prefill(oracle_model(shape, w, "kv_bf16"), toks)["logits"]
    f16 = O.prefill(oracle_model(shape, w, "fp16"), toks)["logits"]
    assert oracle_model(shape, w).round_points == "kv_bf16"
    assert oracle_model(synth.scaled_shape(SMALL, dtype="f32"), w).round_points == "exact"
    top = np.abs(a).max()
    err, err2, errkv = np.abs(a - b).max() / top, np.abs(a - c).max() / top, np.abs(a - kv).max() / top
    assert 1e-5 < err < 5e-2
    assert 1e-7 < err2 < err          # pairs carry 16 bits; only the cached K/V are single bf16
    assert 1e-7 < errkv < err         # cache rounding alone
    # against the parity definition: pairs add about 2^-16 per stored tensor, halves about 2^-11
    assert np.abs(c - kv).max() / top < 2.0 ** -12
    assert np.abs(c - kv).max() < np.abs(f16 - kv).max() < np.abs(b - kv).max()


def test_kv_bf16_rounds_what_enters_the_cache_and_nothing_else():
    """Where the parity definition of a bf16 model rounds (Sec. 3.1's single pass over all drafts must equal
    verifying them one by one on the same cache): the new keys and values are bf16 numbers by the time any row --
    of the same pass or of a later one -- attends to them, and nothing else is rounded."""
    shape = synth.scaled_shape(SMALL, dtype="bf16")
    w = synth.SynthWeights(shape, seed=5, std=0.2)
    om, ex = oracle_model(shape, w, "kv_bf16"), oracle_model(shape, w, "exact")
    ctx = synth.context_tokens(9, shape.vocab, seed=3)
    pf = O.prefill(om, ctx)
    for name in ("K", "V"):   # what the cache holds is representable in bf16
        t = torch.from_numpy(pf[name])
        assert torch.equal(t.to(torch.bfloat16).to(torch.float64), t)
    # layer 0 sees identical inputs in both modes: its cached rows are the rounded exact rows
    pe = O.prefill(ex, ctx)
    assert np.array_equal(pf["K"][0], O.bf16_round(pe["K"][0])) and np.array_equal(pf["V"][0], O.bf16_round(pe["V"][0]))
    assert not np.array_equal(pf["K"][0], pe["K"][0])
    # one pass over [pending, d1..d4] == five single-row passes, each appending its rounded K/V
    toks = [int(t) for t in synth.context_tokens(5, shape.vocab, seed=4)]
    one = O.verify_batch(om, [{"tokens": toks, "K": pf["K"], "V": pf["V"]}])[0]
    K, V, rows = pf["K"], pf["V"], []
    for t in toks:
        r = O.verify_batch(om, [{"tokens": [t], "K": K, "V": V}])[0]
        rows.append(r["logits"][0])
        K, V = np.concatenate([K, r["K_new"]], axis=1), np.concatenate([V, r["V_new"]], axis=1)
    assert np.abs(np.stack(rows) - one["logits"]).max() < 1e-12 * np.abs(one["logits"]).max()
    assert np.array_equal(K[:, 9:], one["K_new"]) or np.abs(K[:, 9:] - one["K_new"]).max() < 1e-12
    # a single token on an empty cache: its only key is its own, the softmax weight is 1, so the attention output
    # of layer 0 IS the rounded value -- rounding after attention instead of before would leave the logits at "exact"
    lone = O.verify_batch(om, [{"tokens": toks[:1], "K": pf["K"][:, :0], "V": pf["V"][:, :0]}])[0]["logits"]
    lone_ex = O.verify_batch(ex, [{"tokens": toks[:1], "K": pf["K"][:, :0], "V": pf["V"][:, :0]}])[0]["logits"]
    assert np.abs(lone - lone_ex).max() > 1e-6 * np.abs(lone_ex).max()
    # with W_k = W_v = 0 the new keys and values are exact zeros, the cache rounding changes nothing, and so the two
    # modes must agree to the last bit: any other tensor being rounded (q, the normalised activations, the softmax
    # weights, the attention output, the SwiGLU product) would show here
    class NoKV:
        def __init__(self, inner):
            self.inner = inner

        def embed(self):
            return self.inner.embed()

        def final(self):
            return self.inner.final()

        def layer(self, l):
            W = dict(self.inner.layer(l))
            W["wk"], W["wv"] = np.zeros_like(W["wk"]), np.zeros_like(W["wv"])
            return W

    ctx_kv = synth.context_kv(shape, 9, seed=1, req=0)
    req = [{"tokens": toks, "K": synth.as_f64(ctx_kv[0]), "V": synth.as_f64(ctx_kv[1])}]
    outs = []
    for m in (om, ex):
        m2 = O.OracleModel(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab, m.rope_theta,
                           m.rms_eps, NoKV(m.weights), m.round_points)
        outs.append(O.verify_batch(m2, req)[0]["logits"])
    assert np.array_equal(outs[0], outs[1])


def test_stored_cache_numbers_replace_the_rounding_decision_and_are_audited():
    """The oracle can take the cache-rounding decision as a cache under test took it: given the bf16 numbers stored
    for the new rows it attends to those and reports how far they are from the exact values.  Its own numbers change
    nothing and audit clean; numbers one bf16 step off change the logits and show in the audit; one pass still equals
    row-by-row verification on the same stored numbers."""
    shape = synth.scaled_shape(SMALL, dtype="bf16")
    w = synth.SynthWeights(shape, seed=6, std=0.2)
    om = oracle_model(shape, w, "kv_bf16")
    ctx_kv = synth.context_kv(shape, 7, seed=2, req=0)
    toks = [int(t) for t in synth.context_tokens(4, shape.vocab, seed=9)]
    base = {"tokens": toks, "K": synth.as_f64(ctx_kv[0]), "V": synth.as_f64(ctx_kv[1])}
    plain = O.verify_batch(om, [base])[0]
    same = O.verify_batch(om, [dict(base, K_stored=plain["K_new"], V_stored=plain["V_new"])])[0]
    assert np.array_equal(same["logits"], plain["logits"])
    assert same["audit"]["flips"] == 0 and same["audit"]["max_excess"] <= 0.0 and same["audit"]["elements"] == 2 * plain["K_new"].size
    # the spacing helper against torch's bf16 grid (bf16-representable, positive values: the step to the next one up)
    x = np.array([1.0, 1.5, 1.984375, 2.0, 0.30078125, 5.0, 0.0009765625, 448.0])
    xb = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(xb.to(torch.float64).numpy(), x)
    nxt = torch.nextafter(xb, torch.full_like(xb, float("inf")))
    assert np.array_equal(O.bf16_ulp(x), (nxt.to(torch.float64) - xb.to(torch.float64)).numpy())
    assert np.array_equal(O.bf16_ulp(-x), O.bf16_ulp(x)) and np.array_equal(O.bf16_ulp(x * 1.003), O.bf16_ulp(x))
    # three values moved by one bf16 step: used as given, and seen
    K2 = plain["K_new"].copy()
    for (l, j, g, d) in ((0, 1, 0, 3), (1, 2, 1, 5), (0, 3, 1, 0)):
        K2[l, j, g, d] += O.bf16_ulp(K2[l, j, g, d])
    moved = O.verify_batch(om, [dict(base, K_stored=K2, V_stored=plain["V_new"])])[0]
    assert np.array_equal(moved["K_new"], K2) and not np.array_equal(moved["logits"], plain["logits"])
    # (a whole step beyond a correct rounding, on an element of about the vector's size: 2^-8 .. 2^-7 of it and more)
    assert moved["audit"]["flips"] >= 3 and 1e-3 < moved["audit"]["max_excess"] < 0.5
    # rows of one pass attend to the stored numbers of the earlier rows, exactly as a later pass would
    K, V, rows = base["K"], base["V"], []
    for j, t in enumerate(toks):
        r = O.verify_batch(om, [{"tokens": [t], "K": K, "V": V, "K_stored": K2[:, j: j + 1], "V_stored": plain["V_new"][:, j: j + 1]}])[0]
        rows.append(r["logits"][0])
        K, V = np.concatenate([K, K2[:, j: j + 1]], axis=1), np.concatenate([V, plain["V_new"][:, j: j + 1]], axis=1)
    assert np.abs(np.stack(rows) - moved["logits"]).max() < 1e-12 * np.abs(moved["logits"]).max()


def test_pair_contract_stays_within_2_to_minus_12_of_the_parity_definition():
    """The bf16-pair storage study ("bf16x2": what the HIP library stores between its kernels) against the parity
    definition, on the tiny bf16 shape and on two layers of the 8B shape: at most 2^-12 of the largest logit
    (measured 1.5e-5 and 1.2e-4; a pair rounding is 2^-17, but it moves a new key or value across a bf16 rounding
    boundary now and then, and such a flip is a whole 2^-8 of that element)."""
    for shape, ctx_len, k, seed in ((synth.SHAPES["tiny_bf16"], [40, 17, 100], [4, 0, 8], 0),
                                    (synth.scaled_shape(synth.SHAPES["llama8b"], n_layers=2, vocab=4096), [300, 70], [4, 2], 1)):
        w = synth.SynthWeights(shape, seed=seed, device="cpu")
        batch = synth.make_batch(ctx_len, k, shape.vocab, seed=seed)
        KV = [synth.context_kv(shape, L, seed=seed, req=i) for i, L in enumerate(ctx_len)]
        reqs = oracle_requests(batch, [a for a, _ in KV], [b for _, b in KV])
        want = np.concatenate([r["logits"] for r in O.verify_batch(oracle_model(shape, w, "kv_bf16", cache=False), reqs)])
        pair = np.concatenate([r["logits"] for r in O.verify_batch(oracle_model(shape, w, "bf16x2", cache=False), reqs)])
        rel = np.abs(pair - want).max() / np.abs(want).max()
        print(f"{shape.d_model}-wide, {shape.n_layers} layers: pairs vs parity definition {rel:.2e} of the largest logit")
        assert rel < 2.0 ** -12


def test_bf16_pair_rounding():
    x = np.array([1.0, 1.00390625, 3.14159265358979, -2.718281828, 1e-3, 123456.789])
    y = O.bf16x2_round(x)
    hi = O.bf16_round(x)
    assert np.array_equal(y, hi + O.bf16_round(x - hi))
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -16)
    assert np.all(np.abs(hi - x) <= np.abs(x) * 2.0 ** -8)


def test_rounded_softmax_numerators_are_reference_free():
    """bf16 mode: rounding 2^(t - M) for a whole number M gives the same attention output for any
    such M (scaling by a power of two commutes with rounding), and stays within bf16 precision of
    the unrounded softmax."""
    rng = np.random.default_rng(4)
    q = rng.standard_normal((3, 4, 16)) * 2
    K = rng.standard_normal((40, 2, 16))
    V = rng.standard_normal((40, 2, 16))
    exact = O.attention_rows(q, K, V, 37, 2, "exact")
    rounded = O.attention_rows(q, K, V, 37, 2, "bf16")
    assert 1e-6 < np.abs(exact - rounded).max() < 2e-2
    # the same with every reference shifted by +3 whole units, written out by hand for one row
    j, h, g = 1, 2, 1
    s = (K[:39, g, :] @ q[j, h, :]) / math.sqrt(16) * O.LOG2E
    p = np.exp2(s - (math.ceil(s.max()) + 3))
    alt = (O.bf16_round(p) @ V[:39, g, :]) / p.sum()
    assert np.abs(alt - rounded[j, h]).max() < 1e-15
