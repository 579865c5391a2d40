"""Pins of the decoder oracle against things other than itself."""
import numpy as np
import pytest
import torch

from oracle import decoder as dec
from paper_2404_08856_amd import synth

TINY = synth.SHAPES["tiny_target"]


def oracle_cfg(shape, kv_bf16):
    return dec.DecoderConfig(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn,
                             shape.vocab, shape.rms_eps, shape.rope_theta, kv_bf16)


def tiny_model(seed=0, shape=TINY, random_gains=False):
    w = synth.make_weights(shape, seed)
    if random_gains:   # gains != 1 so that a dropped/misplaced gain is caught
        g = torch.Generator().manual_seed(99)
        w["final_norm"] = 1.0 + 0.3 * torch.randn(shape.d_model, generator=g)
        for lw in w["layers"]:
            lw["attn_norm"] = 1.0 + 0.3 * torch.randn(shape.d_model, generator=g)
            lw["mlp_norm"] = 1.0 + 0.3 * torch.randn(shape.d_model, generator=g)
    return w


def test_whole_decoder_matches_library_llama():
    """Independent library implementation of the same architecture (the
    LLaMA decoder in the `transformers` package), float64, image rows +
    token rows as input embeddings.  Pins RoPE pairing and frequencies, the
    epsilon placement in RMSNorm, the 1/sqrt(d_h) scale, the causal mask, the
    SwiGLU wiring, residual adds, final norm and LM head."""
    transformers = pytest.importorskip("transformers")
    shape = TINY
    w = tiny_model(random_gains=True)
    hf_cfg = transformers.LlamaConfig(
        vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
        num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
        num_key_value_heads=shape.n_heads, hidden_act="silu", max_position_embeddings=512,
        rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta, attention_bias=False,
        tie_word_embeddings=False, attn_implementation="eager")
    model = transformers.LlamaForCausalLM(hf_cfg).to(torch.float64).eval()
    sd = {"model.embed_tokens.weight": w["embed"], "lm_head.weight": w["lm_head"],
          "model.norm.weight": w["final_norm"]}
    names = {"attn_norm": "input_layernorm.weight", "wq": "self_attn.q_proj.weight",
             "wk": "self_attn.k_proj.weight", "wv": "self_attn.v_proj.weight",
             "wo": "self_attn.o_proj.weight", "mlp_norm": "post_attention_layernorm.weight",
             "w_gate": "mlp.gate_proj.weight", "w_up": "mlp.up_proj.weight", "w_down": "mlp.down_proj.weight"}
    for l, lw in enumerate(w["layers"]):
        for k, v in lw.items():
            sd[f"model.layers.{l}.{names[k]}"] = v
    missing, unexpected = model.load_state_dict({k: v.to(torch.float64) for k, v in sd.items()}, strict=False)
    assert not [m for m in missing if "rotary" not in m] and not unexpected

    img = synth.image_rows(7, shape.d_model, 3)
    toks = synth.text_tokens(9, shape.vocab, 3)
    wn = synth.weights_to_numpy(w)
    x = np.concatenate([img.astype(np.float64), dec.embed_tokens(wn, toks)], axis=0)
    with torch.no_grad():
        ref = model(inputs_embeds=torch.from_numpy(x)[None]).logits[0].numpy()
    got = dec.full_recompute(oracle_cfg(shape, kv_bf16=False), wn, x)
    assert got.shape == ref.shape
    # the library keeps its rotary cos/sin table in float32, hence ~1e-7 rather than 1e-13;
    # a wrong convention anywhere shows up at 1e-2 or more on logits of spread ~0.3
    assert np.max(np.abs(got - ref)) < 2e-6
    assert np.std(ref) > 0.1


@pytest.mark.parametrize("kv_bf16", [False, True])
def test_cached_forward_equals_full_recompute(kv_bf16):
    shape = TINY
    wn = synth.weights_to_numpy(tiny_model())
    cfg = oracle_cfg(shape, kv_bf16)
    x = np.concatenate([synth.image_rows(6, shape.d_model, 1).astype(np.float64),
                        dec.embed_tokens(wn, synth.text_tokens(11, shape.vocab, 1))])
    full = dec.full_recompute(cfg, wn, x)
    cache = dec.KVCache(cfg, 32)
    a = dec.forward_rows(cfg, wn, cache, x[:12])          # prefill
    b = dec.forward_rows(cfg, wn, cache, x[12:])          # gamma+1 = 5 rows against the cache
    got = np.concatenate([a, b])
    # same row-wise arithmetic; only the BLAS blocking of differently sized products differs
    assert np.max(np.abs(got - full)) < 1e-12


def test_rows_at_once_equal_single_row_calls():
    shape = TINY
    wn = synth.weights_to_numpy(tiny_model())
    cfg = oracle_cfg(shape, True)
    toks = synth.text_tokens(10, shape.vocab, 2)
    c1 = dec.KVCache(cfg, 16)
    dec.forward_tokens(cfg, wn, c1, toks[:5])
    many = dec.forward_tokens(cfg, wn, c1, toks[5:])
    c2 = dec.KVCache(cfg, 16)
    dec.forward_tokens(cfg, wn, c2, toks[:5])
    single = np.concatenate([dec.forward_tokens(cfg, wn, c2, toks[i:i + 1]) for i in range(5, 10)])
    assert np.max(np.abs(many - single)) < 1e-12
    assert c1.length == c2.length == 10


def test_rollback_then_refeed_gives_same_logits():
    shape = TINY
    wn = synth.weights_to_numpy(tiny_model())
    cfg = oracle_cfg(shape, True)
    toks = synth.text_tokens(12, shape.vocab, 4)
    c = dec.KVCache(cfg, 16)
    dec.forward_tokens(cfg, wn, c, toks[:6])
    first = dec.forward_tokens(cfg, wn, c, toks[6:11])
    c.truncate(8)                                        # keep two of the five
    dec.forward_tokens(cfg, wn, c, [int(toks[8])])
    again = dec.forward_tokens(cfg, wn, c, toks[9:11])
    assert np.max(np.abs(again - first[3:5])) < 1e-12


def test_causality():
    shape = TINY
    wn = synth.weights_to_numpy(tiny_model())
    cfg = oracle_cfg(shape, True)
    toks = synth.text_tokens(9, shape.vocab, 5).copy()
    a = dec.full_recompute(cfg, wn, dec.embed_tokens(wn, toks))
    toks2 = toks.copy()
    toks2[6] = (toks2[6] + 1) % shape.vocab
    b = dec.full_recompute(cfg, wn, dec.embed_tokens(wn, toks2))
    assert np.array_equal(a[:6], b[:6])
    assert np.max(np.abs(a[6:] - b[6:])) > 1e-6


def test_rope_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 2, 64))
    # position 0 is the identity
    assert np.array_equal(dec.rope(x, [0, 0, 0], 1e4), x)
    # rotation preserves the norm of every head vector
    y = dec.rope(x, [5, 17, 300], 1e4)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    # <rope(q, m), rope(k, n)> depends on m - n only
    q = rng.standard_normal((1, 1, 64))
    k = rng.standard_normal((1, 1, 64))
    d1 = np.sum(dec.rope(q, [9], 1e4) * dec.rope(k, [4], 1e4))
    d2 = np.sum(dec.rope(q, [105], 1e4) * dec.rope(k, [100], 1e4))
    assert abs(d1 - d2) < 1e-11
    # the first pair (i = 0, i + d_h/2) turns by exactly `position` radians, the last by
    # position * theta^(-(d_h-2)/d_h)
    e = np.zeros((1, 1, 64))
    e[0, 0, 0] = 1.0
    r = dec.rope(e, [2], 1e4)
    assert abs(r[0, 0, 0] - np.cos(2.0)) < 1e-15 and abs(r[0, 0, 32] - np.sin(2.0)) < 1e-15
    e = np.zeros((1, 1, 64))
    e[0, 0, 31] = 1.0
    r = dec.rope(e, [7], 1e4)
    ang = 7.0 * 1e4 ** (-62.0 / 64.0)
    assert abs(r[0, 0, 31] - np.cos(ang)) < 1e-15 and abs(r[0, 0, 63] - np.sin(ang)) < 1e-15


def test_attention_special_cases():
    rng = np.random.default_rng(1)
    H, dh = 2, 8
    # a single visible key: output is its value
    q = rng.standard_normal((1, H, dh))
    k = rng.standard_normal((1, H, dh))
    v = rng.standard_normal((1, H, dh))
    assert np.allclose(dec.causal_attention(q, k, v, 0), v.reshape(1, -1), atol=1e-15)
    # zero queries -> uniform weights -> running mean of the values (causal)
    M = 4
    q = np.zeros((M, H, dh))
    k = rng.standard_normal((M, H, dh))
    v = rng.standard_normal((M, H, dh))
    out = dec.causal_attention(q, k, v, 0).reshape(M, H, dh)
    for i in range(M):
        assert np.allclose(out[i], v[:i + 1].mean(axis=0), atol=1e-14)


def test_attention_matches_library_sdpa():
    rng = np.random.default_rng(2)
    H, dh, P0, M = 3, 16, 5, 4
    q = rng.standard_normal((M, H, dh))
    k = rng.standard_normal((P0 + M, H, dh))
    v = rng.standard_normal((P0 + M, H, dh))
    got = dec.causal_attention(q, k, v, P0)
    mask = torch.from_numpy(np.arange(P0 + M)[None, :] <= (P0 + np.arange(M))[:, None])
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2)[None], torch.from_numpy(k).permute(1, 0, 2)[None],
        torch.from_numpy(v).permute(1, 0, 2)[None], attn_mask=mask)
    ref = ref[0].permute(1, 0, 2).reshape(M, H * dh).numpy()
    assert np.max(np.abs(got - ref)) < 1e-13


def test_elementwise_pieces_match_library():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 32))
    g = rng.standard_normal(32)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.max(np.abs(dec.rmsnorm(x, g, 1e-6) - ref)) < 1e-14
    # eps matters for tiny rows: sqrt(mean + eps), not sqrt(mean) + eps
    tiny = np.full((1, 4), 1e-4)
    assert np.allclose(dec.rmsnorm(tiny, np.ones(4), 1e-6), 1e-4 / np.sqrt(1e-8 + 1e-6))
    z = rng.standard_normal(100) * 4
    assert np.max(np.abs(dec.silu(z) - torch.nn.functional.silu(torch.from_numpy(z)).numpy())) < 1e-15
    s = rng.standard_normal((4, 9))
    assert np.max(np.abs(dec.softmax_rows(s) - torch.softmax(torch.from_numpy(s), -1).numpy())) < 1e-15


def test_bf16_helpers_match_library_conversions():
    g = torch.Generator().manual_seed(0)
    x = torch.randn(20000, generator=g, dtype=torch.float64) * 3
    ref = x.to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(dec.round_to_bf16(x.numpy()), ref)
    # exact ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert dec.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert dec.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    b = x.to(torch.bfloat16)
    assert np.array_equal(dec.to_f64(synth.bf16_bits(b)), b.to(torch.float64).numpy())


def test_table1_parameter_counts():
    """Sizes the paper prints (tests/golden/table1_model_sizes.txt)."""
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_model_sizes.txt")) as f:
        for line in f:
            p = line.split()
            if p and p[0] in ("draft", "target"):
                rows[p[0]] = [float(v) for v in p[1:]]
    for name, (layers, heads, ffn, hidden, stated) in rows.items():
        n = dec.parameter_count(int(layers), int(hidden), int(ffn), 32000, tied_embeddings=False)
        assert abs(n - stated) / stated < 0.05, (name, n)
    # the synthetic shapes used by the benchmarks are these shapes
    s = synth.SHAPES["draft_paper_115m"]
    assert (s.n_layers, s.n_heads, s.d_ffn, s.d_model) == (4, 8, 2816, 1024)
    s = synth.SHAPES["llama7b"]
    assert (s.n_layers, s.n_heads, s.d_ffn, s.d_model) == (32, 32, 11008, 4096)
    assert s.n_params() == dec.parameter_count(32, 4096, 11008, 32000, False)
