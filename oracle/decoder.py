"""Oracle: LLaMA-style decoder forward with a KV cache (TEST INFRASTRUCTURE ONLY).

What the paper fixes (Section 2.2, Eq. 1; Section 3; Appendix A.1, Table 1):
the target and the draft language models are LLaMA-architecture decoders with
the Table-1 sizes and SiLU activation; the target conditions on the image
embeddings V_1..V_m followed by the text-token embeddings X_1..X_n, i.e. its
input is a matrix of embedding rows, not only token ids; the draft conditions
on the text tokens alone.  The paper gives nothing below that level, so this
file writes out the public definition of a LLaMA decoder layer:

    a  = RMSNorm(h; g_attn)                    a_i = h_i / sqrt(mean_j h_ij^2 + eps) * g
    q, k, v = a Wq^T, a Wk^T, a Wv^T           (no biases), split into heads
    q, k <- RoPE(q, k; position)               half-split pairing (i, i + d_h/2)
    cache[position] <- k, v                    (rounded to bf16 if the cache is bf16)
    o_i = sum_j softmax_j(q_i.k_j / sqrt(d_h)) v_j     over cached positions j <= position_i
    h += o Wo^T
    b  = RMSNorm(h; g_mlp)
    h += (silu(b Wg^T) * (b Wu^T)) Wd^T        silu(z) = z / (1 + exp(-z))
    logits = RMSNorm(h_L; g_final) Wlm^T

Everything is float64.  Weight arrays may be float64/float32 or uint16 holding
bfloat16 bit patterns; they are widened exactly.  No blocking, fusion or
reordering: each line above is one numpy statement below.

Readings of points the paper leaves open (listed in the design notes too):
RoPE pairs element i with i + d_h/2 and uses inverse frequency
theta^(-2i/d_h); RMSNorm epsilon sits inside the square root; the KV cache of
a bf16 model stores K (after RoPE) and V rounded to bfloat16.

Pins (tests/test_oracle_decoder.py): equality with an independent library
implementation of the same architecture on a tiny model, cached == full
recompute, M rows at once == M single-row calls, closed forms for RoPE and
attention special cases, causality.
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class DecoderConfig:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e4
    kv_bf16: bool = True      # KV cache stores bfloat16-rounded values


def to_f64(a):
    """Widen a weight/activation array to float64 exactly.

    uint16 arrays are bfloat16 bit patterns: a bfloat16 is the upper half of
    an IEEE float32, so shifting into the high 16 bits of a uint32 and
    re-reading as float32 is exact.
    """
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def round_to_bf16(x):
    """Round float64 values to the nearest bfloat16 value (ties to even).

    A bfloat16 has 8 significant binary digits.  Write x = m * 2^e with
    0.5 <= |m| < 1, round m * 2^8 to an integer (numpy rounds halves to even)
    and scale back.  Values here are O(1): no overflow/subnormal handling.
    """
    m, e = np.frexp(np.asarray(x, dtype=np.float64))
    return np.ldexp(np.round(m * 256.0), e - 8)


def rmsnorm(x, gain, eps):
    """Root-mean-square layer norm of each row of x (LLaMA; Appendix A.1)."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * to_f64(gain)


def silu(z):
    """SiLU activation (Table 1): z * sigmoid(z)."""
    return z / (1.0 + np.exp(-z))


def rope(x, positions, theta):
    """Rotary position embedding on x[M, H, d_h] for absolute positions[M].

    Pair (i, i + d_h/2) is rotated by angle position * theta^(-2i/d_h).
    """
    x = np.asarray(x, dtype=np.float64)
    d_h = x.shape[-1]
    half = d_h // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d_h)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]   # [M, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1 = x[..., :half]
    x2 = x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_rows(s):
    """Softmax along the last axis (entries may be -inf)."""
    s = s - np.max(s, axis=-1, keepdims=True)
    e = np.exp(s)
    return e / np.sum(e, axis=-1, keepdims=True)


def causal_attention(q, k_all, v_all, first_pos):
    """Attention of M queries over a cached prefix.

    q[M, H, d_h] are the queries at absolute positions first_pos + i;
    k_all, v_all[P, H, d_h] hold the keys/values of positions 0..P-1 with
    P = first_pos + M (the new rows already appended).  Query i sees keys
    j <= first_pos + i.  Returns o[M, H * d_h].
    """
    M, H, d_h = q.shape
    P = k_all.shape[0]
    assert P == first_pos + M
    key_pos = np.arange(P)[None, :]
    qry_pos = first_pos + np.arange(M)[:, None]
    visible = key_pos <= qry_pos                                   # [M, P]
    out = np.empty((M, H, d_h), dtype=np.float64)
    for h in range(H):
        s = (q[:, h, :] @ k_all[:, h, :].T) / np.sqrt(float(d_h))   # [M, P]
        s = np.where(visible, s, -np.inf)
        w = softmax_rows(s)
        out[:, h, :] = w @ v_all[:, h, :]
    return out.reshape(M, H * d_h)


class KVCache:
    """Keys (after RoPE) and values of every position fed so far, per layer."""

    def __init__(self, cfg, max_positions):
        shape = (cfg.n_layers, max_positions, cfg.n_heads, cfg.head_dim)
        self.k = np.zeros(shape, dtype=np.float64)
        self.v = np.zeros(shape, dtype=np.float64)
        self.length = 0

    def truncate(self, length):
        """Forget every position >= length (rollback after a rejection)."""
        assert 0 <= length <= self.length
        self.length = length


def embed_tokens(weights, tokens):
    """Token-embedding rows E[tok] as float64 [len(tokens), d]."""
    return to_f64(np.asarray(weights["embed"])[np.asarray(tokens, dtype=np.int64)])


def forward_rows(cfg, weights, cache, x):
    """One decoder forward over M new input-embedding rows x[M, d].

    The rows take absolute positions cache.length .. cache.length + M - 1;
    their K, V are appended to the cache and cache.length grows by M.
    Returns logits[M, vocab] (float64): row i is the distribution over the
    token that follows input row i.

    This is the one target call that scores all drafted positions at once
    (Section 2.1) when x = E[[t, d_1 .. d_gamma]], the
    prefill when x = [V_1..V_m ; E[X_1..X_n]] (Section 2.2, Eq. 1), and one
    draft step when M is 1 or 2 and the model is the draft (Section 3).
    """
    h = np.array(x, dtype=np.float64)
    M = h.shape[0]
    P0 = cache.length
    positions = P0 + np.arange(M)
    H, d_h = cfg.n_heads, cfg.head_dim
    assert P0 + M <= cache.k.shape[1], "KV cache overflow"
    for l, lw in enumerate(weights["layers"]):
        a = rmsnorm(h, lw["attn_norm"], cfg.rms_eps)
        q = (a @ to_f64(lw["wq"]).T).reshape(M, H, d_h)
        k = (a @ to_f64(lw["wk"]).T).reshape(M, H, d_h)
        v = (a @ to_f64(lw["wv"]).T).reshape(M, H, d_h)
        q = rope(q, positions, cfg.rope_theta)
        k = rope(k, positions, cfg.rope_theta)
        if cfg.kv_bf16:
            k = round_to_bf16(k)
            v = round_to_bf16(v)
        cache.k[l, P0:P0 + M] = k
        cache.v[l, P0:P0 + M] = v
        o = causal_attention(q, cache.k[l, :P0 + M], cache.v[l, :P0 + M], P0)
        h = h + o @ to_f64(lw["wo"]).T
        b = rmsnorm(h, lw["mlp_norm"], cfg.rms_eps)
        g = b @ to_f64(lw["w_gate"]).T
        u = b @ to_f64(lw["w_up"]).T
        h = h + (silu(g) * u) @ to_f64(lw["w_down"]).T
    cache.length = P0 + M
    hn = rmsnorm(h, weights["final_norm"], cfg.rms_eps)
    lm = weights["lm_head"] if weights.get("lm_head") is not None else weights["embed"]
    return hn @ to_f64(lm).T


def forward_tokens(cfg, weights, cache, tokens):
    """forward_rows on the embedding rows of the given token ids."""
    return forward_rows(cfg, weights, cache, embed_tokens(weights, tokens))


def full_recompute(cfg, weights, x_all):
    """Logits of every row of x_all[S, d] computed from an empty cache."""
    cache = KVCache(cfg, x_all.shape[0])
    return forward_rows(cfg, weights, cache, x_all)


def parameter_count(n_layers, d_model, d_ffn, vocab, tied_embeddings):
    """Parameters of the language-model part (matrices only; Table 1 sizes)."""
    per_layer = 4 * d_model * d_model + 3 * d_model * d_ffn
    emb = vocab * d_model * (1 if tied_embeddings else 2)
    return n_layers * per_layer + emb
