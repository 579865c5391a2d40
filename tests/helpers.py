"""Shared helpers of the test-suite (not collected by pytest)."""
import numpy as np
import torch

from oracle import decoder as dec
from paper_2404_08856_amd import synth

# spec tolerance for logits: bf16 weights, float32 accumulation
LOGIT_MAX_ABS = 3e-2
LOGIT_MEAN_ABS = 3e-3


def oracle_cfg(shape, kv_bf16=True):
    return dec.DecoderConfig(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn,
                             shape.vocab, shape.rms_eps, shape.rope_theta, kv_bf16)


def to_device(w, device="cuda"):
    out = {k: (v.to(device) if isinstance(v, torch.Tensor) else v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: v.to(device) for k, v in lw.items()} for lw in w["layers"]]
    return out


def randomize_gains(w, seed=99):
    """Gains != 1, so that a dropped or misplaced gain cannot hide."""
    g = torch.Generator().manual_seed(seed)
    d = w["final_norm"].numel()
    w["final_norm"] = (1.0 + 0.3 * torch.randn(d, generator=g)).float()
    for lw in w["layers"]:
        lw["attn_norm"] = (1.0 + 0.3 * torch.randn(d, generator=g)).float()
        lw["mlp_norm"] = (1.0 + 0.3 * torch.randn(d, generator=g)).float()
    return w


def check_logits(got, want, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite logits"
    err = np.abs(got - want)
    assert err.max() <= LOGIT_MAX_ABS and err.mean() <= LOGIT_MEAN_ABS, \
        f"{what}: max-abs {err.max():.3e} (limit {LOGIT_MAX_ABS}), mean-abs {err.mean():.3e} (limit {LOGIT_MEAN_ABS})"
    return err.max(), err.mean()


def accept_margins(T_rows, D_rows, d_tokens, u):
    """Relative distance of every accept test u * D(d) < T(d) from equality: a decision may differ between two
    float paths only where this is tiny."""
    return [abs(float(u[j]) * float(D_rows[j, d_tokens[j]]) - float(T_rows[j, d_tokens[j]])) /
            max(float(T_rows[j, d_tokens[j]]), 1e-30) for j in range(len(d_tokens))]


def drawn_token_is_valid(T_rows, D_rows, k, u_last, y, tol=1e-4):
    """Is y what the fixed-point inverse-CDF sampler draws from row k's residual (bonus row for k = gamma),
    up to a perturbation of the cumulative sums by tol * (total mass)?  With tol = 0 this is y == the oracle's
    token.  Two softmax implementations that agree to ~1e-6 move the cumulative sums by that much, so the
    drawn token may differ only when the threshold sits that close to a bucket boundary."""
    from oracle import spec_sampling as ss
    gamma = D_rows.shape[0]
    r = ss.residual(T_rows[k], D_rows[k]) if k < gamma else np.asarray(T_rows[gamma], dtype=np.float32)
    w = ss.fixed_point_weights(r)
    S = int(np.sum(w, dtype=np.uint64))
    if S == 0:
        r = np.asarray(T_rows[min(k, gamma)], dtype=np.float32)
        w = ss.fixed_point_weights(r)
        S = int(np.sum(w, dtype=np.uint64))
        if S == 0:
            return y == 0
    k_u = int(np.float64(np.float32(u_last)) * float(1 << 24))
    thr = (k_u * S) >> 24
    run = np.cumsum(w, dtype=np.uint64)
    lo = int(run[y - 1]) if y > 0 else 0            # bucket of y: [lo, hi)
    hi = int(run[y])
    slack = int(tol * S)
    return hi > lo and lo <= thr + slack and thr < hi + slack
