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
