"""Seeded synthetic inputs: model shapes, random weights, prefixes, uniforms.

This module only *generates data* (shapes, value distributions, seeds).  It
holds none of the method's arithmetic: no norm, projection, attention,
softmax, accept rule or sampler lives here.  Both the HIP path and the CPU
reference are fed from it so that they see identical inputs; neither of them
is imported here.

Recipe (stands in for LLaVA-7B weights, the trained 115M drafts and the
image/text benchmarks of Section 4, none of which are available offline):
matrices and embeddings ~ N(0, 0.02^2) rounded to bfloat16, RMSNorm gains 1,
image-position input embeddings ~ N(0, 1), text tokens uniform over the
vocabulary, uniforms on the grid j / 2^24 from a Philox stream.
"""
from dataclasses import dataclass, asdict

import numpy as np
import torch


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    tied_embeddings: bool = False
    rms_eps: float = 1e-6
    rope_theta: float = 1e4

    def n_params(self):
        per_layer = 4 * self.d_model * self.d_model + 3 * self.d_model * self.d_ffn
        emb = self.vocab * self.d_model * (1 if self.tied_embeddings else 2)
        return self.n_layers * per_layer + emb

    def streamed_weight_bytes(self):
        """bf16 bytes one decode/verify step has to read: every layer matrix
        and the LM head once (the embedding table is only gathered)."""
        per_layer = 4 * self.d_model * self.d_model + 3 * self.d_model * self.d_ffn
        return 2 * (self.n_layers * per_layer + self.vocab * self.d_model)


SHAPES = {
    # correctness pair (tiny): target 2 layers d=256, draft 1 layer d=128
    "tiny_target": ModelShape(2, 256, 4, 64, 688, 1024),
    "tiny_draft": ModelShape(1, 128, 2, 64, 344, 1024),
    # ~110M stand-in for the paper's 115M text-only draft
    "draft_110m": ModelShape(12, 768, 12, 64, 2048, 32000, tied_embeddings=True),
    # the paper's own draft shape (Appendix A.1, Table 1), vocab 32000 untied
    "draft_paper_115m": ModelShape(4, 1024, 8, 128, 2816, 32000),
    # LLaMA-7B backbone of LLaVA-7B (Table 1 with hidden dim 4096)
    "llama7b": ModelShape(32, 4096, 32, 128, 11008, 32000),
}


def llama7b_layers(n_layers):
    """LLaMA-7B layer shape with fewer layers (routine parity cases)."""
    base = asdict(SHAPES["llama7b"])
    base["n_layers"] = n_layers
    return ModelShape(**base)


def _tensor_seed(seed, name, layer):
    # a fixed, readable mixing of (seed, tensor name, layer) into a 63-bit seed
    h = np.uint64(1469598103934665603)
    for b in f"{seed}/{name}/{layer}".encode():
        h = np.uint64((int(h) ^ b) * 1099511628211 & 0xFFFFFFFFFFFFFFFF)
    return int(h) & 0x7FFFFFFFFFFFFFFF


def normal_bf16(shape, seed, std, device="cpu"):
    """N(0, std^2) samples rounded to bfloat16 (torch tensor on `device`).

    The stream depends on the device type (torch's CPU and GPU generators
    differ); every consumer of one test gets the same tensor."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return (x * std).to(torch.bfloat16)


def make_weights(shape, seed, std=0.02, device="cpu"):
    """Random-init weights of a LLaMA-style decoder as bf16 torch tensors.

    Layout: row-major [out_features, in_features].  Norm gains are float32
    ones (a 0.02-scale gain would shrink every activation ~50x per norm and
    make any parity check vacuous).
    """
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    hd = shape.n_heads * shape.head_dim

    def mat(name, layer, rows, cols):
        return normal_bf16((rows, cols), _tensor_seed(seed, name, layer), std, device)

    w = {
        "embed": mat("embed", -1, V, d),
        "lm_head": None if shape.tied_embeddings else mat("lm_head", -1, V, d),
        "final_norm": torch.ones(d, dtype=torch.float32, device=device),
        "layers": [],
    }
    for l in range(shape.n_layers):
        w["layers"].append({
            "attn_norm": torch.ones(d, dtype=torch.float32, device=device),
            "wq": mat("wq", l, hd, d),
            "wk": mat("wk", l, hd, d),
            "wv": mat("wv", l, hd, d),
            "wo": mat("wo", l, d, hd),
            "mlp_norm": torch.ones(d, dtype=torch.float32, device=device),
            "w_gate": mat("w_gate", l, F, d),
            "w_up": mat("w_up", l, F, d),
            "w_down": mat("w_down", l, d, F),
        })
    return w


def projected_draft(target_weights, target_shape, draft_shape, seed):
    """A draft whose weights are the target's first layers seen through fixed random orthogonal maps
    (the full-loop benchmark configuration's draft): with R [d_t, d_d] and S [F_t, F_d] of
    orthonormal columns (QR of seeded Gaussians), Wq' = R^T Wq R (likewise Wk, Wv, Wo),
    Wgate' = S^T Wgate R (likewise Wup), Wdown' = R^T Wdown S, E' = E R (tied head), gains 1,
    everything rounded to bf16; the draft's head structure is imposed on the projected
    matrices as they are.  Input tensors may live on any device; the result lives there too.
    """
    dev = target_weights["embed"].device
    dt, dd, Ft, Fd = target_shape.d_model, draft_shape.d_model, target_shape.d_ffn, draft_shape.d_ffn
    assert target_shape.n_heads * target_shape.head_dim == dt and draft_shape.n_heads * draft_shape.head_dim == dd
    assert draft_shape.tied_embeddings and draft_shape.vocab == target_shape.vocab
    assert draft_shape.n_layers <= target_shape.n_layers

    def ortho(rows, cols, name):
        g = torch.Generator().manual_seed(_tensor_seed(seed, name, -1))
        q, _ = torch.linalg.qr(torch.randn((rows, cols), generator=g, dtype=torch.float64))
        return q.to(torch.float32).to(dev)

    R, S = ortho(dt, dd, "proj_R"), ortho(Ft, Fd, "proj_S")
    f = lambda t: t.to(torch.float32)
    b = lambda t: t.to(torch.bfloat16).contiguous()
    w = {"embed": b(f(target_weights["embed"]) @ R), "lm_head": None,
         "final_norm": torch.ones(dd, dtype=torch.float32, device=dev), "layers": []}
    for l in range(draft_shape.n_layers):
        lw = target_weights["layers"][l]
        w["layers"].append({
            "attn_norm": torch.ones(dd, dtype=torch.float32, device=dev),
            "wq": b(R.T @ f(lw["wq"]) @ R), "wk": b(R.T @ f(lw["wk"]) @ R), "wv": b(R.T @ f(lw["wv"]) @ R),
            "wo": b(R.T @ f(lw["wo"]) @ R),
            "mlp_norm": torch.ones(dd, dtype=torch.float32, device=dev),
            "w_gate": b(S.T @ f(lw["w_gate"]) @ R), "w_up": b(S.T @ f(lw["w_up"]) @ R),
            "w_down": b(R.T @ f(lw["w_down"]) @ S),
        })
    return w


def bf16_bits(t):
    """bf16 torch tensor -> numpy uint16 array of its bit patterns (host)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def weights_to_numpy(w):
    """Same weights as plain numpy arrays (uint16 bf16 bits / float32), the
    form the CPU reference takes."""
    def conv(t):
        if t is None:
            return None
        if t.dtype == torch.bfloat16:
            return bf16_bits(t)
        return t.detach().cpu().numpy()
    out = {k: conv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: conv(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


def image_rows(m, d, seed):
    """m image-position input embeddings ~ N(0, 1) (float32 numpy [m, d])."""
    g = torch.Generator().manual_seed(_tensor_seed(seed, "image_rows", m))
    return torch.randn((m, d), generator=g, dtype=torch.float32).numpy()


def text_tokens(n, vocab, seed):
    """n token ids uniform over the vocabulary (int32 numpy)."""
    rng = np.random.Generator(np.random.Philox(key=_tensor_seed(seed, "text", n)))
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def uniforms(shape, seed):
    """float32 uniforms on the grid j / 2^24, j in [0, 2^24), Philox stream."""
    rng = np.random.Generator(np.random.Philox(key=_tensor_seed(seed, "uniform", 0)))
    raw = rng.integers(0, 1 << 32, size=shape, dtype=np.uint64).astype(np.uint32)
    return ((raw >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)


def accept_workload(n_seqs, gamma, vocab, sigma, seed):
    """Logit rows for the accept step in isolation.

    target logits ~ N(0, 2^2) [n_seqs, gamma+1, V]; draft logits = target
    logits of the same position + N(0, sigma^2) [n_seqs, gamma, V]; sigma
    sweeps the acceptance rate.  float32 numpy arrays.
    """
    g = torch.Generator().manual_seed(_tensor_seed(seed, "accept", int(sigma * 1000)))
    lt = torch.randn((n_seqs, gamma + 1, vocab), generator=g, dtype=torch.float32) * 2.0
    noise = torch.randn((n_seqs, gamma, vocab), generator=g, dtype=torch.float32) * float(sigma)
    ld = lt[:, :gamma, :] + noise
    return lt.numpy(), ld.numpy()
