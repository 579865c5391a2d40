"""The seeded input generators (shared by the oracle and the device path; no arithmetic of the method)."""
import numpy as np
import torch

from paper_2404_08856_amd import synth


def test_generators_are_deterministic_and_seed_dependent():
    shape = synth.SHAPES["tiny_draft"]
    a, b, c = synth.make_weights(shape, 3), synth.make_weights(shape, 3), synth.make_weights(shape, 4)
    assert torch.equal(a["layers"][0]["wq"], b["layers"][0]["wq"]) and not torch.equal(a["layers"][0]["wq"], c["layers"][0]["wq"])
    assert not torch.equal(a["layers"][0]["wq"], a["layers"][0]["wk"])          # one stream per tensor
    assert np.array_equal(synth.text_tokens(50, 1024, 1), synth.text_tokens(50, 1024, 1))
    u = synth.uniforms((1000,), 5)
    assert u.dtype == np.float32 and u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2.0 ** 24 == np.round(u * 2.0 ** 24))                      # on the 2^-24 grid
    lt, ld = synth.accept_workload(4, 3, 256, 1.0, seed=2)
    assert lt.shape == (4, 4, 256) and ld.shape == (4, 3, 256)
    assert abs(float(lt.std()) - 2.0) < 0.1 and abs(float((ld - lt[:, :3]).std()) - 1.0) < 0.1


def test_weights_have_the_stated_distribution():
    w = synth.make_weights(synth.SHAPES["tiny_target"], 0)
    x = w["layers"][1]["w_gate"].float()
    assert abs(float(x.std()) - 0.02) < 1e-3 and abs(float(x.mean())) < 1e-3
    assert torch.all(w["layers"][0]["attn_norm"] == 1.0) and torch.all(w["final_norm"] == 1.0)


def test_projected_draft_keeps_scale_and_is_a_projection():
    ts = synth.ModelShape(2, 256, 4, 64, 688, 1024)
    ds = synth.ModelShape(1, 128, 2, 64, 344, 1024, tied_embeddings=True)
    tw = synth.make_weights(ts, 0)
    d1, d2 = synth.projected_draft(tw, ts, ds, 1), synth.projected_draft(tw, ts, ds, 1)
    lw = d1["layers"][0]
    assert lw["wq"].shape == (128, 128) and lw["w_gate"].shape == (344, 128) and lw["w_down"].shape == (128, 344)
    assert d1["embed"].shape == (1024, 128) and d1["lm_head"] is None
    assert torch.equal(lw["wo"], d2["layers"][0]["wo"])
    # orthonormal maps keep the N(0, 0.02) scale of every matrix
    for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        assert abs(float(lw[k].float().std()) - 0.02) < 2e-3, k
    # projecting E with R: the Gram matrix of E R equals R^T (E^T E) R, in particular its trace is bounded by that of E^T E
    E, Ed = tw["embed"].float(), d1["embed"].float()
    assert float((Ed * Ed).sum()) <= float((E * E).sum()) * 1.001
