"""GPU parity of the whole speculative-decoding block loop (Section 2.1 + Section 3):
gamma draft steps, one target call over gamma + 1 tokens, accept / resample, rollback of
both KV caches -- every step through the C ABI, with the host only sequencing the calls.

The oracle runs beside the device in lock step on the device's own token history (two
float paths that agree to 3e-2 in the logits may still draw different tokens, after which
the histories would no longer be comparable).  The oracle side keeps NO cache: every
reference row is a recompute from scratch over the true history (prompt, every token
emitted so far, this block's drafted tokens before the row; the draft without the image
rows), so a mistake in the rollback bookkeeping cannot be mirrored on both sides.  Per
block it checks

  * the draft rows D_j and the target logits against that recompute (spec tolerance),
  * every drafted token against the oracle's sampler applied to the device's own D_j with
    the same uniform (bit-exact),
  * (k, y) against the oracle's accept / resample on the same T, D, tokens and uniforms
    (bit-exact),
  * the cache lengths after the rollback.
"""
import numpy as np
import pytest
import torch

from oracle import decoder as dec
from oracle import spec_sampling as ss
from paper_2404_08856_amd import synth
from tests.helpers import accept_margins, check_logits, drawn_token_is_valid, oracle_cfg, randomize_gains, to_device

pytestmark = pytest.mark.gpu


def spd_mod():
    from paper_2404_08856_amd import spd
    return spd


def make_pair(t_shape, d_shape, seed, cap, aligned, noise):
    """target + draft; `aligned` makes the draft a perturbed copy of the target so that
    a useful share of the drafts is accepted (needs equal shapes)."""
    spd = spd_mod()
    tw = randomize_gains(synth.make_weights(t_shape, seed))
    if aligned:
        dw = randomize_gains(synth.make_weights(d_shape, seed))
        g = torch.Generator().manual_seed(seed + 1)
        noise = torch.randn(dw["lm_head"].shape, generator=g) * noise
        dw["lm_head"] = (dw["lm_head"].float() + noise).to(torch.bfloat16)
    else:
        dw = randomize_gains(synth.make_weights(d_shape, seed + 50), seed=5)
    target = spd.Model(spd.make_config(t_shape, 1, cap), to_device(tw))
    draft = spd.Model(spd.make_config(d_shape, 1, cap), to_device(dw))
    return target, draft, synth.weights_to_numpy(tw), synth.weights_to_numpy(dw)


def draft_row_ref(dc, dwn, history, temperature):
    """D(. | history): the draft's distribution after the text-only history, recomputed from an empty cache."""
    x = dec.embed_tokens(dwn, np.asarray(history, dtype=np.int64))
    return dec.full_recompute(dc, dwn, x)[-1]


def target_rows_ref(tc, twn, image, history, n_last):
    """Target logits of the last n_last positions of [image rows ; E[history]], recomputed from an empty cache."""
    x = dec.embed_tokens(twn, np.asarray(history, dtype=np.int64))
    if image is not None:
        x = np.concatenate([image.astype(np.float64), x])
    return dec.full_recompute(tc, twn, x)[-n_last:]


def check_draft_row(D_j, ref_logits, temperature):
    D_ref = ss.softmax_probs(ref_logits, temperature)
    if temperature > 0:
        big = D_ref > 1e-12
        assert np.max(np.abs(np.log(D_j[big].astype(np.float64)) - np.log(D_ref[big].astype(np.float64)))) < 2 * 3e-2 / temperature
    else:                                                  # greedy: one-hot rows; the argmax may differ only at a near-tie
        top = np.sort(ref_logits)[-2:]
        assert D_j.sum() == 1.0 and (int(np.argmax(D_j)) == int(np.argmax(ref_logits)) or top[1] - top[0] < 6e-2)


def run_loop(t_shape, d_shape, m_img, n_text, gamma, n_blocks, temperature, seed, aligned, noise=0.02):
    spd = spd_mod()
    cap = m_img + n_text + n_blocks * (gamma + 1) + 8
    target, draft, twn, dwn = make_pair(t_shape, d_shape, seed, cap, aligned, noise)
    tc, dc = oracle_cfg(t_shape), oracle_cfg(d_shape)
    V = t_shape.vocab
    toks = synth.text_tokens(n_text, V, seed)
    image = None if m_img == 0 else synth.image_rows(m_img, t_shape.d_model, seed)

    # prefill: target sees [image rows ; text], the draft the text alone (Section 3)
    x_text = dec.embed_tokens(twn, toks)
    x = x_text if m_img == 0 else np.concatenate([image.astype(np.float64), x_text])
    ref_last = target_rows_ref(tc, twn, image, toks, 1)[0]
    last = torch.empty(V, dtype=torch.float32, device="cuda")
    target.spd_prefill(0, torch.from_numpy(x.astype(np.float32)).cuda(), last)
    draft.spd_prefill_tokens(0, torch.from_numpy(toks).cuda())
    check_logits(last.cpu().numpy(), ref_last, "prefill")

    u_first = synth.uniforms((1,), seed + 1)[0]
    u_draft = synth.uniforms((n_blocks, gamma), seed + 2)
    u_accept = synth.uniforms((n_blocks, gamma + 1), seed + 3)
    t = ss.sample_row(ss.softmax_probs(last.cpu().numpy(), temperature), u_first)

    D_dev = torch.empty((1, gamma, V), dtype=torch.float32, device="cuda")
    tok_dev = torch.empty((1,), dtype=torch.int32, device="cuda")
    logits_dev = torch.empty((1, gamma + 1, V), dtype=torch.float32, device="cuda")
    k_dev = torch.empty((1,), dtype=torch.int32, device="cuda")
    y_dev = torch.empty((1,), dtype=torch.int32, device="cuda")
    pending = [t]
    out, ks = [t], []
    history = [int(x) for x in toks]                       # text prompt + every emitted token before t
    for b in range(n_blocks):
        print(f"loop block {b} t={t} pending={pending}", flush=True)
        d_tokens = []
        for j in range(gamma):
            ref = draft_row_ref(dc, dwn, history + [t] + d_tokens, temperature)
            draft.spd_draft_step(torch.tensor([pending], dtype=torch.int32, device="cuda"), temperature,
                                 torch.from_numpy(u_draft[b, j:j + 1]).cuda(), D_dev[:, j], tok_dev)
            D_j = D_dev[0, j].cpu().numpy()
            check_draft_row(D_j, ref, temperature)
            d_j = int(tok_dev.item())
            assert d_j == ss.sample_row(D_j, u_draft[b, j]), (b, j)
            d_tokens.append(d_j)
            pending = [d_j]
        block = [t] + d_tokens
        ref_t = target_rows_ref(tc, twn, image, history + block, gamma + 1)
        target.spd_verify_forward(torch.tensor([block], dtype=torch.int32, device="cuda"), logits_dev)
        lg = logits_dev[0].cpu().numpy()
        check_logits(lg, ref_t, f"verify block {b}")
        # accept on exactly the rows the oracle sees: T from the device logits, D from the draft steps
        T_rows = ss.softmax_probs(lg, temperature)
        D_rows = D_dev[0].cpu().numpy()
        spd.spd_speculative_accept(torch.from_numpy(T_rows).cuda()[None].contiguous(), D_dev,
                                   torch.tensor([d_tokens], dtype=torch.int32, device="cuda"),
                                   torch.from_numpy(u_accept[b:b + 1]).cuda(), temperature,
                                   spd.SPD_TARGET_IS_PROBS | spd.SPD_DRAFT_IS_PROBS, k_dev, y_dev)
        k, y = int(k_dev.item()), int(y_dev.item())
        assert (k, y) == ss.speculative_accept(T_rows, D_rows, d_tokens, u_accept[b]), b
        # the product call (target given as logits) must take the same decision away from ties
        k2 = torch.empty_like(k_dev)
        y2 = torch.empty_like(y_dev)
        spd.spd_speculative_accept(logits_dev, D_dev, torch.tensor([d_tokens], dtype=torch.int32, device="cuda"),
                                   torch.from_numpy(u_accept[b:b + 1]).cuda(), temperature,
                                   spd.SPD_DRAFT_IS_PROBS, k2, y2)
        if min(accept_margins(T_rows, D_rows, d_tokens, u_accept[b])) > 1e-3:
            assert int(k2.item()) == k, b
        assert drawn_token_is_valid(T_rows, D_rows, int(k2.item()), u_accept[b, gamma], int(y2.item())), b
        # rollback: target keeps t, d_1..d_k; draft keeps t, d_1..d_min(k, gamma-1).  Expected lengths follow
        # from the history alone: the target holds image + everything before y, the draft the text before y
        # minus the drafted token it has not consumed yet after a full acceptance
        history = history + [t] + d_tokens[:k]
        t_len = m_img + len(history)
        d_len = len(history) - (1 if k == gamma else 0)
        target.spd_kv_set_len([t_len])
        draft.spd_kv_set_len([d_len])
        pending = [d_tokens[gamma - 1], y] if k == gamma else [y]
        out.extend(d_tokens[:k])
        out.append(y)
        ks.append(k)
        t = y
    target.close()
    draft.close()
    return out, ks


def test_block_loop_text_only_draft_sampling():
    # tiny correctness configuration: 32 image rows + 32 text tokens, gamma 4, independent draft
    out, ks = run_loop(synth.SHAPES["tiny_target"], synth.SHAPES["tiny_draft"], 32, 32, 4, 6, 1.0, 21, False)
    assert len(out) == 1 + sum(k + 1 for k in ks)


def test_block_loop_aligned_draft_accepts_and_double_input_path():
    # a draft that mostly agrees with the target: exercises k = gamma (two-token draft input)
    out, ks = run_loop(synth.SHAPES["tiny_target"], synth.SHAPES["tiny_target"], 0, 24, 3, 8, 1.0, 22, True)
    print("accepted per block", ks)
    assert max(ks) == 3 and min(ks) < 3


def test_block_loop_greedy_equals_autoregressive_on_device():
    """Greedy SPD reproduces greedy autoregressive decoding of the target token for token
    (Section 2.1: the output distribution is the target's); both run on the device."""
    spd = spd_mod()
    shape = synth.SHAPES["tiny_target"]
    gamma, n_blocks, seed = 4, 6, 23
    out, ks = run_loop(shape, shape, 8, 16, gamma, n_blocks, 0.0, seed, True, noise=0.004)
    cap = 8 + 16 + len(out) + 8
    tw = randomize_gains(synth.make_weights(shape, seed))
    model = spd.Model(spd.make_config(shape, 1, cap), to_device(tw))
    twn = synth.weights_to_numpy(tw)
    x = np.concatenate([synth.image_rows(8, shape.d_model, seed).astype(np.float64),
                        dec.embed_tokens(twn, synth.text_tokens(16, shape.vocab, seed))])
    last = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    model.spd_prefill(0, torch.from_numpy(x.astype(np.float32)).cuda(), last)
    ar = [int(torch.argmax(last).item())]
    lg = torch.empty((1, 1, shape.vocab), dtype=torch.float32, device="cuda")
    margins = []
    while len(ar) < len(out):
        model.spd_verify_forward(torch.tensor([[ar[-1]]], dtype=torch.int32, device="cuda"), lg)
        top = torch.topk(lg[0, 0], 2).values
        margins.append(float(top[0] - top[1]))
        ar.append(int(torch.argmax(lg[0, 0]).item()))
    model.close()
    print("greedy accepted per block", ks, "min top-2 margin", min(margins))
    # M = 1 and M = gamma + 1 calls sum in different orders; only a margin far above that noise is decisive
    first_unsafe = next((i for i, mg in enumerate(margins) if mg < 1e-3), len(margins))
    assert out[:first_unsafe + 1] == ar[:first_unsafe + 1]
    assert first_unsafe >= len(margins) // 2


# ---------------------------------------------------------------------------------------------
# the block loop with KV lengths, tokens and the commit kept on the device
# ---------------------------------------------------------------------------------------------
class DeviceLoop:
    """Buffers and the fixed launch sequence of one block (what a HIP graph captures)."""

    def __init__(self, target, draft, n_seqs, gamma, V, temperature, out_cap):
        self.spd = spd_mod()
        self.target, self.draft, self.n_seqs, self.gamma, self.V, self.temperature = target, draft, n_seqs, gamma, V, temperature
        dev = "cuda"
        self.vt = torch.zeros((n_seqs, gamma + 1), dtype=torch.int32, device=dev)        # t, d_1 .. d_gamma
        self.din = torch.zeros((n_seqs, 2), dtype=torch.int32, device=dev)               # draft's first inputs
        self.D = torch.zeros((n_seqs, gamma, V), dtype=torch.float32, device=dev)
        self.logits = torch.zeros((n_seqs, gamma + 1, V), dtype=torch.float32, device=dev)
        self.u_draft = torch.zeros((n_seqs, gamma), dtype=torch.float32, device=dev)     # this block's uniforms (staging)
        self.u_accept = torch.zeros((n_seqs, gamma + 1), dtype=torch.float32, device=dev)
        self.k = torch.zeros((n_seqs,), dtype=torch.int32, device=dev)
        self.y = torch.zeros((n_seqs,), dtype=torch.int32, device=dev)
        self.out = torch.zeros((n_seqs, out_cap), dtype=torch.int32, device=dev)
        self.n_out = torch.zeros((n_seqs,), dtype=torch.int32, device=dev)
        self.ws = torch.empty(self.spd.spd_accept_workspace_bytes(n_seqs, gamma, V), dtype=torch.uint8, device=dev)

    def block(self):
        g, V, n = self.gamma, self.V, self.n_seqs
        vt_flat, D_flat, u_flat = self.vt.view(-1), self.D.view(-1), self.u_draft.view(-1)
        self.draft.spd_draft_step_strided(self.din, 2, n, 2, self.temperature, u_flat, g, D_flat, g * V, vt_flat[1:], g + 1)
        for j in range(1, g):
            self.draft.spd_draft_step_strided(vt_flat[j:], g + 1, n, 1, self.temperature, u_flat[j:], g,
                                              D_flat[j * V:], g * V, vt_flat[j + 1:], g + 1)
        self.target.spd_verify_forward(self.vt, self.logits)
        self.spd.spd_block_finish(self.target, self.draft, self.logits, self.D, self.vt, self.u_accept, self.temperature,
                                  self.k, self.y, self.din, self.out, self.n_out, self.ws)


def setup_device_loop(n_seqs, gamma, n_blocks, temperature, seed, m_img):
    """Prefill target ([image ; text]) and draft (text) for n_seqs ragged prompts, on device and in the oracle."""
    spd = spd_mod()
    t_shape, d_shape = synth.SHAPES["tiny_target"], synth.SHAPES["tiny_draft"]
    V = t_shape.vocab
    cap = m_img + 12 + 9 * n_seqs + n_blocks * (gamma + 1) + 8
    tw = randomize_gains(synth.make_weights(t_shape, seed))
    dw = randomize_gains(synth.make_weights(d_shape, seed + 50), seed=5)
    target = spd.Model(spd.make_config(t_shape, n_seqs, cap), to_device(tw))
    draft = spd.Model(spd.make_config(d_shape, n_seqs, cap), to_device(dw))
    twn, dwn = synth.weights_to_numpy(tw), synth.weights_to_numpy(dw)
    tc, dc = oracle_cfg(t_shape), oracle_cfg(d_shape)
    loop = DeviceLoop(target, draft, n_seqs, gamma, V, temperature, n_blocks * (gamma + 1))
    oracle = []
    u_first = synth.uniforms((n_seqs,), seed + 1)
    for s in range(n_seqs):
        n_text = 12 + 9 * s
        toks = synth.text_tokens(n_text, V, seed + s)
        image = synth.image_rows(m_img, t_shape.d_model, seed + s)
        x = np.concatenate([image.astype(np.float64), dec.embed_tokens(twn, toks)])
        ref_last = target_rows_ref(tc, twn, image, toks, 1)[0]
        last = torch.empty(V, dtype=torch.float32, device="cuda")
        target.spd_prefill(s, torch.from_numpy(x.astype(np.float32)).cuda(), last)
        draft.spd_prefill_tokens(s, torch.from_numpy(toks).cuda())
        check_logits(last.cpu().numpy(), ref_last, f"prefill seq {s}")
        t = ss.sample_row(ss.softmax_probs(last.cpu().numpy(), temperature), u_first[s])
        # history = text prompt + every emitted token before t (the oracle side keeps no cache)
        oracle.append(dict(image=image, history=[int(v) for v in toks], t=t, out=[]))
        loop.vt[s, 0] = t
        loop.din[s, 0] = int(toks[-1])
        loop.din[s, 1] = t
    # loop convention: the draft's cache ends before the token that precedes t
    draft.spd_kv_set_len([len(o["history"]) - 1 for o in oracle])
    target.spd_kv_lens_to_device()
    draft.spd_kv_lens_to_device()
    return loop, oracle, (tc, twn, dc, dwn, m_img)


def expected_lengths(oracle, m_img):
    """KV lengths the loop convention implies for the current histories: the target holds image + everything
    before t, the draft the text before the token that precedes t."""
    return [m_img + len(o["history"]) for o in oracle], [len(o["history"]) - 1 for o in oracle]


def check_block_against_oracle(loop, oracle, models, u_draft_b, u_accept_b, b):
    tc, twn, dc, dwn, m_img = models
    g, temperature = loop.gamma, loop.temperature
    D_all, lg_all = loop.D.cpu().numpy(), loop.logits.cpu().numpy()
    k_all, y_all = loop.k.cpu().numpy(), loop.y.cpu().numpy()
    ks = []
    for s, o in enumerate(oracle):
        d_tokens = []
        for j in range(g):
            ref = draft_row_ref(dc, dwn, o["history"] + [o["t"]] + d_tokens, temperature)
            D_j = D_all[s, j]
            check_draft_row(D_j, ref, temperature)
            d_j = ss.sample_row(D_j, u_draft_b[s, j])          # the device must have drawn exactly this token
            d_tokens.append(d_j)
        ref_t = target_rows_ref(tc, twn, o["image"], o["history"] + [o["t"]] + d_tokens, g + 1)
        check_logits(lg_all[s], ref_t, f"block {b} seq {s}")
        # the product decides on its own float32 softmax of the logits; the oracle's float64 softmax of the
        # same logits may differ at near-ties only
        T_rows = ss.softmax_probs(lg_all[s], temperature)
        k_ref, y_ref = ss.speculative_accept(T_rows, D_all[s], d_tokens, u_accept_b[s])
        k, y = int(k_all[s]), int(y_all[s])
        if min(accept_margins(T_rows, D_all[s], d_tokens, u_accept_b[s])) > 1e-3:
            assert k == k_ref, (b, s, k, k_ref)
        if temperature > 0:
            assert drawn_token_is_valid(T_rows, D_all[s], k, u_accept_b[s, g], y), (b, s, k, y, k_ref, y_ref)
        else:                                              # greedy: y = argmax of the target row, up to a near-tie of the logits
            top = np.sort(lg_all[s][k])[-2:]
            assert y == int(np.argmax(lg_all[s][k])) or top[1] - top[0] < 1e-5, (b, s, k, y)
        emitted = d_tokens[:k] + [y]
        o["out"].extend(emitted)
        o["history"] = o["history"] + [o["t"]] + d_tokens[:k]
        o["t"] = y
        ks.append(k)
    return ks


@pytest.mark.parametrize("n_seqs,gamma,temperature", [(1, 4, 1.0), (3, 3, 1.0), (2, 5, 1.0), (8, 7, 1.0), (2, 4, 0.0), (2, 3, 0.6)])
def test_device_block_loop_lockstep(n_seqs, gamma, temperature):
    """No host decision between blocks: lengths, tokens and the commit stay on the device."""
    n_blocks, seed = 6, 31
    loop, oracle, models = setup_device_loop(n_seqs, gamma, n_blocks, temperature, seed, m_img=16)
    u_draft = synth.uniforms((n_blocks, n_seqs, gamma), seed + 2)
    u_accept = synth.uniforms((n_blocks, n_seqs, gamma + 1), seed + 3)
    all_ks = []
    for b in range(n_blocks):
        print(f"device loop block {b}", flush=True)
        loop.u_draft.copy_(torch.from_numpy(u_draft[b]))
        loop.u_accept.copy_(torch.from_numpy(u_accept[b]))
        loop.block()
        all_ks.append(check_block_against_oracle(loop, oracle, models, u_draft[b], u_accept[b], b))
    print("accepted per block", all_ks)
    loop.target.spd_kv_lens_from_device()
    loop.draft.spd_kv_lens_from_device()
    t_lens, d_lens = expected_lengths(oracle, 16)
    assert loop.target.spd_kv_get_len(n_seqs) == t_lens
    assert loop.draft.spd_kv_get_len(n_seqs) == d_lens
    n_out = loop.n_out.cpu().numpy()
    out = loop.out.cpu().numpy()
    for s, o in enumerate(oracle):
        assert n_out[s] == len(o["out"]) and list(out[s, :n_out[s]]) == o["out"]
    loop.target.close()
    loop.draft.close()


def test_device_block_loop_as_graph_replays_equal_eager():
    """One block captured in a graph and replayed: every replay (with eager copies of the next
    uniforms and host synchronisation in between) gives what the eager launches give."""
    n_seqs, gamma, n_blocks, temperature, seed = 2, 4, 5, 1.0, 37
    u_draft = synth.uniforms((n_blocks, n_seqs, gamma), seed + 2)
    u_accept = synth.uniforms((n_blocks, n_seqs, gamma + 1), seed + 3)
    results = {}
    for mode in ("eager", "graph"):
        loop, oracle, _ = setup_device_loop(n_seqs, gamma, n_blocks + 2, temperature, seed, m_img=8)
        graph = None
        if mode == "graph":
            # warm-up launches on a side stream (as the capture API asks), then restore the state they changed
            saved = [t.clone() for t in (loop.vt, loop.din, loop.out, loop.n_out)]
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                loop.block()
            torch.cuda.current_stream().wait_stream(s)
            torch.cuda.synchronize()
            loop.target.spd_kv_lens_from_device()
            loop.draft.spd_kv_lens_from_device()
            t_lens, d_lens = expected_lengths(oracle, 8)
            loop.target.spd_kv_set_len(t_lens)
            loop.draft.spd_kv_set_len(d_lens)
            loop.target.spd_kv_lens_to_device()
            loop.draft.spd_kv_lens_to_device()
            for t, sv in zip((loop.vt, loop.din, loop.out, loop.n_out), saved):
                t.copy_(sv)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                loop.block()
            # capture runs nothing: state is still the restored one
        ks, ys = [], []
        for b in range(n_blocks):
            loop.u_draft.copy_(torch.from_numpy(u_draft[b]))
            loop.u_accept.copy_(torch.from_numpy(u_accept[b]))
            if graph is None:
                loop.block()
            else:
                graph.replay()
            torch.cuda.synchronize()
            ks.append(loop.k.cpu().numpy().copy())
            ys.append(loop.y.cpu().numpy().copy())
        loop.target.spd_kv_lens_from_device()
        loop.draft.spd_kv_lens_from_device()
        results[mode] = (np.stack(ks), np.stack(ys), loop.out.cpu().numpy().copy(), loop.n_out.cpu().numpy().copy(),
                         loop.target.spd_kv_get_len(n_seqs), loop.draft.spd_kv_get_len(n_seqs), loop.logits.cpu().numpy().copy())
        loop.target.close()
        loop.draft.close()
    for a, b in zip(results["eager"], results["graph"]):
        assert np.array_equal(np.asarray(a), np.asarray(b))
    assert results["eager"][3].min() >= n_blocks
