"""The fused QKV + attention kernel at its production width (32 heads of 128, d_model 4096: 256
workgroups that wait for each other per head) against the oracle -- launched call by call, replayed
from a captured graph with new tokens before every replay, and called eagerly right after a capture
(which advances host state without running anything).  The wait between the workgroups takes its
target from device state alone, so every one of these must give the oracle's logits."""
import numpy as np
import pytest
import torch

from oracle import decoder as dec
from paper_2404_08856_amd import synth
from tests.helpers import check_logits, oracle_cfg, randomize_gains, to_device

pytestmark = pytest.mark.gpu

P0 = 37          # prefix positions (text only: the oracle's cost grows with the prefix)


@pytest.fixture(scope="module")
def pair():
    from paper_2404_08856_amd import spd
    shape = synth.llama7b_layers(2)                    # Table 1 target layer shape, 2 layers
    print("building the 2-layer 7B-shape pair", flush=True)
    w = randomize_gains(synth.make_weights(shape, 77))
    model = spd.Model(spd.make_config(shape, 1, 64), to_device(w))
    wn = synth.weights_to_numpy(w)
    del w
    cfg = oracle_cfg(shape)
    cache = dec.KVCache(cfg, 64)
    toks = synth.text_tokens(P0, shape.vocab, 77)
    ref_last = dec.forward_tokens(cfg, wn, cache, toks)[-1]
    last = torch.empty(shape.vocab, dtype=torch.float32, device="cuda")
    model.spd_prefill_tokens(0, torch.from_numpy(toks).cuda(), last)
    check_logits(last.cpu().numpy(), ref_last, "prefill")
    yield model, wn, cfg, cache, shape
    model.close()


def oracle_step(cfg, wn, cache, tokens):
    cache.truncate(P0)
    return dec.forward_tokens(cfg, wn, cache, tokens)


@pytest.mark.parametrize("M", [5, 6, 8])
def test_fused_kernel_at_32_heads_eager(pair, M):
    """M = 5: one row group, 12 waves; M = 6, 8: the two-row-group variant (8 waves, two query groups)."""
    model, wn, cfg, cache, shape = pair
    print(f"case fused 32 heads eager M={M}", flush=True)
    out = torch.empty((1, M, shape.vocab), dtype=torch.float32, device="cuda")
    for step in range(2):
        toks = synth.text_tokens(M, shape.vocab, 1000 + 10 * M + step)
        model.spd_kv_set_len([P0])
        model.spd_verify_forward(torch.from_numpy(toks).cuda()[None].contiguous(), out)
        check_logits(out.cpu().numpy()[0], oracle_step(cfg, wn, cache, toks), f"M={M} step {step}")
    model.spd_device_status()


@pytest.mark.parametrize("M", [5, 8])
def test_fused_kernel_graph_replays_with_new_tokens_match_the_oracle(pair, M):
    model, wn, cfg, cache, shape = pair
    print(f"case fused 32 heads graph M={M}", flush=True)
    vt = torch.zeros((1, M), dtype=torch.int32, device="cuda")
    out = torch.empty((1, M, shape.vocab), dtype=torch.float32, device="cuda")

    def run_eager(seed, what):
        toks = synth.text_tokens(M, shape.vocab, seed)
        vt.copy_(torch.from_numpy(toks)[None])
        model.spd_kv_set_len([P0])
        out.zero_()
        model.spd_verify_forward(vt, out)
        torch.cuda.synchronize()
        check_logits(out.cpu().numpy()[0], oracle_step(cfg, wn, cache, toks), what)

    run_eager(2000 + M, "eager before capture")
    # warm-up on a side stream, as the capture API asks
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        model.spd_kv_set_len([P0])
        model.spd_verify_forward(vt, out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    model.spd_kv_set_len([P0])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.spd_verify_forward(vt, out)
    # the capture enqueued nothing; an eager call right after it must still be synchronised correctly
    run_eager(2100 + M, "eager right after the capture")
    for rep in range(4):
        toks = synth.text_tokens(M, shape.vocab, 2200 + 10 * M + rep)
        vt.copy_(torch.from_numpy(toks)[None])
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        check_logits(out.cpu().numpy()[0], oracle_step(cfg, wn, cache, toks), f"replay {rep}")
        if rep % 2 == 0:                                # eager work between replays
            run_eager(2300 + 10 * M + rep, f"eager between replays {rep}")
    model.spd_device_status()
    model.spd_kv_set_len([P0])


def test_wait_spin_limit_is_reported_and_every_kernel_exits():
    """Failure path of the wait between workgroups, driven from the host: with a spin limit of one poll a
    workgroup that has to wait gives up at once, the kernel finishes normally (results meaningless, every
    access in bounds) and spd_device_status reports it."""
    from paper_2404_08856_amd import spd
    shape = synth.ModelShape(1, 4096, 32, 128, 256, 1024)
    model = spd.Model(spd.make_config(shape, 1, 32), to_device(synth.make_weights(shape, 5)))
    model.spd_prefill_tokens(0, torch.from_numpy(synth.text_tokens(9, shape.vocab, 5)).cuda())
    model.spd_device_status()
    model.spd_model_set_tuning(wait_spin_limit=1)
    out = torch.empty((1, 5, shape.vocab), dtype=torch.float32, device="cuda")
    vt = torch.from_numpy(synth.text_tokens(5, shape.vocab, 6)).cuda()[None].contiguous()
    tripped = False
    for _ in range(20):                                 # a wait that lasts longer than one poll happens within a few calls
        model.spd_kv_set_len([9])
        model.spd_verify_forward(vt, out)
        torch.cuda.synchronize()
        try:
            model.spd_device_status()
        except spd.SpdError as e:
            assert e.code == spd.SPD_ERR_HIP
            tripped = True
            break
    assert tripped
    model.close()


def test_batched_projection_kernel_graph_replays_match_the_oracle():
    """The batched projection kernel keeps its arrival counters on the device (the last arriver of a tile group
    clears its counter), so a captured 20-row call can be replayed any number of times: 4 sequences x 5 rows on a
    model with K-sliced matrices (d_model 4096), new tokens before every replay, eager calls in between."""
    from paper_2404_08856_amd import spd
    shape = synth.ModelShape(1, 4096, 2, 128, 3072, 1024)
    n_seqs, M, cap = 4, 5, 48
    print("case batched kernel graph replay", flush=True)
    w = randomize_gains(synth.make_weights(shape, 58))
    model = spd.Model(spd.make_config(shape, n_seqs, cap), to_device(w))
    model.spd_model_set_tuning(batch_kernel=1)
    wn = synth.weights_to_numpy(w)
    del w
    cfg = oracle_cfg(shape)
    caches, lens = [], []
    for s in range(n_seqs):
        toks = synth.text_tokens(3 + 4 * s, shape.vocab, 500 + s)
        c = dec.KVCache(cfg, cap)
        dec.forward_tokens(cfg, wn, c, toks)
        caches.append(c)
        lens.append(len(toks))
        model.spd_prefill_tokens(s, torch.from_numpy(toks).cuda())
    vt = torch.zeros((n_seqs, M), dtype=torch.int32, device="cuda")
    out = torch.empty((n_seqs, M, shape.vocab), dtype=torch.float32, device="cuda")

    def check(toks, what):
        got = out.cpu().numpy()
        for s in range(n_seqs):
            caches[s].truncate(lens[s])
            check_logits(got[s], dec.forward_tokens(cfg, wn, caches[s], toks[s]), f"{what} seq {s}")

    def run_eager(seed, what):
        toks = synth.text_tokens(n_seqs * M, shape.vocab, seed).reshape(n_seqs, M)
        vt.copy_(torch.from_numpy(toks))
        model.spd_kv_set_len(lens)
        out.zero_()
        model.spd_verify_forward(vt, out)
        torch.cuda.synchronize()
        check(toks, what)

    run_eager(3000, "eager before capture")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        model.spd_kv_set_len(lens)
        model.spd_verify_forward(vt, out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    model.spd_kv_set_len(lens)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.spd_verify_forward(vt, out)
    run_eager(3100, "eager right after the capture")
    for rep in range(4):
        toks = synth.text_tokens(n_seqs * M, shape.vocab, 3200 + rep).reshape(n_seqs, M)
        vt.copy_(torch.from_numpy(toks))
        model.spd_kv_set_len(lens)                      # host-side lengths: the captured call reads them at capture time
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        check(toks, f"replay {rep}")
        if rep % 2 == 0:
            run_eager(3300 + rep, f"eager between replays {rep}")
    model.spd_device_status()
    model.close()
