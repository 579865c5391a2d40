"""spd_speculative_accept_static (scratch memory inside the library, nothing allocated) against
spd_speculative_accept (caller's workspace): same k, y and accept probabilities bit for bit, on two calls in
a row, the second with a smaller input (so the shared array still holds the first call's larger contents)."""
import numpy as np
import pytest
import torch

from paper_2404_08856_amd import synth

pytestmark = pytest.mark.gpu


def both_ways(spd, n_seqs, gamma, V, seed, flags, probs):
    lt, ld = synth.accept_workload(n_seqs, gamma, V, 1.0, seed=seed)
    t, d = torch.from_numpy(lt).cuda(), torch.from_numpy(ld).cuda()
    if probs:
        t, d = torch.softmax(t, -1).contiguous(), torch.softmax(d, -1).contiguous()
    g = torch.Generator(device="cuda").manual_seed(seed)
    dtok = torch.multinomial(torch.softmax(torch.from_numpy(ld).cuda().reshape(-1, V), -1), 1, generator=g).to(torch.int32).reshape(n_seqs, gamma)
    u = torch.from_numpy(synth.uniforms((n_seqs, gamma + 1), seed + 1)).cuda()
    res = []
    for static in (False, True):
        k = torch.full((n_seqs,), -5, dtype=torch.int32, device="cuda")
        y = torch.full((n_seqs,), -5, dtype=torch.int32, device="cuda")
        ap = torch.full((n_seqs, gamma), -5.0, dtype=torch.float32, device="cuda")
        if static:
            spd.spd_speculative_accept_static(t, d, dtok, u, 0.9, flags, k, y, ap)
        else:
            spd.spd_speculative_accept(t, d, dtok, u, 0.9, flags, k, y, ap)
        torch.cuda.synchronize()
        res.append((k.cpu().numpy(), y.cpu().numpy(), ap.cpu().numpy()))
    return res


def test_accept_without_allocation_equals_the_workspace_call_twice_in_a_row():
    from paper_2404_08856_amd import spd
    # first call: 64 sequences x (gamma 4) x 32000 logits; second call right after: 3 sequences x (gamma 2) x 1000
    for n_seqs, gamma, V, seed, flags, probs in ((64, 4, 32000, 21, 0, False), (3, 2, 1000, 22, 0, False),
                                                 (5, 3, 2048, 23, spd.SPD_TARGET_IS_PROBS | spd.SPD_DRAFT_IS_PROBS, True)):
        (k0, y0, ap0), (k1, y1, ap1) = both_ways(spd, n_seqs, gamma, V, seed, flags, probs)
        assert np.array_equal(k0, k1) and np.array_equal(y0, y1) and np.array_equal(ap0, ap1), (n_seqs, gamma, V)
        assert k0.min() >= 0 and y0.min() >= 0 and y0.max() < V


def test_accept_without_allocation_rejects_sizes_beyond_its_array():
    from paper_2404_08856_amd import spd
    n_seqs, gamma, V = 64, 40, 16                          # 64 * 81 = 5184 rows > 4096
    t = torch.zeros((n_seqs, gamma + 1, V), dtype=torch.float32, device="cuda")
    d = torch.zeros((n_seqs, gamma, V), dtype=torch.float32, device="cuda")
    dtok = torch.zeros((n_seqs, gamma), dtype=torch.int32, device="cuda")
    u = torch.zeros((n_seqs, gamma + 1), dtype=torch.float32, device="cuda")
    k = torch.zeros((n_seqs,), dtype=torch.int32, device="cuda")
    y = torch.zeros((n_seqs,), dtype=torch.int32, device="cuda")
    with pytest.raises(spd.SpdError) as e:
        spd.spd_speculative_accept_static(t, d, dtok, u, 1.0, 0, k, y)
    assert e.value.code == spd.SPD_ERR_CAPACITY and "4096" in str(e.value)
