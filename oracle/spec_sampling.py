"""Oracle: speculative sampling (TEST INFRASTRUCTURE ONLY).

Notation.  The paper (Section 2.1) writes p for the draft and q for the
target; other texts swap the letters.  To keep them apart this file writes
T(x) for the target probability and D(x) for the draft probability.

The method (Section 2.1 and Section 3), for one block of gamma drafted tokens
d_1..d_gamma with draft distributions D_1..D_gamma and target distributions
T_1..T_{gamma+1} obtained from ONE target call on [t, d_1..d_gamma]:

  * d_j is accepted with probability min{1, T_j(d_j) / D_j(d_j)};
  * at the first rejection, position k+1, a replacement token is drawn from
    the residual distribution proportional to max(0, T_{k+1}(x) - D_{k+1}(x));
  * if nothing is rejected one more token is drawn from T_{gamma+1} (implied
    by the stated maximum of gamma + 1 tokens per block, Section 4 Metrics);
  * with greedy decoding the output equals the target's own greedy output
    (Section 4, Decoding).

Readings of what the paper leaves open (also listed in the design notes):

  accept test   accept  <=>  u * D(d) < T(d)  with u uniform on the grid
                {0, 1, .., 2^24-1} / 2^24, evaluated with ONE float32 multiply
                and one compare (no division).  P(accept) = min(1, T/D) up to
                the 2^-24 grid.  The decision is taken in float32 on both
                the oracle and the device so that it can be compared bit for
                bit.
  residual      the printed residual is unnormalised; it is normalised by its
                sum, inside the sampler.
  sampler       fixed-point inverse CDF, independent of summation order:
                w(x) = floor(r(x) * 2^32) (exact for a float32 r), S = sum w,
                threshold = floor(k_u * S / 2^24) with k_u = u * 2^24, and the
                sample is the first x whose running sum of w exceeds the
                threshold.  If S = 0 for a residual (all mass below 2^-32) the
                sampler is applied to T_{k+1} itself; if that is 0 too, x = 0.
  greedy        temperature 0 makes every distribution one-hot at its argmax
                (lowest index on ties); the rules above then reduce to
                "accept iff d_j = argmax T_j, replacement = argmax T_{k+1}".
  bookkeeping   the target cache keeps t, d_1..d_k (k+1 new positions); the
                draft cache keeps t, d_1..d_min(k, gamma-1); the next block
                starts from [y], or from [d_gamma, y] after a full acceptance
                because the draft has not consumed d_gamma yet.

Pins (tests/test_oracle_spec_sampling.py): P(accept) = sum_x min(T, D) by brute
force, the identity that makes the output distribution equal T, chi-square of
sampled outputs against T, D == T and disjoint-support special cases, greedy
speculative == greedy autoregressive token for token, closed-form block
efficiency, exhaustive checks of the fixed-point sampler on the u grid.
"""
import numpy as np

from . import decoder as dec

U_BITS = 24                 # uniforms live on the grid j / 2^24
W_BITS = 32                 # sampler weights are floor(r * 2^32)


def softmax_probs(logits, temperature):
    """Probability row(s) as float32 from float64 logits.

    temperature > 0: softmax(logits / temperature) in float64, then rounded
    to float32 (the sampler and the accept test are defined on float32).
    temperature == 0: one-hot at the argmax, lowest index on ties.
    """
    logits = np.asarray(logits, dtype=np.float64)
    if temperature == 0.0:
        out = np.zeros(logits.shape, dtype=np.float32)
        idx = np.argmax(logits, axis=-1)            # numpy returns the first maximum
        np.put_along_axis(out, np.expand_dims(idx, -1), np.float32(1.0), axis=-1)
        return out
    return dec.softmax_rows(logits / temperature).astype(np.float32)


def accept_test(T_x, D_x, u):
    """True iff the drafted token is accepted: u * D(d) < T(d), in float32."""
    return bool(np.float32(u) * np.float32(D_x) < np.float32(T_x))


def accept_probability(T_x, D_x):
    """min{1, T(d)/D(d)} (Section 2.1), float64; D(d) = 0 counts as ratio +inf."""
    T_x = float(T_x)
    D_x = float(D_x)
    if D_x == 0.0:
        return 1.0 if T_x > 0.0 else 0.0
    return min(1.0, T_x / D_x)


def residual(T_row, D_row):
    """Unnormalised residual max(0, T - D) (Section 2.1), float32 arithmetic."""
    T_row = np.asarray(T_row, dtype=np.float32)
    D_row = np.asarray(D_row, dtype=np.float32)
    return np.maximum(np.float32(0.0), T_row - D_row)


def fixed_point_weights(r):
    """w(x) = floor(r(x) * 2^32) as uint64; exact because r is float32 >= 0."""
    r = np.asarray(r, dtype=np.float32).astype(np.float64)
    return np.floor(r * float(1 << W_BITS)).astype(np.uint64)


def sample_fixed_point(r, u):
    """Inverse-CDF sample from the distribution proportional to r (float32 >= 0).

    Returns the index, or None when every weight truncates to zero.
    """
    w = fixed_point_weights(r)
    S = int(np.sum(w, dtype=np.uint64))
    if S == 0:
        return None
    k_u = int(np.float64(np.float32(u)) * float(1 << U_BITS))
    assert 0 <= k_u < (1 << U_BITS)
    threshold = (k_u * S) >> U_BITS             # python integers: no overflow
    running = np.cumsum(w, dtype=np.uint64)
    return int(np.searchsorted(running, np.uint64(threshold), side="right"))


def sample_row(p_row, u):
    """Draw a token from a probability row (draft sampling, bonus token)."""
    y = sample_fixed_point(p_row, u)
    return 0 if y is None else y


def count_accepted(T, D, draft_tokens, u):
    """k = number of leading accepted draft tokens (sequential verification)."""
    gamma = len(draft_tokens)
    k = 0
    for j in range(gamma):
        d = int(draft_tokens[j])
        if accept_test(T[j, d], D[j, d], u[j]):
            k += 1
        else:
            break
    return k


def speculative_accept(T, D, draft_tokens, u):
    """Accept/reject + replacement for one sequence and one block.

    T[gamma+1, V], D[gamma, V]: float32 probability rows (row j of T is the
    target distribution of the token d_{j+1} stands for; the last row of T is
    the bonus row).  draft_tokens[gamma]; u[gamma+1] float32 uniforms: the
    first gamma drive the accept tests, the last the replacement/bonus draw.
    Returns (k, y): k accepted tokens and the next token y.
    """
    T = np.asarray(T, dtype=np.float32)
    D = np.asarray(D, dtype=np.float32)
    gamma = len(draft_tokens)
    assert T.shape[0] == gamma + 1 and D.shape[0] == gamma
    k = count_accepted(T, D, draft_tokens, u)
    if k < gamma:
        y = sample_fixed_point(residual(T[k], D[k]), u[gamma])
        if y is None:
            y = sample_row(T[k], u[gamma])
    else:
        y = sample_row(T[gamma], u[gamma])
    return k, y


def spd_generate(target, draft, image_rows, text_tokens, gamma, n_new, temperature,
                 u_first, u_draft, u_accept, max_positions=None):
    """Whole speculative-decoding loop for one sequence.

    target, draft: (DecoderConfig, weights).  image_rows[m, d_target] are the
    image embeddings V_1..V_m (Section 2.2); text_tokens[n] the prompt.  The
    target is prefilled with [V ; E[X]] at positions 0..m+n-1; the draft is
    prefilled with E_d[X] alone at positions 0..n-1 (text-only draft,
    Section 3).  u_first: uniform for the first token, drawn from the target's
    last prefill row.  u_draft[b, gamma], u_accept[b, gamma+1]: uniforms of
    block b.  Generates at least n_new tokens and truncates to n_new.

    Returns dict(tokens, blocks) where blocks is a list of dict(draft_tokens,
    k, y, T, D) in order.
    """
    (tc, tw), (dc, dw) = target, draft
    m = 0 if image_rows is None else image_rows.shape[0]
    n = len(text_tokens)
    cap = max_positions or (m + n + n_new + gamma + 2)
    t_cache = dec.KVCache(tc, cap)
    d_cache = dec.KVCache(dc, cap)

    x_text = dec.embed_tokens(tw, text_tokens)
    x_prefix = x_text if m == 0 else np.concatenate([np.asarray(image_rows, dtype=np.float64), x_text], axis=0)
    logits = dec.forward_rows(tc, tw, t_cache, x_prefix)
    dec.forward_tokens(dc, dw, d_cache, text_tokens)

    t = sample_row(softmax_probs(logits[-1], temperature), u_first)
    out = [t]
    blocks = []
    pending = [t]                      # tokens the draft has not consumed yet
    b = 0
    while len(out) < n_new:
        # gamma autoregressive draft steps
        d_tokens, D_rows = [], []
        for j in range(gamma):
            lg = dec.forward_tokens(dc, dw, d_cache, pending)
            D_j = softmax_probs(lg[-1], temperature)
            d_j = sample_row(D_j, u_draft[b, j])
            d_tokens.append(d_j)
            D_rows.append(D_j)
            pending = [d_j]
        # one target call over [t, d_1 .. d_gamma]
        P = t_cache.length
        lg_t = dec.forward_tokens(tc, tw, t_cache, [t] + d_tokens)
        T_rows = softmax_probs(lg_t, temperature)
        D_rows = np.stack(D_rows)
        k, y = speculative_accept(T_rows, D_rows, d_tokens, u_accept[b])
        blocks.append(dict(draft_tokens=list(d_tokens), k=k, y=y, T=T_rows, D=D_rows))
        out.extend(d_tokens[:k])
        out.append(y)
        # commit: target keeps t, d_1..d_k
        t_cache.truncate(P + k + 1)
        # draft holds (..., t, d_1..d_{gamma-1}); keep t, d_1..d_min(k, gamma-1)
        d_cache.truncate(d_cache.length - (gamma - 1) + min(k, gamma - 1))
        pending = [d_tokens[gamma - 1], y] if k == gamma else [y]
        t = y
        b += 1
    return dict(tokens=out[:n_new], blocks=blocks)


def ar_generate(target, image_rows, text_tokens, n_new, temperature, u):
    """Plain autoregressive generation with the target alone (the baseline
    the paper's token rate is relative to, Section 4 Metrics).  u[i] is the
    uniform of the i-th generated token."""
    tc, tw = target
    m = 0 if image_rows is None else image_rows.shape[0]
    n = len(text_tokens)
    cache = dec.KVCache(tc, m + n + n_new + 1)
    x_text = dec.embed_tokens(tw, text_tokens)
    x_prefix = x_text if m == 0 else np.concatenate([np.asarray(image_rows, dtype=np.float64), x_text], axis=0)
    logits = dec.forward_rows(tc, tw, cache, x_prefix)
    out = []
    for i in range(n_new):
        t = sample_row(softmax_probs(logits[-1], temperature), u[i])
        out.append(t)
        if i + 1 < n_new:
            logits = dec.forward_tokens(tc, tw, cache, [t])
    return out
