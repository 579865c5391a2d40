"""Oracle: the paper's efficiency metrics (TEST INFRASTRUCTURE ONLY).

Section 4, Metrics: block efficiency tau is the average number of tokens
generated per block (= per target-model run), at most gamma + 1; the
memory-bound speed-up (MBSU) is the hypothetical speed-up for a given tau and
relative latency c, the ratio of draft to target parameter counts.

Reading of the MBSU formula.  As printed the numerator carries a factor c,
which with c = draft/target ~ 0.016 would put every value below 1 and cannot
give the reported 2.37x.  In the memory-bound model a block costs gamma draft
passes of relative cost c plus one target pass and yields tau tokens, against
one target pass per token without speculation:
    MBSU = tau / (c * gamma + 1).
(The printed form is this one written with c as the target-to-draft ratio:
c' * tau / (gamma + c') with c' = 1/c.)
"""


def block_efficiency(tokens_per_block):
    """tau: mean number of tokens emitted per target run."""
    tokens_per_block = list(tokens_per_block)
    return sum(tokens_per_block) / len(tokens_per_block)


def mbsu(tau, c, gamma):
    """Memory-bound speed-up with c = draft parameters / target parameters."""
    return tau / (c * gamma + 1.0)


def expected_block_efficiency_iid(alpha, gamma):
    """E[tau] when every draft token is accepted independently w.p. alpha:
    E[k + 1] = sum_{i=0..gamma} alpha^i = (1 - alpha^(gamma+1)) / (1 - alpha)."""
    if alpha == 1.0:
        return gamma + 1.0
    return (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)
