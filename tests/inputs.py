"""Test inputs whose recipe includes a statistic of the method: the encoder-FFN configuration's
per-token activation scales are the value training starts them from, 2 * mean|A| per token.  The
seeded generators hold no method arithmetic, so the tests derive the scales with the oracle and
hand the same values to both sides."""
import oracle
import synth


def config2(which, M=4096):
    c = synth.config2(which, M=M)
    c["s_a"] = oracle.act_scale(c["A"])
    return c
