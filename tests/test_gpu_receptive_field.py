"""Functional check of the multi-layer receptive field (Section 3.1: the mask is the adjacency matrix of a
DAG, and information of token j can reach token i through l layers iff j is reachable from i in at most l
steps; Appendix A: the sets B_k).  Layers are chained on the GPU with V_{l+1} = O_l (one head, Q = K = 0 so
that every attended key has weight 1/count and nothing can cancel).  V is zero except for one token; after
l layers the output is non-zero exactly at the tokens whose l-step receptive field (composition of the
oracle's token mask) contains that token."""
import numpy as np
import pytest
import torch

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa

pytestmark = pytest.mark.gpu


def run_layers(pat, v0, layers):
    n = v0.shape[2]
    cnt, idx, _ = pa.mask_build(pat, n)
    q = torch.zeros_like(v0)
    k = torch.zeros_like(v0)
    outs = []
    v = v0
    for _ in range(layers):
        o, _ = pa.prefill(pat, cnt, idx, q, k, v)
        outs.append(o)
        v = o
    torch.cuda.synchronize()
    return outs


@pytest.mark.parametrize("B,W,S,nb,flags", [
    (64, 2, 0, 16, pa.POWER),     # pure pattern plus a two-block window
    (64, 2, 1, 32, pa.POWER),     # with the sink block
    (64, 1, 0, 16, pa.POWER),     # Theorem B.1's edge set at block level
    (64, 2, 1, 16, 0),            # sliding window + sink: most early tokens stay out of reach
])
def test_influence_is_exactly_the_receptive_field(B, W, S, nb, flags):
    n, d, layers = nb * B, 64, 5
    pat = pa.Pattern(B, W, S, flags)
    opat = orc.Pattern(B, W, S, power=bool(flags & pa.POWER))
    depth = orc.reach_depth(orc.token_mask(n, opat))          # depth[i, j]: layers needed from j to i
    for tok in (5, 3 * B + 17, (nb // 2) * B - 1):
        v0 = torch.zeros(1, 1, n, d, dtype=torch.bfloat16)
        v0[0, 0, tok] = 1.0
        outs = run_layers(pat, v0.cuda(), layers)
        for l in range(layers):
            got = (outs[l].float().abs().amax(dim=3)[0, 0] > 0).cpu().numpy()
            expect = (depth[:, tok] >= 0) & (depth[:, tok] <= l + 1)
            # the value itself stays where it is only through the diagonal: token `tok` attends itself
            assert np.array_equal(got, expect), (tok, l, int(got.sum()), int(expect.sum()))
