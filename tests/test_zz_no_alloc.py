"""lp_attention_static (the entry point for callers that cannot allocate) against lp_attention.

Two calls in a row on the one device-resident scratch array, the second with a smaller input,
each compared with the workspace entry point on the same inputs (same kernels, same split of
the work: bit-identical) and with the oracle at the attention tolerance.
"""
import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth

pytestmark = pytest.mark.gpu


def _static(q, k, v):
    import torch
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    n, heads, d = q.shape
    qd, kd, vd = g.to_dev_bf16(q), g.to_dev_bf16(k), g.to_dev_bf16(v)
    od = torch.full((n, heads, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    lp.lp_attention_static(qd, kd, vd, od, n, heads, d, heads * d, d, 0.0, g.stream())
    torch.cuda.synchronize()
    return g.from_dev_bf16(od)


def test_static_scratch_two_calls_second_smaller():
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    assert lp.lp_attention_static_scratch_bytes() >= lp.lp_attention_workspace_size(128)
    # shapes whose query tiles are shared between workgroups, so the scratch really carries
    # partial results: first the larger, then a smaller one that leaves most slots untouched
    for n, heads, hd, seed in ((3000, 3, 128, 811), (700, 2, 128, 812), (333, 5, 64, 813)):
        q, k, v = synth.qkv_bf16(seed, n, heads, hd)
        got = _static(q, k, v)
        ref = g.hip_attention(q, k, v, balanced=True)
        assert np.array_equal(got, ref), "n=%d: differs from lp_attention with a workspace" % n
        g.assert_attention_close(got, orc.attention(q, k, v), "static n=%d" % n)
