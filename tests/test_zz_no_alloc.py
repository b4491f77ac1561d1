"""The entry point that allocates nothing, eoq_conv_bwd_weight_static (for callers that cannot call hipMalloc: graph
capture, tight loops), against eoq_conv_bwd_weight with a caller workspace and against the CPU oracle (Eq.4, g_w
before Q_g), bit for bit: two calls in a row on one context, the second on a smaller input, so that whatever the
first call left in the library's static scratch array must not leak into the second."""
import numpy as np
import pytest

import seeded_inputs as si

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

from oracle import ops as oo            # noqa: E402
from oracle.ops import ConvShape        # noqa: E402


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_pair(ctx, d, seed):
    from paper_2105_13890_amd import eoq
    desc = eoq.ConvDesc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, d.stride, d.pad)
    u = si.uniform_int8(seed, "u", (d.N, d.H, d.W, d.C))
    e = si.uniform_int8(seed, "e", (d.N, d.P, d.Q, d.K))
    ud, ed = dev(u), dev(e)
    ws = torch.zeros((max(eoq.Context.workspace_bytes(desc, eoq.OP_CONV_BWD_WEIGHT), 16),), dtype=torch.uint8, device="cuda")
    g_ref = torch.zeros((d.K, d.R, d.S, d.C), dtype=torch.int32, device="cuda")
    g_new = torch.full((d.K, d.R, d.S, d.C), 7, dtype=torch.int32, device="cuda")
    slots = torch.zeros((2,), dtype=torch.int32, device="cuda")
    ctx.conv_bwd_weight(desc, ed, ud, g_ref, slots[0:1], ws)
    ctx.conv_bwd_weight_static(desc, ed, ud, g_new, slots[1:2])
    torch.cuda.synchronize()
    want = oo.conv_bwd_weight(d, e, u)
    assert np.array_equal(g_new.cpu().numpy(), g_ref.cpu().numpy()), d
    assert np.array_equal(g_new.cpu().numpy(), want), d
    sl = slots.cpu().numpy()
    assert sl[0] == sl[1] == int(np.abs(want).max())


def test_static_scratch_entry_point_two_calls_second_smaller():
    from paper_2105_13890_amd import eoq
    ctx = eoq.Context()
    # a 3x3 layer whose reduction is split into many ranges (large partial-sum footprint), then smaller problems
    # of other kernel families: 1x1, strided 3x3, the few-channel stem (staged input in front of the partial sums)
    run_pair(ctx, ConvShape(6, 28, 28, 64, 128, 3, 3, 1, 1), 51)
    run_pair(ctx, ConvShape(2, 14, 14, 32, 48, 3, 3, 1, 1), 52)
    run_pair(ctx, ConvShape(3, 17, 13, 64, 32, 1, 1, 1, 0), 53)
    run_pair(ctx, ConvShape(2, 15, 15, 32, 32, 3, 3, 2, 1), 54)
    run_pair(ctx, ConvShape(2, 33, 33, 3, 64, 7, 7, 2, 3), 55)
    run_pair(ctx, ConvShape(1, 9, 9, 20, 16, 3, 3, 1, 1), 56)       # odd channel count: explicit im2col in the scratch
    assert ctx.status() == 0
    # beyond the limit: the filter alone (2048 x 3 x 3 x 2048 int32 = 144 MiB per partial buffer) cannot fit 32 MiB
    big = eoq.ConvDesc(1, 4, 4, 2048, 2048, 3, 3, 1, 1)
    t8 = torch.zeros((16,), dtype=torch.int8, device="cuda")
    t32 = torch.zeros((16,), dtype=torch.int32, device="cuda")
    with pytest.raises(eoq.EoqError, match="workspace"):
        ctx.conv_bwd_weight_static(big, t8, t8, t32, t32[0:1])
    assert ctx.status() == 0
    ctx.close()
