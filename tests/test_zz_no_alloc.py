"""The grouped decode step on the library's built-in scratch buffer (no workspace argument, no allocation).

Checked through the C ABI against the workspace call it mirrors, omni_slim_decode_grouped: same kernels, so the
outputs must agree to the bit (which is inside the parity bar), and against the oracle's slimmed decode.  Two calls in
a row share the buffer; the second is the smaller one, so it runs over what the first left behind.
"""
import numpy as np
import pytest
import torch

from oracle import omni_oracle as oc
from paper_2511_12201_amd import binding as ob
from tests.helpers import lists_to_padded, to_device, to_host
from tests.test_gpu_parity import CFG_BF16, CFG_BF16_64, CFG_F32, TOL_OUT, _decode_case

pytestmark = pytest.mark.gpu


def _step(cfg, batch):
    """One decode step's device tensors, group lists built by the library, and the oracle's result."""
    c, q, Kc, Vc, ctx, probe, vis = _decode_case(cfg, batch)
    tau = 0.08
    H = cfg.n_q_heads
    b = len(c.o_kvidx[0][0])
    kv_idx, _ = lists_to_padded([list(c.o_kvidx[0])] * batch, H, b)
    budget = torch.full((batch,), b, dtype=torch.int32, device="cuda")
    ldesc = ob.make_layer_desc(c.dQ.expand(batch, -1, -1, -1).contiguous(), c.dK.expand(batch, -1, -1, -1).contiguous(),
                               cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)
    grp = ob.omni_group_subset(ldesc, kv_idx, budget, b)
    dq, dKc, dVc = (to_device(x, cfg.dtype) for x in (q, Kc, Vc))
    dctx = torch.from_numpy(ctx).cuda()
    dprobe = torch.from_numpy(probe.astype(np.float32)).cuda()
    desc = ob.make_decode_desc(dq, dKc, cfg.vis_begin, cfg.vis_end, tau)
    want = oc.slim_decode(q, Kc, Vc, ctx, probe.astype(np.float32), vis, tau, cfg.vis_begin, cfg.vis_end, cfg.scale)
    return desc, (dq, dKc, dVc, dctx, dprobe) + tuple(grp), want, tau


def _check(cfg, desc, args, want, tau):
    q = args[0]
    O_ws, act_ws = ob.omni_slim_decode_grouped(desc, *args)
    O_st = torch.full_like(q, float("nan"))
    act_st = torch.full((desc.batch, desc.n_q_heads), 7, dtype=torch.uint8, device="cuda")
    ob.omni_slim_decode_grouped_static(desc, *args, O_st, act_st)
    torch.cuda.synchronize()
    view = torch.int16 if q.dtype == torch.bfloat16 else torch.int32
    assert torch.equal(O_st.view(view), O_ws.view(view))
    assert torch.equal(act_st, act_ws)
    Oo, acto, sc = want
    act = to_host(act_st)
    clear = np.abs(sc - tau) > 1e-5
    np.testing.assert_array_equal(act[clear], acto[clear])
    same = act == acto
    assert np.max(np.abs(to_host(O_st)[same] - Oo[same])) <= TOL_OUT[cfg.dtype]


def test_grouped_decode_on_the_built_in_scratch_buffer_two_calls_in_a_row():
    assert ob.workspace_bytes(ob.CALL_SLIM_DECODE, _step(CFG_BF16, 3)[0]) <= ob.omni_static_scratch_bytes()
    big = _step(CFG_BF16, 3)                 # 8 query heads, 1859 tokens, batch 3
    small = _step(CFG_BF16_64, 1)            # 4 query heads, 537 tokens, batch 1: a smaller footprint in the buffer
    _check(CFG_BF16, *big)
    _check(CFG_BF16_64, *small)
    _check(CFG_BF16, *big)                   # and back, over the small call's leftovers
    _check(CFG_F32, *_step(CFG_F32, 2))


def test_shapes_beyond_the_built_in_buffer_are_refused():
    desc, args, _, _ = _step(CFG_BF16_64, 1)
    big = ob.DecodeDesc.from_buffer_copy(desc)
    big.batch = 20000                         # the partial states of 20000 sequences do not fit 16 MiB
    assert ob.workspace_bytes(ob.CALL_SLIM_DECODE, big) > ob.omni_static_scratch_bytes()
    O = torch.empty(1, device="cuda")
    with pytest.raises(ob.OmniError, match="built-in buffer"):
        ob.omni_slim_decode_grouped_static(big, *args, O, O)
