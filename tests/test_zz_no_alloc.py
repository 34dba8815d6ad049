"""The entry point that allocates nothing (im_decode_attn_with_readout_static: attention partials in a
buffer built into the library's device code) against im_decode_attn_with_readout on the same state,
through the raw C ABI: two calls in a row, the second with a smaller input, so that the buffer still
holds the first call's records when the second runs."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2605_25475_amd as im
from paper_2605_25475_amd import binding as B
from parity import LockStep, assert_out_close
from workloads import WORKLOADS

pytestmark = pytest.mark.gpu


def _both(ls, max_live, tag):
    """Attention + readout over the lock-step layer's current state through both entry points."""
    lib = im.load_library()
    w, g = ls.w, ls.gpu
    q = ls.Q[:, w.context + 1].contiguous().cuda()
    out_ws = torch.empty_like(g.out); res_ws = torch.empty_like(g.readout)
    im.im_set_max_live(ls.handle, max_live)
    im.im_decode_attn_with_readout(ls.handle, ls.params, g.st, q, out_ws, res_ws)
    out_st = torch.full_like(g.out, float("nan")); res_st = torch.full_like(g.readout, float("nan"))
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    cfg = ls.handle.cfg.c_struct()
    free_before = torch.cuda.mem_get_info()[0]
    rc = lib.im_decode_attn_with_readout_static(
        C.byref(cfg), max_live, C.byref(ls.params.c), C.byref(g.st.c), q.data_ptr(), out_st.data_ptr(),
        res_st.data_ptr(), status.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == im.IM_OK, lib.im_last_error(None).decode()
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, f"{tag}: device memory changed hands during the call"
    assert int(status.item()) == 0 and im.im_query_status(ls.handle) == 0
    # the same kernels on the same inputs: the same bits; and the benchmark spec's bar on top
    assert torch.equal(out_st, out_ws), tag
    assert torch.equal(res_st, res_ws), tag
    assert_out_close(tag, out_st.double().cpu().numpy(), out_ws.double().cpu().numpy())
    return out_st


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    big = LockStep(WORKLOADS["cfg3"].scaled(n_layers=1, batch=3, context=1500, budget=700, decode_steps=2))
    big.event(0, big.w.context, big.w.budget, "prefill 1500 -> 700")            # 6 chunks of 128 keys, ragged
    small = LockStep(WORKLOADS["cfg4"].scaled(n_layers=1, batch=1, context=400, budget=150, decode_steps=2))
    small.event(0, small.w.context, small.w.budget, "prefill 400 -> 150")       # 7 heads per group, 2 chunks
    o1 = _both(big, 701, "first call")
    o2 = _both(small, 151, "second call, smaller")
    o3 = _both(big, 701, "third call, the first again")
    assert torch.equal(o1, o3)
    assert o2.shape != o1.shape
    # the oracle agrees with what both entry points return
    q = big.Q[:, big.w.context + 1].contiguous()
    out, _ = big.ref.decode_attn_with_readout(q.double().numpy())
    assert_out_close("oracle", o1.double().cpu().numpy().reshape(out.shape), out)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    lib = im.load_library()
    ls = LockStep(WORKLOADS["cfg1"].scaled(context=200, budget=64, decode_steps=1))
    ls.event(0, 200, 64, "prefill")
    g = ls.gpu
    q = ls.Q[:, 200].contiguous().cuda()
    out = torch.zeros_like(g.out)
    # a shape whose partials exceed the built-in buffer: batch 64 x 64 heads x 128 chunks of records
    huge = im.Config(batch=64, n_q_heads=64, n_kv_heads=8, capacity=16384, n_idx_heads=16).c_struct()
    rc = lib.im_decode_attn_with_readout_static(C.byref(huge), 16384, C.byref(ls.params.c), C.byref(g.st.c),
                                                q.data_ptr(), out.data_ptr(), None, None, 0)
    assert rc == im.IM_ERR_INVALID_ARG
    assert b"IM_STATIC_SCRATCH_BYTES" in lib.im_last_error(None)
    torch.cuda.synchronize()
    assert not out.any()
    with pytest.raises(im.IndexMemError):
        im.im_decode_attn_with_readout_static(ls.handle.cfg, ls.handle.cfg.capacity + 1, ls.params, g.st, q, out)
