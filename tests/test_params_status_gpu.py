"""GPU parity on parameter values the benchmark's recipe never takes (norm weights other than one,
NULL norm pointers, a gate bias, lambda = 1, eta other than 0.5, other sink and recent-window sizes,
per-sequence position offsets, queries behind their tokens), and the device-side status bits
of a broken live-length promise and of a unit above the budget.  Every case runs through the
step-by-step calls AND the fused step, in both state layouts."""
import numpy as np
import pytest
import torch

import paper_2605_25475_amd as im
from helpers import f64
from parity import LockStep, LockStepShared
from workloads import WORKLOADS

pytestmark = pytest.mark.gpu


def _norm_weights(p):
    g = torch.Generator().manual_seed(77)
    for k in ("norm_q_w", "norm_k_w"):
        p[k] = (1.0 + 0.1 * torch.randn(p[k].shape, generator=g)).to(torch.bfloat16)


def _cg(v):
    def mod(p):
        p["cg"] = v
    return mod


VARIANTS = {
    "norm-weights": dict(params_mod=_norm_weights),
    "null-norm-pointers": dict(null_norms=True),
    "gate-bias-plus": dict(params_mod=_cg(1.5)),
    "gate-bias-minus": dict(params_mod=_cg(-1.5)),
    "lambda-one": dict(scale=dict(lam=1.0)),
    "eta-two": dict(scale=dict(eta=2.0)),
    "no-sinks": dict(scale=dict(n_sink=0)),
    "nine-sinks-five-recent": dict(scale=dict(n_sink=9, n_recent=5)),
}


@pytest.mark.parametrize("variant", sorted(VARIANTS))
@pytest.mark.parametrize("fused", [False, True], ids=["steps", "fused"])
@pytest.mark.parametrize("shared", [False, True], ids=["per-unit", "head-shared"])
def test_parameter_values_outside_the_benchmark_recipe(variant, fused, shared):
    v = dict(VARIANTS[variant])
    kw = dict(context=330, budget=90, decode_steps=3, batch=2, n_layers=1, **v.pop("scale", {}))
    w = WORKLOADS["cfg1"].shared(**kw) if shared else WORKLOADS["cfg1"].scaled(**kw)
    cls = LockStepShared if shared else LockStep
    ls = cls(w, capacity=max(w.capacity, w.budget + 2), **v)
    ls.run_schedule(fused_decode=fused)
    if variant.startswith("gate-bias"):
        # the bias is at work: the residual's size follows sigmoid(c_g + w_g . q), far from its value at 0
        assert float(ls.gpu.readout.abs().max()) > 0


def _snapshot(st):
    return {k: getattr(st, k).clone() for k in ("K", "V", "Kidx", "pos", "len", "n_projected", "M", "b")}


def _new_token(ls, t, shared):
    w = ls.w
    d = lambda x: x.to(ls.dev)
    k = d(ls.K[:, :, t:t + 1].contiguous()); v = d(ls.V[:, :, t:t + 1].contiguous())
    q = d(ls.Q[:, t:t + 1].contiguous())
    pos = torch.full((w.batch, 1), t, dtype=torch.int32, device=ls.dev)
    x = d(ls.X[:, t:t + 1].contiguous()) if shared else None
    return k, v, q, pos, x


@pytest.mark.parametrize("fused", [False, True], ids=["steps", "fused"])
@pytest.mark.parametrize("shared", [False, True], ids=["per-unit", "head-shared"])
def test_broken_live_length_promise_sets_the_status_bit_and_evicts_nothing(fused, shared):
    # 200 entries per unit, nothing evicted so far; the caller then promises at most 150 live entries
    # and runs one more step with a budget of 100.  The unit is flagged, the new token is appended,
    # and nothing else changes: no entry leaves, the memory stays as it is, the length is 201.
    kw = dict(context=200, budget=400, decode_steps=2, batch=2, n_layers=1)
    w = WORKLOADS["cfg1"].shared(**kw) if shared else WORKLOADS["cfg1"].scaled(**kw)
    ls = (LockStepShared if shared else LockStep)(w, capacity=420)
    ls.event(0, w.context, w.budget, "prefill, nothing evicted")
    assert im.im_query_status(ls.handle) == 0
    g, st = ls.gpu, ls.gpu.st
    before = _snapshot(st)
    im.im_set_max_live(ls.handle, 150)
    t = w.context
    k, v, q, pos, x = _new_token(ls, t, shared)
    qh = q.view(w.batch, w.n_q_heads, w.head_dim)
    xg = x.view(w.batch, -1) if shared else q.view(w.batch, -1)
    if fused:
        g.decode_step(k, v, pos.view(-1), qh, xg, pos.view(-1), 100, w.lam, w.eta, debug=True)
    else:
        g.step(k, v, pos, q, x if shared else q.view(w.batch, 1, -1), pos, qh, 100, w.lam, w.eta, x_new=x)
    torch.cuda.synchronize()
    status = im.im_query_status(ls.handle)
    assert status & im.IM_STATUS_LIVE_EXCEEDED, status
    assert not status & im.IM_STATUS_APPEND_OVERFLOW
    n0 = w.context
    assert (st.len == n0 + 1).all()
    assert torch.equal(st.M, before["M"]) and torch.equal(st.b, before["b"])
    for name in ("K", "V"):
        assert torch.equal(getattr(st, name)[:, :, :n0], before[name][:, :, :n0])
        assert torch.equal(getattr(st, name)[:, :, n0], (k if name == "K" else v)[:, :, 0])
    assert torch.equal(st.pos[..., :n0], before["pos"][..., :n0]) and (st.pos[..., n0] == t).all()
    assert torch.equal(st.Kidx[..., :n0, :], before["Kidx"][..., :n0, :])
    if fused:
        assert (g.evicted == -1).all()
    else:
        assert (g.n_evict == 0).all()
    # with the promise withdrawn the state is a valid one: the next event matches the oracle, which has
    # seen the same append and no eviction
    im.im_set_max_live(ls.handle, 420)
    if shared:
        ls.ref.append_kv_hidden(f64(k.cpu()), f64(v.cpu()), f64(x.cpu()), pos.cpu().numpy())
    else:
        ls.ref.append_kv(f64(k.cpu()), f64(v.cpu()), pos.cpu().numpy())   # (projected at its next scoring call)
    ls.event(t + 1, t + 2, 100, "event after the promise was withdrawn")
    assert im.im_query_status(ls.handle) == 0


@pytest.mark.parametrize("shared", [False, True], ids=["per-unit", "head-shared"])
def test_unit_above_the_budget_loses_one_entry_and_sets_the_status_bit(shared):
    # every unit enters im_decode_step with 103 entries and a budget of 100: exactly one entry leaves
    # (the one the selection order ranks last, as an oracle step that keeps n - 1 = 103 shows) and the
    # status word says so
    kw = dict(context=300, budget=103, decode_steps=2, batch=2, n_layers=1)
    w = WORKLOADS["cfg1"].shared(**kw) if shared else WORKLOADS["cfg1"].scaled(**kw)
    ls = (LockStepShared if shared else LockStep)(w, capacity=300)
    ls.event(0, w.context, w.budget, "prefill to 103")
    im.im_set_max_live(ls.handle, 110)
    g = ls.gpu
    t = w.context
    k, v, q, pos, x = _new_token(ls, t, shared)
    qh = q.view(w.batch, w.n_q_heads, w.head_dim)
    g.decode_step(k, v, pos.view(-1), qh, x.view(w.batch, -1) if shared else q.view(w.batch, -1), pos.view(-1),
                  100, w.lam, w.eta, debug=True)
    torch.cuda.synchronize()
    status = im.im_query_status(ls.handle)
    assert status == im.IM_STATUS_OVER_BUDGET, status
    posn = pos.cpu().numpy()
    qn = f64(q.cpu())
    if shared:
        xn = f64(x.cpu())
        ref = ls.ref.step(f64(k.cpu()), f64(v.cpu()), xn, posn, qn, xn, posn, qn[:, 0], 103, w.lam, w.eta)
    else:
        ref = ls.ref.step(f64(k.cpu()), f64(v.cpu()), posn, qn, qn.reshape(w.batch, 1, -1), posn, qn[:, 0], 103,
                          w.lam, w.eta)
    ls.compare(*ref, "over budget", fused=True)
    assert (g.st.len == 103).all()


@pytest.mark.parametrize("fused", [False, True], ids=["steps", "fused"])
@pytest.mark.parametrize("shared", [False, True], ids=["per-unit", "head-shared"])
def test_sequences_with_different_token_positions(fused, shared):
    # the benchmark's sequences all count their tokens from 0; here the three sequences of a batch start at
    # 0, 7 and 900, so only the first holds sink positions and every per-sequence position (the new
    # token's, the query's, the recent window's newest) is a different number in each
    kw = dict(context=330, budget=90, decode_steps=4, batch=3, n_layers=1, n_recent=3)
    w = WORKLOADS["cfg1"].shared(**kw) if shared else WORKLOADS["cfg1"].scaled(**kw)
    ls = (LockStepShared if shared else LockStep)(w, capacity=max(w.capacity, w.budget + 2))
    ls.pos_off = torch.tensor([[0], [7], [900]], dtype=torch.int32)
    ls.run_schedule(fused_decode=fused)
    pos = ls.gpu.st.pos.cpu()
    n = int(ls.gpu.st.len.flatten()[0])
    assert int(pos[0].flatten()[:4].max()) <= 3 and int(pos[2].min()) >= 900 and n == w.budget


@pytest.mark.parametrize("fused", [False, True], ids=["steps", "fused"])
@pytest.mark.parametrize("shared", [False, True], ids=["per-unit", "head-shared"])
def test_queries_that_do_not_see_the_newest_tokens(fused, shared):
    # query positions 6 behind their tokens' (Algorithm 1's causal mask is by position, not by slot): the
    # newest cached tokens are invisible to every query that scores them, their importance is -inf and,
    # not being forced, they are the first to leave: among equal -inf scores the older position stays
    kw = dict(context=330, budget=90, decode_steps=4, batch=2, n_layers=1)
    w = WORKLOADS["cfg1"].shared(**kw) if shared else WORKLOADS["cfg1"].scaled(**kw)
    ls = (LockStepShared if shared else LockStep)(w, capacity=max(w.capacity, w.budget + 2))
    ls.qpos_shift = 6
    ls.run_schedule(fused_decode=fused)
    # each decode step's new token was invisible to its own query, so it is the one that left again
    assert (ls.gpu.st.len == w.budget).all()
    assert int(ls.gpu.st.pos[..., :w.budget].max()) < w.context
