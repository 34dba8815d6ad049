"""Lock-step runner for the parity tests: the same seeded inputs go through the HIP path (via
the C ABI binding) and through the oracle, and every observable is compared after every event.

Bars (from the benchmark spec):
  * scores' induced decisions, keep / evict lists, counts, lengths, positions and the moved
    K / V / indexer-key rows: bit-exact;
  * fp32 memory state (M, b): max |diff| <= 1e-4 * rms(oracle);
  * bf16 attention output: |diff| <= 1e-2 + 1e-2 |oracle| elementwise;
  * fp32 readout residual g(q) m(q): max |diff| <= 1e-3 * max |oracle| (it is ~1e-2 or smaller
    in size, so the output bar alone would not see it).
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_25475_amd as im
from helpers import f64, make_oracle_layer
from workloads import Workload, hidden_stream, layer_params, token_stream


def rms(x):
    return float(np.sqrt(np.mean(np.square(x)))) if x.size else 0.0


def assert_state_close(tag, M_gpu, M_ref, rel=1e-4):
    d = float(np.max(np.abs(M_gpu - M_ref))) if M_ref.size else 0.0
    assert d <= rel * rms(M_ref), f"{tag}: max diff {d:.3e} vs rms {rms(M_ref):.3e}"


def assert_out_close(tag, got, want, atol=1e-2, rtol=1e-2):
    bad = np.abs(got - want) > atol + rtol * np.abs(want)
    assert not bad.any(), f"{tag}: {int(bad.sum())} elements off, max diff {np.max(np.abs(got - want)):.3e}"


class LockStep:
    """One layer on the GPU and in the oracle, fed the same events."""

    def __init__(self, w: Workload, layer: int = 0, capacity=None, max_queries=None, device="cuda",
                 gen_device="cpu", kv_heads=None, batch_ids=None, ref_capacity=None, params_mod=None,
                 null_norms=False):
        """params_mod: a function that edits the generated weights (a dict) before both sides get them;
        null_norms: the library gets NULL norm-weight pointers (the oracle keeps the ones)."""
        self.w = w
        self.dev = device
        cap = w.capacity if capacity is None else capacity
        self.cap = cap
        p = layer_params(w, layer, gen_device)
        if params_mod is not None:
            params_mod(p)
        cfg = im.Config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, capacity=cap,
                        n_idx_heads=w.n_idx_heads, n_sink=w.n_sink, n_recent=w.n_recent,
                        fold_block=w.fold_block,
                        max_queries=max_queries or max(w.context if w.prefill_chunk is None else w.prefill_chunk, 1))
        self.handle = im.Handle(cfg, device)
        pd = {k: (v.to(device) if torch.is_tensor(v) else v) for k, v in p.items()}
        self.params = im.Params(pd["Uq"], pd["G"], pd["Uk"], pd["Wtheta"], pd["wg"], pd["cg"],
                                None if null_norms else pd["norm_q_w"], None if null_norms else pd["norm_k_w"])
        self.gpu = im.Layer(self.handle, self.params, device)
        # the oracle may follow a subset of units (all by default)
        self.batch_ids = list(range(w.batch)) if batch_ids is None else list(batch_ids)
        self.kv_heads = list(range(w.n_kv_heads)) if kv_heads is None else list(kv_heads)
        self.ref = make_oracle_layer(w, layer, gen_device, params=p, capacity=ref_capacity or cap,
                                     batch=len(self.batch_ids), kv_head_ids=self.kv_heads)
        self.K, self.V, self.Q = token_stream(w, layer, gen_device)

    # -- one event on both sides ---------------------------------------------------------------
    def pos_offsets(self):
        """Per-sequence offsets added to every token position ([batch, 1] int32; zeros unless a test sets
        `self.pos_off`): sequences then differ in what the causal mask, the sinks and the position
        tie-break see."""
        off = getattr(self, "pos_off", None)
        return torch.zeros((self.w.batch, 1), dtype=torch.int32) if off is None else off

    def event(self, t0: int, t1: int, budget: int, tag: str, check=True):
        """Tokens [t0, t1) enter; their queries score the cache; evict to `budget`; attend with
        the last token's query."""
        w, dev = self.w, self.dev
        n_new = t1 - t0
        k_new = self.K[:, :, t0:t1].contiguous()
        v_new = self.V[:, :, t0:t1].contiguous()
        q_new = self.Q[:, t0:t1].contiguous()
        pos = (torch.arange(t0, t1, dtype=torch.int32).repeat(w.batch, 1) + self.pos_offsets()).contiguous()
        q_attn = self.Q[:, t1 - 1].contiguous()
        d = lambda t: t.to(dev)
        bi_t = torch.tensor(self.batch_ids, device=k_new.device)
        hs_t = torch.tensor(self.kv_heads, device=k_new.device)
        qd = d(q_new)
        qpos = pos - getattr(self, "qpos_shift", 0)   # (a test may let the queries lag behind their tokens)
        self.gpu.step(d(k_new), d(v_new), d(pos), qd, qd.view(w.batch, n_new, -1), d(qpos), d(q_attn),
                      budget, w.lam, w.eta)
        torch.cuda.synchronize()
        bi = self.batch_ids
        # only the sampled units travel to the host (the inputs may live on the GPU)
        sel = lambda x: f64(x.index_select(0, bi_t).index_select(1, hs_t))
        qn = f64(q_new.index_select(0, bi_t))
        posn = pos.numpy()[bi]
        scores, keep, evict, out, res = self.ref.step(
            sel(k_new), sel(v_new), posn, qn, qn.reshape(len(bi), n_new, -1), qpos.numpy()[bi],
            f64(q_attn.index_select(0, bi_t)), budget, w.lam, w.eta)
        if check:
            self.compare(scores, keep, evict, out, res, tag)
        return scores, keep, evict, out, res

    def event_fused(self, t: int, budget: int, tag: str, check=True):
        """One decode token through im_decode_step on the GPU and the step-by-step oracle."""
        w, dev = self.w, self.dev
        k_new = self.K[:, :, t:t + 1].contiguous()
        v_new = self.V[:, :, t:t + 1].contiguous()
        q_new = self.Q[:, t:t + 1].contiguous()
        pos = torch.full((w.batch, 1), t, dtype=torch.int32) + self.pos_offsets()
        d = lambda x: x.to(dev)
        bi_t = torch.tensor(self.batch_ids, device=k_new.device)
        hs_t = torch.tensor(self.kv_heads, device=k_new.device)
        qd = d(q_new).view(w.batch, w.n_q_heads, w.head_dim)
        posd = d(pos).view(w.batch)
        qpos = pos - getattr(self, "qpos_shift", 0)
        self.gpu.decode_step(d(k_new), d(v_new), posd, qd, qd.view(w.batch, -1), d(qpos).view(w.batch), budget,
                             w.lam, w.eta, debug=True)
        torch.cuda.synchronize()
        bi = self.batch_ids
        sel = lambda x: f64(x.index_select(0, bi_t).index_select(1, hs_t))
        qn = f64(q_new.index_select(0, bi_t))
        posn = pos.numpy()[bi]
        scores, keep, evict, out, res = self.ref.step(
            sel(k_new), sel(v_new), posn, qn, qn.reshape(len(bi), 1, -1), qpos.numpy()[bi], qn[:, 0],
            budget, w.lam, w.eta)
        if check:
            self.compare(scores, keep, evict, out, res, tag, fused=True)
        return scores, keep, evict, out, res

    def compare_decision(self, evict, tag):
        """The cheap part of a fused decode step's comparison, for every step of a long trajectory: the
        evicted slot and the new length of the sampled units, bit for bit."""
        evicted = self.gpu.evicted.cpu().numpy(); lens = self.gpu.st.len.cpu().numpy()
        for ib, b in enumerate(self.batch_ids):
            for ih, h in enumerate(self.kv_heads):
                er = evict[ib][ih]
                assert len(er) <= 1, f"{tag} unit(b={b},h={h})"
                want = int(er[0]) if len(er) else -1
                assert evicted[b, h] == want, f"{tag} unit(b={b},h={h}): evicted slot {evicted[b, h]} != {want}"
                assert lens[b, h] == int(self.ref.len[ib, ih]), f"{tag} unit(b={b},h={h}): length"

    def compare(self, scores, keep, evict, out, res, tag, fused=False, lists=True, outputs=True):
        w, g = self.w, self.gpu
        G = w.group
        n_keep = g.n_keep.cpu().numpy(); n_evict = g.n_evict.cpu().numpy()
        keep_idx = g.keep_idx.cpu().numpy(); evict_idx = g.evict_idx.cpu().numpy()
        sc = g.scores.cpu().numpy()
        evicted = g.evicted.cpu().numpy()
        st = g.st
        lens = st.len.cpu().numpy(); nproj = st.n_projected.cpu().numpy()
        pos = st.pos.cpu().numpy()
        out_g = f64(g.out).reshape(w.batch, w.n_kv_heads, G, w.head_dim)
        res_g = g.readout.cpu().numpy().astype(np.float64).reshape(w.batch, w.n_kv_heads, G, w.head_dim)
        Mg = st.M.cpu().numpy().astype(np.float64); bg = st.b.cpu().numpy().astype(np.float64)
        for ib, b in enumerate(self.batch_ids):
            for ih, h in enumerate(self.kv_heads):
                u = f"{tag} unit(b={b},h={h})"
                if lists:
                    kr, er = keep[ib][ih], evict[ib][ih]
                    n_before = len(kr) + len(er)
                    # scores: same fp32 value (a mismatch is reported with its size)
                    s_ref = scores[ib, ih, :n_before]; s_gpu = sc[b, h, :n_before].astype(np.float64)
                    same = (s_ref == s_gpu) | (np.isneginf(s_ref) & np.isneginf(s_gpu))
                    assert same.all(), (f"{u}: {int((~same).sum())} of {n_before} scores differ, max "
                                        f"{np.nanmax(np.abs(np.where(same, 0, s_ref - s_gpu))):.3e}")
                    if fused:
                        assert len(er) <= 1, u
                        want_e = int(er[0]) if len(er) else -1
                        assert evicted[b, h] == want_e, f"{u}: evicted slot {evicted[b, h]} != {want_e}"
                    else:
                        assert n_keep[b, h] == len(kr) and n_evict[b, h] == len(er), u
                        assert np.array_equal(keep_idx[b, h, :len(kr)], kr), f"{u}: keep list differs"
                        assert np.array_equal(evict_idx[b, h, :len(er)], er), f"{u}: evict list differs"
                n = int(self.ref.len[ib, ih])
                assert lens[b, h] == n, u
                if lists:
                    assert nproj[b, h] == n, u
                assert np.array_equal(pos[b, h, :n], self.ref.pos[ib, ih, :n]), f"{u}: positions"
                assert np.array_equal(f64(st.K[b, h, :n]), self.ref.K[ib, ih, :n]), f"{u}: K rows"
                assert np.array_equal(f64(st.V[b, h, :n]), self.ref.V[ib, ih, :n]), f"{u}: V rows"
                if lists:   # (rows appended since the last scoring call have no indexer key yet)
                    assert np.array_equal(f64(st.Kidx[b, h, :n]), self.ref.Kidx[ib, ih, :n]), f"{u}: indexer keys"
                assert_state_close(u + " M", Mg[b, h], self.ref.M[ib, ih])
                assert_state_close(u + " b", bg[b, h], self.ref.b[ib, ih])
                if outputs:
                    assert_out_close(u + " out", out_g[b, h], out[ib, ih])
                    rr = res[ib, ih]
                    dmax = float(np.max(np.abs(res_g[b, h] - rr)))
                    assert dmax <= 1e-3 * float(np.max(np.abs(rr))) + 1e-30, f"{u}: readout diff {dmax:.3e}"

    # -- a follower layer of an index-sharing group (Appendix, IndexCache-style reuse) -------------
    def _keep_from(self, evict):
        return [[np.setdiff1d(np.arange(int(self.ref.len[ib, ih])), evict[ib][ih]).astype(np.int64)
                 for ih in range(len(self.kv_heads))] for ib in range(len(self.batch_ids))]

    def follow_event(self, t0: int, t1: int, leader: "LockStep", evict, tag: str):
        """Tokens [t0, t1) enter this layer; the LEADER's evict lists (oracle's, per sampled unit)
        are applied on both sides; attend with the last token's query."""
        w, dev = self.w, self.dev
        d = lambda x: x.to(dev)
        k_new = self.K[:, :, t0:t1].contiguous(); v_new = self.V[:, :, t0:t1].contiguous()
        pos = (torch.arange(t0, t1, dtype=torch.int32).repeat(w.batch, 1) + self.pos_offsets()).contiguous()
        q_attn = self.Q[:, t1 - 1].contiguous()
        self.gpu.follow_event(d(k_new), d(v_new), d(pos), d(q_attn), leader.gpu, w.lam, w.eta)
        torch.cuda.synchronize()
        bi = self.batch_ids
        bi_t = torch.tensor(bi, device=k_new.device); hs_t = torch.tensor(self.kv_heads, device=k_new.device)
        sel = lambda x: f64(x.index_select(0, bi_t).index_select(1, hs_t))
        self.ref.append_kv(sel(k_new), sel(v_new), pos.numpy()[bi])
        keep = self._keep_from(evict)
        self.ref.memory_update(evict, w.lam, w.eta)
        self.ref.compact_kv(keep, evict)
        out, res = self.ref.decode_attn_with_readout(f64(q_attn.index_select(0, bi_t)))
        self.compare(None, None, None, out, res, tag, lists=False)

    def follow_step(self, t: int, leader: "LockStep", evict, tag: str):
        """One decode token through im_decode_step_shared with the slot the leader evicted."""
        w, dev = self.w, self.dev
        d = lambda x: x.to(dev)
        k_new = self.K[:, :, t:t + 1].contiguous(); v_new = self.V[:, :, t:t + 1].contiguous()
        q = self.Q[:, t].contiguous()
        pos = torch.full((w.batch,), t, dtype=torch.int32)
        self.gpu.follow_step(d(k_new), d(v_new), d(pos), d(q), leader.gpu.evicted, w.lam, w.eta, debug=True)
        torch.cuda.synchronize()
        bi = self.batch_ids
        bi_t = torch.tensor(bi, device=k_new.device); hs_t = torch.tensor(self.kv_heads, device=k_new.device)
        sel = lambda x: f64(x.index_select(0, bi_t).index_select(1, hs_t))
        self.ref.append_kv(sel(k_new), sel(v_new), pos.numpy()[bi].reshape(-1, 1))
        keep = self._keep_from(evict)
        self.ref.memory_update(evict, w.lam, w.eta)
        self.ref.compact_kv(keep, evict)
        out, res = self.ref.decode_attn_with_readout(f64(q.index_select(0, bi_t)))
        self.compare(None, None, None, out, res, tag, lists=False)

    def window(self, t0: int, tau: int, budget: int, tag: str, fused=True):
        """The paper's decode schedule (Section 4, setup): tau tokens are appended and attended to one
        by one, then the interval's queries score the cache and it is cut back to `budget`."""
        w, dev = self.w, self.dev
        d = lambda x: x.to(dev)
        bi_t = torch.tensor(self.batch_ids, device=self.K.device)
        hs_t = torch.tensor(self.kv_heads, device=self.K.device)
        sel = lambda x: f64(x.index_select(0, bi_t).index_select(1, hs_t))
        bi = self.batch_ids
        for t in range(t0, t0 + tau):
            k_new = self.K[:, :, t:t + 1].contiguous(); v_new = self.V[:, :, t:t + 1].contiguous()
            q_attn = self.Q[:, t].contiguous()
            pos = torch.full((w.batch, 1), t, dtype=torch.int32) + self.pos_offsets()
            self.gpu.attend_step(d(k_new), d(v_new), d(pos), d(q_attn), fused=fused)
            torch.cuda.synchronize()
            self.ref.append_kv(sel(k_new), sel(v_new), pos.numpy()[bi])
            out, res = self.ref.decode_attn_with_readout(f64(q_attn.index_select(0, bi_t)))
            self.compare(None, None, None, out, res, f"{tag} attend@{t}", lists=False)
            if fused:   # the fused entry point projects the new key on the way
                assert np.array_equal(self.gpu.st.n_projected.cpu().numpy(), self.gpu.st.len.cpu().numpy())
        q_win = self.Q[:, t0:t0 + tau].contiguous()
        posw = torch.arange(t0, t0 + tau, dtype=torch.int32).repeat(w.batch, 1).contiguous()
        qd = d(q_win)
        self.gpu.compress(qd, qd.view(w.batch, tau, -1), d(posw), budget, w.lam, w.eta)
        torch.cuda.synchronize()
        qn = f64(q_win.index_select(0, bi_t))
        scores = self.ref.index_score(qn, qn.reshape(len(bi), tau, -1), posw.numpy()[bi])
        keep, evict = self.ref.topb_select(scores, budget)
        self.ref.memory_update(evict, w.lam, w.eta)
        self.ref.compact_kv(keep, evict)
        self.compare(scores, keep, evict, None, None, f"{tag} compress@{t0 + tau}", outputs=False)

    # -- schedules --------------------------------------------------------------------------------
    def run_window_schedule(self, tau: int, n_windows: int, fused=True):
        """Prefill eviction, then n_windows compression intervals of tau tokens each."""
        w = self.w
        L = w.context
        if w.prefill_chunk is None:
            self.event(0, L, w.budget, "prefill")
        else:
            for c0 in range(0, L, w.prefill_chunk):
                self.event(c0, min(L, c0 + w.prefill_chunk), w.budget, f"chunk@{c0}")
        im.im_set_max_live(self.handle, min(self.cap, w.budget + tau))
        for k in range(n_windows):
            self.window(L + k * tau, tau, w.budget, f"window {k}", fused=fused)
        assert im.im_query_status(self.handle) == 0

    def run_schedule(self, decode_steps=None, fused_decode=False, full_every=1):
        """full_every = k > 1 (fused decode only): every observable is compared at every k-th decode step
        and at the last one; the steps between compare the decision (evicted slot, length) alone."""
        w = self.w
        steps = w.decode_steps if decode_steps is None else decode_steps
        L = w.context
        if w.prefill_chunk is None:
            self.event(0, L, w.budget, "prefill")
        else:
            for c0 in range(0, L, w.prefill_chunk):
                self.event(c0, min(L, c0 + w.prefill_chunk), w.budget, f"chunk@{c0}")
        im.im_set_max_live(self.handle, min(self.cap, w.budget + 1))
        for i, t in enumerate(range(L, L + steps)):
            if fused_decode:
                full = (i + 1) % full_every == 0 or i == steps - 1
                ref = self.event_fused(t, w.budget, f"fused decode@{t} (step {i + 1} of {steps})", check=full)
                if not full:
                    self.compare_decision(ref[2], f"fused decode@{t} (step {i + 1} of {steps})")
            else:
                self.event(t, t + 1, w.budget, f"decode@{t}")
        assert im.im_query_status(self.handle) == 0


class LockStepShared:
    """The same for the head-shared layout (one indexer key per token from its hidden state, one
    eviction set and one memory per sequence): events through the step-by-step entry points.  The
    oracle follows a subset of the sequences, with all their KV heads."""

    def __init__(self, w: Workload, layer: int = 0, device="cuda", gen_device="cpu", batch_ids=None, capacity=None,
                 params_mod=None, null_norms=False):
        assert w.head_shared
        self.w, self.dev = w, device
        self.cap = cap = w.capacity if capacity is None else capacity
        p = layer_params(w, layer, gen_device)
        if params_mod is not None:
            params_mod(p)
        cfg = im.Config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, capacity=cap,
                        n_idx_heads=w.n_idx_heads, idx_dim=w.idx_dim, n_sink=w.n_sink, n_recent=w.n_recent,
                        fold_block=w.fold_block, head_shared=1,
                        max_queries=max(w.context if w.prefill_chunk is None else w.prefill_chunk, 1))
        self.handle = im.Handle(cfg, device)
        pd = {k: (v.to(device) if torch.is_tensor(v) else v) for k, v in p.items()}
        self.params = im.Params(pd["Uq"], pd["G"], pd["Uk"], pd["Wtheta"], pd["wg"], pd["cg"],
                                None if null_norms else pd["norm_q_w"], None if null_norms else pd["norm_k_w"])
        self.gpu = im.Layer(self.handle, self.params, device)
        self.batch_ids = list(range(w.batch)) if batch_ids is None else list(batch_ids)
        self.ref = make_oracle_layer(w, layer, gen_device, params=p, batch=len(self.batch_ids), capacity=cap)
        self.K, self.V, self.Q = token_stream(w, layer, gen_device)
        self.X = hidden_stream(w, layer, gen_device)

    def pos_offsets(self):
        """Per-sequence offsets added to every token position ([batch, 1] int32; zeros unless a test sets
        `self.pos_off`): sequences then differ in what the causal mask, the sinks and the position
        tie-break see."""
        off = getattr(self, "pos_off", None)
        return torch.zeros((self.w.batch, 1), dtype=torch.int32) if off is None else off

    def event(self, t0: int, t1: int, budget: int, tag: str):
        w, dev = self.w, self.dev
        d = lambda t: t.to(dev)
        k_new = self.K[:, :, t0:t1].contiguous(); v_new = self.V[:, :, t0:t1].contiguous()
        q_new = self.Q[:, t0:t1].contiguous(); x_new = self.X[:, t0:t1].contiguous()
        pos = (torch.arange(t0, t1, dtype=torch.int32).repeat(w.batch, 1) + self.pos_offsets()).contiguous()
        q_attn = self.Q[:, t1 - 1].contiguous()
        xd = d(x_new)
        qpos = pos - getattr(self, "qpos_shift", 0)
        self.gpu.step(d(k_new), d(v_new), d(pos), d(q_new), xd, d(qpos), d(q_attn), budget, w.lam, w.eta, x_new=xd)
        torch.cuda.synchronize()
        bi_t = torch.tensor(self.batch_ids, device=k_new.device)
        sel = lambda x: f64(x.index_select(0, bi_t))
        posn = pos.numpy()[self.batch_ids]
        xn = sel(x_new)
        ref = self.ref.step(sel(k_new), sel(v_new), xn, posn, sel(q_new), xn, qpos.numpy()[self.batch_ids],
                            sel(q_attn), budget, w.lam, w.eta)
        self.compare(*ref, tag)
        return ref

    def event_fused(self, t: int, budget: int, tag: str, check=True):
        """One decode token through im_decode_step (four launches in this layout)."""
        w, dev = self.w, self.dev
        d = lambda x: x.to(dev)
        k_new = self.K[:, :, t:t + 1].contiguous(); v_new = self.V[:, :, t:t + 1].contiguous()
        q_new = self.Q[:, t:t + 1].contiguous(); x_new = self.X[:, t:t + 1].contiguous()
        pos = torch.full((w.batch, 1), t, dtype=torch.int32) + self.pos_offsets()
        posd = d(pos).view(w.batch)
        self.gpu.decode_step(d(k_new), d(v_new), posd, d(q_new).view(w.batch, w.n_q_heads, w.head_dim),
                             d(x_new).view(w.batch, -1), d(pos - getattr(self, "qpos_shift", 0)).view(w.batch),
                             budget, w.lam, w.eta, debug=True)
        torch.cuda.synchronize()
        bi_t = torch.tensor(self.batch_ids, device=k_new.device)
        sel = lambda x: f64(x.index_select(0, bi_t))
        posn = pos.numpy()[self.batch_ids]
        xn = sel(x_new)
        ref = self.ref.step(sel(k_new), sel(v_new), xn, posn, sel(q_new), xn,
                            (pos - getattr(self, "qpos_shift", 0)).numpy()[self.batch_ids], sel(q_new)[:, 0], budget,
                            w.lam, w.eta)
        if check:
            self.compare(*ref, tag, fused=True)
        return ref

    # -- a follower layer of an index-sharing group (Appendix, IndexCache-style reuse) -------------
    def _follow(self, k_new, v_new, x_new, pos, q_attn, evict, tag):
        bi_t = torch.tensor(self.batch_ids)
        sel = lambda x: f64(x.index_select(0, bi_t))
        self.ref.append_kv_hidden(sel(k_new), sel(v_new), sel(x_new), pos.numpy()[self.batch_ids])
        keep = [np.setdiff1d(np.arange(int(self.ref.len[ib])), evict[ib]).astype(np.int64)
                for ib in range(len(self.batch_ids))]
        self.ref.memory_update(evict, self.w.lam, self.w.eta)
        self.ref.compact_kv(keep, evict)
        out, res = self.ref.decode_attn_with_readout(sel(q_attn))
        self.compare(None, None, None, out, res, tag, lists=False)

    def follow_event(self, t0: int, t1: int, leader: "LockStepShared", evict, tag: str):
        w, d = self.w, (lambda x: x.to(self.dev))
        k_new = self.K[:, :, t0:t1].contiguous(); v_new = self.V[:, :, t0:t1].contiguous()
        x_new = self.X[:, t0:t1].contiguous()
        pos = (torch.arange(t0, t1, dtype=torch.int32).repeat(w.batch, 1) + self.pos_offsets()).contiguous()
        q_attn = self.Q[:, t1 - 1].contiguous()
        self.gpu.follow_event(d(k_new), d(v_new), d(pos), d(q_attn), leader.gpu, w.lam, w.eta, x_new=d(x_new))
        torch.cuda.synchronize()
        self._follow(k_new, v_new, x_new, pos, q_attn, evict, tag)

    def follow_step(self, t: int, leader: "LockStepShared", evict, tag: str):
        w, d = self.w, (lambda x: x.to(self.dev))
        k_new = self.K[:, :, t:t + 1].contiguous(); v_new = self.V[:, :, t:t + 1].contiguous()
        x_new = self.X[:, t:t + 1].contiguous(); q = self.Q[:, t].contiguous()
        pos = torch.full((w.batch, 1), t, dtype=torch.int32) + self.pos_offsets()
        self.gpu.follow_step(d(k_new), d(v_new), d(pos).view(-1), d(q), leader.gpu.evicted, w.lam, w.eta, debug=True,
                             x_new=d(x_new))
        torch.cuda.synchronize()
        self._follow(k_new, v_new, x_new, pos, q, evict, tag)

    def compare_decision(self, evict, tag):
        evicted = self.gpu.evicted.cpu().numpy(); lens = self.gpu.st.len.cpu().numpy()
        for ib, b in enumerate(self.batch_ids):
            assert len(evict[ib]) <= 1, f"{tag} sequence {b}"
            want = int(evict[ib][0]) if len(evict[ib]) else -1
            assert evicted[b] == want, f"{tag} sequence {b}: evicted slot {evicted[b]} != {want}"
            assert lens[b] == int(self.ref.len[ib]), f"{tag} sequence {b}: length"

    def compare(self, scores, keep, evict, out, res, tag, fused=False, lists=True, outputs=True):
        w, g, st = self.w, self.gpu, self.gpu.st
        G = w.group
        n_keep = g.n_keep.cpu().numpy(); n_evict = g.n_evict.cpu().numpy()
        keep_idx = g.keep_idx.cpu().numpy(); evict_idx = g.evict_idx.cpu().numpy()
        sc = g.scores.cpu().numpy()
        lens = st.len.cpu().numpy(); nproj = st.n_projected.cpu().numpy(); pos = st.pos.cpu().numpy()
        out_g = f64(g.out).reshape(w.batch, w.n_kv_heads, G, w.head_dim)
        res_g = g.readout.cpu().numpy().astype(np.float64).reshape(w.batch, w.n_kv_heads, G, w.head_dim)
        Mg = st.M.cpu().numpy().astype(np.float64); bg = st.b.cpu().numpy().astype(np.float64)
        for ib, b in enumerate(self.batch_ids):
            u = f"{tag} sequence {b}"
            if lists:
                kr, er = keep[ib], evict[ib]
                n_before = len(kr) + len(er)
                s_ref = scores[ib, :n_before]; s_gpu = sc[b, :n_before].astype(np.float64)
                same = (s_ref == s_gpu) | (np.isneginf(s_ref) & np.isneginf(s_gpu))
                assert same.all(), (f"{u}: {int((~same).sum())} of {n_before} scores differ, max "
                                    f"{np.nanmax(np.abs(np.where(same, 0, s_ref - s_gpu))):.3e}")
                if fused:
                    assert len(er) <= 1, u
                    want_e = int(er[0]) if len(er) else -1
                    got_e = int(g.evicted.cpu().numpy()[b])
                    assert got_e == want_e, f"{u}: evicted slot {got_e} != {want_e}"
                else:
                    assert n_keep[b] == len(kr) and n_evict[b] == len(er), u
                    assert np.array_equal(keep_idx[b, :len(kr)], kr), f"{u}: keep list differs"
                    assert np.array_equal(evict_idx[b, :len(er)], er), f"{u}: evict list differs"
            n = int(self.ref.len[ib])
            assert lens[b] == n and nproj[b] == n, u
            assert np.array_equal(pos[b, :n], self.ref.pos[ib, :n]), f"{u}: positions"
            assert np.array_equal(f64(st.Kidx[b, :n]), self.ref.Kidx[ib, :n]), f"{u}: indexer keys"
            assert np.array_equal(f64(st.K[b, :, :n]), self.ref.K[ib, :, :n]), f"{u}: K rows"
            assert np.array_equal(f64(st.V[b, :, :n]), self.ref.V[ib, :, :n]), f"{u}: V rows"
            assert_state_close(u + " M", Mg[b], self.ref.M[ib])
            assert_state_close(u + " b", bg[b], self.ref.b[ib])
            if outputs:
                assert_out_close(u + " out", out_g[b], out[ib])
                dmax = float(np.max(np.abs(res_g[b] - res[ib])))
                assert dmax <= 1e-3 * float(np.max(np.abs(res[ib]))) + 1e-30, f"{u}: readout diff {dmax:.3e}"

    def window(self, t0: int, tau: int, budget: int, tag: str, fused=True):
        """The paper's decode schedule (Section 4, setup): tau tokens are appended and attended to one
        by one, then the interval's queries score the cache and it is cut back to `budget`."""
        w, dev = self.w, self.dev
        d = lambda x: x.to(dev)
        bi_t = torch.tensor(self.batch_ids, device=self.K.device)
        sel = lambda x: f64(x.index_select(0, bi_t))
        bi = self.batch_ids
        for t in range(t0, t0 + tau):
            k_new = self.K[:, :, t:t + 1].contiguous(); v_new = self.V[:, :, t:t + 1].contiguous()
            x_new = self.X[:, t:t + 1].contiguous(); q_attn = self.Q[:, t].contiguous()
            pos = torch.full((w.batch, 1), t, dtype=torch.int32) + self.pos_offsets()
            self.gpu.attend_step(d(k_new), d(v_new), d(pos), d(q_attn), fused=fused, x_new=d(x_new))
            torch.cuda.synchronize()
            self.ref.append_kv_hidden(sel(k_new), sel(v_new), sel(x_new), pos.numpy()[bi])
            out, res = self.ref.decode_attn_with_readout(sel(q_attn))
            self.compare(None, None, None, out, res, f"{tag} attend@{t}", lists=False)
        q_win = self.Q[:, t0:t0 + tau].contiguous(); x_win = self.X[:, t0:t0 + tau].contiguous()
        posw = torch.arange(t0, t0 + tau, dtype=torch.int32).repeat(w.batch, 1).contiguous()
        self.gpu.compress(d(q_win), d(x_win), d(posw), budget, w.lam, w.eta)
        torch.cuda.synchronize()
        scores = self.ref.index_score(sel(q_win), sel(x_win), posw.numpy()[bi])
        keep, evict = self.ref.topb_select(scores, budget)
        self.ref.memory_update(evict, w.lam, w.eta)
        self.ref.compact_kv(keep, evict)
        self.compare(scores, keep, evict, None, None, f"{tag} compress@{t0 + tau}", outputs=False)

    def run_window_schedule(self, tau: int, n_windows: int, fused=True):
        w = self.w
        self.event(0, w.context, w.budget, "prefill")
        im.im_set_max_live(self.handle, min(self.cap, w.budget + tau))
        for k in range(n_windows):
            self.window(w.context + k * tau, tau, w.budget, f"window {k}", fused=fused)
        assert im.im_query_status(self.handle) == 0

    def run_schedule(self, decode_steps=None, fused_decode=False, full_every=1):
        w = self.w
        steps = w.decode_steps if decode_steps is None else decode_steps
        L = w.context
        if w.prefill_chunk is None:
            self.event(0, L, w.budget, "prefill")
        else:
            for c0 in range(0, L, w.prefill_chunk):
                self.event(c0, min(L, c0 + w.prefill_chunk), w.budget, f"chunk@{c0}")
        im.im_set_max_live(self.handle, min(self.cap, w.budget + 1))
        for i, t in enumerate(range(L, L + steps)):
            if fused_decode:
                full = (i + 1) % full_every == 0 or i == steps - 1
                ref = self.event_fused(t, w.budget, f"fused decode@{t} (step {i + 1} of {steps})", check=full)
                if not full:
                    self.compare_decision(ref[2], f"fused decode@{t} (step {i + 1} of {steps})")
            else:
                self.event(t, t + 1, w.budget, f"decode@{t}")
        assert im.im_query_status(self.handle) == 0
