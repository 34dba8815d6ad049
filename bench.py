#!/usr/bin/env python3
"""Benchmark of the bounded-budget KV decode step on one MI355X.

A "step" is one pass of the whole hot path (append -> index score -> top-B select -> memory
update -> compaction -> decode attention + readout) over every layer of the workload, layers
issued one after another on one stream, inputs already resident in HBM.  The default workload
is configuration 3 (32/8 x 128 heads, 32 layers, batch 4, a 16384-token context evicted to a
budget of 2048): the 16K-context case the headline metric is quoted on.

Prints ONE JSON line with the whole-job decode throughput, the roofline record of the dominant
kernel and the CPU oracle's throughput on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

import numpy as np
import torch

import paper_2605_25475_amd as im
from workloads import WORKLOADS, Workload, hidden_stream, layer_params, token_stream

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(w: Workload) -> dict:
    """Bytes the method itself must move per layer-step of steady-state decode (n = B + 1 live
    entries per unit, one eviction): what the roofline fraction is priced against."""
    Bg, D = w.budget, w.head_dim
    units = w.batch * w.n_kv_heads
    if w.head_shared:
        # one indexer key (16 values), one decision and one memory per sequence; K / V per unit
        per_unit = {"kv": 2 * 2 * D * Bg, "evicted_row": 2 * 2 * D, "compaction_row": 2 * 2 * 2 * D}
        per_seq = {
            "indexer_keys": 2 * w.idx_dim * (Bg + 1),
            "new_key": 2 * w.gate_in_dim + 2 * w.idx_dim,      # the hidden state in, its indexer key out
            "memory_state": 2 * 4 * w.mem_dim * D + 2 * 4 * w.mem_dim,
            "compaction_row": 2 * (2 * w.idx_dim + 4),
        }
        per_layer = {
            "indexer_weights": 2 * (w.n_idx_heads * w.idx_dim * w.n_q_heads * D + w.n_idx_heads * w.gate_in_dim
                                    + w.idx_dim * w.gate_in_dim),
            "q_and_out": w.batch * w.n_q_heads * D * 2 * 2,
        }
        unit_total = sum(per_unit.values())
        layer_total = units * unit_total + w.batch * sum(per_seq.values()) + sum(per_layer.values())
        return {"per_unit": unit_total, "per_layer_step": layer_total, "main_kernel_per_launch": units * per_unit["kv"],
                "attention_kv_per_layer": units * per_unit["kv"], "detail": {**per_unit, **per_seq, **per_layer}}
    per_unit = {
        "indexer_keys": 2 * w.idx_dim * (Bg + 1),          # stream the indexer-key cache
        "kv": 2 * 2 * D * Bg,                              # stream retained K and V
        "new_key": 2 * D + 2 * w.idx_dim,                  # project the new key, store its indexer key
        "evicted_row": 2 * 2 * D,                          # K and V of the evicted entry
        "memory_state": 2 * 4 * w.mem_dim * D + 2 * 4 * w.mem_dim,   # M, b read + write
        "compaction_row": 2 * (2 * 2 * D + 2 * w.idx_dim + 4),
    }
    per_layer = {
        "indexer_weights": 2 * (w.n_idx_heads * w.idx_dim * w.n_q_heads * D + w.n_idx_heads * w.gate_in_dim),
        "q_and_out": w.batch * w.n_q_heads * D * 2 * 2,
    }
    unit_total = sum(per_unit.values())
    layer_total = units * unit_total + sum(per_layer.values())
    # the main kernel of the fused step (k_dec_main) streams the retained cache: the indexer key and
    # the K / V rows of the B entries its 128-key splits cover (the newest entry is the tail kernel's)
    main_kernel = units * (2 * w.idx_dim * Bg + per_unit["kv"])
    return {"per_unit": unit_total, "per_layer_step": layer_total, "main_kernel_per_launch": main_kernel,
            "attention_kv_per_layer": units * per_unit["kv"], "detail": {**per_unit, **per_layer}}


class Job:
    """All layers of a workload after their prefill eviction, plus pre-generated decode inputs."""

    def __init__(self, w: Workload, n_steps: int, device="cuda", log=lambda s: None, tau: int = 0, share: int = 1):
        self.w, self.dev = w, device
        cap = w.capacity
        n_q_max = w.context if w.prefill_chunk is None else w.prefill_chunk
        cfg = im.Config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, capacity=cap,
                        n_idx_heads=w.n_idx_heads, idx_dim=w.idx_dim, n_sink=w.n_sink, n_recent=w.n_recent,
                        fold_block=w.fold_block, max_queries=n_q_max, head_shared=int(w.head_shared))
        self.handle = im.Handle(cfg, device)
        self.layers, self.dec, self.qwin, self.tau, self.share, self.xdec, self.xwin = [], [], [], tau, share, [], []
        L = w.context
        # (the configuration's own number of decode steps is a parity-test size; the benchmark draws as
        # many tokens from the same seeded streams as it is asked to time)
        for li in range(w.n_layers):
            p = layer_params(w, li, device)
            params = im.Params(p["Uq"], p["G"], p["Uk"], p["Wtheta"], p["wg"], p["cg"],
                               p["norm_q_w"], p["norm_k_w"])
            layer = im.Layer(self.handle, params, device)
            K, V, Q = token_stream(w, li, device, n_tokens=L + n_steps)
            X = hidden_stream(w, li, device, n_tokens=L + n_steps) if w.head_shared else None
            im.im_set_max_live(self.handle, cap)
            chunk = L if w.prefill_chunk is None else w.prefill_chunk
            for c0 in range(0, L, chunk):
                c1 = min(L, c0 + chunk)
                pos = torch.arange(c0, c1, dtype=torch.int32, device=device).repeat(w.batch, 1).contiguous()
                q = Q[:, c0:c1].contiguous()
                if w.head_shared and li % share:
                    layer.follow_event(K[:, :, c0:c1].contiguous(), V[:, :, c0:c1].contiguous(), pos,
                                       Q[:, c1 - 1].contiguous(), self.layers[li - li % share], w.lam, w.eta,
                                       x_new=X[:, c0:c1].contiguous())
                elif w.head_shared:
                    x = X[:, c0:c1].contiguous()
                    layer.step(K[:, :, c0:c1].contiguous(), V[:, :, c0:c1].contiguous(), pos, q, x, pos,
                               Q[:, c1 - 1].contiguous(), w.budget, w.lam, w.eta, x_new=x)
                elif li % share:   # a follower of an index-sharing group applies its leader's lists
                    layer.follow_event(K[:, :, c0:c1].contiguous(), V[:, :, c0:c1].contiguous(), pos,
                                       Q[:, c1 - 1].contiguous(), self.layers[li - li % share], w.lam, w.eta)
                else:
                    layer.step(K[:, :, c0:c1].contiguous(), V[:, :, c0:c1].contiguous(), pos, q,
                               q.view(w.batch, c1 - c0, -1), pos, Q[:, c1 - 1].contiguous(), w.budget,
                               w.lam, w.eta)
            # decode inputs, one contiguous slab per step
            kd = K[:, :, L:].permute(2, 0, 1, 3).contiguous().unsqueeze(3)      # [S, B, Hkv, 1, D]
            vd = V[:, :, L:].permute(2, 0, 1, 3).contiguous().unsqueeze(3)
            qd = Q[:, L:].permute(1, 0, 2, 3).contiguous().unsqueeze(2)         # [S, B, 1, H, D]
            self.layers.append(layer)
            self.dec.append((kd, vd, qd))
            if w.head_shared:
                self.xdec.append(X[:, L:].permute(1, 0, 2).contiguous().unsqueeze(2))   # [S, B, 1, d_model]
            if tau:   # the query set of every compression interval, [B, tau, H, D] each
                self.qwin.append([Q[:, L + k * tau:L + (k + 1) * tau].contiguous() for k in range(n_steps // tau)])
                if w.head_shared:
                    self.xwin.append([X[:, L + k * tau:L + (k + 1) * tau].contiguous() for k in range(n_steps // tau)])
            del K, V, Q, X
            torch.cuda.synchronize()
            log(f"layer {li + 1}/{w.n_layers} prefilled")
        self.pos = (torch.arange(L, L + n_steps, dtype=torch.int32, device=device)
                    .view(n_steps, 1, 1).repeat(1, w.batch, 1).contiguous())
        im.im_set_max_live(self.handle, min(cap, w.budget + max(1, tau)))
        if tau:
            self.posw = [torch.arange(L + k * tau, L + (k + 1) * tau, dtype=torch.int32, device=device)
                         .repeat(w.batch, 1).contiguous() for k in range(n_steps // tau)]
        assert im.im_query_status(self.handle) == 0

    def step(self, s: int, path: str = "fused"):
        """One decode step over every layer, layers in order on the current stream."""
        w = self.w
        pos = self.pos[s]
        for li, layer in enumerate(self.layers):
            kd, vd, qd = self.dec[li]
            q = qd[s]
            if w.head_shared:
                x = self.xdec[li][s]
                if path == "shared" and li % self.share:
                    layer.follow_step(kd[s], vd[s], pos.view(w.batch), q.view(w.batch, w.n_q_heads, -1),
                                      self.layers[li - li % self.share].evicted, w.lam, w.eta, x_new=x)
                elif path in ("fused", "shared"):
                    layer.decode_step(kd[s], vd[s], pos.view(w.batch), q.view(w.batch, w.n_q_heads, -1),
                                      x.view(w.batch, -1), pos.view(w.batch), w.budget, w.lam, w.eta,
                                      want_evicted=(path == "shared"))
                elif path == "periodic":
                    layer.attend_step(kd[s], vd[s], pos, q.view(w.batch, w.n_q_heads, -1), debug=False, x_new=x)
                else:
                    layer.step(kd[s], vd[s], pos, q, x, pos, q.view(w.batch, w.n_q_heads, -1), w.budget, w.lam,
                               w.eta, x_new=x)
            elif path == "shared":
                if li % self.share:
                    layer.follow_step(kd[s], vd[s], pos.view(w.batch), q.view(w.batch, w.n_q_heads, -1),
                                      self.layers[li - li % self.share].evicted, w.lam, w.eta)
                else:
                    layer.decode_step(kd[s], vd[s], pos.view(w.batch), q.view(w.batch, w.n_q_heads, -1),
                                      q.view(w.batch, -1), pos.view(w.batch), w.budget, w.lam, w.eta,
                                      want_evicted=True)
            elif path == "periodic":
                layer.attend_step(kd[s], vd[s], pos, q.view(w.batch, w.n_q_heads, -1), debug=False)
            elif path == "fused":
                layer.decode_step(kd[s], vd[s], pos.view(w.batch), q.view(w.batch, w.n_q_heads, -1),
                                  q.view(w.batch, -1), pos.view(w.batch), w.budget, w.lam, w.eta)
            else:
                layer.step(kd[s], vd[s], pos, q, q.view(w.batch, 1, -1), pos, q.view(w.batch, w.n_q_heads, -1),
                           w.budget, w.lam, w.eta)
        if path == "periodic" and (s + 1) % self.tau == 0:
            k = s // self.tau
            for li, layer in enumerate(self.layers):
                qw = self.qwin[li][k]
                xg = self.xwin[li][k] if w.head_shared else qw.view(w.batch, self.tau, -1)
                layer.compress(qw, xg, self.posw[k], w.budget, w.lam, w.eta)


def stream_read_ceiling(nbytes: int, log) -> dict:
    """What a plain read achieves at the dominant kernel's bytes per launch: a hand-written kernel of
    16-byte streaming loads (im_stream_read), one launch per `nbytes` slab, the launches back to back in
    a HIP graph over more than 1.2 GB of distinct memory (so that no slab is found in the 256 MB
    last-level cache), replayed a few times."""
    nbytes = (nbytes + 15) // 16 * 16
    n_slabs = max(8, -(-1_300_000_000 // nbytes))
    buf = torch.empty(n_slabs * nbytes // 4, dtype=torch.int32, device="cuda")
    buf.random_(0, 1 << 30)                      # touched, non-constant pages
    sink = torch.zeros(64, dtype=torch.int32, device="cuda")
    flat = buf.view(torch.uint8)

    def launches():
        for i in range(n_slabs):
            im.im_stream_read(flat[i * nbytes:(i + 1) * nbytes], nbytes, 0xFFFFFFFF, sink)

    launches()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        launches()
    g.replay()
    torch.cuda.synchronize()
    reps = 5
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (reps * n_slabs)
    gbs = nbytes / (us * 1e-6) / 1e9
    log(f"plain streaming read of {nbytes / 1e6:.2f} MB per launch ({n_slabs} slabs, graph replay): "
        f"{us:.2f} us per launch -> {gbs:.0f} GB/s")
    del buf
    return {"ceiling_GBps": gbs, "ceiling_us_per_launch": us, "ceiling_bytes_per_launch": nbytes,
            "ceiling_kind": "k_stream_read: 16-byte streaming loads, one launch per slab, back-to-back launches "
                            f"in a HIP graph over {n_slabs} distinct slabs"}


def cpu_baseline(w: Workload, budget_s: float = 20.0) -> dict:
    """The oracle, as it stands, on one unit of the same workload: its own prefill eviction at
    full context (untimed here, it only builds a realistic state), then timed decode steps."""
    from helpers import f64, make_oracle_layer
    try:
        from threadpoolctl import threadpool_info
        threads = max([t.get("num_threads", 1) for t in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    n_steps = min(512, w.decode_steps)
    nb = min(4, w.batch)
    heads = list(range(w.n_kv_heads))
    ws = w.scaled(batch=nb)
    L = w.context
    spent, done_pairs, done = 0.0, 0, 0
    for layer in range(min(2, w.n_layers)):       # up to two layers' worth of pairs, within the budget
        K, V, Q = token_stream(w, layer, "cpu", n_tokens=w.context + n_steps + 64)
        if w.head_shared:
            ref = make_oracle_layer(ws, layer, "cpu", capacity=w.context + 1, batch=nb)
            X = f64(hidden_stream(w, layer, "cpu", n_tokens=w.context + n_steps + 64)[:nb])
        else:
            ref = make_oracle_layer(ws, layer, "cpu", capacity=w.context + 1, batch=nb, kv_head_ids=heads)
        K, V, Q = f64(K[:nb]), f64(V[:nb]), f64(Q[:nb])
        # build the post-prefill state cheaply, for TIMING purposes only: score with the last 64
        # prompt queries (the parity tests, not this leg, check the full-context event)
        nq = 64
        pos = np.tile(np.arange(L, dtype=np.int32), (nb, 1))
        q = Q[:, L - nq:L]
        if w.head_shared:
            ref.append_kv_hidden(K[:, :, :L], V[:, :, :L], X[:, :L], pos)
            sc = ref.index_score(q, X[:, L - nq:L], pos[:, L - nq:])
        else:
            ref.append_kv(K[:, :, :L], V[:, :, :L], pos)
            sc = ref.index_score(q, q.reshape(nb, nq, -1), pos[:, L - nq:])
        keep, evict = ref.topb_select(sc, w.budget)
        ref.memory_update(evict, w.lam, w.eta)
        ref.compact_kv(keep, evict)
        t0 = time.perf_counter()
        for s in range(n_steps):
            t = L + s
            p = np.full((nb, 1), t, np.int32)
            qs = Q[:, t:t + 1]
            if w.head_shared:
                ref.step(K[:, :, t:t + 1], V[:, :, t:t + 1], X[:, t:t + 1], p, qs, X[:, t:t + 1], p, Q[:, t],
                         w.budget, w.lam, w.eta)
            else:
                ref.step(K[:, :, t:t + 1], V[:, :, t:t + 1], p, qs, qs.reshape(nb, 1, -1), p, Q[:, t], w.budget,
                         w.lam, w.eta)
            done_pairs += nb
            done += 1
            if spent + time.perf_counter() - t0 > budget_s:
                break
        spent += time.perf_counter() - t0
        if spent > budget_s:
            break
    dt = spent / done_pairs                        # one decode step of one (layer, batch element)
    pairs = w.batch * w.n_layers
    # the same steps with the numerical library held to ONE thread (the oracle's python loops are
    # single-threaded anyway; only its matrix products fan out), on the state the timed run left
    single = None
    try:
        from threadpoolctl import threadpool_limits
        n1 = max(1, min(done, 64, int(6.0 / (dt * nb))))
        with threadpool_limits(limits=1):
            t1 = time.perf_counter()
            for s in range(n_steps, n_steps + n1):
                t = L + s
                if t >= K.shape[2]:
                    break
                p = np.full((nb, 1), t, np.int32)
                qs = Q[:, t:t + 1]
                if w.head_shared:
                    ref.step(K[:, :, t:t + 1], V[:, :, t:t + 1], X[:, t:t + 1], p, qs, X[:, t:t + 1], p, Q[:, t],
                             w.budget, w.lam, w.eta)
                else:
                    ref.step(K[:, :, t:t + 1], V[:, :, t:t + 1], p, qs, qs.reshape(nb, 1, -1), p, Q[:, t], w.budget,
                             w.lam, w.eta)
                n1_done = s - n_steps + 1
            dt1 = (time.perf_counter() - t1) / (n1_done * nb)
        single = {"value": w.batch / (dt1 * pairs), "unit": "tokens/s", "threads": 1,
                  "sample": f"{n1_done} further decode steps of the same pairs, {dt1 * 1e3:.2f} ms per pair-step"}
    except Exception as exc:   # threadpoolctl missing or the sample ran out of tokens: all-threads figure only
        single = {"value": None, "note": f"not measured: {exc}"}
    return {"value": w.batch / (dt * pairs), "unit": "tokens/s", "cores": int(threads), "threads": int(threads),
            "kind": "oracle", "single_thread": single,
            "sample": (f"{done} decode steps of all {w.n_kv_heads} KV heads of {nb} (layer, batch element) pairs at a time "
                       f"(from the first {min(2, w.n_layers)} layer(s); {done_pairs} pair-steps in all, the workload has {pairs} pairs) at budget {w.budget}: "
                       f"{dt * 1e3:.2f} ms per pair-step, {spent:.1f} s of CPU work, extrapolated to all pairs run one "
                       f"after another; `cores` is the thread count of the numerical library's pool ({threads}), the oracle's "
                       "own loops are single-threaded")}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg3", choices=sorted(WORKLOADS))
    ap.add_argument("--path", default="fused", choices=["fused", "steps", "periodic", "shared"],
                    help="fused: im_decode_step (3 launches per layer); steps: the six separate calls; "
                         "periodic: the paper's decode schedule (append + attention every step, one "
                         "compression event per --tau steps with the interval's queries as the query set); "
                         "shared: index reuse over groups of --share consecutive layers (the first layer "
                         "of a group scores and selects, the others apply its decision)")
    ap.add_argument("--head-shared", action="store_true",
                    help="the workload's cache shape in the head-shared layout (indexer keys of 16 values from "
                         "hidden states, one eviction set and one memory per sequence)")
    ap.add_argument("--share", type=int, default=4, help="layers per index-sharing group of --path shared")
    ap.add_argument("--tau", type=int, default=128, help="compression interval of --path periodic")
    ap.add_argument("--no-graph", action="store_true", help="launch the fused path eagerly")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (torch copy_) so that a counter run "
                         "has a dispatch of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quiet", action="store_true")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
                 "(units would shard by batch or by KV head with no communication)")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    w = WORKLOADS[a.workload]
    if a.head_shared:
        w = w.shared()
    log = (lambda s: None) if a.quiet else (lambda s: print("[bench] " + s, file=sys.stderr, flush=True))
    torch.cuda.set_device(0)
    tau = a.tau if a.path == "periodic" else 0
    if tau:
        if a.steps % tau or a.warmup % tau:
            sys.exit(f"bench.py: with --path periodic, --steps and --warmup must be multiples of --tau ({tau})")
        assert w.budget + tau <= w.capacity
    n_total = a.warmup + (1 if tau else 2) * a.steps
    if a.steps < 1 or a.warmup < 0 or n_total > 8192:
        sys.exit("bench.py: --steps must be >= 1, --warmup >= 0, and warmup + 2 x steps at most 8192")
    t_setup = time.perf_counter()
    job = Job(w, n_total, log=log, tau=tau, share=a.share if a.path == "shared" else 1)
    torch.cuda.synchronize()
    log(f"setup (generation + prefill eviction of {w.n_layers} layers) {time.perf_counter() - t_setup:.1f} s")

    if a.pmc_calibration:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    use_graph = (a.path in ("fused", "periodic", "shared")) and not a.no_graph

    def run(s0, s1):
        for s in range(s0, s1):
            job.step(s, a.path)

    def graphed(s0, s1):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run(s0, s1)
        return g

    # warm-up, then EXACTLY a.steps timed steps.  With --path fused the steps are replayed from
    # HIP graphs (one graph holds all timed steps, each with its own input slices), so the host's
    # launch cost is outside the loop; the state advances exactly as in eager execution.
    w0, t0s, t1s = 0, a.warmup, a.warmup + a.steps
    if use_graph:
        gw = graphed(w0, t0s) if a.warmup > 0 else None
        gt = graphed(t0s, t1s)
        if gw is not None:
            gw.replay()
    else:
        run(w0, t0s)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    if use_graph:
        gt.replay()
    else:
        run(t0s, t1s)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / a.steps
    log(f"timed {a.steps} steps ({'graph replay' if use_graph else 'eager'}): {ms_per_step:.4f} ms/step wall, "
        f"{e0.elapsed_time(e1) / a.steps:.4f} ms/step between stream events")
    assert im.im_query_status(job.handle) == 0

    # dominant kernel: the same number of further steps, eager, with HIP events that the library
    # records on the launch stream.  An event pair around one launch also spans the hand-over
    # between the event and the dispatch, so the main kernel is timed as it runs behind the prep
    # kernel: (prep + main, no event between them) - (prep alone), half of the steps each.
    ab = algorithmic_bytes(w)
    roof = None
    if a.path == "fused":
        half = max(1, a.steps // 2)
        im.im_profile_start(job.handle, half * w.n_layers, im.IM_PROFILE_PREP_AND_MAIN)
        run(t1s, t1s + half)
        d_pm = im.im_profile_stop(job.handle)
        im.im_profile_start(job.handle, half * w.n_layers, im.IM_PROFILE_PREP)
        run(t1s + half, t1s + 2 * half)
        d_p = im.im_profile_stop(job.handle)
        k_ms = float(np.mean(d_pm)) - float(np.mean(d_p))
        durs = d_pm
        kname = "k_att_main" if w.head_shared else "k_dec_main"   # the launch that streams the cache
        achieved = ab["main_kernel_per_launch"] / (k_ms * 1e-3) / 1e9
        traffic = None
        tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{w.name}.json")
        if os.path.exists(tpath):   # HBM bytes per launch from the committed rocprofv3 --pmc summary
            with open(tpath) as f:
                traffic = json.load(f)["kernels"].get(f"{kname}<{w.group}>", {}).get("total_bytes")
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "kernel": kname,
                "avg_launch_us": k_ms * 1e3, "launches_timed": len(durs),
                "prep_and_main_us": float(np.mean(d_pm)) * 1e3, "prep_us": float(np.mean(d_p)) * 1e3,
                "bytes_per_launch": ab["main_kernel_per_launch"]}
        log(f"{kname}: {k_ms * 1e3:.2f} us per launch over {len(durs)} launches -> {achieved:.0f} GB/s")
        # the measured ceiling beside the published peak: a plain read of the same bytes per launch
        roof.update(stream_read_ceiling(ab["main_kernel_per_launch"], log))
        roof["frac_of_ceiling"] = achieved / roof["ceiling_GBps"]
        # ... and the whole step (every launch of every layer) against both
        whole = ab["per_layer_step"] * w.n_layers / (wall / a.steps) / 1e9
        roof["whole_step"] = {"achieved": whole, "frac": whole / HBM_PEAK_GBS,
                              "frac_of_ceiling": whole / roof["ceiling_GBps"],
                              "bytes_per_step": ab["per_layer_step"] * w.n_layers}
    assert im.im_query_status(job.handle) == 0

    step_s = wall / a.steps
    rec = {
        "metric": "decode tokens/s with eviction+memory at 16K ctx; achieved HBM GB/s vs peak",
        "value": w.batch / step_s, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_q_heads}/{w.n_kv_heads}x{w.head_dim} heads, {w.n_layers} layers, "
                               f"batch {w.batch}, context {w.context} -> budget {w.budget}, "
                               + (f"one compression event per {tau} decode steps" if tau else "one eviction per decode step")
                               + (f", index decisions shared by groups of {a.share} layers" if a.path == "shared" else "")
                               + (", head-shared layout (indexer keys of 16 values from hidden states, one "
                                  "eviction set and one memory per sequence)" if w.head_shared else ""),
                   "layers": w.n_layers, "batch": w.batch, "budget": w.budget, "context": w.context,
                   "path": a.path, "hip_graph": use_graph,
                   "algorithmic_bytes_per_step": ab["per_layer_step"] * w.n_layers,
                   "whole_step_GBps": ab["per_layer_step"] * w.n_layers / step_s / 1e9,
                   "whole_step_frac_of_peak": ab["per_layer_step"] * w.n_layers / step_s / 1e9 / HBM_PEAK_GBS},
        "roofline": roof,
    }
    if not a.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        rec["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
