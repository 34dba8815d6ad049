"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs, event by event (see parity.py for the bars)."""
import numpy as np
import pytest
import torch

import paper_2605_25475_amd as im
from oracle import indexmem_oracle as O
from helpers import f64
from parity import LockStep, LockStepShared
from workloads import WORKLOADS

pytestmark = pytest.mark.gpu


def test_cfg1_full_trajectory():
    # configuration 1 as stated: 1024 -> 256, 16 decode steps, all 8 units
    LockStep(WORKLOADS["cfg1"]).run_schedule()


@pytest.mark.parametrize("name,kw", [
    # reduced copies of the other configurations: same head shapes and distributions, sizes that
    # span several tiles of every kernel (64-row projection tiles, 256-key score / attention
    # chunks, 16-row memory sub-tiles, 64-row fold blocks) and leave ragged tails
    ("cfg2", dict(batch=2, context=1100, budget=300, decode_steps=3)),
    ("cfg3", dict(batch=2, context=1500, budget=333, decode_steps=3)),
    ("cfg4", dict(batch=3, context=1300, budget=130, decode_steps=3)),
    ("cfg5", dict(batch=1, context=1536, budget=512, decode_steps=3, prefill_chunk=512)),
])
def test_reduced_configurations(name, kw):
    LockStep(WORKLOADS[name].scaled(n_layers=1, **kw)).run_schedule()


def test_cfg1_full_trajectory_fused_decode():
    # the same trajectory with every decode step through im_decode_step (three launches per step)
    LockStep(WORKLOADS["cfg1"]).run_schedule(fused_decode=True)


@pytest.mark.parametrize("name,kw", [
    ("cfg2", dict(batch=2, context=1100, budget=300, decode_steps=4)),
    ("cfg3", dict(batch=2, context=1500, budget=333, decode_steps=4)),
    ("cfg4", dict(batch=3, context=1300, budget=130, decode_steps=4)),       # 7 query heads per KV head
    ("cfg4", dict(batch=2, context=700, budget=128, decode_steps=3)),        # n = 129: a one-key last split
    ("cfg4", dict(batch=1, context=1500, budget=1200, decode_steps=3)),      # 10 splits: two staging rounds in the tail
    ("cfg5", dict(batch=1, context=1536, budget=512, decode_steps=4, prefill_chunk=512)),
    ("cfg1", dict(context=40, budget=64, decode_steps=30)),                  # grows to the budget, then evicts
    ("cfg1", dict(context=300, budget=64, decode_steps=3, n_recent=8)),      # recent window forced
    ("cfg1", dict(n_q_heads=40, context=600, budget=150, decode_steps=3)),   # 10 indexer heads, 5 per group
    ("cfg1", dict(n_q_heads=16, context=600, budget=150, decode_steps=3)),   # 4 indexer heads, 2 per group
    ("cfg1", dict(n_q_heads=64, context=500, budget=140, decode_steps=3)),   # 16 indexer heads, 8 per group
    ("cfg1", dict(n_q_heads=8, context=500, budget=140, decode_steps=3)),    # 2 indexer heads, 1 per group
    ("cfg1", dict(batch=64, n_kv_heads=2, n_q_heads=8, context=150, budget=40, decode_steps=2)),   # the largest batch
    ("cfg1", dict(batch=11, context=260, budget=4, decode_steps=3)),         # budget = the sinks alone; projection blocks of 8 + 3 batch rows
    ("cfg1", dict(batch=5, context=200, budget=48, decode_steps=2)),         # projection blocks of 4 + 1 batch rows
    ("cfg1", dict(batch=12, n_kv_heads=2, n_q_heads=8, context=150, budget=40, decode_steps=2)),   # three blocks of 4 batch rows
])
def test_reduced_configurations_fused_decode(name, kw):
    w = WORKLOADS[name].scaled(n_layers=1, **kw)
    LockStep(w, capacity=max(w.capacity, w.budget + 2)).run_schedule(fused_decode=True)


@pytest.mark.parametrize("name,kw,tau,n_win", [
    ("cfg1", dict(context=600, budget=200, decode_steps=96), 32, 3),
    ("cfg1", dict(context=500, budget=160, decode_steps=80, n_recent=16), 40, 2),   # recent window kept
    ("cfg4", dict(batch=2, context=700, budget=130, decode_steps=128), 128, 1),      # the paper's tau
    ("cfg3", dict(batch=1, context=900, budget=300, decode_steps=48), 24, 2),
    ("cfg1", dict(context=500, budget=200, decode_steps=114), 57, 2),    # live bound 257: one key beyond the splits
    ("cfg1", dict(batch=2, context=300, budget=100, decode_steps=15), 5, 3),    # 5 queries < 8 indexer heads: the few-query scoring kernel
    ("cfg4", dict(batch=2, context=300, budget=70, decode_steps=12), 6, 2),     # 6 queries < 7 heads
    ("cfg1", dict(batch=2, context=300, budget=100, decode_steps=22), 11, 2),   # 8 heads <= 11 queries < 16: one ragged query block of the many-query kernel
    ("cfg1", dict(batch=1, context=260, budget=90, decode_steps=16), 8, 2),     # exactly as many queries as indexer heads
])
@pytest.mark.parametrize("fused", [True, False])
def test_periodic_compression_schedule(name, kw, tau, n_win, fused):
    # Section 4 (setup): attention every step, compression once per interval with the interval's
    # queries as the query set; the cache grows to budget + tau between compressions
    w = WORKLOADS[name].scaled(n_layers=1, **kw)
    ls = LockStep(w, capacity=max(w.context, w.budget + tau), max_queries=max(w.context, tau))
    ls.run_window_schedule(tau, n_win, fused=fused)


@pytest.mark.parametrize("name,kw", [
    ("cfg1", dict(context=700, budget=256, decode_steps=6)),
    ("cfg4", dict(batch=2, context=600, budget=130, decode_steps=5)),     # 7 query heads per KV head
    ("cfg3", dict(batch=1, context=2900, budget=2700, decode_steps=3)),   # 22 splits: two staging rounds
])
def test_index_reuse_across_layers(name, kw):
    # Appendix "From Running Mean to IndexCache": layer 0 scores and selects; layer 1 (its own
    # weights and K / V / Q) applies layer 0's lists at the prefill event and layer 0's evicted slot
    # at every decode step
    w = WORKLOADS[name].scaled(n_layers=2, **kw)
    lead = LockStep(w, layer=0, capacity=max(w.capacity, w.budget + 2))
    foll = LockStep(w, layer=1, capacity=max(w.capacity, w.budget + 2))
    _, _, evict, _, _ = lead.event(0, w.context, w.budget, "leader prefill")
    foll.follow_event(0, w.context, lead, evict, "follower prefill")
    for ls in (lead, foll):
        im.im_set_max_live(ls.handle, w.budget + 1)
    for t in range(w.context, w.context + w.decode_steps):
        _, _, evict, _, _ = lead.event_fused(t, w.budget, f"leader decode@{t}")
        foll.follow_step(t, lead, evict, f"follower decode@{t}")
    assert im.im_query_status(lead.handle) == 0 and im.im_query_status(foll.handle) == 0
    # a follower never reads its indexer keys, but the keys of the tokens it appended while decoding
    # must still be those tokens' keys wherever the hole filling has moved them
    from helpers import f64, oracle_params
    from workloads import layer_params
    p = oracle_params(layer_params(w, 1))
    st = foll.gpu.st
    pos = st.pos.cpu().numpy(); lens = st.len.cpu().numpy()
    seen = 0
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            n = int(lens[b, h])
            new = np.nonzero(pos[b, h, :n] >= w.context)[0]
            want = O.key_feature(f64(st.K[b, h, :n])[new], p.Uk, p.norm_k_w, float(np.float32(1e-6)))
            assert np.array_equal(f64(st.Kidx[b, h, :n])[new], want), f"follower unit ({b},{h}): moved indexer keys"
            seen += len(new)
    assert seen > 0


@pytest.mark.parametrize("name,kw", [
    ("cfg1", dict(batch=2, context=700, budget=256, decode_steps=6)),
    ("cfg4", dict(batch=2, context=600, budget=130, decode_steps=5)),     # 7 query heads per KV head
])
def test_index_reuse_across_layers_head_shared_layout(name, kw):
    w = WORKLOADS[name].shared(n_layers=2, **kw)
    cap = max(w.capacity, w.budget + 2)
    lead, foll = LockStepShared(w, layer=0, capacity=cap), LockStepShared(w, layer=1, capacity=cap)
    _, _, evict, _, _ = lead.event(0, w.context, w.budget, "leader prefill")
    foll.follow_event(0, w.context, lead, evict, "follower prefill")
    for ls in (lead, foll):
        im.im_set_max_live(ls.handle, w.budget + 1)
    for t in range(w.context, w.context + w.decode_steps):
        _, _, evict, _, _ = lead.event_fused(t, w.budget, f"leader decode@{t}")
        foll.follow_step(t, lead, evict, f"follower decode@{t}")
    assert im.im_query_status(lead.handle) == 0 and im.im_query_status(foll.handle) == 0
    # a follower never reads its indexer keys, but the keys of the tokens it appended while decoding
    # must still be those tokens' keys wherever the hole filling has moved them
    from helpers import f64, oracle_params
    from workloads import layer_params
    p = oracle_params(layer_params(w, 1))
    st = foll.gpu.st
    pos = st.pos.cpu().numpy(); lens = st.len.cpu().numpy()
    seen = 0
    for b in range(w.batch):
        n = int(lens[b])
        new = np.nonzero(pos[b, :n] >= w.context)[0]
        want = O.key_feature(f64(foll.X[b])[pos[b, :n][new]], p.Uk, p.norm_k_w, float(np.float32(1e-6)))
        assert np.array_equal(f64(st.Kidx[b, :n])[new], want), f"follower sequence {b}: moved indexer keys"
        seen += len(new)
    assert seen > 0


def test_fused_decode_ties_evict_newest_then_largest_slot():
    # a zero gate makes every visible score 0: the entry ranked last is the newest position
    w = WORKLOADS["cfg1"].scaled(context=200, budget=200, decode_steps=5, param_std=0.0)
    ls = LockStep(w, capacity=256)
    ls.run_schedule(fused_decode=True)
    assert int(ls.gpu.st.len.max()) == 200


def test_recent_window_and_budget_above_context():
    w = WORKLOADS["cfg1"].scaled(context=300, budget=64, decode_steps=2, n_recent=8)
    LockStep(w).run_schedule()
    # budget >= context: nothing evicted, memory untouched, plain attention
    w2 = WORKLOADS["cfg1"].scaled(context=200, budget=256, decode_steps=2)
    ls = LockStep(w2, capacity=300)
    ls.run_schedule()
    assert float(ls.gpu.st.M.abs().max()) == 0.0 and float(ls.gpu.st.b.abs().max()) == 0.0
    assert int(ls.gpu.st.len.min()) == 202


def _select_case(scores_np, pos_np, budget, n_sink=4, n_recent=0, lens=None):
    """Run im_topb_select on hand-made scores; compare with the oracle's select()."""
    Bz, Hk, Cc = scores_np.shape
    cfg = im.Config(batch=Bz, n_q_heads=Hk, n_kv_heads=Hk, capacity=Cc, n_idx_heads=1,
                    n_sink=n_sink, n_recent=n_recent)
    h = im.Handle(cfg)
    st = im.State(cfg)
    lens = np.full((Bz, Hk), Cc, np.int32) if lens is None else lens
    st.len.copy_(torch.tensor(lens)); st.pos.copy_(torch.tensor(pos_np))
    sc = torch.tensor(scores_np, dtype=torch.float32, device="cuda")
    keep = torch.full((Bz, Hk, Cc), -1, dtype=torch.int32, device="cuda")
    evict = torch.full((Bz, Hk, Cc), -1, dtype=torch.int32, device="cuda")
    nk = torch.zeros((Bz, Hk), dtype=torch.int32, device="cuda"); ne = torch.zeros_like(nk)
    im.im_topb_select(h, sc, st, budget, keep, evict, nk, ne)
    torch.cuda.synchronize()
    for b in range(Bz):
        for hh in range(Hk):
            n = int(lens[b, hh])
            k_ref, e_ref = O.select(scores_np[b, hh, :n].astype(np.float32).astype(np.float64),
                                    pos_np[b, hh, :n], budget, n_sink, n_recent)
            assert int(nk[b, hh]) == len(k_ref) and int(ne[b, hh]) == len(e_ref)
            assert np.array_equal(keep[b, hh, :len(k_ref)].cpu().numpy(), k_ref)
            assert np.array_equal(evict[b, hh, :len(e_ref)].cpu().numpy(), e_ref)


def test_select_ties_infinities_and_degenerate_sizes():
    rng = np.random.default_rng(7)
    Cc = 3000
    pos = np.stack([rng.permutation(Cc) for _ in range(6)]).reshape(2, 3, Cc).astype(np.int32)
    cases = {
        "quantised": rng.integers(0, 4, (2, 3, Cc)).astype(np.float32),
        "all_equal": np.zeros((2, 3, Cc), np.float32),
        "signed_zero": np.where(rng.integers(0, 2, (2, 3, Cc)) == 0, 0.0, -0.0).astype(np.float32),
        "infs": rng.choice(np.array([-np.inf, np.inf, 0.0, 1.5, -2.0], np.float32), (2, 3, Cc)),
        "random": rng.standard_normal((2, 3, Cc)).astype(np.float32),
        "tiny_spread": (1.0 + 1e-7 * rng.integers(0, 5, (2, 3, Cc))).astype(np.float32),
    }
    lens = np.array([[Cc, 1, 0], [5, 1025, 2047]], np.int32)
    for name, sc in cases.items():
        for budget in (4, 5, 1024, 2999, 3000):
            _select_case(sc, pos, budget, lens=lens)
        _select_case(sc, pos, 100, n_sink=0, n_recent=3, lens=lens)
    # duplicate positions: the slot index breaks the remaining ties
    pos_dup = (pos // 7).astype(np.int32)
    _select_case(cases["quantised"], pos_dup, 500, lens=lens)
    _select_case(cases["all_equal"], pos_dup, 77, lens=lens)
    # exactly one entry leaves (units of 3000, 1025 and 5 entries): the slot index decides among equal
    # (score, position) pairs there too
    for budget in (2999, 1024, 4):
        _select_case(cases["quantised"], pos_dup, budget, lens=lens)
        _select_case(cases["all_equal"], pos_dup, budget, lens=lens)
        _select_case(cases["infs"], pos_dup, budget, n_sink=0, n_recent=2, lens=lens)


@pytest.mark.parametrize("shared", [False, True], ids=["per-unit", "head-shared"])
def test_events_of_one_to_six_new_tokens(shared):
    # events that append m tokens and evict m entries, m = 1 .. 6: the sizes around which the kernels of the
    # step-by-step calls change paths (up to 4 new rows are projected, and up to 4 evicted rows folded into
    # the memory, without the matrix-core tiles; a single eviction is selected by one reduction; the
    # compaction probes the shorter of its two lists)
    kw = dict(context=300, budget=140, decode_steps=32, batch=2, n_layers=1)
    w = WORKLOADS["cfg1"].shared(**kw) if shared else WORKLOADS["cfg1"].scaled(**kw)
    ls = (LockStepShared if shared else LockStep)(w, capacity=w.context + 32)
    ls.event(0, w.context, w.budget, "prefill")
    t = w.context
    for m in (1, 2, 3, 4, 5, 6, 4, 1):
        ls.event(t, t + m, w.budget, f"event of {m} tokens at {t}")
        t += m
    assert im.im_query_status(ls.handle) == 0


def test_empty_and_single_entry_units_through_the_whole_step():
    # a unit with nothing cached attends to nothing: output = gated readout of an empty memory = 0
    w = WORKLOADS["cfg1"].scaled(context=1, budget=8, decode_steps=2)
    ls = LockStep(w, capacity=16)
    ls.run_schedule()
    cfg = ls.handle.cfg
    st = im.State(cfg)
    q = torch.randn((1, 32, 128), device="cuda").to(torch.bfloat16)
    out = torch.full((1, 32, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    im.im_decode_attn_with_readout(ls.handle, ls.params, st, q, out, None)
    torch.cuda.synchronize()
    assert float(out.float().abs().max()) == 0.0


def test_append_overflow_sets_status_and_leaves_state():
    cfg = im.Config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=8, n_idx_heads=2)
    h = im.Handle(cfg); st = im.State(cfg)
    k = torch.ones((1, 2, 5, 128), dtype=torch.bfloat16, device="cuda")
    p = torch.arange(5, dtype=torch.int32, device="cuda").view(1, 5)
    im.im_append_kv(h, st, k, k, p)
    assert im.im_query_status(h) == 0 and st.len.tolist() == [[5, 5]]
    im.im_append_kv(h, st, k, k, p)
    assert im.im_query_status(h) == im.IM_STATUS_APPEND_OVERFLOW
    assert st.len.tolist() == [[5, 5]] and float(st.K[0, 0, 5:].float().abs().max()) == 0.0
    assert im.im_query_status(h) == 0


@pytest.mark.parametrize("shared", [False, True])
def test_decode_step_in_a_hip_graph_matches_eager_replay_by_replay(shared):
    # the benchmark replays decode steps from HIP graphs: a captured step, replayed with fresh
    # inputs copied into its static buffers, must leave the same state and output as the same step
    # launched eagerly on a twin layer (both layouts)
    w = WORKLOADS["cfg1"].scaled(batch=2, context=700, budget=256, decode_steps=8)
    if shared:
        w = w.shared()
    twins = [(LockStepShared if shared else LockStep)(w) for _ in range(2)]
    for ls in twins:
        if shared:
            ls.event(0, w.context, w.budget, "prefill")
        else:
            ls.event(0, w.context, w.budget, "prefill", check=False)
        im.im_set_max_live(ls.handle, w.budget + 1)
    g_ls, e_ls = twins
    dev = "cuda"
    k_s = torch.empty((w.batch, w.n_kv_heads, 1, 128), dtype=torch.bfloat16, device=dev)
    v_s = torch.empty_like(k_s)
    q_s = torch.empty((w.batch, w.n_q_heads, 128), dtype=torch.bfloat16, device=dev)
    x_s = torch.empty((w.batch, w.gate_in_dim), dtype=torch.bfloat16, device=dev)
    p_s = torch.empty((w.batch,), dtype=torch.int32, device=dev)

    def load(t):
        k_s.copy_(g_ls.K[:, :, t:t + 1]); v_s.copy_(g_ls.V[:, :, t:t + 1]); q_s.copy_(g_ls.Q[:, t])
        x_s.copy_(g_ls.X[:, t] if shared else g_ls.Q[:, t].reshape(w.batch, -1))
        p_s.fill_(t)

    def step(ls):
        ls.gpu.decode_step(k_s, v_s, p_s, q_s, x_s, p_s, w.budget, w.lam, w.eta, debug=True)

    load(w.context)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):   # capture records the launches; nothing runs yet
        step(g_ls)
    for t in range(w.context, w.context + 6):
        load(t)
        graph.replay()
        step(e_ls)
        torch.cuda.synchronize()
        for n in ("len", "pos", "K", "V", "Kidx", "M", "b"):
            assert torch.equal(getattr(g_ls.gpu.st, n), getattr(e_ls.gpu.st, n)), f"replay@{t}: {n} differs"
        assert torch.equal(g_ls.gpu.out, e_ls.gpu.out), f"replay@{t}: output differs"
        assert torch.equal(g_ls.gpu.evicted, e_ls.gpu.evicted), f"replay@{t}: evicted slot differs"
        # eager work between the replays, as in a real program
        _ = (g_ls.gpu.st.M.sum() + e_ls.gpu.st.M.sum()).item()
    assert im.im_query_status(g_ls.handle) == 0 and im.im_query_status(e_ls.handle) == 0


@pytest.mark.parametrize("name,kw", [
    ("cfg1", dict()),                                                        # 1024 -> 256, 16 decode steps
    ("cfg2", dict(batch=2, context=1100, budget=300, decode_steps=3)),
    ("cfg3", dict(batch=2, context=1500, budget=333, decode_steps=3)),
    ("cfg4", dict(batch=3, context=1300, budget=130, decode_steps=3)),       # 4 KV heads of 7 query heads, 7 indexer heads
    ("cfg5", dict(batch=1, context=1536, budget=512, decode_steps=3, prefill_chunk=512)),
    ("cfg1", dict(context=40, budget=64, decode_steps=30)),                  # grows to the budget, then evicts
    ("cfg1", dict(batch=3, context=300, budget=64, decode_steps=3, n_recent=8)),
])
def test_head_shared_layout(name, kw):
    # the layer-wide form of the paper's text (Section 3.1: one indexer key per token from the hidden
    # state; Algorithm 1 mem_write: rows summed across heads into one memory per layer; d_index 16)
    LockStepShared(WORKLOADS[name].shared(n_layers=1, **kw)).run_schedule()


@pytest.mark.parametrize("name,kw", [
    ("cfg1", dict()),
    ("cfg2", dict(batch=2, context=1100, budget=300, decode_steps=4)),
    ("cfg3", dict(batch=2, context=1500, budget=333, decode_steps=4)),
    ("cfg4", dict(batch=3, context=1300, budget=130, decode_steps=4)),       # 4 KV heads of 7 query heads
    ("cfg4", dict(batch=2, context=700, budget=128, decode_steps=3)),        # n = 129: one key beyond the splits
    ("cfg4", dict(batch=1, context=1500, budget=1200, decode_steps=3)),      # 10 splits
    ("cfg5", dict(batch=1, context=1536, budget=512, decode_steps=4, prefill_chunk=512)),
    ("cfg1", dict(context=40, budget=64, decode_steps=30)),                  # grows to the budget, then evicts
    ("cfg1", dict(batch=3, context=300, budget=64, decode_steps=3, n_recent=8)),   # recent window forced
    ("cfg1", dict(n_q_heads=64, context=500, budget=140, decode_steps=3)),   # 16 indexer heads, 8 per group
    ("cfg1", dict(n_q_heads=8, n_kv_heads=1, context=500, budget=140, decode_steps=3)),   # a single KV head
    ("cfg1", dict(batch=11, context=260, budget=4, decode_steps=3)),         # budget = the sinks alone
    ("cfg1", dict(batch=2, n_kv_heads=16, context=400, budget=150, decode_steps=3)),   # 16 KV heads: two rounds of row sums
    ("cfg1", dict(batch=64, n_kv_heads=2, n_q_heads=8, context=150, budget=40, decode_steps=2)),   # the largest batch
])
def test_head_shared_layout_fused_decode(name, kw):
    w = WORKLOADS[name].shared(n_layers=1, **kw)
    LockStepShared(w).run_schedule(fused_decode=True)


@pytest.mark.parametrize("name,kw,tau,n_win", [
    ("cfg1", dict(context=600, budget=200, decode_steps=96), 32, 3),
    ("cfg4", dict(batch=2, context=700, budget=130, decode_steps=128), 128, 1),      # the paper's tau
    ("cfg1", dict(batch=2, context=500, budget=200, decode_steps=114), 57, 2),       # live bound 257: one key beyond the splits
    ("cfg1", dict(batch=2, context=300, budget=100, decode_steps=15), 5, 3),         # 5 queries < 8 indexer heads: the few-query scoring kernel
])
@pytest.mark.parametrize("fused", [True, False])
def test_head_shared_layout_periodic_schedule(name, kw, tau, n_win, fused):
    w = WORKLOADS[name].shared(n_layers=1, **kw)
    LockStepShared(w, capacity=max(w.context, w.budget + tau)).run_window_schedule(tau, n_win, fused=fused)


def test_head_shared_layout_rejects_what_is_not_built_for_it():
    w = WORKLOADS["cfg1"].shared()
    ls = LockStepShared(w)
    g = ls.gpu
    d = lambda t: t.cuda()
    k = d(ls.K[:, :, :1].contiguous()); q = d(ls.Q[:, 0].contiguous()); pos = torch.zeros(w.batch, dtype=torch.int32).cuda()
    with pytest.raises(im.IndexMemError):
        im.im_attend_step(ls.handle, ls.params, g.st, q, k, k, pos, g.out)
    with pytest.raises(im.IndexMemError):
        im.im_decode_step_shared(ls.handle, ls.params, g.st, q, k, k, pos, pos, 0.9, 0.5, g.out)
    per_head = LockStep(WORKLOADS["cfg1"])
    with pytest.raises(im.IndexMemError):
        im.im_decode_step_shared_hidden(per_head.handle, per_head.params, per_head.gpu.st, q, q.view(1, -1), k, k, pos,
                                        pos, 0.9, 0.5, g.out)
    with pytest.raises(im.IndexMemError):
        im.im_append_kv(ls.handle, g.st, k, k, pos.view(-1, 1))


def test_pre_eviction_prompt_buffers_in_place_then_a_budget_sized_cache():
    # Section 3.1 ("pre-eviction": cache only the selected KV).  The prompt's K / V sit in buffers of
    # their own, as a model's projections leave them; a state of capacity L adopts them in place
    # (im_append_kv with no rows), the step runs on it, and only the kept entries are written
    # (im_gather_kept) to the cache that decoding uses, which holds budget + 2 entries.  The oracle
    # takes the ordinary path.  A destination too small for the kept set is refused and flagged.
    w = WORKLOADS["cfg3"].scaled(n_layers=1, batch=2, context=1500, budget=333, decode_steps=4)
    L = w.context
    ls = LockStep(w, capacity=w.budget + 2, ref_capacity=L, max_queries=L)
    big_h = im.Handle(im.Config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, capacity=L,
                                n_idx_heads=w.n_idx_heads, n_sink=w.n_sink, fold_block=w.fold_block, max_queries=L))
    big = im.Layer(big_h, ls.params)
    d = lambda t: t.cuda()
    big.st.K[:, :, :L] = d(ls.K[:, :, :L]); big.st.V[:, :, :L] = d(ls.V[:, :, :L])     # "written by the projections"
    pos = torch.arange(L, dtype=torch.int32).repeat(w.batch, 1).contiguous()
    q = d(ls.Q[:, :L].contiguous())
    im.im_append_kv(big_h, big.st, None, None, d(pos))
    # score -> select -> memory update on the adopted buffers, then ONE launch that writes the kept entries
    # (and the memory state) straight into the budget-sized cache; the prompt's buffers are only read
    im.im_index_score(big_h, ls.params, big.st, q, q.view(w.batch, L, -1), d(pos), big.scores)
    im.im_topb_select(big_h, big.scores, big.st, w.budget, big.keep_idx, big.evict_idx, big.n_keep, big.n_evict)
    im.im_memory_update(big_h, ls.params, big.st, big.evict_idx, big.n_evict, w.lam, w.eta)
    snap = {k: getattr(big.st, k).clone() for k in ("K", "V", "pos", "len")}
    small = ls.gpu.st
    im.im_gather_kept(big_h, big.st, small, w.budget + 2, big.keep_idx, big.n_keep, big.evict_idx, big.n_evict)
    torch.cuda.synchronize()
    assert im.im_query_status(big_h) == 0
    n = w.budget
    assert (big.st.len == L).all() and all(torch.equal(getattr(big.st, k), v) for k, v in snap.items())
    assert (small.len == n).all() and (small.n_projected == n).all()
    # the oracle's ordinary prefill event; everything the cache holds must match it
    f = lambda t: t.to(torch.float64).numpy()
    qn = f(ls.Q[:, :L])
    ls.ref.append_kv(f(ls.K[:, :, :L]), f(ls.V[:, :, :L]), pos.numpy())
    scores = ls.ref.index_score(qn, qn.reshape(w.batch, L, -1), pos.numpy())
    keep, evict = ls.ref.topb_select(scores, w.budget)
    ls.ref.memory_update(evict, w.lam, w.eta)
    ls.ref.compact_kv(keep, evict)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            assert np.array_equal(big.keep_idx[b, h, :n].cpu().numpy(), keep[b][h])
            assert np.array_equal(big.evict_idx[b, h, :L - n].cpu().numpy(), evict[b][h])
    ls.compare(None, None, None, None, None, "adopted cache", lists=False, outputs=False)
    for b in range(w.batch):   # the indexer keys travelled along (compare() skips them without lists)
        for h in range(w.n_kv_heads):
            assert np.array_equal(f(small.Kidx[b, h, :n].cpu()), ls.ref.Kidx[b, h, :n])
    im.im_set_max_live(ls.handle, w.budget + 1)
    for t in range(L, L + w.decode_steps):
        ls.event_fused(t, w.budget, f"fused decode@{t}")
    assert im.im_query_status(ls.handle) == 0
    # a destination with fewer slots than the kept set: nothing is written, the status word says so
    tiny = im.State(im.Config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, capacity=w.budget - 1,
                              n_idx_heads=w.n_idx_heads))
    im.im_gather_kept(big_h, big.st, tiny, w.budget - 1, big.keep_idx, big.n_keep, big.evict_idx, big.n_evict)
    torch.cuda.synchronize()
    assert im.im_query_status(big_h) == im.IM_STATUS_APPEND_OVERFLOW
    assert not tiny.K.any() and not tiny.len.any() and not tiny.M.any()


@pytest.mark.parametrize("shared", [False, True])
def test_fused_decode_from_an_empty_cache(shared):
    # no prompt at all: the cache grows one token per step through the fused entry point, reaches the
    # budget and starts evicting (sinks included in the budget)
    w = WORKLOADS["cfg1"].scaled(batch=2, context=0, budget=9, decode_steps=24)
    if shared:
        w = w.shared()
    ls = (LockStepShared(w, capacity=16) if shared else LockStep(w, capacity=16, max_queries=1))
    im.im_set_max_live(ls.handle, w.budget + 1)
    for t in range(w.decode_steps):
        ls.event_fused(t, w.budget, f"fused decode@{t}")
    assert im.im_query_status(ls.handle) == 0


def _random_shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        n_kv = int(rng.choice([1, 2, 4, 8]))
        g = int(rng.choice([1, 2, 3, 4, 5, 7, 8]))
        n_q = n_kv * g
        if n_q % 4 or n_q // 4 > 16:        # H_index = H / 4 must be an integer in 1..16
            continue
        context = int(rng.integers(5, 700))
        budget = int(rng.integers(4, max(6, context)))
        n_recent = int(rng.choice([0, 0, 3]))
        if budget < 4 + n_recent:
            budget = 4 + n_recent
        out.append(dict(batch=int(rng.integers(1, 6)), n_kv_heads=n_kv, n_q_heads=n_q, context=context,
                        budget=budget, decode_steps=int(rng.integers(2, 6)), n_recent=n_recent))
    return out


@pytest.mark.parametrize("kw", _random_shapes(20260525, 14), ids=lambda kw: "-".join(str(v) for v in kw.values()))
@pytest.mark.parametrize("shared", [False, True])
def test_seeded_random_shapes_fused_decode(kw, shared):
    # shapes drawn from a fixed seed: head counts, ragged contexts and budgets, recent windows
    w = WORKLOADS["cfg1"].scaled(n_layers=1, **kw)
    if shared:
        LockStepShared(w.shared(), capacity=max(w.capacity, w.budget + 2)).run_schedule(fused_decode=True)
    else:
        LockStep(w, capacity=max(w.capacity, w.budget + 2)).run_schedule(fused_decode=True)


@pytest.mark.parametrize("kw", _random_shapes(7, 9), ids=lambda kw: "-".join(str(v) for v in kw.values()))
@pytest.mark.parametrize("shared", [False, True])
def test_seeded_random_shapes_periodic_schedule(kw, shared):
    # the two-launch attend-only step and the compression event on the same kind of shapes
    tau = 3 + kw["decode_steps"] * 7
    w = WORKLOADS["cfg1"].scaled(n_layers=1, **{**kw, "decode_steps": 2 * tau})
    if w.context == 0 or w.budget < 4 + w.n_recent:
        pytest.skip("degenerate draw")
    cap = max(w.context, w.budget + tau)
    if shared:
        LockStepShared(w.shared(), capacity=cap).run_window_schedule(tau, 2)
    else:
        LockStep(w, capacity=cap, max_queries=max(w.context, tau)).run_window_schedule(tau, 2)


def test_few_queries_score_a_cache_with_many_rows_not_yet_projected():
    # 300 rows are appended without a scoring call in between, then ONE query scores the cache: the
    # decode-size scoring call has to project all of them (its projection workgroups walk over the unit's
    # tiles), bit for bit as the prefill-size call would, and the scores follow the oracle's
    w = WORKLOADS["cfg1"].scaled(batch=2, context=371, budget=400, decode_steps=1, n_layers=1)
    ls = LockStep(w, capacity=400)
    g, ref, dev = ls.gpu, ls.ref, "cuda"
    n0 = 70
    ls.event(0, n0, w.budget, "first rows")                       # 70 rows, projected by a 70-query call
    t1 = w.context
    k = ls.K[:, :, n0:t1].contiguous(); v = ls.V[:, :, n0:t1].contiguous()
    pos = torch.arange(n0, t1, dtype=torch.int32).repeat(w.batch, 1).contiguous()
    im.im_append_kv(ls.handle, g.st, k.to(dev), v.to(dev), pos.to(dev))
    ref.append_kv(f64(k), f64(v), pos.numpy())
    q = ls.Q[:, t1 - 1:t1].contiguous()
    qpos = torch.full((w.batch, 1), t1 - 1, dtype=torch.int32)
    qd = q.to(dev)
    im.im_index_score(ls.handle, ls.params, g.st, qd, qd.view(w.batch, 1, -1), qpos.to(dev), g.scores)
    torch.cuda.synchronize()
    want = ref.index_score(f64(q), f64(q).reshape(w.batch, 1, -1), qpos.numpy())
    assert (g.st.n_projected == t1).all()
    assert np.array_equal(f64(g.st.Kidx[:, :, :t1]), ref.Kidx[:, :, :t1])
    assert np.array_equal(g.scores[:, :, :t1].cpu().numpy().astype(np.float64), want[:, :, :t1])
    assert im.im_query_status(ls.handle) == 0
