"""Parity at the benchmark's full size and launch configuration: configuration 3 (batch 4, 8 KV
heads, a 16384-token prompt evicted to 2048, then decode through im_decode_step with the live
bound the benchmark sets).  The GPU runs every unit of one layer; the oracle follows a sample of
units (they are independent) through the same events and every observable of those units is
compared to the usual bars.  Configuration 4's head shape (7 query heads per KV head, 7 indexer
heads) gets the same treatment at a reduced batch; configuration 2 (batch 8, 4096 -> 1024) and
configuration 5 (one sequence of 131072 tokens in 32 chunks of 4096, running cache evicted to
4096 after every chunk) run one layer at their stated sizes; configuration 4 also at its own batch
of 16.  The other decode paths of the benchmark run at configuration 3's size as well: the periodic
schedule (128 attend-only steps, then one compression event) and a leader / follower pair of an
index-sharing group."""
import pytest

from parity import LockStep, LockStepShared
from workloads import WORKLOADS

pytestmark = pytest.mark.gpu


def test_cfg3_full_size_sampled_units():
    w = WORKLOADS["cfg3"].scaled(n_layers=1, decode_steps=6)
    ls = LockStep(w, gen_device="cuda", batch_ids=[1, 3], kv_heads=[2, 5])
    ls.run_schedule(fused_decode=True)


def test_cfg4_shape_full_context_sampled_units():
    w = WORKLOADS["cfg4"].scaled(n_layers=1, batch=4, decode_steps=4)
    ls = LockStep(w, gen_device="cuda", batch_ids=[2], kv_heads=[0, 3])
    ls.run_schedule(fused_decode=True)


def test_cfg4_full_batch_sampled_units():
    # the benchmark's own launch configuration of configuration 4: batch 16 x 4 KV heads (projection blocks
    # of 8 batch rows, the per-unit tail: 64 units x 7 heads do not fit the chip once)
    w = WORKLOADS["cfg4"].scaled(n_layers=1, decode_steps=3)
    ls = LockStep(w, gen_device="cuda", batch_ids=[11], kv_heads=[1, 2])
    ls.run_schedule(fused_decode=True)


def test_cfg3_full_size_periodic_schedule_sampled_units():
    # the paper's decode schedule at the benchmark's size: 128 attend-only steps (two launches each, 2049 ..
    # 2176 live entries), then one compression event with the interval's 128 queries
    w = WORKLOADS["cfg3"].scaled(n_layers=1, decode_steps=128)
    ls = LockStep(w, gen_device="cuda", batch_ids=[2], kv_heads=[0, 7], capacity=w.context,
                  max_queries=w.context)
    ls.run_window_schedule(128, 1, fused=True)


def test_cfg3_full_size_index_reuse_sampled_units():
    # two layers of an index-sharing group at the benchmark's size: layer 1 applies layer 0's lists at the
    # prefill event and layer 0's evicted slot at every decode step (its two-launch follower step)
    import paper_2605_25475_amd as im
    w = WORKLOADS["cfg3"].scaled(n_layers=2, decode_steps=4)
    kw = dict(gen_device="cuda", batch_ids=[0], kv_heads=[4, 6])
    lead, foll = LockStep(w, layer=0, **kw), LockStep(w, layer=1, **kw)
    _, _, evict, _, _ = lead.event(0, w.context, w.budget, "leader prefill")
    foll.follow_event(0, w.context, lead, evict, "follower prefill")
    for ls in (lead, foll):
        im.im_set_max_live(ls.handle, w.budget + 1)
    for t in range(w.context, w.context + w.decode_steps):
        _, _, evict, _, _ = lead.event_fused(t, w.budget, f"leader decode@{t}")
        foll.follow_step(t, lead, evict, f"follower decode@{t}")
    assert im.im_query_status(lead.handle) == 0 and im.im_query_status(foll.handle) == 0


def test_cfg2_full_size_sampled_units():
    w = WORKLOADS["cfg2"].scaled(n_layers=1, decode_steps=6)
    ls = LockStep(w, gen_device="cuda", batch_ids=[0, 5], kv_heads=[1, 6])
    ls.run_schedule(fused_decode=True)


def test_cfg5_full_size_chunked_prefill_sampled_unit():
    # 31 chunk evictions of 4096 out of 8192 live entries, then decode at 4097 live entries
    w = WORKLOADS["cfg5"].scaled(n_layers=1, decode_steps=4)
    ls = LockStep(w, gen_device="cuda", kv_heads=[3])
    ls.run_schedule(fused_decode=True)


def test_cfg3_head_shared_full_size_sampled_sequence():
    # configuration 3's cache shape in the head-shared layout: one 16384-query scoring pass over 16384
    # keys of 16 dims per sequence, one eviction set per sequence, rows of 8 KV heads summed into one memory
    w = WORKLOADS["cfg3"].shared(n_layers=1, decode_steps=3)
    LockStepShared(w, gen_device="cuda", batch_ids=[2]).run_schedule()


def test_cfg3_head_shared_full_size_fused_decode():
    w = WORKLOADS["cfg3"].shared(n_layers=1, decode_steps=5)
    LockStepShared(w, gen_device="cuda", batch_ids=[1]).run_schedule(fused_decode=True)
