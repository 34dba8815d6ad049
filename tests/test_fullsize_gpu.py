"""Parity at the configurations' stated sizes, in the launch configuration the benchmark times.
The GPU runs every unit of one layer; the oracle follows a sample of units (they are independent)
through the same events, and every observable of those units is compared to the usual bars.
Configurations 2-5 run their own trajectories (stated context, budget, batch and all 256 / 512 /
256 / 1024 decode steps through im_decode_step; configuration 5 after its 31 chunk evictions).  The
other decode paths of the benchmark run at configuration 3's size as well: the periodic schedule
(128 attend-only steps, then one compression event), a leader / follower pair of an index-sharing
group, the six separate calls at decode size, and the head-shared layout (step by step, and its fused
step over 512 decode steps)."""
import pytest

from parity import LockStep, LockStepShared
from workloads import WORKLOADS

pytestmark = pytest.mark.gpu


# The configurations' own trajectories: the stated context, budget, batch AND number of decode steps,
# every step through im_decode_step in the launch configuration the benchmark times.  The oracle
# follows the sampled units in lock step; the decision (evicted slot, length) is compared at every
# step, every observable (fp32 scores, rows, positions, M, b, output, readout) at every 32nd step and
# at the last one.  Same bars as everywhere else.
@pytest.mark.parametrize("name,layer,kw,units", [
    ("cfg2", 0, dict(decode_steps=256), dict(batch_ids=[0, 5], kv_heads=[1, 6])),
    ("cfg3", 0, dict(decode_steps=512), dict(batch_ids=[1, 3], kv_heads=[2, 5])),
    # configuration 4's launch configuration: batch 16 x 4 KV heads (projection blocks of 8 batch rows, the
    # per-unit tail: 64 units x 7 heads do not fit the chip once)
    ("cfg4", 0, dict(decode_steps=256), dict(batch_ids=[11], kv_heads=[1, 2])),
    # ... and its head shape at a reduced batch (the per-(unit, head) tail), on a layer other than the first
    ("cfg4", 5, dict(decode_steps=256, batch=4), dict(batch_ids=[2], kv_heads=[0, 3])),
    # 31 chunk evictions of 4096 out of 8192 live entries, then decode at 4097 live entries
    ("cfg5", 0, dict(decode_steps=1024), dict(kv_heads=[3])),
], ids=["cfg2-256-steps", "cfg3-512-steps", "cfg4-256-steps", "cfg4-batch4-layer5-256-steps", "cfg5-1024-steps"])
def test_full_size_trajectory_sampled_units(name, layer, kw, units):
    w = WORKLOADS[name].scaled(n_layers=layer + 1, **kw)
    ls = LockStep(w, layer=layer, gen_device="cuda", **units)
    ls.run_schedule(fused_decode=True, full_every=32)


@pytest.mark.parametrize("name,units", [
    ("cfg3", dict(batch_ids=[0, 2], kv_heads=[3, 6])),
    ("cfg4", dict(batch_ids=[7], kv_heads=[0, 3])),
], ids=["cfg3", "cfg4"])
def test_full_size_step_by_step_decode_sampled_units(name, units):
    # the six separate calls at the benchmark's sizes (bench.py --path steps): after the prompt's event, 8
    # decode steps of one new token and one eviction each, through the decode-size paths of the generic
    # kernels (single-eviction selection, few-row projection and memory update, matrix-core attention
    # partials with 4 and 7 query heads per KV head)
    w = WORKLOADS[name].scaled(n_layers=1, decode_steps=8)
    LockStep(w, gen_device="cuda", **units).run_schedule()


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


def test_cfg3_head_shared_full_size_sampled_sequence():
    # configuration 3's cache shape in the head-shared layout: one 16384-query scoring pass over 16384
    # keys of 16 dims per sequence, one eviction set per sequence, rows of 8 KV heads summed into one memory
    w = WORKLOADS["cfg3"].shared(n_layers=1, decode_steps=3)
    LockStepShared(w, gen_device="cuda", batch_ids=[2]).run_schedule()


def test_cfg3_head_shared_full_size_fused_decode():
    # configuration 3's own 512 decode steps through the four-launch step of this layout
    w = WORKLOADS["cfg3"].shared(n_layers=1, decode_steps=512)
    LockStepShared(w, gen_device="cuda", batch_ids=[1]).run_schedule(fused_decode=True, full_every=32)
