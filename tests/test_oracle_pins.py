"""Pins of the CPU oracle: each test checks an oracle function against something the paper or
the mathematics fixes and that is computed here WITHOUT the oracle's own formula: library
routines (torch SDPA, torch Linear / RMS statistics, torch bf16 conversion), closed forms,
brute force and invariants.  The paper prints no worked numeric example; the parameter counts of Section 4 are
the only printed numbers that touch this path: they are kept in tests/golden/ with their
citation and pinned in test_parameter_counts."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import indexmem_oracle as O
from workloads import WORKLOADS, hidden_stream, layer_params, token_stream
from helpers import f64, make_oracle_layer, oracle_params

RNG = np.random.default_rng(1234)


def bf(x):
    """numpy fp64 -> bf16-representable fp64 via torch (library conversion from fp32)."""
    return torch.tensor(np.asarray(x, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


# ----------------------------------------------------------------------------- roundings
def test_round_bf16_matches_torch_on_fp32_inputs():
    x = np.concatenate([RNG.standard_normal(20000) * 10.0 ** RNG.integers(-6, 6, 20000),
                        [0.0, -0.0, 1.0, -1.0, 3.0e-40, 1.0e-45]]).astype(np.float32)
    want = torch.tensor(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_bf16(x.astype(np.float64))
    assert np.array_equal(got, want)


def test_round_bf16_is_a_single_rounding():
    # 1 + 2^-8 is the midpoint of the bf16 neighbours 1 and 1 + 2^-7.  A value just below the
    # midpoint, but so close that fp32 rounds it onto the midpoint, must still go DOWN.
    mid = 1.0 + 2.0 ** -8
    below = mid - 2.0 ** -40
    above = mid + 2.0 ** -40
    assert np.float32(below) == np.float32(mid)          # the double-rounding trap is armed
    assert O.round_bf16(below)[0] == 1.0
    assert O.round_bf16(above)[0] == 1.0 + 2.0 ** -7
    assert O.round_bf16(mid)[0] == 1.0                   # tie -> even mantissa
    mid_odd = 1.0 + 2.0 ** -7 + 2.0 ** -8                # tie whose lower neighbour is odd
    assert O.round_bf16(mid_odd)[0] == 1.0 + 2.0 ** -6
    assert O.round_bf16(-below)[0] == -1.0


# ----------------------------------------------------------------------------- P4 shapes
def test_parameter_counts():
    # Section 4 "Parameter and Efficiency Analysis": 19.92 M indexer and 0.52 M memory
    # parameters on Llama-3.1-8B (32 layers, H=32, d_head=128, d_model=4096) with the paper's
    # H_idx = H/4 and d_idx = d_head/8.
    golden = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "parameter_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                golden[k] = float(v)
    idx, mem = O.param_count(n_heads=32, head_dim=128, d_model=4096, n_idx_heads=8, idx_dim=16,
                             mem_dim=128, n_layers=32)
    assert idx == 19_922_944 and round(idx / 1e6, 2) == golden["indexer_millions"]
    assert mem == 524_288 and round(mem / 1e6, 2) == golden["memory_millions"]
    # the head-shared layout's weights at configuration 3's shape are exactly these modules: the
    # generated tensors add up to the printed counts
    w = WORKLOADS["cfg3"].shared()
    p = layer_params(w, 0)
    per_layer_idx = p["Uq"].numel() + p["Uk"].numel() + p["G"].numel()
    assert per_layer_idx * w.n_layers == idx and p["Wtheta"].numel() * w.n_layers == mem
    assert tuple(p["Uk"].shape) == (16, 4096) and tuple(p["Uq"].shape) == (8 * 16, 4096)


# ----------------------------------------------------------------------------- a1 indexer
def test_key_feature_against_torch_linear_and_rms():
    K = bf(RNG.standard_normal((37, 128)))
    Uk = bf(RNG.standard_normal((64, 128)) * 0.02)
    w = bf(1.0 + 0.1 * RNG.standard_normal(64))
    got = O.key_feature(K, Uk, w, 1e-6)
    u = torch.nn.functional.linear(torch.tensor(K), torch.tensor(Uk))       # [out,in] weight
    want = torch.nn.functional.rms_norm(u, (64,), torch.tensor(w), eps=1e-6)
    assert got.shape == (37, 64)
    assert np.allclose(got, want.numpy(), rtol=2 ** -8, atol=0)             # bf16 rounding only
    assert np.array_equal(got, bf(got))                                     # stored as bf16


def test_query_feature_and_gate_against_torch():
    H, D, Hi, di, nq = 8, 128, 2, 64, 5
    Q = bf(RNG.standard_normal((nq, H * D)))
    Uq = bf(RNG.standard_normal((Hi * di, H * D)) * 0.02)
    G = bf(RNG.standard_normal((Hi, H * D)) * 0.02)
    w = bf(1.0 + 0.1 * RNG.standard_normal(di))
    got = O.query_feature(Q, Uq, w, Hi, di, 1e-6)
    y = torch.nn.functional.linear(torch.tensor(Q), torch.tensor(Uq)).view(nq, Hi, di)
    want = torch.nn.functional.rms_norm(y, (di,), torch.tensor(w), eps=1e-6).numpy()
    assert np.allclose(got, want, rtol=1e-6, atol=0)
    assert np.array_equal(got, got.astype(np.float32).astype(np.float64))
    a = O.head_gate(Q, G, Hi, di)
    want_a = (torch.tensor(Q) @ torch.tensor(G).T).numpy() / math.sqrt(Hi * di)
    assert np.allclose(a, want_a, rtol=1e-6, atol=0)


def _rand_indexer(nq, n, Hi=8, di=64):
    qhat = RNG.standard_normal((nq, Hi, di)).astype(np.float32).astype(np.float64)
    alpha = (RNG.standard_normal((nq, Hi)) * 0.1).astype(np.float32).astype(np.float64)
    khat = bf(RNG.standard_normal((n, di)))
    return qhat, alpha, khat


def test_importance_against_explicit_loops():
    # the definition, as scalar loops over query, key, head and feature
    nq, n, Hi, di = 4, 9, 3, 8
    qhat, alpha, khat = _rand_indexer(nq, n, Hi, di)
    q_pos = np.array([3, 5, 7, 20]); k_pos = np.array([0, 1, 2, 4, 6, 8, 9, 21, 20])
    want = np.full(n, -np.inf)
    for t in range(n):
        for s in range(nq):
            if k_pos[t] > q_pos[s]:
                continue
            a = 0.0
            for h in range(Hi):
                z = sum(qhat[s, h, c] * khat[t, c] for c in range(di))
                a += alpha[s, h] * max(z, 0.0)
            want[t] = max(want[t], a)
    got = O.importance(qhat, alpha, q_pos, khat, k_pos)
    assert np.isneginf(got[7]) and np.isfinite(got[8])      # key newer than every query
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin)
    assert np.allclose(got[fin], want[fin], rtol=1e-6, atol=1e-9)


def test_importance_single_head_is_relu_cosine():
    # H_idx = 1, alpha = 1, unit norm weights: score = ReLU(d_idx * cos(q, k)) up to rms_eps
    di, n = 64, 50
    yq = RNG.standard_normal((1, 1, di)); ku = RNG.standard_normal((n, di))
    qhat = O.rms_norm(yq, np.ones(di), 0.0)
    khat = O.rms_norm(ku, np.ones(di), 0.0)
    got = O.importance(qhat, np.ones((1, 1)), np.array([10 ** 6]), khat, np.arange(n))
    cos = (ku @ yq[0, 0]) / (np.linalg.norm(ku, axis=1) * np.linalg.norm(yq))
    assert np.allclose(got, np.maximum(di * cos, 0.0), rtol=1e-6, atol=1e-6)


def test_importance_invariants():
    nq, n = 6, 40
    qhat, alpha, khat = _rand_indexer(nq, n)
    q_pos = np.arange(100, 100 + nq); k_pos = np.arange(n)
    imp = O.importance(qhat, alpha, q_pos, khat, k_pos)
    # max-decomposition over a split of the query set
    a = O.importance(qhat[:2], alpha[:2], q_pos[:2], khat, k_pos)
    b = O.importance(qhat[2:], alpha[2:], q_pos[2:], khat, k_pos)
    assert np.array_equal(imp, np.maximum(a, b))
    # bound: |q_h . k| <= |q_h| |k|  =>  |imp| <= max_s sum_h |alpha_sh| |q_sh| |k_t|
    bound = np.max(np.sum(np.abs(alpha)[:, :, None] * np.linalg.norm(qhat, axis=2)[:, :, None]
                          * np.linalg.norm(khat, axis=1)[None, None, :], axis=1), axis=0)
    assert np.all(np.abs(imp) <= bound * (1 + 1e-6))
    # one query: linear in the gate
    one = O.importance(qhat[:1], alpha[:1], q_pos[:1], khat, k_pos)
    two = O.importance(qhat[:1], 2 * alpha[:1], q_pos[:1], khat, k_pos)
    assert np.allclose(two, 2 * one, rtol=1e-6)
    # zero gate -> every visible score is 0
    z = O.importance(qhat, 0 * alpha, q_pos, khat, k_pos)
    assert np.all(z == 0.0)


def test_key_feature_scale_invariance():
    # RMSNorm removes the key's scale, so a planted high-norm key keeps its indexer key
    K = bf(RNG.standard_normal((20, 128)))
    Uk = bf(RNG.standard_normal((64, 128)) * 0.02)
    one = np.ones(64)
    a = O.key_feature(K, Uk, one, 1e-12)
    b = O.key_feature(4.0 * K, Uk, one, 1e-12)
    assert np.max(np.abs(a - b)) <= 2 ** -7 * np.max(np.abs(a))   # at most one bf16 ulp
    assert np.mean(a != b) < 0.01


# ----------------------------------------------------------------------------- a2 selection
def _brute_select(scores, pos, budget, n_sink, n_recent):
    n = len(scores)
    mx = max(pos) if n else 0
    s = [math.inf if (pos[t] < n_sink or pos[t] > mx - n_recent) else scores[t] for t in range(n)]
    keep, evict = [], []
    for t in range(n):
        rank = sum(1 for u in range(n) if s[u] > s[t] or (s[u] == s[t] and pos[u] < pos[t]))
        (keep if rank < budget else evict).append(t)
    return keep, evict


@pytest.mark.parametrize("kind", ["random", "quantised", "all_equal", "infs"])
def test_select_against_brute_force(kind):
    for n in [0, 1, 3, 7, 16, 33]:
        for trial in range(3):
            pos = RNG.permutation(n + 5)[:n]
            if kind == "random":
                sc = RNG.standard_normal(n)
            elif kind == "quantised":
                sc = RNG.integers(0, 3, n).astype(np.float64)
            elif kind == "all_equal":
                sc = np.zeros(n)
            else:
                sc = RNG.choice([-np.inf, np.inf, 0.0, 1.0], n)
            sc = sc.astype(np.float32).astype(np.float64)
            for n_recent in (0, 2):
                for budget in range(4 + n_recent, n + 2):
                    keep, evict = O.select(sc, pos, budget, 4, n_recent)
                    bk, be = _brute_select(list(sc), list(pos), budget, 4, n_recent)
                    assert list(keep) == bk and list(evict) == be


def test_select_invariants_and_ties():
    n, B = 500, 100
    pos = np.arange(n)
    sc = RNG.integers(0, 8, n).astype(np.float64)
    keep, evict = O.select(sc, pos, B, 4)
    assert len(keep) == B and len(evict) == n - B
    assert sorted(set(keep) | set(evict)) == list(range(n)) and not set(keep) & set(evict)
    assert all(t in set(keep) for t in range(4))                       # sinks kept
    nonforced = [t for t in keep if pos[t] >= 4]
    worst_kept = min((sc[t], -pos[t]) for t in nonforced)
    best_evicted = max((sc[t], -pos[t]) for t in evict)
    assert worst_kept > best_evicted
    # all scores equal -> the B oldest positions survive
    keep0, _ = O.select(np.zeros(n), pos[::-1].copy(), B, 4)
    assert sorted(pos[::-1][keep0]) == list(range(B))
    # -0.0 and +0.0 are the same score
    sz = np.where(RNG.integers(0, 2, n) == 0, 0.0, -0.0)
    keepz, _ = O.select(sz, pos, B, 4)
    assert list(keepz) == list(range(B))


# ----------------------------------------------------------------------------- a3 memory write
def test_memory_write_against_outer_product_loop():
    ne = 7
    K = bf(RNG.standard_normal((ne, 128))); V = bf(RNG.standard_normal((ne, 128)))
    W = bf(RNG.standard_normal((128, 128)) * 0.02)
    M0 = RNG.standard_normal((128, 128)); b0 = np.abs(RNG.standard_normal(128))
    lam, eta = 0.9, 0.5
    M, b = O.memory_write(M0, b0, K, V, W, lam, eta)
    Mw, bw = lam * M0, lam * b0
    for i in range(ne):
        phi = torch.nn.functional.linear(torch.tensor(K[i]), torch.tensor(W)).numpy()
        Mw = Mw + eta * np.outer(phi, V[i])
        bw = bw + eta * phi ** 2
    assert np.allclose(M, Mw, rtol=1e-12, atol=1e-14) and np.allclose(b, bw, rtol=1e-12, atol=1e-14)


def test_memory_write_chunks_are_order_independent_and_sum_to_batch_update():
    ne = 200
    K = bf(RNG.standard_normal((ne, 128))); V = bf(RNG.standard_normal((ne, 128)))
    W = bf(RNG.standard_normal((128, 128)) * 0.02)
    M0 = RNG.standard_normal((128, 128)); b0 = np.abs(RNG.standard_normal(128))
    # lam = 1: any partition into blocks, in any order, equals the one-shot update
    M1, b1 = O.memory_write(M0, b0, K, V, W, 1.0, 0.5)
    perm = RNG.permutation(ne)
    M2, b2 = M0, b0
    for blk in np.array_split(perm, 7):
        M2, b2 = O.memory_write(M2, b2, K[blk], V[blk], W, 1.0, 0.5)
    assert np.allclose(M1, M2, rtol=1e-12, atol=1e-13) and np.allclose(b1, b2, rtol=1e-12, atol=1e-13)
    # lam < 1 is applied once per event: event(lam, E1) then event(1, E2) == event(lam, E1 u E2)
    Ma, ba = O.memory_write(M0, b0, K, V, W, 0.9, 0.5)
    Mb, bb = O.memory_write(M0, b0, K[:64], V[:64], W, 0.9, 0.5)
    Mb, bb = O.memory_write(Mb, bb, K[64:], V[64:], W, 1.0, 0.5)
    assert np.allclose(Ma, Mb, rtol=1e-12, atol=1e-13) and np.allclose(ba, bb, rtol=1e-12, atol=1e-13)
    # nothing evicted is not an event: no decay
    Mn, bn = O.memory_write(M0, b0, K[:0], V[:0], W, 0.5, 0.5)
    assert Mn is M0 and bn is b0


# ----------------------------------------------------------------------------- a5 readout
def test_associative_recall_closed_form():
    # W_theta = I, one evicted token k = e_j with value v, lam = 1:
    # M = eta e_j v^T, b = eta e_j, so reading with q = k returns v (eps -> 0)
    I = np.eye(128); j = 17
    k = np.zeros((1, 128)); k[0, j] = 1.0
    v = bf(RNG.standard_normal((1, 128)))
    M, b = O.memory_write(np.zeros((128, 128)), np.zeros(128), k, v, I, 1.0, 0.5)
    m = O.memory_read(k, M, b, I, 1e-30)
    assert np.allclose(m[0], v[0], rtol=1e-12)
    # a transposed state would return v_j e_j instead
    assert not np.allclose(O.memory_read(k, M.T, b, I, 1e-30)[0], v[0])


def test_single_token_readout_closed_form_and_eta_invariance():
    W = bf(RNG.standard_normal((128, 128)) * 0.1)
    k = bf(RNG.standard_normal((1, 128))); v = bf(RNG.standard_normal((1, 128)))
    q = bf(RNG.standard_normal((3, 128)))
    fk = np.array([sum(W[c, d] * k[0, d] for d in range(128)) for c in range(128)])
    for eta in (0.5, 3.0):
        M, b = O.memory_write(np.zeros((128, 128)), np.zeros(128), k, v, W, 0.7, eta)
        m = O.memory_read(q, M, b, W, 0.0)
        for r in range(3):
            fq = np.array([sum(W[c, d] * q[r, d] for d in range(128)) for c in range(128)])
            want = (fq @ fk) * v[0] / np.sum(fq ** 2 * fk ** 2)
            assert np.allclose(m[r], want, rtol=1e-10)


def test_empty_memory_reads_zero_and_closed_gate_falls_back_to_attention():
    q = bf(RNG.standard_normal((4, 128)))
    W = bf(RNG.standard_normal((128, 128)) * 0.02)
    m = O.memory_read(q, np.zeros((128, 128)), np.zeros(128), W, 1e-6)
    assert np.all(m == 0.0)
    g = O.read_gate(q, bf(RNG.standard_normal(128) * 0.02), -1e4)
    assert np.all(g == 0.0)
    o = RNG.standard_normal((4, 128))
    out, res = O.fuse(o, g, RNG.standard_normal((4, 128)))
    assert np.array_equal(out, O.round_bf16(o)) and np.all(res == 0.0)
    g1 = O.read_gate(q, np.zeros(128), 0.0)
    assert np.all(g1 == 0.5)


@pytest.mark.parametrize("cg", [0.0, 1.5, -1.5])
def test_read_gate_is_the_logistic_of_the_weighted_query(cg):
    # g(q) in [0, 1] (Section 3.2, "Readout as residual compensation"): sigmoid(w_g . q + c_g), one
    # value per query head.  Weights large enough that the w_g . q term moves the gate far from 0.5.
    q = bf(RNG.standard_normal((5, 128)))
    wg = bf(RNG.standard_normal(128) * 0.15)
    got = O.read_gate(q, wg, cg)
    assert got.shape == (5,)
    for r in range(5):   # scalar loop, term by term
        z = cg
        for d in range(128):
            z += wg[d] * q[r, d]
        assert abs(got[r] - 1.0 / (1.0 + math.exp(-z))) <= 1e-14
    want = torch.sigmoid(torch.nn.functional.linear(torch.tensor(q), torch.tensor(wg)[None]) + cg)[:, 0].numpy()
    assert np.allclose(got, want, rtol=0, atol=1e-14)
    assert np.ptp(got) > 0.2                       # the heads' gates differ: the query term is at work
    # reflecting the query reflects the gate around the bias' own value
    assert np.allclose(got + O.read_gate(-q, wg, -cg), 1.0, atol=1e-14)


@pytest.mark.parametrize("gval", [0.25, 1.0])
def test_fuse_adds_the_gated_readout_once_and_rounds_once(gval):
    # Eq. latent_residual_fuse: o = o_attn + g(q) m(q), per element; stored in bf16, the residual in fp32
    o = RNG.standard_normal((3, 128)); m = RNG.standard_normal((3, 128)) * 0.3
    gate = np.array([gval, gval * 0.5, gval])
    out, res = O.fuse(o, gate, m)
    for r in range(3):
        for d in range(128):
            exact = o[r, d] + gate[r] * m[r, d]
            assert out[r, d] == bf(out[r, d])[()]                                 # a bf16 value ...
            assert abs(out[r, d] - exact) <= 2.0 ** -8 * abs(exact) + 1e-300     # ... half an ulp from the sum at most
            assert res[r, d] == float(np.float32(gate[r] * m[r, d]))
    # linear in the gate: twice the gate doubles the residual (a squared gate would quadruple it)
    _, res2 = O.fuse(o, 2.0 * gate, m)
    assert np.allclose(res2, 2.0 * res, rtol=1e-6)
    # the bf16 result is the rounding of the exact sum, not of separately rounded terms
    want = torch.tensor(o + gate[:, None] * m, dtype=torch.float64).to(torch.float32)
    exact_in_f32 = want.to(torch.float64).numpy() == (o + gate[:, None] * m)
    assert np.array_equal(out[exact_in_f32], want.to(torch.bfloat16).to(torch.float64).numpy()[exact_in_f32])


def test_layer_on_a_subset_of_kv_heads_reproduces_those_heads_of_the_full_layer():
    # the full-size GPU tests let the oracle follow a few KV heads (kv_head_ids): local index hi then stands
    # for global head heads[hi], whose g query heads are heads[hi] g .. heads[hi] g + g - 1
    w, K, V, Q = _small_layer(context=72, budget=24, steps=3)
    heads = [2, 5]
    full = make_oracle_layer(w)
    sub = make_oracle_layer(w, kv_head_ids=heads)
    L = w.context

    def both(t0, t1):
        pos = np.tile(np.arange(t0, t1, dtype=np.int32), (w.batch, 1))
        q = Q[:, t0:t1]
        xg = q.reshape(w.batch, t1 - t0, -1)
        rf = full.step(K[:, :, t0:t1], V[:, :, t0:t1], pos, q, xg, pos, Q[:, t1 - 1], w.budget, w.lam, w.eta)
        rs = sub.step(K[:, heads, t0:t1], V[:, heads, t0:t1], pos, q, xg, pos, Q[:, t1 - 1], w.budget, w.lam, w.eta)
        return rf, rs

    for t0, t1 in [(0, L)] + [(t, t + 1) for t in range(L, L + w.decode_steps)]:
        (sf, kf, ef, of, rf), (ss, ks, es, os_, rs) = both(t0, t1)
        for hi, h in enumerate(heads):
            for bi in range(w.batch):
                assert np.array_equal(sf[bi, h], ss[bi, hi], equal_nan=True)
                assert np.array_equal(kf[bi][h], ks[bi][hi]) and np.array_equal(ef[bi][h], es[bi][hi])
                assert np.array_equal(of[bi, h], os_[bi, hi]) and np.array_equal(rf[bi, h], rs[bi, hi])
                assert np.array_equal(full.M[bi, h], sub.M[bi, hi]) and np.array_equal(full.b[bi, h], sub.b[bi, hi])
                assert np.array_equal(full.K[bi, h], sub.K[bi, hi]) and np.array_equal(full.pos[bi, h], sub.pos[bi, hi])
    # the heads' outputs differ from one another, so a mix-up of local and global index would show
    assert not np.array_equal(of[0, 2], of[0, 0]) and np.max(np.abs(rf[0, 2] - rf[0, 0])) > 0


# ----------------------------------------------------------------------------- a5 attention
@pytest.mark.parametrize("n", [1, 5, 300])
def test_attend_equals_library_softmax_attention(n):
    g, D = 4, 128
    q = bf(RNG.standard_normal((g, D))); K = bf(RNG.standard_normal((n, D))); V = bf(RNG.standard_normal((n, D)))
    scale = 1 / math.sqrt(D)
    got = O.attend(q, K, V, scale)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None], torch.tensor(K)[None], torch.tensor(V)[None], scale=scale)[0].numpy()
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)
    perm = RNG.permutation(n)
    assert np.allclose(O.attend(q, K[perm], V[perm], scale), got, rtol=1e-12, atol=1e-14)
    assert np.all(O.attend(q, K[:0], V[:0], scale) == 0)


# ----------------------------------------------------------------------------- a4 compaction
def test_compaction_moves_fill_holes():
    for n, B in [(10, 4), (33, 32), (64, 1), (20, 20), (7, 0)]:
        for _ in range(20):
            keep = np.sort(RNG.permutation(n)[:B]); evict = np.setdiff1d(np.arange(n), keep)
            slots = list(range(n))
            moves = O.compaction_moves(keep, evict)
            assert all(s >= B > d for s, d in moves)
            assert [s for s, _ in moves] == sorted(s for s, _ in moves)
            assert [d for _, d in moves] == sorted(d for _, d in moves)
            for s, d in moves:
                slots[d] = slots[s]
            assert sorted(slots[:B]) == list(keep)


# ----------------------------------------------------------------------------- whole layer
def _small_layer(context=96, budget=32, steps=3, name="cfg1", batch=None):
    w = WORKLOADS[name].scaled(context=context, budget=budget, decode_steps=steps,
                               batch=WORKLOADS[name].batch if batch is None else batch)
    K, V, Q = token_stream(w, 0)
    return w, f64(K), f64(V), f64(Q)


def _prefill(layer, w, K, V, Q, budget, lam=None, eta=None):
    L = w.context
    pos = np.tile(np.arange(L, dtype=np.int32), (w.batch, 1))
    q = Q[:, :L]
    return layer.step(K[:, :, :L], V[:, :, :L], pos, q, q.reshape(w.batch, L, -1), pos,
                      Q[:, L - 1], budget, w.lam if lam is None else lam, w.eta if eta is None else eta)


def test_budget_at_least_context_is_plain_attention_and_leaves_memory_untouched():
    w, K, V, Q = _small_layer()
    layer = make_oracle_layer(w)
    scores, keep, evict, out, res = _prefill(layer, w, K, V, Q, budget=w.context + 5)
    assert all(len(e) == 0 for row in evict for e in row)
    assert np.all(layer.M == 0) and np.all(layer.b == 0) and np.all(res == 0)
    assert np.all(layer.len == w.context)
    L, g = w.context, w.group
    qh = torch.tensor(Q[:, L - 1]).view(w.batch, w.n_kv_heads, g, w.head_dim)
    want = torch.nn.functional.scaled_dot_product_attention(
        qh, torch.tensor(K[:, :, :L]), torch.tensor(V[:, :, :L]), scale=1 / math.sqrt(w.head_dim)).numpy()
    assert np.array_equal(out, O.round_bf16(want).reshape(out.shape)) or \
        np.max(np.abs(out - want)) <= 2 ** -8 * np.max(np.abs(want))


def test_trajectory_indices_do_not_depend_on_values_or_memory():
    w, K, V, Q = _small_layer(context=80, budget=24, steps=4)
    L = w.context

    def run(Vx, eta):
        layer = make_oracle_layer(w)
        traj = []
        _, keep, evict, _, _ = _prefill(layer, w, K, Vx, Q, w.budget, eta=eta)
        traj.append((keep, evict))
        for t in range(L, L + w.decode_steps):
            p = np.full((w.batch, 1), t, np.int32)
            q = Q[:, t:t + 1]
            _, keep, evict, _, _ = layer.step(K[:, :, t:t + 1], Vx[:, :, t:t + 1], p, q,
                                              q.reshape(w.batch, 1, -1), p, Q[:, t], w.budget, w.lam, eta)
            traj.append((keep, evict))
        return traj, layer

    t1, l1 = run(V, 0.5)
    t2, l2 = run(V[:, :, ::-1].copy(), 2.0)
    for (k1, e1), (k2, e2) in zip(t1, t2):
        for bi, hi in l1.units():
            assert np.array_equal(k1[bi][hi], k2[bi][hi]) and np.array_equal(e1[bi][hi], e2[bi][hi])
    assert np.all(l1.len == w.budget)
    # decode steps evict exactly one entry and the compacted cache holds exactly the kept set
    for (k, e) in t1[1:]:
        assert all(len(x) == 1 for row in e for x in row)
    for bi, hi in l1.units():
        assert len(set(l1.pos[bi, hi, :w.budget].tolist())) == w.budget
        assert set(range(4)) <= set(l1.pos[bi, hi, :w.budget].tolist())


def test_compacted_cache_is_the_kept_multiset():
    w, K, V, Q = _small_layer(context=70, budget=20, steps=0)
    layer = make_oracle_layer(w)
    ref = make_oracle_layer(w)
    L = w.context
    pos = np.tile(np.arange(L, dtype=np.int32), (w.batch, 1))
    ref.append_kv(K[:, :, :L], V[:, :, :L], pos)
    q = Q[:, :L]
    ref.index_score(q, q.reshape(w.batch, L, -1), pos)
    _, keep, evict, _, _ = _prefill(layer, w, K, V, Q, w.budget)
    for bi, hi in layer.units():
        kept = keep[bi][hi]
        got = {int(layer.pos[bi, hi, s]): (layer.K[bi, hi, s].tobytes(), layer.V[bi, hi, s].tobytes(),
                                           layer.Kidx[bi, hi, s].tobytes()) for s in range(w.budget)}
        want = {int(ref.pos[bi, hi, s]): (ref.K[bi, hi, s].tobytes(), ref.V[bi, hi, s].tobytes(),
                                          ref.Kidx[bi, hi, s].tobytes()) for s in kept}
        assert got == want


def test_planted_high_norm_keys_change_attention_but_not_selection():
    w = WORKLOADS["cfg2"].scaled(context=128, budget=32, decode_steps=0, batch=1, n_layers=1)
    K, V, Q = (f64(t) for t in token_stream(w, 0))
    w_plain = w.scaled(dist="normal")
    K0, _, _ = (f64(t) for t in token_stream(w_plain, 0))
    ratio = np.linalg.norm(K, axis=-1) / np.linalg.norm(K0, axis=-1)
    assert int(np.sum(ratio[0, 0] > 3.9)) == int(0.05 * 128)             # exactly floor(5% of L) planted
    la, lb = make_oracle_layer(w), make_oracle_layer(w)
    _, ka, _, oa, _ = _prefill(la, w, K, V, Q, w.budget)
    _, kb, _, ob, _ = _prefill(lb, w, K0, V, Q, w.budget)
    same = np.mean([len(set(ka[0][h]) & set(kb[0][h])) / w.budget for h in range(w.n_kv_heads)])
    assert same > 0.95                                                   # up to bf16 ties in the indexer keys
    assert np.max(np.abs(oa - ob)) > 1e-2


# --------------------------------------------------------------------------------------------
# the head-shared layout (OracleLayerShared)
# --------------------------------------------------------------------------------------------
def _shared_inputs(context=60, budget=18, steps=3, batch=2, **kw):
    w = WORKLOADS["cfg1"].shared(context=context, budget=budget, decode_steps=steps, batch=batch, **kw)
    K, V, Q = (f64(t) for t in token_stream(w, 0))
    X = f64(hidden_stream(w, 0))
    return w, K, V, Q, X


def _shared_event(layer, w, K, V, Q, X, t0, t1, budget, lam=None, eta=None):
    pos = np.tile(np.arange(t0, t1, dtype=np.int32), (w.batch, 1))
    return layer.step(K[:, :, t0:t1], V[:, :, t0:t1], X[:, t0:t1], pos, Q[:, t0:t1], X[:, t0:t1], pos,
                      Q[:, t1 - 1], budget, w.lam if lam is None else lam, w.eta if eta is None else eta)


def test_shared_layout_with_one_kv_head_fed_its_key_rows_is_the_per_head_layout():
    # one KV head, d_model = d_head, hidden state := the key row, same d_index: nothing is left to
    # share, so every observable must equal the (separately pinned) per-head layer's
    w = WORKLOADS["cfg1"].scaled(n_q_heads=4, n_kv_heads=1, batch=2, context=50, budget=14, decode_steps=3)
    K, V, Q = (f64(t) for t in token_stream(w, 0))
    p = oracle_params(layer_params(w, 0))
    rng = np.random.default_rng(5)
    p.G = O.round_bf16(rng.normal(size=(w.n_idx_heads, w.head_dim)) * 0.02).reshape(w.n_idx_heads, w.head_dim)
    from helpers import oracle_config
    a, b = O.OracleLayer(oracle_config(w), p), O.OracleLayerShared(oracle_config(w), p)
    for t0, t1 in [(0, w.context)] + [(t, t + 1) for t in range(w.context, w.n_tokens)]:
        pos = np.tile(np.arange(t0, t1, dtype=np.int32), (w.batch, 1))
        x = K[:, 0, t0:t1]
        ra = a.step(K[:, :, t0:t1], V[:, :, t0:t1], pos, Q[:, t0:t1], x, pos, Q[:, t1 - 1], w.budget, w.lam, w.eta)
        rb = b.step(K[:, :, t0:t1], V[:, :, t0:t1], x, pos, Q[:, t0:t1], x, pos, Q[:, t1 - 1], w.budget, w.lam, w.eta)
        assert np.array_equal(ra[0][:, 0], rb[0], equal_nan=True)
        for bi in range(w.batch):
            assert np.array_equal(ra[1][bi][0], rb[1][bi]) and np.array_equal(ra[2][bi][0], rb[2][bi])
        assert np.array_equal(ra[3], rb[3]) and np.array_equal(ra[4], rb[4])
        assert np.array_equal(a.M[:, 0], b.M) and np.array_equal(a.b[:, 0], b.b)
        assert np.array_equal(a.K, b.K) and np.array_equal(a.Kidx[:, 0], b.Kidx) and np.array_equal(a.pos[:, 0], b.pos)


def test_shared_memory_write_is_the_double_sum_over_heads():
    # M = eta sum_i Linear_theta(sum_h k_{h,i}) (sum_h' v_{h',i})^T, expanded by bilinearity into
    # explicit loops over tokens and head pairs (Algorithm 1 `mem_write`, rows summed across heads)
    w, K, V, Q, X = _shared_inputs(context=40, budget=30, steps=0, batch=1)
    layer = make_oracle_layer(w)
    _, keep, evict, _, _ = _shared_event(layer, w, K, V, Q, X, 0, w.context, w.budget)
    e = evict[0]
    assert len(e) == 10
    W = f64(layer_params(w, 0)["Wtheta"])
    M = np.zeros((w.mem_dim, w.head_dim)); bvec = np.zeros(w.mem_dim)
    ref = make_oracle_layer(w)
    pos = np.arange(w.context, dtype=np.int32)[None]
    ref.append_kv_hidden(K[:, :, :w.context], V[:, :, :w.context], X[:, :w.context], pos)
    for i in e:
        phi = np.zeros(w.mem_dim)
        for h in range(w.n_kv_heads):
            phi += W @ ref.K[0, h, i]
        for h in range(w.n_kv_heads):
            M += w.eta * np.outer(phi, ref.V[0, h, i])
        bvec += w.eta * phi * phi
    assert np.allclose(layer.M[0], M, rtol=1e-12, atol=1e-12) and np.allclose(layer.b[0], bvec, rtol=1e-12, atol=1e-12)


def test_shared_layout_keeps_the_same_tokens_in_the_same_slots_of_every_head():
    w, K, V, Q, X = _shared_inputs()
    # tag every row with (head, token) so that a row's origin can be read back after the moves
    for h in range(w.n_kv_heads):
        K[:, h, :, 0] = np.arange(K.shape[2]) + 1000 * h
        V[:, h, :, 1] = np.arange(V.shape[2]) + 1000 * h
    layer = make_oracle_layer(w)
    _shared_event(layer, w, K, V, Q, X, 0, w.context, w.budget)
    for t in range(w.context, w.n_tokens):
        _, keep, evict, _, _ = _shared_event(layer, w, K, V, Q, X, t, t + 1, w.budget)
        assert all(len(e) == 1 for e in evict)
    for bi in range(w.batch):
        n = int(layer.len[bi])
        assert n == w.budget and set(range(4)) <= set(layer.pos[bi, :n].tolist())
        for h in range(w.n_kv_heads):
            assert np.array_equal(layer.K[bi, h, :n, 0], layer.pos[bi, :n] + 1000 * h)
            assert np.array_equal(layer.V[bi, h, :n, 1], layer.pos[bi, :n] + 1000 * h)
        # the indexer key travels with its token: it is the key of the hidden state at that position
        want = O.key_feature(X[bi, layer.pos[bi, :n]], f64(layer_params(w, 0)["Uk"]),
                             f64(layer_params(w, 0)["norm_k_w"]), float(np.float32(1e-6)))
        assert np.array_equal(layer.Kidx[bi, :n], want)


def test_shared_scores_against_explicit_loops():
    w, K, V, Q, X = _shared_inputs(context=24, budget=24, steps=0, batch=1)
    layer = make_oracle_layer(w)
    scores, *_ = _shared_event(layer, w, K, V, Q, X, 0, w.context, w.budget)
    p = layer_params(w, 0)
    Uq, G, Uk = f64(p["Uq"]), f64(p["G"]), f64(p["Uk"])
    Hi, di, eps = w.n_idx_heads, w.idx_dim, float(np.float32(1e-6))
    assert di == 16 and Uk.shape == (16, w.gate_in_dim)
    for t in range(w.context):
        kt = Uk @ X[0, t]
        kt = O.round_bf16(kt / math.sqrt(sum(v * v for v in kt) / di + eps))
        best = -math.inf
        for s in range(t, w.context):                       # causal: queries at or after the key
            y = (Uq @ Q[0, s].reshape(-1)).reshape(Hi, di)
            a = 0.0
            for j in range(Hi):
                qj = O.round_f32(y[j] / math.sqrt(sum(v * v for v in y[j]) / di + eps))
                al = float(O.round_f32(G[j] @ X[0, s] / math.sqrt(Hi * di)))
                a += al * max(0.0, float(qj @ kt))
            best = max(best, a)
        assert abs(float(O.round_f32(best)) - scores[0, t]) <= 1e-12 * max(1.0, abs(best))


@pytest.mark.parametrize("shared", [False, True], ids=["per-unit", "head-shared"])
def test_sequences_of_a_batch_are_independent_and_keep_their_own_positions(shared):
    # Batch elements share nothing but the weights: a layer of 3 sequences whose token positions differ
    # (offsets 0, 7 and 900: only the first sequence holds sink positions, and the causal mask and the
    # position tie-break see different numbers in each) must give, for every sequence, exactly what a
    # layer of that one sequence gives.  Pins every per-sequence index of the layer classes (positions,
    # query positions, gate inputs, hidden states, queries).
    kw = dict(batch=3, context=40, budget=16, decode_steps=3, n_recent=2)
    w = WORKLOADS["cfg1"].shared(**kw) if shared else WORKLOADS["cfg1"].scaled(**kw)
    K, V, Q = (f64(t) for t in token_stream(w, 0))
    X = f64(hidden_stream(w, 0)) if shared else None
    offs = np.array([0, 7, 900], np.int32)

    def run(layer, rows):
        outs = []
        for t0, t1 in [(0, w.context)] + [(t, t + 1) for t in range(w.context, w.n_tokens)]:
            pos = (np.arange(t0, t1, dtype=np.int32)[None] + offs[rows, None]).astype(np.int32)
            k, v, q = K[rows][:, :, t0:t1], V[rows][:, :, t0:t1], Q[rows][:, t0:t1]
            if shared:
                x = X[rows][:, t0:t1]
                outs.append(layer.step(k, v, x, pos, q, x, pos, Q[rows][:, t1 - 1], w.budget, w.lam, w.eta))
            else:
                xg = q.reshape(len(rows), t1 - t0, -1)
                outs.append(layer.step(k, v, pos, q, xg, pos, Q[rows][:, t1 - 1], w.budget, w.lam, w.eta))
        return outs

    full = make_oracle_layer(w)
    got = run(full, [0, 1, 2])
    decisions = []
    for bi in range(3):
        one = make_oracle_layer(w, batch=1)
        want = run(one, [bi])
        for g, r in zip(got, want):
            assert np.array_equal(g[0][bi], r[0][0], equal_nan=True)                 # scores
            flat = (lambda x: [x]) if shared else (lambda x: x)
            for a, b in zip(flat(g[1][bi]), flat(r[1][0])):
                assert np.array_equal(a, b)                                          # keep lists
            for a, b in zip(flat(g[2][bi]), flat(r[2][0])):
                assert np.array_equal(a, b)                                          # evict lists
            assert np.array_equal(g[3][bi], r[3][0]) and np.array_equal(g[4][bi], r[4][0])
        assert np.array_equal(full.M[bi], one.M[0]) and np.array_equal(full.b[bi], one.b[0])
        assert np.array_equal(full.pos[bi], one.pos[0]) and np.array_equal(full.K[bi], one.K[0])
        decisions.append(got[0][2][bi] if shared else got[0][2][bi][0])
    # the offsets matter: the sequence that holds the sink positions evicts a different set
    assert not np.array_equal(decisions[0], decisions[2])
