"""CPU oracle for the bounded-budget KV step of IndexMem.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy implementation of what the hot path computes, written from the
paper's definitions: the indexer score (Section 3.1 "Architecture"; Algorithm 1, `indexer`),
the score -> TopK -> Gather eviction framework (Section 2.2), the latent-memory write and
read (Section 3.2, Eqs. latent_write_A / latent_write_b / latent_readout; Algorithm 1,
`mem_write` / `mem_read`) and decode attention with the gated residual (Section 2.1
"KV Caching"; Eq. latent_residual_fuse).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It shares no code with the HIP path and never imports it.  Nothing here is blocked, fused
or tuned: one numpy expression per equation, python loops over units and over queries.

Precision: every input is a bf16 value held exactly in fp64; all arithmetic is fp64.  The
roundings the method's *stored* quantities undergo are explicit and happen exactly once:
indexer keys are stored in bf16, query features / head gates / scores in fp32, the attention
output in bf16, the memory state in fp32 (rounded only when compared).

Every function below is pinned by tests/test_oracle_pins.py against closed forms, invariants,
brute force, scalar loops and library routines (read_gate and fuse on random inputs with gates
strictly inside (0, 1); a layer that follows a subset of KV heads against the same heads of a
full layer; a batch of sequences with different positions against layers of one sequence each);
none is "parity unpinned".  The paper prints no worked numeric example, so there
are no golden values of the paper's to compare with.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------------------
# roundings
# --------------------------------------------------------------------------------------
def round_bf16(x) -> np.ndarray:
    """Nearest bf16 value of each fp64 element (round-to-nearest-even, ONE rounding),
    returned as fp64.  Picks between the two bf16 neighbours by exact fp64 distance, so
    there is no double rounding through fp32."""
    x = np.atleast_1d(np.asarray(x, dtype=F64))
    f = x.astype(np.float32)                      # only used to find the bracketing bf16 pair
    bits = f.view(np.uint32)
    lo_bits = bits & np.uint32(0xFFFF0000)        # bf16 neighbour toward zero
    hi_bits = lo_bits + np.uint32(0x00010000)     # bf16 neighbour away from zero
    lo = lo_bits.view(np.float32).astype(F64)
    hi = hi_bits.view(np.float32).astype(F64)
    d_lo = np.abs(x - lo)
    d_hi = np.abs(hi - x)
    lo_is_odd = ((lo_bits >> np.uint32(16)) & np.uint32(1)) == 1
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & lo_is_odd)
    return np.where(pick_hi, hi, lo)


def round_f32(x) -> np.ndarray:
    """Nearest fp32 value (round-to-nearest-even), returned as fp64."""
    return np.asarray(x, dtype=F64).astype(np.float32).astype(F64)


# --------------------------------------------------------------------------------------
# step a1: indexer  (Section 3.1 "Architecture"; Algorithm 1 `indexer`)
# --------------------------------------------------------------------------------------
def rms_norm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm over the last axis: x / sqrt(mean(x^2) + eps) * w."""
    r = np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x / r * w


def key_feature(K_rows: np.ndarray, Uk: np.ndarray, norm_k_w: np.ndarray, rms_eps: float) -> np.ndarray:
    """Indexer key of each cached key row: k = Norm(U_k K_t), stored in bf16.
    K_rows [n, D], Uk [d_idx, D] -> [n, d_idx].  One shared key per token (MQA-style)."""
    u = K_rows @ Uk.T
    return round_bf16(rms_norm(u, norm_k_w, rms_eps))


def query_feature(Q_flat: np.ndarray, Uq: np.ndarray, norm_q_w: np.ndarray,
                  n_idx_heads: int, idx_dim: int, rms_eps: float) -> np.ndarray:
    """Indexer queries: q_s = U_q flatten(Q_s), viewed as [H_idx, d_idx], RMSNorm per head.
    Q_flat [n_q, H*D], Uq [H_idx*d_idx, H*D] -> [n_q, H_idx, d_idx], kept in fp32."""
    y = (Q_flat @ Uq.T).reshape(Q_flat.shape[0], n_idx_heads, idx_dim)
    return round_f32(rms_norm(y, norm_q_w, rms_eps))


def head_gate(X: np.ndarray, G: np.ndarray, n_idx_heads: int, idx_dim: int) -> np.ndarray:
    """Head-gating vector alpha_s = G X_s / sqrt(H_idx d_idx).  X [n_q, gate_in], G [H_idx, gate_in]
    -> [n_q, H_idx], kept in fp32."""
    return round_f32((X @ G.T) / np.sqrt(F64(n_idx_heads * idx_dim)))


def importance(qhat: np.ndarray, alpha: np.ndarray, q_pos: np.ndarray,
               khat: np.ndarray, k_pos: np.ndarray) -> np.ndarray:
    """imp_t = max over queries s that may see key t (pos_t <= pos_s) of
    A_{s,t} = sum_h alpha_{s,h} * ReLU(q_{s,h} . k_t);  -inf where no query sees the key.
    qhat [n_q, H_idx, d_idx], alpha [n_q, H_idx], khat [n, d_idx] -> [n], kept in fp32."""
    n = khat.shape[0]
    imp = np.full(n, -np.inf, dtype=F64)
    for s in range(qhat.shape[0]):
        z = np.maximum(qhat[s] @ khat.T, 0.0)            # [H_idx, n]   act = ReLU
        A_s = alpha[s] @ z                               # [n]
        visible = k_pos <= q_pos[s]                      # causal mask by token position
        imp = np.where(visible, np.maximum(imp, A_s), imp)
    return round_f32(imp)


# --------------------------------------------------------------------------------------
# step a2: top-B selection  (Section 2.2; sinks: Section 4 "Models and Evaluation Setup")
# --------------------------------------------------------------------------------------
def select(scores: np.ndarray, pos: np.ndarray, budget: int, n_sink: int,
           n_recent: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Keep min(budget, n) entries: the forced ones (the first n_sink token positions and the
    n_recent newest positions) and then the largest scores; total order = score descending,
    then token position ascending (the older token wins a tie).
    Returns (keep, evict): slot indices, each ascending."""
    n = scores.shape[0]
    if n == 0:
        return np.zeros(0, np.int32), np.zeros(0, np.int32)
    forced = (pos < n_sink) | (pos > pos.max() - n_recent)
    s = np.where(forced, np.inf, scores)
    order = np.lexsort((pos, -s))                        # primary: -score, secondary: position
    n_keep = min(budget, n)
    keep = np.sort(order[:n_keep]).astype(np.int32)
    evict = np.sort(order[n_keep:]).astype(np.int32)
    return keep, evict


# --------------------------------------------------------------------------------------
# step a3: latent-memory write  (Eqs. latent_write_A, latent_write_b; Algorithm 1 `mem_write`)
# --------------------------------------------------------------------------------------
def memory_write(M: np.ndarray, b: np.ndarray, K_E: np.ndarray, V_E: np.ndarray,
                 Wtheta: np.ndarray, lam: float, eta: float) -> Tuple[np.ndarray, np.ndarray]:
    """M <- lam M + eta sum_i phi(k_i) v_i^T ;  b <- lam b + eta sum_i phi(k_i) * phi(k_i),
    phi = Linear_theta (no bias).  One call = one eviction event: the decay is applied once.
    An empty evicted set is not an event: the state is returned untouched."""
    if K_E.shape[0] == 0:
        return M, b
    Phi = K_E @ Wtheta.T                                  # [n_e, d_mem]
    M_new = lam * M + eta * (Phi.T @ V_E)                 # [d_mem, D]
    b_new = lam * b + eta * np.sum(Phi * Phi, axis=0)     # [d_mem]
    return M_new, b_new


# --------------------------------------------------------------------------------------
# step a4: compaction (the Gather of Section 2.2, done in place)
# --------------------------------------------------------------------------------------
def compaction_moves(keep: Sequence[int], evict: Sequence[int]) -> List[Tuple[int, int]]:
    """Hole filling: kept entries sitting in slots >= n_keep move, in ascending order, into the
    evicted slots < n_keep, in ascending order.  Returns (src, dst) pairs."""
    n_keep = len(keep)
    movers = [int(s) for s in keep if s >= n_keep]
    holes = [int(s) for s in evict if s < n_keep]
    assert len(movers) == len(holes)
    return list(zip(movers, holes))


# --------------------------------------------------------------------------------------
# step a5: decode attention + gated memory readout
# (Section 2.1 "KV Caching"; Eqs. latent_readout, latent_residual_fuse)
# --------------------------------------------------------------------------------------
def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """Softmax attention of g query heads over the retained entries of their KV head.
    q [g, D], K, V [n, D] -> [g, D].  Zero when nothing is retained."""
    if K.shape[0] == 0:
        return np.zeros_like(q)
    logits = scale * (q @ K.T)                            # [g, n]
    logits = logits - logits.max(axis=-1, keepdims=True)
    p = np.exp(logits)
    p = p / p.sum(axis=-1, keepdims=True)
    return p @ V


def memory_read(q: np.ndarray, M: np.ndarray, b: np.ndarray, Wtheta: np.ndarray,
                mem_eps: float) -> np.ndarray:
    """m(q) = phi(q)^T M / (phi(q)^{.2 T} b + eps).  q [g, D] -> [g, D]."""
    phi = q @ Wtheta.T                                    # [g, d_mem]
    den = (phi * phi) @ b + mem_eps                       # [g]
    return (phi @ M) / den[:, None]


def read_gate(q: np.ndarray, wg: np.ndarray, cg: float) -> np.ndarray:
    """g(q) = sigmoid(w_g . q + c_g), one value in [0, 1] per query head."""
    return 1.0 / (1.0 + np.exp(-(q @ wg + cg)))


def fuse(o_attn: np.ndarray, gate: np.ndarray, m: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """o = o_attn + g(q) m(q), stored in bf16; also returns the residual g(q) m(q) in fp32."""
    res = gate[:, None] * m
    return round_bf16(o_attn + res), round_f32(res)


# --------------------------------------------------------------------------------------
# parameter counts (Section 4 "Parameter and Efficiency Analysis")
# --------------------------------------------------------------------------------------
def param_count(n_heads: int, head_dim: int, d_model: int, n_idx_heads: int, idx_dim: int,
                mem_dim: int, n_layers: int) -> Tuple[int, int]:
    """(indexer parameters, memory parameters) of the module shapes used here:
    U_q [H_idx d_idx, H d_head], U_k [d_idx, d_model], G [H_idx, d_model]; Linear_theta
    [mem_dim, head_dim]."""
    indexer = n_idx_heads * idx_dim * n_heads * head_dim + idx_dim * d_model + n_idx_heads * d_model
    memory = mem_dim * head_dim
    return n_layers * indexer, n_layers * memory


# --------------------------------------------------------------------------------------
# one layer's state, laid out like the library's (slots, lengths), and the calls on it
# --------------------------------------------------------------------------------------
@dataclass
class OracleConfig:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    capacity: int
    n_idx_heads: int
    head_dim: int = 128
    idx_dim: int = 64
    mem_dim: int = 128
    n_sink: int = 4
    n_recent: int = 0
    rms_eps: float = 1e-6
    mem_eps: float = 1e-6
    softmax_scale: float = 1.0 / np.sqrt(128.0)
    # which global KV heads the state's head axis holds (a subset lets a test check a few units)
    kv_head_ids: Optional[Sequence[int]] = None

    def head_ids(self) -> List[int]:
        return list(range(self.n_kv_heads)) if self.kv_head_ids is None else list(self.kv_head_ids)


@dataclass
class OracleParams:
    Uq: np.ndarray
    G: np.ndarray
    Uk: np.ndarray
    norm_q_w: np.ndarray
    norm_k_w: np.ndarray
    Wtheta: np.ndarray
    wg: np.ndarray
    cg: float


class OracleLayer:
    """State of one attention layer: per (batch, KV head) unit a slot array of K, V, indexer
    keys and token positions, a live length, and the memory state (M, b), all zero / empty at
    start.  Methods mirror the library's calls and apply the per-unit functions above."""

    def __init__(self, cfg: OracleConfig, params: OracleParams):
        self.cfg, self.p = cfg, params
        B, Hs, C, D = cfg.batch, len(cfg.head_ids()), cfg.capacity, cfg.head_dim
        self.K = np.zeros((B, Hs, C, D), F64)
        self.V = np.zeros((B, Hs, C, D), F64)
        self.Kidx = np.zeros((B, Hs, C, cfg.idx_dim), F64)
        self.pos = np.zeros((B, Hs, C), np.int32)
        self.len = np.zeros((B, Hs), np.int32)
        self.n_projected = np.zeros((B, Hs), np.int32)
        self.M = np.zeros((B, Hs, cfg.mem_dim, D), F64)
        self.b = np.zeros((B, Hs, cfg.mem_dim), F64)

    def units(self):
        for bi in range(self.cfg.batch):
            for hi in range(len(self.cfg.head_ids())):
                yield bi, hi

    # helper: new tokens enter the cache
    def append_kv(self, k_new: np.ndarray, v_new: np.ndarray, pos_new: np.ndarray) -> None:
        """k_new, v_new [B, Hs, n_new, D]; pos_new [B, n_new]."""
        n_new = k_new.shape[2]
        for bi, hi in self.units():
            n = int(self.len[bi, hi])
            assert n + n_new <= self.cfg.capacity
            self.K[bi, hi, n:n + n_new] = k_new[bi, hi]
            self.V[bi, hi, n:n + n_new] = v_new[bi, hi]
            self.pos[bi, hi, n:n + n_new] = pos_new[bi]
            self.len[bi, hi] = n + n_new

    # a1
    def index_score(self, q_new: np.ndarray, x_gate: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
        """q_new [B, n_q, H, D]; x_gate [B, n_q, gate_in]; q_pos [B, n_q].
        Projects the keys not yet projected, then returns scores [B, Hs, C] (fp32 values;
        slots >= len are NaN here: the library leaves them untouched)."""
        cfg, p = self.cfg, self.p
        scores = np.full((cfg.batch, len(cfg.head_ids()), cfg.capacity), np.nan, F64)
        for bi in range(cfg.batch):
            n_q = q_new.shape[1]
            qhat = query_feature(q_new[bi].reshape(n_q, -1), p.Uq, p.norm_q_w,
                                 cfg.n_idx_heads, cfg.idx_dim, cfg.rms_eps)
            alpha = head_gate(x_gate[bi], p.G, cfg.n_idx_heads, cfg.idx_dim)
            for hi in range(len(cfg.head_ids())):
                n, n0 = int(self.len[bi, hi]), int(self.n_projected[bi, hi])
                if n > n0:
                    self.Kidx[bi, hi, n0:n] = key_feature(self.K[bi, hi, n0:n], p.Uk,
                                                         p.norm_k_w, cfg.rms_eps)
                    self.n_projected[bi, hi] = n
                scores[bi, hi, :n] = importance(qhat, alpha, q_pos[bi],
                                                self.Kidx[bi, hi, :n], self.pos[bi, hi, :n])
        return scores

    # a2
    def topb_select(self, scores: np.ndarray, budget: int):
        """Returns per-unit lists keep[b][h], evict[b][h] (ascending slot indices)."""
        cfg = self.cfg
        keep = [[None] * len(cfg.head_ids()) for _ in range(cfg.batch)]
        evict = [[None] * len(cfg.head_ids()) for _ in range(cfg.batch)]
        for bi, hi in self.units():
            n = int(self.len[bi, hi])
            keep[bi][hi], evict[bi][hi] = select(scores[bi, hi, :n], self.pos[bi, hi, :n],
                                                 budget, cfg.n_sink, cfg.n_recent)
        return keep, evict

    # a3
    def memory_update(self, evict, lam: float, eta: float) -> None:
        for bi, hi in self.units():
            e = evict[bi][hi]
            self.M[bi, hi], self.b[bi, hi] = memory_write(
                self.M[bi, hi], self.b[bi, hi], self.K[bi, hi, e], self.V[bi, hi, e],
                self.p.Wtheta, lam, eta)

    # a4
    def compact_kv(self, keep, evict) -> None:
        for bi, hi in self.units():
            for src, dst in compaction_moves(keep[bi][hi], evict[bi][hi]):
                self.K[bi, hi, dst] = self.K[bi, hi, src]
                self.V[bi, hi, dst] = self.V[bi, hi, src]
                self.Kidx[bi, hi, dst] = self.Kidx[bi, hi, src]
                self.pos[bi, hi, dst] = self.pos[bi, hi, src]
            self.len[bi, hi] = len(keep[bi][hi])
            self.n_projected[bi, hi] = len(keep[bi][hi])

    # a5
    def decode_attn_with_readout(self, q: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
        """q [B, H, D] -> (out [B, Hs, g, D] bf16 values, residual g(q) m(q) [B, Hs, g, D] fp32 values);
        the g query heads of global KV head h are heads h*g .. h*g+g-1."""
        cfg, p = self.cfg, self.p
        g = cfg.n_q_heads // cfg.n_kv_heads
        heads = cfg.head_ids()
        out = np.zeros((cfg.batch, len(heads), g, cfg.head_dim), F64)
        res = np.zeros_like(out)
        for bi, hi in self.units():
            h = heads[hi]
            qg = q[bi, h * g:(h + 1) * g]
            n = int(self.len[bi, hi])
            o_attn = attend(qg, self.K[bi, hi, :n], self.V[bi, hi, :n], cfg.softmax_scale)
            m = memory_read(qg, self.M[bi, hi], self.b[bi, hi], p.Wtheta, cfg.mem_eps)
            out[bi, hi], res[bi, hi] = fuse(o_attn, read_gate(qg, p.wg, p.cg), m)
        return out, res

    # one whole step of the path, in the canonical order
    def step(self, k_new, v_new, pos_new, q_new, x_gate, q_pos, q_attn, budget, lam, eta):
        """append -> score -> select -> memory update -> compact -> attention + readout.
        Returns (scores, keep, evict, out, residual)."""
        self.append_kv(k_new, v_new, pos_new)
        scores = self.index_score(q_new, x_gate, q_pos)
        keep, evict = self.topb_select(scores, budget)
        self.memory_update(evict, lam, eta)
        self.compact_kv(keep, evict)
        out, res = self.decode_attn_with_readout(q_attn)
        return scores, keep, evict, out, res


# --------------------------------------------------------------------------------------
# the layer-wide (head-shared) form of the paper's text
# --------------------------------------------------------------------------------------
class OracleLayerShared:
    """One attention layer in the form the paper's text and Algorithm 1 describe literally:

      * the indexer key of a token is made from its hidden state, k_t = Norm(U_k X_t), one key
        for all heads (Section 3.1 "Architecture"; Algorithm 1 `indexer`), with d_index =
        d_head / 8 (Section 4, hyper-parameters);
      * hence one importance per token and ONE eviction set per sequence: every KV head keeps
        the same tokens in the same slots;
      * one latent memory per layer shared by all heads (Section 3.2, "Slow and fast weights");
        a write sums the evicted rows across heads per token (Algorithm 1 `mem_write`) - here
        both the key row fed to Linear_theta and the value row, so the state stays
        [d_mem, d_head]; every query head reads the same state (Eq. latent_readout).

    State per sequence b: Kidx [C, d_index], pos [C], len, (M, b); per (b, KV head): K, V
    [C, D].  Built from the same per-equation functions as OracleLayer; `cfg.batch` counts the
    sequences followed, all KV heads are always followed (the write needs their sum)."""

    def __init__(self, cfg: OracleConfig, params: OracleParams):
        assert cfg.kv_head_ids is None
        self.cfg, self.p = cfg, params
        B, Hk, C, D = cfg.batch, cfg.n_kv_heads, cfg.capacity, cfg.head_dim
        self.K = np.zeros((B, Hk, C, D), F64)
        self.V = np.zeros((B, Hk, C, D), F64)
        self.Kidx = np.zeros((B, C, cfg.idx_dim), F64)
        self.pos = np.zeros((B, C), np.int32)
        self.len = np.zeros(B, np.int32)
        self.M = np.zeros((B, cfg.mem_dim, D), F64)
        self.b = np.zeros((B, cfg.mem_dim), F64)

    def append_kv_hidden(self, k_new, v_new, x_new, pos_new) -> None:
        """k_new, v_new [B, H_kv, n_new, D]; x_new [B, n_new, d_model]; pos_new [B, n_new]."""
        n_new = k_new.shape[2]
        for bi in range(self.cfg.batch):
            n = int(self.len[bi])
            assert n + n_new <= self.cfg.capacity
            self.K[bi, :, n:n + n_new] = k_new[bi]
            self.V[bi, :, n:n + n_new] = v_new[bi]
            self.Kidx[bi, n:n + n_new] = key_feature(x_new[bi], self.p.Uk, self.p.norm_k_w, self.cfg.rms_eps)
            self.pos[bi, n:n + n_new] = pos_new[bi]
            self.len[bi] = n + n_new

    def index_score(self, q_new, x_gate, q_pos) -> np.ndarray:
        """q_new [B, n_q, H, D]; x_gate [B, n_q, d_model] (the queries' hidden states); q_pos [B, n_q]
        -> scores [B, C] (NaN beyond len)."""
        cfg, p = self.cfg, self.p
        scores = np.full((cfg.batch, cfg.capacity), np.nan, F64)
        for bi in range(cfg.batch):
            n_q, n = q_new.shape[1], int(self.len[bi])
            qhat = query_feature(q_new[bi].reshape(n_q, -1), p.Uq, p.norm_q_w,
                                 cfg.n_idx_heads, cfg.idx_dim, cfg.rms_eps)
            alpha = head_gate(x_gate[bi], p.G, cfg.n_idx_heads, cfg.idx_dim)
            scores[bi, :n] = importance(qhat, alpha, q_pos[bi], self.Kidx[bi, :n], self.pos[bi, :n])
        return scores

    def topb_select(self, scores, budget: int):
        keep, evict = [], []
        for bi in range(self.cfg.batch):
            n = int(self.len[bi])
            k, e = select(scores[bi, :n], self.pos[bi, :n], budget, self.cfg.n_sink, self.cfg.n_recent)
            keep.append(k)
            evict.append(e)
        return keep, evict

    def memory_update(self, evict, lam: float, eta: float) -> None:
        for bi in range(self.cfg.batch):
            e = evict[bi]
            K_E = self.K[bi][:, e].sum(axis=0)            # rows summed across heads per token
            V_E = self.V[bi][:, e].sum(axis=0)
            self.M[bi], self.b[bi] = memory_write(self.M[bi], self.b[bi], K_E, V_E, self.p.Wtheta, lam, eta)

    def compact_kv(self, keep, evict) -> None:
        for bi in range(self.cfg.batch):
            for src, dst in compaction_moves(keep[bi], evict[bi]):
                self.K[bi, :, dst] = self.K[bi, :, src]
                self.V[bi, :, dst] = self.V[bi, :, src]
                self.Kidx[bi, dst] = self.Kidx[bi, src]
                self.pos[bi, dst] = self.pos[bi, src]
            self.len[bi] = len(keep[bi])

    def decode_attn_with_readout(self, q) -> Tuple[np.ndarray, np.ndarray]:
        """q [B, H, D] -> (out, residual), each [B, H_kv, g, D]."""
        cfg, p = self.cfg, self.p
        g = cfg.n_q_heads // cfg.n_kv_heads
        out = np.zeros((cfg.batch, cfg.n_kv_heads, g, cfg.head_dim), F64)
        res = np.zeros_like(out)
        for bi in range(cfg.batch):
            n = int(self.len[bi])
            for h in range(cfg.n_kv_heads):
                qg = q[bi, h * g:(h + 1) * g]
                o_attn = attend(qg, self.K[bi, h, :n], self.V[bi, h, :n], cfg.softmax_scale)
                m = memory_read(qg, self.M[bi], self.b[bi], p.Wtheta, cfg.mem_eps)
                out[bi, h], res[bi, h] = fuse(o_attn, read_gate(qg, p.wg, p.cg), m)
        return out, res

    def step(self, k_new, v_new, x_new, pos_new, q_new, x_gate, q_pos, q_attn, budget, lam, eta):
        """append -> score -> select -> memory update -> compact -> attention + readout."""
        self.append_kv_hidden(k_new, v_new, x_new, pos_new)
        scores = self.index_score(q_new, x_gate, q_pos)
        keep, evict = self.topb_select(scores, budget)
        self.memory_update(evict, lam, eta)
        self.compact_kv(keep, evict)
        out, res = self.decode_attn_with_readout(q_attn)
        return scores, keep, evict, out, res
