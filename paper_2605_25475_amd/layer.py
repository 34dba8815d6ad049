"""One attention layer's buffers and the canonical order of the library calls on them.

Pure sequencing: every method enqueues library calls on the current stream; nothing is
computed in Python."""
from __future__ import annotations

import torch

from . import binding as B


class Layer:
    def __init__(self, handle: B.Handle, params: B.Params, device="cuda"):
        cfg = handle.cfg
        self.h, self.p, self.cfg = handle, params, cfg
        self.st = B.State(cfg, device)
        Bz, Cc, S = cfg.batch, cfg.capacity, cfg.set_shape()
        self.scores = torch.empty(S + (Cc,), dtype=torch.float32, device=device)
        self.keep_idx = torch.empty(S + (Cc,), dtype=torch.int32, device=device)
        self.evict_idx = torch.empty(S + (Cc,), dtype=torch.int32, device=device)
        self.n_keep = torch.zeros(S, dtype=torch.int32, device=device)
        self.n_evict = torch.zeros(S, dtype=torch.int32, device=device)
        self.out = torch.empty((Bz, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device=device)
        self.readout = torch.empty((Bz, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device=device)
        self.evicted = torch.full(S, -1, dtype=torch.int32, device=device)

    def step(self, k_new, v_new, pos_new, q_new, x_gate, q_pos, q_attn, budget, lam, eta, x_new=None):
        """append -> score -> select -> memory update -> compact -> attention + readout.
        x_new: the new tokens' hidden states (head-shared layout only)."""
        h, p, st = self.h, self.p, self.st
        if self.cfg.head_shared:
            B.im_append_kv_hidden(h, p, st, k_new, v_new, x_new, pos_new)
        else:
            B.im_append_kv(h, st, k_new, v_new, pos_new)
        B.im_index_score(h, p, st, q_new, x_gate, q_pos, self.scores)
        B.im_topb_select(h, self.scores, st, budget, self.keep_idx, self.evict_idx, self.n_keep, self.n_evict)
        B.im_memory_update(h, p, st, self.evict_idx, self.n_evict, lam, eta)
        B.im_compact_kv(h, st, self.keep_idx, self.n_keep, self.evict_idx, self.n_evict)
        B.im_decode_attn_with_readout(h, p, st, q_attn, self.out, self.readout)
        return self.out

    def attend_step(self, k_new, v_new, pos_new, q_attn, fused=True, debug=True, x_new=None):
        """One token of the periodic schedule (Section 4, setup: compress every tau steps): append,
        then attention + readout over everything cached; nothing is scored or evicted.  fused: the
        three-launch entry point; else the two separate calls.  x_new [B, 1, d_model]: the token's
        hidden state (head-shared layout only)."""
        hs = self.cfg.head_shared
        if fused and hs:
            B.im_attend_step_hidden(self.h, self.p, self.st, q_attn, x_new.view(self.cfg.batch, -1), k_new, v_new,
                                    pos_new.view(-1), self.out, self.readout if debug else None)
        elif fused:
            B.im_attend_step(self.h, self.p, self.st, q_attn, k_new, v_new, pos_new.view(-1), self.out,
                             self.readout if debug else None)
        else:
            if hs:
                B.im_append_kv_hidden(self.h, self.p, self.st, k_new, v_new, x_new, pos_new)
            else:
                B.im_append_kv(self.h, self.st, k_new, v_new, pos_new)
            B.im_decode_attn_with_readout(self.h, self.p, self.st, q_attn, self.out, self.readout)
        return self.out

    def compress(self, q_win, x_gate_win, q_pos_win, budget, lam, eta):
        """The compression event of the periodic schedule: the queries of the interval score the
        cache, the cache is cut back to the budget, the evicted entries go to the memory."""
        h, p, st = self.h, self.p, self.st
        B.im_index_score(h, p, st, q_win, x_gate_win, q_pos_win, self.scores)
        B.im_topb_select(h, self.scores, st, budget, self.keep_idx, self.evict_idx, self.n_keep, self.n_evict)
        B.im_memory_update(h, p, st, self.evict_idx, self.n_evict, lam, eta)
        B.im_compact_kv(h, st, self.keep_idx, self.n_keep, self.evict_idx, self.n_evict)

    def follow_event(self, k_new, v_new, pos_new, q_attn, leader: "Layer", lam, eta, x_new=None):
        """An eviction event of a follower layer of an index-sharing group: the leader's keep / evict
        lists are applied to this layer's cache (same slot layout), nothing is scored here (a follower
        keeps no indexer keys of its own use: its Kidx rows are moved along but never read)."""
        h, p, st = self.h, self.p, self.st
        if self.cfg.head_shared:
            B.im_append_kv_hidden(h, p, st, k_new, v_new, x_new, pos_new)
        else:
            B.im_append_kv(h, st, k_new, v_new, pos_new)
        B.im_memory_update(h, p, st, leader.evict_idx, leader.n_evict, lam, eta)
        B.im_compact_kv(h, st, leader.keep_idx, leader.n_keep, leader.evict_idx, leader.n_evict)
        B.im_decode_attn_with_readout(h, p, st, q_attn, self.out, self.readout)
        return self.out

    def follow_step(self, k_new, v_new, pos_new, q, evict_slot, lam, eta, debug=False, x_new=None):
        """One decode token of a follower layer: the slot its leader evicted leaves here too."""
        if self.cfg.head_shared:
            B.im_decode_step_shared_hidden(self.h, self.p, self.st, q, x_new.view(self.cfg.batch, -1), k_new, v_new,
                                           pos_new, evict_slot, lam, eta, self.out, self.readout if debug else None)
        else:
            B.im_decode_step_shared(self.h, self.p, self.st, q, k_new, v_new, pos_new, evict_slot, lam, eta,
                                    self.out, self.readout if debug else None)
        return self.out

    def decode_step(self, k_new, v_new, pos_new, q, x_gate, q_pos, budget, lam, eta, debug=False,
                    want_evicted=False):
        """The same step for one new token per sequence through the fused entry point."""
        B.im_decode_step(self.h, self.p, self.st, q, x_gate, q_pos, k_new, v_new, pos_new, budget, lam, eta,
                         self.out, self.readout if debug else None,
                         self.evicted if (debug or want_evicted) else None, self.scores if debug else None)
        return self.out
