"""Glue used by the tests: exact bf16 -> fp64 conversion of the seeded inputs and the oracle's
parameter / config objects for a workload."""
from __future__ import annotations

import numpy as np
import torch

from oracle import indexmem_oracle as O
from workloads import Workload, layer_params


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact conversion of a (bf16 / fp32 / int) tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_params(p: dict) -> O.OracleParams:
    return O.OracleParams(Uq=f64(p["Uq"]), G=f64(p["G"]), Uk=f64(p["Uk"]),
                          norm_q_w=f64(p["norm_q_w"]), norm_k_w=f64(p["norm_k_w"]),
                          Wtheta=f64(p["Wtheta"]), wg=f64(p["wg"]), cg=float(p["cg"]))


def oracle_config(w: Workload, capacity=None, batch=None, kv_head_ids=None) -> O.OracleConfig:
    return O.OracleConfig(batch=w.batch if batch is None else batch,
                          n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                          capacity=w.capacity if capacity is None else capacity,
                          n_idx_heads=w.n_idx_heads, head_dim=w.head_dim, idx_dim=w.idx_dim,
                          mem_dim=w.mem_dim, n_sink=w.n_sink, n_recent=w.n_recent,
                          # the library takes these three as fp32; the oracle uses the same values
                          rms_eps=float(np.float32(1e-6)), mem_eps=float(np.float32(1e-6)),
                          softmax_scale=float(np.float32(float(w.head_dim) ** -0.5)),
                          kv_head_ids=kv_head_ids)


def make_oracle_layer(w: Workload, layer: int = 0, device="cpu", params=None, **kw):
    """params: the layer's weights as layer_params returns them (default: generated here)."""
    cls = O.OracleLayerShared if w.head_shared else O.OracleLayer
    return cls(oracle_config(w, **kw), oracle_params(layer_params(w, layer, device) if params is None else params))
