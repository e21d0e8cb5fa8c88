"""Glue shared by the GPU parity tests, the smoke check and the benchmark:
moves a Workload to the device, calls the library through its C ABI, and calls
the oracle on the same bits.  No attention arithmetic lives here."""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np
import torch

import oracle
from paper_2602_01053_amd.runner import DeviceWorkload
from paper_2602_01053_amd.workloads import Workload

REL_L2_TOL = 5e-3      # relative L2 over the whole output and per query
MAX_ABS_TOL = 2e-2


def run_decode(w: Workload, dev, head_major: bool = False) -> np.ndarray:
    dw = DeviceWorkload(w, dev, head_major)
    dw.alloc_workspace()
    dw.out.fill_(float("nan"))
    dw.decode()
    torch.cuda.synchronize()
    return dw.out.to(torch.float64).cpu().numpy()


def run_prefill(w: Workload, dev) -> np.ndarray:
    dw = DeviceWorkload(w, dev)
    dw.alloc_workspace()
    dw.out.fill_(float("nan"))
    dw.prefill()
    torch.cuda.synchronize()
    return dw.out.to(torch.float64).cpu().numpy()


def _f64(t: Optional[torch.Tensor]):
    return None if t is None else t.to(torch.float64).numpy()


def oracle_decode(w: Workload) -> np.ndarray:
    return oracle.decode(_f64(w.q), _f64(w.k_base), _f64(w.v_base), _f64(w.l), _f64(w.b_k),
                         _f64(w.b_v), w.query_adapter.numpy(), w.seq_query_start.numpy(),
                         w.seq_lens, w.scale, block_size=w.block_size,
                         block_table=None if w.block_table is None else w.block_table.numpy())


def oracle_prefill(w: Workload, rows=None) -> np.ndarray:
    a = int(w.query_adapter[0])
    return oracle.prefill(_f64(w.q), _f64(w.k_base), _f64(w.v_base), _f64(w.l), _f64(w.b_k[a]),
                          _f64(w.b_v[a]), n=w.seq_lens[0], scale=w.scale, rows=rows)


def oracle_prefill_by_blocks(w: Workload, key_rope_theta: float = 0.0, block: int = 256) -> np.ndarray:
    """Every new-token row of a prefill workload from the oracle, evaluated in blocks of rows (rows are
    independent) so that the fp64 score matrix of one call stays small; prints a line per block."""
    a = int(w.query_adapter[0])
    args = (_f64(w.q), _f64(w.k_base), _f64(w.v_base), _f64(w.l), _f64(w.b_k[a]), _f64(w.b_v[a]))
    parts = []
    for r0 in range(0, w.n_new, block):
        rows = np.arange(r0, min(r0 + block, w.n_new))
        parts.append(oracle.prefill(*args, n=w.seq_lens[0], scale=w.scale, rows=rows, key_rope_theta=key_rope_theta))
        print(f"oracle rows {r0}..{rows[-1]} done", flush=True)
    return np.concatenate(parts)


def errors(got: np.ndarray, ref: np.ndarray) -> Tuple[float, float]:
    """(worst relative L2 over the whole tensor and over each leading-index slice,
    max abs error).  Non-finite outputs count as infinite error."""
    if not np.isfinite(got).all():
        return float("inf"), float("inf")
    rel_all = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    rel_each = max(np.linalg.norm(got[i] - ref[i]) / np.linalg.norm(ref[i]) for i in range(len(ref)))
    return float(max(rel_all, rel_each)), float(np.abs(got - ref).max())
