"""Helpers of the GPU parity tests: drive the library and the oracle over the same stream."""
from __future__ import annotations

import numpy as np
import torch

from oracle import ltri_oracle as O
from paper_2412_04757_amd import LtriContext, config_from_workload
from workloads import theta_default


def make_pair(w, K, V, device, *, max_tokens, seg_map=O.MAP_LOGIT, theta=None, phi=0.0,
              max_spans_per_chunk=0, window=None, n_sink=None, k_max=None, budget_tokens=None,
              chunk_max=None, max_spans=0, rep_mode=0, lam=3.0, index_min=1, index_max=0, ratio_mode=0,
              theta_quantile=0.0, unit_tokens=0, kv_offload=0, index_block_max=0):
    """A library context with K/V resident in its arenas and the matching oracle stream."""
    theta = theta_default(w.head_dim) if theta is None else theta
    cfg = config_from_workload(w, max_tokens=max_tokens, theta=theta, phi=phi, seg_map=seg_map,
                               n_layers=1, n_seqs=1, max_spans_per_chunk=max_spans_per_chunk,
                               window=window, n_sink=n_sink, k_max=k_max, budget_tokens=budget_tokens,
                               chunk_max=chunk_max, max_spans=max_spans, rep_mode=rep_mode,
                               lam=lam, index_min=index_min, index_max=index_max, ratio_mode=ratio_mode,
                               theta_quantile=theta_quantile, unit_tokens=unit_tokens, kv_offload=kv_offload,
                               index_block_max=index_block_max)
    ctx = LtriContext(cfg, device)
    ka, va = ctx.arena_views()
    T = K.shape[1]
    if kv_offload:          # the arenas are host memory that the appends fill: poison them so that a row read before
        ka.fill_(float("nan")); va.fill_(float("nan"))          # its append would show
    else:
        ka[0, 0, :, :T].copy_(K)
        va[0, 0, :, :T].copy_(V)
    ocfg = O.OracleConfig(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, cfg.n_sink, cfg.window,
                          k_max=cfg.k_max, budget_tokens=cfg.budget_tokens, seg_map=seg_map,
                          theta=float(np.float32(theta)), phi=float(np.float32(phi)),
                          max_spans_per_chunk=max_spans_per_chunk, rep_mode=rep_mode,
                          lam=float(np.float32(lam)), n_min=index_min, n_max=index_max, ratio_mode=ratio_mode,
                          theta_quantile=float(np.float32(theta_quantile)), unit_tokens=unit_tokens,
                          block_max=index_block_max)
    st = O.OracleStream(ocfg, K.double().cpu().numpy(), V.double().cpu().numpy())
    return ctx, st


def spans_equal(ctx, st, h):
    s, l = ctx.get_spans(0, 0, h)
    return list(s) == st.starts[h] and list(l) == st.lens[h]


def rep_keys_diff(ctx, st, h):
    got = ctx.get_rep_keys(0, 0, h).double().numpy()
    want = np.stack(st.krep[h])
    return float(np.abs(got - want).max())
