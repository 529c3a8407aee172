"""Random model parameters: Glorot-uniform weights, small uniform biases.

A model is a list of per-layer dicts. Keys:
  d_in, d_hidden (0 = single linear map), d_out,
  agg  'sum' | 'mean' | 'wsum' (needs edge weights) | 'max' | 'min' | 'attn' (graph attention, one head;
       extra key att: a_src followed by a_dst, d_out float32 each; self must be 'none'),
  self 'none' | 'concat' (GraphSAGE: rows [0,d_in) of W0 multiply the vertex's
       own embedding, rows [d_in,2*d_in) the aggregate) | 'add' (GIN:
       (1+eps)*own + aggregate),
  eps, act_inner, act_out ('none' | 'relu'),
  W0 [K x (d_hidden or d_out)], b0, and for d_hidden > 0 also W1 [d_hidden x d_out], b1;
  all float32, row-major, K = d_in or 2*d_in.
The last layer has no output activation (logits); hidden layers use ReLU.
"""
from __future__ import annotations

import numpy as np


def glorot(rng: np.random.Generator, fan_in: int, fan_out: int) -> np.ndarray:
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-a, a, size=(fan_in, fan_out)).astype(np.float32)


def _bias(rng: np.random.Generator, n: int) -> np.ndarray:
    return rng.uniform(-0.1, 0.1, size=n).astype(np.float32)


def make_model(kind: str, widths, seed: int, last_act: str = "none"):
    rng = np.random.default_rng(seed)
    layers = []
    L = len(widths) - 1
    for l in range(L):
        d_in, d_out = int(widths[l]), int(widths[l + 1])
        act_out = "relu" if l < L - 1 else last_act
        lay = dict(d_in=d_in, d_hidden=0, d_out=d_out, eps=0.0,
                   act_inner="none", act_out=act_out, W1=None, b1=None)
        if kind == "gcn_sum":
            lay.update(agg="sum", self="none", W0=glorot(rng, d_in, d_out), b0=_bias(rng, d_out))
        elif kind == "gcn_mean":
            lay.update(agg="mean", self="none", W0=glorot(rng, d_in, d_out), b0=_bias(rng, d_out))
        elif kind in ("gcn_max", "gcn_min"):
            lay.update(agg=kind.split("_")[1], self="none", W0=glorot(rng, d_in, d_out), b0=_bias(rng, d_out))
        elif kind == "gat":                   # single-head graph attention: att = a_src then a_dst (d_out each)
            lay.update(agg="attn", self="none", W0=glorot(rng, d_in, d_out), b0=_bias(rng, d_out),
                       att=glorot(rng, 2 * d_out, 1).reshape(-1))
        elif kind == "gcn_wsum":
            lay.update(agg="wsum", self="none", W0=glorot(rng, d_in, d_out), b0=_bias(rng, d_out))
        elif kind in ("sage_mean", "sage_sum", "sage_wsum", "sage_max", "sage_min"):
            w_self, w_neigh = glorot(rng, d_in, d_out), glorot(rng, d_in, d_out)
            lay.update(agg=kind.split("_")[1], self="concat",
                       W0=np.ascontiguousarray(np.vstack([w_self, w_neigh])), b0=_bias(rng, d_out))
        elif kind == "gin_sum":
            d_h = 256 if max(widths) >= 256 else int(max(widths))
            lay.update(agg="sum", self="add", d_hidden=d_h, act_inner="relu",
                       W0=glorot(rng, d_in, d_h), b0=_bias(rng, d_h),
                       W1=glorot(rng, d_h, d_out), b1=_bias(rng, d_out))
        else:
            raise ValueError(kind)
        layers.append(lay)
    return layers
