"""JSON serialisation of logit-lens results, "indexed by layer and activation type" (paper Sec. 3.1,
Stage 3).  The paper does not print its schema; this one is

    {"meta": {...},
     "layers": {"<layer>": {"<activation type>": [ {"position": t,
                                                    "topk": [{"id": i, "token": s, "p": x}, ...],
                                                    "target_logp": x, "entropy": x}, ... ]}}}

Host code only: it takes the arrays the library returned (already copied to the host or not).
"""
from __future__ import annotations

import json

import numpy as np


def _host(x):
    if x is None:
        return None
    return x.detach().cpu().numpy() if hasattr(x, "detach") else np.asarray(x)


def lens_to_dict(topk_ids, topk_p, L: int, T: int, *, target_logp=None, entropy=None, activation_type: str = "block",
                 layer_names=None, id_to_token=None, meta=None) -> dict:
    """Rows are r = l*T + t (the packed trajectories).  layer_names defaults to "embed", "layer_1", ..."""
    ids, p = _host(topk_ids), _host(topk_p)
    lp, ent = _host(target_logp), _host(entropy)
    if ids.shape != p.shape or ids.ndim != 2 or ids.shape[0] != L * T:
        raise ValueError("topk_ids / topk_p must both be [L*T, k]")
    if layer_names is None:
        layer_names = ["embed"] + [f"layer_{l}" for l in range(1, L)]
    if len(layer_names) != L:
        raise ValueError("need one name per layer")
    out = {"meta": dict(meta or {}, L=L, T=T, k=int(ids.shape[1])), "layers": {}}
    for l in range(L):
        rows = []
        for t in range(T):
            r = l * T + t
            entry = {"position": t,
                     "topk": [dict({"id": int(i), "p": float(q)},
                                   **({"token": id_to_token(int(i))} if id_to_token else {}))
                              for i, q in zip(ids[r], p[r])]}
            if lp is not None:
                v = float(lp[r])
                entry["target_logp"] = None if np.isnan(v) else v
            if ent is not None:
                entry["entropy"] = float(ent[r])
            rows.append(entry)
        out["layers"][layer_names[l]] = {activation_type: rows}
    return out


def lens_to_json(*args, indent=None, **kwargs) -> str:
    return json.dumps(lens_to_dict(*args, **kwargs), indent=indent)
