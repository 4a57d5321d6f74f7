"""Host-side check of the JSON writer (layer / activation-type index of the paper's Stage 3)."""
import json

import numpy as np
import pytest

from paper_2604_06483_amd import serialize as S


def test_json_is_indexed_by_layer_and_activation_type():
    L, T, k = 3, 4, 2
    ids = np.arange(L * T * k, dtype=np.int32).reshape(L * T, k)
    p = np.linspace(0.9, 0.1, L * T * k, dtype=np.float32).reshape(L * T, k)
    lp = np.full(L * T, -1.5, dtype=np.float32)
    lp[5] = np.nan
    ent = np.full(L * T, 2.0, dtype=np.float32)
    d = json.loads(S.lens_to_json(ids, p, L, T, target_logp=lp, entropy=ent, activation_type="mlp",
                                  id_to_token=lambda i: f"<{i}>", meta={"model": "synthetic"}))
    assert set(d["layers"]) == {"embed", "layer_1", "layer_2"}
    rows = d["layers"]["layer_1"]["mlp"]
    assert len(rows) == T and rows[1]["position"] == 1
    r = 1 * T + 1
    assert rows[1]["topk"][0] == {"id": int(ids[r, 0]), "p": pytest.approx(float(p[r, 0])), "token": f"<{ids[r, 0]}>"}
    assert rows[1]["target_logp"] is None            # NaN (target outside the vocabulary) -> null
    assert rows[0]["target_logp"] == pytest.approx(-1.5) and rows[0]["entropy"] == pytest.approx(2.0)
    assert d["meta"] == {"model": "synthetic", "L": L, "T": T, "k": k}
    with pytest.raises(ValueError):
        S.lens_to_dict(ids[:-1], p[:-1], L, T)
