"""Writes tests/golden/oracle_stream_cfg1.json: what the CPU oracle computes on a small seeded
stream (config 1 shape, 768 tokens in chunks of 128). Calls only `oracle/` and the seeded input
generator. The stored values pin the oracle's arithmetic against silent changes and give the GPU
tests a reference that does not depend on the oracle code of the day.

    python tests/golden/make_oracle_stream_fixture.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ltri_oracle as O                                    # noqa: E402
from workloads import CONFIGS, planted_stream, theta_default         # noqa: E402

SEED, T, L = 7, 768, 128
ROWS = (0, 1, 63, 127)


def build():
    w = CONFIGS["cfg1"]
    K, V, Q, _ = planted_stream(w, SEED, device="cpu", context=T)
    Kn, Vn, Qn = K.double().numpy(), V.double().numpy(), Q.double().numpy()
    cfg = O.OracleConfig(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, w.n_sink, w.window,
                         k_max=w.k_max, budget_tokens=w.budget_tokens,
                         theta=float(np.float32(theta_default(w.head_dim))))
    st = O.OracleStream(cfg, Kn, Vn)
    chunks = []
    for c0 in range(0, T, L):
        q = Qn[c0:c0 + L]
        st.append_chunk(L, q_seg=None)
        sel = st.retrieve(q)
        out, lse = st.attend(q, rows=list(ROWS))
        chunks.append({
            "chunk_start": c0,
            "bounds": [[int(x) for x in st.last_bounds[h]] for h in range(w.n_kv_heads)],
            "selected": [[int(i) for i in sel[h]] for h in range(w.n_kv_heads)],
            "context_tokens": [len(st.context_tokens(h)) for h in range(w.n_kv_heads)],
            "out_rows": list(ROWS),
            "out_head0_first8": [[float(f"{v:.12e}") for v in out[r, 0, :8]] for r in range(len(ROWS))],
            "lse_head0": [float(f"{lse[r, 0]:.12e}") for r in range(len(ROWS))],
        })
    return {"seed": SEED, "tokens": T, "chunk": L, "config": "cfg1", "chunks": chunks}


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_stream_cfg1.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", path)
