#!/usr/bin/env python3
"""Writes tests/golden/cfg1_rollout.json: what the CPU oracle computes on the tiny workload cfg1.

The paper prints no intermediate values (no worked example), so this fixture is not a pin of the
oracle against the paper: it freezes the oracle's own results (block sets of Eq. 10-11, block scores
and slot assignments of Eq. 7-9, a few attention rows of Eq. 3-5, the summary counts) so that a later
change to the oracle's arithmetic or to the input generator shows up as a diff.  It calls only oracle/
and the seeded input generator.  Run from the repository root: python tests/golden/make_cfg1_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle.rollout import run_chunk, state_for_workload  # noqa: E402
from harness import synth  # noqa: E402

ROWS_T = [0, 63, 64, 130, 255]      # tokens whose attention rows are stored (both heads)
DIMS = [0, 1, 31, 63]               # output dimensions stored per row


def build():
    w = synth.WORKLOADS["cfg1"]
    st, g0 = state_for_workload(w)
    hh = np.repeat(np.arange(w.H, dtype=np.int32), len(ROWS_T))
    tt = np.tile(np.array(ROWS_T, np.int32), w.H)
    chunks = []
    for g in range(g0, g0 + 3):
        r = run_chunk(st, w, 0, g, rows=(hh, tt))
        chunks.append({
            "chunk": g,
            "sel": r["sel"].tolist(),
            # fp32 values that decide integers are stored as bit patterns
            "scores_bits": r["scores"].view(np.uint32).tolist(),
            "slot_src": r["slot_src"].tolist(),
            "p_id": st.p_id.tolist(),
            "p_len": st.p_len.tolist(),
            "S_cnt_sum": int(st.S_cnt.sum()),
            "O_rows": np.round(r["O"][:, DIMS].astype(np.float64), 6).tolist(),
            "lse_rows": np.round(r["lse"].astype(np.float64), 6).tolist(),
        })
    return {"workload": "cfg1", "rows_t": ROWS_T, "dims": DIMS, "chunks": chunks}


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_rollout.json")
    with open(out, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", out)
