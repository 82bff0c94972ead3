"""Writes tests/golden/c1_mini_oracle.json: inputs drawn by `workloads` and the results the CPU oracle gives for
them.  Calls only `workloads` and `oracle/`.  The stored values guard the oracle against silent drift; they are
not an independent pin (those are in tests/test_oracle_pins.py and algorithm1_worked_rows.txt).

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
import workloads as W  # noqa: E402


def main():
    cfg = W.config("C1", B=6, rows_scale=2e-4, c=4.0)          # 1 table, 20 rows x 64, 6 bags of 20 uniform ids
    tab = W.weight_rows(cfg, 0, torch.arange(cfg.rows[0])).numpy()
    idx, off = (x.numpy() for x in W.make_batch(cfg, 0))
    gout = W.make_grad_out(cfg, 0).numpy()
    out = oracle.forward([tab], idx, off, cfg.B, cfg.pooling)
    state = np.zeros(cfg.rows[0], dtype=np.float32)
    res = oracle.backward_rowwise_adagrad([tab], state, gout, idx, off, cfg.B, cfg.pooling, cfg.lr, cfg.eps, cfg.c)
    doc = {
        "config": {"name": "C1", "B": 6, "rows_scale": 2e-4, "c": 4.0, "rows": cfg.rows, "D": cfg.D},
        "indices": idx.tolist(), "offsets": off.tolist(),
        "out_hex": out.astype(np.float32).tobytes().hex(),
        "weights_after_hex": tab.astype(np.float32).tobytes().hex(),
        "state_after_hex": state.tobytes().hex(),
        "order": res.order.tolist(), "unique_rows": res.unique_rows.tolist(), "seg_start": res.seg_start.tolist(),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_mini_oracle.json")
    with open(path, "w") as f:
        json.dump(doc, f)
    print("wrote", path)


if __name__ == "__main__":
    main()
