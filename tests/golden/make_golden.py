"""Write the expected values for the full-size configurations.

Runs ONLY the CPU oracle (oracle/cfdetr_oracle.py) on the seeded workloads of
the two largest configurations and stores, per configuration, the integer
selection outputs in full and a seeded sample of output rows.  The GPU parity
test compares the same rows.  Usage:  python tests/golden/make_golden.py [4 5]
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import cfdetr_oracle as O          # noqa: E402
from paper_2505_23317_amd import synth         # noqa: E402

N_ROWS = 48


def make(cfg_id: int) -> None:
    cfg = synth.config(cfg_id)
    wl = synth.make_workload(cfg_id)
    t0 = time.time()
    yc, ym, tok, cu, counts = O.multilevel_batch(wl["images"], wl["boxes"], wl["tier"],
                                                 wl["box_offsets"], cfg.patch, wl["weights"],
                                                 cfg.heads)
    rng = np.random.default_rng(100 + cfg_id)
    rows_c = np.sort(rng.choice(len(yc), size=N_ROWS, replace=False))
    # sample the mixed output from every frame, ends of each sequence included
    rows_m = set()
    for i in range(cfg.B):
        rows_m.update([int(cu[i]), int(cu[i + 1]) - 1])
    rows_m.update(rng.choice(len(ym), size=N_ROWS, replace=False).tolist())
    rows_m = np.sort(np.asarray(sorted(rows_m)))
    out = os.path.join(HERE, f"cfg{cfg_id}_oracle.npz")
    np.savez_compressed(
        out, tok_desc=O.pack_tok_desc(tok), cu_seqlens=cu.astype(np.int32),
        level_counts=counts.astype(np.int32), rows_coarse=rows_c, rows_mixed=rows_m,
        y_coarse=yc[rows_c].astype(np.float32), y_mixed=ym[rows_m].astype(np.float32),
        max_abs_coarse=np.abs(yc).max(), max_abs_mixed=np.abs(ym).max())
    print(f"cfg{cfg_id}: T={int(cu[-1])} lens={np.diff(cu).tolist()} "
          f"oracle {time.time() - t0:.1f}s -> {out}", flush=True)


if __name__ == "__main__":
    for cid in [int(a) for a in sys.argv[1:]] or [4, 5]:
        make(cid)
