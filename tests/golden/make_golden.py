"""Write the expected values for the full-size configurations.

Runs ONLY the CPU oracle (oracle/cfdetr_oracle.py) on the seeded workloads of
the two largest configurations and stores, per configuration, the integer
selection outputs in full and a dense sample of output rows.  The GPU parity
test compares the same rows.  Usage:  python tests/golden/make_golden.py [4 5]

The sample is laid out in the row order of one merged run (the coarse grids of all
frames, then the mixed token sets): one row of every block of 32 consecutive rows (at
a position that rotates through the block), every multiple of 64 with the row before
and the row after it (these are the edges of row tiles of 64, 128, 192 and 256 rows),
and the first and last row of every sequence.  A mistake confined to one row tile of
any of these sizes, or to a sequence boundary, hits a stored row.
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import cfdetr_oracle as O          # noqa: E402
from paper_2505_23317_amd import synth         # noqa: E402

def sample_rows(n_coarse: int, cu: np.ndarray) -> np.ndarray:
    """Rows of a merged run (coarse rows first, then mixed rows) that the sample keeps."""
    total = n_coarse + int(cu[-1])
    rows = set()
    for b in range((total + 31) // 32):
        rows.add(min(32 * b + (7 * b) % 32, total - 1))
    for m in range(0, total + 64, 64):
        rows.update(r for r in (m - 1, m, m + 1) if 0 <= r < total)
    n0 = n_coarse // (len(cu) - 1)
    for i in range(len(cu) - 1):
        rows.update([i * n0, (i + 1) * n0 - 1])
        if cu[i + 1] > cu[i]:
            rows.update([n_coarse + int(cu[i]), n_coarse + int(cu[i + 1]) - 1])
    return np.asarray(sorted(rows), dtype=np.int64)


def make(cfg_id: int) -> None:
    cfg = synth.config(cfg_id)
    wl = synth.make_workload(cfg_id)
    t0 = time.time()
    yc, ym, tok, cu, counts = O.multilevel_batch(wl["images"], wl["boxes"], wl["tier"],
                                                 wl["box_offsets"], cfg.patch, wl["weights"],
                                                 cfg.heads)
    rows = sample_rows(len(yc), cu)
    rows_c = rows[rows < len(yc)]
    rows_m = rows[rows >= len(yc)] - len(yc)
    out = os.path.join(HERE, f"cfg{cfg_id}_oracle.npz")
    np.savez_compressed(
        out, tok_desc=O.pack_tok_desc(tok), cu_seqlens=cu.astype(np.int32),
        level_counts=counts.astype(np.int32), rows_coarse=rows_c, rows_mixed=rows_m,
        y_coarse=yc[rows_c].astype(np.float32), y_mixed=ym[rows_m].astype(np.float32),
        max_abs_coarse=np.abs(yc).max(), max_abs_mixed=np.abs(ym).max())
    print(f"cfg{cfg_id}: T={int(cu[-1])} lens={np.diff(cu).tolist()} rows stored "
          f"{len(rows_c)} + {len(rows_m)} oracle {time.time() - t0:.1f}s -> {out}", flush=True)


if __name__ == "__main__":
    for cid in [int(a) for a in sys.argv[1:]] or [4, 5]:
        make(cid)
