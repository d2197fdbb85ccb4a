"""HBM traffic of the hot path from rocprofv3 counters.

Two steps, both on the GPU machine:

  rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT/fetch -o t -- \
      python3 hbm_probe.py run --config 3
  rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d OUT/write -o t -- \
      python3 hbm_probe.py run --config 3
  python3 hbm_probe.py report OUT/fetch/t_counter_collection.csv \
      OUT/write/t_counter_collection.csv --config 3 > profiles/<name>.txt

`run` first copies a buffer of known size with a plain device-to-device copy kernel
(the calibration: it reads and writes exactly COPY_BYTES), then runs a few
cfdetr_multilevel_batch steps.  `report` scales each counter by what it read for the
copy and prints bytes per launch for every kernel family.
"""
from __future__ import annotations

import argparse
import collections
import csv
import os
import re
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

COPY_BYTES = 1 << 30
STEPS = 3

FAMILIES = [
    ("attention", r"attention_bf16_kernel"),
    ("gemm_qkv", r"gemm_bf16_(direct|persist)_kernel.*EpiQkv"),
    ("gemm_ffn1_gelu", r"gemm_bf16_(direct|persist)_kernel.*EpiAct<unsigned short, (true|1)>"),
    ("gemm_residual", r"gemm_bf16_(direct|persist)_kernel.*EpiResidual|gemm_bf16_rowln_kernel"),
    ("layer_tail", r"layer_tail_kernel"),
    ("layer_head", r"layer_head_kernel"),
    ("embed", r"gemm_bf16_gather_kernel|gemm_bf16_direct_kernel.*EpiEmbed"),
    ("layernorm", r"layernorm4?_kernel"),
    ("select_hit", r"select_hit_kernel"),
    ("select_compact", r"select_compact_kernel"),
    ("gather_coarse", r"gather_coarse_kernel"),
    ("plan", r"plan_kernel"),
]


def run(cfg_id: int) -> None:
    import torch
    from paper_2505_23317_amd import cfdetr, synth
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)                       # the calibration kernel (elementwise copy)
    torch.cuda.synchronize()
    cfg = synth.config(cfg_id)
    wl = synth.make_workload(cfg_id)
    enc = cfdetr.Encoder(cfg, wl["weights"])
    img = enc.upload_images(wl["images"])
    b, t, o = enc.upload_boxes(wl["boxes"], wl["tier"], wl["box_offsets"])
    out = enc.alloc_outputs(cfg.B)
    for _ in range(STEPS):
        enc.multilevel_batch(img, cfg.B, b, t, o, out)
    enc.sync_status()
    enc.close()


def _read(path: str):
    """kernel name -> list of counter values (one per dispatch, in dispatch order), and
    the counter's name."""
    vals = collections.defaultdict(list)
    name = None
    with open(path) as f:
        rows = sorted(csv.DictReader(f), key=lambda r: int(r["Dispatch_Id"]))
    for r in rows:
        name = r["Counter_Name"]
        vals[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return vals, name


def _copy_reading(vals):
    """Counter value of the calibration copy: the largest single dispatch of a copy kernel."""
    best = 0.0
    for k, v in vals.items():
        if "copy" in k.lower() or "elementwise" in k.lower():
            best = max(best, max(v))
    return best


def _alternate(v, sel):
    """Every second dispatch of one kernel name, restarting with each of the STEPS steps."""
    per = len(v) // STEPS
    if per == 1:   # the instantiation that ends a run (final LayerNorm): a second FFN projection
        return list(v) if sel == 1 else []
    return [x for s0 in range(0, per * STEPS, per) for x in v[s0:s0 + per][sel::2]]


def report(fetch_csv: str, write_csv: str, cfg_id: int) -> None:
    fetch, fname = _read(fetch_csv)
    write, wname = _read(write_csv)
    cf, cw = _copy_reading(fetch), _copy_reading(write)
    if cf <= 0 or cw <= 0:
        sys.exit("calibration copy not found in the counter files")
    kf, kw = COPY_BYTES / cf, COPY_BYTES / cw        # bytes per counter unit
    print(f"# HBM traffic per launch, cfdetr_multilevel_batch, config {cfg_id}")
    print("# commands, from the repository root on the MI355X box (OUT = any scratch folder):")
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        print(f"#   rocprofv3 --pmc {c} --kernel-trace --output-format csv -d OUT/{c.lower()} -o t "
              f"-- python3 hbm_probe.py run --config {cfg_id}")
    print(f"#   python3 hbm_probe.py report OUT/fetch_size/t_counter_collection.csv "
          f"OUT/write_size/t_counter_collection.csv --config {cfg_id}")
    print(f"# counters: {fname}, {wname}; calibration: a {COPY_BYTES} byte device copy read "
          f"{cf:.1f} / {cw:.1f} counter units -> {kf:.1f} / {kw:.1f} bytes per unit "
          f"(1024 would mean KiB)")
    print("# family launches fetch_bytes_per_launch write_bytes_per_launch")
    for fam, pat in FAMILIES:
        rx = re.compile(pat)
        f = [x for k, v in fetch.items() if rx.search(k) for x in v]
        w = [x for k, v in write.items() if rx.search(k) for x in v]
        if not f or not w:
            continue
        if fam == "gemm_residual":
            # the two residual contractions of a layer alternate: output projection, then
            # second FFN projection (the last one of a run may be another instantiation,
            # which keeps the alternation per kernel name)
            for part, sel in (("gemm_out_proj", 0), ("gemm_ffn2", 1)):
                fp = [x for k, v in fetch.items() if rx.search(k) for x in _alternate(v, sel)]
                wp = [x for k, v in write.items() if rx.search(k) for x in _alternate(v, sel)]
                if fp and wp:
                    print(f"{part} {len(fp)} {kf * sum(fp) / len(fp):.0f} {kw * sum(wp) / len(wp):.0f}")
            continue
        print(f"{fam} {len(f)} {kf * sum(f) / len(f):.0f} {kw * sum(w) / len(w):.0f}")


def counters(csvs, cfg_id: int, names) -> None:
    """Per-launch averages of every counter in rocprofv3 counter files of `run`, by kernel
    family (same families as `report`), plus each counter as a fraction of GRBM_GUI_ACTIVE
    times the number of SIMDs where that is a meaningful ratio."""
    print(f"# Shader counters per launch, cfdetr_multilevel_batch, config {cfg_id}")
    print("# command, from the repository root on the MI355X box (OUT = any scratch folder):")
    print(f"#   rocprofv3 --pmc {' '.join(names)} --kernel-trace --output-format csv -d OUT -o t "
          f"-- python3 hbm_probe.py run --config {cfg_id}")
    print(f"#   python3 hbm_probe.py counters OUT/t_counter_collection.csv "
          f"--config {cfg_id}")
    print("# values are sums over the chip (SQ counters: over its 1024 SIMDs = 256 CUs x 4;")
    print("# GRBM_GUI_ACTIVE: over its 8 XCDs), averaged over the launches of a family.")
    print("# 'per SIMD-cycle' divides by the SIMD-cycles the kernel had: GRBM_GUI_ACTIVE / 8 x 1024.")
    print("# For SQ_VALU_MFMA_BUSY_CYCLES that is the share of time the matrix unit was busy (it")
    print("# equals SQ_INSTS_MFMA x 32 cycles for 32x32x16 bf16); for SQ_ACTIVE_INST_* the share of")
    print("# time an instruction of that kind was executing; SQ_ACTIVE_INST_* and SQ_WAIT_* count in")
    print("# units of 4 cycles (SQ_ACTIVE_INST_VALU / SQ_INSTS_VALU = 1.2-1.3 is the mix of 4- and")
    print("# 16-cycle instructions), so their shares are printed times 4.")
    tot = collections.defaultdict(lambda: collections.defaultdict(float))
    cnt = collections.defaultdict(lambda: collections.defaultdict(int))
    for path in csvs:
        with open(path) as f:
            for r in csv.DictReader(f):
                for fam, pat in FAMILIES:
                    if re.search(pat, r["Kernel_Name"]):
                        tot[fam][r["Counter_Name"]] += float(r["Counter_Value"])
                        cnt[fam][r["Counter_Name"]] += 1
                        break
    for fam, _ in FAMILIES:
        if fam not in tot:
            continue
        avg = {c: tot[fam][c] / cnt[fam][c] for c in tot[fam]}
        active = avg.get("GRBM_GUI_ACTIVE", 0.0)
        print(f"{fam} ({max(cnt[fam].values())} launches)")
        for c in sorted(avg):
            line = f"   {c:30s} {avg[c]:16.0f}"
            if active > 0 and c != "GRBM_GUI_ACTIVE":
                quad = 4.0 if c.startswith("SQ_ACTIVE_INST") or c.startswith("SQ_WAIT") else 1.0
                line += f"   {quad * avg[c] / (active * 128):8.3f} per SIMD-cycle"
            print(line)


def main() -> None:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    r = sub.add_parser("run")
    r.add_argument("--config", type=int, default=3)
    p = sub.add_parser("report")
    p.add_argument("fetch_csv")
    p.add_argument("write_csv")
    p.add_argument("--config", type=int, default=3)
    c = sub.add_parser("counters")
    c.add_argument("csv", nargs="+")
    c.add_argument("--config", type=int, default=3)
    c.add_argument("--names", nargs="*", default=["GRBM_GUI_ACTIVE", "SQ_VALU_MFMA_BUSY_CYCLES",
                                                  "SQ_ACTIVE_INST_VALU", "SQ_ACTIVE_INST_LDS",
                                                  "SQ_ACTIVE_INST_VMEM", "SQ_INSTS_MFMA",
                                                  "SQ_INSTS_VALU", "SQ_WAIT_INST_ANY"])
    a = ap.parse_args()
    if a.cmd == "counters":
        counters(a.csv, a.config, a.names)
        return
    if a.cmd == "run":
        run(a.config)
    else:
        report(a.fetch_csv, a.write_csv, a.config)


if __name__ == "__main__":
    main()
