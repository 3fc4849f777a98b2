"""Per-kernel-family summary of rocprofv3 --pmc counter dumps of the slide step: matrix-core utilisation and the
stall / LDS figures that explain it.

    python -m paper_2403_04865_amd.pmc_summary PASS1_DIR [PASS2_DIR ...]

Each PASS_DIR is the output directory of one
    rocprofv3 --pmc <counters> --kernel-trace --output-format csv -d PASS_DIR -o t -- python3 bench.py ...
run (one counter group per run; the directory holds t_counter_collection.csv and t_kernel_trace.csv).  Counters
used when present: SQ_VALU_MFMA_BUSY_CYCLES, SQ_BUSY_CU_CYCLES, SQ_INSTS_VALU_MFMA_MOPS_BF16, SQ_WAVE_CYCLES,
SQ_WAIT_INST_ANY, SQ_WAIT_INST_LDS, SQ_ACTIVE_INST_VALU, SQ_LDS_BANK_CONFLICT, SQ_LDS_IDX_ACTIVE,
TCP_PENDING_STALL_CYCLES_sum, GRBM_GUI_ACTIVE.  Prints one block per family (average per launch):
  mfma_busy      = SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES): share of the SIMDs' busy time the matrix pipe works
  tflops_counter = SQ_INSTS_VALU_MFMA_MOPS_BF16 * 512 flop / launch time (kernel trace of the same run)
  frac_of_peak   = tflops_counter / 2500 (dense bf16 peak of the chip)
  wait_any, wait_lds, valu_active = the wave-cycle counters over SQ_WAVE_CYCLES
  lds_conflict   = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE
  tcp_pending    = TCP_PENDING_STALL_CYCLES_sum / (compute units * kernel clocks), kernel clocks = GRBM_GUI_ACTIVE / 8 XCDs
  clock_ghz      = kernel clocks / launch time: the clock the chip held during the kernel (frac_of_peak is against the
                   peak at 2.4 GHz, mfma_busy against the cycles that actually passed)
"""
from __future__ import annotations

import collections
import csv
import os
import sys

from .pmc_traffic import FAMILIES, family_of

PEAK_TFLOPS = 2500.0
CUS, XCDS = 256, 8


def main(dirs):
    cnt = collections.defaultdict(lambda: collections.defaultdict(float))   # family -> counter -> sum over launches
    n = collections.defaultdict(collections.Counter)                        # family -> counter -> launches seen
    dur = collections.defaultdict(list)                                     # family -> launch durations (ns)
    for d in dirs:
        cc = os.path.join(d, "t_counter_collection.csv")
        with open(cc) as f:
            for r in csv.DictReader(f):
                fam = family_of(r["Kernel_Name"])
                if fam:
                    cnt[fam][r["Counter_Name"]] += float(r["Counter_Value"])
                    n[fam][r["Counter_Name"]] += 1
        kt = os.path.join(d, "t_kernel_trace.csv")
        if os.path.exists(kt) and not dur:
            with open(kt) as f:
                for r in csv.DictReader(f):
                    fam = family_of(r["Kernel_Name"])
                    if fam:
                        dur[fam].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    for fam, _ in FAMILIES:
        if fam not in cnt:
            continue
        c = {k: v / max(n[fam][k], 1) for k, v in cnt[fam].items()}   # per launch
        ms = sum(dur[fam]) / len(dur[fam]) / 1e6 if dur.get(fam) else None
        out = [f"{fam}: launches {len(dur[fam]) if dur.get(fam) else min(n[fam].values())}" + (f", avg {ms:.4f} ms" if ms else "")]

        def ratio(a, b, scale=1.0):
            return c[a] / (c[b] * scale) if a in c and b in c and c[b] > 0 else None
        fields = [("mfma_busy", ratio("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", 4.0)),
                  ("wait_any", ratio("SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES")),
                  ("wait_lds", ratio("SQ_WAIT_INST_LDS", "SQ_WAVE_CYCLES")),
                  ("valu_active", ratio("SQ_ACTIVE_INST_VALU", "SQ_WAVE_CYCLES")),
                  ("lds_conflict", ratio("SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE")),
                  ("tcp_pending", ratio("TCP_PENDING_STALL_CYCLES_sum", "GRBM_GUI_ACTIVE", CUS / XCDS))]
        if "SQ_INSTS_VALU_MFMA_MOPS_BF16" in c and ms:
            tf = c["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512 / (ms * 1e-3) / 1e12
            fields += [("tflops_counter", tf), ("frac_of_peak", tf / PEAK_TFLOPS)]
        if "GRBM_GUI_ACTIVE" in c and ms:
            fields += [("clock_ghz", c["GRBM_GUI_ACTIVE"] / XCDS / (ms * 1e-3) / 1e9)]
        out.append("   " + "  ".join(f"{k} {v:.3f}" for k, v in fields if v is not None))
        print("\n".join(out))


if __name__ == "__main__":
    main(sys.argv[1:])
