"""Turn four rocprofv3 --pmc counter dumps into HBM bytes per launch of each kernel family.

    python -m paper_2403_04865_amd.pmc_traffic WORKLOAD FETCH.csv WRITE.csv COPY_FETCH.csv COPY_WRITE.csv COPY_BYTES [COMMIT]

FETCH.csv / WRITE.csv: `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of `bench.py --workload WORKLOAD`
(counter_collection csv, one row per dispatch and counter).  COPY_*.csv: the same two counters over
`bench.py --calib-copy COPY_BYTES`; what they read for that plain copy of known size gives the scale of each
counter (bytes per count).  Writes profiles/traffic_WORKLOAD.json:
    {family: {"hbm_bytes_per_launch", "fetch_bytes_per_launch", "write_bytes_per_launch", "launches"}, ...,
     "_scale": {...}}
Kernel families are the names the library's timing hooks use (gemm_nt, gemm_tn, attn_fwd, ...; for the ResNet step
conv_nt = conv_fwd + conv_dgrad, conv_wgrad, bn_stats, bn_apply, bn_bwd, pooling).
COMMIT (optional) is recorded as "_commit": the source revision the counters were collected on; bench.py prints it
beside the traffic figures it reads from this file.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

FAMILIES = [("gemm_nt", ("gemm_nt_",)), ("gemm_tn", ("gemm_tn_",)), ("attn_fwd", ("attn_fwd",)),
            ("attn_bwd", ("attn_bwd",)), ("ln_fwd", ("ln_fwd",)), ("ln_bwd", ("ln_bwd",)),
            ("pool_fwd", ("pool_gate", "pool_combine", "pool_alpha", "pool_cast")), ("pool_bwd", ("pool_bwd",)),
            ("cls_lane", ("lane_",)),
            # convolutional encoders: forward and input gradient are launches of one kernel (family conv_nt)
            ("conv_nt", ("conv_nt_",)), ("conv_wgrad", ("conv_wgrad_",)), ("bn_stats", ("bn_stats_",)),
            ("bn_apply", ("bn_apply_",)), ("bn_bwd", ("bn_bwd_",)), ("pooling", ("maxpool_", "avgpool_"))]


def per_dispatch(path, counter):
    """[(kernel name, counter value)] per dispatch."""
    out = []
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                out.append((r["Kernel_Name"], float(r["Counter_Value"])))
    return out


def family_of(name):
    for fam, keys in FAMILIES:
        if any(k in name for k in keys):
            return fam
    return None


def main(argv):
    workload, fetch, write, cfetch, cwrite, copy_bytes = argv[0], argv[1], argv[2], argv[3], argv[4], int(argv[5])
    scale = {}
    for counter, path in (("FETCH_SIZE", cfetch), ("WRITE_SIZE", cwrite)):
        vals = [v for k, v in per_dispatch(path, counter) if "calib_copy" in k]
        if not vals:
            raise SystemExit(f"no calib_copy dispatch in {path}")
        scale[counter] = copy_bytes / (sum(vals) / len(vals))   # bytes per count
    agg = collections.defaultdict(lambda: {"FETCH_SIZE": 0.0, "WRITE_SIZE": 0.0, "n": 0})
    for counter, path in (("FETCH_SIZE", fetch), ("WRITE_SIZE", write)):
        for k, v in per_dispatch(path, counter):
            fam = family_of(k)
            if fam is None:
                continue
            agg[fam][counter] += v * scale[counter]
            if counter == "FETCH_SIZE":
                agg[fam]["n"] += 1
    out = {"_commit": argv[6] if len(argv) > 6 else None,
           "_scale": {"bytes_per_count": scale, "copy_bytes": copy_bytes,
                      "note": "counter readings of a plain copy of copy_bytes bytes define the scale"}}
    for fam, d in agg.items():
        n = max(d["n"], 1)
        out[fam] = {"hbm_bytes_per_launch": round((d["FETCH_SIZE"] + d["WRITE_SIZE"]) / n),
                    "fetch_bytes_per_launch": round(d["FETCH_SIZE"] / n),
                    "write_bytes_per_launch": round(d["WRITE_SIZE"] / n), "launches": d["n"]}
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    path = os.path.join(root, "profiles", f"traffic_{workload}.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main(sys.argv[1:])
