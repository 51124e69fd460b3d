"""HBM traffic per launch from rocprofv3 counter collections, written to profiles/traffic.json.

Two counter runs of one program of this library (bench.py --headline-only --calibrate-copy), one with
`--pmc FETCH_SIZE` and one with `--pmc WRITE_SIZE` (KiB per dispatch), each also holding launches of
the library's plain copy kernel (torq_diag_copy) of a known size:

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d prof/fetch -o p -- \
        python3 bench.py --headline-only --calibrate-copy --no-cpu-baseline --no-board-sample --steps 5 --warmup 2
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d prof/write -o p -- \
        python3 bench.py --headline-only --calibrate-copy --no-cpu-baseline --no-board-sample --steps 5 --warmup 2
    python3 -m paper_2605_19561_amd.traffic --fetch prof/fetch --write prof/write

The copy kernel reads COPY_BYTES and writes COPY_BYTES; bytes = counter * 1024 * (COPY_BYTES / (1024 *
the counter's value for the copy)).  bench.py reads the file and calls its figures stale when the kernel
sources they were taken on are not the ones in the tree.
"""
import argparse
import csv
import glob
import hashlib
import json
import os
import statistics
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
OUT = os.path.join(ROOT, "profiles", "traffic.json")
COPY_BYTES = 1 << 30

# what bench.py's headline step launches: key -> (kernel name without spaces, grid size in work-items, sources)
KERNELS = {
    "mxfp4_gemm/llama3_70b_up": ("torq::mxfp4_gemm_kernel<4,4,true,false,false,0,true>", 256 * 256,
                                 ["mxfp4_gemm.hip", "torq_device.h"]),
    "torq_rotate_quantize/llama3_70b_up": ("torq::rotate_ring_kernel32<8,0,0>", 745 * 256,
                                           ["rotate_quant.hip", "rotate16_body.h", "torq_device.h"]),
}
COPY_KERNEL = "torq::diag_copy_kernel"


def source_digest(files):
    h = hashlib.sha256()
    for f in files:
        h.update(open(os.path.join(HERE, "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def _rows(directory):
    paths = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not paths:
        raise SystemExit(f"no *counter_collection.csv under {directory}")
    for p in paths:
        with open(p, newline="") as fh:
            for row in csv.DictReader(fh):
                yield row


def _medians(directory, counter):
    """{(kernel name without spaces and argument list, grid size): median counter value} over the dispatches"""
    vals = {}
    for row in _rows(directory):
        if row.get("Counter_Name") != counter:
            continue
        name = row["Kernel_Name"].replace(" ", "")
        if name.startswith("void"):
            name = name[4:]
        name = name.split("(")[0]
        vals.setdefault((name, int(row["Grid_Size"])), []).append(float(row["Counter_Value"]))
    return {k: (statistics.median(v), len(v)) for k, v in vals.items()}


def _find(meds, name, grid=None):
    hits = [(k, v) for k, v in meds.items() if k[0] == name and (grid is None or k[1] == grid)]
    if not hits:
        raise SystemExit(f"kernel {name} (grid {grid}) not in the counter run; has: {sorted({k[0] for k in meds})}")
    return max(hits, key=lambda kv: kv[1][1])[1]      # the variant with the most dispatches


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch", required=True, help="output directory of the --pmc FETCH_SIZE run")
    ap.add_argument("--write", required=True, help="output directory of the --pmc WRITE_SIZE run")
    ap.add_argument("--out", default=OUT)
    args = ap.parse_args()
    fetch, write = _medians(args.fetch, "FETCH_SIZE"), _medians(args.write, "WRITE_SIZE")
    copy_f, n_cf = _find(fetch, COPY_KERNEL)
    copy_w, n_cw = _find(write, COPY_KERNEL)
    f_scale, w_scale = COPY_BYTES / (copy_f * 1024.0), COPY_BYTES / (copy_w * 1024.0)
    try:
        head = subprocess.run(["git", "rev-parse", "--short=12", "HEAD"], cwd=ROOT, capture_output=True, text=True).stdout.strip()
    except OSError:
        head = ""
    doc = {"what": "HBM bytes per launch: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, medians), scaled by "
                   "the same counter's reading for torq_diag_copy of 1 GiB in the same run",
           "git_head": head,
           "calibration": {"copy_bytes": COPY_BYTES, "copy_fetch_kib": copy_f, "copy_write_kib": copy_w,
                           "copy_dispatches": [n_cf, n_cw], "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4)},
           "kernels": {}}
    for key, (name, grid, files) in KERNELS.items():
        (kf, nf), (kw, nw) = _find(fetch, name, grid), _find(write, name, grid)
        rd, wr = kf * 1024.0 * f_scale, kw * 1024.0 * w_scale
        doc["kernels"][key] = {"kernel": name, "grid_size": grid, "dispatches": [nf, nw], "fetch_kib": kf, "write_kib": kw,
                               "bytes_read": round(rd), "bytes_written": round(wr), "bytes": round(rd + wr),
                               "sources": files, "source_digest": source_digest(files)}
    with open(args.out, "w") as fh:
        json.dump(doc, fh, indent=1)
        fh.write("\n")
    print(json.dumps(doc, indent=1))


def lookup(key):
    """(bytes per launch or None, stale flag or None) for bench.py"""
    try:
        doc = json.load(open(OUT))
        k = doc["kernels"][key]
    except (OSError, KeyError, ValueError):
        return None, None
    return k["bytes"], k["source_digest"] != source_digest(k["sources"])


if __name__ == "__main__":
    main()
