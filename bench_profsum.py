"""Condense rocprofv3 CSV output of a bench.py run into the short text tables kept under profiles/.

    python bench_profsum.py stats  <dir with *_kernel_stats.csv>
    python bench_profsum.py traffic <FETCH_SIZE dir> <WRITE_SIZE dir>
    python bench_profsum.py mfma    <dir of a --pmc SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE --kernel-trace run>

`traffic` scales the FETCH_SIZE / WRITE_SIZE counters (KiB per dispatch as rocprofv3 reports them) by
what the same counters read for the 1 GiB device-to-device copy that `bench.py --copy-calibration`
runs, whose traffic is known (1 GiB read, 1 GiB written).
"""
from __future__ import annotations

import collections
import csv
import glob
import sys


def short(name: str) -> str:
    name = name.replace("void ", "").replace("(anonymous namespace)::", "")
    cut = name.find("(")
    if cut > 0:
        name = name[:cut]
    return name if len(name) <= 70 else name[:67] + "..."


def stats(d: str) -> None:
    f = glob.glob(d + "/*kernel_stats.csv")[0]
    rows = list(csv.DictReader(open(f)))
    total = sum(int(r["TotalDurationNs"]) for r in rows)
    print(f"{'kernel':70s} {'calls':>7s} {'total ms':>10s} {'avg us':>9s} {'min us':>9s} {'max us':>9s} {'%':>6s}")
    gemm_calls = gemm_ns = 0
    for r in rows:
        t = int(r["TotalDurationNs"])
        if t < 0.002 * total:
            continue
        print(f"{short(r['Name']):70s} {int(r['Calls']):7d} {t / 1e6:10.3f} {float(r['AverageNs']) / 1e3:9.2f} "
              f"{int(r['MinNs']) / 1e3:9.2f} {int(r['MaxNs']) / 1e3:9.2f} {100.0 * t / total:6.2f}")
        if "gemm_bf16_kernel" in r["Name"]:
            gemm_calls += int(r["Calls"])
            gemm_ns += t
    if gemm_calls:
        print(f"\nall gemm_bf16_kernel instances: {gemm_calls} launches, {gemm_ns / 1e6:.3f} ms, "
              f"average {gemm_ns / gemm_calls / 1e3:.2f} us per launch")


def per_kernel(d: str, counter: str):
    f = glob.glob(d + "/*counter_collection.csv")[0]
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(f)):
        if r["Counter_Name"] == counter:
            acc[(short(r["Kernel_Name"]), int(r["Grid_Size"]))].append(float(r["Counter_Value"]))
    return acc


def traffic(dfetch: str, dwrite: str) -> None:
    fe, wr = per_kernel(dfetch, "FETCH_SIZE"), per_kernel(dwrite, "WRITE_SIZE")
    GIB_KIB = float(1 << 20)
    # the calibration copy is the largest __amd_rocclr_copyBuffer dispatch of the run (a same-dtype
    # tensor copy is a runtime device-to-device copy)
    def cal(acc):
        vs = [v for (n, g), vals in acc.items() if "copyBuffer" in n for v in vals]
        top = max(vs) if vs else 0.0
        return [v for v in vs if v > 0.9 * top] if top > 0 else []
    cal_f, cal_w = cal(fe), cal(wr)
    if not cal_f or not cal_w:
        print("no 1 GiB copy dispatch found: run bench.py with --copy-calibration")
        return
    sf, sw = GIB_KIB / (sum(cal_f) / len(cal_f)), GIB_KIB / (sum(cal_w) / len(cal_w))
    print(f"calibration: 1 GiB copy reads FETCH_SIZE={sum(cal_f) / len(cal_f):.0f} KiB, WRITE_SIZE={sum(cal_w) / len(cal_w):.0f} KiB "
          f"-> scale factors {sf:.4f} (fetch), {sw:.4f} (write)")
    print(f"{'kernel':70s} {'grid':>10s} {'n':>5s} {'fetch MB':>10s} {'write MB':>10s}   (per dispatch, scaled)")
    for key in sorted(fe, key=lambda k: -sum(fe[k])):
        n, g = key
        if n.startswith("at::") or "rocclr" in n or n.startswith("pack_rows") or n.startswith("kv_ingest"):
            continue  # set-up work of the benchmark script (weight generation, loading, context upload)
        f_mb = sum(fe[key]) / len(fe[key]) * sf * 1024 / 1e6
        w_mb = (sum(wr[key]) / len(wr[key]) * sw * 1024 / 1e6) if key in wr else float("nan")
        if f_mb + (w_mb if w_mb == w_mb else 0) < 1.0:
            continue
        print(f"{n:70s} {g:10d} {len(fe[key]):5d} {f_mb:10.2f} {w_mb:10.2f}")


def mfma(d: str) -> None:
    """MFMA pipe occupancy of the projection kernels: SQ_VALU_MFMA_BUSY_CYCLES (summed over all SIMDs) over the SIMD
    cycles of the dispatch, GRBM_GUI_ACTIVE (summed over the 8 XCDs) / 8 x 256 CUs x 4 SIMDs; and the shader clock
    that GRBM_GUI_ACTIVE implies for the dispatch's duration."""
    busy, act = per_kernel(d, "SQ_VALU_MFMA_BUSY_CYCLES"), per_kernel(d, "GRBM_GUI_ACTIVE")
    dur = collections.defaultdict(list)
    for r in csv.DictReader(open(glob.glob(d + "/*kernel_trace.csv")[0])):
        grid = int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"])
        dur[(short(r["Kernel_Name"]), grid)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    print(f"{'kernel':40s} {'grid':>9s} {'n':>5s} {'avg us':>9s} {'MFMA busy':>10s} {'clock GHz':>10s}")
    for key in sorted(busy, key=lambda k: -sum(busy[k])):
        if "gemm_bf16" not in key[0] or key not in act or key not in dur:
            continue
        b, a, t = sum(busy[key]) / len(busy[key]), sum(act[key]) / len(act[key]), sum(dur[key]) / len(dur[key])
        print(f"{key[0]:40s} {key[1]:9d} {len(busy[key]):5d} {t:9.1f} {b / (a / 8 * 1024):10.3f} {a / 8 / (t * 1e3):10.2f}")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 4 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3])
    elif len(sys.argv) >= 3 and sys.argv[1] == "mfma":
        mfma(sys.argv[2])
    else:
        print(__doc__)
        sys.exit(2)
