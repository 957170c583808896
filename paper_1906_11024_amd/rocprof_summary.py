"""Turn rocprofv3 output of a bench.py run into the short text summaries kept
under profiles/.

  python -m paper_1906_11024_amd.rocprof_summary kernels  <results.db>
      per-kernel count / total / average / min / max duration (kernel-trace run)
  python -m paper_1906_11024_amd.rocprof_summary attention <results.db> --config base
      decode-attention launches split by role (block head / follower / enc-dec
      head) and by cache length n, with algorithmic GB/s
  python -m paper_1906_11024_amd.rocprof_summary pmc <counter_collection.csv> --copy-mib 512 --config base
      FETCH_SIZE or WRITE_SIZE per launch, scaled by the reading of the plain
      copy kernel of known size that bench.py --calib-copy-mb adds to the run

  python -m paper_1906_11024_amd.rocprof_summary mfma <counter_collection.csv> --dtype f32 [--trace <results.db>]
      matrix-core use of every GEMM shape: SQ_VALU_MFMA_BUSY_CYCLES (summed over the SIMDs)
      against GRBM_GUI_ACTIVE x 1024 SIMDs, and the flops the MFMA op counter saw
      (SQ_INSTS_VALU_MFMA_MOPS_* x 512) against the algorithmic 2 M N K where the shape is known

Only reads files; nothing here runs on the GPU.
"""
from __future__ import annotations

import argparse
import csv
import re
import sqlite3
import sys

from . import workloads as wl


def _short(name: str) -> str:
    name = re.sub(r"\(.*", "", name).replace("san::", "").replace("void ", "")
    return name[:58]


def kernels(db: str) -> None:
    cur = sqlite3.connect(db).cursor()
    rows = cur.execute(
        "select name, grid_x, grid_y, grid_z, workgroup_x, lds_size, vgpr_count, accum_vgpr_count, scratch_size,"
        " count(*), sum(duration), avg(duration), min(duration), max(duration)"
        " from kernels group by name, grid_x, grid_y, grid_z order by sum(duration) desc").fetchall()
    total = sum(r[10] for r in rows)
    print(f"total kernel time {total / 1e6:.3f} ms over {sum(r[9] for r in rows)} dispatches")
    print(f"{'kernel':58s} {'grid(threads)':>18s} {'wg':>5s} {'lds':>7s} {'vgpr':>7s} {'scr':>4s} {'calls':>6s} "
          f"{'total_us':>10s} {'avg_us':>8s} {'min_us':>8s} {'max_us':>8s} {'%':>5s}")
    for r in rows[:30]:
        grid = f"{r[1]}x{r[2]}x{r[3]}"
        print(f"{_short(r[0]):58s} {grid:>18s} {r[4]:5d} {r[5]:7d} {r[6]:4d}+{r[7]:<3d}{r[8]:4d} {r[9]:6d} "
              f"{r[10] / 1e3:10.1f} {r[11] / 1e3:8.2f} {r[12] / 1e3:8.2f} {r[13] / 1e3:8.2f} {100 * r[10] / total:5.1f}")


def _roles(cfg):
    """Order of the decode-attention launches inside one step."""
    heads_s, heads_c = [], []
    start = 0
    for p in cfg["self_pi"]:
        heads_s += [start] * p
        start += p
    start = 0
    for p in cfg["encdec_pi"]:
        heads_c += [start] * p
        start += p
    order = []
    for n in range(cfg["n_dec"]):
        if cfg["self_kind"] != "aan":
            order.append("head" if heads_s[n] == n else "apply")
        if heads_c[n] == n:
            order.append("ctx")
    return order


def attention(db: str, cfg_name: str) -> None:
    cfg = wl.get_config(cfg_name)
    order = _roles(cfg)
    T, B, d = cfg["steps"], cfg["batch"] * cfg["beam"], cfg["d"]
    esz = 2 if cfg["dtype"] == "bf16" else 4
    cur = sqlite3.connect(db).cursor()
    # every attention launch in start order: the encoder's n_enc launches come first (bench.py encodes once
    # and rewinds), then `per` launches per decode step; the run ends on a decode boundary
    durs = [r[0] for r in cur.execute("select duration from kernels where name like '%attention_kernel%' order by start")]
    per = len(order)
    ndec = (len(durs) - cfg["n_enc"]) // (T * per)
    durs = durs[len(durs) - ndec * T * per:]                     # whole decodes only, from the end
    acc = {r: [[0.0, 0] for _ in range(T)] for r in set(order)}
    for i, dur in enumerate(durs):
        t = (i // per) % T
        a = acc[order[i % per]][t]
        a[0] += dur
        a[1] += 1
    print(f"{cfg_name}: {ndec} decode(s) of {T} steps, {per} attention launches per step: {order}")
    print("role   n   avg_us   algorithmic_MB   GB/s")
    for role in ("head", "apply"):
        if role not in acc:
            continue
        mult = 2 if role == "head" else 1
        tot_b = tot_t = 0.0
        for t in list(range(0, T, max(1, T // 8))) + [T - 1]:
            s, c = acc[role][t]
            nb = mult * B * (t + 1) * d * esz
            print(f"{role:6s} {t + 1:3d} {s / c / 1e3:8.2f} {nb / 1e6:12.2f} {nb / (s / c):10.1f}")
        for t in range(T):
            s, c = acc[role][t]
            tot_b += mult * B * (t + 1) * d * esz
            tot_t += s / c
        print(f"{role:6s} all steps: avg {tot_t / T / 1e3:.2f} us per launch, {tot_b / T / 1e6:.2f} MB per launch, "
              f"{tot_b / tot_t:.1f} GB/s = {tot_b / tot_t / 8000:.3f} of 8 TB/s")
    if "ctx" in acc:
        s = sum(a[0] for a in acc["ctx"])
        c = sum(a[1] for a in acc["ctx"])
        print(f"ctx    all steps: avg {s / c / 1e3:.2f} us per launch")


def pmc(path: str, copy_mib: int, cfg_name: str) -> None:
    cfg = wl.get_config(cfg_name)
    order = _roles(cfg)
    rows = sorted(csv.DictReader(open(path)), key=lambda r: int(r["Dispatch_Id"]))
    counter = rows[0]["Counter_Name"]
    copies = [float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]
              and float(r["Counter_Value"]) > copy_mib * 1024 * 0.2]
    if not copies:
        sys.exit("no calibration copy found (run bench.py with --calib-copy-mb)")
    factor = copy_mib * 1024.0 / copies[-1]
    print(f"{counter}: copy kernel of {copy_mib} MiB read back as {copies[-1]:.0f} KiB -> scale factor {factor:.3f}")
    att = [float(r["Counter_Value"]) for r in rows if "attention_kernel" in r["Kernel_Name"]]
    per, T = len(order), cfg["steps"]
    att = att[len(att) - T * per:]
    sums = {}
    for i, v in enumerate(att):
        sums.setdefault(order[i % per], []).append(v)
    for role, vals in sums.items():
        kib = sum(vals) / len(vals)
        print(f"attention {role:6s}: {kib:10.1f} KiB raw per launch -> {kib * factor * 1024 / 1e6:8.2f} MB per launch")
    agg = {}
    for r in rows:
        agg.setdefault(_short(r["Kernel_Name"]) + " g" + r["Grid_Size"], []).append(float(r["Counter_Value"]))
    print("per kernel (scaled MB per launch):")
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1]))[:12]:
        print(f"  {k:70s} n={len(v):5d} {sum(v) / len(v) * factor * 1024 / 1e6:10.2f}")


def mfma(path: str, dtype: str) -> None:
    """Per GEMM shape (kernel name + grid): MFMA-busy cycles summed over all SIMDs
    (SQ_VALU_MFMA_BUSY_CYCLES; a 32x32x2 fp32 MFMA holds the pipe 64 cycles = its 4096 flops at
    the 64 flops/cycle/SIMD behind the 157.3 TFLOP/s peak, so busy cycles / (SIMDs x cycles) IS
    the fraction of the dense peak), set against
      - the dispatch's own GPU-active cycles: GRBM_GUI_ACTIVE, which the CSV holds summed over the
        8 XCDs, hence /8 (the profiler's MfmaUtil expression takes the max over XCDs instead);
      - the dispatch's duration in this run (End - Start time stamps) at 2.4 GHz.
    Kernels run slower while counters are collected (each dispatch is serialised), so both are
    lower bounds of the utilisation in a normal run; the flops the MFMA op counter saw
    (MOPS x 512) are printed to be checked against the algorithmic 2 M N K."""
    simds, xcds, ghz = 256 * 4, 8, 2.4
    rows = list(csv.DictReader(open(path)))
    per = {}
    for r in rows:
        if "gemm_kernel" not in r["Kernel_Name"]:
            continue
        key = (_short(r["Kernel_Name"]), r["Grid_Size"])
        d = per.setdefault(key, {})
        d.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
        if r["Counter_Name"] == "GRBM_GUI_ACTIVE":
            d.setdefault("dur_ns", []).append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
    mops_name = "SQ_INSTS_VALU_MFMA_MOPS_BF16" if dtype == "bf16" else "SQ_INSTS_VALU_MFMA_MOPS_F32"
    peak = 2500.0 if dtype == "bf16" else 157.3
    print(f"{'kernel':50s} {'grid':>8s} {'calls':>5s} {'GFLOP':>8s} {'mfma_busy_cyc':>14s} {'active_cyc/XCD':>15s} {'dur_us':>8s} "
          f"{'util(active)':>13s} {'util(dur)':>10s} {'TFLOP/s(dur)':>13s}")
    for (name, grid), d in sorted(per.items(), key=lambda kv: -sum(kv[1].get("dur_ns", [0]))):
        busy, act, mops, dur = (d.get(k, []) for k in ("SQ_VALU_MFMA_BUSY_CYCLES", "GRBM_GUI_ACTIVE", mops_name, "dur_ns"))
        if not busy or not act or not dur:
            continue
        b, a, t = sum(busy) / len(busy), sum(act) / len(act) / xcds, sum(dur) / len(dur)
        gf = (sum(mops) / len(mops)) * 512 / 1e9 if mops else float("nan")
        print(f"{name:50s} {grid:>8s} {len(busy):5d} {gf:8.3f} {b:14.0f} {a:15.0f} {t / 1e3:8.2f} {b / (a * simds):13.3f} "
              f"{b / (t * ghz * simds):10.3f} {gf / t * 1e6:13.1f}")
    print(f"(dense peak for {dtype}: {peak} TFLOP/s; util = MFMA-busy cycles / (1024 SIMDs x cycles of the dispatch))")


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("mode", choices=["kernels", "attention", "pmc", "mfma"])
    ap.add_argument("--dtype", default="f32")
    ap.add_argument("path")
    ap.add_argument("--config", default="base")
    ap.add_argument("--copy-mib", type=int, default=512)
    a = ap.parse_args()
    if a.mode == "kernels":
        kernels(a.path)
    elif a.mode == "attention":
        attention(a.path, a.config)
    elif a.mode == "mfma":
        mfma(a.path, a.dtype)
    else:
        pmc(a.path, a.copy_mib, a.config)


if __name__ == "__main__":
    main()
