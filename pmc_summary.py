"""HBM traffic per kernel class and training step from rocprofv3 counter runs.

    python pmc_summary.py <dir>
    python pmc_summary.py --by-kernel <dir>     (any workload; no calibration runs needed:
                                                 FETCH_SIZE x 2, WRITE_SIZE x 1 as calibrated)
    python pmc_summary.py --l1-latency <dir>    (<dir> = one rocprofv3 --pmc output with the vector-L1 counters
                                                 TCP_TCC_READ_REQ_sum TCP_TCC_READ_REQ_LATENCY_sum
                                                 TCP_PENDING_STALL_CYCLES_sum GRBM_GUI_ACTIVE)

<dir> holds four rocprofv3 --pmc outputs (csv), one counter each:
    bench_FETCH_SIZE/ bench_WRITE_SIZE/   python3 bench.py --steps 40 --warmup 10 --no-cpu-baseline
    copy_FETCH_SIZE/  copy_WRITE_SIZE/    python3 bench.py --workload copy-calibration --steps 10
and optionally bench_MFMA/ (--pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE,
the same bench command): matrix-core busy cycles of the matrix products against the cycles
the device was active during them.
The counters are in KiB per dispatch.  They are scaled by what the same counter reads for the
plain copy kernel (1 GiB read and 1 GiB written per launch): on this machine FETCH_SIZE reads
half the bytes actually fetched.  Dispatches are walked in order; a step starts at the pooling
kernel, matrix products before the loss kernel are the forward pass, those after it the
data-gradient chain (gemm_bwd) and the per-shard weight gradients (gemm_wgrad).  The first five
steps are dropped.
"""
import collections
import csv
import glob
import sys


def _rows(d, counter=None):
    path = glob.glob(f"{d}/**/*counter_collection.csv", recursive=True)[0]
    rows = [r for r in csv.DictReader(open(path)) if counter is None or r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def class_totals(rows):
    out, cur, after_head = collections.defaultdict(list), None, False
    for r in rows:
        k, v = r["Kernel_Name"], float(r["Counter_Value"])
        if "pool_tile" in k or "pool_kernel" in k:
            if cur is not None:
                for c, x in cur.items():
                    out[c].append(x)
            cur, after_head, cls = collections.defaultdict(float), False, "pool"
        elif cur is None:
            continue
        elif "head_tile" in k or "head_kernel" in k:
            after_head, cls = True, "head"
        elif "head_reduce" in k:
            cls = "head_reduce"
        elif "wgrad_update" in k:
            cls = "wgrad_adagrad"
        elif "transpose" in k:
            cls = "transpose"
        elif "gemm_" in k:  # the grouped instantiations (last template argument true) are the weight gradients
            cls = "gemm_fwd" if not after_head else ("gemm_wgrad" if "true>" in k else "gemm_bwd")
        elif "seg_reduce" in k:
            cls = "sparse_adagrad"
        elif "seg_chunk" in k or "seg_finish" in k:
            cls = "seg_reduce_long"
        elif "dense_adagrad" in k:
            cls = "dense_adagrad"
        elif "sort_" in k:
            cls = "sort"
        elif "seg_" in k:
            cls = "segments"
        else:
            cls = "other"
        cur[cls] += v
    return {c: sum(x[5:]) / max(len(x[5:]), 1) for c, x in out.items()}


def main(d):
    fs = float(_rows(f"{d}/copy_FETCH_SIZE")[-1]["Counter_Value"])
    ws = float(_rows(f"{d}/copy_WRITE_SIZE")[-1]["Counter_Value"])
    fscale, wscale = 1048576.0 / fs, 1048576.0 / ws
    print(f"copy kernel (1048576 KiB read, 1048576 KiB written): FETCH_SIZE {fs:.0f}, WRITE_SIZE {ws:.0f} "
          f"-> scale factors {fscale:.3f} (fetch), {wscale:.3f} (write)")
    f = class_totals(_rows(f"{d}/bench_FETCH_SIZE"))
    w = class_totals(_rows(f"{d}/bench_WRITE_SIZE"))
    print(f"{'class':18s} {'fetched MB':>11s} {'written MB':>11s} {'total MB':>10s}   per step, scaled")
    for c in sorted(f):
        fm, wm = f[c] * fscale * 1024 / 1e6, w.get(c, 0.0) * wscale * 1024 / 1e6
        print(f"{c:18s} {fm:11.1f} {wm:11.1f} {fm + wm:10.1f}")


    if glob.glob(f"{d}/bench_MFMA"):
        mfma_summary(f"{d}/bench_MFMA")


def mfma_summary(d, simds=1024, xcds=8):
    """Matrix-core utilisation of the matrix-product classes: busy cycles summed over the SIMDs,
    divided by (cycles the device was active in those dispatches x number of SIMDs); and the
    flops the counters saw (512 per counted operation).  The active-cycle counter is reported
    summed over the device's XCDs (one instance each), so it is divided by their number."""
    busy = class_totals(_rows(d, "SQ_VALU_MFMA_BUSY_CYCLES"))
    mops = class_totals(_rows(d, "SQ_INSTS_VALU_MFMA_MOPS_BF16"))
    act = class_totals(_rows(d, "GRBM_GUI_ACTIVE"))
    print(f"{'class':18s} {'MFMA busy cycles':>17s} {'active cycles':>14s} {'utilisation':>12s} {'GFLOP counted':>14s}   per step")
    for c in sorted(busy):
        if not c.startswith("gemm"):
            continue
        active = act.get(c, 0.0) / xcds
        util = busy[c] / max(active * simds, 1.0)
        print(f"{c:18s} {busy[c]:17.0f} {active:14.0f} {100 * util:11.1f}% {mops.get(c, 0.0) * 512 / 1e9:14.2f}")


def by_kernel(d, fscale=2.0, wscale=1.0):
    """MB per launch of every kernel, from <d>/bench_FETCH_SIZE and <d>/bench_WRITE_SIZE."""
    tot = collections.defaultdict(lambda: [0, 0.0, 0.0])
    for sub, idx, scale in (("bench_FETCH_SIZE", 1, fscale), ("bench_WRITE_SIZE", 2, wscale)):
        for r in _rows(f"{d}/{sub}"):
            k = r["Kernel_Name"].replace("antdt::(anonymous namespace)::", "").replace("antdt::", "").replace("void ", "")
            if idx == 1:
                tot[k][0] += 1
            tot[k][idx] += float(r["Counter_Value"]) * scale * 1024 / 1e6
    print(f"{'kernel':72s} {'launches':>8s} {'fetched MB':>11s} {'written MB':>11s}   per launch")
    for k, (n, f, w) in sorted(tot.items(), key=lambda kv: -(kv[1][1] + kv[1][2])):
        if n and (f + w) / n >= 1.0 and "at::native" not in k and "fill_tables" not in k:
            print(f"{k[:72]:72s} {n:8d} {f / n:11.1f} {w / n:11.1f}")


def l1_latency(d):
    """Per kernel: vector-L1 read requests to L2 per launch and their mean latency in cycles, from a run with
    --pmc TCP_TCC_READ_REQ_sum TCP_TCC_READ_REQ_LATENCY_sum TCP_PENDING_STALL_CYCLES_sum GRBM_GUI_ACTIVE."""
    tot = collections.defaultdict(lambda: collections.defaultdict(float))
    n = collections.defaultdict(int)
    for r in _rows(d):
        k = r["Kernel_Name"].replace("antdt::(anonymous namespace)::", "").replace("antdt::", "").replace("void ", "")
        tot[k][r["Counter_Name"]] += float(r["Counter_Value"])
        if r["Counter_Name"] == "TCP_TCC_READ_REQ_sum":
            n[k] += 1
    print(f"{'kernel':64s} {'launches':>8s} {'L1->L2 reads':>13s} {'mean latency':>13s} {'pending stall':>14s} {'active':>10s}   per launch")
    for k, c in sorted(tot.items(), key=lambda kv: -kv[1].get("TCP_TCC_READ_REQ_sum", 0.0)):
        if not n[k] or "at::native" in k or "fill_tables" in k:
            continue
        req = c.get("TCP_TCC_READ_REQ_sum", 0.0)
        if req / n[k] < 1000:
            continue
        print(f"{k[:64]:64s} {n[k]:8d} {req / n[k]:13.0f} {c.get('TCP_TCC_READ_REQ_LATENCY_sum', 0.0) / max(req, 1):13.0f} "
              f"{c.get('TCP_PENDING_STALL_CYCLES_sum', 0.0) / n[k]:14.0f} {c.get('GRBM_GUI_ACTIVE', 0.0) / n[k] / 8:10.0f}")


if __name__ == "__main__":
    if sys.argv[1] == "--by-kernel":
        by_kernel(sys.argv[2])
    elif sys.argv[1] == "--l1-latency":
        l1_latency(sys.argv[2])
    else:
        main(sys.argv[1])
