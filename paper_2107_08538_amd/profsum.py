"""Turns rocprofv3 CSV output into the short tables kept under profiles/, and reads them back.

Three tables:
  * kernel statistics of a `--kernel-trace --stats` run (calls, total / average / min / max time);
  * HBM-side bytes per launch from two `--pmc` runs (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch),
    each scaled by what the same counter reads for the bench's plain copy kernel of known size, with
    the hash of each kernel's source file beside it: a figure is only valid for the kernel it was
    measured on, and bench.py drops it (traffic = null) once the source has changed;
  * which kernels overlapped in time on which CU partitions, from a `--kernel-trace` run of a mix
    with MGB_TAG_PARTITIONS set (start / end timestamps per dispatch; a tag dispatch in front of
    every task names its partition), and derived counters per kernel and partition size.

Usage:  python -m paper_2107_08538_amd.profsum stats   <kernel_stats.csv>
        python -m paper_2107_08538_amd.profsum traffic <fetch_counter_collection.csv> <write_counter_collection.csv>
        python -m paper_2107_08538_amd.profsum overlap <kernel_trace.csv> [<tasks per pass> [<fetch csv> <write csv>]]
        python -m paper_2107_08538_amd.profsum utilisation <MfmaUtil csv> <VALUBusy csv> <MeanOccupancyPerActiveCU csv>
        python -m paper_2107_08538_amd.profsum gaps <kernel_trace.csv> <tasks per pass>
        python -m paper_2107_08538_amd.profsum counters <counter_collection.csv> <Counter1,Counter2>
Each prints markdown on stdout."""
import csv
import hashlib
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")

SOURCE_OF = (("gemm_f32", "gemm_f32.hip"), ("gemm_bf16", "gemm_bf16.hip"), ("jacobi", "jacobi.hip"), ("bfs", "bfs.hip"),
             ("conv", "conv3x3.hip"), ("stream_copy", "cu_trace.hip"), ("mfma_loop", "cu_trace.hip"),
             ("fetch_rate", "cu_trace.hip"), ("lds_read_rate", "cu_trace.hip"))


def source_hash(kernel_name):
    """First 16 hex digits of the SHA-256 of the source file that defines the kernel followed by the
    device headers of csrc/ it may include ('' if unknown)."""
    for frag, src in SOURCE_OF:
        if frag in kernel_name:
            h = hashlib.sha256()
            for name in [src] + sorted(n for n in os.listdir(CSRC) if n.endswith(".h")):
                with open(os.path.join(CSRC, name), "rb") as f:
                    h.update(f.read())
            return h.hexdigest()[:16]
    return ""


def short(name):
    name = name.replace("void ", "").replace("(anonymous namespace)::", "")
    return name.split("(")[0] if not name.startswith("at::") else name[:60]


def stats_md(path, keep=14):
    rows = list(csv.DictReader(open(path)))
    out = ["| kernel | calls | total us | avg us | min us | max us | % |", "|---|---|---|---|---|---|---|"]
    for r in rows[:keep]:
        out.append("| %s | %s | %.1f | %.2f | %.2f | %.2f | %s |" % (
            short(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e3, float(r["AverageNs"]) / 1e3,
            float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, r["Percentage"]))
    return "\n".join(out)


def _pmc(path, counter):
    agg = {}
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        agg.setdefault(short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    return agg


def traffic_md(fetch_csv, write_csv, copy_bytes=1 << 30):
    """Per kernel: mean FETCH_SIZE / WRITE_SIZE per dispatch, scaled so that the copy kernel reads
    and writes exactly copy_bytes."""
    f, w = _pmc(fetch_csv, "FETCH_SIZE"), _pmc(write_csv, "WRITE_SIZE")
    mean = lambda v: sum(v) / len(v)
    copy = [k for k in f if "stream_copy" in k]
    assert copy, "the run must contain the bench's copy kernel (calibration point)"
    sf = copy_bytes / 1024.0 / mean(f[copy[0]])
    sw = copy_bytes / 1024.0 / mean(w[copy[0]])
    out = ["Calibration: `stream_copy_kernel` copies %d bytes; FETCH_SIZE reads %.1f KiB for it -> scale %.4f; "
           "WRITE_SIZE reads %.1f KiB -> scale %.4f." % (copy_bytes, mean(f[copy[0]]), sf, mean(w[copy[0]]), sw), "",
           "| kernel | launches | FETCH_SIZE KiB (raw mean) | WRITE_SIZE KiB (raw mean) | read MB | write MB | total bytes per launch | source sha256/16 |",
           "|---|---|---|---|---|---|---|---|"]
    for k in sorted(f):
        if k not in w or k.startswith("at::") or "rocclr" in k:
            continue
        rb, wb = mean(f[k]) * 1024 * sf, mean(w[k]) * 1024 * sw
        out.append("| %s | %d | %.1f | %.1f | %.1f | %.1f | %d | %s |" % (k, len(f[k]), mean(f[k]), mean(w[k]), rb / 1e6, wb / 1e6,
                                                                    round(rb + wb), source_hash(k)))
    return "\n".join(out)


def read_traffic(md_path):
    """{kernel name as in the table: (bytes per launch, launches, source hash)} from a traffic table."""
    out = {}
    if not os.path.exists(md_path):
        return out
    for line in open(md_path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) == 8 and re.fullmatch(r"\d+", cells[6] or "x") and re.fullmatch(r"[0-9a-f]{16}", cells[7] or "x"):
            out[cells[0]] = (int(cells[6]), int(cells[1]), cells[7])
    return out


def traffic_for(md_path, kernel_fragment):
    """Launch-weighted mean bytes per launch over the table rows whose name contains the fragment,
    or None if there is no such row or a row's kernel source has changed since it was measured."""
    rows = [(k, v) for k, v in read_traffic(md_path).items() if kernel_fragment in k]
    if not rows or any(v[2] != source_hash(k) for k, v in rows):
        return None
    n = sum(v[1] for _, v in rows)
    return sum(v[0] * v[1] for _, v in rows) / n


UTIL_COUNTERS = ("MfmaUtil", "VALUBusy", "MeanOccupancyPerActiveCU")


def utilisation_md(csv_by_counter):
    """Per kernel: mean over its dispatches of MfmaUtil (share of cycles the matrix pipes are busy, per
    cent), VALUBusy (the same for the vector units) and MeanOccupancyPerActiveCU, one --pmc run each
    ({counter: counter_collection.csv}); with the kernel's source hash, like the traffic table."""
    agg = {c: _pmc(path, c) for c, path in csv_by_counter.items()}
    mean = lambda v: sum(v) / len(v)
    kernels = sorted({k for a in agg.values() for k in a if not k.startswith("at::") and "rocclr" not in k})
    out = ["| kernel | dispatches | " + " | ".join(UTIL_COUNTERS) + " | source sha256/16 (utilisation) |", "|---|---|" + "---|" * (len(UTIL_COUNTERS) + 1)]
    for k in kernels:
        n = max(len(agg[c].get(k, [])) for c in agg)
        cells = ["%.2f" % mean(agg[c][k]) if c in agg and k in agg[c] else "" for c in UTIL_COUNTERS]
        out.append("| %s | %d | %s | %s |" % (k, n, " | ".join(cells), source_hash(k)))
    return "\n".join(out)


def utilisation_for(md_path, kernel_fragment, counter):
    """Dispatch-weighted mean of a counter of utilisation_md's table over the rows whose kernel name
    contains the fragment; None if there is none or the kernel's source has changed since."""
    col = 2 + UTIL_COUNTERS.index(counter)
    tot = n = 0.0
    if not os.path.exists(md_path):
        return None
    for line in open(md_path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) != 3 + len(UTIL_COUNTERS) or kernel_fragment not in cells[0] or not re.fullmatch(r"[0-9a-f]{16}", cells[-1] or "x"):
            continue
        if cells[-1] != source_hash(cells[0]) or not cells[col]:
            return None
        tot += float(cells[col]) * int(cells[1])
        n += int(cells[1])
    return tot / n if n else None


def _tag_of(name, threads):
    """(first granule, number of granules) if the dispatch is a partition tag, else None."""
    if "partition_tag_kernel" not in name:
        return None
    v = threads // 64
    return v // 64, v % 64


def _trace_rows(trace_csv):
    """[(start ns, end ns, kernel, queue, threads)] of a --kernel-trace CSV, library kernels only."""
    rows = []
    for r in csv.DictReader(open(trace_csv)):
        name = short(r["Kernel_Name"])
        if name.startswith("at::") or "rocclr" in name:
            continue
        threads = int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1) * int(r.get("Grid_Size_Z", 1) or 1)
        rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), name, int(r["Queue_Id"]), threads))
    rows.sort()
    return rows


def _last_pass_bytes(counter_csv, counter, n_tasks, copy_bytes=1 << 30):
    """Sum of a traffic counter (KiB per dispatch, scaled by the copy kernel's reading) over the
    library's dispatches that follow the n_tasks-th last partition tag."""
    rows = [r for r in csv.DictReader(open(counter_csv)) if r["Counter_Name"] == counter]
    copy = [float(r["Counter_Value"]) for r in rows if "stream_copy" in r["Kernel_Name"]]
    scale = copy_bytes / 1024.0 / (sum(copy) / len(copy))
    tags = [i for i, r in enumerate(rows) if "partition_tag_kernel" in r["Kernel_Name"]]
    first = tags[-n_tasks] if len(tags) >= n_tasks else 0
    total = 0.0
    for r in rows[first:]:
        name = short(r["Kernel_Name"])
        if name.startswith("at::") or "rocclr" in name or "partition_tag" in name:
            continue
        total += float(r["Counter_Value"]) * 1024.0 * scale
    return total, scale


def overlap_md(trace_csv, n_tasks=None, fetch_csv=None, write_csv=None, granule_cus=32, keep=30):
    """Which kernels ran at the same time on which partitions, from a kernel trace of a run with
    MGB_TAG_PARTITIONS set: every task's kernels follow, on their queue, a tag dispatch that names
    the task's granules.  Reports (over the last pass of the mix, i.e. after the last long gap)
    how many CUs were held by running kernels over time, busy time per partition, and the pairs
    of kernels on different partitions whose [start, end) intervals intersect."""
    rows = _trace_rows(trace_csv)
    # every dispatch belongs to the partition of the last tag seen on its queue; the last pass of
    # the mix starts with the n_tasks-th last tag
    tag_starts = [s for s, e, name, q, threads in rows if _tag_of(name, threads) is not None]
    begin = tag_starts[-n_tasks] if n_tasks and len(tag_starts) >= n_tasks else 0
    part_of_queue, tagged = {}, []
    for s, e, name, q, threads in rows:
        tag = _tag_of(name, threads)
        if tag is not None:
            part_of_queue[q] = tag
        elif q in part_of_queue and s >= begin:
            tagged.append((s, e, name, part_of_queue[q]))
    if not tagged:
        return "no tagged dispatches in the trace (was MGB_TAG_PARTITIONS set?)"
    t0, t1 = tagged[0][0], max(t[1] for t in tagged)
    span = t1 - t0
    mask = lambda p: "%d-%d" % (p[0] * granule_cus, (p[0] + p[1]) * granule_cus - 1)
    # CUs held by running kernels over time
    ev = sorted([(s, p[1] * granule_cus, 1) for s, e, n, p in tagged] + [(e, -p[1] * granule_cus, -1) for s, e, n, p in tagged])
    cus = disp = 0
    last = t0
    cu_time, hist = 0.0, {}
    for t, dc, dd in ev:
        cu_time += cus * (t - last)
        hist[disp] = hist.get(disp, 0) + (t - last)
        cus += dc
        disp += dd
        last = t
    out = ["Traced pass: %d kernel dispatches on %d different partitions in %.3f ms; CUs held by a running kernel, averaged over the pass: %.1f of 256."
           % (len(tagged), len({p for *_, p in tagged}), span / 1e6, cu_time / span), ""]
    if fetch_csv and write_csv and n_tasks:
        rd, sf = _last_pass_bytes(fetch_csv, "FETCH_SIZE", n_tasks)
        wr, sw = _last_pass_bytes(write_csv, "WRITE_SIZE", n_tasks)
        out += ["HBM-side bytes of the same pass from the counter runs (FETCH_SIZE x %.4f + WRITE_SIZE x %.4f, the factors the 1 GiB copy kernel gives; "
                "counter collection runs one dispatch at a time, so the bytes are per kernel and the time is the un-instrumented pass above): "
                "%.1f MB read + %.1f MB written = %.1f GB/s over the pass = %.1f %% of 8 TB/s." % (sf, sw, rd / 1e6, wr / 1e6, (rd + wr) / span, 100.0 * (rd + wr) / span / 8000.0), ""]
    out += [
           "| kernels running at once | time us | share of the pass |", "|---|---|---|"]
    for k in sorted(hist):
        if hist[k]:
            out.append("| %d | %.1f | %.1f %% |" % (k, hist[k] / 1e3, 100.0 * hist[k] / span))
    per = {}
    for s, e, n, p in tagged:
        a = per.setdefault(p, [0, 0, set()])
        a[0] += 1
        a[1] += e - s
        a[2].add(n.split("<")[0])
    out += ["", "| partition (CU-mask bits) | CUs | dispatches | kernel time us | busy share of the pass | kernels |", "|---|---|---|---|---|---|"]
    for p in sorted(per):
        a = per[p]
        out.append("| %s | %d | %d | %.1f | %.1f %% | %s |" % (mask(p), p[1] * granule_cus, a[0], a[1] / 1e3, 100.0 * a[1] / span,
                                                         ", ".join(sorted(a[2]))))
    pairs = {}
    active = []
    for s, e, n, p in tagged:
        active = [a for a in active if a[1] > s]
        for a in active:
            if a[3] != p:
                ka, kb = (a[2].split("<")[0], a[3]), (n.split("<")[0], p)
                lo, hi = sorted((ka, kb))
                q = pairs.setdefault((lo, hi), [0, 0, None])
                q[0] += 1
                q[1] += min(a[1], e) - s
                if q[2] is None:
                    ia, ib = (a[0] - t0, a[1] - t0), (s - t0, e - t0)
                    q[2] = ia + ib if ka == lo else ib + ia
        active.append((s, e, n, p))
    overlapping_partitions_disjoint = all(
        k[0][1][0] + k[0][1][1] <= k[1][1][0] or k[1][1][0] + k[1][1][1] <= k[0][1][0] for k in pairs)
    out += ["", "Pairs of kernels on different partitions that overlapped in time (%d distinct pairs; every such pair of partitions is disjoint: %s).  "
            "Example = the first such pair of dispatches, [start, end) in us from the start of the pass:" % (len(pairs), overlapping_partitions_disjoint), "",
            "| kernel A | CUs of A | kernel B | CUs of B | overlapping dispatch pairs | total overlap us | example A | example B |", "|---|---|---|---|---|---|---|---|"]
    for (a, b), (cnt, ov, ex) in sorted(pairs.items(), key=lambda kv: -kv[1][1])[:keep]:
        out.append("| %s | %s | %s | %s | %d | %.1f | [%.1f, %.1f) | [%.1f, %.1f) |" % (a[0], mask(a[1]), b[0], mask(b[1]), cnt, ov / 1e3,
                                                                                 ex[0] / 1e3, ex[1] / 1e3, ex[2] / 1e3, ex[3] / 1e3))
    return "\n".join(out)


def gaps_md(trace_csv, n_tasks):
    """Where the device idles inside the last pass of a mix (run with MGB_TAG_PARTITIONS): every
    interval during which no kernel runs, attributed to the kernel that ended before it and the one
    that starts after it; a tag dispatch marks the first kernel of a task."""
    rows = _trace_rows(trace_csv)
    tag_starts = [s for s, e, name, q, threads in rows if _tag_of(name, threads) is not None]
    begin = tag_starts[-n_tasks] if len(tag_starts) >= n_tasks else 0
    rows = [r for r in rows if r[0] >= begin]
    work = [(s, e, n.split("<")[0]) for s, e, n, q, th in rows]
    busy = sum(e - s for s, e, n in work if "partition_tag" not in n)
    t0, t1 = work[0][0], max(e for s, e, n in work)
    kinds = {}
    end, prev, after_tag = work[0][1], work[0][2], False
    for s, e, n in work[1:]:
        if "partition_tag" in n:
            after_tag = True
        if s > end:
            what = "between two tasks (%s -> %s)" % (prev, "next task") if after_tag or "partition_tag" in n else \
                   "inside a task (%s -> %s)" % (prev, n)
            k = kinds.setdefault(what, [0, 0])
            k[0] += 1
            k[1] += s - end
        if e > end:
            end = e
            if "partition_tag" not in n:
                prev, after_tag = n, False
    idle = sum(v[1] for v in kinds.values())
    out = ["Last pass: %.3f ms from the first dispatch to the end of the last, kernels busy %.3f ms (summed over queues), device idle %.3f ms (%.1f %%):"
           % ((t1 - t0) / 1e6, busy / 1e6, idle / 1e6, 100.0 * idle / (t1 - t0)), "",
           "| idle interval | count | total us | mean us |", "|---|---|---|---|"]
    for what, (cnt, tot) in sorted(kinds.items(), key=lambda kv: -kv[1][1]):
        out.append("| %s | %d | %.1f | %.2f |" % (what, cnt, tot / 1e3, tot / 1e3 / cnt))
    return "\n".join(out)


def partition_counters_md(counter_csv, counters, granule_cus=32):
    """Mean of derived counters per (kernel, partition size) from a --pmc run with MGB_TAG_PARTITIONS
    set (counter collection runs one dispatch at a time: these are figures of each kernel inside
    its partition, not of the overlap)."""
    part_of_queue, agg, order = {}, {}, []
    for r in csv.DictReader(open(counter_csv)):
        name = short(r["Kernel_Name"])
        q = int(r["Queue_Id"])
        tag = _tag_of(name, int(r["Grid_Size"]))
        if tag is not None:
            part_of_queue[q] = tag
            continue
        if name.startswith("at::") or "rocclr" in name or q not in part_of_queue or r["Counter_Name"] not in counters:
            continue
        key = (name.split("(")[0], part_of_queue[q][1] * granule_cus)
        if key not in agg:
            order.append(key)
        agg.setdefault(key, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    # MfmaUtil, VALUBusy and MeanOccupancyPerCU are normalised by the whole device's SIMDs / CUs: the
    # same figure inside the partition is the reading x 256 / (CUs of the partition)
    whole = {"MfmaUtil", "VALUBusy", "MeanOccupancyPerCU"}
    head = []
    for c in counters:
        head += [c] + (["%s x 256 / CUs" % c] if c in whole else [])
    out = ["| kernel | CUs of its partition | dispatches | " + " | ".join(head) + " |", "|---|---|---|" + "---|" * len(head)]
    for key in sorted(order):
        vals = agg[key]
        n = max(len(v) for v in vals.values())
        cells = []
        for c in counters:
            if c not in vals:
                cells += [""] * (2 if c in whole else 1)
                continue
            m = sum(vals[c]) / len(vals[c])
            cells.append("%.2f (%.2f - %.2f)" % (m, min(vals[c]), max(vals[c])))
            if c in whole:
                cells.append("%.1f" % (m * 256.0 / key[1]))
        out.append("| %s | %d | %d | %s |" % (key[0], key[1], n, " | ".join(cells)))
    return "\n".join(out)


if __name__ == "__main__":
    cmd = sys.argv[1] if len(sys.argv) > 1 else ""
    if cmd == "stats":
        print(stats_md(sys.argv[2]))
    elif cmd == "traffic":
        print(traffic_md(sys.argv[2], sys.argv[3]))
    elif cmd == "overlap":
        a = sys.argv[2:] + [None] * 4
        print(overlap_md(a[0], int(a[1]) if a[1] else None, a[2], a[3]))
    elif cmd == "utilisation":
        print(utilisation_md(dict(zip(UTIL_COUNTERS, sys.argv[2:5]))))
    elif cmd == "gaps":
        print(gaps_md(sys.argv[2], int(sys.argv[3])))
    elif cmd == "counters":
        print(partition_counters_md(sys.argv[2], sys.argv[3].split(",")))
    else:
        print(__doc__)
        sys.exit(2)
