"""Turn rocprofv3 result databases into the short text summaries kept under profiles/.

    python -m paper_2601_12212_amd.profile_summary kernels RESULTS.db [--cmd "..."]
    python -m paper_2601_12212_amd.profile_summary pmc FETCH.db WRITE.db --copy-bytes N [--json OUT] [--cmd "..."]
    python -m paper_2601_12212_amd.profile_summary counters RESULTS.db [--cmd "..."]

`kernels`: per-kernel launch count and average / min / max duration from a
`rocprofv3 --kernel-trace --stats` run.
`pmc`: per-kernel HBM traffic from two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE, both
in KiB per dispatch).  The counters are scaled by what they read for a plain device copy of
known size in the same run (bench.py --calibration-copy-mb): factor = copy bytes / counter.
`counters`: every counter of one `rocprofv3 --pmc` run per kernel (average per dispatch), and -- when the
counters are there -- the matrix pipe's busy cycles per SIMD as a share of the cycles its compute unit is busy,
the share of them that overlap vector work, and the share of LDS bank-conflict cycles in the LDS's active cycles.
"""
import argparse
import json
import sqlite3
import sys

OURS = "dt::"
COPY = "copyBuffer"


def short(name):
    name = name.replace("void ", "")
    cut = name.find("(")
    return name[:cut] if cut > 0 else name


def kernels(db, cmd):
    c = sqlite3.connect(db)
    rows = c.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start), "
                     "grid_x, grid_y, grid_z, workgroup_x from kernels group by name, grid_x, grid_y, grid_z "
                     "order by sum(end-start) desc").fetchall()
    if cmd:
        print("# command: %s" % cmd)
    print("# rocprofv3 --kernel-trace --stats; durations in microseconds; grid in work-items")
    print("%-44s %7s %9s %9s %9s  %-18s %5s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "grid", "wg"))
    for r in rows:
        if OURS not in r[0]:
            continue
        print("%-44s %7d %9.2f %9.2f %9.2f  %-18s %5d" % (short(r[0])[:44], r[1], r[2] / 1e3, r[3] / 1e3, r[4] / 1e3,
                                                         "%dx%dx%d" % (r[6], r[7], r[8]), r[9]))
    tot = sum(r[5] for r in rows if OURS in r[0])
    calls = max((r[1] for r in rows if "tree_kernel" in r[0]), default=0)
    if calls:
        print("# sum of the library's kernels per step: %.2f us over %d steps" % (tot / 1e3 / calls, calls))


def counter_table(db, counter):
    c = sqlite3.connect(db)
    rows = c.execute("select kernel_name, count(*), avg(value), max(value) from counters_collection "
                     "where counter_name = ? group by kernel_name", (counter,)).fetchall()
    return {r[0]: (r[1], r[2], r[3]) for r in rows}


def pmc(db_fetch, db_write, copy_bytes, out_json, cmd):
    f = counter_table(db_fetch, "FETCH_SIZE")
    w = counter_table(db_write, "WRITE_SIZE")
    fcopy = max((v[2] for k, v in f.items() if COPY in k), default=0.0)
    wcopy = max((v[2] for k, v in w.items() if COPY in k), default=0.0)
    if not fcopy or not wcopy:
        sys.exit("no calibration copy found in the counter runs")
    ff, wf = copy_bytes / (fcopy * 1024.0), copy_bytes / (wcopy * 1024.0)
    if cmd:
        print("# command: %s" % cmd)
    print("# rocprofv3 --pmc FETCH_SIZE / --pmc WRITE_SIZE (KiB per dispatch, averaged over dispatches)")
    print("# calibration: a %d-byte device copy read %.1f KiB (FETCH_SIZE) and wrote %.1f KiB (WRITE_SIZE):"
          % (copy_bytes, fcopy, wcopy))
    print("#   scale factors %.4f (fetch) and %.4f (write) bytes per counted byte" % (ff, wf))
    print("%-44s %7s %12s %12s %14s %14s" % ("kernel", "calls", "FETCH_KiB", "WRITE_KiB", "read_bytes", "write_bytes"))
    res = {}
    for k in sorted(f):
        if OURS not in k:
            continue
        fk = f[k][1]
        wk = w.get(k, (0, 0.0, 0.0))[1]
        rb, wb = fk * 1024.0 * ff, wk * 1024.0 * wf
        res[short(k)] = dict(read_bytes=round(rb), write_bytes=round(wb), hbm_bytes=round(rb + wb), calls=f[k][0])
        print("%-44s %7d %12.1f %12.1f %14.0f %14.0f" % (short(k)[:44], f[k][0], fk, wk, rb, wb))
    if out_json:
        with open(out_json, "w") as fh:
            json.dump(dict(fetch_scale=ff, write_scale=wf, kernels=res), fh, indent=1, sort_keys=True)
            fh.write("\n")


def counters(db, cmd):
    c = sqlite3.connect(db)
    rows = c.execute("select kernel_name, counter_name, count(*), avg(value) from counters_collection "
                     "group by kernel_name, counter_name").fetchall()
    names = sorted({r[1] for r in rows})
    per = {}
    for k, n, cnt, avg in rows:
        if OURS in k:
            per.setdefault(short(k), {})[n] = (cnt, avg)
    if cmd:
        print("# command: %s" % cmd)
    print("# rocprofv3 --pmc %s; averages per dispatch (summed over the chip's shader engines / units)" % " ".join(names))
    print("%-44s %7s %s" % ("kernel", "calls", " ".join("%26s" % n for n in names)))
    for k in sorted(per):
        calls = max(v[0] for v in per[k].values())
        print("%-44s %7d %s" % (k[:44], calls, " ".join("%26.1f" % per[k].get(n, (0, 0.0))[1] for n in names)))
    for k in sorted(per):
        g = lambda n: per[k].get(n, (0, 0.0))[1]
        notes = []
        if g("SQ_VALU_MFMA_BUSY_CYCLES") and g("SQ_BUSY_CU_CYCLES"):
            # the first is summed over SIMDs, the second over compute units (four SIMDs each)
            notes.append("matrix pipe busy %.3f of the cycles its compute unit is busy"
                         % (g("SQ_VALU_MFMA_BUSY_CYCLES") / (4.0 * g("SQ_BUSY_CU_CYCLES"))))
        if g("SQ_VALU_MFMA_BUSY_CYCLES") and g("SQ_VALU_MFMA_COEXEC_CYCLES"):
            notes.append("co-executing with vector work %.3f of the matrix pipe's busy cycles"
                         % (g("SQ_VALU_MFMA_COEXEC_CYCLES") / g("SQ_VALU_MFMA_BUSY_CYCLES")))
        if g("SQ_LDS_IDX_ACTIVE"):
            notes.append("LDS bank conflicts / LDS active cycles = %.3f" % (g("SQ_LDS_BANK_CONFLICT") / g("SQ_LDS_IDX_ACTIVE")))
        if notes:
            print("# %s: %s" % (k, "; ".join(notes)))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    k = sub.add_parser("kernels")
    k.add_argument("db")
    k.add_argument("--cmd", default="")
    p = sub.add_parser("pmc")
    p.add_argument("fetch_db")
    p.add_argument("write_db")
    p.add_argument("--copy-bytes", type=int, required=True)
    p.add_argument("--json", default="")
    p.add_argument("--cmd", default="")
    q = sub.add_parser("counters")
    q.add_argument("db")
    q.add_argument("--cmd", default="")
    a = ap.parse_args()
    if a.what == "kernels":
        kernels(a.db, a.cmd)
    elif a.what == "counters":
        counters(a.db, a.cmd)
    else:
        pmc(a.fetch_db, a.write_db, a.copy_bytes, a.json, a.cmd)


if __name__ == "__main__":
    main()
