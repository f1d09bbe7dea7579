"""Check the checksums in a sweep result file against the CPU oracle.

    python tests/verify_sweep.py results.jsonl [--threads N] [--max-reads 3e8]

The experiment driver (paper_2405_11425_amd/sweep.py) uses only the HIP library and prints the
checksum of every measured point; this script recomputes them with the oracle from what each
row says about itself (region size, line shape, reads, seeds, window map) and reports, row by
row, "match", "MISMATCH" or why the row is skipped (rows that carry no checksum, or more
reads than --max-reads).  Exit status 1 if any row mismatches.  Runs on the CPU only.
"""
import argparse
import json
import os
import sys

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), ".."))

from oracle import randline as orc   # noqa: E402

GiB, MiB = 1 << 30, 1 << 20
FILL_SEED, READ_SEED = 1, 7          # the driver's fixed seeds (workloads.py)


def expected(row, threads):
    """(value in the row, oracle's value) for a row that can be checked, else a string saying why not."""
    e = row.get("experiment")
    if e in ("region", "lines", "windows", "beyond"):
        R, B, I = int(row["region_gib"] * GiB), row["line_bytes"], row["iters_per_wave"]
        W = row["n_reads"] // I
        wog, nw = None, 1
        if (e == "windows" and row.get("scheme") != "none") or (e == "beyond" and row["scheme"].startswith("windows")):
            if "window_of_group" not in row:
                return "row does not say which window each group reads"
            wog, nw = row["window_of_group"], row["n_windows"]
        return row["checksum_first_seed"], orc.checksum(R, B, W, I, FILL_SEED, READ_SEED, nw, wog, n_threads=threads)
    if e == "pieces-size":
        if "n_reads" not in row:
            return "row does not say how many reads"
        R, I = int(row["region_mib"] * MiB), row["iters_per_wave"]
        return row["checksum_uniform"], orc.checksum(R, 128, row["n_reads"] // I, I, FILL_SEED, READ_SEED, n_threads=threads)
    if e == "probe":
        if "n_reads" not in row:
            return "row does not say how many reads"
        if row.get("distinct_checksums") != 1:
            return row["distinct_checksums"], 1          # every pair must have returned the same checksum
        R, I = int(row["region_gib"] * GiB), row["iters_per_wave"]
        return row["checksum"], orc.checksum(R, 128, row["n_reads"] // I, I, FILL_SEED, READ_SEED, n_threads=threads)
    if e == "stream" and "checksum" in row:
        return row["checksum"], orc.sum_words(FILL_SEED, 0, row["region_gib"] * GiB // 4, n_threads=threads)
    if e in ("latency", "beyond-latency"):
        R = row["footprint_mib"] * MiB
        return (row["final_line"], row["word_sum"]), orc.chase(R, 128, FILL_SEED, 0, 0, 0xFFFFFFFF, row["hops"])
    if e == "beyond-pages":
        stride = row["distance_bytes"] + 128
        return ((row["final_line"], row["word_sum"]),
                orc.chase(row["n_lines"] * stride, 128, FILL_SEED, 0, stride // 128, 0, row["hops"]))
    if e == "latency-per-xcd":
        R = row["footprint_mib"] * MiB
        if not row["all_cus_agree"]:
            return "walks differ", "one walk"
        return (row["final_line"], row["word_sum"]), orc.chase(R, 128, FILL_SEED, 0, 0, 0xFFFFFFFF, row["hops"])
    if e == "updates":
        if "value_seed" not in row:
            return "row does not give the value seed"
        R, I = row["region_gib"] * GiB, row["iters_per_wave"]
        return row["checksum_first_seed"], orc.update_checksum(R, 128, row["n_updates"] // I, I, READ_SEED, row["value_seed"])
    return "no checksum in this kind of row"


def work(row):
    return row.get("n_reads") or row.get("n_updates") or 0


def verify(path, threads, max_reads, out=sys.stdout):
    n_match = n_bad = n_skip = 0
    for line in open(path):
        line = line.strip()
        if not line:
            continue
        row = json.loads(line)
        key = row.get("key", "?")
        if work(row) > max_reads:
            verdict = f"skipped ({work(row)} reads exceed --max-reads)"
            n_skip += 1
        elif row.get("experiment") == "stream" and row.get("region_gib", 0) * GiB // 4 > 16 * max_reads:   # a word costs 1/16 of a read
            verdict = "skipped (region exceeds --max-reads)"
            n_skip += 1
        else:
            res = expected(row, threads)
            if isinstance(res, str):
                verdict = f"skipped ({res})"
                n_skip += 1
            elif res[0] == res[1]:
                verdict = "match"
                n_match += 1
            else:
                verdict = f"MISMATCH: row has {res[0]}, oracle says {res[1]}"
                n_bad += 1
        print(f"{key}: {verdict}", file=out, flush=True)
    print(f"{n_match} match, {n_bad} mismatch, {n_skip} skipped", file=out)
    return n_match, n_bad, n_skip


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("results")
    ap.add_argument("--threads", type=int, default=len(os.sched_getaffinity(0)))
    ap.add_argument("--max-reads", type=float, default=3e8,
                    help="skip rows with more reads than this (the line-width rows have 2^30: about a minute each)")
    args = ap.parse_args(argv)
    _, bad, _ = verify(args.results, args.threads, args.max_reads)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main())
