"""How much of the forward aggregation's gather traffic a cache could remove on a synthetic workload (host only).

The aggregation of eq. (2) reads one source row per entry of a partition's operator rows: a full row of F
elements for a local column, the k kept elements for a halo column. This script counts, for one partition
and one layer width, how often every source row is referred to, and prints the share of those bytes an ideal
cache of a given size would save if it held the most-referred-to rows for the whole launch (every reference
after the first is a hit). That is an upper bound for any replacement policy that keeps whole rows, and
what a node order or a row schedule could at most gain from reuse inside a cache of that size.

  python -m paper_2406_17611_amd.source_row_reuse <workload> [partition] [width] [ratio]
"""
from __future__ import annotations

import sys

import numpy as np

from . import synth

CACHE_MB = (0.5, 1, 2, 4, 8, 16, 64, 256)


def reuse_counts(w: synth.Workload, p: int, width: int, ratio: int, elem_bytes: int) -> dict:
    """Per distinct source row of partition p: references and bytes; plus the entry count and the local share."""
    g, part = w.graph, np.asarray(w.part)
    rows = np.nonzero(part == p)[0]
    lens = (g.rowptr[rows + 1] - g.rowptr[rows]).astype(np.int64)
    total = int(lens.sum())
    first = np.concatenate([[0], np.cumsum(lens)[:-1]])
    entry = np.repeat(g.rowptr[rows].astype(np.int64) - first, lens) + np.arange(total)
    cols = g.colidx[entry]
    src, refs = np.unique(cols, return_counts=True)
    local = part[src] == p
    k = max(1, width // ratio)
    row_bytes = np.where(local, width * elem_bytes, k * elem_bytes).astype(np.int64)
    return {"entries": total, "local_entries": int(refs[local].sum()), "k": k, "refs": refs, "row_bytes": row_bytes,
            "local": local, "per_entry_bytes": int((refs * row_bytes).sum()), "per_row_bytes": int(row_bytes.sum())}


def reuse_table(w: synth.Workload, p: int, width: int, ratio: int, elem_bytes: int) -> list[str]:
    c = reuse_counts(w, p, width, ratio, elem_bytes)
    refs, row_bytes, local, streaming = c["refs"], c["row_bytes"], c["local"], c["per_entry_bytes"]
    out = [f"workload {w.name}, partition {p} of {w.n_parts}, width {width}, k {c['k']}, {elem_bytes} bytes per element",
           f"entries {c['entries']} ({100.0 * c['local_entries'] / max(1, c['entries']):.1f} % refer to local rows), "
           f"distinct source rows {len(refs)} ({int(local.sum())} local, {int((~local).sum())} halo)",
           f"source-row bytes: {streaming / 1e9:.3f} GB with one fetch per entry, {c['per_row_bytes'] / 1e9:.3f} GB with one "
           f"fetch per row",
           f"references per source row: median {int(np.median(refs))}, 90 % {int(np.quantile(refs, .9))}, "
           f"99 % {int(np.quantile(refs, .99))}, 99.9 % {int(np.quantile(refs, .999))}, max {int(refs.max())}",
           "", "ideal cache   rows held   fewest references of a held row   share of the per-entry bytes saved"]
    order = np.argsort(-refs, kind="stable")          # same bytes saved per cached byte for both kinds of row
    held = np.cumsum(row_bytes[order])
    saved = np.cumsum(((refs - 1) * row_bytes)[order])
    for mb in CACHE_MB:
        n = int(np.searchsorted(held, mb * 1e6))
        if n == 0:
            continue
        out.append(f"{mb:8g} MB  {n:10d}  {int(refs[order][n - 1]):33d}  {saved[n - 1] / streaming:36.3f}")
    return out


def main(argv: list[str]) -> int:
    if not argv:
        print(__doc__)
        return 2
    w = synth.make_workload(argv[0])
    p = int(argv[1]) if len(argv) > 1 else 0
    width = int(argv[2]) if len(argv) > 2 else w.widths[1]
    ratio = int(argv[3]) if len(argv) > 3 else w.ratios[0][0] // w.ratios[0][1]
    print("\n".join(reuse_table(w, p, width, ratio, 2 if w.dtype == "bf16" else 4)))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
