"""Whole-span parity bars of the full-shape GPU tests, derived from the stored error floor of the bf16
precision contract (tests/golden/precision_floor.txt: the numpy precision model against the fp32
oracle, no GPU involved).  Importable without torch or the HIP library."""
import os

_GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "precision_floor.txt")
MARGIN = 1.25      # largest row error / largest element error: the GPU path may exceed the contract's own floor by a
                   # quarter.  Its roundings fall on other elements than the model's (running softmax maximum, split
                   # accumulation, fp32 sums in another order flip one bf16 rounding in a thousand, and every later
                   # rounding of a value that moved by a fraction of a bf16 step is drawn afresh), so the two maxima
                   # over a few thousand rows are two draws from the same distribution.
RMS_MARGIN = 1.05  # rms element error: a bulk statistic over 10^6..10^7 elements, reproducible to a fraction of a
                   # per cent between two realisations of the same contract.  A path that added an error of its own of
                   # a third of the floor (one more rounding point, a sloppy exponential) would show +5 % here.


def read_floor():
    """{(workload, session, kind, blocks, rows): (max_row_err, median_row_err, max_elem_err, rms_elem_err)}"""
    out = {}
    with open(_GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            c = line.split()
            out[(c[0], int(c[1]), c[2], int(c[3]), c[4])] = tuple(float(v) for v in c[5:9])
    return out


def _bars(rows):
    return MARGIN * max(r[0] for r in rows), MARGIN * max(r[2] for r in rows), RMS_MARGIN * max(r[3] for r in rows)


def deep_span_bars(workload: str, n_blocks: int = 0, rows: str = ""):
    """(row bar, element bar, rms bar) for outputs of the whole span of `workload` (or of its first n_blocks
    blocks): the margins above times the largest stored floor over the sessions the table holds and over the
    row groups (or for the group `rows` = "prefix" / "decode" alone)."""
    g = read_floor()
    depth = n_blocks or max(k[3] for k in g if k[0] == workload and k[2] == "span")
    sel = [v for k, v in g.items() if k[0] == workload and k[2] == "span" and k[3] == depth and (not rows or k[4] == rows)]
    if not sel:
        raise KeyError(f"no stored floor for {workload} at depth {depth}")
    return _bars(sel)


def alone_bars(workload: str, block: int = 0, rows: str = ""):
    """The same for one block of `workload` on its own, fed the oracle's input (block = 1-based index, 0 = the
    largest over all blocks).  The row bar of a single block that the tests apply is the benchmark spec's 2e-2 itself;
    the floor must stay under it (tests/test_precision_model.py)."""
    sel = [v for k, v in read_floor().items()
           if k[0] == workload and k[2] == "alone" and (not block or k[3] == block) and (not rows or k[4] == rows)]
    if not sel:
        raise KeyError(f"no stored floor for {workload}")
    return _bars(sel)


def floor_of(workload: str, kind: str, n_blocks: int):
    """Largest stored row floor (no margin) of `workload`: kind = "span" after n_blocks blocks, or "alone" for block n_blocks."""
    sel = [v[0] for k, v in read_floor().items() if k[0] == workload and k[2] == kind and k[3] == n_blocks]
    return max(sel)
