"""Writes tests/golden/precision_floor.txt: the error floor of the bf16 precision contract at the full
shapes of the benchmark configurations, CPU only (numpy): `python tests/golden/make_precision_floor.py`.

For the sessions the GPU parity tests follow (70B-shaped span: session 0 of the 2048 + 128-token
workload and the shortest and the median-length session of the fail-over workload; BLOOM-176B-shaped
span: sessions 0 and 9; 7B-shaped span: all four sessions) it runs, block by block on the same seeded weights and inputs,

  * the fp32 oracle (oracle/span_oracle.py),
  * the bf16 precision model (tests/precision_model.py) through the whole span  -> rows "span",
  * the model on one block alone, fed the oracle's input of that block          -> rows "alone",

and records how far the model lies from the oracle after every block: the largest and the median
relative row error ||model_t - oracle_t|| / ||oracle_t||, and the largest and the rms element error
|model - oracle| / rms(oracle row), separately for the prefix rows and the decode-step rows.  No
kernel and no GPU takes part: the numbers are what the contract "bf16 operands, fp32 accumulation,
bf16 cache" costs on these synthetic inputs, and the GPU tests derive their whole-span bars from them.
About 20 minutes on 8 cores; `... make_precision_floor.py 7b` (or 70b, bloom) recomputes one group only.
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import precision_model as pm  # noqa: E402
from oracle import span_oracle as so  # noqa: E402
from workloads import WORKLOADS, SpanWeights, draw_hidden  # noqa: E402


def followed_sessions(name):
    """(session index, prefix length, decode steps) of the sessions the parity tests follow."""
    wl = WORKLOADS[name]
    if name == "failover70b":
        order = np.argsort(wl.prefix_lens)
        picks = [int(order[0]), int(order[len(order) // 2])]
    elif name == "bloom176b":
        picks = [0, 9]
    elif name == "llama7b":
        picks = [0, 1, 2, 3]
    else:
        picks = [0]
    return [(i, wl.prefix_lens[i], wl.decode_steps) for i in picks]


def stats(got, ref):
    l2, el = pm.row_l2_rel(got, ref), pm.elem_rel(got, ref)
    return float(l2.max()), float(np.median(l2)), float(el.max()), float(np.sqrt(np.mean(el * el)))


def run(names, out):
    shape = WORKLOADS[names[0]].shape
    W = SpanWeights(shape, seed=WORKLOADS[names[0]].seed, bf16=True, cache=False, threads=8)
    sess = []
    for name in names:
        for i, L, n_dec in followed_sessions(name):
            x = draw_hidden(shape, WORKLOADS[name].seed, i, L + n_dec).astype(np.float32)
            sess.append({"name": name, "i": i, "L": L, "ref": x, "mod": x, "carry": {}})
    empty = np.zeros((0, shape.n_kv_heads, shape.head_dim), np.float32)
    for b in range(shape.n_blocks):
        t0 = time.time()
        w = W[b]
        for s in sess:
            ref_in = s["ref"]
            s["ref"] = so.block_forward(shape, w, ref_in, empty, empty, dtype=np.float32, matrix_attention=True)[0]
            s["mod"] = pm.block_forward(shape, w, s["mod"], empty, empty, pm.ALL_POINTS, folded_norm1=b > 0, carry=s["carry"])[0]
            alone = pm.block_forward(shape, w, ref_in, empty, empty, pm.ALL_POINTS, folded_norm1=False)[0]
            for kind, got in (("span", s["mod"]), ("alone", alone)):
                for part, sl in (("prefix", slice(0, s["L"])), ("decode", slice(s["L"], None))):
                    st = stats(got[sl], s["ref"][sl])
                    out.write(f"{s['name']} {s['i']} {kind} {b + 1} {part} " + " ".join(f"{v:.4e}" for v in st) + "\n")
                    out.flush()
        del w
        print(f"  {names}: block {b} done in {time.time() - t0:.0f} s", file=sys.stderr, flush=True)


GROUPS = {"70b": ["llama70b", "failover70b"], "bloom": ["bloom176b"], "7b": ["llama7b"]}   # a group shares its weights
HEADER = ("# Error floor of the bf16 precision contract (tests/precision_model.py against oracle/span_oracle.py, fp32),\n"
          "# written by tests/golden/make_precision_floor.py; no GPU involved.\n"
          "# 'span N': after N blocks of the whole span; 'alone N': block N on its own, fed the oracle's input.\n"
          "# workload session kind blocks rows  max_row_rel_err median_row_rel_err max_elem_err rms_elem_err\n")


def main():
    """No arguments: everything.  With group names (70b, bloom, 7b): only those are recomputed, the
    other workloads' lines are kept as they stand."""
    groups = sys.argv[1:] or list(GROUPS)
    redo = {w for g in groups for w in GROUPS[g]}
    path = os.path.join(HERE, "precision_floor.txt")
    kept = []
    if os.path.exists(path):
        kept = [l for l in open(path) if not l.startswith("#") and l.split() and l.split()[0] not in redo]
    with open(path + ".tmp", "w") as out:
        out.write(HEADER)
        out.writelines(kept)
        for g in groups:
            run(GROUPS[g], out)
    os.replace(path + ".tmp", path)


if __name__ == "__main__":
    main()
