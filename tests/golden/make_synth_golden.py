"""Writes tests/golden/synth_golden.txt: a few values of the seeded generator, so
that a change to the hash or to the draw shows up as a test failure.  Calls only
the generator (no inference code of any kind)."""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import synth  # noqa: E402


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]


def lines():
    yield "# key value   (written by make_synth_golden.py; generator bits only)"
    for k in range(5):
        c = synth.config(k)
        idx = synth.gen_layer(c["N"], 1, c["seed"], c["window"])
        yield "cfg%d_layer1_cols_sha %s" % (k, digest(idx))
        yield "cfg%d_layer1_neuron7 %s" % (k, ",".join(str(int(x)) for x in idx[7]))
        y = synth.gen_y0(c["batch"], c["N"], c["seed"], rows=[0, 17, c["batch"] - 1])
        yield "cfg%d_y0_rows_sha %s" % (k, digest(y))
        yield "cfg%d_y0_row17_ones %d" % (k, int(y[1].sum()))
    ym = synth.gen_y0(64, 1024, 5, density="mixed")
    yield "mixed_y0_sha %s" % digest(ym)
    ptr, idx, val = synth.gen_layer_general(2048, 2, 20200799, 0, 80)
    yield "general_layer2_sha %s %s %s" % (digest(ptr), digest(idx), digest(val))
    yield "general_layer2_neuron5 %s" % ",".join(str(int(x)) for x in idx[ptr[5]:ptr[6]])
    sc = synth.scatter_columns(synth.gen_layer(8192, 1, 31, 1024), 8192, 1, 31)
    yield "scattered_layer1_sha %s" % digest(sc)


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "synth_golden.txt")
    with open(out, "w") as f:
        f.write("\n".join(lines()) + "\n")
    print(open(out).read())
