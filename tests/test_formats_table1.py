"""The storage formats of the boundary (4-byte node ids, 8-byte (src, ctx) samples, fp32 embedding
elements) reproduce the sizes the paper prints in Table I, to the printed precision."""
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

ID_BYTES = np.dtype(np.int32).itemsize            # node id in pairs_dev / neg_out_dev
PAIR_BYTES = 2 * ID_BYTES                         # one (src, ctx) sample
ELEM_BYTES = np.dtype(np.float32).itemsize        # one embedding element

BYTES_PER_ITEM = {"nodes": ID_BYTES, "edges": PAIR_BYTES, "augmented_edges": PAIR_BYTES,
                  "vertex_embeddings": ELEM_BYTES, "context_embeddings": ELEM_BYTES}


def test_table1_sizes():
    rows = 0
    for line in open(os.path.join(HERE, "golden", "table1_memory.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, count, printed, unit = [c.strip() for c in line.split("|")]
        n = 1.0
        for f in count.split("*"):
            n *= float(f)
        size = n * BYTES_PER_ITEM[name] / 2**30
        if unit == "GiB/1000":
            size /= 1000.0
        printed_v = float(printed)
        decimals = len(printed.split(".")[1]) if "." in printed else 0
        assert abs(size - printed_v) <= 0.5 * 10 ** (-decimals) + 1e-9, (name, size, printed_v)
        rows += 1
    assert rows == 5
