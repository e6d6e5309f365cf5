"""Reader for the small text fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_sections(name):
    """'NAME' lines start a section; following lines are rows of numbers (0x.. = integer)."""
    out, cur = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            tok = line.split()
            try:
                row = [int(t, 16) if t.lower().startswith("0x") else float(t) for t in tok]
            except ValueError:
                cur = line
                out[cur] = []
                continue
            out[cur].append(row)
    return {k: np.array(v) for k, v in out.items()}


def read_lemma_table():
    rows = []
    with open(os.path.join(GOLDEN, "lemma_extra_sparsity.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                t = line.split()
                rows.append((int(t[0]), int(t[1]), float(t[2]), len(t) > 3))
    return rows
