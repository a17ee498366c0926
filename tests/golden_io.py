"""Reader for the small text fixtures under tests/golden/.

A file is a list of ``case <name>`` blocks; inside a block ``key value`` lines hold
scalars and ``key d0 d1 ... : v v v`` lines hold row-major arrays.  ``#`` starts a comment.
"""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_cases(filename):
    cases, cur = {}, None
    with open(os.path.join(GOLDEN, filename)) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            if line.startswith("case "):
                cur = {}
                cases[line.split()[1]] = cur
                continue
            if ":" in line:
                head, vals = line.split(":", 1)
                name, *dims = head.split()
                arr = np.array([float(v) for v in vals.split()], np.float64)
                cur[name] = arr.reshape([int(d) for d in dims])
            else:
                name, val = line.split()
                cur[name] = int(val)
    return cases
