"""Small shared helpers for the tests (parsing the golden text fixtures, error metrics)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    """'key v v v' lines -> dict of float lists; a bare 'A' line starts a matrix."""
    out, mat = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "A" and len(tok) == 1:
                mat = []
                out["A"] = mat
                continue
            try:
                vals = [float(t) for t in tok]
                if mat is not None:
                    mat.append(vals)
                    continue
            except ValueError:
                pass
            mat = None
            out[tok[0]] = [float(t) for t in tok[1:]]
    return out


def rel_max_err(got, ref):
    """Norm-wise relative error: max|got-ref| / max(max|ref|, 1e-30)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30)) if ref.size else 0.0
