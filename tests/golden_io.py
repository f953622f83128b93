"""Reader for the small text fixtures under tests/golden/.

Format: '#' comment lines; 'name value' scalar lines; 'name rows cols' followed by that many
rows of numbers.
"""
import numpy as np


def read_golden(path):
    out = {}
    with open(path) as f:
        lines = [ln.strip() for ln in f if ln.strip() and not ln.lstrip().startswith("#")]
    i = 0
    while i < len(lines):
        parts = lines[i].split()
        if len(parts) == 2:
            out[parts[0]] = float(parts[1])
            i += 1
        elif len(parts) == 3:
            r, c = int(parts[1]), int(parts[2])
            rows = [[float(v) for v in lines[i + 1 + j].split()] for j in range(r)]
            a = np.array(rows, dtype=np.float64)
            assert a.shape == (r, c), (path, parts[0])
            out[parts[0]] = a
            i += 1 + r
        else:
            raise ValueError(f"{path}: cannot parse {lines[i]!r}")
    return out
