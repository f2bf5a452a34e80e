"""Reader for the hand-written text fixtures under tests/golden/."""
import os
import numpy as np

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_case(name):
    """Parse a decode_*.txt fixture into a dict of plain arrays."""
    out = {"codebook": [], "W": [], "q": [], "tables": [], "levels": [], "codes": []}
    with open(os.path.join(GOLDEN_DIR, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(":")
            key, rest = key.strip(), rest.strip()
            if key == "format":
                out["format"] = {k: int(v) for k, v in (kv.split("=") for kv in rest.split())}
            elif key == "idx_hex":
                out["idx"] = np.array([int(t, 16) for t in rest.split()], dtype=np.uint8)
            elif key in ("codebook", "W"):
                out[key].append([float(t) for t in rest.split()])
            elif key == "q":          # int8 lookup table of one group
                out["q"].append([int(t) for t in rest.split()])
            elif key == "scale":      # one scale per group
                out["scale"] = np.array([float(t) for t in rest.split()], dtype=np.float64)
            elif key == "tables_hex":   # raw bytes of an interchange table buffer (lines are concatenated)
                out["tables"].extend(int(t, 16) for t in rest.split())
            elif key == "levels":     # the 16 block-scale levels of one group
                out["levels"].append([float(t) for t in rest.split()])
            elif key == "codes":      # the 4-bit block codes of one row
                out["codes"].append([int(t) for t in rest.split()])
            elif key in ("x", "y"):
                out[key] = np.array([float(t) for t in rest.split()], dtype=np.float64)
            else:
                raise ValueError(f"unknown key {key!r} in {name}")
    fmt = out["format"]
    out["codebook"] = np.array(out["codebook"], dtype=np.float64).reshape(-1, fmt["k"], fmt["d"])
    out["q"] = np.array(out["q"], dtype=np.int64).reshape(-1, fmt["k"], fmt["d"])
    out["W"] = np.array(out["W"], dtype=np.float64)
    out["tables"] = np.array(out["tables"], dtype=np.uint8)
    out["levels"] = np.array(out["levels"], dtype=np.float64)
    out["codes"] = np.array(out["codes"], dtype=np.uint8)
    return out


def read_bpv_table():
    rows = []
    with open(os.path.join(GOLDEN_DIR, "bpv_table.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bpv, d, k, l, bc = line.split()
            rows.append((float(bpv), int(d), int(k), int(l), int(bc)))
    return rows
