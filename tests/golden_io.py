"""Reader for the hand-worked examples under tests/golden/."""
import math
import os

import numpy as np

_SYMS = {"ln3": math.log(3.0), "ln3/2": math.log(3.0) / 2.0}


def _num(tok: str) -> float:
    neg = tok.startswith("-")
    body = tok[1:] if neg else tok
    v = _SYMS[body] if body in _SYMS else float(body)
    return -v if neg else v


def load_example(name: str) -> dict:
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    rows = {"W": [], "U": [], "x": [], "c": [], "h": []}
    ex = {"bias": None}
    with open(path) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, *toks = line.split()
            if key == "cell":
                ex["cell"] = toks[0]
            elif key in ("d", "k"):
                ex[key] = int(toks[0])
            elif key in rows:
                rows[key].append([_num(t) for t in toks])
            elif key in ("bias", "c_init", "h_init"):
                ex[key] = np.array([_num(t) for t in toks], np.float64)
            else:
                raise ValueError(f"{name}: unknown key {key}")
    d, k = ex["d"], ex.get("k", 1)
    ex["W"] = np.array(rows["W"], np.float64).astype(np.float32)
    if ex["cell"] == "lstm":
        ex["U"] = np.array(rows["U"], np.float64).astype(np.float32)
        assert ex["W"].shape == (4 * d, d) and ex["U"].shape == (4 * d, d)
    else:
        assert ex["W"].shape == (3 * d, k * d)
    ex["x"] = np.array(rows["x"], np.float32)
    ex["c"] = np.array(rows["c"], np.float64)
    ex["h"] = np.array(rows["h"], np.float64)
    if ex["bias"] is not None:
        ex["bias"] = ex["bias"].astype(np.float32)
    return ex
