"""Parser for tests/golden/handbuilt_cases.txt (text fixtures, no arithmetic)."""
import os

import numpy as np

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _words(tokens, w):
    out = []
    for tok in tokens:
        if "*" in tok:
            word, count = tok.split("*")
            out.extend([int(word, 16)] * int(count))
        else:
            out.append(int(tok, 16))
    dtype = np.uint32 if w == 4 else np.uint16
    return np.array(out, dtype=dtype)


def load_handbuilt(filename="handbuilt_cases.txt"):
    cases, cur = [], None
    with open(os.path.join(GOLDEN_DIR, filename)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(" ")
            toks = rest.split()
            if key == "case":
                cur = {"name": rest}
                cases.append(cur)
            elif key in ("n", "w", "bytes", "window"):
                cur[key] = int(rest)
            elif key in ("in", "relu"):
                cur[key] = _words(toks, cur["w"])
            elif key == "stream":
                cur["stream"] = np.array([int(t, 16) for t in toks], dtype=np.uint8)
            elif key == "offsets":
                cur["offsets"] = np.array([int(t) for t in toks], dtype=np.uint64)
            elif key == "masks":
                cur["masks"] = _words(toks, 4)
            elif key == "values":
                cur["values"] = _words(toks, cur["w"])
    for c in cases:
        assert c["in"].size == c["n"], c["name"]
    return cases


def load_window_cases():
    return load_handbuilt("window_cases.txt")


def load_relu_cases():
    return load_handbuilt("relu_cases.txt")


def load_paper_numbers():
    vals = {}
    with open(os.path.join(GOLDEN_DIR, "paper_closed_forms.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, value = line.split()[:2]
            vals[name] = float(value)
    return vals
