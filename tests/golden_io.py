"""Parser for the hand-written text fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _clean(lines):
    for ln in lines:
        ln = ln.split("#", 1)[0].rstrip()
        yield ln


def load_mask(name):
    hdr, rows, in_mask = {}, [], False
    with open(os.path.join(GOLDEN, name)) as f:
        for ln in _clean(f):
            if not ln.strip():
                continue
            if in_mask:
                rows.append([int(x) for x in ln.split()])
            elif ln.startswith("mask:"):
                in_mask = True
            else:
                k, v = ln.split(":", 1)
                hdr[k.strip()] = v.strip()
    gamma, K, bp = int(hdr["gamma"]), int(hdr["K"]), int(hdr["beta_p"])
    branch = [int(x) for x in hdr["branch"].split()]
    return gamma, K, bp, branch, np.array(rows, dtype=bool)


def load_traces(name):
    traces, cur = [], {}
    with open(os.path.join(GOLDEN, name)) as f:
        for ln in list(_clean(f)) + [""]:
            if not ln.strip():
                if cur:
                    traces.append(cur)
                    cur = {}
                continue
            k, v = ln.split(":", 1)
            cur[k.strip()] = v.split()
    out = []
    for t in traces:
        d = {k: int(t[k][0]) for k in ("gamma", "K", "beta_p", "A", "path", "n_accept", "bonus")}
        d["branch"] = [int(x) for x in t["branch"]]
        d["root"] = None if t["root"][0] == "none" else int(t["root"][0])
        for k in ("tok", "argmax", "Ahat", "idx"):
            d[k] = np.array([int(x) for x in t[k]], dtype=np.int32)
        out.append(d)
    return out


def meta_from_layout(gamma, K, beta_p, branch):
    """(pid, boff) int16 arrays for a block laid out as main draft then K phrases."""
    T = gamma + K * beta_p
    pid = np.zeros(T, dtype=np.int16)
    boff = np.zeros(T, dtype=np.int16)
    boff[:gamma] = np.arange(gamma)
    for j in range(1, K + 1):
        lo = gamma + (j - 1) * beta_p
        pid[lo:lo + beta_p] = j
        boff[lo:lo + beta_p] = branch[j - 1]
    return pid, boff


def load_commit_examples(name):
    """Paragraphs of kv_commit_example.txt as dicts of int arrays."""
    out, cur = [], {}
    with open(os.path.join(GOLDEN, name)) as f:
        for ln in list(_clean(f)) + [""]:
            if not ln.strip():
                if cur:
                    out.append(cur)
                    cur = {}
                continue
            k, v = ln.split(":", 1)
            cur[k.strip()] = np.array([int(x) for x in v.split()], dtype=np.int64)
    return out
