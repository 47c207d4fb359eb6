"""Readers for the small text fixtures under tests/golden/."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def accept_cases():
    cases = []
    with open(os.path.join(GOLDEN, "accept_cases.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            name, y, d, a, nl, w, vd, tau, bonus = [p.strip() for p in line.split(";")]
            ints = lambda s: np.array([int(x) for x in s.split(",")], np.int32)
            cases.append(dict(name=name, y=ints(y), d=ints(d),
                              a=np.array([float(x) for x in a.split(",")], np.float32),
                              n_loose=int(nl), pst_window=int(w), verdict=ints(vd).astype(np.uint8),
                              tau=int(tau), bonus=int(bonus)))
    return cases


def entropy_cases():
    cases = []
    ints = lambda s: np.array([int(x) for x in s.split(",")], np.int32)
    with open(os.path.join(GOLDEN, "entropy_cases.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            name, y, d, h, th, w, vd, tau, bonus = [p.strip() for p in line.split(";")]
            cases.append(dict(name=name, y=ints(y), d=ints(d),
                              h=np.array([float(x) for x in h.split(",")], np.float32),
                              threshold=float(th), window=int(w),
                              verdict=ints(vd).astype(np.uint8), tau=int(tau), bonus=int(bonus)))
    return cases


def paper_constants():
    out = {}
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                out[k.strip()] = float(v)
    return out


def tree_cases():
    cases = []
    ints = lambda s: np.array([int(x) for x in s.split(",")], np.int32)
    with open(os.path.join(GOLDEN, "tree_cases.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            name, nl, w, chains, taus, kept = [p.strip() for p in line.split(";")]
            ch = []
            for c in chains.split("|"):
                y, d, a = [p.strip() for p in c.split("/")]
                ch.append(dict(y=ints(y), d=ints(d),
                               a=np.array([float(x) for x in a.split(",")], np.float32)))
            cases.append(dict(name=name, n_loose=int(nl), pst_window=int(w), chains=ch,
                              tau=ints(taus), kept=int(kept)))
    return cases


def commit_cases():
    cases = []
    ints = lambda s: np.array([int(x) for x in s.split(",")], np.int32)
    with open(os.path.join(GOLDEN, "commit_cases.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            name, cap, ctx, nbr, K, taus, kept, rows, new_len = [p.strip() for p in line.split(";")]
            cases.append(dict(name=name, cap=int(cap), ctx=int(ctx), n_branches=int(nbr),
                              chain_len=int(K), accept_len=ints(taus), kept=int(kept),
                              rows=ints(rows), new_len=int(new_len)))
    return cases
