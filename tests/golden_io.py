"""Readers for the small text fixtures under tests/golden/."""
import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _ints(s):
    return [int(v) for v in s.split(",")] if s else []


def read_plan_trace(name="plan_trace.txt"):
    """Returns (E, S, W, calls); each call is a dict of the fields listed after a 'call' line."""
    head, calls, cur = {}, [], None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, _, v = line.partition(" ")
            if k in ("E", "S", "W"):
                head[k] = int(v)
            elif k == "call":
                parts = dict(p.split("=") for p in v.split())
                cur = {"layer": int(parts["layer"]), "ids": _ints(parts["ids"]), "entries": []}
                calls.append(cur)
            elif k == "entry":
                cur["entries"].append(tuple(int(t) for t in v.split()))
            elif k in ("cursor", "g"):
                cur[k] = int(v)
            else:
                cur[k] = _ints(v)
    return head["E"], head["S"], head["W"], calls


def read_serve_trace(name="serve_trace.txt"):
    """Returns (head, batches): head has E, S, W, lookahead, policy, fifo_misses; each batch is a
    list of calls as in read_plan_trace."""
    head, batches, cur = {}, [], None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, _, v = line.partition(" ")
            if k in ("E", "S", "W", "lookahead", "fifo_misses"):
                head[k] = int(v)
            elif k == "policy":
                head[k] = v
            elif k == "batch":
                batches.append([])
            elif k == "call":
                parts = dict(p.split("=") for p in v.split())
                cur = {"layer": int(parts["layer"]), "ids": _ints(parts["ids"]), "entries": []}
                batches[-1].append(cur)
            elif k == "entry":
                cur["entries"].append(tuple(int(t) for t in v.split()))
            elif k == "g":
                cur[k] = int(v)
            else:
                cur[k] = _ints(v)
    return head, batches


def read_table2():
    rows = {}
    with open(os.path.join(GOLDEN, "table2_moe_size.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, model, moe, pct = line.split()
            rows[name] = (float(model), float(moe), float(pct))
    return rows


def read_attention_cases(name="sparse_attention_2tok.txt"):
    """Returns {case: (h rows, out rows)} as lists of lists of floats."""
    cases, cur = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, _, v = line.partition(" ")
            if k == "case":
                cur = cases.setdefault(v, ([], []))
            else:
                cur[0 if k == "h" else 1].append([float(t) for t in v.split()])
    return cases
