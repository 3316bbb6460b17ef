import os


def load_golden(name="paper_stated_values.txt"):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    out = {}
    with open(path) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = [s.strip() for s in line.split("=", 1)]
            vals = [float(t) for t in v.split()]
            out[k] = vals[0] if len(vals) == 1 else vals
    return out
