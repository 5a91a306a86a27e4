import os


def paper_values():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            k, v = [t.strip() for t in line.split("=")]
            vals = [float(t) for t in v.split()]
            out[k] = vals if len(vals) > 1 else vals[0]
    return out
