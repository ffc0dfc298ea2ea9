import os


def load():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")
    out = {}
    for line in open(path):
        line = line.split("#", 1)[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out
