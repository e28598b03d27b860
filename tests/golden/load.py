import os


def paper_constants():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "paper_constants.txt")) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if line:
                k, v = line.split()
                out[k] = float(v)
    return out
