"""Reader for the small text fixtures under tests/golden/.

Format: '#' starts a comment; 'name: v v v ...' defines a vector (ints, floats or
hex words); 'name: [a b c; d e f]' defines a matrix, rows separated by ';'."""
import os


def _num(s):
    if s.lower().startswith("0x"):
        return int(s, 16)
    try:
        return int(s)
    except ValueError:
        return float(s)


def load(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            name, val = line.split(":", 1)
            val = val.strip()
            if val.startswith("["):
                rows = val.strip("[]").split(";")
                out[name.strip()] = [[_num(x) for x in r.split()] for r in rows]
            else:
                out[name.strip()] = [_num(x) for x in val.split()]
    return out


def path(name):
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
