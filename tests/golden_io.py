"""Reader for the small text fixtures under tests/golden/."""
import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_cases(name):
    """Yield (kind, params dict, [(a, b, value)], {word: value}) for each 'case' block."""
    cases = []
    cur = None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "case":
                cur = (tok[1], {k: int(v) for k, v in (t.split("=") for t in tok[2:])}, [], {})
                cases.append(cur)
            elif tok[0] == "set":
                cur[2].append((int(tok[1]), int(tok[2]), int(tok[3])))
            elif tok[0] == "expect":
                cur[3][int(tok[1])] = int(tok[2], 16)
            else:
                raise ValueError(line)
    return cases


def read_dequant(name="dequant.txt"):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            lhs, rhs = line.split("->")
            l = lhs.split()
            rows.append((float(l[0]), int(l[1]), [int(t) for t in l[2:]], [float(t) for t in rhs.split()]))
    return rows
