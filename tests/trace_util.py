"""Parser for tests/golden/*_trace.txt (hand-derived file-system traces)."""
import os


def load_trace(name):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    steps = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        lhs, rhs = line.split("|")
        op, *args = lhs.split()
        exp = dict(kv.split("=", 1) for kv in rhs.split())
        steps.append((op, args, exp))
    return steps


def parse_expect(exp):
    out = {}
    if "h" in exp:
        out["h"] = int(exp["h"])
    if "len" in exp:
        out["len"] = int(exp["len"])
    if "free" in exp:
        out["free"] = int(exp["free"])
    if "rc" in exp:
        out["rc"] = [int(x) for x in exp["rc"].split(",")]
    if "pages" in exp:
        out["pages"] = [] if exp["pages"] == "-" else [int(x) for x in exp["pages"].split(",")]
    if "moves" in exp:          # src page:slot > dst page:slot
        out["moves"] = [] if exp["moves"] == "-" else [
            tuple(int(y) for side in x.split(">") for y in side.split(":")) for x in exp["moves"].split(",")]
    if "swaps" in exp:          # a>b pairs
        out["swaps"] = [] if exp["swaps"] == "-" else [tuple(int(y) for y in x.split(">")) for x in exp["swaps"].split(",")]
    if "slots" in exp:
        out["slots"] = [tuple(int(y) for y in x.split(":")) for x in exp["slots"].split(",")]
    if "cow" in exp:
        out["cow"] = [] if exp["cow"] == "-" else [
            (int(x.split(">")[0]), int(x.split(">")[1].split(":")[0]), int(x.split(":")[1])) for x in exp["cow"].split(",")]
    return out
