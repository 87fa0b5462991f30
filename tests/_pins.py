"""Reader for tests/golden/paper_pins.txt."""
import os


def load_pins():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_pins.txt")
    pins = {}
    for line in open(path):
        line = line.split("#", 1)[0].strip()
        if not line:
            continue
        name, *vals = line.split()
        vals = [int(v) for v in vals]
        pins[name] = vals[0] if len(vals) == 1 else tuple(vals)
    return pins
