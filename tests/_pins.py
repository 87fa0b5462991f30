"""Readers for tests/golden/paper_pins.txt and for the feasibility limits the library's header states."""
import os
import re


def lib_limits():
    """The three limits include/wt.h states as #defines, as the keyword arguments the oracle takes them by:
    (for select.read_table / DualTable) ws_elems, max_split_tiles; (for fit.fit_tables) max_anchors."""
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "wt.h")
    text = open(path).read()

    def define(name):
        m = re.search(r"#define\s+" + name + r"\s+\(?\s*(\d+)\s*(?:<<\s*(\d+))?\s*\)?", text)
        assert m, name
        return int(m.group(1)) << int(m.group(2) or 0)

    return {"ws_elems": define("WT_SPLITK_WS_FLOATS"), "max_split_tiles": define("WT_SPLITK_MAX_TILES"),
            "max_anchors": define("WT_MAX_ANCHORS")}


def split_limits():
    d = lib_limits()
    return {"ws_elems": d["ws_elems"], "max_split_tiles": d["max_split_tiles"]}


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
