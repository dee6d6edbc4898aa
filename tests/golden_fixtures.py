"""Readers of the text fixtures under tests/golden/."""

import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fig3_displacement.txt")


def read_fig3():
    """The worked example of the paper's Figure 3: (token, productions, per-character stacks,
    final input stack, final output stack) with symbols as strings."""
    prods, steps, token, res_i, res_o = [], [], None, None, None
    for line in open(GOLDEN):
        line = line.rstrip("\n")
        if not line or line.startswith("#"):
            continue
        key, _, val = line.partition(":")
        val = val.strip()
        if key == "token":
            token = val
        elif key in ("production", "extra"):
            parts = val.split()
            prods.append((parts[0], parts[1], tuple(parts[2:])))
        elif key == "step":
            ch, si, so = [x.strip() for x in val.split(";")]
            steps.append((ch, tuple(si.split()), tuple(so.split())))
        elif key == "result_input":
            res_i = tuple(val.split())
        elif key == "result_output":
            res_o = tuple(val.split())
    return token, prods, steps, res_i, res_o


