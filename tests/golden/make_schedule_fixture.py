"""Writes tests/golden/completion_schedules.txt from the oracle alone.

The paper prints no worked schedule (its Fig. 3a is an image), so this fixture is
not a paper value: it freezes what the oracle's planner emits for n = 4 and 8 so
that a change of a tie-break shows up as a diff.  Run from the repository root:
    python tests/golden/make_schedule_fixture.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import schedule as S  # noqa: E402

KIND = {0: "COPY", 1: "REDUCE", 2: "EXCHANGE"}


def render():
    lines = ["# completion schedules of Alg. 1 as the oracle emits them (logical ranks, straggler = n-1)",
             "# format: n round src dst chunk kind"]
    for n in (4, 8):
        for r, ops in enumerate(S.completion_logical(n)):
            for s, d, c, k in ops:
                lines.append("%d %d %d %d %d %s" % (n, r, s, d, c, KIND[k]))
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "completion_schedules.txt")
    with open(out, "w") as f:
        f.write(render())
    print("wrote", out)
