"""Writes worked_example_g0_4.txt from the oracle (and only the oracle).

G0 = 4, uniform prior, c = (0, 2, 4), budgets 0..12.  The paper prints no worked
allocation; rows without ties follow from exact rationals (checked in
tests/test_oracle_allocate.py), the tied rows record this library's tie rule
(canonical binary64 gain, then prompt index; Sec. 3.2's argmax states none).
Run: python tests/golden/make_worked_example.py
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import hora_oracle  # noqa: E402

c = np.array([0, 2, 4], dtype=np.int32)
out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "worked_example_g0_4.txt")
with open(out, "w") as f:
    f.write("# G0=4, prior Beta(1,1), c=(0,2,4); columns: budget delta_0 delta_1 delta_2\n")
    f.write("# written by make_worked_example.py from oracle/ (Alg. 1 Phase B; tie rule: fp64 gain, then index)\n")
    for budget in range(13):
        d = hora_oracle.allocate(c, 4, budget)
        f.write(f"{budget} {d[0]} {d[1]} {d[2]}\n")
