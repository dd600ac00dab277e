"""Writes constant_gradient_closed_form.txt from the closed-form sum alone (no oracle, no GPU code).

With the same constant gradient c on every worker, Algorithm 3 of arXiv 1911.09030 gives
acc_T = b0^2 + T c^2 and, because the value under the root is the accumulator of the last
sync (b0^2 + H floor((t-1)/H) c^2) plus t' eps^2 with t' = (t-1) mod H + 1,
    x_T = x0 - eta c sum_{t=1..T} 1 / sqrt(b0^2 + H floor((t-1)/H) c^2 + ((t-1) mod H + 1) eps^2).
"""
import os
from math import sqrt

ETA, EPS, B0, T = 0.5, 1.0, 1.0, 8
rows = []
for c in (1.0, 2.0):
    for H in (1, 2, 4, 8):
        x = -ETA * c * sum(1.0 / sqrt(B0 * B0 + H * ((t - 1) // H) * c * c + ((t - 1) % H + 1) * EPS * EPS)
                           for t in range(1, T + 1))
        rows.append(f"{c:g} {H} {x:.10f} {B0 * B0 + T * c * c:g}")
head = """# Constant gradient g = c on every worker and coordinate; eta = 0.5, eps = 1, b0 = 1, x0 = 0, T = 8.
# Closed form of Algorithm 3 for that input (see make_closed_form.py, which wrote this file).
# For c^2 = eps^2 the sum is sum_t 1/sqrt(b0^2 + t eps^2): independent of H.
# columns: c H x_T acc_T
"""
with open(os.path.join(os.path.dirname(__file__), "constant_gradient_closed_form.txt"), "w") as f:
    f.write(head + "\n".join(rows) + "\n")
