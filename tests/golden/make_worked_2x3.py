"""Writes tests/golden/worked_2x3.json: two CAME steps on a 2 x 3 matrix.

The paper prints no worked numeric example, so this fixture is DERIVED, not
quoted: Algorithm 2 (CAME) is evaluated entry by entry with 60-digit mpmath
arithmetic, written as scalar expressions over explicit index sets -- a second
route to the numbers that shares nothing with oracle/came_oracle.c (no arrays,
no loops over a dense buffer, different precision).  Parts that can be checked
by hand are listed under "hand" with the arithmetic spelled out.

Run from the repository root:  python tests/golden/make_worked_2x3.py
"""
import json
import os

from mpmath import mp, mpf, sqrt

mp.dps = 60

b1, b2, b3 = mpf("0.9"), mpf("0.999"), mpf("0.9999")
e1, e2, d, lr = mpf("1e-30"), mpf("1e-16"), mpf(1), mpf("2e-4")
n, m = 2, 3
theta = [[mpf("0.1"), mpf("-0.2"), mpf("0.3")], [mpf("-0.4"), mpf("0.5"), mpf("-0.6")]]
grads = [
    [[mpf("0.01"), mpf("-0.02"), mpf("0.03")], [mpf("0.04"), mpf("0.005"), mpf("-0.06")]],
    [[mpf("-0.02"), mpf("0.01"), mpf("0.03")], [mpf("0.05"), mpf("-0.04"), mpf("0.002")]],
]
I, J = range(n), range(m)
M = [[mpf(0)] * m for _ in I]
r = [mpf(0)] * n
c = [mpf(0)] * m
R = [mpf(0)] * n
C = [mpf(0)] * m
steps = []
for g in grads:
    r = [b2 * r[i] + (1 - b2) * sum(g[i][j] ** 2 + e1 for j in J) for i in I]
    c = [b2 * c[j] + (1 - b2) * sum(g[i][j] ** 2 + e1 for i in I) for j in J]
    sr = sum(r)
    u = [[g[i][j] / sqrt(r[i] * c[j] / sr) for j in J] for i in I]
    rms = sqrt(sum(u[i][j] ** 2 for i in I for j in J) / (n * m))
    k = max(mpf(1), rms / d)
    uh = [[u[i][j] / k for j in J] for i in I]
    M = [[b1 * M[i][j] + (1 - b1) * uh[i][j] for j in J] for i in I]
    U = [[(uh[i][j] - M[i][j]) ** 2 for j in J] for i in I]
    R = [b3 * R[i] + (1 - b3) * sum(U[i][j] + e2 for j in J) for i in I]
    C = [b3 * C[j] + (1 - b3) * sum(U[i][j] + e2 for i in I) for j in J]
    sR = sum(R)
    theta = [[theta[i][j] - lr * M[i][j] / sqrt(R[i] * C[j] / sR) for j in J] for i in I]
    f = lambda x: float(x)
    steps.append({
        "g": [[f(x) for x in row] for row in g],
        "rms_u": f(rms),
        "r": [f(x) for x in r], "c": [f(x) for x in c],
        "R": [f(x) for x in R], "C": [f(x) for x in C],
        "M": [[f(x) for x in row] for row in M],
        "theta": [[f(x) for x in row] for row in theta],
    })

out = {
    "source": "derived from Algorithm 2 (CAME) with 60-digit mpmath; the paper prints no worked example",
    "hyper": {"beta1": 0.9, "beta2": 0.999, "beta3": 0.9999, "eps1": 1e-30, "eps2": 1e-16,
              "clip_d": 1.0, "lr": 2e-4},
    "theta0": [[0.1, -0.2, 0.3], [-0.4, 0.5, -0.6]],
    "hand": {
        "r1": [1.4e-6, 5.225e-6],
        "r1_why": "(1-0.999)*(1e-4+4e-4+9e-4) and (1-0.999)*(1.6e-3+2.5e-5+3.6e-3); eps1 is below the last digit",
        "c1": [1.7e-6, 4.25e-7, 4.5e-6],
        "c1_why": "(1-0.999)*(1e-4+1.6e-3), (1-0.999)*(4e-4+2.5e-5), (1-0.999)*(9e-4+3.6e-3)",
        "rms_uhat_1": 1.0,
        "rms_uhat_1_why": "RMS(u_1) > d = 1, so Eq. 1 scales u_1 to RMS exactly d",
    },
    "steps": steps,
}
path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "worked_2x3.json")
with open(path, "w") as fh:
    json.dump(out, fh, indent=1)
print("wrote", path)
