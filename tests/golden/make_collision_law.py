"""Writes the p(s) values of tests/golden/e2lsh_collision_law.txt by numerical
quadrature of the paper's Eq. 2 (Sec. 2.2): p(s) = int_0^w f_{|sX|}(t) (1 - t/w) dt,
with f_{|sX|}(t) = (2/s) phi(t/s).  Calls nothing but scipy."""
import math
import os

from scipy.integrate import quad


def p_collision(s, w):
    f = lambda t: (2.0 / s) * math.exp(-0.5 * (t / s) ** 2) / math.sqrt(2 * math.pi) * (1 - t / w)
    val, _ = quad(f, 0.0, w, epsabs=1e-13, epsrel=1e-13, limit=200)
    return val


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(__file__), "e2lsh_collision_law.txt")
    with open(path) as fh:
        head = [ln for ln in fh if ln.startswith("#")]
    with open(path, "w") as fh:
        fh.writelines(head)
        for w in (4.0, 1.5):
            for s in (0.5, 1.0, 2.0, 4.0, 8.0, 16.0):
                fh.write(f"{w} {s} {p_collision(s, w):.10f}\n")
