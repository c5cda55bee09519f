"""CPU oracle of the decode-attention latency fit (test infrastructure only).

The paper's Profiler fits f_DA = a * c_DA + h * g + b by linear regression (latency-model section, the
decode-attention equation; System Implementation, Profiler).  This is that regression written out from
its definition: the normal equations of the three-parameter least-squares problem, solved by Cramer's
rule in exact rational arithmetic on the fp64 inputs.  It shares nothing with the product's fit.

Pinned in the tests by planted coefficients (exact recovery), by numpy's polynomial fit on the
one-variable reductions, and by the orthogonality of the residual to the three regressors.
"""
from fractions import Fraction


def _det3(m):
    return (m[0][0] * (m[1][1] * m[2][2] - m[1][2] * m[2][1])
            - m[0][1] * (m[1][0] * m[2][2] - m[1][2] * m[2][0])
            + m[0][2] * (m[1][0] * m[2][1] - m[1][1] * m[2][0]))


def fit(c_da, g, t):
    """Returns (a, h, b) minimising sum (a c + h g + b - t)^2."""
    cs = [Fraction(float(x)) for x in c_da]
    gs = [Fraction(float(x)) for x in g]
    ts = [Fraction(float(x)) for x in t]
    n = len(cs)
    cols = [cs, gs, [Fraction(1)] * n]
    gram = [[sum(x * y for x, y in zip(cols[i], cols[j])) for j in range(3)] for i in range(3)]
    rhs = [sum(x * y for x, y in zip(cols[i], ts)) for i in range(3)]
    det = _det3(gram)
    if det == 0:
        raise ValueError("singular normal equations")
    sol = []
    for k in range(3):
        m = [row[:] for row in gram]
        for i in range(3):
            m[i][k] = rhs[i]
        sol.append(float(_det3(m) / det))
    return tuple(sol)
