#!/usr/bin/env python3
"""Coefficients of the degree-10 polynomial that exp_softmax (spec_accept.hip) evaluates on the reduced argument.

The polynomial takes the values of exp at the 11 Chebyshev nodes of [-a, a], a = ln2 / 2 widened by 0.05 %; the
linear system is solved by Gaussian elimination in x87 extended precision (numpy.longdouble) and the result rounded
to fp64.  Prints the coefficients (constant term first) and the largest relative error of the fp64 Horner
evaluation over the interval.  Run it to check or regenerate the constants in the kernel source."""
import numpy as np

LD = np.longdouble
DEGREE = 10


def coefficients(n=DEGREE):
    a = LD(0.34657359027997264311) * LD(1.0005)
    k = np.arange(n + 1)
    x = np.cos((np.pi * (2 * k + 1) / (2 * (n + 1))).astype(LD)) * a
    A = np.vander(np.asarray(x, dtype=LD), n + 1, increasing=True)
    b = np.exp(x)
    m = n + 1
    for i in range(m):  # elimination with partial pivoting, all in long double
        p = int(np.argmax(np.abs(A[i:, i]))) + i
        A[[i, p]], b[[i, p]] = A[[p, i]], b[[p, i]]
        for j in range(i + 1, m):
            f = A[j, i] / A[i, i]
            A[j] -= f * A[i]
            b[j] -= f * b[i]
    c = np.zeros(m, dtype=LD)
    for i in range(m - 1, -1, -1):
        c[i] = (b[i] - A[i, i + 1:] @ c[i + 1:]) / A[i, i]
    return c.astype(np.float64)


def max_relative_error(c, samples=200001):
    x = np.linspace(-0.34657359027997264311, 0.34657359027997264311, samples)
    p = np.full_like(x, c[-1])
    for q in c[-2::-1]:
        p = p * x + q
    return float(np.max(np.abs(p.astype(LD) / np.exp(x.astype(LD)) - 1)))


if __name__ == "__main__":
    c = coefficients()
    for i, v in enumerate(c):
        print(f"c{i} = {float(v)!r}")
    print(f"max relative error of the fp64 Horner evaluation on [-ln2/2, ln2/2]: {max_relative_error(c):.2e}")
