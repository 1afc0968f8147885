"""Writes the closed-form Cholesky fixtures in this folder.

The paper (arXiv 1710.08717) prints no worked numerical example for potrf, trsm,
trmm, syrk or the potrf backward expression, so the stored values are textbook
closed forms, written from their formulas alone (no oracle, no GPU code):

* pascal_lower_n8.txt   - lower Pascal matrix L_ij = C(i, j); the symmetric Pascal
                          matrix S_ij = C(i + j, i) satisfies S = L L^T (classical
                          identity, Vandermonde convolution), so potrf(S) = L.
* tridiag_factor_n8.txt - the second-difference matrix tridiag(-1, 2, -1) has the
                          factor l_ii = sqrt((i+1)/i), l_{i+1,i} = -sqrt(i/(i+1))
                          (1-based i), from its pivots (i+1)/i.

Run:  python tests/golden/make_golden.py
"""
import math
import os

HERE = os.path.dirname(os.path.abspath(__file__))


def write(name, header, rows):
    with open(os.path.join(HERE, name), "w") as f:
        for line in header:
            f.write("# " + line + "\n")
        for r in rows:
            f.write(" ".join(repr(float(v)) for v in r) + "\n")


def main():
    n = 8
    write(
        "pascal_lower_n8.txt",
        ["lower Pascal matrix, L_ij = C(i,j) (0-based); potrf of S_ij = C(i+j,i) must return it",
         "pins: operator table row potrf (A = L L^T, l_ij = 0 for i<j) and section 4.2 (positive diagonal)"],
        [[math.comb(i, j) if j <= i else 0 for j in range(n)] for i in range(n)],
    )
    rows = []
    for i in range(1, n + 1):
        r = [0.0] * n
        r[i - 1] = math.sqrt((i + 1) / i)
        if i >= 2:
            r[i - 2] = -math.sqrt((i - 1) / i)
        rows.append(r)
    write(
        "tridiag_factor_n8.txt",
        ["Cholesky factor of tridiag(-1,2,-1), n=8: l_ii = sqrt((i+1)/i), l_{i,i-1} = -sqrt((i-1)/i), 1-based",
         "pins: operator table row potrf and section 4.2 first paragraph"],
        rows,
    )


if __name__ == "__main__":
    main()
