"""TEST INFRASTRUCTURE: exact nodal (Kirchhoff) solution of one small resistive crossbar tile.

Used only to pin the approximate analytical model of the oracle (Sec. IV-D of the paper compares
that model with the full circuit solution and reports that the error vanishes when the device
resistance is far above the wire resistance).  Geometry: row i is driven from the column-0 side
through r_source, every cell adds one r_row segment along the row wire; column j is sensed at the
far end (beyond the last row) through r_sense to ground, every cell adds one r_col segment along
the column wire.  Device (i, j) connects row-wire node (i, j) with column-wire node (i, j).
"""
import numpy as np


def effective_conductance(G, r_row, r_col, r_source=0.0, r_sense=0.0):
    """G: [R][C] device conductances.  Returns E[R][C] with I_col[j] = sum_i V_row[i] * E[i][j],
    the exact linear map from row voltages to sensed column currents."""
    G = np.asarray(G, dtype=np.float64)
    R, C = G.shape
    nn = 2 * R * C                      # unknown node voltages: row-wire nodes, then column-wire nodes

    def rn(i, j):
        return i * C + j

    def cn(i, j):
        return R * C + i * C + j

    A = np.zeros((nn, nn))
    B = np.zeros((nn, R))               # right-hand side per unit voltage on each row driver
    g_row = 1.0 / r_row
    g_col = 1.0 / r_col
    g_first = 1.0 / (r_source + r_row)  # driver -> first row node
    g_last = 1.0 / (r_col + r_sense)    # last column node -> ground
    for i in range(R):
        for j in range(C):
            a = rn(i, j)
            # towards the driver
            if j == 0:
                A[a, a] += g_first
                B[a, i] += g_first
            else:
                A[a, a] += g_row
                A[a, rn(i, j - 1)] -= g_row
            if j + 1 < C:
                A[a, a] += g_row
                A[a, rn(i, j + 1)] -= g_row
            # the device
            b = cn(i, j)
            A[a, a] += G[i, j]
            A[a, b] -= G[i, j]
            A[b, b] += G[i, j]
            A[b, a] -= G[i, j]
            # column wire
            if i > 0:
                A[b, b] += g_col
                A[b, cn(i - 1, j)] -= g_col
            if i + 1 < R:
                A[b, b] += g_col
                A[b, cn(i + 1, j)] -= g_col
            else:
                A[b, b] += g_last
    V = np.linalg.solve(A, B)           # node voltages per unit drive of each row
    E = np.zeros((R, C))
    for j in range(C):
        E[:, j] = V[cn(R - 1, j), :] * g_last
    return E


def effective_conductance_sparse(G, r_row, r_col, r_source=0.0, r_sense=0.0):
    """Same circuit and same result as effective_conductance, assembled as a sparse matrix and
    factorised once (sparse LU) so that full-size tiles (128 x 128: 32768 node voltages) are solved in
    seconds.  Kirchhoff's current law at every wire node; unknowns: row-wire nodes, then column-wire
    nodes."""
    import scipy.sparse as sp
    import scipy.sparse.linalg as spla

    G = np.asarray(G, dtype=np.float64)
    R, C = G.shape
    n = R * C
    ii, jj = np.meshgrid(np.arange(R), np.arange(C), indexing="ij")
    rn = (ii * C + jj).ravel()
    cn = rn + n
    g = G.ravel()
    rows, cols, vals = [], [], []

    def add(a, b, v):
        rows.append(a); cols.append(b); vals.append(np.broadcast_to(v, a.shape))

    def link(a, b, cond):                       # conductance cond between nodes a and b
        add(a, a, cond); add(b, b, cond); add(a, b, -cond); add(b, a, -cond)

    link(rn, cn, g)                             # devices
    right = (jj < C - 1).ravel()
    link(rn[right], rn[right] + 1, 1.0 / r_row)     # row-wire segments
    down = (ii < R - 1).ravel()
    link(cn[down], cn[down] + C, 1.0 / r_col)       # column-wire segments
    first = (jj == 0).ravel()
    g_first = 1.0 / (r_source + r_row)
    add(rn[first], rn[first], g_first)              # driver side (the drive goes to the right-hand side)
    last = (ii == R - 1).ravel()
    g_last = 1.0 / (r_col + r_sense)
    add(cn[last], cn[last], g_last)                 # sense side to ground
    A = sp.csc_matrix((np.concatenate(vals), (np.concatenate(rows), np.concatenate(cols))), shape=(2 * n, 2 * n))
    B = np.zeros((2 * n, R))
    B[np.arange(R) * C, np.arange(R)] = g_first
    V = spla.splu(A).solve(B)
    return (V[n + (R - 1) * C + np.arange(C), :] * g_last).T
