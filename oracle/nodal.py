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
