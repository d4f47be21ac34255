"""TEST INFRASTRUCTURE: circuit-level crossbar model of the oracle (Sec. IV-A, IV-D: the model that
solves Ohm's and Kirchhoff's laws for every crossbar instance, and the distortion profile
D = (G_ideal - G_nonideal) / G_ideal that the interpolated variant stores and reuses).

Per crossbar instance, slice and polarity array the exact nodal solution (oracle/nodal.py) gives the
linear map from row voltages to column currents; its entry (i, j) is the non-ideal conductance of
device (i, j).  Rows / columns beyond the weight matrix hold no device (conductance 0), the wires of
a partial tile still run the full tile length.
"""
import numpy as np

from . import nodal
from . import xbar_oracle as xo


def fcm_profile(cfg, W, w_max, step=0):
    """D[S][2][K][N] (float64) for the weights W under the parameters of cfg."""
    G = xo.device_conductances(cfg, W, w_max, step)
    S, _, K, N = G.shape
    R, C = cfg.xbar_rows, cfg.xbar_cols
    D = np.zeros_like(G)
    for s in range(S):
        for pol in range(2):
            for k0 in range(0, K, R):
                for n0 in range(0, N, C):
                    tile = np.zeros((R, C))
                    rows, cols = min(R, K - k0), min(C, N - n0)
                    tile[:rows, :cols] = G[s, pol, k0:k0 + rows, n0:n0 + cols]
                    E = nodal.effective_conductance_sparse(tile, cfg.r_row, cfg.r_col, cfg.r_source, cfg.r_sense)
                    g = tile[:rows, :cols]
                    D[s, pol, k0:k0 + rows, n0:n0 + cols] = (g - E[:rows, :cols]) / g
    return D
