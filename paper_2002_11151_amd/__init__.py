"""MI355X-native emulation of non-ideal resistive-crossbar training operations (TxSim hot path).

`paper_2002_11151_amd.xbar` is the thin binding over the C-ABI library `libxbar.so` (HIP kernels for
gfx950).  Importing the package does not load the library; the first call does and fails loudly if
the library has not been built.
"""
