"""Operation-count model of the paper's efficiency analysis (sec. 4.1).

A standard convolution costs c*N_W*N_I high-precision operations per filter; the binary
convolution costs c*N_W*N_I binary operations plus N_I non-binary ones.  With `lanes`
binary operations per clock the speed-up is
    S = c*N_W*N_I / (c*N_W*N_I/lanes + N_I) = lanes*c*N_W / (c*N_W + lanes),
independent of the input size N_I.  The paper evaluates it with lanes = 64.
Used only for reporting next to measured numbers.
"""


def standard_conv_ops(c: int, n_w: int, n_i: int) -> int:
    return c * n_w * n_i


def binary_conv_ops(c: int, n_w: int, n_i: int):
    """(binary operations, non-binary operations) per filter."""
    return c * n_w * n_i, n_i


def theoretical_speedup(c: int, n_w: int, n_i: int = 1, lanes: int = 64) -> float:
    binary, non_binary = binary_conv_ops(c, n_w, n_i)
    return standard_conv_ops(c, n_w, n_i) / (binary / lanes + non_binary)
