"""A deviation matrix written out by hand for the layer-range profiler's tests (Section 4.2, Eq. 2-4).

Five tokens, twelve layers.  Layer l's deviations are (1 - s_l) * (1 + 0.1 (rank - 3)), so the layer mean is exactly
1 - s_l and the token ranking of every layer is the permutation listed below.  With n = 5 and no ties the Spearman
correlation of two rankings is 1 - sum(delta^2) / 20.

  layer  ranks of tokens 0..4   sum delta^2 to the layer before   rho_l
    0    1 2 3 4 5
    1    5 4 3 2 1              16+4+0+4+16 = 40                  -1.0
    2    1 4 3 2 5              16+0+0+0+16 = 32                  -0.6
    3    4 1 2 3 5               9+9+1+1+0  = 20                   0.0
    4    3 1 2 5 4               1+0+0+4+1  =  6                   0.7
    5    3 2 1 5 4               0+1+1+0+0  =  2                   0.9
    6..11 as layer 5                          0                    1.0

Second difference alpha_l = rho_l - 2 rho_{l-1} + rho_{l-2} (rho_l compares layers l-1 and l, so alpha exists from l = 3):
  alpha_3 =  0.0 + 1.2 - 1.0 = +0.2
  alpha_4 =  0.7 - 0.0 - 0.6 = +0.1
  alpha_5 =  0.9 - 1.4 + 0.0 = -0.5      <- first layer whose alpha is negative right after a positive one: l* = 5
  alpha_6 =  1.0 - 1.8 + 0.7 = -0.1
  alpha_7 =  1.0 - 2.0 + 0.9 = -0.1
  alpha_8.. = 0
so the detection layer is l* + 1 = 6.  (Had l* been the last positive layer, or the "+ 1" been dropped, the answer
would be 5; had rho_l compared layers l and l+1, alpha would move one layer down and the answer would be 5 as well.)

Similarity profile: s = 0.999 0.995 0.992 0.97 0.90 0.85 0.88 0.93 0.95 0.955 0.953 0.956, worked by hand:
minimum at layer 5; deepest layer <= 5 with s >= 0.99 is 2; last five layers have mean 0.9488 and population
standard deviation 0.00962, so b = 0.93918 and 2 sigma = 0.01924; scanning from layer 5, layer 8 is the first one
followed by two layers that stay above b with steps below 2 sigma (0.005, 0.002): l_end = 8.  6 lies in (2, 8].
"""
import numpy as np

RANKS = [[1, 2, 3, 4, 5], [5, 4, 3, 2, 1], [1, 4, 3, 2, 5], [4, 1, 2, 3, 5], [3, 1, 2, 5, 4]] + [[3, 2, 1, 5, 4]] * 7
S = [0.999, 0.995, 0.992, 0.97, 0.90, 0.85, 0.88, 0.93, 0.95, 0.955, 0.953, 0.956]
RHO = [0.0, -1.0, -0.6, 0.0, 0.7, 0.9, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0]          # rho_0 is undefined (reported as 0)
ALPHA = [0.0, 0.0, 0.0, 0.2, 0.1, -0.5, -0.1, -0.1, 0.0, 0.0, 0.0, 0.0]       # alpha_0..2 undefined (reported as 0)
TRIPLE = (2, 6, 8)                                                            # (l_start, l_det, l_end)


def deviations(ranks=RANKS, s=S) -> np.ndarray:
    """d[token][layer], float64."""
    r = np.asarray(ranks, np.float64).T                    # [token][layer]
    return (1.0 - np.asarray(s, np.float64))[None, :] * (1.0 + 0.1 * (r - 3.0))
