"""Tolerance for gradient-descent weights when the inputs of every product are rounded to bfloat16.

The task fixes 1e-4 for float32 weights and 5e-3 for single reduced-precision operators, and nothing for the
weights the reduced-precision variant reaches after N iterations of Alg. 1.  This bound is derived from the
arithmetic; ``tests/test_oracle_pins.py`` checks it on the CPU against an emulation of that arithmetic
(``oracle.gd_bf16_inputs``) before the device tests use it.

Notation: u = 2^-8 is the unit roundoff of bfloat16 (8 significant bits, round to nearest), H = T^T T / r_T,
gamma the learning rate, x_max = gamma * lambda_max(H) (< 2: the iteration is stable), rho = max(0, x_max - 1).

1. Weights.  The variant multiplies by rd(w) = w + dw with |dw| <= u |w| componentwise, so its iteration is
   w+ = w - gamma (H (w + dw) - b): Alg. 1 with the extra term -gamma H dw_t in every step.  The difference d_t
   to the exact iterates obeys d_{t+1} = (I - gamma H) d_t - gamma H dw_t, hence
   ||d_N|| <= sum_s ||gamma H (I - gamma H)^s|| * u * max_t ||w_t||,   s = 0 .. N-1.
   All matrices are functions of H, so the norm is max over eigenvalues x = gamma*lambda in [0, x_max] of
   |x (1 - x)^s|.  For x <= 1 the maximum is at x = 1/(s+1) and is at most 1 (s = 0) or 1/(2 (s+1)) (s >= 1,
   because (1 + 1/s)^s >= 2); for 1 < x <= x_max it is at most x_max rho^s.  Summed over s:
   1 + ln(N)/2 + x_max rho / (1 - rho).
2. Table, residual and segment-sum rounding perturb the gradient by products of independent relative errors
   of size <= u with the data; for tables with independent entries such a sum over r_T rows, divided by r_T,
   is of relative size u sqrt(c_T / r_T) per source of error (the usual square-root law of rounding-error
   sums).  Four such terms are allowed for: 4 u sqrt(c_T / r_T).  This part is a statistical estimate, which is
   why the CPU test checks the whole bound against the emulation on every kind of schema the device tests use.

Relative to ||w_N|| (from w_0 = 0 the exact iterates grow towards the least-squares solution, so
max_t ||w_t|| is ||w_N|| to first order):

    tol = u * (1 + ln(N)/2 + x_max rho / (1 - rho) + 4 sqrt(c_T / r_T)).
"""
import math

import numpy as np

BF16_UNIT_ROUNDOFF = 2.0 ** -8


def lambda_max(gram: np.ndarray, r_T: int) -> float:
    """Largest eigenvalue of H = T^T T / r_T, from the Gram matrix of the target table."""
    return float(np.linalg.eigvalsh(np.asarray(gram, dtype=np.float64) / r_T)[-1])


def bf16_gd_weight_tol(iters: int, c_T: int, r_T: int, lr: float, lam_max: float) -> float:
    x_max = float(lr) * float(lam_max)
    assert 0.0 <= x_max < 2.0, f"learning rate {lr} is outside the stable range of Alg. 1 (lambda_max {lam_max})"
    rho = max(0.0, x_max - 1.0)
    return BF16_UNIT_ROUNDOFF * (1.0 + 0.5 * math.log(max(iters, 1)) + x_max * rho / (1.0 - rho)
                                 + 4.0 * math.sqrt(c_T / r_T))
