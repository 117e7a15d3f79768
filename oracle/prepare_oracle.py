"""Oracle for the host-side model preparation (test infrastructure, not the product).

Two small definitions from the paper, written out plainly in float64 numpy:

* ternary weights (Eq. 4): Delta = 0.7/n * sum|W_i|;  W~_i = +1 if W_i > Delta, 0 if |W_i| <= Delta,
  -1 otherwise;  alpha = (sum over nonzero W~ of |W_i|) / n_Delta.  Taken per output filter: the
  paper keeps a single full-precision scale per feature channel (section 2, last paragraph).
* the activation of Eq. 6 applied to y = a*acc + b, where a and b collect the weight scale alpha
  and the batch-norm affine (section 2: batch-norm sits between the ternary convolution and the
  activation):  code(acc) = +1 if y > 0.5, 0 if |y| <= 0.5, -1 otherwise, evaluated in float64.

* ternary weights with a prescribed sparsity (section 2, the remark after Eq. 9): Delta is not
  taken from Eq. 4 but placed so that a given number of entries of every kernel falls at or
  below it (the paper's example: exactly half).  Reading taken here, the paper gives no more than
  that sentence: "kernel" = one output filter (the unit that has its own alpha); the `zeros`
  entries of smallest magnitude become 0, equal magnitudes in index order; the others get their
  sign (an entry that is exactly 0 stays 0); alpha as in Eq. 4, the mean magnitude of the entries
  kept.  How this halves the bit-counts is not explained in the paper and is not modelled.

Pins: tests/test_prepare.py (hand-worked vectors, scale equivariance, Gaussian zero fraction,
exhaustive agreement of integer cut points with the float64 evaluation; for the prescribed
sparsity: hand-worked vector with ties, zero count, separation by a threshold, agreement with
Eq. 4 when given Eq. 4's own zero count, Gaussian median).
"""
import numpy as np


def ternarize_filters(w: np.ndarray):
    """w: float [C_out][...].  Returns (int8 codes of the same shape, float64 alpha[C_out])."""
    w64 = np.asarray(w, dtype=np.float64)
    flat = w64.reshape(w64.shape[0], -1)
    codes = np.zeros(flat.shape, dtype=np.int8)
    alpha = np.zeros(flat.shape[0], dtype=np.float64)
    for co in range(flat.shape[0]):
        row = flat[co]
        delta = 0.7 * np.sum(np.abs(row)) / row.size
        t = np.where(row > delta, 1, np.where(np.abs(row) <= delta, 0, -1)).astype(np.int8)
        n_delta = int(np.count_nonzero(t))
        alpha[co] = (np.sum(np.abs(row)[t != 0]) / n_delta) if n_delta else 0.0
        codes[co] = t
    return codes.reshape(w64.shape), alpha


def ternarize_filters_sparse(w: np.ndarray, zeros: int):
    """w: float [C_out][...]; zeros: entries per filter that become 0 (0 <= zeros <= entries).
    Returns (int8 codes of the same shape, float64 alpha[C_out])."""
    w64 = np.asarray(w, dtype=np.float64)
    flat = w64.reshape(w64.shape[0], -1)
    if not 0 <= zeros <= flat.shape[1]:
        raise ValueError("zeros out of range")
    codes = np.zeros(flat.shape, dtype=np.int8)
    alpha = np.zeros(flat.shape[0], dtype=np.float64)
    for co in range(flat.shape[0]):
        row = flat[co]
        order = np.argsort(np.abs(row), kind="stable")     # smallest magnitude first, ties by index
        keep = order[zeros:]
        t = np.zeros(row.size, dtype=np.int8)
        t[keep] = np.sign(row[keep]).astype(np.int8)
        n_kept = int(np.count_nonzero(t))
        alpha[co] = (np.sum(np.abs(row)[t != 0]) / n_kept) if n_kept else 0.0
        codes[co] = t
    return codes.reshape(w64.shape), alpha


def bn_affine(alpha, gamma, beta, mean, var, eps):
    """y = a*acc + b for conv scale alpha followed by batch-norm (gamma, beta, mean, var, eps)."""
    alpha, gamma, beta, mean, var = (np.asarray(v, dtype=np.float64) for v in (alpha, gamma, beta, mean, var))
    inv = 1.0 / np.sqrt(var + eps)
    return alpha * gamma * inv, beta - gamma * mean * inv


def activation_code(acc, a, b):
    """Eq. 6 on y = a*acc + b in float64, for integer acc (any shape) and scalars a, b."""
    y = np.float64(a) * np.asarray(acc, dtype=np.float64) + np.float64(b)
    return np.where(y > 0.5, 1, np.where(np.abs(y) <= 0.5, 0, -1)).astype(np.int8)
