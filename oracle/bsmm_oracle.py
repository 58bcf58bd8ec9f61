"""CPU oracle for the general block-sparse products.  TEST INFRASTRUCTURE ONLY.

Only tests/ may import this module; the product (the HIP library and its binding) never does.

What is computed, and from where in the paper: Section 4.2 names the block-sparse products by the sparsity of
output and inputs (SDD: sparse output, dense inputs; DSD: dense output, sparse left input) and Section 5.1 lists
the transposed variants that a two-layer network's backward pass needs.  With S a matrix whose 128x128 blocks are
present where `mask` is nonzero and absent (zero) elsewhere, the definitions are simply dense products:

    SDD   S = (X W)   restricted to the mask          SDD^T  S = (X W^T) restricted to the mask
    DSD   Y = S W                                      DSD^T  Y = S W^T
    DS^TD Y = S^T X                                    DD^TS  Y = X^T S
    DDS   Y = X S     (dense output, sparse right input; named in Section 5.1.1, not used by the layer)

and the remaining combinations of transposed inputs that Section 5.1.1 counts (a T after the operand's letter):

    SD^TD   S = (X^T W)   on the mask                  SD^TD^T  S = (X^T W^T) on the mask
    DS^TD^T Y = S^T X^T                                DDS^T    Y = X S^T            DD^TS^T  Y = X^T S^T

and that is what this file writes out: densify, multiply in float64, restrict.  The values of S travel as
[nnz, 128, 128] in the row-wise order of the nonzero blocks (ascending row, ascending column inside a row), which is
the order of the blocked-CSR encoding (Section 5.1.3).

Pins (tests/test_oracle_bsmm.py): scipy.sparse block-CSR matrices built from the same blocks (an independent
library's notion of block order, products and transposes), the all-ones mask against plain dense products, the
empty mask, and the algebraic identity <S, X W> = <Y, S W^T ...> style adjoint checks between forward and
transposed products.
"""
from __future__ import annotations

import numpy as np

BLOCK = 128


def block_order(mask: np.ndarray):
    """(rows, cols) of the nonzero blocks in row-wise order."""
    r, c = np.nonzero(np.asarray(mask) != 0)       # numpy returns row-major order: ascending row, then column
    return r.astype(np.int64), c.astype(np.int64)


def densify(values: np.ndarray, mask: np.ndarray, block: int = BLOCK) -> np.ndarray:
    """[nnz, block, block] -> dense [R*block, C*block] float64 with zeros where the mask is zero."""
    R, C = mask.shape
    out = np.zeros((R * block, C * block), dtype=np.float64)
    r, c = block_order(mask)
    assert values.shape == (len(r), block, block)
    for b in range(len(r)):
        out[r[b] * block:(r[b] + 1) * block, c[b] * block:(c[b] + 1) * block] = values[b]
    return out


def sample(dense: np.ndarray, mask: np.ndarray, block: int = BLOCK) -> np.ndarray:
    """dense [R*block, C*block] -> [nnz, block, block]: the blocks the mask keeps, row-wise order."""
    r, c = block_order(mask)
    out = np.empty((len(r), block, block), dtype=np.float64)
    for b in range(len(r)):
        out[b] = dense[r[b] * block:(r[b] + 1) * block, c[b] * block:(c[b] + 1) * block]
    return out


def sdd(x: np.ndarray, w: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """S = (X W) on the mask.  x [M, D], w [D, N]."""
    return sample(x.astype(np.float64) @ w.astype(np.float64), mask)


def sddt(x: np.ndarray, w: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """S = (X W^T) on the mask.  x [M, D], w [N, D]."""
    return sample(x.astype(np.float64) @ w.astype(np.float64).T, mask)


def dsd(s: np.ndarray, w: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = S W.  s [nnz, 128, 128], w [N, D]."""
    return densify(s.astype(np.float64), mask) @ w.astype(np.float64)


def dsdt(s: np.ndarray, w: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = S W^T.  w [D, N]."""
    return densify(s.astype(np.float64), mask) @ w.astype(np.float64).T


def dstd(s: np.ndarray, x: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = S^T X.  x [M, D], Y [N, D]."""
    return densify(s.astype(np.float64), mask).T @ x.astype(np.float64)


def ddts(x: np.ndarray, s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = X^T S.  x [M, D], Y [D, N]."""
    return x.astype(np.float64).T @ densify(s.astype(np.float64), mask)


def dds(x: np.ndarray, s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = X S.  x [D, M], Y [D, N]."""
    return x.astype(np.float64) @ densify(s.astype(np.float64), mask)


# ---- the remaining combinations of transposed inputs (Section 5.1.1)
def sdtd(x: np.ndarray, w: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """S = (X^T W) on the mask.  x [D, M], w [D, N]."""
    return sample(x.astype(np.float64).T @ w.astype(np.float64), mask)


def sdtdt(x: np.ndarray, w: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """S = (X^T W^T) on the mask.  x [D, M], w [N, D]."""
    return sample(x.astype(np.float64).T @ w.astype(np.float64).T, mask)


def dstdt(s: np.ndarray, x: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = S^T X^T.  x [D, M], Y [N, D]."""
    return densify(s.astype(np.float64), mask).T @ x.astype(np.float64).T


def ddst(x: np.ndarray, s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = X S^T.  x [D, N], Y [D, M]."""
    return x.astype(np.float64) @ densify(s.astype(np.float64), mask).T


def ddtst(x: np.ndarray, s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Y = X^T S^T.  x [N, D], Y [D, M]."""
    return x.astype(np.float64).T @ densify(s.astype(np.float64), mask).T
