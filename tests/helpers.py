"""Small shared helpers for the tests (input construction only)."""
import numpy as np

import oracle


def csc_from_dense(counts: np.ndarray) -> oracle.CSC:
    """counts[d][w] (integers) -> CSC with documents as columns."""
    D, V = counts.shape
    colptr = [0]
    rowidx, val = [], []
    for d in range(D):
        nz = np.nonzero(counts[d])[0]
        rowidx.extend(nz.tolist())
        val.extend(counts[d, nz].tolist())
        colptr.append(len(rowidx))
    return oracle.CSC(D, V, np.array(colptr, np.int32), np.array(rowidx, np.int32), np.array(val, np.float32))


def corpus_to_csc(c) -> oracle.CSC:
    return oracle.CSC(c.D, c.V, c.colptr.cpu().numpy(), c.rowidx.cpu().numpy(), c.val.cpu().numpy())
