"""k-nearest-neighbour index tensors (self included), int32 [K,N]."""
import numpy as np


def knn_bruteforce(pts, k, chunk=1024):
    """Exact k-NN by the full distance matrix; ties by (d^2, index)."""
    p = np.asarray(pts, np.float64)
    n = p.shape[0]
    out = np.empty((n, k), np.int32)
    for r0 in range(0, n, chunk):
        q = p[r0:r0 + chunk]
        d2 = np.zeros((q.shape[0], n))
        for a in range(p.shape[1]):
            d2 += (q[:, a:a + 1] - p[None, :, a]) ** 2
        if k < n:
            # candidates: everything not farther than the k-th smallest distance
            kth = np.partition(d2, k - 1, axis=1)[:, k - 1:k]
            for r in range(q.shape[0]):
                cand = np.nonzero(d2[r] <= kth[r, 0])[0]          # ascending index
                sel = cand[np.argsort(d2[r, cand], kind="stable")[:k]]
                out[r0 + r] = sel
        else:
            out[r0:r0 + chunk] = np.argsort(d2, axis=1, kind="stable")[:, :k]
    return np.ascontiguousarray(out.T)


def knn_kdtree(pts, k, workers=-1):
    """Exact k-NN with a kD-tree (neighbourhoods computed once upfront)."""
    from scipy.spatial import cKDTree
    p = np.asarray(pts, np.float64)
    tree = cKDTree(p)
    _, idx = tree.query(p, k=k, workers=workers)
    if k == 1:
        idx = idx[:, None]
    return np.ascontiguousarray(idx.T.astype(np.int32))
