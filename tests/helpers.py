"""Independent numpy formulations used to pin the oracle (none of them calls the oracle)."""
import numpy as np


def to_np(index):
    return {k: (v.detach().cpu().numpy() if hasattr(v, "detach") else np.asarray(v)) for k, v in index.items()}


def list_of(index):
    """List number of every list-major row."""
    off = index["list_offsets"]
    return np.repeat(np.arange(len(off) - 1), np.diff(off))


def reconstruct(index):
    """x_hat[i] = C[list(i)] + concat_j CB[j][code[i][j]] in fp64, list-major rows."""
    C = index["centroids"].astype(np.float64)
    CB = index["codebooks"].astype(np.float64)
    codes = index["codes"]
    m = CB.shape[0]
    parts = [CB[j][codes[:, j]] for j in range(m)]
    return C[list_of(index)] + np.concatenate(parts, axis=1)


def topk_desc(keys, ids, k):
    """Best k by (key descending, id ascending) via a full lexicographic sort."""
    order = np.lexsort((ids, -keys))[:k]
    return ids[order], keys[order]
