"""Oracle of the copy steps around the attention call -- TEST INFRASTRUCTURE ONLY.

The definitions written out in numpy on raw bf16 bits (uint16): grouping q, k, v of a batch side
by side in one row per request (Sec. 3.2.1, step 2), and placing returned rows among the rows of
the decode batch's output (the "merging outputs" kernel of Sec. 3.2.2).  Shares nothing with the
library."""
import numpy as np


def pack_qkv(q, k, v, width=None, fill=0):
    """q [B,Hq,d], k, v [B,Hkv,d] (uint16 bits) -> [B, width] with q | k | v at the row start."""
    B = q.shape[0]
    row = [np.concatenate([q[b].reshape(-1), k[b].reshape(-1), v[b].reshape(-1)]) for b in range(B)]
    n = row[0].size if B else 0
    width = n if width is None else width
    out = np.full((B, width), fill, dtype=np.uint16)
    for b in range(B):
        out[b, :n] = row[b]
    return out


def scatter_rows(dst, src, row_index):
    """dst[row_index[i]] = src[i]; an index outside dst's rows skips the row.  Returns a copy."""
    out = dst.copy()
    for i, r in enumerate(row_index):
        if 0 <= r < out.shape[0]:
            out[r] = src[i]
    return out
