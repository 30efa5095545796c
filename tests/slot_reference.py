"""Expected contents of the ring store, built on the CPU from the oracle's own shard splitting.

Test helper (not a test): the rows / columns of a shard come from the oracle's `_split_rows` / `_split_cols`
(the partition the rotated oracle computes on), so a slot written by rtp_pack_shards can be compared byte for byte
with what the oracle would hold in `home[k]`.  A partition that does not divide evenly is zero-padded to the width
the library documents (include/rtp.h, rtp_shard_width) before it is split: the padding rows / columns are extra
zeros, nothing else moves."""
import numpy as np

import oracle as orc


def _pad_to(W, rows, cols):
    out = np.zeros((rows, cols), dtype=W.dtype)
    out[:W.shape[0], :W.shape[1]] = W
    return out


def matrix_parts(W, n, split_out, width):
    """The n shard parts of W[O, I], each flattened in storage order: row blocks [w, I] (output partition) or
    column blocks stored [O, w] (input partition)."""
    O, I = W.shape
    if split_out:
        parts = orc._impl._split_rows(_pad_to(W, n * width, I), n)
    else:
        parts = orc._impl._split_cols(_pad_to(W, O, n * width), n)
    assert all(p.shape == ((width, I) if split_out else (O, width)) for p in parts)
    return [np.ascontiguousarray(p).reshape(-1) for p in parts]


def vector_parts(b, n, width):
    """Bias entries [k w, (k+1) w) per shard, zero-padded: a vector is a one-column matrix split by rows."""
    return matrix_parts(np.asarray(b).reshape(-1, 1), n, True, width)


def slots(n, slot_elems, placed):
    """`placed`: list of (element offset, parts) -> array [n, slot_elems] with every part at its offset, zero elsewhere."""
    dtype = placed[0][1][0].dtype
    out = np.zeros((n, slot_elems), dtype=dtype)
    for off, parts in placed:
        for k in range(n):
            out[k, off:off + parts[k].size] = parts[k]
    return out
