"""Integer oracle for the graph layout -- TEST INFRASTRUCTURE.

The transition matrix T of the paper (Matrix-based implementation section)
stores only the arcs that are not the semiring zero (Using-the-Julia-language
section).  The forward recursion multiplies by T transposed, i.e. gathers the
arcs that *enter* a state; the backward recursion multiplies by T, i.e.
gathers the arcs that *leave* it.  The two compressed layouts are therefore
the arc list stably sorted by destination and by source; the pdf grouping is
the state list stably sorted by pdf id.  "Stable" = ties keep ascending
original index, which makes each layout unique.  numpy's stable argsort is the
library primitive used as the definition.
"""
from __future__ import annotations

import numpy as np


def compressed(keys: np.ndarray, n_keys: int):
    """(ptr[n_keys+1], perm) with perm the stable ascending order of keys."""
    keys = np.asarray(keys, dtype=np.int64)
    perm = np.argsort(keys, kind="stable").astype(np.int32)
    ptr = np.zeros(n_keys + 1, dtype=np.int32)
    np.cumsum(np.bincount(keys, minlength=n_keys), out=ptr[1:])
    return ptr, perm


def graph_layout(K: int, D: int, src, dst, logw, pdf) -> dict:
    src = np.asarray(src, dtype=np.int32)
    dst = np.asarray(dst, dtype=np.int32)
    logw = np.asarray(logw, dtype=np.float32)
    in_ptr, in_perm = compressed(dst, K)
    out_ptr, out_perm = compressed(src, K)
    pdf_ptr, pdf_states = compressed(pdf, D)
    return {
        "in_ptr": in_ptr, "in_perm": in_perm, "in_src": src[in_perm], "in_w": logw[in_perm],
        "out_ptr": out_ptr, "out_perm": out_perm, "out_dst": dst[out_perm], "out_w": logw[out_perm],
        "pdf_ptr": pdf_ptr, "pdf_states": pdf_states,
    }
