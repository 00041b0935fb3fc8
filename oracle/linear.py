"""fp64 oracle: a linear layer over the tokens of a pass (TEST INFRASTRUCTURE).

The forward pass whose cost the paper reasons about (Sec. 3.1: a pass is bound by reading the
weights while it holds few tokens and by compute once it holds many, which is what fixes a
sensible token budget) consists, besides attention, of dense projections applied to every
token of the ragged batch: the query/key/value and output projections and the gated MLP of the
served model family (Sec. 4.1, Llama-2).  Each is the textbook linear map

    y[t, o] = sum_k x[t, k] * w[o, k]            t: token of the pass, o: output feature

with the weight stored one output feature per row (``w`` is ``[n_out, k]``, the layout in which
such models keep their weights).  The oracle is that definition written out in float64 on the
exactly converted storage values; numpy's matmul is the only library step.  No blocking, no
reordering, no rounding of the result.
"""
from __future__ import annotations

import numpy as np

from .attention import to_f64


def linear(x: np.ndarray, w: np.ndarray, dtype: str) -> np.ndarray:
    """``x [n_tokens, k]``, ``w [n_out, k]`` as storage arrays -> ``float64 [n_tokens, n_out]``."""
    assert x.ndim == 2 and w.ndim == 2 and x.shape[1] == w.shape[1]
    return to_f64(x, dtype) @ to_f64(w, dtype).T
