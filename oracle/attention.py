"""fp64 oracle: blocked KV-cache append and ragged causal attention (TEST INFRASTRUCTURE).

What is computed (own words, following the paper):

* A sequence is served in forward passes.  A pass hands the model ``n_new`` tokens of
  the sequence while ``n_cached`` earlier tokens already sit in the KV cache: a prompt
  pass hands over many tokens, a generation pass exactly one (Sec. 2, the two phases).
* The cache is a pool of fixed-size blocks; a sequence owns a list of block ids that
  need not be contiguous (Sec. 2.1).
* Dynamic SplitFuse may cut one prompt into chunks that run in different passes
  (Sec. 3.2, rule 1).  That changes scheduling only: every token must still attend to
  all earlier tokens of its own sequence, wherever and whenever they were cached.

The paper does not print the attention formula; it is the textbook causal scaled
dot-product attention of the model families it serves (Sec. 5, supported models).  For
new row ``i`` of a sequence (absolute position ``p = n_cached + i``), query head ``hq``
sharing KV head ``hk = hq // g`` with ``g = Hq // Hkv``::

    J   = { j : 0 <= j <= p  and (window == 0 or p - j < window) }
    s_j = scale * <q[i, hq, :], k[j, hk, :]>
    o   = sum_{j in J} softmax_J(s)_j * v[j, hk, :]

Everything is dense, two-pass (max, then exp/sum), in float64.  No tiling, no running
softmax, no reordering.  numpy's matmul is the only library step.

Storage conventions shared with the library's public header (a format, not code):

* caches:       ``[num_blocks, Hkv, block_size, d]``, K and V separate
* token tensors ``[T, H, d]``, sequences back to back in descriptor order
* descriptor    ``(n_new, n_cached, q_offset, seq_id)`` as int32
* block table   ``int32 [S, max_blocks]``, unused entries ``-1``
* bf16 is carried as its uint16 bit pattern (numpy has no bf16)

Append happens first; attention then reads all ``n_cached + n_new`` tokens from the cache.
"""
from __future__ import annotations

import numpy as np

DESC_N_NEW, DESC_N_CACHED, DESC_Q_OFFSET, DESC_SEQ_ID = 0, 1, 2, 3


# --------------------------------------------------------------------------------------
# exact storage -> float64 conversion
# --------------------------------------------------------------------------------------
def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Convert stored values to float64 exactly (every bf16/f16/f32 is an f64)."""
    if dtype == "f32":
        assert x.dtype == np.float32
        return x.astype(np.float64)
    if dtype == "f16":
        assert x.dtype == np.float16
        return x.astype(np.float64)
    if dtype == "bf16":
        assert x.dtype == np.uint16, "bf16 travels as uint16 bit patterns"
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------------------
# blocked cache: append and gather  (Sec. 2.1)
# --------------------------------------------------------------------------------------
def kv_append(k_cache, v_cache, k_new, v_new, descs, block_tables, block_size: int) -> None:
    """Copy this pass's new K/V rows into their cache slots, bit for bit, in place.

    Token ``i`` of sequence ``s`` has position ``p = n_cached + i`` and lands in physical
    block ``block_tables[s, p // block_size]`` at slot ``p % block_size``.  No other
    slot is touched.
    """
    descs = np.asarray(descs)
    for s in range(descs.shape[0]):
        n_new = int(descs[s, DESC_N_NEW])
        n_cached = int(descs[s, DESC_N_CACHED])
        q_off = int(descs[s, DESC_Q_OFFSET])
        for i in range(n_new):
            p = n_cached + i
            blk = int(block_tables[s, p // block_size])
            slot = p % block_size
            assert blk >= 0, "position falls on an unassigned block-table entry"
            k_cache[blk, :, slot, :] = k_new[q_off + i]
            v_cache[blk, :, slot, :] = v_new[q_off + i]


def f32_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the storage type, nearest with ties to even (bf16 as uint16 bits)."""
    assert x.dtype == np.float32
    if dtype == "f32":
        return x.copy()
    if dtype == "f16":
        return x.astype(np.float16)           # numpy rounds to nearest even
    if dtype == "bf16":
        bits = x.view(np.uint32).astype(np.uint64)
        keep, drop = bits >> np.uint64(16), bits & np.uint64(0xFFFF)
        up = (drop > 0x8000) | ((drop == 0x8000) & ((keep & np.uint64(1)) == 1))
        return (keep + up.astype(np.uint64)).astype(np.uint16)   # finite inputs; a carry moves to the exponent
    raise ValueError(f"unknown dtype {dtype!r}")


def rotary_table(n_positions: int, head_dim: int, theta: float = 10000.0) -> np.ndarray:
    """``float32 [n_positions, head_dim // 2, 2]``: cos and sin of ``p * theta ** (-2 i / head_dim)``,
    evaluated in float64 and rounded once (the rotary position embedding of the Llama family,
    which the paper's evaluation serves, Sec. 4.1)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    ang = np.arange(n_positions, dtype=np.float64)[:, None] * theta ** (-2.0 * i / head_dim)[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def rotate_row(k_row: np.ndarray, cos_sin_p: np.ndarray, dtype: str) -> np.ndarray:
    """Rotate one stored K row ``[Hkv, d]`` by its position's angles (half-split pairing: element
    ``i`` pairs with ``i + d/2``)::

        k'[i]       = k[i] * cos_i - k[i + d/2] * sin_i
        k'[i + d/2] = k[i + d/2] * cos_i + k[i] * sin_i

    The arithmetic is fixed so that the cache stays bit-exact: every product and the sum or
    difference of the two products is a float32 operation rounded to nearest even (no fused
    multiply-add), and the result is rounded once more to the storage type."""
    d = k_row.shape[-1]
    k = to_f64(k_row, dtype).astype(np.float32)      # exact: storage values are float32 values
    a, b = k[..., : d // 2], k[..., d // 2:]
    c, s = cos_sin_p[:, 0][None, :], cos_sin_p[:, 1][None, :]
    lo = (a * c).astype(np.float32) - (b * s).astype(np.float32)
    hi = (b * c).astype(np.float32) + (a * s).astype(np.float32)
    return f32_to_storage(np.concatenate([lo, hi], axis=-1).astype(np.float32), dtype)


def kv_append_rotary(k_cache, v_cache, k_new, v_new, descs, block_tables, block_size: int,
                     cos_sin: np.ndarray, dtype: str) -> None:
    """As :func:`kv_append`, but every K row is rotated by the angles of its position before it
    is stored (V is copied bit for bit)."""
    descs = np.asarray(descs)
    for s in range(descs.shape[0]):
        n_new = int(descs[s, DESC_N_NEW])
        n_cached = int(descs[s, DESC_N_CACHED])
        q_off = int(descs[s, DESC_Q_OFFSET])
        for i in range(n_new):
            p = n_cached + i
            blk = int(block_tables[s, p // block_size])
            slot = p % block_size
            assert blk >= 0, "position falls on an unassigned block-table entry"
            k_cache[blk, :, slot, :] = rotate_row(k_new[q_off + i], cos_sin[p], dtype)
            v_cache[blk, :, slot, :] = v_new[q_off + i]


def rotate_queries(q, descs, cos_sin: np.ndarray, dtype: str) -> np.ndarray:
    """The pass's query rows ``[T, Hq, d]`` rotated like the keys (:func:`rotate_row`): row ``i`` of
    sequence ``s`` by the angles of its position ``n_cached + i``.  Returns a new array."""
    descs = np.asarray(descs)
    out = np.empty_like(q)
    for s in range(descs.shape[0]):
        n_new, n_cached, q_off = int(descs[s, DESC_N_NEW]), int(descs[s, DESC_N_CACHED]), int(descs[s, DESC_Q_OFFSET])
        for i in range(n_new):
            out[q_off + i] = rotate_row(q[q_off + i], cos_sin[n_cached + i], dtype)
    return out


def gather_history(cache, block_table_row, n_tokens: int, block_size: int) -> np.ndarray:
    """Logical history ``[n_tokens, Hkv, d]`` of one sequence, in position order."""
    n_heads, d = cache.shape[1], cache.shape[3]
    out = np.empty((n_tokens, n_heads, d), dtype=cache.dtype)
    for j in range(n_tokens):
        blk = int(block_table_row[j // block_size])
        assert blk >= 0
        out[j] = cache[blk, :, j % block_size, :]
    return out


# --------------------------------------------------------------------------------------
# dense attention for one sequence
# --------------------------------------------------------------------------------------
def visible_mask(n_new: int, n_cached: int, window: int) -> np.ndarray:
    """Boolean ``[n_new, n_cached + n_new]``: may row i look at key j?"""
    p = n_cached + np.arange(n_new)[:, None]
    j = np.arange(n_cached + n_new)[None, :]
    vis = j <= p
    if window > 0:
        vis &= (p - j) < window
    return vis


def softmax_weights(q_s, k_s, n_cached: int, scale: float, window: int, group: int) -> np.ndarray:
    """Attention weights ``[Hq, n_new, L]`` (rows sum to one, hidden keys get zero)."""
    n_new, n_q_heads, _ = q_s.shape
    vis = visible_mask(n_new, n_cached, window)
    w = np.zeros((n_q_heads, n_new, k_s.shape[0]), dtype=np.float64)
    for hq in range(n_q_heads):
        hk = hq // group
        s = scale * (q_s[:, hq, :] @ k_s[:, hk, :].T)
        s = np.where(vis, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        w[hq] = e / e.sum(axis=1, keepdims=True)
    return w


def attention_one_sequence(q_s, k_s, v_s, n_cached: int, scale: float, window: int = 0) -> np.ndarray:
    """``q_s [n_new, Hq, d]``, ``k_s, v_s [n_cached + n_new, Hkv, d]`` (all float64)."""
    n_new, n_q_heads, d = q_s.shape
    n_kv_heads = k_s.shape[1]
    assert k_s.shape[0] == n_cached + n_new and v_s.shape == k_s.shape
    assert n_q_heads % n_kv_heads == 0
    group = n_q_heads // n_kv_heads
    w = softmax_weights(q_s, k_s, n_cached, scale, window, group)
    out = np.empty((n_new, n_q_heads, d), dtype=np.float64)
    for hq in range(n_q_heads):
        out[:, hq, :] = w[hq] @ v_s[:, hq // group, :]
    return out


# --------------------------------------------------------------------------------------
# the ragged batch
# --------------------------------------------------------------------------------------
def ragged_attention(q, k_cache, v_cache, descs, block_tables, *, block_size: int, scale: float,
                     window: int = 0, dtype: str = "f32", seq_subset=None) -> np.ndarray:
    """Attention outputs ``float64 [T, Hq, d]`` for a whole ragged batch.

    The caches must already contain this pass's tokens (call :func:`kv_append` first).
    ``seq_subset`` restricts the work to some descriptor indices; other rows stay NaN.
    """
    descs = np.asarray(descs)
    out = np.full(q.shape, np.nan, dtype=np.float64)
    seqs = range(descs.shape[0]) if seq_subset is None else seq_subset
    for s in seqs:
        n_new = int(descs[s, DESC_N_NEW])
        n_cached = int(descs[s, DESC_N_CACHED])
        q_off = int(descs[s, DESC_Q_OFFSET])
        total = n_cached + n_new
        k_s = to_f64(gather_history(k_cache, block_tables[s], total, block_size), dtype)
        v_s = to_f64(gather_history(v_cache, block_tables[s], total, block_size), dtype)
        q_s = to_f64(q[q_off:q_off + n_new], dtype)
        out[q_off:q_off + n_new] = attention_one_sequence(q_s, k_s, v_s, n_cached, scale, window)
    return out
