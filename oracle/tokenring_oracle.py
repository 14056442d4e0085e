"""Plain fp64 CPU oracle for TokenRing's per-device compute path.

TEST INFRASTRUCTURE.  Slow, unblocked, unfused, written to be checked against the paper
by eye.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may call
it; the HIP library never does, and the two share no code.

What is computed, and where the paper defines it:

* ``attention_block`` / ``attention_full`` / ``attention_rows`` - the per-step operation
  ``block_out, block_lse <- Attention(Q, K, V)`` of Algorithm 1 (Sec. 3.2): scaled
  dot-product softmax attention of one Query chunk against one K/V chunk, returning the
  normalised output and the row-wise natural-log log-sum-exp of the scaled scores
  (Sec. 3.1 describes block_out as (N,H,D) and block_lse as (H,N)).  The paper never
  writes the softmax out ("typical self-attention"), so this is the textbook definition:
      s_k = scale * <q, k_k>,  lse = ln sum_k exp(s_k),  out = sum_k exp(s_k - lse) v_k
  over the allowed keys (all keys, or key position <= query position for the causal
  LLM case of Sec. 3.3.2).
* ``merge_pair_sigmoid_form`` - the Update equations of Sec. 3.1 exactly as printed:
      out <- out - sigmoid(block_lse - lse) * (out - block_out)
      lse <- lse - ln(sigmoid(lse - block_lse))
* ``merge_pair`` - the same Update made total: the accumulator starts as the identity
  element (out = 0, lse = -inf), which Algorithm 1 needs at its first Update but the
  printed sigmoid form turns into NaN.  Equal to the printed form wherever that is finite.
* ``merge_nary`` - the order-free definition the pairwise Update must reach:
      lse = ln sum_i exp(lse_i),  out = sum_i exp(lse_i - lse) out_i.
* ``ring_schedule`` / ``ring_attention`` - Algorithm 1's iteration order replayed on one
  device: at iteration i "device" j holds Query chunk (j - i) mod N and attends it to its
  own K_j, V_j; the block result is merged into the accumulators of that Query chunk.
  (Reading of the garbled index in Algorithm 1: "step" is the loop variable i; this
  matches the four-device walk-through of Sec. 3.3.1.)

Layout: [B, H, S, D] for Q/K/V/out and [B, H, S] for lse (the paper's (N,H,D)/(H,N)
with a batch axis in front and heads before tokens).  Grouped-query attention: query
head h reads K/V head h // (Hq // Hkv).  All arithmetic is float64.

Parity pins (tests/test_oracle_*.py): 50-digit mpmath brute force on tiny inputs,
closed forms (zero queries, causal prefix means, single dominant key), library special
cases (torch scaled_dot_product_attention in fp64, scipy logsumexp), the invariants the
formulation fixes (softmax rows sum to one, chunk-count and merge-order invariance,
GQA == MHA with repeated K/V) and the paper's four-device walk-through for the schedule.
The paper prints no numeric example, so no pin comes from printed values.
"""
from __future__ import annotations

import numpy as np

NEG_INF = -np.inf


def _kv_head(h: int, Hq: int, Hkv: int) -> int:
    if Hq % Hkv:
        raise ValueError("query heads must be a multiple of K/V heads")
    return h // (Hq // Hkv)


def _allowed(q_pos: np.ndarray, k_pos: np.ndarray, causal: bool) -> np.ndarray:
    """Boolean [len(q_pos), len(k_pos)]: may query position attend key position (Sec. 3.3.2)."""
    if not causal:
        return np.ones((len(q_pos), len(k_pos)), dtype=bool)
    return k_pos[None, :] <= q_pos[:, None]


def _rows(q, k, v, scale, allowed):
    """Softmax attention of query rows q [R,D] over keys k [K,D], values v [K,D], fp64.

    Two passes per row: all scores, then their log-sum-exp, then the weighted value sum.
    Rows with no allowed key give out = 0 and lse = -inf.
    """
    s = scale * (q @ k.T)                                   # [R, K] scaled scores
    s = np.where(allowed, s, NEG_INF)
    m = np.max(s, axis=1, initial=NEG_INF)                  # row max, for a stable exp only
    m_safe = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(s - m_safe[:, None])                         # masked entries -> exp(-inf) = 0
    l = np.sum(e, axis=1)
    with np.errstate(divide="ignore"):
        lse = m_safe + np.log(l)                            # ln sum_k exp(s_k); -inf when l == 0
    w = np.exp(s - np.where(np.isfinite(lse), lse, 0.0)[:, None])   # exp(s_k - lse) = softmax weights
    w = np.where(np.isfinite(lse)[:, None], w, 0.0)
    return w @ v, lse, w


def attention_block(q, k, v, scale, causal_diag=False, q_offset=0, k_offset=0):
    """One block step of Algorithm 1: Attention(Q chunk, K chunk, V chunk) -> block_out, block_lse.

    q [B,Hq,Sq,D], k/v [B,Hkv,Sk,D] float64.  ``causal_diag`` applies the causal rule with
    query row r at position q_offset + r and key c at position k_offset + c; with both
    offsets 0 and Sq == Sk this is the diagonal chunk's mask (key index <= query index).
    Returns out [B,Hq,Sq,D], lse [B,Hq,Sq].
    """
    q, k, v = (np.asarray(x, dtype=np.float64) for x in (q, k, v))
    B, Hq, Sq, D = q.shape
    _, Hkv, Sk, _ = k.shape
    allowed = _allowed(q_offset + np.arange(Sq), k_offset + np.arange(Sk), causal_diag)
    out = np.empty((B, Hq, Sq, D))
    lse = np.empty((B, Hq, Sq))
    for b in range(B):
        for h in range(Hq):
            g = _kv_head(h, Hq, Hkv)
            out[b, h], lse[b, h], _ = _rows(q[b, h], k[b, g], v[b, g], scale, allowed)
    return out, lse


def attention_full(q, k, v, scale, causal=False):
    """Unchunked attention over the whole sequence: the result every chunked schedule must reach."""
    return attention_block(q, k, v, scale, causal_diag=causal)


def attention_rows(q_rows, row_pos, k, v, scale, causal):
    """Exact attention for a sample of query rows of one (batch, head).

    q_rows [R,D] are the queries at global positions row_pos [R]; k, v [S,D] are the whole
    K/V of the matching K/V head.  Used where the full problem is too large for the CPU.
    """
    q_rows, k, v = (np.asarray(x, dtype=np.float64) for x in (q_rows, k, v))
    row_pos = np.asarray(row_pos)
    out = np.empty_like(q_rows)
    lse = np.empty(len(row_pos))
    step = 64                                               # rows per slab: bounds the score matrix
    for a in range(0, len(row_pos), step):
        pos = row_pos[a:a + step]
        kmax = int(pos.max()) + 1 if causal else k.shape[0]
        allowed = _allowed(pos, np.arange(kmax), causal)
        out[a:a + step], lse[a:a + step], _ = _rows(q_rows[a:a + step], k[:kmax], v[:kmax], scale, allowed)
    return out, lse


def softmax_weights(q, k, scale, causal=False):
    """exp(s - lse) for one head: q [Sq,D], k [Sk,D] -> [Sq,Sk]; rows sum to one."""
    q, k = np.asarray(q, dtype=np.float64), np.asarray(k, dtype=np.float64)
    allowed = _allowed(np.arange(q.shape[0]), np.arange(k.shape[0]), causal)
    return _rows(q, k, np.zeros((k.shape[0], 1)), scale, allowed)[2]


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def merge_pair_sigmoid_form(out, lse, block_out, block_lse):
    """The Update of Sec. 3.1 exactly as printed (finite inputs only).

    out [...,D], lse [...] accumulators; block_out / block_lse the new partial result.
    """
    out, lse, block_out, block_lse = (np.asarray(x, dtype=np.float64) for x in (out, lse, block_out, block_lse))
    new_out = out - _sigmoid(block_lse - lse)[..., None] * (out - block_out)
    new_lse = lse - np.log(_sigmoid(lse - block_lse))
    return new_out, new_lse


def merge_pair(out, lse, block_out, block_lse):
    """Update(block_out, block_lse) of Algorithm 1 with the identity element (0, -inf) handled.

    m = max(lse, block_lse); both -inf -> (0, -inf); otherwise
    lse' = m + ln(exp(lse - m) + exp(block_lse - m)), w = exp(block_lse - lse'),
    out' = out + w (block_out - out)   [= out - sigmoid(block_lse - lse)(out - block_out)].
    """
    out, lse, block_out, block_lse = (np.asarray(x, dtype=np.float64) for x in (out, lse, block_out, block_lse))
    m = np.maximum(lse, block_lse)
    empty = np.isneginf(m)
    m_safe = np.where(empty, 0.0, m)
    with np.errstate(divide="ignore"):
        new_lse = m_safe + np.log(np.exp(lse - m_safe) + np.exp(block_lse - m_safe))
    w = np.where(empty, 0.0, np.exp(block_lse - np.where(empty, 0.0, new_lse)))
    new_out = out + w[..., None] * (block_out - out)
    new_out = np.where(empty[..., None], 0.0, new_out)
    new_lse = np.where(empty, NEG_INF, new_lse)
    return new_out, new_lse


def merge_nary(outs, lses):
    """Order-free merge of any number of partial results: lse = ln sum_i exp(lse_i),
    out = sum_i exp(lse_i - lse) out_i (max-subtracted for stability; all -inf -> (0, -inf))."""
    outs = np.stack([np.asarray(o, dtype=np.float64) for o in outs])    # [n, ..., D]
    lses = np.stack([np.asarray(l, dtype=np.float64) for l in lses])    # [n, ...]
    m = np.max(lses, axis=0)
    empty = np.isneginf(m)
    m_safe = np.where(empty, 0.0, m)
    with np.errstate(divide="ignore"):
        lse = m_safe + np.log(np.sum(np.exp(lses - m_safe), axis=0))
    w = np.exp(lses - np.where(empty, 0.0, lse))                        # [n, ...]
    w = np.where(empty, 0.0, w)
    out = np.sum(w[..., None] * outs, axis=0)
    return out, np.where(empty, NEG_INF, lse)


def ring_schedule(n_chunks, causal):
    """Algorithm 1's steps in execution order, all devices replayed on one.

    Returns a list of (i, j, c): at iteration i, device j (owner of K_j, V_j) attends
    Query chunk c = (j - i) mod N, whose accumulators live on device c.  With contiguous
    causal chunks, steps whose K/V chunk lies after the Query chunk (j > c) are dropped
    and j == c is the diagonal (masked) step.
    """
    steps = []
    for i in range(n_chunks):
        for j in range(n_chunks):
            c = (j - i) % n_chunks
            if causal and j > c:
                continue
            steps.append((i, j, c))
    return steps


def ring_attention(q, k, v, n_chunks, causal, scale, order=None):
    """Chunked attention by Algorithm 1: block attention per step, pairwise Update into
    per-Query-chunk accumulators that start at (0, -inf).

    ``order`` optionally replaces the TokenRing step order by any other sequence of
    (q_chunk, kv_chunk) pairs (e.g. Ring Attention's, or a shuffle) - the result must not
    depend on it.  Returns out [B,Hq,S,D], lse [B,Hq,S] in float64.
    """
    q, k, v = (np.asarray(x, dtype=np.float64) for x in (q, k, v))
    B, Hq, S, D = q.shape
    if S % n_chunks:
        raise ValueError("sequence length must be a multiple of n_chunks")
    C = S // n_chunks
    out = np.zeros((B, Hq, S, D))
    lse = np.full((B, Hq, S), NEG_INF)
    pairs = [(c, j) for (_, j, c) in ring_schedule(n_chunks, causal)] if order is None else list(order)
    for c, j in pairs:
        qs, ks = slice(c * C, (c + 1) * C), slice(j * C, (j + 1) * C)
        bout, blse = attention_block(q[:, :, qs], k[:, :, ks], v[:, :, ks], scale,
                                     causal_diag=causal, q_offset=c * C, k_offset=j * C)
        out[:, :, qs], lse[:, :, qs] = merge_pair(out[:, :, qs], lse[:, :, qs], bout, blse)
    return out, lse


def zigzag_segments(n_devices):
    """Zigzag partition of Sec. 3.3.2: the sequence is cut into 2N segments and device g
    holds segments g and 2N-1-g (four devices, eight segments: device 0 holds 0 and 7)."""
    return [(g, 2 * n_devices - 1 - g) for g in range(n_devices)]


def ring_attention_order(n_chunks, causal):
    """Ring Attention (Sec. 2.1) as (q_chunk, kv_chunk) pairs in execution order: device j keeps
    Q_j and, at iteration i, holds the K/V chunk that started on device (j - i) mod N."""
    pairs = []
    for i in range(n_chunks):
        for j in range(n_chunks):
            kv = (j - i) % n_chunks
            if causal and kv > j:
                continue
            pairs.append((j, kv))
    return pairs


def zigzag_steps(n_devices):
    """TokenRing on the zigzag partition (Sec. 3.3.2), causal: (i, j, q_segment, kv_segment) in
    execution order over 2N segments.  Device j keeps the K/V of its two segments; at iteration
    i it holds the Query pair of device c = (j - i) mod N.  A pair of segments is computed iff
    the K/V segment does not lie after the Query segment."""
    owned = zigzag_segments(n_devices)
    steps = []
    for i in range(n_devices):
        for j in range(n_devices):
            c = (j - i) % n_devices
            for qs in owned[c]:
                for ks in owned[j]:
                    if ks <= qs:
                        steps.append((i, j, qs, ks))
    return steps


def zigzag_order(n_devices):
    """zigzag_steps as plain (q_segment, kv_segment) pairs, the form ring_attention's ``order`` takes."""
    return [(qs, ks) for (_, _, qs, ks) in zigzag_steps(n_devices)]


def hybrid_order(n_nodes, per_node, causal):
    """Multi-node scheme of Sec. 3.3.3 as (q_chunk, kv_chunk) pairs: K/V move between nodes as
    in Ring Attention (after outer step t, device p of node m holds the K/V that started on
    device p of node (m - t) mod M); inside every node Algorithm 1 circulates the node's own
    Query chunks among its ``per_node`` devices."""
    pairs = []
    for t in range(n_nodes):
        for i in range(per_node):
            for m in range(n_nodes):
                for p in range(per_node):
                    qc = m * per_node + (p - i) % per_node
                    kv = ((m - t) % n_nodes) * per_node + p
                    if causal and kv > qc:
                        continue
                    pairs.append((qc, kv))
    return pairs
