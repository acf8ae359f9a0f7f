"""Plain, slow, dense-masked fp64 reference of the Dynamic Mask Attention hot path.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Everything here is NumPy
in float64, written from the paper's definitions, with no blocking or fusion
beyond row-chunking of the dense score matrix to bound memory.

What is computed (paper: Section 4 "Method", Eq. 3-10, Alg. 1-2, Listing 1):

* content scores       z[h, j] = exp(A_h * softplus(w_h . v_{g(h), j}))      (Eq. 3)
* kept set of row i    the min(k, #candidates) best candidate keys of row i
                       under "larger z first, lower index first on ties";
                       candidates = keys j <= i of the same document when
                       causal, else all keys of the document           (Eq. 4, Listing 1)
* attention            S_ij = scale * q_i . k_j + z_j on the kept set,
                       P = softmax over the kept set, exactly 0 elsewhere,
                       O = P V, LSE = log sum exp S                     (Eq. 5-6, Alg. 1)
* gradients            dV, dS = P o (dP - D), dz = column sums of dS,
                       dQ, dK                                          (Eq. 7-10, Alg. 2)

Readings of the paper taken here (the paper is ambiguous on these points):
the mask is *added* to the scaled scores (the case formula of Eq. 5, Alg. 1 and
the listing agree; the words "element-wise multiplied" do not); the activation
tau is softplus (Listing 1); the bias is delta itself, not its log; the
sparsifier f acts element-wise; the top-w is taken per query row over that
row's causal prefix (Listing 1); rows with fewer than k candidates keep all of
them; Alg. 2's "rowsum(dS)" into dM is a sum over the query rows of a column
(Eq. 9 summed over time steps); no gradient flows through the selection
(Section 6, "Fully Differentiable Design").  Each q-head h uses its own vector
w_h on the values of its kv-head g(h) = h // (H_q / H_kv); z_scores_xhead is the
paper's full form, in which the score of head h contracts the token's values of
ALL heads (Delta in R^{n_h x d_h x n_h}, Eq. 3; Listing 1 flattens the heads'
values before the projection).

Layouts: Q, O, dO, dQ [T, H_q, d]; K, V, dK, dV [T, H_kv, d]; z, dz, LSE
[H_q, T]; cu_seqlens [n_docs + 1] with cu[0] = 0, cu[-1] = T.

Pins (tests/test_oracle_*.py): reduction to textbook causal softmax attention
and to torch SDPA (k >= L, constant z), sliding-window / sink closed forms,
k = 1, all-equal z (tie rule), row sums, exact zeros, finite differences for
all four gradients, algebraic identities, scalar triple-loop brute force, and
the gather-loop formulation of Listing 1; mask_backward: central finite
differences of Eq. 3 and torch autograd of the forward formula; dma_decode:
the last rows of the dense forward oracle and of topk_indices; z_scores_xhead /
xhead_backward: a block-structured Delta reproduces the per-head functions,
torch's linear + softplus + exp and its autograd, central finite differences;
the bias argument / expand_bias / bias_backward: torch SDPA with the bias as attn_mask
(forward and autograd, all four broadcast forms), finite differences, and a kept
set that must not move with the bias; O_stored: the closed form of its shift.
No function here is unpinned.
"""
from __future__ import annotations

import bisect
import math

import numpy as np

__all__ = [
    "softplus", "z_scores", "kept_mask_definition", "kept_mask_ranked",
    "expiry_from_kept", "expiry_sequential", "topk_indices", "dma_forward",
    "dma_backward", "dma_forward_gather_loop", "dma_scalar_bruteforce",
    "n_active_pairs", "dma_rows", "dma_keys", "mask_backward", "dma_decode",
    "z_scores_xhead", "xhead_backward", "expand_bias", "bias_backward",
]


# --------------------------------------------------------------------------- scores
def softplus(x):
    """log(1 + exp(x)), evaluated without overflow (Listing 1 uses softplus for tau)."""
    x = np.asarray(x, dtype=np.float64)
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def z_scores(V, W, A, H_q):
    """Eq. 3: z[h, j] = exp(A_h * softplus(w_h . v_{g(h), j})).

    V [T, H_kv, d], W [H_q, d], A [H_q]  ->  z [H_q, T] (float64).
    """
    V = np.asarray(V, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    T, H_kv, d = V.shape
    G = H_q // H_kv
    z = np.empty((H_q, T), dtype=np.float64)
    for h in range(H_q):
        x = V[:, h // G, :] @ W[h]
        z[h] = np.exp(A[h] * softplus(x))
    return z


def mask_backward(V, W, A, dz, H_q):
    """Gradient of Eq. 3 by the chain rule, given dz [H_q, T] (the gradient that reaches the
    scores through the attention bias, Eq. 9 / Alg. 2).  With x = w_h . v_{g(h), j},
    z = exp(A_h softplus(x)) and softplus' = logistic sigmoid:

        dx[h, j]  = dz[h, j] z[h, j] A_h sigmoid(x[h, j])
        dA[h]     = sum_j dz[h, j] z[h, j] softplus(x[h, j])
        dW[h, :]  = sum_j dx[h, j] v_{g(h), j}
        dVz[j, g] = sum_{h in group g} dx[h, j] w_h     (the part of dV that flows through z)

    Returns dW [H_q, d], dA [H_q], dVz [T, H_kv, d] (float64).  No gradient flows through the
    top-k selection (Section 6).
    """
    V = np.asarray(V, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    dz = np.asarray(dz, dtype=np.float64)
    T, H_kv, d = V.shape
    G = H_q // H_kv
    dW = np.zeros((H_q, d))
    dA = np.zeros(H_q)
    dVz = np.zeros((T, H_kv, d))
    for h in range(H_q):
        g = h // G
        x = V[:, g, :] @ W[h]
        sp = softplus(x)
        z = np.exp(A[h] * sp)
        sig = 1.0 / (1.0 + np.exp(-x))
        dx = dz[h] * z * A[h] * sig
        dA[h] = np.sum(dz[h] * z * sp)
        dW[h] = dx @ V[:, g, :]
        dVz[:, g, :] += np.outer(dx, W[h])
    return dW, dA, dVz


def z_scores_xhead(V, Delta, A):
    """Eq. 3 with the full sampling tensor: the score of head h contracts the token's value
    vectors of all kv-heads, z[h, j] = exp(A_h * softplus(sum_{g, c} v_{g, j, c} Delta[h, g, c])).

    V [T, H_kv, d], Delta [H_q, H_kv * d] (row h = the flattened [H_kv, d] weights of head h, the
    layout of a linear layer's weight), A [H_q]  ->  z [H_q, T] (float64).
    """
    V = np.asarray(V, dtype=np.float64)
    Delta = np.asarray(Delta, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    T = V.shape[0]
    x = V.reshape(T, -1) @ Delta.T                  # [T, H_q]
    return np.exp(A[None, :] * softplus(x)).T


def xhead_backward(V, Delta, A, dz):
    """Chain rule of z_scores_xhead, given dz [H_q, T]:

        dx[h, j]        = dz[h, j] z[h, j] A_h sigmoid(x[h, j])
        dA[h]           = sum_j dz[h, j] z[h, j] softplus(x[h, j])
        dDelta[h, g, c] = sum_j dx[h, j] v_{g, j, c}
        dVz[j, g, c]    = sum_h dx[h, j] Delta[h, g, c]

    Returns dDelta [H_q, H_kv * d], dA [H_q], dVz [T, H_kv, d] (float64).
    """
    V = np.asarray(V, dtype=np.float64)
    Delta = np.asarray(Delta, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    dz = np.asarray(dz, dtype=np.float64)
    T, H_kv, d = V.shape
    Vf = V.reshape(T, -1)
    x = Vf @ Delta.T                                # [T, H_q]
    sp = softplus(x)
    z = np.exp(A[None, :] * sp)
    sig = 1.0 / (1.0 + np.exp(-x))
    dzt = dz.T                                      # [T, H_q]
    dx = dzt * z * A[None, :] * sig
    dA = np.sum(dzt * z * sp, axis=0)
    dDelta = dx.T @ Vf
    dVz = (dx @ Delta).reshape(T, H_kv, d)
    return dDelta, dA, dVz


# --------------------------------------------------------------------------- kept sets
def kept_mask_definition(z_doc, k, causal=True):
    """Eq. 4 by its definition: for each row, stable-sort the candidates by
    descending z and keep the first min(k, #candidates).

    z_doc [n] (one document, one head) -> bool [n, n], entry (i, j) true iff
    key j is kept by query row i.
    """
    z_doc = np.asarray(z_doc, dtype=np.float64)
    n = z_doc.shape[0]
    keep = np.zeros((n, n), dtype=bool)
    for i in range(n):
        ncand = i + 1 if causal else n
        order = np.argsort(-z_doc[:ncand], kind="stable")  # ties: lower index first
        keep[i, order[: min(k, ncand)]] = True
    return keep


def kept_mask_ranked(z_doc, k, causal=True):
    """Same set as kept_mask_definition, computed densely: rank all keys once
    (stable), then key j is kept by row i iff fewer than k candidates of row i
    rank ahead of it."""
    z_doc = np.asarray(z_doc, dtype=np.float64)
    n = z_doc.shape[0]
    order = np.argsort(-z_doc, kind="stable")
    rank = np.empty(n, dtype=np.int64)
    rank[order] = np.arange(n)
    ahead = rank[None, :] < rank[:, None]          # ahead[j, j2]: j2 ranks ahead of j
    if causal:
        # cnt[i, j] = #{j2 <= i : j2 ahead of j}
        cnt = np.cumsum(ahead.T, axis=0)           # cumsum over j2 (rows) -> [i, j]
        cand = np.tril(np.ones((n, n), dtype=bool))
        return cand & (cnt < k)
    cnt = ahead.sum(axis=1)                        # [j]
    return np.broadcast_to(cnt[None, :] < k, (n, n)).copy()


def expiry_from_kept(keep):
    """Encode a causal kept mask as one integer per key: e[j] = first row >= j
    that does not keep key j (n if kept to the end, j if never kept).  Raises if
    the rows keeping a key are not one contiguous interval starting at j."""
    n = keep.shape[0]
    e = np.empty(n, dtype=np.int64)
    for j in range(n):
        col = keep[j:, j]
        dropped = np.flatnonzero(~col)
        e[j] = j + (dropped[0] if dropped.size else n - j)
        if col[e[j] - j:].any() or keep[:j, j].any():
            raise AssertionError(f"key {j}: kept rows are not a contiguous interval [j, e)")
    return e


def expiry_sequential(z_doc, k):
    """Causal expiry by walking the rows once with the kept set held as a
    sorted list (an iteration, not the definition: pinned against
    kept_mask_definition in the tests).  Row i: key i joins the candidates; if
    more than k are then held, the worst one (lowest z, highest index among
    equals) is dropped and its expiry is i."""
    z_doc = np.asarray(z_doc, dtype=np.float64)
    n = z_doc.shape[0]
    e = np.full(n, n, dtype=np.int64)
    held = []                                      # sorted ascending by (z, -index): held[0] is the worst
    for i in range(n):
        bisect.insort(held, (z_doc[i], -i))
        if len(held) > k:
            _, neg = held.pop(0)
            e[-neg] = i
    return e


def topk_indices(z_doc, k, causal=True):
    """Kept key indices of every row in ascending order, -1 padded: int32 [n, k]."""
    keep = kept_mask_definition(z_doc, k, causal)
    n = keep.shape[0]
    out = np.full((n, k), -1, dtype=np.int32)
    for i in range(n):
        idx = np.flatnonzero(keep[i])
        out[i, : idx.size] = idx
    return out


def n_active_pairs(n, k):
    """Number of (row, key) pairs the causal mask keeps in a document of n rows."""
    if k >= n:
        return n * (n + 1) // 2
    return k * n - k * (k - 1) // 2


# --------------------------------------------------------------------------- attention
def _doc_keep_provider(z_doc, k, causal, mask_method):
    """Returns f(r0, r1) -> bool [r1 - r0, n] for one (document, head)."""
    n = z_doc.shape[0]
    if mask_method == "definition":
        full = kept_mask_definition(z_doc, k, causal)
        return lambda r0, r1: full[r0:r1]
    if mask_method != "sequential":
        raise ValueError(mask_method)
    cols = np.arange(n)[None, :]
    if causal:
        e = expiry_sequential(z_doc, k)

        def prov(r0, r1):
            rows = np.arange(r0, r1)[:, None]
            return (cols <= rows) & (rows < e[None, :])
        return prov
    order = np.argsort(-z_doc, kind="stable")
    kept = np.zeros(n, dtype=bool)
    kept[order[: min(k, n)]] = True
    return lambda r0, r1: np.broadcast_to(kept[None, :], (r1 - r0, n))


def _softmax_rows(S, keep):
    """Masked softmax of a chunk of rows: returns (P, LSE); P is exactly 0 off the kept set."""
    S = np.where(keep, S, -np.inf)
    m = S.max(axis=1, keepdims=True)
    Pu = np.exp(S - m)                             # exp(-inf) == 0.0 exactly
    l = Pu.sum(axis=1, keepdims=True)
    return Pu / l, (m + np.log(l))[:, 0]


def _as64(x):
    return np.asarray(x, dtype=np.float64)


def expand_bias(bias, H_q, cu_seqlens, per_token=True):
    """A caller-supplied attention bias with head / batch broadcasting, written out per (head, key):
    bias [Hb, T] (per_token) or [Hb, n_max] indexed by the key's position in its document and shared
    by all documents (batch broadcast); Hb = H_q or 1 (head broadcast).  Returns float64 [H_q, T]."""
    bias = _as64(bias)
    cu = [int(c) for c in cu_seqlens]
    T = cu[-1]
    Hb = bias.shape[0]
    assert Hb in (1, H_q)
    out = np.empty((H_q, T))
    for h in range(H_q):
        row = bias[h if Hb == H_q else 0]
        if per_token:
            out[h] = row[:T]
        else:
            for a, b in zip(cu[:-1], cu[1:]):
                out[h, a:b] = row[: b - a]
    return out


def bias_backward(dz, bias_heads, cu_seqlens, per_token=True, n_max=None):
    """Gradient of the broadcast bias from dz [H_q, T] (the bias enters the score exactly like z, so
    d(loss)/d(bias as applied)[h, j] = dz[h, j]): summed over the heads and documents that share an
    entry.  Returns [bias_heads, T] (per_token) or [bias_heads, n_max]."""
    dz = _as64(dz)
    H_q, T = dz.shape
    cu = [int(c) for c in cu_seqlens]
    d = dz if bias_heads == H_q else dz.sum(axis=0, keepdims=True)
    if per_token:
        return d.copy()
    out = np.zeros((bias_heads, n_max))
    for a, b in zip(cu[:-1], cu[1:]):
        out[:, : b - a] += d[:, a:b]
    return out


def dma_forward(Q, K, V, z, cu_seqlens, k, causal=True, scale=None, heads=None,
                mask_method="sequential", row_chunk=1024, bias=None):
    """Eq. 5-6 / Alg. 1 result: O [T, H_q, d], LSE [H_q, T].

    bias [H_q, T] (optional): a further additive attention bias per (head, key), broadcast over the
    query rows (Section 1, "Kernel Design": the kernel takes masks and biases with batch, head and
    query broadcasting).  It is added to the scores of the kept pairs, S_ij = scale q_i.k_j + z_j +
    b_j; the kept set is selected on z alone (Eq. 4 ranks the content scores).

    heads: iterable of q-head indices to compute (others are left as NaN).
    mask_method: "definition" (per-row stable sort, O(n^2 log n)) or
    "sequential" (interval encoding from expiry_sequential; causal) -- the two
    are asserted equal in the tests.
    """
    Q, K, V, z = _as64(Q), _as64(K), _as64(V), _as64(z)
    T, H_q, d = Q.shape
    H_kv = K.shape[1]
    G = H_q // H_kv
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    heads = range(H_q) if heads is None else heads
    O = np.full((T, H_q, d), np.nan)
    LSE = np.full((H_q, T), np.nan)
    cu = [int(c) for c in cu_seqlens]
    for h in heads:
        g = h // G
        for a, b in zip(cu[:-1], cu[1:]):
            n = b - a
            if n == 0:
                continue
            q, kk, v, zb = Q[a:b, h], K[a:b, g], V[a:b, g], z[h, a:b]
            prov = _doc_keep_provider(zb, k, causal, mask_method)
            sb = zb if bias is None else zb + _as64(bias)[h, a:b]
            for r0 in range(0, n, row_chunk):
                r1 = min(n, r0 + row_chunk)
                S = scale * (q[r0:r1] @ kk.T) + sb[None, :]
                P, lse = _softmax_rows(S, prov(r0, r1))
                O[a + r0:a + r1, h] = P @ v
                LSE[h, a + r0:a + r1] = lse
    return O, LSE


def dma_backward(Q, K, V, z, dO, cu_seqlens, k, causal=True, scale=None, heads=None,
                 mask_method="sequential", row_chunk=1024, abs_out=None, O_stored=None, bias=None,
                 LSE_stored=None):
    """Eq. 7-10 / Alg. 2 result: dQ [T, H_q, d], dK, dV [T, H_kv, d], dz [H_q, T].

    bias [H_q, T]: as in dma_forward.  z and the bias enter the score as a sum, so dz is also the
    gradient with respect to the bias as applied (see bias_backward for the broadcast forms).

    dK and dV are summed over the q-heads listed in `heads` that share a
    kv-head (all heads by default).  dV is the attention-path gradient only
    (the path V -> z is not part of this function).

    O_stored [T, H_q, d]: Alg. 2 does not recompute O: it loads the forward's output from memory and
    forms D_i = rowsum(dO_i o O_i) from it.  With O_stored given, D_i is formed from that array (the
    buffer a backward kernel is handed, e.g. the forward result rounded to bf16); without it D_i uses
    the exact O of Eq. 5 (then D_i equals the sum_j p_ij dp_ij of Eq. 8).  dS = P o (dP - D) is linear
    in D, so the two results differ by dD_i = dO_i . (O_stored_i - O_i) entering as -P_ij dD_i.

    LSE_stored [H_q, T]: Alg. 2 does not renormalise either: it loads the forward's row statistics
    (l_i and m_i, stored here as one LSE_i = m_i + ln l_i) and forms P_ij = exp(S_ij - LSE_i) from them.
    With LSE_stored given, P is formed that way from the array (e.g. the forward result rounded to
    fp32); without it P is the exact softmax of Eq. 5.  A stored LSE_i + e_i scales row i of P by
    exp(-e_i), and with it that row's contributions to every gradient.  (The exact O of the default D_i
    is always the exact softmax's.)

    A dict passed as abs_out receives the magnitudes of the summands of dK and dV,
    "dK": scale * sum_i |dS_ij| |q_ic| and "dV": sum_i P_ij |do_ic|, both [T, H_kv, d] (no part of the
    result: the yardstick for a sum of many reduced-precision terms).
    """
    Q, K, V, z, dO = _as64(Q), _as64(K), _as64(V), _as64(z), _as64(dO)
    T, H_q, d = Q.shape
    H_kv = K.shape[1]
    G = H_q // H_kv
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    heads = range(H_q) if heads is None else heads
    dQ = np.full((T, H_q, d), np.nan)
    dz = np.full((H_q, T), np.nan)
    dK = np.zeros((T, H_kv, d))
    dV = np.zeros((T, H_kv, d))
    cu = [int(c) for c in cu_seqlens]
    dK_abs = np.zeros((T, H_kv, d)) if abs_out is not None else None
    dV_abs = np.zeros((T, H_kv, d)) if abs_out is not None else None
    O_st = None if O_stored is None else _as64(O_stored)
    L_st = None if LSE_stored is None else _as64(LSE_stored)
    for h in heads:
        g = h // G
        for a, b in zip(cu[:-1], cu[1:]):
            n = b - a
            if n == 0:
                continue
            q, kk, v, zb, do = Q[a:b, h], K[a:b, g], V[a:b, g], z[h, a:b], dO[a:b, h]
            prov = _doc_keep_provider(zb, k, causal, mask_method)
            sb = zb if bias is None else zb + _as64(bias)[h, a:b]
            dzd = np.zeros(n)
            for r0 in range(0, n, row_chunk):
                r1 = min(n, r0 + row_chunk)
                S = scale * (q[r0:r1] @ kk.T) + sb[None, :]
                keep = prov(r0, r1)
                P, _ = _softmax_rows(S, keep)
                o = P @ v
                if L_st is not None:                                # Alg. 2 loads l_i, m_i from memory
                    P = np.where(keep, np.exp(np.where(keep, S, -np.inf) - L_st[h, a + r0:a + r1, None]), 0.0)
                if O_st is not None:
                    o = O_st[a + r0:a + r1, h]                      # Alg. 2 loads O_i from memory
                D = (do[r0:r1] * o).sum(axis=1, keepdims=True)      # Alg. 2: D_i
                dP = do[r0:r1] @ v.T                                # Eq. 8: dp_j = v_j . do
                dS = P * (dP - D)                                   # Eq. 8
                dV[a:b, g] += P.T @ do[r0:r1]                       # Eq. 7
                dQ[a + r0:a + r1, h] = scale * (dS @ kk)            # Eq. 10
                dK[a:b, g] += scale * (dS.T @ q[r0:r1])             # Eq. 10
                dzd += dS.sum(axis=0)                               # Eq. 9, summed over rows
                if dK_abs is not None:
                    dK_abs[a:b, g] += scale * (np.abs(dS).T @ np.abs(q[r0:r1]))
                    dV_abs[a:b, g] += P.T @ np.abs(do[r0:r1])
            dz[h, a:b] = dzd
    if abs_out is not None:
        abs_out["dK"] = dK_abs
        abs_out["dV"] = dV_abs
    return dQ, dK, dV, dz


def dma_forward_gather_loop(Q, K, V, z, cu_seqlens, k, causal=True, scale=None):
    """The second formulation (Listing 1's per-query loop): for every query
    gather its kept keys, softmax over just those, weighted sum of the gathered
    values.  Small inputs only."""
    Q, K, V, z = _as64(Q), _as64(K), _as64(V), _as64(z)
    T, H_q, d = Q.shape
    G = H_q // K.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    O = np.zeros((T, H_q, d))
    cu = [int(c) for c in cu_seqlens]
    for h in range(H_q):
        g = h // G
        for a, b in zip(cu[:-1], cu[1:]):
            idx_all = topk_indices(z[h, a:b], k, causal)
            for i in range(b - a):
                idx = idx_all[i][idx_all[i] >= 0] + a
                s = (K[idx, g] * Q[a + i, h][None, :]).sum(axis=1) * scale + z[h, idx]
                w = np.exp(s - s.max())
                w /= w.sum()
                O[a + i, h] = (w[:, None] * V[idx, g]).sum(axis=0)
    return O


def dma_scalar_bruteforce(Q, K, V, z, dO, k, scale):
    """Root of trust for tiny inputs: one document, one head (H_q = H_kv = 1),
    causal, pure-Python scalar loops.  Q, K, V, dO: [n][d] nested sequences,
    z: [n].  Returns (O, LSE, dQ, dK, dV, dz) as nested lists."""
    n, d = len(Q), len(Q[0])
    O = [[0.0] * d for _ in range(n)]
    LSE = [0.0] * n
    dQ = [[0.0] * d for _ in range(n)]
    dK = [[0.0] * d for _ in range(n)]
    dV = [[0.0] * d for _ in range(n)]
    dz = [0.0] * n
    for i in range(n):
        cand = list(range(i + 1))
        cand.sort(key=lambda j: (-z[j], j))
        kept = sorted(cand[:k])
        s = {}
        for j in kept:
            acc = 0.0
            for c in range(d):
                acc += Q[i][c] * K[j][c]
            s[j] = acc * scale + z[j]
        m = max(s.values())
        tot = sum(math.exp(s[j] - m) for j in kept)
        LSE[i] = m + math.log(tot)
        p = {j: math.exp(s[j] - m) / tot for j in kept}
        for j in kept:
            for c in range(d):
                O[i][c] += p[j] * V[j][c]
        dp = {j: sum(dO[i][c] * V[j][c] for c in range(d)) for j in kept}
        dot = sum(p[j] * dp[j] for j in kept)
        for j in kept:
            ds = p[j] * (dp[j] - dot)
            dz[j] += ds
            for c in range(d):
                dV[j][c] += p[j] * dO[i][c]
                dQ[i][c] += ds * K[j][c] * scale
                dK[j][c] += ds * Q[i][c] * scale
    return O, LSE, dQ, dK, dV, dz


# --------------------------------------------------------------------------- sampled outputs
# For inputs too large for the dense path: single rows / single keys computed one by one from the
# same definitions (pinned against the dense functions above on small inputs in the tests).
def _doc_of(cu, t):
    for a, b in zip(cu[:-1], cu[1:]):
        if a <= t < b:
            return int(a), int(b)
    raise ValueError(t)


class _ExpiryCache:
    def __init__(self, z, cu, k):
        self.z, self.cu, self.k, self.c = z, [int(c) for c in cu], k, {}

    def get(self, h, a, b):
        if (h, a) not in self.c:
            self.c[(h, a)] = expiry_sequential(self.z[h, a:b], self.k) + a
        return self.c[(h, a)]


def dma_rows(Q, K, V, z, dO, cu_seqlens, k, rows, scale=None, O_stored=None):
    """Eq. 5-6 and the dQ half of Eq. 10 for single (head, row) pairs, causal.

    rows: iterable of (h, i) with i a global row index.  Returns a list of dicts with keys
    O [d], LSE, dQ [d] (dQ only if dO is given), kept (global key indices, ascending).
    O_stored: as in dma_backward (D_i from the stored output, Alg. 2).
    """
    Q, K, V, z = _as64(Q), _as64(K), _as64(V), _as64(z)
    dO = None if dO is None else _as64(dO)
    T, H_q, d = Q.shape
    G = H_q // K.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    cache = _ExpiryCache(z, cu_seqlens, k)
    out = []
    for h, i in rows:
        a, b = _doc_of(cache.cu, i)
        e = cache.get(h, a, b)
        j = np.arange(a, i + 1)
        kept = j[e[: i + 1 - a] > i]
        g = h // G
        s = scale * (K[kept, g] @ Q[i, h]) + z[h, kept]
        m = s.max()
        w = np.exp(s - m)
        tot = w.sum()
        p = w / tot
        o = p @ V[kept, g]
        rec = dict(O=o, LSE=m + math.log(tot), kept=kept)
        if dO is not None:
            dp = V[kept, g] @ dO[i, h]
            o_D = o if O_stored is None else _as64(O_stored[i, h])
            ds = p * (dp - float(dO[i, h] @ o_D))
            rec["dQ"] = scale * (ds @ K[kept, g])
        out.append(rec)
    return out


def dma_keys(Q, K, V, z, dO, LSE, O, cu_seqlens, k, keys, scale=None):
    """Eq. 7, 9 and the dK half of Eq. 10 for single (kv-head, key) pairs, causal, given the
    oracle's own LSE [H_q, T] and O [T, H_q, d] for the q-heads of those kv-heads.

    keys: iterable of (g, j).  Returns a list of dicts: dK [d], dV [d] (summed over the q-heads of
    group g) and dz {h: value}.  D_i is formed from the O passed in (Alg. 2): pass the exact O of
    Eq. 5 or the stored array a backward kernel was handed.
    """
    Q, K, V, z, dO, LSE, O = _as64(Q), _as64(K), _as64(V), _as64(z), _as64(dO), _as64(LSE), _as64(O)
    T, H_q, d = Q.shape
    G = H_q // K.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    cache = _ExpiryCache(z, cu_seqlens, k)
    out = []
    for g, j in keys:
        a, b = _doc_of(cache.cu, j)
        dK = np.zeros(d)
        dV = np.zeros(d)
        dz = {}
        for h in range(g * G, (g + 1) * G):
            e = int(cache.get(h, a, b)[j - a])
            rows = np.arange(j, e)
            if rows.size == 0:
                dz[h] = 0.0
                continue
            s = scale * (Q[rows, h] @ K[j, g]) + z[h, j]
            p = np.exp(s - LSE[h, rows])
            D = (dO[rows, h] * O[rows, h]).sum(axis=1)
            ds = p * (dO[rows, h] @ V[j, g] - D)
            dz[h] = float(ds.sum())
            dV += p @ dO[rows, h]
            dK += scale * (ds @ Q[rows, h])
        out.append(dict(dK=dK, dV=dV, dz=dz))
    return out


# --------------------------------------------------------------------------- decode (one new row per sequence)
def dma_decode(q, K, V, z, cu_seqlens, k, scale=None):
    """Eq. 4-6 for the newest row of every sequence: the row is the last one of its document, so
    its candidates are all n keys of the document; it keeps the min(k, n) best by (z descending,
    index ascending), and o = softmax(scale q.K_kept + z_kept) V_kept.

    q [n_docs, H_q, d]; K, V [T, H_kv, d]; z [H_q, T].  Returns o [n_docs, H_q, d],
    lse [H_q, n_docs] and kept: list over documents of int arrays [H_q, min(k, n)] (global row
    indices, ascending).  An empty document gives o = 0 and lse = -inf.
    """
    q, K, V, z = _as64(q), _as64(K), _as64(V), _as64(z)
    n_docs, H_q, d = q.shape
    H_kv = K.shape[1]
    G = H_q // H_kv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    o = np.zeros((n_docs, H_q, d))
    lse = np.full((H_q, n_docs), -np.inf)
    kept = []
    for b in range(n_docs):
        a, e = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        n = e - a
        kk = min(k, n)
        kept_b = np.zeros((H_q, kk), dtype=np.int64)
        for h in range(H_q):
            if n == 0:
                continue
            zz = z[h, a:e]
            order = sorted(range(n), key=lambda j: (-zz[j], j))   # larger z first, lower index on ties
            idx = np.array(sorted(order[:kk]), dtype=np.int64)
            s = scale * (K[a + idx, h // G, :] @ q[b, h]) + zz[idx]
            mx = s.max()
            p = np.exp(s - mx)
            lse[h, b] = mx + math.log(p.sum())
            o[b, h] = (p / p.sum()) @ V[a + idx, h // G, :]
            kept_b[h] = a + idx
        kept.append(kept_b)
    return o, lse, kept
