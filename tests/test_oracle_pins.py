"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no worked numerical example, so the oracle is pinned by:
reduction to textbook causal softmax attention / torch SDPA, closed forms for
special score sequences, invariants of Eq. 5, finite differences for Eq. 7-10,
algebraic identities, a scalar triple-loop brute force and the gather-loop
formulation of Listing 1.  Each test names the mistake it is there to catch.
"""
import math

import numpy as np
import pytest
import torch

import oracle as orc

RNG = np.random.default_rng(7)


def rand_case(n=48, H_q=4, H_kv=2, d=8, seed=0, ties=False):
    r = np.random.default_rng(seed)
    Q = r.standard_normal((n, H_q, d))
    K = r.standard_normal((n, H_kv, d))
    V = r.standard_normal((n, H_kv, d))
    dO = r.standard_normal((n, H_q, d))
    z = r.uniform(0.05, 1.0, size=(H_q, n))
    if ties:
        z = np.round(z * 4) / 4            # heavy ties: 5 distinct values
    return Q, K, V, dO, z


def textbook_causal(Q, K, V, scale, bias=None, band=None):
    """Independent five-line reference: dense causal softmax attention, one head."""
    n = Q.shape[0]
    S = scale * Q @ K.T
    if bias is not None:
        S = S + bias[None, :]
    i, j = np.arange(n)[:, None], np.arange(n)[None, :]
    ok = j <= i
    if band is not None:
        ok &= (i - j) < band
    S = np.where(ok, S, -np.inf)
    P = np.exp(S - S.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    return P @ V, P


# ----------------------------------------------------------------------------- scores (Eq. 3)
def test_softplus_matches_library_and_limits():
    x = np.linspace(-40, 40, 161)
    ref = torch.nn.functional.softplus(torch.tensor(x, dtype=torch.float64), threshold=1e9).numpy()
    assert np.allclose(orc.softplus(x), ref, rtol=1e-14, atol=0)
    assert orc.softplus(0.0) == pytest.approx(math.log(2.0), abs=1e-15)
    assert orc.softplus(800.0) == 800.0          # no overflow
    assert orc.softplus(-800.0) == 0.0 or orc.softplus(-800.0) < 1e-300


def test_z_scores_closed_form_and_head_grouping():
    # W = 0 => x = 0 => z = exp(A ln 2) = 2**A, for every key
    V = RNG.standard_normal((10, 2, 4))
    A = np.array([-1.0, -0.5, -2.0, -1.5])
    z = orc.z_scores(V, np.zeros((4, 4)), A, 4)
    assert np.allclose(z, (2.0 ** A)[:, None], rtol=1e-15)
    # one-hot w_h picks one channel of the head's own kv-head (g = h // 2)
    W = np.zeros((4, 4)); W[0, 1] = 1; W[1, 2] = 1; W[2, 0] = 1; W[3, 3] = 1
    z = orc.z_scores(V, W, A, 4)
    for h, (g, c) in enumerate([(0, 1), (0, 2), (1, 0), (1, 3)]):
        x = V[:, g, c]
        assert np.allclose(z[h], np.exp(A[h] * np.log1p(np.exp(x))), rtol=1e-13)


# ----------------------------------------------------------------------------- kept sets (Eq. 4)
@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("n,k", [(1, 1), (7, 3), (64, 16), (200, 64), (50, 80)])
def test_kept_mask_formulations_agree(n, k, ties):
    r = np.random.default_rng(n * 100 + k)
    z = r.uniform(0, 1, n)
    if ties:
        z = np.round(z * 3) / 3
    ref = orc.kept_mask_definition(z, k)
    assert (orc.kept_mask_ranked(z, k) == ref).all()
    e = orc.expiry_from_kept(ref)                       # raises unless contiguous intervals [j, e)
    assert (orc.expiry_sequential(z, k) == e).all()
    i, j = np.arange(n)[:, None], np.arange(n)[None, :]
    assert (((j <= i) & (i < e[None, :])) == ref).all()
    # every row keeps exactly min(i + 1, k) keys, all of them causal
    assert (ref.sum(1) == np.minimum(np.arange(n) + 1, k)).all()
    assert not np.triu(ref, 1).any()
    assert ref.sum() == orc.n_active_pairs(n, k)


def test_kept_mask_noncausal():
    z = np.array([0.3, 0.9, 0.3, 0.5, 0.9])
    m = orc.kept_mask_definition(z, 3, causal=False)
    assert (m == np.array([0, 1, 0, 1, 1], bool)[None, :]).all()     # 0.9, 0.9, 0.5
    assert (orc.kept_mask_ranked(z, 3, causal=False) == m).all()
    m2 = orc.kept_mask_definition(z, 4, causal=False)
    assert (m2[0] == np.array([1, 1, 0, 1, 1], bool)).all()          # tie 0.3: lower index wins


def test_tie_rule_lower_index_wins():
    # all scores equal: the kept set of every row is keys 0..k-1
    n, k = 20, 5
    m = orc.kept_mask_definition(np.full(n, 0.25), k)
    for i in range(n):
        assert (np.flatnonzero(m[i]) == np.arange(min(i + 1, k))).all()
    e = orc.expiry_sequential(np.full(n, 0.25), k)
    assert (e[:k] == n).all() and (e[k:] == np.arange(k, n)).all()   # later keys never kept


def test_increasing_and_decreasing_scores_closed_forms():
    n, k = 30, 6
    inc = np.linspace(0.1, 0.9, n)
    m = orc.kept_mask_definition(inc, k)
    i, j = np.arange(n)[:, None], np.arange(n)[None, :]
    assert (m == ((j <= i) & (i - j < k))).all()                     # sliding window
    dec = inc[::-1].copy()
    m = orc.kept_mask_definition(dec, k)
    assert (m == ((j <= i) & (j < k))).all()                         # attention sink


def test_topk_indices_ascending_and_padded():
    z = np.array([0.5, 0.1, 0.9, 0.7])
    idx = orc.topk_indices(z, 2)
    assert idx.tolist() == [[0, -1], [0, 1], [0, 2], [2, 3]]


# ----------------------------------------------------------------------------- forward (Eq. 5-6)
def test_reduces_to_causal_attention_textbook_and_sdpa():
    """k >= L with constant z: softmax is shift-invariant, so the result is
    plain causal attention.  Catches a wrong scale, a transposed operand, a
    wrong head grouping or a bias applied multiplicatively."""
    n, H_q, H_kv, d = 40, 4, 2, 8
    Q, K, V, dO, _ = rand_case(n, H_q, H_kv, d, seed=3)
    for const in (0.0, 0.37):
        z = np.full((H_q, n), const)
        O, LSE = orc.dma_forward(Q, K, V, z, [0, n], k=n + 5)
        dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, [0, n], k=n + 5)
        tq = torch.tensor(Q.transpose(1, 0, 2)[None], dtype=torch.float64, requires_grad=True)
        tk = torch.tensor(K.transpose(1, 0, 2)[None], dtype=torch.float64, requires_grad=True)
        tv = torch.tensor(V.transpose(1, 0, 2)[None], dtype=torch.float64, requires_grad=True)
        tkr = tk.repeat_interleave(H_q // H_kv, dim=1)
        tvr = tv.repeat_interleave(H_q // H_kv, dim=1)
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tkr, tvr, is_causal=True)
        ref.backward(torch.tensor(dO.transpose(1, 0, 2)[None]))
        assert np.allclose(O, ref.detach()[0].numpy().transpose(1, 0, 2), atol=1e-12)
        assert np.allclose(dQ, tq.grad[0].numpy().transpose(1, 0, 2), atol=1e-12)
        assert np.allclose(dK, tk.grad[0].numpy().transpose(1, 0, 2), atol=1e-12)
        assert np.allclose(dV, tv.grad[0].numpy().transpose(1, 0, 2), atol=1e-12)
        for h in range(H_q):
            Oh, P = textbook_causal(Q[:, h], K[:, h // 2], V[:, h // 2], 1 / math.sqrt(d))
            assert np.allclose(O[:, h], Oh, atol=1e-12)
            S = np.where(np.tril(np.ones((n, n), bool)), Q[:, h] @ K[:, h // 2].T / math.sqrt(d), -np.inf)
            lse = np.log(np.exp(S).sum(1)) + const
            assert np.allclose(LSE[h], lse, atol=1e-12)


def test_increasing_scores_equal_banded_attention_with_bias():
    """z strictly increasing => sliding window of width k with z as additive
    bias; compared with torch SDPA given an explicit additive mask."""
    n, d, k = 36, 8, 7
    Q, K, V, dO, _ = rand_case(n, 1, 1, d, seed=5)
    z = np.linspace(0.05, 0.95, n)[None, :]
    O, _ = orc.dma_forward(Q, K, V, z, [0, n], k=k)
    i, j = np.arange(n)[:, None], np.arange(n)[None, :]
    add = np.where((j <= i) & (i - j < k), z[0][None, :], -np.inf)
    t = lambda a: torch.tensor(a.transpose(1, 0, 2)[None], dtype=torch.float64)
    ref = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V), attn_mask=torch.tensor(add)[None, None])
    assert np.allclose(O, ref[0].numpy().transpose(1, 0, 2), atol=1e-12)
    Oh, _ = textbook_causal(Q[:, 0], K[:, 0], V[:, 0], 1 / math.sqrt(d), bias=z[0], band=k)
    assert np.allclose(O[:, 0], Oh, atol=1e-12)


def test_k_equals_one_picks_first_prefix_maximum():
    n, d = 25, 4
    Q, K, V, dO, z = rand_case(n, 2, 1, d, seed=9, ties=True)
    O, LSE = orc.dma_forward(Q, K, V, z, [0, n], k=1)
    for h in range(2):
        for i in range(n):
            j = int(np.argmax(z[h, : i + 1]))               # first maximum
            assert np.allclose(O[i, h], V[j, 0], atol=1e-14)
            assert LSE[h, i] == pytest.approx(Q[i, h] @ K[j, 0] / math.sqrt(d) + z[h, j], abs=1e-12)


def test_rows_sum_to_one_and_masked_weights_exactly_zero():
    n, k = 64, 9
    Q, K, V, dO, z = rand_case(n, 2, 2, 8, seed=11, ties=True)
    for h in range(2):
        keep = orc.kept_mask_definition(z[h], k)
        S = Q[:, h] @ K[:, h].T / math.sqrt(8) + z[h][None, :]
        from oracle.dma_oracle import _softmax_rows
        P, lse = _softmax_rows(S, keep)
        assert np.allclose(P.sum(1), 1.0, atol=1e-14)
        assert (P[~keep] == 0.0).all()                        # exact zeros (Eq. 5, second case)
        assert (P[keep] > 0.0).all()
        assert ((P != 0).sum(1) == np.minimum(np.arange(n) + 1, k)).all()
        O, LSE = orc.dma_forward(Q, K, V, z, [0, n], k=k, heads=[h])
        assert np.allclose(O[:, h], P @ V[:, h], atol=1e-13)
        assert np.allclose(LSE[h], lse, atol=1e-13)


@pytest.mark.parametrize("ties", [False, True])
def test_dense_masked_equals_gather_loop_and_both_mask_methods(ties):
    n, k = 40, 6
    Q, K, V, dO, z = rand_case(n, 4, 2, 8, seed=13, ties=ties)
    cu = [0, 13, 13, 40]                                       # includes an empty document
    O1, L1 = orc.dma_forward(Q, K, V, z, cu, k, mask_method="definition")
    O2, L2 = orc.dma_forward(Q, K, V, z, cu, k, mask_method="sequential", row_chunk=7)
    O3 = orc.dma_forward_gather_loop(Q, K, V, z, cu, k)
    assert np.allclose(O1, O2, atol=1e-13) and np.allclose(L1, L2, atol=1e-13)
    assert np.allclose(O1, O3, atol=1e-12)
    g1 = orc.dma_backward(Q, K, V, z, dO, cu, k, mask_method="definition")
    g2 = orc.dma_backward(Q, K, V, z, dO, cu, k, mask_method="sequential", row_chunk=5)
    for a, b in zip(g1, g2):
        assert np.allclose(a, b, atol=1e-12)


def test_documents_are_independent():
    n1, n2, k = 17, 23, 5
    Q, K, V, dO, z = rand_case(n1 + n2, 2, 1, 8, seed=17)
    O, LSE = orc.dma_forward(Q, K, V, z, [0, n1, n1 + n2], k)
    Oa, La = orc.dma_forward(Q[:n1], K[:n1], V[:n1], z[:, :n1], [0, n1], k)
    Ob, Lb = orc.dma_forward(Q[n1:], K[n1:], V[n1:], z[:, n1:], [0, n2], k)
    assert np.allclose(O, np.concatenate([Oa, Ob]), atol=1e-14)
    assert np.allclose(LSE, np.concatenate([La, Lb], axis=1), atol=1e-14)


def test_vectorised_oracle_equals_scalar_bruteforce():
    """Root of trust: pure-Python loops written from Eq. 6-10 (Eq. 8's sum form
    for the softmax Jacobian rather than Alg. 2's D_i)."""
    n, d, k = 24, 5, 4
    Q, K, V, dO, z = rand_case(n, 1, 1, d, seed=19, ties=True)
    scale = 0.31
    ref = orc.dma_scalar_bruteforce(Q[:, 0].tolist(), K[:, 0].tolist(), V[:, 0].tolist(), z[0].tolist(),
                                    dO[:, 0].tolist(), k, scale)
    O, LSE = orc.dma_forward(Q, K, V, z, [0, n], k, scale=scale)
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, [0, n], k, scale=scale)
    for got, want in zip((O[:, 0], LSE[0], dQ[:, 0], dK[:, 0], dV[:, 0], dz[0]), ref):
        assert np.allclose(got, np.array(want), atol=1e-12)


# ----------------------------------------------------------------------------- backward (Eq. 7-10)
def _loss(Q, K, V, z, dO, cu, k, scale):
    O, _ = orc.dma_forward(Q, K, V, z, cu, k, scale=scale, mask_method="definition")
    return float((O * dO).sum())


def test_gradients_match_finite_differences():
    """Central differences of sum(O o dO) w.r.t. Q, K, V and z.  Pins the
    column-sum reading of the mask gradient, the scale factors, the GQA sum
    over q-heads and the sign of the softmax Jacobian.  z is perturbed by much
    less than its smallest gap, so the kept sets do not change (no gradient
    flows through the selection)."""
    n, H_q, H_kv, d, k = 12, 4, 2, 6, 4
    r = np.random.default_rng(23)
    Q, K, V, dO = (r.standard_normal(s) for s in [(n, H_q, d), (n, H_kv, d), (n, H_kv, d), (n, H_q, d)])
    z = np.stack([r.permutation(n) for _ in range(H_q)]) * 0.05 + 0.1      # gaps of 0.05
    cu, scale, eps = [0, 5, n], 0.4, 1e-5
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, cu, k, scale=scale, mask_method="definition")
    args = dict(Q=Q, K=K, V=V, z=z)
    for name, grad in (("Q", dQ), ("K", dK), ("V", dV), ("z", dz)):
        base = args[name]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            hi = {**args, name: base.copy()}; hi[name][idx] += eps
            lo = {**args, name: base.copy()}; lo[name][idx] -= eps
            num[idx] = (_loss(dO=dO, cu=cu, k=k, scale=scale, **hi) -
                        _loss(dO=dO, cu=cu, k=k, scale=scale, **lo)) / (2 * eps)
        assert np.allclose(grad, num, atol=2e-8), name


def test_gradient_identities():
    n, H_q, H_kv, d, k = 50, 4, 2, 8, 7
    Q, K, V, dO, z = rand_case(n, H_q, H_kv, d, seed=29)
    cu = [0, 20, n]
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, cu, k)
    # rows of the softmax Jacobian sum to zero => sum_j dz = 0 per (document, head)
    for a, b in zip(cu[:-1], cu[1:]):
        assert np.allclose(dz[:, a:b].sum(1), 0.0, atol=1e-12)
    # scores are bilinear in (q, k): sum_i q_i.dQ_i over a kv-group == sum_j k_j.dK_j
    for g in range(H_kv):
        lhs = sum((Q[:, h] * dQ[:, h]).sum() for h in (2 * g, 2 * g + 1))
        assert lhs == pytest.approx((K[:, g] * dK[:, g]).sum(), abs=1e-10)
    # adding a constant to z leaves O unchanged and shifts LSE by that constant
    O0, L0 = orc.dma_forward(Q, K, V, z, cu, k)
    O1, L1 = orc.dma_forward(Q, K, V, z + 0.7, cu, k)
    assert np.allclose(O0, O1, atol=1e-13) and np.allclose(L1 - L0, 0.7, atol=1e-12)
    # keys that are never kept receive exactly zero gradient
    for h in range(H_q):
        for a, b in zip(cu[:-1], cu[1:]):
            e = orc.expiry_sequential(z[h, a:b], k)
            never = np.flatnonzero(e == np.arange(b - a)) + a
            assert (dz[h, never] == 0.0).all()


def test_heads_subset_matches_full():
    n = 30
    Q, K, V, dO, z = rand_case(n, 4, 2, 8, seed=31)
    full = orc.dma_backward(Q, K, V, z, dO, [0, n], 5)
    sub = orc.dma_backward(Q, K, V, z, dO, [0, n], 5, heads=[2, 3])     # one whole kv-group
    assert np.allclose(sub[0][:, 2:], full[0][:, 2:], atol=1e-14)
    assert np.allclose(sub[1][:, 1], full[1][:, 1], atol=1e-14)
    assert np.allclose(sub[2][:, 1], full[2][:, 1], atol=1e-14)
    assert (sub[1][:, 0] == 0).all()


def test_sampled_rows_and_keys_match_dense_oracle():
    """The one-by-one functions used at full size are the same mathematics as the dense path."""
    n1, n2, H_q, H_kv, d, k = 37, 50, 4, 2, 8, 6
    Q, K, V, dO, z = rand_case(n1 + n2, H_q, H_kv, d, seed=41, ties=True)
    cu = [0, n1, n1 + n2]
    O, LSE = orc.dma_forward(Q, K, V, z, cu, k)
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, cu, k)
    rows = [(h, i) for h in range(H_q) for i in (0, 5, n1 - 1, n1, n1 + 7, n1 + n2 - 1)]
    for (h, i), rec in zip(rows, orc.dma_rows(Q, K, V, z, dO, cu, k, rows)):
        assert np.allclose(rec["O"], O[i, h], atol=1e-13)
        assert rec["LSE"] == pytest.approx(LSE[h, i], abs=1e-13)
        assert np.allclose(rec["dQ"], dQ[i, h], atol=1e-13)
        a = 0 if i < n1 else n1
        assert rec["kept"].tolist() == (np.flatnonzero(orc.kept_mask_definition(z[h, a:cu[1 if i < n1 else 2]], k)[i - a]) + a).tolist()
    keys = [(g, j) for g in range(H_kv) for j in (0, 3, n1 - 1, n1, n1 + 11, n1 + n2 - 1)]
    for (g, j), rec in zip(keys, orc.dma_keys(Q, K, V, z, dO, LSE, O, cu, k, keys)):
        assert np.allclose(rec["dK"], dK[j, g], atol=1e-12)
        assert np.allclose(rec["dV"], dV[j, g], atol=1e-12)
        for h, val in rec["dz"].items():
            assert val == pytest.approx(dz[h, j], abs=1e-12)


# ----------------------------------------------------------------------------- D_i from a stored O (Alg. 2)
def _bf16_round(x):
    """Round-to-nearest-even to 8 significant bits, written out on the bit pattern (a stand-in for a
    stored low-precision O; independent of the workload module's converter)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def test_stored_o_equal_to_exact_o_changes_nothing():
    """Alg. 2's D_i = rowsum(dO o O) equals Eq. 8's sum_j p_ij dp_ij when O is the exact forward
    result: the O_stored mode must then reproduce the default (a wrong row / head index into
    O_stored, or D formed before the substitution, fails here)."""
    n1, n2, k = 23, 30, 5
    Q, K, V, dO, z = rand_case(n1 + n2, 4, 2, 8, seed=51, ties=True)
    cu = [0, n1, n1 + n2]
    O, _ = orc.dma_forward(Q, K, V, z, cu, k)
    a = orc.dma_backward(Q, K, V, z, dO, cu, k)
    b = orc.dma_backward(Q, K, V, z, dO, cu, k, O_stored=O, row_chunk=7)
    for x, y in zip(a, b):
        assert np.allclose(x, y, atol=1e-13)
    rows = [(h, i) for h in range(4) for i in (0, 4, n1, n1 + n2 - 1)]
    for ra, rb in zip(orc.dma_rows(Q, K, V, z, dO, cu, k, rows), orc.dma_rows(Q, K, V, z, dO, cu, k, rows, O_stored=O)):
        assert np.allclose(ra["dQ"], rb["dQ"], atol=1e-13)


def test_stored_o_rounded_shifts_the_gradients_by_the_closed_form():
    """dS = P o (dP - D) is linear in D.  With a rounded O the row term moves by
    dD_i = dO_i . (O~_i - O_i), hence exactly: dz_j -= sum_i P_ij dD_i, dQ_i -= scale dD_i sum_j P_ij k_j,
    dK_j -= scale sum_i P_ij dD_i q_i, and dV does not move.  The shifts are written out with
    explicit loops over (head, row, kept key); a sign slip, a missing scale or D applied to dV fails."""
    n, H_q, H_kv, d, k = 26, 4, 2, 8, 4
    G = H_q // H_kv
    scale = 1.0 / math.sqrt(d)
    Q, K, V, dO, z = rand_case(n, H_q, H_kv, d, seed=52)
    cu = [0, n]
    O, LSE = orc.dma_forward(Q, K, V, z, cu, k)
    Or = _bf16_round(O)
    assert np.abs(Or - O).max() > 1e-4                      # the rounding is visible
    dQ0, dK0, dV0, dz0 = orc.dma_backward(Q, K, V, z, dO, cu, k)
    dQ1, dK1, dV1, dz1 = orc.dma_backward(Q, K, V, z, dO, cu, k, O_stored=Or)
    sdQ, sdK, sdz = np.zeros_like(dQ0), np.zeros_like(dK0), np.zeros_like(dz0)
    for h in range(H_q):
        keep = orc.kept_mask_definition(z[h], k)
        for i in range(n):
            dD = float(dO[i, h] @ (Or[i, h] - O[i, h]))
            for j in np.flatnonzero(keep[i]):
                p = math.exp(scale * float(Q[i, h] @ K[j, h // G]) + z[h, j] - LSE[h, i])
                sdz[h, j] -= p * dD
                sdQ[i, h] -= scale * p * dD * K[j, h // G]
                sdK[j, h // G] -= scale * p * dD * Q[i, h]
    assert np.allclose(dz1 - dz0, sdz, atol=1e-13) and np.abs(sdz).max() > 1e-5
    assert np.allclose(dQ1 - dQ0, sdQ, atol=1e-13)
    assert np.allclose(dK1 - dK0, sdK, atol=1e-13)
    assert np.array_equal(dV1, dV0)
    # the one-by-one functions take the same buffer
    rows = [(h, i) for h in range(H_q) for i in (0, 3, n - 1)]
    for (h, i), rec in zip(rows, orc.dma_rows(Q, K, V, z, dO, cu, k, rows, O_stored=Or)):
        assert np.allclose(rec["dQ"], dQ1[i, h], atol=1e-13)
    keys = [(g, j) for g in range(H_kv) for j in (0, 5, n - 1)]
    for (g, j), rec in zip(keys, orc.dma_keys(Q, K, V, z, dO, LSE, Or, cu, k, keys)):
        assert np.allclose(rec["dK"], dK1[j, g], atol=1e-12)
        for h, val in rec["dz"].items():
            assert val == pytest.approx(dz1[h, j], abs=1e-12)


def test_stored_lse_equal_to_exact_lse_changes_nothing():
    """Alg. 2 forms P_ij = exp(S_ij - LSE_i) from the stored row statistics; with the exact LSE that is
    the softmax of Eq. 5, so the LSE_stored mode must reproduce the default (a head / row index slip
    into LSE_stored, or P exponentiated off the kept set, fails here).  Two documents, ties, non-causal too."""
    n1, n2, k = 21, 33, 6
    Q, K, V, dO, z = rand_case(n1 + n2, 4, 2, 8, seed=53, ties=True)
    cu = [0, n1, n1 + n2]
    for causal in (True, False):
        _, LSE = orc.dma_forward(Q, K, V, z, cu, k, causal=causal)
        a = orc.dma_backward(Q, K, V, z, dO, cu, k, causal=causal)
        b = orc.dma_backward(Q, K, V, z, dO, cu, k, causal=causal, LSE_stored=LSE, row_chunk=5)
        for x, y in zip(a, b):
            assert np.allclose(x, y, atol=1e-13)


def test_stored_lse_off_by_e_scales_the_rows_by_exp_minus_e():
    """With a stored LSE_i + e_i every P_ij of row i is exp(-e_i) times the softmax weight, D_i (from
    the exact O) is unchanged, and the four gradients follow from Eq. 7-10 term by term.  Written out
    with explicit loops over (head, row, kept key) from the exact LSE; together with a stored O
    (both buffers at once, as a backward kernel gets them)."""
    n, H_q, H_kv, d, k = 24, 4, 2, 8, 5
    G = H_q // H_kv
    scale = 1.0 / math.sqrt(d)
    Q, K, V, dO, z = rand_case(n, H_q, H_kv, d, seed=54)
    cu = [0, n]
    O, LSE = orc.dma_forward(Q, K, V, z, cu, k)
    e = 0.03 * np.random.default_rng(55).standard_normal((H_q, n))
    Or = _bf16_round(O)
    for O_used, kw in ((O, {}), (Or, {"O_stored": Or})):
        dQ1, dK1, dV1, dz1 = orc.dma_backward(Q, K, V, z, dO, cu, k, LSE_stored=LSE + e, **kw)
        rQ, rK, rV, rz = np.zeros_like(dQ1), np.zeros_like(dK1), np.zeros_like(dV1), np.zeros_like(dz1)
        for h in range(H_q):
            g = h // G
            keep = orc.kept_mask_definition(z[h], k)
            for i in range(n):
                D = float(dO[i, h] @ O_used[i, h])
                for j in np.flatnonzero(keep[i]):
                    p = math.exp(scale * float(Q[i, h] @ K[j, g]) + z[h, j] - (LSE[h, i] + e[h, i]))
                    ds = p * (float(dO[i, h] @ V[j, g]) - D)
                    rV[j, g] += p * dO[i, h]
                    rz[h, j] += ds
                    rQ[i, h] += scale * ds * K[j, g]
                    rK[j, g] += scale * ds * Q[i, h]
        assert np.allclose(dQ1, rQ, atol=1e-13) and np.allclose(dK1, rK, atol=1e-13)
        assert np.allclose(dV1, rV, atol=1e-13) and np.allclose(dz1, rz, atol=1e-13)
    dV0 = orc.dma_backward(Q, K, V, z, dO, cu, k)[2]
    assert np.abs(dV1 - dV0).max() > 1e-3                   # the offset is visible


def test_summand_masses_of_dk_and_dv_match_triple_loops():
    """abs_out["dK"] = scale sum_i |dS_ij| |q_ic| and abs_out["dV"] = sum_i P_ij |dO_ic| (summed over
    the q-heads of the kv-head): the yardsticks a test may add to the tolerance of dK / dV for keep
    windows of one to three keys.  Recomputed here with scalar loops from the scalar brute force's
    quantities; a missing scale, |.| in the wrong place or a head not summed fails."""
    n, H_q, H_kv, d, k = 14, 2, 1, 3, 3
    scale = 0.7
    Q, K, V, dO, z = rand_case(n, H_q, H_kv, d, seed=53)
    mass = {}
    orc.dma_backward(Q, K, V, z, dO, [0, n], k, scale=scale, abs_out=mass)
    mK = [[0.0] * d for _ in range(n)]
    mV = [[0.0] * d for _ in range(n)]
    for h in range(H_q):
        for i in range(n):
            cand = sorted(range(i + 1), key=lambda j: (-z[h][j], j))[:k]
            s = {j: scale * sum(Q[i, h, c] * K[j, 0, c] for c in range(d)) + z[h, j] for j in cand}
            m = max(s.values())
            tot = sum(math.exp(v - m) for v in s.values())
            p = {j: math.exp(s[j] - m) / tot for j in cand}
            dp = {j: sum(dO[i, h, c] * V[j, 0, c] for c in range(d)) for j in cand}
            dot = sum(p[j] * dp[j] for j in cand)
            for j in cand:
                ds = p[j] * (dp[j] - dot)
                for c in range(d):
                    mK[j][c] += scale * abs(ds) * abs(Q[i, h, c])
                    mV[j][c] += p[j] * abs(dO[i, h, c])
    assert np.allclose(mass["dK"][:, 0], np.array(mK), atol=1e-13)
    assert np.allclose(mass["dV"][:, 0], np.array(mV), atol=1e-13)
    # and they bound the gradients they accompany
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, [0, n], k, scale=scale)
    assert (np.abs(dK) <= mass["dK"] + 1e-12).all() and (np.abs(dV) <= mass["dV"] + 1e-12).all()


# ----------------------------------------------------------------------------- caller-supplied attention bias
@pytest.mark.parametrize("Hb,per_token", [(4, True), (1, True), (4, False), (1, False)])
def test_bias_equals_sdpa_attn_mask_and_its_autograd(Hb, per_token):
    """With k >= n everything causal is kept, so z + bias is an ordinary additive attn_mask of torch's
    SDPA: O, dQ, dK, dV and the bias gradient (reduced over the broadcast dimensions by autograd) must
    match, for a bias per (head, token), shared by the heads, indexed by the position in the document
    (shared by the two documents), or both.  A bias dropped from the backward, added twice, or summed
    over the wrong axis fails."""
    n, H_q, H_kv, d = 19, 4, 2, 8
    G = H_q // H_kv
    Q, K, V, dO, z = rand_case(2 * n, H_q, H_kv, d, seed=61)
    cu = [0, n, 2 * n]
    r = np.random.default_rng(62)
    braw = r.standard_normal((Hb, 2 * n if per_token else n))
    bias = orc.expand_bias(braw, H_q, cu, per_token)
    O, _ = orc.dma_forward(Q, K, V, z, cu, 10 * n, bias=bias)
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, cu, 10 * n, bias=bias)
    dbias = orc.bias_backward(dz, Hb, cu, per_token, n_max=n)
    tb = torch.tensor(braw, requires_grad=True)
    tq, tk, tv = (torch.tensor(x, requires_grad=True) for x in (Q, K, V))
    outs = []
    for doc in range(2):
        a, b = cu[doc], cu[doc + 1]
        brow = tb[:, a:b] if per_token else tb                           # [Hb, n]
        m = torch.tensor(z[:, a:b])[:, None, :] + brow[:, None, :].expand(Hb, n, n)      # [H_q, n, n] by broadcast
        m = m + torch.triu(torch.full((n, n), float("-inf"), dtype=torch.float64), 1)
        q = tq[a:b].permute(1, 0, 2)[None]
        kk = tk[a:b].permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
        vv = tv[a:b].permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
        outs.append(torch.nn.functional.scaled_dot_product_attention(q, kk, vv, attn_mask=m[None])[0].permute(1, 0, 2))
    to = torch.cat(outs)
    to.backward(torch.tensor(dO))
    assert np.allclose(O, to.detach().numpy(), atol=1e-12)
    assert np.allclose(dQ, tq.grad.numpy(), atol=1e-12) and np.allclose(dK, tk.grad.numpy(), atol=1e-12)
    assert np.allclose(dV, tv.grad.numpy(), atol=1e-12)
    assert dbias.shape == braw.shape and np.allclose(dbias, tb.grad.numpy(), atol=1e-12)


def test_bias_does_not_move_the_kept_set_and_zero_bias_changes_nothing():
    """The selection ranks the content scores z alone (Eq. 4): a bias that would reorder z + b must leave
    the kept set where it is (exact zeros of P in the same places), and b = 0 reproduces the unbiased
    result.  Finite differences over the bias confirm dz as its gradient on a sparse window."""
    n, H_q, H_kv, d, k = 24, 2, 1, 6, 4
    Q, K, V, dO, z = rand_case(n, H_q, H_kv, d, seed=63)
    cu = [0, n]
    bias = np.random.default_rng(64).standard_normal((H_q, n)) * 5.0      # large enough to reorder z + b
    O0, L0 = orc.dma_forward(Q, K, V, z, cu, k)
    Oz, Lz = orc.dma_forward(Q, K, V, z, cu, k, bias=np.zeros((H_q, n)))
    assert np.array_equal(O0, Oz) and np.array_equal(L0, Lz)
    Ob, Lb = orc.dma_forward(Q, K, V, z, cu, k, bias=bias)
    # same result as gathering each row's kept keys (chosen on z) and applying softmax with z + b
    scale = 1.0 / math.sqrt(d)
    for h in range(H_q):
        keep = orc.kept_mask_definition(z[h], k)
        for i in range(n):
            idx = np.flatnonzero(keep[i])
            sc = scale * (K[idx, 0] @ Q[i, h]) + z[h, idx] + bias[h, idx]
            w = np.exp(sc - sc.max()); w /= w.sum()
            assert np.allclose(Ob[i, h], w @ V[idx, 0], atol=1e-13)
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, cu, k, bias=bias)
    eps = 1e-6
    for (h, j) in [(0, 0), (1, 3), (0, n - 2), (1, n - 1)]:
        bp, bm = bias.copy(), bias.copy()
        bp[h, j] += eps; bm[h, j] -= eps
        fp = (orc.dma_forward(Q, K, V, z, cu, k, bias=bp)[0] * dO).sum()
        fm = (orc.dma_forward(Q, K, V, z, cu, k, bias=bm)[0] * dO).sum()
        assert (fp - fm) / (2 * eps) == pytest.approx(dz[h, j], abs=1e-7)


# ----------------------------------------------------------------------------- without the causal restriction
@pytest.mark.parametrize("ties", [False, True])
def test_noncausal_is_plain_attention_over_the_gathered_top_k(ties):
    """Without the causal restriction every row of a document keeps the same min(k, n) best keys
    (Eq. 4 over all keys), so the path is dense attention over those gathered keys with their scores
    as a bias.  torch computes that and differentiates it.  Catches: a causal mask left in, a kept set
    that varies with the row, a wrong tie rule, gradients leaking to unselected keys."""
    Q, K, V, dO, z = rand_case(n=50, H_q=4, H_kv=2, d=8, seed=31, ties=ties)
    cu = np.array([0, 20, 50])
    k, scale = 7, 1.0 / math.sqrt(8)
    O, LSE = orc.dma_forward(Q, K, V, z, cu, k, causal=False)
    dQ, dK, dV, dz = orc.dma_backward(Q, K, V, z, dO, cu, k, causal=False)
    Qt, Kt, Vt, zt = (torch.tensor(a, requires_grad=True) for a in (Q, K, V, z))
    outs = []
    for a, b in zip(cu[:-1], cu[1:]):
        per_head = []
        for h in range(4):
            g = h // 2
            sel = np.sort(np.argsort(-z[h, a:b], kind="stable")[:k]) + a
            S = scale * Qt[a:b, h] @ Kt[sel, g].T + zt[h, sel][None, :]
            per_head.append(torch.softmax(S, dim=-1) @ Vt[sel, g])
            assert np.allclose(LSE[h, a:b], torch.logsumexp(S, dim=-1).detach().numpy(), rtol=1e-12)
        outs.append(torch.stack(per_head, dim=1))
    Ot = torch.cat(outs, dim=0)
    assert np.allclose(O, Ot.detach().numpy(), rtol=1e-11, atol=1e-13)
    (Ot * torch.tensor(dO)).sum().backward()
    assert np.allclose(dQ, Qt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dK, Kt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dV, Vt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dz, zt.grad.numpy(), rtol=1e-10, atol=1e-12)
    tk = orc.topk_indices(z[1, 20:50], k, causal=False)
    assert (tk == tk[0]).all() and (tk[0] == np.sort(np.argsort(-z[1, 20:50], kind="stable")[:k])).all()


def test_noncausal_full_window_is_bidirectional_sdpa():
    Q, K, V, dO, z = rand_case(n=33, H_q=2, H_kv=2, d=8, seed=32)
    O, _ = orc.dma_forward(Q, K, V, np.zeros_like(z), np.array([0, 33]), 64, causal=False)
    q, kk, v = (torch.tensor(a).permute(1, 0, 2)[None] for a in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(q, kk, v, is_causal=False)[0].permute(1, 0, 2).numpy()
    assert np.allclose(O, ref, rtol=1e-10, atol=1e-12)


# ----------------------------------------------------------------------------- mask-path backward (chain rule of Eq. 3)
def _mask_case(seed=3, T=23, H_q=6, H_kv=2, d=5):
    r = np.random.default_rng(seed)
    V = r.standard_normal((T, H_kv, d))
    W = r.standard_normal((H_q, d)) / math.sqrt(d)
    A = -r.uniform(0.5, 2.0, H_q)
    dz = r.standard_normal((H_q, T))
    return V, W, A, dz, H_q


def test_mask_backward_matches_finite_differences():
    """Catches: a dropped factor (A, z or the sigmoid), softplus' taken as 1, a wrong head -> kv-head
    map, dVz not summed over the q-heads of a group, dA using x instead of softplus(x)."""
    V, W, A, dz, H_q = _mask_case()
    dW, dA, dVz = orc.mask_backward(V, W, A, dz, H_q)

    def loss(V_, W_, A_):
        return float(np.sum(dz * orc.z_scores(V_, W_, A_, H_q)))

    eps = 1e-6
    r = np.random.default_rng(11)
    for _ in range(12):
        h, c = int(r.integers(H_q)), int(r.integers(W.shape[1]))
        Wp, Wm = W.copy(), W.copy(); Wp[h, c] += eps; Wm[h, c] -= eps
        assert abs((loss(V, Wp, A) - loss(V, Wm, A)) / (2 * eps) - dW[h, c]) <= 1e-6 * (1 + abs(dW[h, c]))
        t, g = int(r.integers(V.shape[0])), int(r.integers(V.shape[1]))
        Vp, Vm = V.copy(), V.copy(); Vp[t, g, c] += eps; Vm[t, g, c] -= eps
        assert abs((loss(Vp, W, A) - loss(Vm, W, A)) / (2 * eps) - dVz[t, g, c]) <= 1e-6 * (1 + abs(dVz[t, g, c]))
    for h in range(H_q):
        Ap, Am = A.copy(), A.copy(); Ap[h] += eps; Am[h] -= eps
        assert abs((loss(V, W, Ap) - loss(V, W, Am)) / (2 * eps) - dA[h]) <= 1e-6 * (1 + abs(dA[h]))


def test_mask_backward_matches_autograd_of_the_forward_formula():
    """Independent derivation: torch differentiates exp(A * softplus(V w)) itself."""
    V, W, A, dz, H_q = _mask_case(seed=5, T=40, H_q=4, H_kv=4, d=7)
    dW, dA, dVz = orc.mask_backward(V, W, A, dz, H_q)
    Vt = torch.tensor(V, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    At = torch.tensor(A, requires_grad=True)
    G = H_q // V.shape[1]
    z = torch.stack([torch.exp(At[h] * torch.nn.functional.softplus(Vt[:, h // G, :] @ Wt[h])) for h in range(H_q)])
    (z * torch.tensor(dz)).sum().backward()
    assert np.allclose(Wt.grad.numpy(), dW, rtol=1e-10, atol=1e-12)
    assert np.allclose(At.grad.numpy(), dA, rtol=1e-10, atol=1e-12)
    assert np.allclose(Vt.grad.numpy(), dVz, rtol=1e-10, atol=1e-12)


def test_mask_backward_special_cases():
    """dz = 0 gives zero gradients; A = 0 makes z constant in V and W (dW = dVz = 0) while
    dA = sum dz * softplus(x); one q-head per kv-head gives dVz = outer(dx, w)."""
    V, W, A, dz, H_q = _mask_case(seed=8, H_q=2, H_kv=2)
    dW, dA, dVz = orc.mask_backward(V, W, A, np.zeros_like(dz), H_q)
    assert not dW.any() and not dA.any() and not dVz.any()
    dW, dA, dVz = orc.mask_backward(V, W, np.zeros_like(A), dz, H_q)
    assert not dW.any() and not dVz.any()
    sp = np.stack([orc.softplus(V[:, h, :] @ W[h]) for h in range(H_q)])
    assert np.allclose(dA, (dz * sp).sum(1))


# ----------------------------------------------------------------------------- cross-head scores (Eq. 3 with the full Delta)
def _xhead_case(seed=4, T=19, H_q=6, H_kv=3, d=5):
    r = np.random.default_rng(seed)
    V = r.standard_normal((T, H_kv, d))
    Delta = r.standard_normal((H_q, H_kv * d)) / math.sqrt(H_kv * d)
    A = -r.uniform(0.5, 2.0, H_q)
    dz = r.standard_normal((H_q, T))
    return V, Delta, A, dz


def test_xhead_scores_match_torch_linear():
    """Listing 1's form, with library routines: a linear layer on the token's flattened values, then
    softplus, gate and exp.  Catches a transposed Delta and a wrong flattening order of (head, channel)."""
    V, Delta, A, _ = _xhead_case()
    z = orc.z_scores_xhead(V, Delta, A)
    x = torch.nn.functional.linear(torch.tensor(V).reshape(V.shape[0], -1), torch.tensor(Delta))
    zt = torch.exp(torch.tensor(A) * torch.nn.functional.softplus(x)).T
    assert z.shape == (Delta.shape[0], V.shape[0])
    assert np.allclose(z, zt.numpy(), rtol=1e-12, atol=0)


def test_xhead_with_block_structure_is_the_per_head_form():
    """Delta[h] zero outside the block of kv-head g(h) reduces both functions to z_scores /
    mask_backward with w_h = that block."""
    V, W, A, dz, H_q = _mask_case(seed=9, T=31, H_q=6, H_kv=3, d=4)
    H_kv, d = V.shape[1], V.shape[2]
    G = H_q // H_kv
    Delta = np.zeros((H_q, H_kv * d))
    for h in range(H_q):
        Delta[h, (h // G) * d:(h // G + 1) * d] = W[h]
    assert np.allclose(orc.z_scores_xhead(V, Delta, A), orc.z_scores(V, W, A, H_q), rtol=1e-13, atol=0)
    dD, dA, dVz = orc.xhead_backward(V, Delta, A, dz)
    dW, dA2, dVz2 = orc.mask_backward(V, W, A, dz, H_q)
    for h in range(H_q):
        assert np.allclose(dD[h, (h // G) * d:(h // G + 1) * d], dW[h], rtol=1e-12, atol=1e-14)
    assert np.allclose(dA, dA2, rtol=1e-12, atol=1e-14)
    assert np.allclose(dVz, dVz2, rtol=1e-12, atol=1e-14)


def test_xhead_backward_matches_finite_differences_and_autograd():
    """Catches: dDelta missing the off-group blocks, dVz summed over one group only, a dropped
    factor, dA using x instead of softplus(x)."""
    V, Delta, A, dz = _xhead_case(seed=6)
    dD, dA, dVz = orc.xhead_backward(V, Delta, A, dz)

    def loss(V_, D_, A_):
        return float(np.sum(dz * orc.z_scores_xhead(V_, D_, A_)))

    eps = 1e-6
    r = np.random.default_rng(12)
    for _ in range(12):
        h, c = int(r.integers(Delta.shape[0])), int(r.integers(Delta.shape[1]))
        Dp, Dm = Delta.copy(), Delta.copy(); Dp[h, c] += eps; Dm[h, c] -= eps
        assert abs((loss(V, Dp, A) - loss(V, Dm, A)) / (2 * eps) - dD[h, c]) <= 1e-6 * (1 + abs(dD[h, c]))
        t, g, cc = int(r.integers(V.shape[0])), int(r.integers(V.shape[1])), int(r.integers(V.shape[2]))
        Vp, Vm = V.copy(), V.copy(); Vp[t, g, cc] += eps; Vm[t, g, cc] -= eps
        assert abs((loss(Vp, Delta, A) - loss(Vm, Delta, A)) / (2 * eps) - dVz[t, g, cc]) <= 1e-6 * (1 + abs(dVz[t, g, cc]))
    for h in range(len(A)):
        Ap, Am = A.copy(), A.copy(); Ap[h] += eps; Am[h] -= eps
        assert abs((loss(V, Delta, Ap) - loss(V, Delta, Am)) / (2 * eps) - dA[h]) <= 1e-6 * (1 + abs(dA[h]))
    Vt, Dt, At = (torch.tensor(a, requires_grad=True) for a in (V, Delta, A))
    z = torch.exp(At * torch.nn.functional.softplus(torch.nn.functional.linear(Vt.reshape(V.shape[0], -1), Dt))).T
    (z * torch.tensor(dz)).sum().backward()
    assert np.allclose(Dt.grad.numpy(), dD, rtol=1e-10, atol=1e-12)
    assert np.allclose(At.grad.numpy(), dA, rtol=1e-10, atol=1e-12)
    assert np.allclose(Vt.grad.numpy(), dVz, rtol=1e-10, atol=1e-12)


# ----------------------------------------------------------------------------- decode (last row of every document)
@pytest.mark.parametrize("ties", [False, True])
def test_decode_equals_last_rows_of_the_dense_forward(ties):
    """Catches: candidates not being the whole document, a wrong tie rule in the selection, the bias
    left out, a kv-head mix-up under GQA, k larger than a document."""
    Q, K, V, dO, z = rand_case(n=90, H_q=4, H_kv=2, d=8, seed=21, ties=ties)
    cu = np.array([0, 37, 37, 60, 90])            # includes an empty document and one shorter than k
    k = 25
    last = [int(e) - 1 for a, e in zip(cu[:-1], cu[1:])]
    q = np.stack([Q[max(i, 0)] for i in last])     # (the empty document's query is never used)
    o, lse, kept = orc.dma_decode(q, K, V, z, cu, k)
    O, LSE = orc.dma_forward(Q, K, V, z, cu, k)
    for b, (a, e) in enumerate(zip(cu[:-1], cu[1:])):
        if e == a:
            assert not o[b].any() and np.isneginf(lse[:, b]).all() and kept[b].shape[1] == 0
            continue
        assert np.allclose(o[b], O[e - 1], rtol=1e-12, atol=1e-14)
        assert np.allclose(lse[:, b], LSE[:, e - 1], rtol=1e-12, atol=1e-14)
        for h in range(4):
            ref = orc.topk_indices(z[h, a:e], k)[-1]
            assert (kept[b][h] == ref[ref >= 0] + a).all()
