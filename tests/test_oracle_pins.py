"""Pins of the float64 CPU oracle against things other than itself.

Each test names the fact it rests on: a definition or identity of the paper (arXiv
2410.09397, Sec. 3.1 and App. B.4 / C.1), a closed form, finite differences of the forward
loss, or an independent library evaluation.  None of them needs a GPU.
"""
import json
import os

import numpy as np
import pytest

from oracle import attn_oracle as orc

RNG = np.random.default_rng(20241009)
HERE = os.path.dirname(os.path.abspath(__file__))


def rand(*shape, std=1.0):
    return RNG.standard_normal(shape) * std


def tri_blocks(nblk):
    return np.tril(np.ones((nblk, nblk), dtype=np.uint8))


MASKS = {
    "dense": dict(causal=False, keep=None, block=1),
    "causal": dict(causal=True, keep=None, block=1),
    "blocks": dict(causal=False, block=3,
                   keep=np.array([[1, 0, 1], [0, 1, 0], [1, 1, 1]], dtype=np.uint8)),
    "causal+blocks": dict(causal=True, block=3,
                          keep=np.array([[1, 0, 0], [0, 1, 0], [1, 1, 1]], dtype=np.uint8)),
}


def loss(Q, K, V, dO, scale, **mask):
    O, _ = orc.attn_fwd(Q, K, V, scale, **mask)
    return float((O * dO).sum())


# --------------------------------------------------------------------- finite differences
@pytest.mark.parametrize("mask", list(MASKS))
def test_backward_matches_central_differences_of_forward(mask):
    """dQ, dK, dV are the gradients of L = sum(O o dO): every entry, step 1e-5."""
    n, d, scale, m = 9, 4, 0.7, MASKS[mask]
    Q, K, V, dO = (rand(1, 1, n, d) for _ in range(4))
    O, LSE = orc.attn_fwd(Q, K, V, scale, **m)
    grads = orc.attn_bwd(Q, K, V, O, dO, LSE, scale, **m)
    eps = 1e-5
    for which, g in zip(range(3), grads):
        num = np.zeros_like(g)
        for idx in np.ndindex(*g.shape):
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][idx] += eps
            lp = loss(*args, dO, scale, **m)
            args[which][idx] -= 2 * eps
            lm = loss(*args, dO, scale, **m)
            num[idx] = (lp - lm) / (2 * eps)
        assert np.abs(num - g).max() < 1e-8 * max(1.0, np.abs(g).max()) + 2e-9, (mask, which)


# ------------------------------------------------------- the paper's own gradient (Def. 3.2)
def test_paper_weight_gradient_equals_A1T_dQ_and_finite_differences():
    """With Q = A_1 X, K = A_2, V = A_3 Y and scale 1, dL/dX = A_1^T p A_2 = A_1^T dQ.
    g is evaluated by separate oracle code written from Def. 3.2 (no LSE, no shift)."""
    n, d = 7, 3
    A1, A2, A3, dO = (rand(n, d, std=0.6) for _ in range(4))
    X, Y = rand(d, d, std=0.6), rand(d, d, std=0.6)
    g, f, q, p = orc.wgrad(A1, A2, A3, dO, X, Y)
    Q, K, V = (A1 @ X)[None, None], A2[None, None], (A3 @ Y)[None, None]
    O, LSE = orc.attn_fwd(Q, K, V, 1.0)
    dQ, dK, dV, f2, q2, p2 = orc.attn_bwd_head(Q[0, 0], K[0, 0], V[0, 0], O[0, 0], dO, LSE[0, 0], 1.0)
    assert np.allclose(f, f2, rtol=1e-12, atol=1e-14)
    assert np.allclose(q, q2, rtol=1e-12, atol=1e-14)
    assert np.allclose(p, p2, rtol=1e-10, atol=1e-13)
    assert np.allclose(g, A1.T @ dQ, rtol=1e-10, atol=1e-12)
    # dL/dA_2 by the chain rule is dK; dL/dY = A_3^T dV
    eps = 1e-5
    num = np.zeros_like(X)
    for idx in np.ndindex(d, d):
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += eps
        Xm[idx] -= eps
        num[idx] = (loss((A1 @ Xp)[None, None], K, V, dO[None, None], 1.0)
                    - loss((A1 @ Xm)[None, None], K, V, dO[None, None], 1.0)) / (2 * eps)
    assert np.abs(num - g).max() < 1e-8
    numY = np.zeros_like(Y)
    for idx in np.ndindex(d, d):
        Yp, Ym = Y.copy(), Y.copy()
        Yp[idx] += eps
        Ym[idx] -= eps
        numY[idx] = (loss(Q, K, (A3 @ Yp)[None, None], dO[None, None], 1.0)
                     - loss(Q, K, (A3 @ Ym)[None, None], dO[None, None], 1.0)) / (2 * eps)
    assert np.abs(numY - A3.T @ dV).max() < 1e-8


# ------------------------------------------------- the four-phase small-cache scheme (App. C)
@pytest.mark.parametrize("n,d,B", [(7, 3, 1), (7, 3, 2), (8, 4, 2), (8, 4, 4), (9, 5, 3), (6, 6, 16), (10, 4, 7)])
def test_small_cache_scheme_computes_the_same_gradient(n, d, B):
    """Four phases over B x B blocks, every n x n intermediate through memory, give the g of
    Def. 3.2 (App. C: "calculates the same gradients"), for block edges that divide n and d,
    that do not, and that exceed both."""
    A1, A2, A3, dO = (rand(n, d, std=0.6) for _ in range(4))
    X, Y = rand(d, d, std=0.6), rand(d, d, std=0.6)
    g, _, _, _ = orc.wgrad(A1, A2, A3, dO, X, Y)
    gb, rd, wr = orc.small_cache_wgrad(A1, A2, A3, dO, X, Y, B)
    assert np.allclose(gb, g, rtol=1e-11, atol=1e-13)
    assert rd > 0 and wr > 0


@pytest.mark.parametrize("n,d,B", [(8, 4, 2), (12, 6, 3), (16, 8, 4), (16, 16, 8)])
def test_small_cache_scheme_moves_what_its_lemmas_count(n, d, B):
    """Element transfers of the replayed schedule against the count of its own block loops (B | n,
    B | d): every block product reads two B x B blocks per k-step and writes its block once; the
    elementwise passes read and write n x n.  With B = sqrt(M / 4) the total is
    12 (n^2 d + n d^2) / sqrt(M) + O(n^2): the O((n^2 d + n d^2) / sqrt(M)) of Thm 4.3."""
    A1, A2, A3, dO = (rand(n, d, std=0.4) for _ in range(4))
    X, Y = rand(d, d, std=0.4), rand(d, d, std=0.4)
    _, rd, wr = orc.small_cache_wgrad(A1, A2, A3, dO, X, Y, B)
    nb, db = n // B, d // B
    prod = lambda mb, nb_, kb: 2 * B * B * mb * nb_ * kb  # operand reads of one blocked product
    reads = (2 * prod(nb, db, db)      # S = A_1 X, h = A_3 Y
             + 2 * prod(nb, nb, db)    # S A_2^T, dO h^T
             + prod(db, nb, nb)        # T = A_1^T p
             + prod(db, db, nb)        # g = T A_2
             + n * n + (n * n + n)     # exp / row-sum pass; normalisation pass (reads l)
             + 4 * n * n)              # phase 3: f and q twice
    writes = 2 * n * d + 2 * n * n + (n * n + n) + n * n + n * n + d * n + d * d
    assert rd == reads and wr == writes
    M = 4 * B * B
    lead = 12 * (n * n * d + n * d * d) / np.sqrt(M)
    assert abs(rd - (lead + 6 * n * n + n)) < 1e-9


# ----------------------------------------------------------------------------- invariants
@pytest.mark.parametrize("mask", list(MASKS))
def test_row_identities_of_f_q_p(mask):
    """Rows of f sum to 1; rows of p sum to 0; (f o q) 1 = (O o dO) 1 (the two matrix forms
    of p); <dQ,Q> = <dK,K>; column sums of dV equal those of dO."""
    n, d, scale, m = 9, 5, 0.45, MASKS[mask]
    Q, K, V, dO = (rand(n, d) for _ in range(4))
    O, LSE = orc.attn_fwd(Q[None, None], K[None, None], V[None, None], scale, **m)
    O, LSE = O[0, 0], LSE[0, 0]
    dQ, dK, dV, f, q, p = orc.attn_bwd_head(Q, K, V, O, dO, LSE, scale, **m)
    assert np.allclose(f.sum(1), 1.0, atol=1e-13)
    assert np.abs(p.sum(1)).max() < 1e-13
    assert np.allclose((f * q).sum(1), (O * dO).sum(1), atol=1e-12)
    assert np.isclose((dQ * Q).sum(), (dK * K).sum(), atol=1e-12)
    assert np.allclose(dV.sum(0), dO.sum(0), atol=1e-12)
    # masked entries are exactly zero
    for i in range(n):
        for j in range(n):
            vis = (not m["causal"] or j <= i) and (m["keep"] is None or m["keep"][i // m["block"], j // m["block"]])
            if not vis:
                assert f[i, j] == 0.0 and p[i, j] == 0.0


def test_key_shift_and_key_permutation():
    """Adding one vector c to every key leaves f, O and all gradients unchanged and moves
    LSE_i by scale q_i.c; permuting keys permutes dK, dV and fixes O, dQ (no mask)."""
    n, d, scale = 10, 4, 0.5
    Q, K, V, dO = (rand(1, 1, n, d) for _ in range(4))
    c = rand(d)
    O, LSE = orc.attn_fwd(Q, K, V, scale)
    O2, LSE2 = orc.attn_fwd(Q, K + c, V, scale)
    assert np.allclose(O, O2, atol=1e-13)
    assert np.allclose(LSE2 - LSE, scale * (Q @ c), atol=1e-12)
    g = orc.attn_bwd(Q, K, V, O, dO, LSE, scale)
    g2 = orc.attn_bwd(Q, K + c, V, O2, dO, LSE2, scale)
    for a, b in zip(g, g2):
        assert np.allclose(a, b, atol=1e-12)
    perm = RNG.permutation(n)
    O3, LSE3 = orc.attn_fwd(Q, K[:, :, perm], V[:, :, perm], scale)
    g3 = orc.attn_bwd(Q, K[:, :, perm], V[:, :, perm], O3, dO, LSE3, scale)
    assert np.allclose(O3, O, atol=1e-13) and np.allclose(g3[0], g[0], atol=1e-12)
    assert np.allclose(g3[1], g[1][:, :, perm], atol=1e-12)
    assert np.allclose(g3[2], g[2][:, :, perm], atol=1e-12)


# --------------------------------------------------------------------------- closed forms
def test_closed_form_single_key():
    """n = 1: f = 1, O = V, LSE = scale q.k, dV = dO, dQ = dK = 0."""
    d, scale = 5, 0.3
    Q, K, V, dO = (rand(1, 1, 1, d) for _ in range(4))
    O, LSE = orc.attn_fwd(Q, K, V, scale)
    assert np.allclose(O, V) and np.isclose(LSE[0, 0, 0], scale * (Q * K).sum())
    dQ, dK, dV = orc.attn_bwd(Q, K, V, O, dO, LSE, scale)
    assert np.allclose(dV, dO) and np.abs(dQ).max() < 1e-15 and np.abs(dK).max() < 1e-15


def test_closed_form_zero_queries():
    """Q = 0, no mask: f = 1/n, O = column mean of V, LSE = log n, dV_j = mean_i dO_i,
    dK = 0 and dQ_i = scale/n sum_j (dO_i.V_j - dO_i.mean V) K_j."""
    n, d, scale = 8, 3, 0.9
    K, V, dO = (rand(1, 1, n, d) for _ in range(3))
    Q = np.zeros_like(K)
    O, LSE = orc.attn_fwd(Q, K, V, scale)
    assert np.allclose(O, V.mean(2, keepdims=True)) and np.allclose(LSE, np.log(n))
    dQ, dK, dV = orc.attn_bwd(Q, K, V, O, dO, LSE, scale)
    assert np.allclose(dV, np.broadcast_to(dO.mean(2, keepdims=True), dV.shape))
    assert np.abs(dK).max() < 1e-15
    dP = dO[0, 0] @ V[0, 0].T
    dS = (dP - dP.mean(1, keepdims=True)) / n
    assert np.allclose(dQ[0, 0], scale * dS @ K[0, 0], atol=1e-13)


def test_closed_form_causal_first_row():
    """Causal: query 0 sees only key 0, so O_0 = V_0, LSE_0 = scale q_0.k_0, dQ_0 = 0."""
    n, d, scale = 6, 4, 0.5
    Q, K, V, dO = (rand(1, 1, n, d) for _ in range(4))
    O, LSE = orc.attn_fwd(Q, K, V, scale, causal=True)
    assert np.allclose(O[0, 0, 0], V[0, 0, 0])
    assert np.isclose(LSE[0, 0, 0], scale * Q[0, 0, 0] @ K[0, 0, 0])
    dQ, dK, dV = orc.attn_bwd(Q, K, V, O, dO, LSE, scale, causal=True)
    assert np.abs(dQ[0, 0, 0]).max() < 1e-15
    # the last key is seen by the last query only
    f_last = np.exp(scale * Q[0, 0, -1] @ K[0, 0, -1] - LSE[0, 0, -1])
    assert np.allclose(dV[0, 0, -1], f_last * dO[0, 0, -1])


def test_hand_worked_example():
    """n = 2, d = 1 example worked by hand from the definitions (fixture cites them)."""
    with open(os.path.join(HERE, "golden", "hand_n2_d1.json")) as fh:
        g = json.load(fh)
    a = lambda k: np.array(g[k], dtype=np.float64).reshape(1, 1, 2, 1)
    O, LSE = orc.attn_fwd(a("Q"), a("K"), a("V"), g["scale"])
    assert np.allclose(O.ravel(), g["O"], atol=1e-14) and np.allclose(LSE.ravel(), g["LSE"], atol=1e-14)
    dQ, dK, dV = orc.attn_bwd(a("Q"), a("K"), a("V"), O, a("dO"), LSE, g["scale"])
    assert np.allclose(dQ.ravel(), g["dQ"], atol=1e-14)
    assert np.allclose(dK.ravel(), g["dK"], atol=1e-14)
    assert np.allclose(dV.ravel(), g["dV"], atol=1e-14)


# ------------------------------------------------------------------ brute-force equalities
def test_all_ones_block_mask_is_dense_and_triangular_unit_blocks_is_causal():
    n, d, scale = 12, 4, 0.5
    Q, K, V, dO = (rand(2, 2, n, d) for _ in range(4))
    ref = orc.attn_fwd(Q, K, V, scale)
    ones = orc.attn_fwd(Q, K, V, scale, keep=np.ones((3, 3), np.uint8), block=4)
    assert all(np.array_equal(a, b) for a, b in zip(ref, ones))
    gr = orc.attn_bwd(Q, K, V, *[ref[0], dO, ref[1]], scale)
    go = orc.attn_bwd(Q, K, V, *[ones[0], dO, ones[1]], scale, keep=np.ones((3, 3), np.uint8), block=4)
    assert all(np.array_equal(a, b) for a, b in zip(gr, go))
    cz = orc.attn_fwd(Q, K, V, scale, causal=True)
    tz = orc.attn_fwd(Q, K, V, scale, keep=tri_blocks(n), block=1)
    assert all(np.array_equal(a, b) for a, b in zip(cz, tz))
    gc = orc.attn_bwd(Q, K, V, cz[0], dO, cz[1], scale, causal=True)
    gt = orc.attn_bwd(Q, K, V, tz[0], dO, tz[1], scale, keep=tri_blocks(n), block=1)
    assert all(np.array_equal(a, b) for a, b in zip(gc, gt))


def test_sampled_backward_equals_full_backward():
    n, d, scale = 24, 6, 0.4
    keep = np.array([[1, 1, 0], [0, 1, 1], [1, 0, 1]], dtype=np.uint8)
    Q, K, V, dO = (rand(n, d) for _ in range(4))
    for m in (dict(causal=False, keep=None, block=1), dict(causal=True, keep=None, block=1),
              dict(causal=False, keep=keep, block=8)):
        O, LSE = orc.attn_fwd(Q[None, None], K[None, None], V[None, None], scale, **m)
        dQ, dK, dV, *_ = orc.attn_bwd_head(Q, K, V, O[0, 0], dO, LSE[0, 0], scale, **m)
        qr, kr = [0, 5, 23, 11], [23, 0, 7]
        sQ, sK, sV = orc.attn_bwd_sampled(Q, K, V, O[0, 0], dO, LSE[0, 0], scale, qr, kr, **m)
        assert np.allclose(sQ, dQ[qr], atol=1e-14) and np.allclose(sK, dK[kr], atol=1e-14)
        assert np.allclose(sV, dV[kr], atol=1e-14)


def test_fully_masked_row_is_zero():
    """A query block row that keeps no key block: O = 0, LSE = -inf, no gradient from it."""
    n, d = 4, 2
    keep = np.array([[1, 0], [0, 0]], dtype=np.uint8)
    Q, K, V, dO = (rand(1, 1, n, d) for _ in range(4))
    O, LSE = orc.attn_fwd(Q, K, V, 1.0, keep=keep, block=2)
    assert np.all(O[0, 0, 2:] == 0) and np.all(np.isneginf(LSE[0, 0, 2:]))
    dQ, dK, dV = orc.attn_bwd(Q, K, V, O, dO, LSE, 1.0, keep=keep, block=2)
    assert np.all(dQ[0, 0, 2:] == 0) and np.all(dK[0, 0, 2:] == 0) and np.all(dV[0, 0, 2:] == 0)
    assert np.all(np.isfinite(dQ)) and np.all(np.isfinite(dK)) and np.all(np.isfinite(dV))


# ------------------------------------------------------ independent library evaluation
@pytest.mark.parametrize("mask", list(MASKS))
def test_against_float64_softmax_autograd(mask):
    """Second opinion: torch.softmax + autograd in float64 on the same inputs."""
    import torch
    n, d, scale, m = 9, 6, 0.37, MASKS[mask]
    b, h = 2, 3
    Q, K, V, dO = (rand(b, h, n, d) for _ in range(4))
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    s = scale * tq @ tk.transpose(-1, -2)
    vis = torch.ones(n, n, dtype=torch.bool)
    if m["causal"]:
        vis &= torch.tril(torch.ones(n, n, dtype=torch.bool))
    if m["keep"] is not None:
        kb = torch.tensor(m["keep"], dtype=torch.bool)
        vis &= kb.repeat_interleave(m["block"], 0).repeat_interleave(m["block"], 1)[:n, :n]
    s = s.masked_fill(~vis, float("-inf"))
    o = torch.softmax(s, -1) @ tv
    (o * torch.tensor(dO)).sum().backward()
    O, LSE = orc.attn_fwd(Q, K, V, scale, **m)
    assert np.allclose(O, o.detach().numpy(), atol=1e-13)
    assert np.allclose(LSE, torch.logsumexp(s, -1).detach().numpy(), atol=1e-13)
    dQ, dK, dV = orc.attn_bwd(Q, K, V, O, dO, LSE, scale, **m)
    assert np.allclose(dQ, tq.grad.numpy(), atol=1e-12)
    assert np.allclose(dK, tk.grad.numpy(), atol=1e-12)
    assert np.allclose(dV, tv.grad.numpy(), atol=1e-12)
