"""Pins of the learning-to-hash oracle (oracle/hash_train_oracle.py) against things it does not
compute itself: central finite differences, closed forms worked with math.tanh, invariants of the
three loss terms, hand-worked label fixtures, torch's SGD and autograd on the CPU."""
import math
import os

import numpy as np
import pytest

from oracle import hash_train_oracle as T

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def small_problem(seed=0, n=24, d=6, r=5):
    rng = np.random.default_rng(seed)
    Q = rng.normal(size=(n, d))
    K = rng.normal(size=(n, d))
    s = np.where(rng.random(n) < 0.2, rng.uniform(1, 20, n), -1.0)
    W = rng.normal(size=(d, r)) * 0.7
    return Q, K, s, W


def test_relaxed_hash_is_tanh_of_half_and_tends_to_the_sign():
    x = np.array([[0.3, -1.2, 2.0]])
    W = np.array([[1.0, -2.0], [0.5, 0.25], [-1.0, 3.0]])
    z = x @ W
    for sig in (0.1, 0.7):
        want = [[math.tanh(sig * v / 2.0) for v in z[0]]]
        assert np.allclose(T.relaxed_hash(x, W, sig), want, rtol=0, atol=1e-15)
    # a steep sigmoid reproduces the sign code of Alg. 2 (h in {-1, 1})
    assert np.array_equal(np.sign(T.relaxed_hash(x, W, 500.0)), np.sign(z))
    assert np.array_equal(T.sign_codes(x, W), (z >= 0).astype(np.uint8))


def test_single_triplet_closed_form():
    # d = r = 1, one triplet: every term has a one-line closed form
    q, k, s, w, sig, eps, eta, lam = 1.5, -0.5, 7.0, 0.8, 0.3, 0.01, 2.0, 1.0
    hq, hk = math.tanh(sig * q * w / 2), math.tanh(sig * k * w / 2)
    want = (eps * s * (hq - hk) ** 2, eta * hk ** 2, lam * abs(w * w - 1.0))
    got = T.loss_terms([[q]], [[k]], [s], [[w]], sig, eps, eta, lam)
    assert np.allclose(got, want, rtol=1e-14, atol=0)
    loss, g = T.loss_and_grad([[q]], [[k]], [s], [[w]], sig, eps, eta, lam)
    assert math.isclose(loss, sum(want), rel_tol=1e-14)
    # derivative by hand: d tanh(c w)/dw = c (1 - tanh^2)
    cq, ck = sig * q / 2, sig * k / 2
    dhq, dhk = cq * (1 - hq * hq), ck * (1 - hk * hk)
    dwant = eps * s * 2 * (hq - hk) * (dhq - dhk) + eta * 2 * hk * dhk + lam * math.copysign(2 * w, w * w - 1)
    assert math.isclose(float(g[0, 0]), dwant, rel_tol=1e-12)


def test_term_invariants():
    Q, K, s, W = small_problem(1)
    # identical query and key of every triplet: the similarity term vanishes
    assert T.loss_terms(K, K, s, W)[0] == 0.0
    # keys in (k, -k) pairs: h is odd, the bit sums cancel, the balance term vanishes
    K2 = np.concatenate([K, -K])
    assert T.loss_terms(np.concatenate([Q, Q]), K2, np.concatenate([s, s]), W)[1] < 1e-28
    # orthonormal columns: W^T W = I, the uncorrelation term vanishes; W = 0 gives ||I||_F = sqrt(r)
    Wo, _ = np.linalg.qr(np.random.default_rng(2).normal(size=(6, 5)))
    assert T.loss_terms(Q, K, s, Wo)[2] < 1e-14
    assert math.isclose(T.loss_terms(Q, K, s, np.zeros((6, 5)))[2], math.sqrt(5.0), rel_tol=1e-15)
    # the similarity term is linear in the labels and in eps; the scale factors multiply their terms
    a = T.loss_terms(Q, K, s, W, eps=0.01)
    b = T.loss_terms(Q, K, 3.0 * s, W, eps=0.02, scale_sim=0.5, scale_bal=0.25)
    assert math.isclose(b[0], 3.0 * a[0], rel_tol=1e-13) and math.isclose(b[1], 0.25 * a[1], rel_tol=1e-13)
    # a positive pair pulled apart costs more than the same pair close together
    far = T.loss_terms([[1.0, 0, 0, 0, 0, 0]], [[-1.0, 0, 0, 0, 0, 0]], [5.0], W)[0]
    near = T.loss_terms([[1.0, 0, 0, 0, 0, 0]], [[0.9, 0, 0, 0, 0, 0]], [5.0], W)[0]
    assert far > near > 0


@pytest.mark.parametrize("which", ["sim", "bal", "unc", "all"])
def test_gradient_matches_central_finite_differences(which):
    Q, K, s, W = small_problem(3)
    kw = dict(sigma=0.4, eps=0.01 if which in ("sim", "all") else 0.0,
              eta=2.0 if which in ("bal", "all") else 0.0, lam=1.0 if which in ("unc", "all") else 0.0,
              scale_sim=0.7, scale_bal=0.3)
    _, g = T.loss_and_grad(Q, K, s, W, **kw)
    num = np.zeros_like(W)
    h = 1e-6
    for i in range(W.shape[0]):
        for j in range(W.shape[1]):
            Wp, Wm = W.copy(), W.copy()
            Wp[i, j] += h
            Wm[i, j] -= h
            num[i, j] = (sum(T.loss_terms(Q, K, s, Wp, **kw)) - sum(T.loss_terms(Q, K, s, Wm, **kw))) / (2 * h)
    assert np.max(np.abs(g - num)) <= 1e-7 * max(1.0, float(np.max(np.abs(num))))
    assert float(np.max(np.abs(num))) > 1e-4  # the check is not vacuous


def test_gradient_matches_torch_autograd():
    torch = pytest.importorskip("torch")
    Q, K, s, W = small_problem(4, n=40, d=8, r=7)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    Qt, Kt, st = (torch.tensor(a, dtype=torch.float64) for a in (Q, K, s))
    hq = 2 * torch.sigmoid(T.SIGMA * Qt @ Wt) - 1
    hk = 2 * torch.sigmoid(T.SIGMA * Kt @ Wt) - 1
    loss = (T.EPSILON * (st * ((hq - hk) ** 2).sum(1)).sum() + T.ETA * (hk.sum(0) ** 2).sum()
            + T.LAMBDA * torch.linalg.matrix_norm(Wt.T @ Wt - torch.eye(7, dtype=torch.float64)))
    loss.backward()
    got_l, got_g = T.loss_and_grad(Q, K, s, W)
    assert math.isclose(got_l, float(loss.detach()), rel_tol=1e-12)
    assert np.allclose(got_g, Wt.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_per_query_balance_closed_form_and_invariants():
    # two queries with one key each, d = r = 1: eta (h(k1)^2 + h(k2)^2) per query against
    # eta (h(k1) + h(k2))^2 when the batch counts as one query
    k1, k2, w, sig, eta = 0.9, -1.7, 1.3, 0.5, 2.0
    h1, h2 = math.tanh(sig * k1 * w / 2), math.tanh(sig * k2 * w / 2)
    args = ([[0.0], [0.0]], [[k1], [k2]], [0.0, 0.0], [[w]], sig, 0.0, eta, 0.0)
    assert math.isclose(T.loss_terms(*args, group=[0, 1])[1], eta * (h1 * h1 + h2 * h2), rel_tol=1e-14)
    assert math.isclose(T.loss_terms(*args)[1], eta * (h1 + h2) ** 2, rel_tol=1e-14)
    assert math.isclose(T.loss_terms(*args, group=[5, 5])[1], eta * (h1 + h2) ** 2, rel_tol=1e-14)
    Q, K, s, W = small_problem(8, n=30)
    # one group for everything is the ungrouped form; the names of the groups do not matter, nor
    # does the order of the triplets
    g = np.array([0] * 7 + [1] * 12 + [2] * 11)
    one = T.loss_and_grad(Q, K, s, W)
    same = T.loss_and_grad(Q, K, s, W, group=np.full(30, 3))
    assert one[0] == same[0] and np.array_equal(one[1], same[1])
    a = T.loss_and_grad(Q, K, s, W, group=g)
    b = T.loss_and_grad(Q, K, s, W, group=np.array([9, 4, 7])[g])
    assert math.isclose(a[0], b[0], rel_tol=1e-14) and np.allclose(a[1], b[1], rtol=1e-12, atol=1e-15)
    perm = np.random.default_rng(9).permutation(30)
    c = T.loss_and_grad(Q[perm], K[perm], s[perm], W, group=g[perm])
    assert math.isclose(a[0], c[0], rel_tol=1e-13) and np.allclose(a[1], c[1], rtol=1e-11, atol=1e-14)
    # the per-query balance term is the sum of the balance terms of the queries taken alone, and
    # it differs from the whole-batch form by the cross terms between queries
    parts = sum(T.loss_terms(Q[g == j], K[g == j], s[g == j], W)[1] for j in range(3))
    assert math.isclose(T.loss_terms(Q, K, s, W, group=g)[1], parts, rel_tol=1e-13)
    assert abs(T.loss_terms(Q, K, s, W, group=g)[1] - T.loss_terms(Q, K, s, W)[1]) > 1e-3
    # every query made of (k, -k) pairs: its bit sums cancel
    K2 = np.concatenate([K, -K])
    assert T.loss_terms(np.concatenate([Q, Q]), K2, np.concatenate([s, s]), W, group=np.concatenate([g, g]))[1] < 1e-28


@pytest.mark.parametrize("which", ["bal", "all"])
def test_per_query_gradient_matches_central_finite_differences(which):
    Q, K, s, W = small_problem(10, n=26)
    g = np.array([0] * 11 + [1] * 15)  # two queries
    kw = dict(sigma=0.4, eps=0.01 if which == "all" else 0.0, eta=2.0, lam=1.0 if which == "all" else 0.0,
              scale_sim=0.7, scale_bal=0.3, group=g)
    _, grad = T.loss_and_grad(Q, K, s, W, **kw)
    num = np.zeros_like(W)
    h = 1e-6
    for i in range(W.shape[0]):
        for j in range(W.shape[1]):
            Wp, Wm = W.copy(), W.copy()
            Wp[i, j] += h
            Wm[i, j] -= h
            num[i, j] = (sum(T.loss_terms(Q, K, s, Wp, **kw)) - sum(T.loss_terms(Q, K, s, Wm, **kw))) / (2 * h)
    assert np.max(np.abs(grad - num)) <= 1e-7 * max(1.0, float(np.max(np.abs(num))))
    assert float(np.max(np.abs(num))) > 1e-4
    # and it is not the gradient of the whole-batch form
    kw0 = dict(kw, group=None)
    assert np.max(np.abs(grad - T.loss_and_grad(Q, K, s, W, **kw0)[1])) > 1e-4


def test_per_query_gradient_matches_torch_autograd():
    torch = pytest.importorskip("torch")
    Q, K, s, W = small_problem(11, n=40, d=8, r=7)
    g = np.array([2] * 9 + [0] * 17 + [1] * 14)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    Qt, Kt, st = (torch.tensor(a, dtype=torch.float64) for a in (Q, K, s))
    hq = 2 * torch.sigmoid(T.SIGMA * Qt @ Wt) - 1
    hk = 2 * torch.sigmoid(T.SIGMA * Kt @ Wt) - 1
    bal = sum((hk[torch.tensor(g == j)].sum(0) ** 2).sum() for j in range(3))
    loss = (T.EPSILON * (st * ((hq - hk) ** 2).sum(1)).sum() + T.ETA * bal
            + T.LAMBDA * torch.linalg.matrix_norm(Wt.T @ Wt - torch.eye(7, dtype=torch.float64)))
    loss.backward()
    got_l, got_g = T.loss_and_grad(Q, K, s, W, group=g)
    assert math.isclose(got_l, float(loss.detach()), rel_tol=1e-12)
    assert np.allclose(got_g, Wt.grad.numpy(), rtol=1e-10, atol=1e-13)


def test_sgd_step_matches_torch_optimizer():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    W = rng.normal(size=(4, 3))
    p = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=T.LR, momentum=T.MOMENTUM, weight_decay=T.WEIGHT_DECAY)
    v = np.zeros_like(W)
    for step in range(4):
        g = rng.normal(size=W.shape)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        W, v = T.sgd_step(W, v, g)
        assert np.allclose(W, p.detach().numpy(), rtol=1e-13, atol=1e-15), step


def test_labels_hand_fixture():
    n = 0
    for line in open(os.path.join(GOLDEN, "labels_hand.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        sc, lab = line.split("|")
        got = T.make_labels([float(x) for x in sc.split()])
        assert np.array_equal(got, np.array([float(x) for x in lab.split()])), line
        n += 1
    assert n == 4


def test_labels_properties():
    rng = np.random.default_rng(6)
    sc = rng.normal(size=1000)
    lab = T.make_labels(sc)
    pos = lab > 0
    assert pos.sum() == 100 and np.all(lab[~pos] == -1.0)
    assert lab.max() == 20.0 and lab[pos].min() == 1.0
    assert sc[pos].min() >= sc[~pos].max()  # positives are the top of the ranking
    # labels decrease with the rank of the score, in equal steps
    order = np.argsort(-sc)[:100]
    steps = np.diff(lab[order])
    assert np.allclose(steps, -19.0 / 99.0, rtol=0, atol=1e-12)


def test_topk_and_recall():
    rng = np.random.default_rng(7)
    K = rng.normal(size=(200, 16))
    q = rng.normal(size=16)
    ex = T.exact_topk(q, K, 20)
    sc = K @ q
    assert set(ex) == set(np.argsort(-sc)[:20]) and np.all(np.diff(ex) > 0)
    assert T.recall(T.exact_topk(q, K, 200), np.arange(200)) == 1.0
    assert T.recall([1, 2, 3, 9], [2, 3, 4, 5]) == 0.5
    # with r = d and W = identity the code of a vector is the sign pattern of its channels
    W = np.eye(16)
    hk = T.hash_topk(q, K, W, 5)
    dist = np.sum((K >= 0) != (q >= 0)[None, :], axis=1)
    assert sorted(dist[hk]) == sorted(np.sort(dist, kind="stable")[:5])
    # a key equal to the query has distance 0 and is always selected
    K[77] = q
    assert 77 in T.hash_topk(q, K, rng.normal(size=(16, 32)), 1)
