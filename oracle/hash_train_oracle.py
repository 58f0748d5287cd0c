"""CPU oracle of the learning-to-hash side of HATA -- TEST INFRASTRUCTURE ONLY.

Plain numpy in fp64, written from the paper (Sec. 3.1 "Learning-to-Hash for Top-k Attention",
App. B "Configuration Details of HATA Training"); no blocking, no fusion.  Only tests, the smoke
check and the benchmark's ``cpu_baseline`` legs may import this module; it shares no code with
the HIP path.

Function -> passage of the paper:
  relaxed_hash     Sec. 3.1.1, the relaxation h(x) = 2 Sigmoid(sigma x W_H) - 1
  loss_terms       Sec. 3.1.1, the final hashing model (the three terms of the multi-query
                   objective): similarity, bit balance, uncorrelation
  loss_and_grad    the same and its gradient with respect to W_H (chain rule, written out)
  sgd_step         App. B.2, SGD with momentum and weight decay (hyper-parameter table)
  make_labels      App. B.1 steps 3-4: top 10 % of the qk scores positive with linearly decayed
                   labels in [1, 20], the rest -1
  exact_topk       Eq. 2, TopK(q K^T, N)
  hash_topk        Alg. 2 + Alg. 3 for one query: sign codes, Hamming distance, the N closest
  recall           overlap of the two index sets / N

Readings (the paper is silent or ambiguous; the HIP path takes the same ones):
  * the final hashing model sums the balance term per query j: eta * sum_j || sum_i h(k_{j,i}) ||^2.
    `group[n]` names the query a triplet belongs to and gives exactly that; without it the batch
    counts as one query (the triplets of a stored batch are shuffled, App. B.1 step 5, and carry
    no query index): eta * || sum_n h(k_n) ||^2;
  * || W^T W - I || is the Frobenius norm, not squared (the other two terms carry an explicit
    square in the paper, this one does not);
  * the sums are as printed; the optional factors scale_sim / scale_bal multiply the two data
    terms (1/N and 1/N^2 give the mean forms, which keep the printed learning rate usable);
  * "top 10 %" is floor(0.1 m) pairs, at least one; the best pair gets 20, the last positive 1,
    linearly in between (a single positive gets 20);
  * SGD follows the common convention g <- g + wd * W, v <- mu * v + g, W <- W - lr * v.
"""
from __future__ import annotations

import numpy as np

# App. B.2, hyper-parameter table
SIGMA = 0.1
EPSILON = 0.01
LAMBDA = 1.0
ETA = 2.0
LR = 0.1
WEIGHT_DECAY = 1e-6
MOMENTUM = 0.9


def relaxed_hash(x: np.ndarray, W: np.ndarray, sigma: float = SIGMA) -> np.ndarray:
    z = sigma * (np.asarray(x, np.float64) @ np.asarray(W, np.float64))
    return 2.0 / (1.0 + np.exp(-z)) - 1.0


def _group_ids(group, n):
    """Per-triplet query ids as consecutive integers 0 .. n_groups - 1 (None: one query)."""
    if group is None:
        return np.zeros(n, dtype=np.int64), 1
    group = np.asarray(group)
    assert group.shape == (n,)
    values, ids = np.unique(group, return_inverse=True)
    return ids.astype(np.int64), int(values.size)


def _group_sums(hk, ids, n_groups):
    """col[j] = sum of h(k_n) over the triplets of query j."""
    col = np.zeros((n_groups, hk.shape[1]))
    for n in range(hk.shape[0]):
        col[ids[n]] += hk[n]
    return col


def loss_terms(Q, K, s, W, sigma=SIGMA, eps=EPSILON, eta=ETA, lam=LAMBDA,
               scale_sim=1.0, scale_bal=1.0, group=None):
    """(similarity, balance, uncorrelation) for N triplets (Q[n], K[n], s[n]); W is [d, r];
    group [N]: the query each triplet belongs to (None: all one query)."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    s = np.asarray(s, np.float64)
    W = np.asarray(W, np.float64)
    hq = relaxed_hash(Q, W, sigma)
    hk = relaxed_hash(K, W, sigma)
    diff = hq - hk
    l_sim = eps * scale_sim * float(np.sum(s * np.sum(diff * diff, axis=1)))
    ids, n_groups = _group_ids(group, hk.shape[0])
    col = _group_sums(hk, ids, n_groups)
    l_bal = eta * scale_bal * float(np.sum(col * col))
    M = W.T @ W - np.eye(W.shape[1])
    l_unc = lam * float(np.sqrt(np.sum(M * M)))
    return l_sim, l_bal, l_unc


def loss_and_grad(Q, K, s, W, sigma=SIGMA, eps=EPSILON, eta=ETA, lam=LAMBDA,
                  scale_sim=1.0, scale_bal=1.0, group=None):
    """Total loss and dL/dW.

    With a = sigma Q W, b = sigma K W, hq = 2 Sigmoid(a) - 1, hk = 2 Sigmoid(b) - 1:
      dh/da = (1 - h^2) / 2
      dL/dhq_n =  2 eps s_n (hq_n - hk_n)
      dL/dhk_n = -2 eps s_n (hq_n - hk_n) + 2 eta sum_{m in the query of n} hk_m
      dL/dW    = sigma (Q^T dL/da + K^T dL/db) + lam * 2 W (W^T W - I) / ||W^T W - I||_F
    """
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    s = np.asarray(s, np.float64)
    W = np.asarray(W, np.float64)
    hq = relaxed_hash(Q, W, sigma)
    hk = relaxed_hash(K, W, sigma)
    diff = hq - hk
    ids, n_groups = _group_ids(group, hk.shape[0])
    col = _group_sums(hk, ids, n_groups)
    M = W.T @ W - np.eye(W.shape[1])
    fro = float(np.sqrt(np.sum(M * M)))
    loss = (eps * scale_sim * float(np.sum(s * np.sum(diff * diff, axis=1)))
            + eta * scale_bal * float(np.sum(col * col)) + lam * fro)
    d_hq = 2.0 * eps * scale_sim * s[:, None] * diff
    d_hk = -d_hq + 2.0 * eta * scale_bal * col[ids]
    d_a = d_hq * (1.0 - hq * hq) * 0.5
    d_b = d_hk * (1.0 - hk * hk) * 0.5
    grad = sigma * (Q.T @ d_a + K.T @ d_b)
    if fro > 0.0:
        grad = grad + lam * 2.0 * (W @ M) / fro
    return loss, grad


def sgd_step(W, v, grad, lr=LR, momentum=MOMENTUM, weight_decay=WEIGHT_DECAY):
    """One SGD update; returns (W_new, v_new)."""
    g = np.asarray(grad, np.float64) + weight_decay * np.asarray(W, np.float64)
    v_new = momentum * np.asarray(v, np.float64) + g
    return np.asarray(W, np.float64) - lr * v_new, v_new


def make_labels(scores) -> np.ndarray:
    """Similarity labels of m (query, key) pairs from their qk scores."""
    scores = np.asarray(scores, np.float64)
    m = scores.shape[0]
    n_pos = max(1, int(np.floor(0.1 * m)))
    order = np.argsort(-scores, kind="stable")  # descending, earlier pair first on equal scores
    labels = np.full(m, -1.0)
    for rank in range(n_pos):
        labels[order[rank]] = 20.0 if n_pos == 1 else 20.0 - 19.0 * rank / (n_pos - 1)
    return labels


def exact_topk(q, K, n_sel: int) -> np.ndarray:
    """Indices of the n_sel largest q . k_i (earlier key first on equal scores), ascending."""
    sc = np.asarray(K, np.float64) @ np.asarray(q, np.float64)
    order = np.argsort(-sc, kind="stable")[:n_sel]
    return np.sort(order)


def sign_codes(x, W) -> np.ndarray:
    """Alg. 2 without the packing: 1 where the projection is >= 0, else 0."""
    return (np.asarray(x, np.float64) @ np.asarray(W, np.float64) >= 0.0).astype(np.uint8)


def hash_topk(q, K, W, n_sel: int) -> np.ndarray:
    """Indices of the n_sel keys closest to q in Hamming space (lower row on ties), ascending."""
    cq = sign_codes(np.asarray(q)[None, :], W)[0]
    ck = sign_codes(K, W)
    dist = np.sum(ck != cq[None, :], axis=1)
    order = np.argsort(dist, kind="stable")[:n_sel]
    return np.sort(order)


def recall(selected, reference) -> float:
    reference = np.asarray(reference)
    if reference.size == 0:
        return 1.0
    return float(np.intersect1d(selected, reference).size) / float(reference.size)
