"""GPU-vs-oracle parity of the learning-to-hash training step (hata_train_step through the C ABI)
against oracle/hash_train_oracle.py (fp64) on the same seeded inputs.

Tolerances (fp32 accumulation of exact bf16 x bf16 products over n rows, partial sums per 128
rows, then a sequential sum over the workgroups; one v_exp_f32 per hash value):
  gradient   max |g - g_ref| <= 2e-5 * max |g_ref|
  loss terms relative 2e-5
  W, v after a step: the gradient bound times lr (plus fp32 rounding of the update itself)
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import hash_train_oracle as T
from paper_2506_02572_amd import synth, train
from tests import harness as H

GRAD_TOL = 2e-5
CASES = [(1000, 128, True), (4096, 256, True), (300, 32, True), (2048, 64, False), (129, 128, False)]


def make_problem(n, r, seed):
    Qb = synth.train_vectors(n, seed=seed, tensor_id=synth.TID_Q)
    Kb = synth.train_vectors(n, seed=seed, tensor_id=synth.TID_K)
    Q = synth.bf16_to_f32(Qb).astype(np.float64)
    K = synth.bf16_to_f32(Kb).astype(np.float64)
    # labels from the qk score of each pair (best tenth positive), as the training data are built
    s = T.make_labels(np.sum(Q * K, axis=1)).astype(np.float32)
    W = synth.fill_f32(seed, synth.TID_WH, (128, r), 1.0 / np.sqrt(128.0))
    return Qb, Kb, Q, K, s, W


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


@pytest.mark.parametrize("n,r,mean_forms", CASES)
def test_train_step_matches_oracle(torch_mod, n, r, mean_forms):
    torch = torch_mod
    print(f"[train] n={n} r={r} mean_forms={mean_forms}", flush=True)
    Qb, Kb, Q, K, s, W = make_problem(n, r, seed=99 + n)
    hp = train.default_hparams(n, mean_forms)
    if not mean_forms:
        hp.lr = 1e-6  # the sums as printed give gradients ~n^2 larger: keep the step finite
    kw = dict(sigma=hp.sigma, eps=hp.eps, eta=hp.eta, lam=hp.lam, scale_sim=hp.scale_sim, scale_bal=hp.scale_bal)
    ctx = train.TrainContext(128, r, max(n, 512))
    Qd, Kd, sd = H.to_dev(Qb), H.to_dev(Kb), H.to_dev(s)
    Wd = H.to_dev(W.copy())
    vd = torch.zeros_like(Wd)
    gd = torch.empty_like(Wd)
    ld = torch.empty(3, dtype=torch.float32, device="cuda")
    Wr, vr = W.astype(np.float64), np.zeros((128, r))
    for step in range(3):
        terms = T.loss_terms(Q, K, s, Wr, **kw)
        _, g_ref = T.loss_and_grad(Q, K, s, Wr, **kw)
        ctx.hata_train_step(Qd, Kd, sd, n, Wd, vd, hp, gd, ld)
        torch.cuda.synchronize()
        g = H.to_host(gd).astype(np.float64)
        gmax = float(np.max(np.abs(g_ref)))
        err = float(np.max(np.abs(g - g_ref)))
        assert err <= GRAD_TOL * gmax, f"step {step}: gradient off by {err:.3e} (max |g| {gmax:.3e})"
        got = H.to_host(ld).astype(np.float64)
        for name, a, b in zip(("similarity", "balance", "uncorrelation"), got, terms):
            assert abs(a - b) <= 2e-5 * max(abs(b), 1e-6 * sum(abs(t) for t in terms)), (step, name, a, b)
        Wr, vr = T.sgd_step(Wr, vr, g_ref, hp.lr, hp.momentum, hp.weight_decay)
        # follow the device weights (fp32) so that the next step compares like with like
        assert np.max(np.abs(H.to_host(Wd) - Wr)) <= hp.lr * GRAD_TOL * gmax * (step + 1) * 2 + 1e-6
        assert np.max(np.abs(H.to_host(vd) - vr)) <= GRAD_TOL * gmax * (step + 1) * 2 + 1e-7
        Wr = H.to_host(Wd).astype(np.float64)
        vr = H.to_host(vd).astype(np.float64)
        print(f"  step {step}: grad err {err:.2e} of {gmax:.2e}; loss {got}", flush=True)
    ctx.close()


def test_per_query_balance_matches_oracle(torch_mod):
    """The balance term summed per query (the final hashing model as printed): blocks of 128
    triplets name their query, in any order; the last block is ragged."""
    torch = torch_mod
    n, r = 11 * train.BLOCK - 40, 128
    Qb, Kb, Q, K, s, W = make_problem(n, r, seed=321)
    blocks = np.array([2, 0, 0, 1, 2, 2, 0, 1, 1, 2, 0], np.int32)  # 3 queries over the 11 blocks
    group = np.repeat(blocks, train.BLOCK)[:n]
    hp = train.default_hparams(n)
    hp.scale_bal = 1.0 / (n * 512)
    kw = dict(sigma=hp.sigma, eps=hp.eps, eta=hp.eta, lam=hp.lam, scale_sim=hp.scale_sim, scale_bal=hp.scale_bal)
    ctx = train.TrainContext(128, r, 2048)
    Wd = H.to_dev(W.copy())
    vd, gd = torch.zeros_like(Wd), torch.empty_like(Wd)
    ld = torch.empty(3, dtype=torch.float32, device="cuda")
    hp.lr = 0.0  # (only the gradient and the loss terms are looked at)
    for blk, grp, n_q in ((H.to_dev(blocks), group, 3), (None, None, 1)):
        terms = T.loss_terms(Q, K, s, W, group=grp, **kw)
        _, g_ref = T.loss_and_grad(Q, K, s, W, group=grp, **kw)
        ctx.hata_train_step(H.to_dev(Qb), H.to_dev(Kb), H.to_dev(s), n, Wd, vd, hp, gd, ld, block_query=blk, n_queries=n_q)
        torch.cuda.synchronize()
        g = H.to_host(gd).astype(np.float64)
        gmax = float(np.max(np.abs(g_ref)))
        assert float(np.max(np.abs(g - g_ref))) <= GRAD_TOL * gmax, n_q
        for name, a, b in zip(("similarity", "balance", "uncorrelation"), H.to_host(ld).astype(np.float64), terms):
            assert abs(a - b) <= 2e-5 * max(abs(b), 1e-6 * sum(abs(t) for t in terms)), (n_q, name, a, b)
    # the two forms really differ on this batch (the test above is not vacuous)
    assert abs(T.loss_terms(Q, K, s, W, group=group, **kw)[1] - T.loss_terms(Q, K, s, W, **kw)[1]) > 1e-3 * T.loss_terms(Q, K, s, W, **kw)[1]
    # more queries than blocks is refused
    from paper_2506_02572_amd import hata
    with pytest.raises(hata.HataError):
        ctx.hata_train_step(H.to_dev(Qb), H.to_dev(Kb), H.to_dev(s), n, Wd, vd, hp, gd, ld, block_query=H.to_dev(blocks), n_queries=12)
    ctx.close()


@pytest.mark.parametrize("m", [1, 7, 10, 300, 4099])
def test_make_labels_matches_oracle(torch_mod, m):
    """hata_train_make_labels (App. B.1 steps 3-4 on the device) against the oracle's make_labels
    fed with exact qk scores; a second case with many exactly tied scores."""
    torch = torch_mod
    ctx = train.TrainContext(128, 128, 4099)
    qb = synth.train_vectors(1, seed=5 + m, tensor_id=synth.TID_Q)[0]
    Kb = synth.train_vectors(m, seed=5 + m, tensor_id=synth.TID_K)
    sd = torch.empty(m, dtype=torch.float32, device="cuda")

    def check(qb, Kb, what):
        q = synth.bf16_to_f32(qb).astype(np.float64)
        K = synth.bf16_to_f32(Kb).astype(np.float64)
        want = T.make_labels(K @ q).astype(np.float32)
        ctx.hata_train_make_labels(H.to_dev(qb), H.to_dev(Kb), m, sd)
        torch.cuda.synchronize()
        assert np.array_equal(H.to_host(sd), want), what
        return want

    check(qb, Kb, "random vectors")
    # small-integer vectors: every score is an exact small integer whatever the summation order, and
    # most scores tie -- the earlier key must win
    rng = np.random.default_rng(m)
    qi = synth.round_to_bf16_bits(rng.integers(-2, 3, 128).astype(np.float32))
    Ki = synth.round_to_bf16_bits(rng.integers(-1, 2, (m, 128)).astype(np.float32))
    want = check(qi, Ki, "tied integer scores")
    if m >= 300:
        sc = synth.bf16_to_f32(Ki).astype(np.float64) @ synth.bf16_to_f32(qi).astype(np.float64)
        assert len(np.unique(sc)) < m // 2 and (want > 0).sum() == m // 10
    ctx.close()


def test_training_raises_the_recall_of_the_hash_topk(torch_mod):
    """The demonstration of Sec. 3.1.2 / App. B on a synthetic head: keys with a few massive,
    query-irrelevant directions (rotated away from the channel axes), where a sign-random-projection
    spends nearly every bit on those directions.  Training data as App. B.1 builds them (sampled
    queries against all keys, labels from hata_train_make_labels), the hyper-parameters of the table
    of App. B.2, 15 epochs x 20 iterations, four queries per batch with the balance term per query;
    the two data terms in their mean forms, the similarity term weighted 30 / n.  The recall of the
    hash top-k against the exact qk top-k (Eq. 2), evaluated by the oracle on HELD-OUT queries, must
    rise by a factor of two at least (measured: 0.06 -> 0.21, where a hash aligned with the
    generator's own basis reaches 0.23); the objective, evaluated by the oracle, must fall."""
    torch = torch_mod
    n_keys, r, k_sel, qpb = 4096, 128, 64, 4
    Kb, Qb = synth.massive_direction_vectors(n_keys, 80, seed=4242)
    K = synth.bf16_to_f32(Kb).astype(np.float64)
    Qf = synth.bf16_to_f32(Qb).astype(np.float64)
    train_q, held_out = list(range(64)), list(range(64, 80))
    W0 = synth.fill_f32(4242, synth.TID_WH, (128, r), 1.0 / np.sqrt(128.0))

    def mean_recall(W):
        return float(np.mean([T.recall(T.hash_topk(Qf[j], K, W, k_sel), T.exact_topk(Qf[j], K, k_sel)) for j in held_out]))

    n = qpb * n_keys
    ctx = train.TrainContext(128, r, n)
    hp = train.default_hparams(n)
    hp.scale_sim = 30.0 / n
    hp.scale_bal = 1.0 / (n * n_keys)
    kw = dict(sigma=hp.sigma, eps=hp.eps, eta=hp.eta, lam=hp.lam, scale_sim=hp.scale_sim, scale_bal=hp.scale_bal)
    Kd, Qd_all = H.to_dev(Kb), H.to_dev(Qb)
    # labels of every training query, built on the device; checked against the oracle for two of them
    labels = torch.empty((len(train_q), n_keys), dtype=torch.float32, device="cuda")
    for j in train_q:
        ctx.hata_train_make_labels(Qd_all[j], Kd, n_keys, labels[j])
    torch.cuda.synchronize()
    for j in (0, 63):
        assert np.array_equal(H.to_host(labels[j]), T.make_labels(K @ Qf[j]).astype(np.float32))
    K_batch = Kd.repeat(qpb, 1).contiguous()
    blocks = torch.arange(qpb, dtype=torch.int32, device="cuda").repeat_interleave(n_keys // train.BLOCK).contiguous()
    group = np.repeat(np.arange(qpb), n_keys)

    def batch(it):
        js = [(it * qpb + i) % len(train_q) for i in range(qpb)]
        Qm = torch.cat([Qd_all[j].expand(n_keys, 128) for j in js]).contiguous()
        return js, Qm, torch.cat([labels[j] for j in js]).contiguous()

    def objective(W):  # on the first batch, by the oracle
        js, _, _ = batch(0)
        Qm = np.concatenate([np.broadcast_to(Qf[j], (n_keys, 128)) for j in js])
        sm = np.concatenate([H.to_host(labels[j]).astype(np.float64) for j in js])
        return float(sum(T.loss_terms(Qm, np.concatenate([K] * qpb), sm, W, group=group, **kw)))

    Wd = H.to_dev(W0.copy())
    vd = torch.zeros_like(Wd)
    for it in range(15 * 20):
        _, Qm, sm = batch(it)
        ctx.hata_train_step(Qm, K_batch, sm, n, Wd, vd, hp, block_query=blocks, n_queries=qpb)
    torch.cuda.synchronize()
    W1 = H.to_host(Wd).astype(np.float64)
    assert np.all(np.isfinite(W1))
    before, after = mean_recall(W0.astype(np.float64)), mean_recall(W1)
    start, end = objective(W0.astype(np.float64)), objective(W1)
    print(f"[train] recall@{k_sel} of the hash top-k against the exact top-k on held-out queries: "
          f"{before:.3f} -> {after:.3f}; objective {start:.3f} -> {end:.3f}", flush=True)
    assert end < start
    assert after >= 2.0 * before and after >= before + 0.08
    ctx.close()


def test_train_validation(torch_mod):
    import ctypes
    from paper_2506_02572_amd import hata
    lib = hata.load_library()
    train._lib()
    n = ctypes.c_size_t(0)
    assert lib.hata_train_workspace_bytes(ctypes.byref(train.hata_train_config(64, 128, 100)), ctypes.byref(n)) == -2
    assert lib.hata_train_workspace_bytes(ctypes.byref(train.hata_train_config(128, 96, 100)), ctypes.byref(n)) == -2
    assert lib.hata_train_workspace_bytes(ctypes.byref(train.hata_train_config(128, 128, 0)), ctypes.byref(n)) == -1
    assert lib.hata_train_step(None, None, None, None, 1, None, 1, None, None, None, None, None, None) == -1
    ctx = train.TrainContext(128, 128, 256)
    with pytest.raises(hata.HataError):
        t = torch_mod.zeros((512, 128), dtype=torch_mod.int16, device="cuda")
        ctx.hata_train_step(t, t, torch_mod.zeros(512, device="cuda"), 512,
                            torch_mod.zeros((128, 128), device="cuda"), torch_mod.zeros((128, 128), device="cuda"),
                            train.default_hparams(512))  # n > n_max
    ctx.close()
