"""Pins for the linear-embedding predictor's oracle (Sec. 7.1, "Linear embedding approximation"):
F(t_<i, t) ~ c + A E(t), predicted KV = c + A Ebar with Ebar the expected embedding.  The oracle is
checked against the identity the approximation rests on (for vectors that are exactly linear in the
embedding, c + A Ebar IS the probability-weighted mean of the candidate vectors, which the pinned C
oracle computes), against explicit loops on a case small enough to read, and against the recovery
bound -- never against itself or the device path."""
import numpy as np
import pytest
import torch

from oracle import plc_oracle_linear as OL
from paper_2604_15356_amd.workloads import make_linear_workload


def _np(t):
    return t.contiguous().numpy()


def _ebar(w):
    return OL.expected_embedding(_np(w.probs_full), _np(w.embed_t)).reshape(w.S, w.n, w.m)


def test_explicit_loops_on_a_case_small_enough_to_read():
    rng = np.random.default_rng(0)
    S, L, H, n, d, m, V = 1, 2, 2, 3, 2, 4, 5
    P = rng.dirichlet(np.ones(V), S * n).astype(np.float16)
    Et = rng.integers(-3, 4, (m, V)).astype(np.float16)
    A = rng.integers(-2, 3, (L, H, 2, d, m)).astype(np.float16)
    bk = rng.integers(-2, 3, (S, L, H, n, d)).astype(np.float16)
    bv = rng.integers(-2, 3, (S, L, H, n, d)).astype(np.float16)
    eb = OL.expected_embedding(P, Et)
    for r in range(S * n):
        for j in range(m):
            want = sum(float(P[r, t]) * float(Et[j, t]) for t in range(V))
            assert eb[r, j] == np.float16(want)
    pred = OL.predict(eb.reshape(S, n, m), A, bk, bv)
    for l in range(L):
        for h in range(H):
            for i in range(n):
                for c, bias in ((0, bk), (1, bv)):
                    for e in range(d):
                        want = float(bias[0, l, h, i, e]) + sum(float(A[l, h, c, e, j]) * float(eb[i, j]) for j in range(m))
                        assert abs(pred[0, l, h, i, c, e] - want) < 1e-12


def test_linear_vectors_make_it_the_weighted_mean_of_the_candidates(oracle):
    """If KV is linear in the embedding, c + A Ebar = sum_t P(t) (c + A E(t)): the prediction of Sec. 7.1
    over the whole (small) vocabulary, as the pinned C oracle computes it from candidate vectors.  The two
    agree up to the fp16 rounding of the candidate vectors and of Ebar."""
    rng = np.random.default_rng(4)
    S, L, H, n, d, m, V = 1, 2, 2, 6, 8, 16, 32
    P = rng.dirichlet(np.full(V, 0.3), S * n).astype(np.float16)
    Et = rng.standard_normal((m, V)).astype(np.float16)
    A = (rng.standard_normal((L, H, 2, d, m)) / 4).astype(np.float16)
    bk = rng.standard_normal((S, L, H, n, d)).astype(np.float16)
    bv = rng.standard_normal((S, L, H, n, d)).astype(np.float16)
    pred = OL.predict(OL.expected_embedding(P, Et).reshape(S, n, m), A, bk, bv)           # [S,L,H,n,2,d]
    # candidate t of every position: c + A E(t)
    lin = np.einsum("lhcem,mt->lhcte", A.astype(np.float64), Et.astype(np.float64))          # [L,H,2,V,d]
    cand = [np.empty((S, L, H, n, V, d), dtype=np.float16) for _ in range(2)]
    for c, bias in ((0, bk), (1, bv)):
        cand[c][:] = (bias.astype(np.float64)[:, :, :, :, None, :] + lin[None, :, :, c, None, :, :]).astype(np.float16)
    dm = oracle.make_dims(S, L, H, n, V, d, 0.02)
    zeros = np.zeros((S, L, H, n, d), dtype=np.float16)
    ref = oracle.predict_residual(dm, cand[0], cand[1], P.astype(np.float32).reshape(S, n, V), zeros, zeros,
                                  want_pred=True)["pred"].reshape(S, L, H, n, 2, d)
    scale = P.astype(np.float64).sum(1).reshape(S, 1, 1, n, 1, 1)       # the fp16 row sums to 1 only nearly
    lin_part = pred - np.stack([bk, bv], axis=4).astype(np.float64)
    bias_part = np.stack([bk, bv], axis=4).astype(np.float64)
    assert np.abs(ref - (bias_part + lin_part / scale)).max() < 4e-3
    # a transposed or mis-indexed operand would be off by O(1)
    assert np.abs(ref - pred).max() < 2e-2 and np.abs(pred).max() > 1.0


def test_token_known_and_no_noise_leaves_no_residual():
    w = make_linear_workload("tiny", one_hot=True, overrides=dict(n=128, m=128, V=256))
    r = OL.predict_residual(_ebar(w), _np(w.A), _np(w.bias_k), _np(w.bias_v), _np(w.act_k), _np(w.act_v), w.delta)
    assert (r["symbols"] == 127).all() and r["esc_cnt"].sum() == 0


def test_recovery_error_is_the_quantiser_error():
    w = make_linear_workload("tiny", overrides=dict(n=128))
    eb = _ebar(w)
    r = OL.predict_residual(eb, _np(w.A), _np(w.bias_k), _np(w.bias_v), _np(w.act_k), _np(w.act_v), w.delta)
    ok, ov = OL.reconstruct(eb, _np(w.A), _np(w.bias_k), _np(w.bias_v), r["symbols"], r["esc_vals"], w.delta)
    sym = r["symbols"].reshape(w.S, w.L, w.H, w.n, 2, w.d)
    for c, (out, act) in enumerate(((ok, w.act_k), (ov, w.act_v))):
        a = _np(act).astype(np.float64)
        o = out.astype(np.float64)
        esc = sym[..., c, :] == 255
        ulp = np.maximum(np.abs(o), 2.0 ** -14) * 2.0 ** -10
        assert (np.abs(a - o)[~esc] <= np.float32(w.delta) / 2 + ulp[~esc] / 2 + 1e-9).all()
        assert np.array_equal(out.view(np.uint16)[esc], _np(act).view(np.uint16)[esc])
    assert 0 < r["esc_cnt"].sum() < 0.03 * sym.size
    # as good a predictor as the weighted mean over the whole vocabulary: about the same bits
    c = np.bincount(r["symbols"].ravel(), minlength=256) / sym.size
    assert 6.8 < -(c[c > 0] * np.log2(c[c > 0])).sum() < 7.8
