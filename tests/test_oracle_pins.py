"""Pins for the float64 oracle: every check here compares the oracle with
something other than itself -- numbers the paper prints, closed forms,
library routines, invariants, brute force on tiny inputs."""
import math
import os

import numpy as np
import pytest
import scipy.linalg
import scipy.special

from oracle import tpla_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            rows[k] = np.array([float(x) for x in v])
    return rows


def _rand_problem(rng, B=2, H=3, d_c=8, d_r=4, d_n=5, d_v=6, lens=(7, 3)):
    q_nope = rng.standard_normal((B, H, d_n))
    q_pe = rng.standard_normal((B, H, d_r))
    W_UK = rng.standard_normal((H, d_n, d_c))
    W_UV = rng.standard_normal((H, d_c, d_v))
    c = [rng.standard_normal((L, d_c)) for L in lens]
    kpe = [rng.standard_normal((L, d_r)) for L in lens]
    return q_nope, q_pe, W_UK, W_UV, c, kpe


def _rand_orthogonal(rng, d):
    q, r = np.linalg.qr(rng.standard_normal((d, d)))
    return q * np.sign(np.diag(r))


# ---------------------------------------------------------------- Hadamard
def test_hadamard_matches_printed_example():
    gold = _golden("hadamard_worked_example.txt")
    U4 = orc.hadamard_U(4)
    printed = np.stack([gold[f"H4_half_row{i}"] for i in range(4)])
    assert np.array_equal(U4, printed)
    assert np.array_equal(gold["vec_a"] @ U4, gold["vec_a_out"])
    assert np.array_equal(gold["vec_q"] @ U4, gold["vec_q_out"])
    assert np.array_equal(gold["vec_c"] @ U4, gold["vec_c_out"])
    # Sec. 4.3.1 counter-example: the two half sums of Q' * c' cancel although
    # each is large (the printed 200/400 are a factor 10 short of 50*40).
    prod = (gold["vec_q"] @ U4) * (gold["vec_c"] @ U4)
    assert np.array_equal(prod, [2000, 2000, -2000, -2000])
    assert prod[:2].sum() == 4000 and prod[2:].sum() == -4000 and prod.sum() == 0


@pytest.mark.parametrize("d", [1, 2, 4, 8, 64, 512])
def test_hadamard_equals_library_and_is_orthogonal(d):
    Hm = orc.sylvester_hadamard(d)
    assert np.array_equal(Hm, scipy.linalg.hadamard(d).astype(np.float64))
    assert np.array_equal(Hm @ Hm.T, d * np.eye(d))
    U = orc.hadamard_U(d)
    assert np.allclose(U @ U.T, np.eye(d), atol=1e-14)


def test_hadamard_sign_diagonal_side_and_orthogonality():
    rng = np.random.default_rng(0)
    d = 16
    s = rng.choice([-1.0, 1.0], size=d)
    U = orc.hadamard_U(d, s)
    x = rng.standard_normal(d)
    # x U = H-transform of (x * s): the diagonal sits on the left of H
    assert np.allclose(x @ U, (x * s) @ scipy.linalg.hadamard(d) / math.sqrt(d), atol=1e-14)
    assert np.allclose(U @ U.T, np.eye(d), atol=1e-14)
    with pytest.raises(ValueError):
        orc.sylvester_hadamard(12)
    with pytest.raises(ValueError):
        orc.hadamard_U(4, [1, 1, 2, 1])


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_textbook_values_and_prop1():
    out = orc.rms_norm_unit(np.array([3.0, 4.0]), 0.0)
    assert np.allclose(out, np.array([3.0, 4.0]) / math.sqrt(12.5), rtol=1e-15)
    out = orc.rms_norm(np.array([2.0, 0.5]), np.array([3.0, 4.0]), 0.5)
    assert np.allclose(out, np.array([6.0, 2.0]) / math.sqrt(13.0), rtol=1e-15)
    # Proposition 1: RMSNorm(1, c) = RMSNorm(1, c U) U^T for orthogonal U
    rng = np.random.default_rng(1)
    c = rng.standard_normal((5, 16))
    for U in (orc.hadamard_U(16), _rand_orthogonal(rng, 16)):
        assert np.allclose(np.linalg.norm(c @ U, axis=1), np.linalg.norm(c, axis=1), rtol=1e-13)
        assert np.allclose(orc.rms_norm_unit(c @ U, 1e-6) @ U.T, orc.rms_norm_unit(c, 1e-6), atol=1e-13)
    row = orc.mla_cache_rows(np.array([[3.0, 4.0]]), np.array([[7.0]]), 0.0)
    assert np.allclose(row, [[3 / math.sqrt(12.5), 4 / math.sqrt(12.5), 7.0]])


def test_sliced_rmsnorm_append():
    gold = _golden("hadamard_worked_example.txt")
    # Sec. 4.3.1: (100,0,0,0) H_4/2 = (50,50,50,50): both halves carry half the energy, so the
    # sliced norm with alpha = 2 is the global one; RMS = 50, every normalised entry is 1
    x = gold["vec_a"] @ orc.hadamard_U(4)
    rows = orc.sliced_rms_rows(x, np.array([7.0]), 2, [2.0, 2.0], 0.0)
    assert np.array_equal(rows[0], [1.0, 1.0, 7.0]) and np.array_equal(rows[1], [1.0, 1.0, 7.0])
    # closed form with unequal halves: x = (3,4 | 0,5), alpha = (2, 2), eps = 0.5
    rows = orc.sliced_rms_rows(np.array([3.0, 4.0, 0.0, 5.0]), np.zeros(0), 2, None, 0.5)
    assert np.allclose(rows[0], np.array([3.0, 4.0]) / math.sqrt(2 * 25 / 4 + 0.5), rtol=1e-15)
    assert np.allclose(rows[1], np.array([0.0, 5.0]) / math.sqrt(2 * 25 / 4 + 0.5), rtol=1e-15)
    # eps is added to the estimated global mean square, not to the slice's own
    rows = orc.sliced_rms_rows(np.array([3.0, 4.0, 0.0, 5.0]), np.zeros(0), 2, [1.5, 3.0], 0.5)
    assert np.allclose(rows[0], np.array([3.0, 4.0]) / math.sqrt(1.5 * 25 / 4 + 0.5), rtol=1e-15)
    assert np.allclose(rows[1], np.array([0.0, 5.0]) / math.sqrt(3.0 * 25 / 4 + 0.5), rtol=1e-15)
    # equal-energy slices + alpha_i = g  ==  global RMSNorm (Condition 1 met exactly), any g
    rng = np.random.default_rng(13)
    for g in (2, 4):
        c = rng.standard_normal((6, 32))
        dl = 32 // g
        e = np.sum(c[:, :dl] ** 2, axis=1, keepdims=True)
        for i in range(1, g):
            sl = c[:, i * dl:(i + 1) * dl]
            sl *= np.sqrt(e / np.sum(sl ** 2, axis=1, keepdims=True))
        rows = orc.sliced_rms_rows(c, np.zeros((6, 0)), g, None, 1e-6)
        assert np.allclose(np.concatenate(rows, axis=1), orc.rms_norm_unit(c, 1e-6), rtol=1e-13)
    # alpha as the reciprocal variance share (PCA reading): exact for a vector whose energy
    # splits exactly in those shares
    c = np.array([[2.0, 2.0, 1.0, 1.0]])            # |x_0|^2 = 8, |x_1|^2 = 2 -> shares 0.8 / 0.2
    rows = orc.sliced_rms_rows(c, np.zeros((1, 0)), 2, [1 / 0.8, 1 / 0.2], 0.0)
    assert np.allclose(np.concatenate(rows, axis=1), orc.rms_norm_unit(c, 0.0), rtol=1e-14)
    # scale invariance at eps = 0, and the k_pe part is passed through untouched
    c = rng.standard_normal((3, 8)); k = rng.standard_normal((3, 2))
    r1 = orc.sliced_rms_rows(c, k, 2, [1.7, 2.4], 0.0); r2 = orc.sliced_rms_rows(5 * c, k, 2, [1.7, 2.4], 0.0)
    assert np.allclose(r1[0], r2[0], rtol=1e-14) and np.array_equal(r1[1][:, 4:], k)
    with pytest.raises(ValueError):
        orc.sliced_rms_rows(np.zeros(6), np.zeros(0), 4, None, 0.0)


# ---------------------------------------------------------------- softmax
def test_shard_attention_against_library_softmax():
    rng = np.random.default_rng(2)
    B, H, dl, dr, L = 2, 3, 6, 4, 11
    Q = rng.standard_normal((B, H, dl))
    qpe = rng.standard_normal((B, H, dr))
    c = [rng.standard_normal((L, dl)) for _ in range(B)]
    k = [rng.standard_normal((L, dr)) for _ in range(B)]
    scale = 0.37
    O, lse = orc.shard_attention(Q, qpe, c, k, scale)
    for b in range(B):
        s = scale * (np.einsum("hd,td->ht", Q[b], c[b]) + np.einsum("hr,tr->ht", qpe[b], k[b]))
        assert np.allclose(O[b], scipy.special.softmax(s, axis=1) @ c[b], rtol=1e-12, atol=1e-14)
        assert np.allclose(lse[b], scipy.special.logsumexp(s, axis=1), rtol=1e-13)


def test_two_token_closed_form():
    # one head, g = 2 slices of width 1, two cached tokens: each shard's
    # softmax is a logistic function of the score difference.
    a, b_, p = 0.7, -1.3, 0.4
    rows = np.array([[1.0, 2.0], [3.0, -1.0]])
    kpe = np.array([[0.5], [-0.25]])
    W_UK = np.array([[[1.0, 0.0], [0.0, 1.0]]])           # Q = q_nope
    W_UV = np.array([[[2.0, -1.0, 0.5], [0.25, 4.0, -3.0]]])
    scale = 0.9
    res = orc.tpla_decode(np.array([[[a, b_]]]), np.array([[[p]]]), W_UK, W_UV, [rows], [kpe], 2, scale)
    s00 = scale * (a * 1.0 + p * 0.5)
    s01 = scale * (a * 3.0 + p * -0.25)
    w0 = 1.0 / (1.0 + math.exp(s01 - s00))                # weight of token 0 on shard 0
    O0 = w0 * 1.0 + (1 - w0) * 3.0
    s10 = scale * (b_ * 2.0 + p * 0.5)
    s11 = scale * (b_ * -1.0 + p * -0.25)
    w1 = 1.0 / (1.0 + math.exp(s11 - s10))
    O1 = w1 * 2.0 + (1 - w1) * -1.0
    assert np.allclose(res["O_lat"][:, 0, 0, 0], [O0, O1], rtol=1e-14)
    assert np.allclose(res["o"][0, 0], O0 * W_UV[0, 0] + O1 * W_UV[0, 1], rtol=1e-14)
    assert np.allclose(res["lse"][:, 0, 0], [s00 + math.log1p(math.exp(s01 - s00)),
                                             s10 + math.log1p(math.exp(s11 - s10))], rtol=1e-14)


def test_softmax_invariants():
    rng = np.random.default_rng(3)
    q_nope, q_pe, W_UK, W_UV, c, kpe = _rand_problem(rng, lens=(9, 1))
    # a latent column equal to 1 everywhere comes back as 1 (weights sum to 1)
    for cb in c:
        cb[:, 3] = 1.0
    res = orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, 2, 0.3)
    assert np.allclose(res["O_lat"][0][:, :, 3], 1.0, rtol=1e-14)
    # outputs lie in the convex hull of the rows (column-wise bounds)
    for i in range(2):
        for b, cb in enumerate(c):
            sl = cb[:, i * 4:(i + 1) * 4]
            assert np.all(res["O_lat"][i, b] <= sl.max(axis=0) + 1e-12)
            assert np.all(res["O_lat"][i, b] >= sl.min(axis=0) - 1e-12)
    # L = 1: the output is that row, lse is its score
    assert np.allclose(res["O_lat"][1, 1], np.broadcast_to(c[1][0, 4:], (3, 4)), rtol=1e-14)
    # shifting every score of a head by a constant (k_pe += v with q_pe . v = const)
    # changes lse by that constant and nothing else
    Q_i = rng.standard_normal((1, 2, 4)); qp = rng.standard_normal((1, 2, 3))
    ci = [rng.standard_normal((6, 4))]; ki = [rng.standard_normal((6, 3))]
    O1, l1 = orc.shard_attention(Q_i, qp, ci, ki, 1.0)
    v = np.linalg.lstsq(qp[0], np.array([2.5, 2.5]), rcond=None)[0]
    O2, l2 = orc.shard_attention(Q_i, qp, ci, [ki[0] + v], 1.0)
    assert np.allclose(O1, O2, rtol=1e-12) and np.allclose(l2 - l1, 2.5, rtol=1e-12)
    # zero queries: uniform weights -> mean of rows, lse = log L
    O3, l3 = orc.shard_attention(np.zeros((1, 2, 4)), np.zeros((1, 2, 3)), ci, ki, 1.0)
    assert np.allclose(O3[0], np.broadcast_to(ci[0].mean(axis=0), (2, 4)), rtol=1e-14)
    assert np.allclose(l3, math.log(6), rtol=1e-15)
    # empty sequence
    O4, l4 = orc.shard_attention(Q_i, qp, [np.zeros((0, 4))], [np.zeros((0, 3))], 1.0)
    assert np.all(O4 == 0) and np.all(np.isneginf(l4))


# ------------------------------------------------------ absorption / MLA
def test_absorbed_equals_naive_equals_bruteforce():
    rng = np.random.default_rng(4)
    q_nope, q_pe, W_UK, W_UV, c, kpe = _rand_problem(rng)
    scale = 1.0 / math.sqrt(5 + 4)
    o_abs = orc.mla_absorbed(q_nope, q_pe, W_UK, W_UV, c, kpe, scale)
    o_nai = orc.mla_naive(q_nope, q_pe, W_UK, W_UV, c, kpe, scale)
    o_bf = orc.tpla_bruteforce(q_nope, q_pe, W_UK, W_UV, c, kpe, 1, scale)
    assert np.allclose(o_abs, o_nai, rtol=1e-12, atol=1e-13)
    assert np.allclose(o_abs, o_bf, rtol=1e-12, atol=1e-13)


def test_absorb_query_definition():
    rng = np.random.default_rng(5)
    q = rng.standard_normal((2, 3, 5)); W = rng.standard_normal((3, 5, 8))
    Q = orc.absorb_query(q, W, 2, mu=[2.0, 0.5])
    for b in range(2):
        for h in range(3):
            full = W[h].T @ q[b, h]                      # k_h = W_UK[h] c  =>  q.k = (W^T q).c
            assert np.allclose(Q[0, b, h], 2.0 * full[:4], rtol=1e-13)
            assert np.allclose(Q[1, b, h], 0.5 * full[4:], rtol=1e-13)
    with pytest.raises(ValueError):
        orc.absorb_query(q, W, 3)


@pytest.mark.parametrize("g", [2, 4])
def test_tpla_equals_bruteforce_with_U_and_mu(g):
    rng = np.random.default_rng(6)
    q_nope, q_pe, W_UK, W_UV, c, kpe = _rand_problem(rng, lens=(5, 2))
    U = orc.hadamard_U(8, rng.choice([-1.0, 1.0], size=8))
    mu = rng.uniform(0.5, 2.0, size=g)
    res = orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, g, 0.41, U=U, mu=mu)
    bf = orc.tpla_bruteforce(q_nope, q_pe, W_UK, W_UV, c, kpe, g, 0.41, U=U.tolist(), mu=mu.tolist())
    assert np.allclose(res["o"], bf, rtol=1e-11, atol=1e-12)
    # a non-symmetric orthogonal U catches a transposed operand
    U2 = _rand_orthogonal(rng, 8)
    res2 = orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, g, 0.41, U=U2, mu=mu)
    bf2 = orc.tpla_bruteforce(q_nope, q_pe, W_UK, W_UV, c, kpe, g, 0.41, U=U2.tolist(), mu=mu.tolist())
    assert np.allclose(res2["o"], bf2, rtol=1e-11, atol=1e-12)


# --------------------------------------------------- TPLA facts of the paper
def test_tpla_g1_is_mla_and_U_is_a_noop_at_g1():
    rng = np.random.default_rng(7)
    q_nope, q_pe, W_UK, W_UV, c, kpe = _rand_problem(rng, d_c=16, lens=(12, 4))
    scale = 0.25
    ref = orc.mla_naive(q_nope, q_pe, W_UK, W_UV, c, kpe, scale)
    assert np.allclose(orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, 1, scale)["o"], ref, rtol=1e-12)
    for U in (orc.hadamard_U(16), orc.hadamard_U(16, rng.choice([-1.0, 1.0], size=16)), _rand_orthogonal(rng, 16)):
        got = orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, 1, scale, U=U)["o"]
        assert np.allclose(got, ref, rtol=1e-11, atol=1e-12)
    # the norm weight folds into the up-projections (Sec. 4.1)
    gamma = rng.uniform(0.5, 1.5, size=16)
    got = orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, 1, scale, gamma=gamma)["o"]
    ref_g = orc.mla_naive(q_nope, q_pe, W_UK, W_UV, [x * gamma for x in c], kpe, scale)
    assert np.allclose(got, ref_g, rtol=1e-11, atol=1e-12)


def test_tpla_differs_from_mla_in_general_but_matches_in_exact_cases():
    rng = np.random.default_rng(8)
    q_nope, q_pe, W_UK, W_UV, c, kpe = _rand_problem(rng, d_c=8, lens=(10, 6))
    scale = 0.5
    mla = orc.mla_naive(q_nope, q_pe, W_UK, W_UV, c, kpe, scale)
    tp = orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, 2, scale)["o"]
    assert np.max(np.abs(tp - mla)) > 1e-3           # per-shard softmaxes differ (Sec. 4.2)
    # (i) q_nope = 0: every shard sees the RoPE-only scores
    z = np.zeros_like(q_nope)
    assert np.allclose(orc.tpla_decode(z, q_pe, W_UK, W_UV, c, kpe, 2, scale)["o"],
                       orc.mla_naive(z, q_pe, W_UK, W_UV, c, kpe, scale), rtol=1e-12, atol=1e-13)
    # (iv) replicated halves with mu_i = g: per-shard scores equal the global ones
    half_c = [rng.standard_normal((L, 4)) for L in (10, 6)]
    c_rep = [np.concatenate([x, x], axis=1) for x in half_c]
    W_half = rng.standard_normal((3, 5, 4))
    W_rep = np.concatenate([W_half, W_half], axis=2)
    got = orc.tpla_decode(q_nope, q_pe, W_rep, W_UV, c_rep, kpe, 2, scale, mu=[2.0, 2.0])["o"]
    assert np.allclose(got, orc.mla_naive(q_nope, q_pe, W_rep, W_UV, c_rep, kpe, scale), rtol=1e-12, atol=1e-13)
    # (v) query supported on slice 0 and the other slice of the cache zero
    W0 = W_UK.copy(); W0[:, :, 4:] = 0.0
    c0 = [x.copy() for x in c]
    for x in c0:
        x[:, 4:] = 0.0
    got = orc.tpla_decode(q_nope, q_pe, W0, W_UV, c0, kpe, 2, scale)["o"]
    assert np.allclose(got, orc.mla_naive(q_nope, q_pe, W0, W_UV, c0, kpe, scale), rtol=1e-12, atol=1e-13)


def test_row_parallel_identity_for_combine():
    rng = np.random.default_rng(9)
    O = rng.standard_normal((4, 2, 3, 5))             # g=4 slices of width 5
    W = rng.standard_normal((3, 20, 7))
    cat = np.concatenate(list(O), axis=-1)            # [B,H,20]
    ref = np.stack([cat[:, h] @ W[h] for h in range(3)], axis=1)
    assert np.allclose(orc.combine_shards(O, W), ref, rtol=1e-13)


def test_output_projection_is_head_major_and_row_parallel():
    rng = np.random.default_rng(14)
    o = rng.standard_normal((3, 4, 5)); W = rng.standard_normal((20, 7))
    ref = np.zeros((3, 7))
    for b in range(3):
        for h in range(4):
            for v in range(5):
                ref[b] += o[b, h, v] * W[h * 5 + v]
    assert np.allclose(orc.output_projection(o, W), ref, rtol=1e-13)
    # row-parallel over head groups (Sec. 4.2): X A = X_1 A_1 + X_2 A_2
    parts = orc.output_projection(o[:, :2], W[:10]) + orc.output_projection(o[:, 2:], W[10:])
    assert np.allclose(parts, ref, rtol=1e-13)
    # absorbing W_UV into W_O (Sec. 3.3) gives the same block output
    q_nope, q_pe, W_UK, W_UV, c, kpe = _rand_problem(rng, H=4, d_v=5, lens=(6, 3))
    res = orc.tpla_decode(q_nope, q_pe, W_UK, W_UV, c, kpe, 1, 0.3)
    W_VO = np.concatenate([W_UV[h] @ W[h * 5:(h + 1) * 5] for h in range(4)], axis=0)      # [H d_c, D]
    direct = res["O_lat"][0].reshape(2, -1) @ W_VO
    assert np.allclose(orc.output_projection(res["o"], W), direct, rtol=1e-12)


def test_reparameterize_weights_layouts():
    rng = np.random.default_rng(10)
    W_UK = rng.standard_normal((2, 3, 4)); W_UV = rng.standard_normal((2, 4, 5))
    U = _rand_orthogonal(rng, 4); gamma = rng.uniform(0.5, 2, 4)
    Wk, Wv = orc.reparameterize_weights(W_UK, W_UV, U, gamma)
    for h in range(2):
        # paper layout: W^UK is [d_c, d_n] = W_UK[h].T ; W_new = U^T W_gamma W
        assert np.allclose(Wk[h].T, U.T @ np.diag(gamma) @ W_UK[h].T, rtol=1e-13)
        assert np.allclose(Wv[h], U.T @ np.diag(gamma) @ W_UV[h], rtol=1e-13)


# ------------------------------------------------------------------- PCA
def test_pca_closed_form_on_diagonal_covariance():
    rng = np.random.default_rng(11)
    lam = np.array([9.0, 4.0, 1.0, 0.25])
    R = _rand_orthogonal(rng, 4)
    n = 200000
    F = (rng.standard_normal((n, 4)) * np.sqrt(lam)) @ R.T
    U, ev = orc.pca_U(F)
    assert np.allclose(ev, lam, rtol=2e-2)
    assert np.allclose(np.abs(U.T @ R), np.eye(4), atol=2e-2)      # columns = +-R columns, sorted
    fr = orc.variance_fractions(lam, 2)
    assert np.allclose(fr, [13.0 / 14.25, 1.25 / 14.25])
    assert np.allclose(orc.default_mu(2, lam), [14.25 / 13.0, 14.25 / 1.25])
    assert np.allclose(orc.default_mu(4), 4.0)


# --------------------------------------------------------------- storage
def test_bf16_rounding_and_paging_helpers():
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: ties go to the even mantissa
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -3.0, 0.0, 1e-3])
    r = orc.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 + 2.0 ** -6 and r[2] == 1.0 + 2.0 ** -7 and r[3] == -3.0 and r[4] == 0.0
    # every rounded value is representable: its float32 bit pattern has 16 zero low bits
    bits = r.astype(np.float32).view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0)
    assert np.array_equal(orc.bf16_bits_to_f64((bits >> 16).astype(np.uint16)), r)
    rng = np.random.default_rng(12)
    y = rng.standard_normal(1000) * 10
    ry = orc.round_to_bf16(y)
    assert np.all(np.abs(ry - y) <= np.abs(y) * 2.0 ** -8)
    pool = np.arange(5 * 4 * 2).reshape(5, 4, 2)
    got = orc.paged_rows(pool, [3, 0, 4], 9)
    ref = np.concatenate([pool[3], pool[0], pool[4][:1]])
    assert np.array_equal(got, ref)


def test_latent_moments_give_the_library_covariance():
    # pinned to numpy's own covariance routine (biased, rows = observations) and to a hand-countable case
    rng = np.random.default_rng(12)
    F = rng.standard_normal((300, 5)) * np.array([3.0, 1.0, 0.5, 2.0, 0.1]) + np.array([0.5, -1.0, 0.0, 2.0, 0.3])
    s, G = orc.latent_moments(F)
    n = F.shape[0]
    assert np.allclose(G / n - np.outer(s / n, s / n), np.cov(F, rowvar=False, bias=True), rtol=1e-12, atol=1e-12)
    s2, G2 = orc.latent_moments(np.array([[1.0, 2.0], [3.0, -1.0]]))
    assert np.array_equal(s2, [4.0, 1.0]) and np.array_equal(G2, [[10.0, -1.0], [-1.0, 5.0]])
    # and pca_U is the eigen-decomposition of exactly that covariance
    U, ev = orc.pca_U(F)
    assert np.allclose(U @ np.diag(ev) @ U.T, G / n - np.outer(s / n, s / n), atol=1e-12)


# ------------------------------------------------------------------- prefill
def test_prefill_is_token_by_token_decode_over_each_sequence_prefix():
    """Causal prefill of packed sequences = for every token, MLA decode (pinned above
    against brute force) whose cache is that sequence's prefix up to and including the token."""
    rng = np.random.default_rng(21)
    H, d_n, d_r, d_c, d_v = 2, 3, 2, 4, 3
    lens = [5, 1, 0, 6]
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    q_nope, q_pe = rng.standard_normal((T, H, d_n)), rng.standard_normal((T, H, d_r))
    W_UK, W_UV = rng.standard_normal((H, d_n, d_c)), rng.standard_normal((H, d_c, d_v))
    c, kpe = rng.standard_normal((T, d_c)), rng.standard_normal((T, d_r))
    scale = 0.37
    o = orc.mla_prefill(q_nope, q_pe, W_UK, W_UV, c, kpe, cu, scale)
    assert o.shape == (T, H, d_v)
    for b, L in enumerate(lens):
        for i in range(L):
            t = cu[b] + i
            ref = orc.mla_naive(q_nope[t:t + 1], q_pe[t:t + 1], W_UK, W_UV, [c[cu[b]:t + 1]], [kpe[cu[b]:t + 1]], scale)
            assert np.allclose(o[t], ref[0], rtol=1e-12, atol=1e-13), (b, i)
        if L:
            # the first token sees only itself: its output is its own value vector
            assert np.allclose(o[cu[b]], np.einsum("c,hcv->hv", c[cu[b]], W_UV), rtol=1e-12, atol=1e-13)
    # scalar-loop check of one entry (second sequence-of-5 token 3, head 1)
    t, h, t0 = 3, 1, 0
    sc = [scale * (sum(q_nope[t, h, n] * sum(W_UK[h, n, a] * c[s_, a] for a in range(d_c)) for n in range(d_n))
                   + sum(q_pe[t, h, r] * kpe[s_, r] for r in range(d_r))) for s_ in range(t0, t + 1)]
    w = np.exp(np.array(sc) - max(sc)); w /= w.sum()
    ref = [sum(w[j] * sum(c[t0 + j, a] * W_UV[h, a, v] for a in range(d_c)) for j in range(len(sc))) for v in range(d_v)]
    assert np.allclose(o[t, h], ref, rtol=1e-12, atol=1e-13)
    # a change in a later token or in another sequence never reaches an earlier output
    c2 = c.copy(); c2[4] += 1.0; c2[7] -= 2.0
    o2 = orc.mla_prefill(q_nope, q_pe, W_UK, W_UV, c2, kpe, cu, scale)
    assert np.array_equal(o2[:4], o[:4]) and np.array_equal(o2[5:7], o[5:7])
