"""Float64 CPU oracle for tensor-parallel latent attention (TPLA) decode.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  This module is a plain, slow,
obviously-correct numpy implementation of what the GPU library computes.  It
shares no code with the HIP path (no common helpers, tables or constants) and
must only be imported by tests, the smoke check and the benchmark's
CPU-baseline leg.  Everything is float64, dense and un-paged: full softmax
(no online/split form), dense orthogonal matrix U (no fast transform).

Notation follows the paper (arXiv 2508.15881):
  d_c  latent width (4*d_h)            d_r  RoPE key/query width
  d_n  per-head no-RoPE query width    d_v  per-head value width
  H    query heads                     g    number of latent slices
  U    orthogonal d_c x d_c matrix     mu   per-slice score factor (Cond. 2)
Weight layouts (per head):  W_UK[h] is [d_n, d_c]  so that k_h = W_UK[h] @ c,
                            W_UV[h] is [d_c, d_v]  so that v_h = c @ W_UV[h].

Parity status: every function below is pinned by tests/test_oracle_pins.py
against facts the paper or the mathematics fix, except
  * default_mu(): the paper is inconsistent about the value of the Condition 2
    factors (Sec. 4.2 vs Sec. 4.3.2) -- "parity unpinned"; mu is an input
    everywhere else, so the choice never enters a parity comparison.
"""
import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# Orthogonal reparameterisation (Sec. 4.1, Sec. 4.3)
# --------------------------------------------------------------------------
def sylvester_hadamard(d):
    """Unnormalised Walsh-Hadamard matrix H_d by the recursion of Sec. 4.3.1:
    H_1 = (1), H_2n = [[H_n, H_n], [H_n, -H_n]] (natural / Sylvester order)."""
    if d < 1 or (d & (d - 1)) != 0:
        raise ValueError("Hadamard size must be a power of two")
    Hm = np.ones((1, 1), dtype=F64)
    while Hm.shape[0] < d:
        Hm = np.block([[Hm, Hm], [Hm, -Hm]])
    return Hm


def hadamard_U(d, signs=None):
    """Orthonormal U = diag(s) @ H_d / sqrt(d)  (Sec. 4.3.1: H_d H_d^T = d I,
    so 1/sqrt(d) makes it orthonormal; the random +-1 diagonal multiplies H_d.
    The paper does not say on which side; this oracle puts it on the left, so
    x U = H-transform of (x * s))."""
    Hm = sylvester_hadamard(d)
    if signs is None:
        signs = np.ones(d, dtype=F64)
    signs = np.asarray(signs, dtype=F64)
    if signs.shape != (d,) or not np.all(np.abs(signs) == 1.0):
        raise ValueError("signs must be d values of +-1")
    return (signs[:, None] * Hm) / np.sqrt(F64(d))


def pca_U(F):
    """PCA basis of calibration latents F [n, d] (Sec. 4.3.2): eigenvectors of
    the covariance matrix, columns sorted by descending eigenvalue.
    Returns (U, eigenvalues)."""
    F = np.asarray(F, dtype=F64)
    Fc = F - F.mean(axis=0, keepdims=True)
    cov = (Fc.T @ Fc) / F64(F.shape[0])
    lam, vec = np.linalg.eigh(cov)
    order = np.argsort(-lam, kind="stable")
    return vec[:, order], lam[order]


def latent_moments(F):
    """First and second raw moments of calibration latents F [n, d] (Sec. 4.3.2,
    the ingredients of the covariance): (sum_r F_r, sum_r F_r^T F_r)."""
    F = np.asarray(F, dtype=F64)
    return F.sum(axis=0), F.T @ F


def variance_fractions(eigenvalues, g=2):
    """alpha, beta, ... of Sec. 4.3.2 as printed: the fraction of total
    variance captured by each contiguous slice of d/g principal components."""
    lam = np.asarray(eigenvalues, dtype=F64)
    parts = lam.reshape(g, -1).sum(axis=1)
    return parts / lam.sum()


def default_mu(g, eigenvalues=None):
    """Per-slice score factors of Condition 2 -- parity unpinned (see header).
    Balanced slices (identity / Hadamard): mu_i = g, the analogue of alpha = 2
    in Sec. 4.3.1.  PCA: the reciprocal of the variance fraction, which is the
    reading consistent with Condition 1 (alpha * ||slice||^2 ~ ||c||^2)."""
    if eigenvalues is None:
        return np.full(g, F64(g))
    return 1.0 / variance_fractions(eigenvalues, g)


def rms_norm_unit(c, eps):
    """RMSNorm(1, c) over the last axis (Sec. 4.1): c / sqrt(mean(c^2) + eps)."""
    c = np.asarray(c, dtype=F64)
    rms = np.sqrt(np.mean(c * c, axis=-1, keepdims=True) + F64(eps))
    return c / rms


def rms_norm(gamma, c, eps):
    """RMSNorm(gamma, c) = RMSNorm(1, c) * gamma (Sec. 4.1)."""
    return rms_norm_unit(c, eps) * np.asarray(gamma, dtype=F64)


def reparameterize_weights(W_UK, W_UV, U, gamma=None):
    """W_new = U^T W_gamma W for both up-projections (Sec. 4.1).  In the
    per-head layouts used here that is W_UK'[h] = W_UK[h] @ W_gamma @ U and
    W_UV'[h] = U^T @ W_gamma @ W_UV[h]."""
    W_UK = np.asarray(W_UK, dtype=F64)
    W_UV = np.asarray(W_UV, dtype=F64)
    U = np.asarray(U, dtype=F64)
    if gamma is not None:
        gamma = np.asarray(gamma, dtype=F64)
        W_UK = W_UK * gamma[None, None, :]
        W_UV = W_UV * gamma[None, :, None]
    W_UK_t = np.einsum("hnc,ck->hnk", W_UK, U)
    W_UV_t = np.einsum("ck,hcv->hkv", U, W_UV)
    return W_UK_t, W_UV_t


def transform_latent(c, U):
    """Cache rows in the U basis: c' = c @ U (Sec. 4.1, W_DKV_new = W_DKV U)."""
    return np.asarray(c, dtype=F64) @ np.asarray(U, dtype=F64)


def mla_cache_rows(c_raw, k_pe, eps):
    """One MLA cache row per token: [RMSNorm(1, c) || k_pe] (Sec. 3.3 with the
    norm weight absorbed into the up-projections, Sec. 4.1)."""
    return np.concatenate([rms_norm_unit(c_raw, eps), np.asarray(k_pe, dtype=F64)], axis=-1)


def sliced_rms_rows(c_t, k_pe, g, alpha, eps):
    """Cache rows of a decode token when every device normalises its own
    latent slice (Sec. 4.1, RMSNorm slicing condition): with x_i the i-th of g
    contiguous slices of c_t (already in the U basis), the global mean square
    |c|^2 / d is replaced by alpha_i |x_i|^2 / d, so
        row_i = [ x_i / sqrt(alpha_i |x_i|^2 / d + eps)  ||  k_pe ].
    Returns a list of g arrays [..., d/g + d_r].  (The paper's last step also
    writes this as sqrt(alpha/2) RMS(x_0); the two differ only in how eps is
    scaled -- this oracle keeps eps unscaled, as in the line before it.)"""
    c_t = np.asarray(c_t, dtype=F64)
    k_pe = np.asarray(k_pe, dtype=F64)
    d = c_t.shape[-1]
    if d % g:
        raise ValueError("d_c must be divisible by g")
    alpha = np.full(g, F64(g)) if alpha is None else np.asarray(alpha, dtype=F64)
    dl = d // g
    rows = []
    for i in range(g):
        x = c_t[..., i * dl:(i + 1) * dl]
        ms = alpha[i] * np.sum(x * x, axis=-1, keepdims=True) / F64(d) + F64(eps)
        rows.append(np.concatenate([x / np.sqrt(ms), k_pe], axis=-1))
    return rows


# --------------------------------------------------------------------------
# Softmax helpers
# --------------------------------------------------------------------------
def _softmax_lse(s):
    """Max-subtracted softmax over the last axis and its log-sum-exp."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    z = np.sum(e, axis=-1, keepdims=True)
    return e / z, (m + np.log(z))[..., 0]


# --------------------------------------------------------------------------
# TPLA decode (Sec. 4, eq. "tpla_softmax_one_device"; Sec. 4.2 for k_pe / mu)
# --------------------------------------------------------------------------
def absorb_query(q_nope, W_UK_t, g, mu=None):
    """Absorbed query Q[b,h,:] = q_nope[b,h,:] @ W_UK'[h] (Sec. 3.3), cut into
    g contiguous slices of the latent axis (Sec. 4) with slice i scaled by
    mu_i (Condition 2, Sec. 4.2).  Returns [g, B, H, d_c/g]."""
    q_nope = np.asarray(q_nope, dtype=F64)
    W_UK_t = np.asarray(W_UK_t, dtype=F64)
    Q = np.einsum("bhn,hnc->bhc", q_nope, W_UK_t)
    B, Hh, d_c = Q.shape
    if d_c % g:
        raise ValueError("d_c must be divisible by g")
    mu = np.ones(g, dtype=F64) if mu is None else np.asarray(mu, dtype=F64)
    Qs = Q.reshape(B, Hh, g, d_c // g).transpose(2, 0, 1, 3)
    return Qs * mu[:, None, None, None]


def shard_attention(Q_i, q_pe, c_i, k_pe, scale):
    """One device's attention over its latent slice (Sec. 4):
        s[h,t] = scale * (Q_i[h] . c_i[t] + q_pe[h] . k_pe[t])     (k_pe replicated, Sec. 4.2)
        O_i[h] = sum_t softmax_t(s[h,:])[t] * c_i[t]
    for every sequence b.  c_i, k_pe: lists (one per sequence) of [L_b, d_c/g]
    and [L_b, d_r].  Returns O_i [B,H,d_c/g] and lse_i [B,H].  A sequence with
    L_b = 0 yields O = 0 and lse = -inf."""
    Q_i = np.asarray(Q_i, dtype=F64)
    q_pe = np.asarray(q_pe, dtype=F64)
    B, Hh, dl = Q_i.shape
    O = np.zeros((B, Hh, dl), dtype=F64)
    lse = np.full((B, Hh), -np.inf, dtype=F64)
    for b in range(B):
        cb = np.asarray(c_i[b], dtype=F64)
        kb = np.asarray(k_pe[b], dtype=F64)
        if cb.shape[0] == 0:
            continue
        s = F64(scale) * (Q_i[b] @ cb.T + q_pe[b] @ kb.T)      # [H, L_b]
        p, lse[b] = _softmax_lse(s)
        O[b] = p @ cb
    return O, lse


def combine_shards(O_lat, W_UV_t):
    """Sum over slices of the per-slice value up-projection (the all-reduce of
    Sec. 4 with W_UV kept separate from W_O, Sec. 3.3):
        o[b,h,:] = sum_i O_lat[i,b,h,:] @ W_UV'[h, S_i, :]."""
    O_lat = np.asarray(O_lat, dtype=F64)
    W_UV_t = np.asarray(W_UV_t, dtype=F64)
    g, B, Hh, dl = O_lat.shape
    o = np.zeros((B, Hh, W_UV_t.shape[2]), dtype=F64)
    for i in range(g):
        o += np.einsum("bhc,hcv->bhv", O_lat[i], W_UV_t[:, i * dl:(i + 1) * dl, :])
    return o


def output_projection(o, W_O):
    """O~ = O W^O (Sec. 3.3): the per-head outputs o [B, H, d_v], flattened
    head-major to [B, H d_v], times W_O [H d_v, D]."""
    o = np.asarray(o, dtype=F64)
    return o.reshape(o.shape[0], -1) @ np.asarray(W_O, dtype=F64)


def tpla_decode(q_nope, q_pe, W_UK, W_UV, c_list, kpe_list, g, scale, U=None, mu=None, gamma=None):
    """Whole TPLA decode step for one layer on cached latents c_list[b]
    ([L_b, d_c], already normalised) and RoPE keys kpe_list[b] ([L_b, d_r]).
    Returns a dict with every intermediate the GPU path exposes."""
    W_UK = np.asarray(W_UK, dtype=F64)
    d_c = W_UK.shape[2]
    if U is None:
        U = np.eye(d_c, dtype=F64)
    W_UK_t, W_UV_t = reparameterize_weights(W_UK, W_UV, U, gamma)
    c_t = [transform_latent(c, U) for c in c_list]
    Q_lat = absorb_query(q_nope, W_UK_t, g, mu)
    dl = d_c // g
    O_lat = []
    lse = []
    for i in range(g):
        c_i = [c[:, i * dl:(i + 1) * dl] for c in c_t]
        O_i, lse_i = shard_attention(Q_lat[i], q_pe, c_i, kpe_list, scale)
        O_lat.append(O_i)
        lse.append(lse_i)
    O_lat = np.stack(O_lat)
    o = combine_shards(O_lat, W_UV_t)
    return {"W_UK_t": W_UK_t, "W_UV_t": W_UV_t, "c_t": c_t, "Q_lat": Q_lat,
            "O_lat": O_lat, "lse": np.stack(lse), "o": o}


def mla_absorbed(q_nope, q_pe, W_UK, W_UV, c_list, kpe_list, scale):
    """Absorbed MLA decode (Sec. 3.1 / 3.3): TPLA with a single slice."""
    return tpla_decode(q_nope, q_pe, W_UK, W_UV, c_list, kpe_list, 1, scale)["o"]


def mla_naive(q_nope, q_pe, W_UK, W_UV, c_list, kpe_list, scale):
    """Un-absorbed MLA (Sec. 3.3, eq. "isolate_rope"): materialise per-head
    keys k = W_UK[h] c and values v = c W_UV[h], then ordinary attention with
    the decoupled RoPE term added to the scores."""
    q_nope = np.asarray(q_nope, dtype=F64)
    q_pe = np.asarray(q_pe, dtype=F64)
    W_UK = np.asarray(W_UK, dtype=F64)
    W_UV = np.asarray(W_UV, dtype=F64)
    B, Hh, _ = q_nope.shape
    o = np.zeros((B, Hh, W_UV.shape[2]), dtype=F64)
    for b in range(B):
        cb = np.asarray(c_list[b], dtype=F64)
        kb = np.asarray(kpe_list[b], dtype=F64)
        if cb.shape[0] == 0:
            continue
        for h in range(Hh):
            k = cb @ W_UK[h].T                    # [L, d_n]
            v = cb @ W_UV[h]                      # [L, d_v]
            s = F64(scale) * (k @ q_nope[b, h] + kb @ q_pe[b, h])
            p, _ = _softmax_lse(s)
            o[b, h] = p @ v
    return o


def mla_prefill(q_nope, q_pe, W_UK, W_UV, c, k_pe, cu_seqlens, scale):
    """Prefill with MLA in its un-absorbed form (Sec. 4.5: prefill stays MLA,
    heads split over devices; Sec. 3.3 for the per-head keys and values): the
    T tokens of all sequences are packed, sequence b owning rows
    cu_seqlens[b]..cu_seqlens[b+1]-1.  Token t of a sequence attends to tokens
    0..t of the same sequence (causal):
        k[s, h] = W_UK[h] c_s,  v[s, h] = c_s W_UV[h]
        score[t, s, h] = scale (q_nope[t, h] . k[s, h] + q_pe[t, h] . k_pe[s]),  s <= t
        o[t, h] = sum_s softmax_s(score[t, :, h]) v[s, h]
    q_nope [T, H, d_n], q_pe [T, H, d_r], c [T, d_c], k_pe [T, d_r].
    Returns o [T, H, d_v]."""
    q_nope = np.asarray(q_nope, dtype=F64)
    q_pe = np.asarray(q_pe, dtype=F64)
    W_UK = np.asarray(W_UK, dtype=F64)
    W_UV = np.asarray(W_UV, dtype=F64)
    c = np.asarray(c, dtype=F64)
    k_pe = np.asarray(k_pe, dtype=F64)
    T, Hh, _ = q_nope.shape
    o = np.zeros((T, Hh, W_UV.shape[2]), dtype=F64)
    for b in range(len(cu_seqlens) - 1):
        t0, t1 = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        L = t1 - t0
        if L == 0:
            continue
        future = np.triu(np.ones((L, L), dtype=bool), k=1)          # [t, s] with s > t
        for h in range(Hh):
            k = c[t0:t1] @ W_UK[h].T                                 # [L, d_n]
            v = c[t0:t1] @ W_UV[h]                                   # [L, d_v]
            s = F64(scale) * (q_nope[t0:t1, h] @ k.T + q_pe[t0:t1, h] @ k_pe[t0:t1].T)
            s = np.where(future, -np.inf, s)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p /= p.sum(axis=1, keepdims=True)
            o[t0:t1, h] = p @ v
    return o


def tpla_bruteforce(q_nope, q_pe, W_UK, W_UV, c_list, kpe_list, g, scale, U=None, mu=None):
    """TPLA decode written with scalar Python loops only (tiny shapes).
    Independent of the vectorised functions above: used to cross-check them."""
    import math
    B = len(q_nope)
    Hh = len(q_nope[0])
    d_n = len(q_nope[0][0])
    d_r = len(q_pe[0][0])
    d_c = len(W_UK[0][0])
    d_v = len(W_UV[0][0])
    dl = d_c // g
    if U is None:
        U = [[1.0 if a == c else 0.0 for c in range(d_c)] for a in range(d_c)]
    if mu is None:
        mu = [1.0] * g
    out = [[[0.0] * d_v for _ in range(Hh)] for _ in range(B)]
    for b in range(B):
        L = len(c_list[b])
        # rows in the U basis
        ct = [[sum(float(c_list[b][t][a]) * float(U[a][j]) for a in range(d_c)) for j in range(d_c)]
              for t in range(L)]
        for h in range(Hh):
            Wk = [[sum(float(W_UK[h][n][a]) * float(U[a][j]) for a in range(d_c)) for j in range(d_c)]
                  for n in range(d_n)]
            Wv = [[sum(float(U[a][j]) * float(W_UV[h][a][v]) for a in range(d_c)) for v in range(d_v)]
                  for j in range(d_c)]
            Q = [sum(float(q_nope[b][h][n]) * Wk[n][j] for n in range(d_n)) for j in range(d_c)]
            for i in range(g):
                cols = range(i * dl, (i + 1) * dl)
                s = []
                for t in range(L):
                    lat = sum(Q[j] * ct[t][j] for j in cols)
                    pe = sum(float(q_pe[b][h][r]) * float(kpe_list[b][t][r]) for r in range(d_r))
                    s.append(float(scale) * (float(mu[i]) * lat + pe))
                if L == 0:
                    continue
                m = max(s)
                e = [math.exp(x - m) for x in s]
                z = sum(e)
                for j in cols:
                    O_j = sum(e[t] / z * ct[t][j] for t in range(L))
                    for v in range(d_v):
                        out[b][h][v] += O_j * Wv[j][v]
    return np.array(out, dtype=F64)


# --------------------------------------------------------------------------
# Storage helpers used when comparing against bf16 device buffers
# --------------------------------------------------------------------------
def round_to_bf16(x):
    """Round float64 values to the nearest bfloat16 (8 significant bits, ties
    to even) in one rounding step; returns float64.  Valid for normal-range
    magnitudes, which is all the synthetic workloads produce."""
    x = np.asarray(x, dtype=F64)
    m, e = np.frexp(x)                       # x = m * 2^e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def bf16_bits_to_f64(u16):
    """Exact value of bfloat16 bit patterns (uint16 array) as float64."""
    u = np.asarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(F64)


def paged_rows(pool, page_ids, L):
    """Rows 0..L-1 of a sequence from a paged pool [P, page_tokens, width]
    (pure integer indexing): token t lives in page page_ids[t // page_tokens]
    at slot t % page_tokens."""
    pool = np.asarray(pool)
    pt = pool.shape[1]
    t = np.arange(L)
    return pool[np.asarray(page_ids)[t // pt], t % pt]
