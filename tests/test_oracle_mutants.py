"""Each plausible mistake planted in the oracle (on the CPU, by patching one
function) must make at least one pin in test_oracle_pins.py fail."""
import numpy as np
import pytest

from oracle import tpla_oracle as orc
import test_oracle_pins as pins

PIN_FUNCS = [
    pins.test_hadamard_matches_printed_example,
    lambda: pins.test_hadamard_equals_library_and_is_orthogonal(8),
    pins.test_hadamard_sign_diagonal_side_and_orthogonality,
    pins.test_rmsnorm_textbook_values_and_prop1,
    pins.test_shard_attention_against_library_softmax,
    pins.test_two_token_closed_form,
    pins.test_softmax_invariants,
    pins.test_absorbed_equals_naive_equals_bruteforce,
    pins.test_absorb_query_definition,
    lambda: pins.test_tpla_equals_bruteforce_with_U_and_mu(2),
    pins.test_tpla_g1_is_mla_and_U_is_a_noop_at_g1,
    pins.test_tpla_differs_from_mla_in_general_but_matches_in_exact_cases,
    pins.test_row_parallel_identity_for_combine,
    pins.test_reparameterize_weights_layouts,
    pins.test_pca_closed_form_on_diagonal_covariance,
    pins.test_bf16_rounding_and_paging_helpers,
    pins.test_sliced_rmsnorm_append,
    pins.test_output_projection_is_head_major_and_row_parallel,
    pins.test_latent_moments_give_the_library_covariance,
    pins.test_prefill_is_token_by_token_decode_over_each_sequence_prefix,
]


def _some_pin_fails():
    for f in PIN_FUNCS:
        try:
            f()
        except (AssertionError, ValueError, IndexError):
            return True
    return False


_orig = {k: getattr(orc, k) for k in dir(orc) if callable(getattr(orc, k))}


def m_hadamard_wrong_block(d):
    Hm = np.ones((1, 1))
    while Hm.shape[0] < d:
        Hm = np.block([[Hm, Hm], [-Hm, Hm]])
    return Hm


def m_hadamard_scale(d, signs=None):
    return _orig["hadamard_U"](d, signs) / np.sqrt(d)


def m_hadamard_signs_right(d, signs=None):
    s = np.ones(d) if signs is None else np.asarray(signs, dtype=float)
    return _orig["sylvester_hadamard"](d) * s[None, :] / np.sqrt(d)


def m_transform_transposed(c, U):
    return np.asarray(c) @ np.asarray(U).T


def m_rms_sum(c, eps):
    c = np.asarray(c, dtype=float)
    return c / np.sqrt(np.sum(c * c, axis=-1, keepdims=True) + eps)


def m_rms_no_eps(c, eps):
    return _orig["rms_norm_unit"](c, 0.0)


def m_attention_no_rope(Q_i, q_pe, c_i, k_pe, scale):
    return _orig["shard_attention"](Q_i, np.zeros_like(q_pe), c_i, k_pe, scale)


def m_attention_scale_latent_only(Q_i, q_pe, c_i, k_pe, scale):
    return _orig["shard_attention"](Q_i, np.asarray(q_pe) / scale, c_i, k_pe, scale)


def m_attention_unnormalised(Q_i, q_pe, c_i, k_pe, scale):
    O, lse = _orig["shard_attention"](Q_i, q_pe, c_i, k_pe, scale)
    return O * np.exp(lse)[..., None], lse


def m_attention_lse_without_max(Q_i, q_pe, c_i, k_pe, scale):
    O, lse = _orig["shard_attention"](Q_i, q_pe, c_i, k_pe, scale)
    return O, lse - 1e-3


def m_combine_reversed(O_lat, W_UV_t):
    return _orig["combine_shards"](np.asarray(O_lat)[::-1], W_UV_t)


def m_combine_first_only(O_lat, W_UV_t):
    O = np.array(O_lat, dtype=float)
    O[1:] = 0
    return _orig["combine_shards"](O, W_UV_t)


def m_absorb_mu_divides(q_nope, W_UK_t, g, mu=None):
    mu = None if mu is None else 1.0 / np.asarray(mu, dtype=float)
    return _orig["absorb_query"](q_nope, W_UK_t, g, mu)


def m_absorb_transposed_slices(q_nope, W_UK_t, g, mu=None):
    Q = _orig["absorb_query"](q_nope, W_UK_t, g, mu)
    return Q[::-1]


def m_reparam_uk_transposed(W_UK, W_UV, U, gamma=None):
    return _orig["reparameterize_weights"](W_UK, W_UV, np.asarray(U).T, gamma)[0], \
        _orig["reparameterize_weights"](W_UK, W_UV, U, gamma)[1]


def m_reparam_no_gamma(W_UK, W_UV, U, gamma=None):
    return _orig["reparameterize_weights"](W_UK, W_UV, U, None)


def m_round_truncate(x):
    m, e = np.frexp(np.asarray(x, dtype=float))
    return np.ldexp(np.trunc(m * 256.0) / 256.0, e)


def m_round_half_away(x):
    m, e = np.frexp(np.asarray(x, dtype=float))
    return np.ldexp(np.sign(m) * np.floor(np.abs(m) * 256.0 + 0.5) / 256.0, e)


def m_paged_rows_transposed(pool, page_ids, L):
    pool = np.asarray(pool)
    pt = pool.shape[1]
    t = np.arange(L)
    return pool[np.asarray(page_ids)[t % len(page_ids)], (t // len(page_ids)) % pt]


def m_pca_ascending(F):
    U, lam = _orig["pca_U"](F)
    return U[:, ::-1], lam[::-1]


def m_fractions_reciprocal(ev, g=2):
    return 1.0 / _orig["variance_fractions"](ev, g)


def m_sliced_rms_local_mean(c_t, k_pe, g, alpha, eps):
    # each slice normalised by its own mean square, without the alpha / g correction
    return _orig["sliced_rms_rows"](c_t, k_pe, g, np.ones(g), eps)


def m_sliced_rms_eps_scaled(c_t, k_pe, g, alpha, eps):
    a = np.full(g, float(g)) if alpha is None else np.asarray(alpha, dtype=float)
    d = np.asarray(c_t).shape[-1]
    dl = d // g
    c = np.asarray(c_t, dtype=float); k = np.asarray(k_pe, dtype=float)
    return [np.concatenate([c[..., i * dl:(i + 1) * dl] /
                            np.sqrt(a[i] / g * (np.sum(c[..., i * dl:(i + 1) * dl] ** 2, axis=-1, keepdims=True) / dl + eps)), k], axis=-1)
            for i in range(g)]


def m_sliced_rms_kpe_normalised(c_t, k_pe, g, alpha, eps):
    rows = _orig["sliced_rms_rows"](c_t, k_pe, g, alpha, eps)
    dl = np.asarray(c_t).shape[-1] // g
    return [np.concatenate([r[..., :dl], r[..., dl:] * 0.5], axis=-1) for r in rows]


def m_output_projection_value_major(o, W_O):
    o = np.asarray(o, dtype=float)
    return o.transpose(0, 2, 1).reshape(o.shape[0], -1) @ np.asarray(W_O, dtype=float)


def _prefill_variant(mask_from, rope, respect_boundaries):
    """Prefill re-typed with one thing changed: first masked key offset, RoPE term, sequence walls."""
    def f(q_nope, q_pe, W_UK, W_UV, c, k_pe, cu_seqlens, scale):
        q_nope, q_pe, c, k_pe = (np.asarray(x, dtype=np.float64) for x in (q_nope, q_pe, c, k_pe))
        T, Hh, _ = q_nope.shape
        o = np.zeros((T, Hh, np.asarray(W_UV).shape[2]))
        cu = list(cu_seqlens) if respect_boundaries else [0, T]
        for b in range(len(cu) - 1):
            t0, t1 = int(cu[b]), int(cu[b + 1])
            L = t1 - t0
            if L == 0:
                continue
            masked = np.triu(np.ones((L, L), dtype=bool), k=mask_from)
            for h in range(Hh):
                k = c[t0:t1] @ np.asarray(W_UK)[h].T
                v = c[t0:t1] @ np.asarray(W_UV)[h]
                s_ = scale * (q_nope[t0:t1, h] @ k.T + (q_pe[t0:t1, h] @ k_pe[t0:t1].T if rope else 0.0))
                s_ = np.where(masked, -1e300, s_)
                p = np.exp(s_ - s_.max(axis=1, keepdims=True))
                o[t0:t1, h] = (p / p.sum(axis=1, keepdims=True)) @ v
        return o
    return f


m_prefill_sees_next_token = _prefill_variant(2, True, True)
m_prefill_sees_next_token.__name__ = "m_prefill_sees_next_token"
m_prefill_not_causal = _prefill_variant(10 ** 6, True, True)
m_prefill_not_causal.__name__ = "m_prefill_not_causal"
m_prefill_no_rope = _prefill_variant(1, False, True)
m_prefill_no_rope.__name__ = "m_prefill_no_rope"
m_prefill_no_sequence_walls = _prefill_variant(1, True, False)
m_prefill_no_sequence_walls.__name__ = "m_prefill_no_sequence_walls"


def m_moments_centered(F):
    F = np.asarray(F, dtype=np.float64)
    Fc = F - F.mean(axis=0, keepdims=True)
    return F.sum(axis=0), Fc.T @ Fc


MUTANTS = [
    ("mla_prefill", m_prefill_sees_next_token),
    ("mla_prefill", m_prefill_not_causal),
    ("mla_prefill", m_prefill_no_rope),
    ("mla_prefill", m_prefill_no_sequence_walls),
    ("latent_moments", m_moments_centered),
    ("output_projection", m_output_projection_value_major),
    ("sliced_rms_rows", m_sliced_rms_local_mean),
    ("sliced_rms_rows", m_sliced_rms_eps_scaled),
    ("sliced_rms_rows", m_sliced_rms_kpe_normalised),
    ("sylvester_hadamard", m_hadamard_wrong_block),
    ("hadamard_U", m_hadamard_scale),
    ("hadamard_U", m_hadamard_signs_right),
    ("transform_latent", m_transform_transposed),
    ("rms_norm_unit", m_rms_sum),
    ("rms_norm_unit", m_rms_no_eps),
    ("shard_attention", m_attention_no_rope),
    ("shard_attention", m_attention_scale_latent_only),
    ("shard_attention", m_attention_unnormalised),
    ("shard_attention", m_attention_lse_without_max),
    ("combine_shards", m_combine_reversed),
    ("combine_shards", m_combine_first_only),
    ("absorb_query", m_absorb_mu_divides),
    ("absorb_query", m_absorb_transposed_slices),
    ("reparameterize_weights", m_reparam_uk_transposed),
    ("reparameterize_weights", m_reparam_no_gamma),
    ("round_to_bf16", m_round_truncate),
    ("round_to_bf16", m_round_half_away),
    ("paged_rows", m_paged_rows_transposed),
    ("pca_U", m_pca_ascending),
    ("variance_fractions", m_fractions_reciprocal),
]


def test_unmutated_oracle_passes_every_pin():
    assert not _some_pin_fails()


@pytest.mark.parametrize("name,mutant", MUTANTS, ids=[f"{n}:{m.__name__}" for n, m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    monkeypatch.setattr(orc, name, mutant)
    assert _some_pin_fails(), f"no pin notices the mistake {mutant.__name__}"
