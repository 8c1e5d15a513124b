"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2508_15881_amd as tp
from paper_2508_15881_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "tpla.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tpla_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = tp.load_library()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert tp.tpla_version() >= 100
    assert isinstance(tp.tpla_last_error(), str)


def _shape(**kw):
    base = dict(B=2, H=64, d_c=512, g=2, d_r=64, d_n=128, d_v=128, page_tokens=64, dtype=tp.TPLA_BF16, sm_scale=0.07)
    base.update(kw)
    return tp.TplaShape(**base)


A = 4096   # a 16-byte aligned fake address: validation must fail before it is ever used


def _code(fn, *args):
    with pytest.raises(tp.TplaError) as e:
        fn(*args)
    assert tp.tpla_last_error() != ""
    return e.value.code


def test_decode_shard_argument_checks():
    s = _shape()
    assert _code(tp.tpla_decode_shard, s, None, A, A, A, 4, A, 0, A, 1 << 30, A, None) == -1
    assert _code(tp.tpla_decode_shard, s, A, A, A, A, 0, A, 0, A, 1 << 30, A, None) == -2
    assert _code(tp.tpla_decode_shard, s, A + 2, A, A, A, 4, A, 0, A, 1 << 30, A, None) == -3
    assert _code(tp.tpla_decode_shard, s, A, A, A, A, 4, A, 2, A, 16, A, None) == -4
    assert _code(tp.tpla_decode_shard, _shape(dtype=7), A, A, A, A, 4, A, 0, A, 1 << 30, A, None) == -5
    assert _code(tp.tpla_decode_shard, _shape(g=3), A, A, A, A, 4, A, 0, A, 1 << 30, A, None) == -2
    assert _code(tp.tpla_decode_shard, _shape(d_r=60), A, A, A, A, 4, A, 0, A, 1 << 30, A, None) == -2
    assert _code(tp.tpla_decode_shard, _shape(sm_scale=0.0), A, A, A, A, 4, A, 0, A, 1 << 30, A, None) == -2
    assert _code(tp.tpla_decode_shard, _shape(g=16, d_c=1024), A, A, A, A, 4, A, 0, A, 1 << 30, A, None) == -2


def test_workspace_bytes():
    s = _shape()
    one = tp.tpla_workspace_bytes(s, 512, 1)
    assert one == 2 * 1 * 64 * (256 + 2) * 4
    assert tp.tpla_workspace_bytes(s, 512, 8) == 8 * one
    assert tp.tpla_workspace_bytes(s, 4, 100) == 4 * one          # never more splits than pages
    auto = tp.tpla_workspace_bytes(s, 512, 0)      # balanced plan: one slot per workgroup and per sequence,
    plan_table = (3 * 2 + 2) * 4                   # then three ints per sequence (B = 2) and two more, in whole 16 bytes
    assert auto > one and (auto - plan_table) % (64 * (256 + 2) * 4) == 0
    assert tp.tpla_workspace_bytes_all(s, 512, 0) >= auto
    assert tp.tpla_workspace_bytes_all(s, 512, 3) == 2 * tp.tpla_workspace_bytes(s, 512, 3)
    assert tp.tpla_workspace_bytes(s, 0, 0) == 0
    assert tp.tpla_workspace_bytes(_shape(H=0), 4, 0) == 0


def test_other_entry_points_argument_checks():
    s = _shape()
    assert _code(tp.tpla_absorb_query, s, None, A, None, A) == -1
    assert _code(tp.tpla_absorb_query, s, A, A + 4, None, A) == -3
    assert _code(tp.tpla_absorb_query, s, A, A, [1.0, float("inf")], A) == -2
    assert _code(tp.tpla_combine_shards, s, A, None, A) == -1
    assert _code(tp.tpla_combine_shards, _shape(B=0), A, A, A) == -2
    assert _code(tp.tpla_transform_latent, s, 9, 0, None, None, A, A, 4, 1) == -2
    assert _code(tp.tpla_transform_latent, _shape(d_c=96), tp.TPLA_U_HADAMARD, 0, None, None, A, A, 4, 1) == -2
    assert _code(tp.tpla_transform_latent, s, tp.TPLA_U_DENSE, 0, None, None, A, A, 4, 1) == -1
    assert _code(tp.tpla_transform_latent, s, tp.TPLA_U_IDENTITY, 0, None, None, None, A, 4, 1) == -1
    assert _code(tp.tpla_transform_latent_paged, s, tp.TPLA_U_IDENTITY, None, None, A, [A, None], None, 3) == -1
    assert _code(tp.tpla_transform_latent_paged, s, tp.TPLA_U_IDENTITY, None, None, A, [A, A + 8], None, 3) == -3
    assert _code(tp.tpla_transform_latent_paged, s, tp.TPLA_U_IDENTITY, None, None, A, [A, A], None, -1) == -2
    assert _code(tp.tpla_write_mla_cache, s, A, A, None, 5, 1e-6, A) == -1
    assert _code(tp.tpla_write_mla_cache, s, A, A, A, -5, 1e-6, A) == -2
    assert _code(tp.tpla_append_token_sliced, s, A, A, None, 1e-6, None, [A, A]) == -1
    assert _code(tp.tpla_append_token_sliced, s, A, A, [2.0, -1.0], 1e-6, A, [A, A]) == -2
    assert _code(tp.tpla_append_token_sliced, s, A, A, None, -1.0, A, [A, A]) == -2
    assert _code(tp.tpla_append_token_sliced, s, A, A, None, 1e-6, A, [A, A + 4]) == -3
    # output projection, PCA moments, prefill
    assert _code(tp.tpla_output_projection, s, A, None, 64, A, 1 << 20, A) == -1
    assert _code(tp.tpla_output_projection, s, A, A, 0, A, 1 << 20, A) == -2
    assert tp.tpla_latent_moments_workspace_bytes(s, 0) == 0 and tp.tpla_latent_moments_workspace_bytes(s, 40) > 0
    assert _code(tp.tpla_latent_moments, s, None, None, None, 4, A, 1 << 30, A, A) == -1
    assert _code(tp.tpla_latent_moments, s, A, None, None, 0, A, 1 << 30, A, A) == -2
    assert _code(tp.tpla_latent_moments, s, A, None, None, 4, A, 16, A, A) == -4
    assert _code(tp.tpla_latent_moments, s, A, None, None, 4, A + 4, 1 << 30, A, A) == -3
    sp = _shape(d_n=128, d_v=128)
    assert tp.tpla_prefill_workspace_bytes(sp, 100) == 100 * 64 * 256 * 2 and tp.tpla_prefill_workspace_bytes(sp, 0) == 0
    assert _code(tp.tpla_prefill_attention, sp, A, A, A, A, A, A, None, 8, 8, A, 1 << 30, A) == -1
    assert _code(tp.tpla_prefill_attention, sp, A, A, A, A, A, A, A, 0, 8, A, 1 << 30, A) == -2
    assert _code(tp.tpla_prefill_attention, sp, A, A, A, A, A, A, A, 8, 0, A, 1 << 30, A) == -2
    assert _code(tp.tpla_prefill_attention, sp, A, A, A, A, A, A, A, 8, 8, A, 64, A) == -4
    assert _code(tp.tpla_prefill_attention, sp, A, A + 2, A, A, A, A, A, 8, 8, A, 1 << 30, A) == -3
    assert _code(tp.tpla_prefill_attention, _shape(d_n=64), A, A, A, A, A, A, A, 8, 8, A, 1 << 30, A) == -7
    # decode + merge + combine in one call: its own pointers, then the decode's checks
    assert _code(tp.tpla_decode_shards_combine, s, A, A, [A, A], A, 4, A, 0, A, 1 << 30, None, A, A, None) == -1
    assert _code(tp.tpla_decode_shards_combine, s, A, A, [A, A], A, 4, A, 0, A, 1 << 30, A, None, A, None) == -1
    assert _code(tp.tpla_decode_shards_combine, s, A, A, [A, A], A, 4, A, 0, A, 1 << 30, A, A, None, None) == -1
    assert _code(tp.tpla_decode_shards_combine, s, A, A, [A, A], A, 4, A, 0, A, 1 << 30, A + 2, A, A, None) == -3
    assert _code(tp.tpla_decode_shards_combine, s, A, A, [A, None], A, 4, A, 0, A, 1 << 30, A, A, A, None) == -1
    assert _code(tp.tpla_decode_shards_combine, s, A, A, [A, A], A, 4, A, 2, A, 16, A, A, A, None) == -4
    # chosen output types; the attention block in one call checks both stages before any launch
    assert _code(tp.tpla_combine_shards_to, s, A, A, A, 9) == -5
    assert _code(tp.tpla_combine_shards_to, s, A, A, None, tp.TPLA_BF16) == -1
    assert _code(tp.tpla_output_projection_to, s, A, A, 64, A, 1 << 20, A, 9) == -5
    assert _code(tp.tpla_decode_shards_combine_to, s, A, A, [A, A], A, 4, A, 0, A, 1 << 30, A, A, 9, A, None) == -5
    big = 1 << 30
    assert _code(tp.tpla_decode_shards_project, s, A, A, [A, A], A, 4, A, 0, A, big, A, None, 7168, A, tp.TPLA_F32, A, A, None) == -1
    assert _code(tp.tpla_decode_shards_project, s, A, A, [A, A], A, 4, A, 0, A, big, A, A, 0, A, tp.TPLA_F32, A, A, None) == -2
    assert _code(tp.tpla_decode_shards_project, s, A, A, [A, A], A, 4, A, 0, A, big, A, A, 7168, A, 3, A, A, None) == -5
    assert _code(tp.tpla_decode_shards_project, s, A, A, [A, A], A, 4, A, 0, A, 64, A, A, 7168, A, tp.TPLA_BF16, A, A, None) == -4
    assert _code(tp.tpla_decode_shards_project, s, A, A, [A, A], A, 4, A, 0, A, big, A, A + 2, 7168, A, tp.TPLA_F32, A, A, None) == -3
    assert tp.tpla_attention_block_workspace_bytes(s, 512, 0, 7168) >= tp.tpla_workspace_bytes_all(s, 512, 0)
    assert tp.tpla_attention_block_workspace_bytes(s, 512, 0, 0) == 0
    # empty work is accepted without a launch
    tp.tpla_transform_latent(s, tp.TPLA_U_IDENTITY, 0, None, None, A, A, 0, 1)
    tp.tpla_transform_latent_paged(s, tp.TPLA_U_IDENTITY, None, None, A, [A, A], None, 0)
    tp.tpla_write_mla_cache(s, A, A, A, 0, 1e-6, A)


def test_validate_block_table_names_the_first_bad_entry():
    s = _shape(B=3)
    bt = np.array([[0, 1, 2, 3], [4, 5, 0, 0], [6, 0, 0, 0]], dtype=np.int32)
    ln = np.array([200, 65, 1], dtype=np.int32)               # 4, 2 and 1 pages in use
    tp.tpla_validate_block_table(s, bt, 4, ln, 7)
    tp.tpla_validate_block_table(s, bt, 4, ln, 7, forbid_shared=True)
    tp.tpla_validate_block_table(s, bt, 4, np.zeros(3, dtype=np.int32), 1)     # nothing in use: ids are not looked at
    assert _code(tp.tpla_validate_block_table, s, bt, 4, ln, 6) == -2 and "block_table[2][0]=6" in tp.tpla_last_error()
    bad = bt.copy(); bad[1, 1] = -1
    assert _code(tp.tpla_validate_block_table, s, bad, 4, ln, 7) == -2 and "block_table[1][1]=-1" in tp.tpla_last_error()
    bad = bt.copy(); bad[1, 3] = 99                            # beyond the pages in use: ignored
    tp.tpla_validate_block_table(s, bad, 4, ln, 7, forbid_shared=True)
    assert _code(tp.tpla_validate_block_table, s, bt, 4, np.array([257, 65, 1], dtype=np.int32), 7) == -2
    assert "seq_lens[0]=257" in tp.tpla_last_error()
    assert _code(tp.tpla_validate_block_table, s, bt, 4, np.array([200, -1, 1], dtype=np.int32), 7) == -2
    shared = bt.copy(); shared[2, 0] = 1
    tp.tpla_validate_block_table(s, shared, 4, ln, 7)           # sharing a page is legal for reading
    assert _code(tp.tpla_validate_block_table, s, shared, 4, ln, 7, True) == -2 and "page 1" in tp.tpla_last_error()
    assert _code(tp.tpla_validate_block_table, s, None, 4, ln, 7) == -1
    assert _code(tp.tpla_validate_block_table, s, bt, 4, ln, 0) == -2
    with pytest.raises(ValueError):
        tp.tpla_validate_block_table(s, bt, 3, ln, 7)          # the binding checks the array shapes itself


def test_missing_library_is_a_loud_error(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libtpla.so")
    with pytest.raises(RuntimeError, match="not found"):
        binding.load_library()


def test_workload_generators_are_seeded_and_consistent():
    import numpy as np
    from paper_2508_15881_amd import workloads as wl
    w = wl.CONFIGS["tiny"]
    a, b = wl.draw_model_side(w), wl.draw_model_side(w)
    assert all(np.array_equal(a[k], b[k]) for k in ("W_UK", "W_UV", "q_nope", "q_pe", "signs", "seq_lens", "block_table"))
    c1, k1 = wl.draw_sequence(w, 0, 128); c2, k2 = wl.draw_sequence(w, 0, 128)
    assert np.array_equal(c1, c2) and np.array_equal(k1, k2) and c1.shape == (128, 64) and k1.shape == (128, 16)
    # bf16 bit patterns: round to nearest even, exact decode
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.14159], dtype=np.float32)
    bits = wl.f32_to_bf16_bits(x)
    assert list(wl.as_f64(bits, "bf16")[:4]) == [1.0, 1.0, 1.015625, -2.5]
    r = wl.CONFIGS["ragged_g4"]
    m = wl.draw_model_side(r)
    assert m["seq_lens"].min() >= 1024 and m["seq_lens"].max() <= 131072 and m["seq_lens"].shape == (128,)
    pages = (m["seq_lens"].astype(np.int64) + 63) // 64
    ids = np.concatenate([m["block_table"][i, :pages[i]] for i in range(128)])
    assert len(np.unique(ids)) == len(ids) and ids.max() < m["n_pool_pages"]
    assert wl.algorithmic_bytes_per_shard(wl.CONFIGS["dsv3_32k"], np.full(32, 32768)) == 671088640
