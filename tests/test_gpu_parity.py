"""GPU parity: every C-ABI entry point against the float64 oracle on the same
seeded inputs.  Tolerances: bit-exact for paging / copies, max|x-r|/max|r| <=
1e-5 (float storage) or 1e-2 (bf16 storage, float accumulation) otherwise."""
import numpy as np
import pytest
import torch

import paper_2508_15881_amd as tp
from paper_2508_15881_amd import pipeline as pl
from paper_2508_15881_amd import workloads as wl
from oracle import tpla_oracle as orc
from gpu_common import elementwise_err, TOL, build_shard_problem, oracle_decode_shard, rel_err, run_decode_shard

pytestmark = pytest.mark.gpu

DSV3 = wl.CONFIGS["dsv3_4k"]
KIMI = wl.CONFIGS["kimi_32k"]
RAGGED = wl.CONFIGS["ragged_g4"]


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------ decode_shard
MFMA_CASES = [
    ("dsv3_g2_H64", DSV3, [1, 63, 64, 65, 700, 2049, 0, 31]),
    ("kimi_g2_H32", KIMI, [129, 1000, 5, 64]),
    ("ragged_g4_H64", RAGGED, [3000, 17, 256, 4097]),
    ("mla_g1_H64", wl.scaled(DSV3, g=1), [333, 64, 1025]),
    # 576-wide rows with 64 heads run as pairs of waves: one tile, whole tiles, odd and even tile counts,
    # ragged tails in the first and the second half of a tile, empty sequences, more than 64 pages per item
    ("mla_g1_H64_tiles", wl.scaled(DSV3, g=1), [1, 15, 16, 17, 32, 33, 48, 63, 64, 65, 96, 97, 0, 127, 129, 4500]),
    ("mla_g1_H32", wl.scaled(KIMI, g=1), [1, 33, 64, 97, 700, 0, 2049]),
    ("dsv3_g2_H128", wl.scaled(DSV3, H=128), [500, 130]),
    ("dsv3_g2_H16", wl.scaled(DSV3, H=16), [500, 130]),
    # the remaining instances of the matrix-core kernel (slice width x head count), so that each is
    # compared with the oracle in both its static-chunk and its balanced form
    ("g4_H16", wl.scaled(RAGGED, H=16), [300, 65, 1]),
    ("g4_H32", wl.scaled(RAGGED, H=32), [300, 65, 1]),
    ("g4_H128", wl.scaled(RAGGED, H=128), [300, 65, 1]),
    ("mla_g1_H16", wl.scaled(DSV3, g=1, H=16), [300, 65, 1]),
    ("mla_g1_H128", wl.scaled(DSV3, g=1, H=128), [300, 65, 1]),
]


@pytest.mark.parametrize("name,w,lens", MFMA_CASES, ids=[c[0] for c in MFMA_CASES])
@pytest.mark.parametrize("n_splits", [0, 1, 3])
def test_decode_shard_bf16_matches_oracle(name, w, lens, n_splits):
    _say(f"decode_shard bf16 {name} lens={lens} n_splits={n_splits}")
    prob = build_shard_problem(w, lens)
    o, lse = run_decode_shard(prob, n_splits)
    ro, rl = oracle_decode_shard(prob)
    nz = np.asarray(lens) > 0
    assert rel_err(o, ro) <= TOL["bf16"]
    assert elementwise_err(o, ro) <= TOL["bf16"]         # |x - r| <= tol (|r| + rms(r)) for every element
    assert np.max(np.abs(lse[nz] - rl[nz])) <= 1e-2
    assert np.all(o[~nz] == 0) and np.all(np.isneginf(lse[~nz]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decode_shard_generic_shapes(dtype):
    # widths the matrix-core kernel does not cover: generic kernel, both storage types
    w = wl.Workload("odd", B=3, H=5, d_c=80, g=2, d_r=24, d_n=16, d_v=16, dtype=dtype, seed=11)
    for n_splits in (0, 1, 2):
        _say(f"decode_shard generic {dtype} n_splits={n_splits}")
        prob = build_shard_problem(w, [200, 0, 65])
        o, lse = run_decode_shard(prob, n_splits)
        ro, rl = oracle_decode_shard(prob)
        assert rel_err(o, ro) <= TOL[dtype]
        assert np.max(np.abs(lse[[0, 2]] - rl[[0, 2]])) <= TOL[dtype] * 10
        assert np.all(o[1] == 0) and np.all(np.isneginf(lse[1]))


def test_decode_shard_many_short_sequences():
    # more sequences than workgroups' page ranges can separate: the automatic plan
    # gives a workgroup pieces of several sequences, and sequences several workgroups
    w = wl.scaled(RAGGED, H=16)
    rng = np.random.default_rng(99)
    lens = rng.integers(0, 400, size=700)
    lens[::97] = 0
    lens[5] = 9000                       # one long sequence among the short ones
    _say(f"decode_shard many short sequences B={len(lens)} tokens={int(lens.sum())}")
    prob = build_shard_problem(w, lens)
    o, lse = run_decode_shard(prob, 0)
    ro, rl = oracle_decode_shard(prob)
    nz = lens > 0
    assert rel_err(o, ro) <= TOL["bf16"]
    assert np.max(np.abs(lse[nz] - rl[nz])) <= 1e-2
    assert np.all(o[~nz] == 0) and np.all(np.isneginf(lse[~nz]))
    o2, lse2 = run_decode_shard(prob, 0)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)


def test_decode_shard_random_batches():
    # seeded random batches (lengths, widths, head counts, split counts) through both plans
    rng = np.random.default_rng(2024)
    shapes = [(DSV3, {}), (KIMI, {}), (RAGGED, {}), (wl.scaled(DSV3, H=16), {}), (wl.scaled(RAGGED, H=32), {})]
    for case in range(12):
        w, _ = shapes[case % len(shapes)]
        Bn = int(rng.integers(1, 40))
        kind = case % 3
        if kind == 0:
            lens = rng.integers(0, 300, size=Bn)
        elif kind == 1:
            lens = np.floor(np.exp(rng.uniform(0, np.log(6000), size=Bn))).astype(np.int64)
        else:
            lens = np.full(Bn, int(rng.integers(1, 1500)))
        n_splits = int(rng.choice([0, 0, 1, 2, 7, 50]))
        _say(f"random batch {case}: {w.name} H={w.H} dl={w.dl} B={Bn} tokens={int(lens.sum())} n_splits={n_splits}")
        prob = build_shard_problem(w, lens, rng_extra=case)
        o, lse = run_decode_shard(prob, n_splits)
        ro, rl = oracle_decode_shard(prob)
        nz = np.asarray(lens) > 0
        if nz.any():
            assert rel_err(o[nz], ro[nz]) <= TOL["bf16"]
            assert np.max(np.abs(lse[nz] - rl[nz])) <= 1e-2
        assert np.all(o[~nz] == 0) and np.all(np.isneginf(lse[~nz]))


def test_profile_brackets_count_decode_launches():
    prob = build_shard_problem(wl.scaled(DSV3, H=16), [100, 300])
    tp.tpla_profile_enable(3)
    for _ in range(5):
        run_decode_shard(prob, 0)
    ms = tp.tpla_profile_collect(8)
    assert len(ms) == 3 and all(0.0 < m < 100.0 for m in ms)      # capped at the enabled count
    assert tp.tpla_profile_collect(8) == []
    tp.tpla_profile_enable(0)
    run_decode_shard(prob, 0)
    assert tp.tpla_profile_collect(8) == []


def test_decode_shard_other_page_sizes_and_one_long_sequence():
    # 16-token pages (generic kernel), bf16 and float
    for dtype in ("bf16", "f32"):
        w = wl.Workload("p16", B=2, H=8, d_c=256, g=2, d_r=64, d_n=16, d_v=16, dtype=dtype, page_tokens=16, seed=12)
        _say(f"decode_shard page_tokens=16 {dtype}")
        prob = build_shard_problem(w, [333, 16])
        o, lse = run_decode_shard(prob, 0)
        ro, rl = oracle_decode_shard(prob)
        assert rel_err(o, ro) <= TOL[dtype] and np.max(np.abs(lse - rl)) <= TOL[dtype] * 10
    # one sequence of 100k tokens: every workgroup holds a piece of it, the merge sums hundreds of partials
    _say("decode_shard single sequence of 100000 tokens")
    prob = build_shard_problem(wl.scaled(DSV3, H=16), [100000])
    o, lse = run_decode_shard(prob, 0)
    ro, rl = oracle_decode_shard(prob)
    assert rel_err(o, ro) <= TOL["bf16"] and np.max(np.abs(lse - rl)) <= 1e-2


def test_decode_shard_paging_is_bit_invariant():
    lens = [700, 65, 1, 2048]
    _say("decode_shard paging invariance")
    a = build_shard_problem(DSV3, lens, permute=True, slack_pages=5, poison=True)
    b = build_shard_problem(DSV3, lens, permute=False, slack_pages=0, poison=False)
    for n_splits in (0, 1, 4):
        oa, la = run_decode_shard(a, n_splits)
        ob, lb = run_decode_shard(b, n_splits)
        assert np.array_equal(oa, ob) and np.array_equal(la, lb)
        oa2, la2 = run_decode_shard(a, n_splits)
        assert np.array_equal(oa, oa2) and np.array_equal(la, la2)     # reproducible bits
    assert np.all(np.isfinite(oa))                                     # NaN tails / spare pages never leak


def test_peaky_softmax_exercises_the_rescale_path():
    """Queries 16x larger: scores spread over hundreds of log2 units, the running reference of the
    online softmax moves on most tiles and almost all weight sits on a few tokens."""
    _say("peaky softmax (decode and prefill)")
    for w, lens in ((DSV3, [700, 65]), (wl.scaled(DSV3, g=1), [300])):
        prob = build_shard_problem(w, lens)
        prob["q_lat"] = wl.to_storage(wl.as_f64(prob["q_lat"], "bf16") * 16.0, "bf16")
        prob["q_pe"] = wl.to_storage(wl.as_f64(prob["q_pe"], "bf16") * 16.0, "bf16")
        for n_splits in (0, 2):
            o, lse = run_decode_shard(prob, n_splits)
            ro, rl = oracle_decode_shard(prob)
            assert rel_err(o, ro) <= TOL["bf16"]
            assert np.max(np.abs(lse - rl) / np.maximum(1.0, np.abs(rl))) <= 1e-2
    p = _prefill_problem(9, [300, 77], 2, 256)
    p["q_nope"] = wl.to_storage(wl.as_f64(p["q_nope"], "bf16") * 16.0, "bf16")
    p["q_pe"] = wl.to_storage(wl.as_f64(p["q_pe"], "bf16") * 16.0, "bf16")
    f64 = {k: wl.as_f64(p[k], "bf16") for k in ("q_nope", "q_pe", "c", "k_pe", "W_UK", "W_UV")}
    ref = orc.mla_prefill(f64["q_nope"], f64["q_pe"], f64["W_UK"], f64["W_UV"], f64["c"], f64["k_pe"], p["cu"], 1.0 / np.sqrt(192.0))
    o, _ = _run_prefill(p, 2, 256, 2, 300)
    assert rel_err(o, ref) <= TOL["bf16"]


def test_lengths_beyond_the_table_are_clipped_not_followed():
    """A length that disagrees with max_pages_per_seq (or cu_seqlens that run past T) is clipped by
    the kernels to what the tables can address: same result as the clipped input, no stray read."""
    _say("lengths beyond the tables are clipped")
    for dtype in ("bf16", "f32"):
        w = wl.scaled(wl.CONFIGS["dsv3_4k"], dtype=dtype, H=16)
        prob = build_shard_problem(w, [256, 128], permute=True)          # table rows hold 4 pages
        good = run_decode_shard(prob)
        wild = run_decode_shard(prob, lens_override=[1 << 20, 128])
        neg = run_decode_shard(prob, lens_override=[256, -7])
        assert np.array_equal(good[0], wild[0]) and np.array_equal(good[1], wild[1])
        assert np.array_equal(good[0][0], neg[0][0]) and np.all(neg[0][1] == 0) and np.all(np.isneginf(neg[1][1]))
    p = _prefill_problem(3, [40, 24], 2, 128)
    ref, _ = _run_prefill(p, 2, 128, 2, 40)
    p2 = dict(p); p2["cu"] = np.array([0, 40, 9999], dtype=np.int32)      # second range runs past T = 64
    got, _ = _run_prefill(p2, 2, 128, 2, 40)
    assert np.array_equal(ref, got)


def test_decode_shard_softmax_properties_at_long_context():
    # one long sequence (spans many tiles and splits): weights sum to one and
    # the output stays inside the rows' column range
    prob = build_shard_problem(DSV3, [20000, 8191])
    w = prob["w"]
    o, lse = run_decode_shard(prob, 0)
    ro, rl = oracle_decode_shard(prob)
    assert rel_err(o, ro) <= TOL["bf16"]
    assert np.max(np.abs(lse - rl)) <= 1e-2
    for b in range(2):
        lat = prob["rows64"][b][:, :w.dl]
        assert np.all(o[b] <= lat.max(axis=0) + 1e-3) and np.all(o[b] >= lat.min(axis=0) - 1e-3)


def test_decode_shards_equals_one_call_per_slice():
    # all slices in one launch == g single-slice calls, bit for bit at equal split count
    w = wl.scaled(DSV3, B=3)
    lens = np.array([700, 65, 2048], dtype=np.int32)
    _say("decode_shards vs decode_shard")
    probs = [build_shard_problem(w, lens, rng_extra=i) for i in range(w.g)]
    shape = pl.make_shape(w)
    dev = "cuda"
    q_lat = pl.to_device(np.stack([p["q_lat"] for p in probs]), "bf16")
    q_pe = pl.to_device(probs[0]["q_pe"], "bf16")
    pools = [pl.to_device(p["pool"], "bf16") for p in probs]
    # the slices share one page table: reuse slice 0's table for every pool
    for i in range(1, w.g):
        pools[i] = pl.to_device(probs[0]["pool"][:, :, ::-1].copy(), "bf16")    # different contents, same paging
    bt = torch.from_numpy(probs[0]["bt"]).to(dev); ln = torch.from_numpy(lens).to(dev)
    mp = probs[0]["max_pages"]
    for n_splits in (0, 4):
        ws_b = tp.tpla_workspace_bytes_all(shape, mp, n_splits)
        ws = torch.empty(ws_b, dtype=torch.uint8, device=dev)
        o_all = torch.full((w.g, 3, w.H, w.dl), float("nan"), dtype=torch.float32, device=dev)
        l_all = torch.full((w.g, 3, w.H), float("nan"), dtype=torch.float32, device=dev)
        tp.tpla_decode_shards(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, o_all, l_all)
        o_one = torch.empty_like(o_all); l_one = torch.empty_like(l_all)
        ws1_b = tp.tpla_workspace_bytes(shape, mp, n_splits)
        ws1 = torch.empty(ws1_b, dtype=torch.uint8, device=dev)
        for i in range(w.g):
            tp.tpla_decode_shard(shape, q_lat[i], q_pe, pools[i], bt, mp, ln, n_splits, ws1, ws1_b, o_one[i], l_one[i])
        torch.cuda.synchronize()
        if n_splits:
            assert torch.equal(o_all, o_one) and torch.equal(l_all, l_one)
        else:
            assert rel_err(o_all.cpu().numpy(), o_one.cpu().numpy()) <= 1e-4
    # and against the oracle for slice 0
    ro, rl = oracle_decode_shard(probs[0])
    assert rel_err(o_all[0].cpu().numpy(), ro) <= TOL["bf16"]


# ------------------------------------------------------------ decode + merge + combine in one call
COMBINE_CASES = [
    # name, workload, lengths (B = their number), split counts
    ("dsv3_two_seq_blocks", DSV3, [700, 65, 2048, 0, 1, 64, 3000, 129, 31, 640, 5, 900, 63, 257, 1100, 2, 333, 77, 1500], (0, 4)),
    ("ragged_g4", RAGGED, [3000, 17, 0, 256, 4097], (0, 3)),
    ("wide_two_chunks", wl.scaled(DSV3, d_c=1024), [500, 130, 1025], (0, 2)),
    ("mla_g1", wl.scaled(DSV3, g=1), [333, 64, 1025], (0,)),
    ("fewer_pages_than_workgroups", DSV3, [1, 64, 0, 33, 7, 60, 12, 64, 2, 50, 64, 31, 9, 40, 3, 64, 20], (0,)),
    ("kimi_H32", KIMI, [129, 1000, 5, 64], (0, 1)),
    # every workgroup of the launch works on the one sequence: hundreds of partial results per
    # (slice, sequence), merged 16 at a time with a moving reference
    ("one_long_sequence", DSV3, [70000], (0, 100)),
    ("generic_f32", wl.Workload("odd", B=3, H=5, d_c=80, g=2, d_r=24, d_n=16, d_v=16, dtype="f32", seed=11), [200, 0, 65], (0, 2)),
]


@pytest.mark.parametrize("name,w,lens,splits", COMBINE_CASES, ids=[c[0] for c in COMBINE_CASES])
def test_decode_shards_combine_matches_oracle_and_the_separate_calls(name, w, lens, splits):
    lens = np.asarray(lens, dtype=np.int32)
    Bn = len(lens)
    w = wl.scaled(w, B=Bn)
    probs = [build_shard_problem(w, lens, rng_extra=i) for i in range(w.g)]
    shape = pl.make_shape(w)
    dev = "cuda"
    dt = w.dtype
    q_lat = pl.to_device(np.stack([p["q_lat"] for p in probs]), dt)
    q_pe = pl.to_device(probs[0]["q_pe"], dt)
    # the slices share one page table and one k_pe (Sec. 4.2): slice i's pool takes slice 0's paging
    # and RoPE columns and its own latent columns
    pools_np = []
    for i in range(w.g):
        pool = probs[0]["pool"].copy()
        src = probs[i]
        for b in range(Bn):
            n = (int(lens[b]) + w.page_tokens - 1) // w.page_tokens
            for j in range(n):
                pool[probs[0]["bt"][b, j], :, :w.dl] = src["pool"][src["bt"][b, j], :, :w.dl]
        pools_np.append(pool)
    pools = [pl.to_device(p, dt) for p in pools_np]
    bt = torch.from_numpy(probs[0]["bt"]).to(dev)
    ln = torch.from_numpy(lens).to(dev)
    mp = probs[0]["max_pages"]
    rng = np.random.default_rng(4242)
    Wv = wl.to_storage(rng.standard_normal((w.H, w.d_c, w.d_v)) * 0.05, dt)
    Wv_d = pl.to_device(Wv, dt)
    # oracle: per-slice attention, then the up-projection and the sum over slices
    qp64 = wl.as_f64(probs[0]["q_pe"], dt)
    kpe = [r[:, w.dl:] for r in probs[0]["rows64"]]
    ref_lat, ref_lse = [], []
    for i in range(w.g):
        c = [r[:, :w.dl] for r in probs[i]["rows64"]]
        o_i, l_i = orc.shard_attention(wl.as_f64(probs[i]["q_lat"], dt), qp64, c, kpe, w.sm_scale)
        ref_lat.append(o_i); ref_lse.append(l_i)
    ref_lat = np.stack(ref_lat); ref_lse = np.stack(ref_lse)
    ref_o = orc.combine_shards(ref_lat, wl.as_f64(Wv, dt))
    nz = lens > 0
    for n_splits in splits:
        _say(f"decode_shards_combine {name} B={Bn} n_splits={n_splits}")
        ws_b = tp.tpla_workspace_bytes_all(shape, mp, n_splits)
        ws = torch.empty(ws_b, dtype=torch.uint8, device=dev)
        nan = float("nan")
        o = torch.full((Bn, w.H, w.d_v), nan, dtype=torch.float32, device=dev)
        o_lat = torch.full((w.g, Bn, w.H, w.dl), nan, dtype=torch.float32, device=dev)
        lse = torch.full((w.g, Bn, w.H), nan, dtype=torch.float32, device=dev)
        tp.tpla_decode_shards_combine(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, Wv_d, o, o_lat, lse)
        torch.cuda.synchronize()
        o_np, lat_np, lse_np = o.cpu().numpy(), o_lat.cpu().numpy(), lse.cpu().numpy()
        assert rel_err(lat_np, ref_lat) <= TOL[dt]
        assert rel_err(o_np, ref_o) <= TOL[dt]
        assert np.max(np.abs(lse_np[:, nz] - ref_lse[:, nz])) <= (1e-2 if dt == "bf16" else 1e-4)
        assert np.all(lat_np[:, ~nz] == 0) and np.all(np.isneginf(lse_np[:, ~nz])) and np.all(o_np[~nz] == 0)
        # the two separate calls: same partial results, the merge summed in another order
        o2 = torch.full_like(o, nan); o_lat2 = torch.full_like(o_lat, nan); lse2 = torch.full_like(lse, nan)
        tp.tpla_decode_shards(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, o_lat2, lse2)
        tp.tpla_combine_shards(shape, o_lat2, Wv_d, o2)
        torch.cuda.synchronize()
        assert rel_err(lat_np, o_lat2.cpu().numpy()) <= 1e-5
        assert rel_err(o_np, o2.cpu().numpy()) <= 1e-5
        assert np.max(np.abs(lse_np[:, nz] - lse2.cpu().numpy()[:, nz])) <= 1e-5
        # reproducible bits
        o3 = torch.full_like(o, nan); o_lat3 = torch.full_like(o_lat, nan)
        tp.tpla_decode_shards_combine(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, Wv_d, o3, o_lat3, None)
        torch.cuda.synchronize()
        assert torch.equal(o, o3) and torch.equal(o_lat, o_lat3)


# ------------------------------------------------------------ tiny config, whole path
def _full_problem(w):
    m = wl.draw_model_side(w)
    c64, k64, cs, ks = [], [], [], []
    for b in range(w.B):
        c, k = wl.draw_sequence(w, b, int(m["seq_lens"][b]), heavy=m["heavy"])
        cs.append(c); ks.append(k)
        c64.append(wl.as_f64(c, w.dtype)); k64.append(wl.as_f64(k, w.dtype))
    pool = wl.nan_fill((m["n_pool_pages"], w.page_tokens, w.d_c + w.d_r), w.dtype)
    for b in range(w.B):
        n = (int(m["seq_lens"][b]) + w.page_tokens - 1) // w.page_tokens
        wl.place_rows(pool, m["block_table"][b, :n], np.concatenate([cs[b], ks[b]], axis=1))
    return m, pool, c64, k64


def _run_full(w, m, mla_pool_np, mode, signs_np, U_np, mu, g=None):
    g = w.g if g is None else g
    wg = wl.scaled(w, g=g)
    shape = pl.make_shape(wg)
    dev = "cuda"
    W_UK = pl.to_device(m["W_UK"], w.dtype); W_UV = pl.to_device(m["W_UV"], w.dtype)
    q_nope = pl.to_device(m["q_nope"], w.dtype); q_pe = pl.to_device(m["q_pe"], w.dtype)
    signs = None if signs_np is None else torch.from_numpy(signs_np).to(dev)
    U = None if U_np is None else torch.from_numpy(np.ascontiguousarray(U_np, dtype=np.float32)).to(dev)
    W_UK_t, W_UV_t = pl.transform_weights(shape, mode, signs, U, W_UK, W_UV)
    mla_pool = pl.to_device(mla_pool_np, w.dtype)
    P = mla_pool.shape[0]
    pools = [torch.full((P, w.page_tokens, wg.dl + w.d_r), float("nan"), dtype=pl.torch_dtype(w.dtype), device=dev)
             for _ in range(g)]
    used = np.unique(np.concatenate([m["block_table"][b, :(int(m["seq_lens"][b]) + w.page_tokens - 1) // w.page_tokens]
                                     for b in range(w.B)])).astype(np.int32)
    page_ids = torch.from_numpy(used).to(dev)
    tp.tpla_transform_latent_paged(shape, mode, signs, U, mla_pool, pools, page_ids, len(used))
    step = pl.DecodeStep(shape, m["max_pages"])
    bt = torch.from_numpy(m["block_table"]).to(dev); lens = torch.from_numpy(m["seq_lens"]).to(dev)
    o = step.run(q_nope, q_pe, W_UK_t, W_UV_t, pools, bt, lens, mu)
    torch.cuda.synchronize()
    return {"o": o.cpu().numpy(), "O_lat": step.o_lat.cpu().numpy(), "lse": step.lse.cpu().numpy(),
            "Q_lat": wl.as_f64(pl.from_device_bits(step.q_lat), w.dtype)}


@pytest.mark.parametrize("mode", ["identity", "hadamard", "dense"])
def test_tiny_config_whole_path_fp32(mode):
    w = wl.CONFIGS["tiny"]
    _say(f"tiny config whole path, U={mode}")
    m, pool, c64, k64 = _full_problem(w)
    args = (wl.as_f64(m["q_nope"], "f32"), wl.as_f64(m["q_pe"], "f32"), wl.as_f64(m["W_UK"], "f32"),
            wl.as_f64(m["W_UV"], "f32"), c64, k64)
    if mode == "identity":
        U64, code, signs, Unp = None, tp.TPLA_U_IDENTITY, None, None
    elif mode == "hadamard":
        U64, code, signs, Unp = orc.hadamard_U(w.d_c, m["signs"]), tp.TPLA_U_HADAMARD, m["signs"], None
    else:
        q, r = np.linalg.qr(np.random.default_rng(5).standard_normal((w.d_c, w.d_c)))
        U64 = (q * np.sign(np.diag(r))).astype(np.float32).astype(np.float64)
        code, signs, Unp = tp.TPLA_U_DENSE, None, U64
    mu = [2.0, 2.0]
    ref = orc.tpla_decode(*args, 2, w.sm_scale, U=U64, mu=mu)
    got = _run_full(w, m, pool, code, signs, Unp, mu)
    for key in ("Q_lat", "O_lat", "o"):
        assert rel_err(got[key], ref[key]) <= TOL["f32"], key
    assert np.max(np.abs(got["lse"] - ref["lse"])) <= 1e-5
    # one slice: TPLA is MLA, whatever U is
    got1 = _run_full(w, m, pool, code, signs, Unp, None, g=1)
    mla = orc.mla_naive(*args, w.sm_scale)
    assert rel_err(got1["o"], mla) <= TOL["f32"]


# ------------------------------------------------------------ transform
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mode", ["hadamard", "dense", "identity"])
def test_transform_latent_weights(dtype, mode):
    _say(f"transform_latent {dtype} {mode}")
    d_c, H, d_n, d_v = 128, 3, 8, 24
    rng = np.random.default_rng(21)
    shape = tp.TplaShape(1, H, d_c, 2, 16, d_n, d_v, 64, tp.TPLA_F32 if dtype == "f32" else tp.TPLA_BF16, 1.0)
    W_UK = wl.to_storage(rng.standard_normal((H, d_n, d_c)), dtype)
    W_UV = wl.to_storage(rng.standard_normal((H, d_c, d_v)), dtype)
    signs_np = rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d_c)
    if mode == "hadamard":
        U64, code, signs, U = orc.hadamard_U(d_c, signs_np), tp.TPLA_U_HADAMARD, torch.from_numpy(signs_np).cuda(), None
    elif mode == "dense":
        q, r = np.linalg.qr(rng.standard_normal((d_c, d_c)))
        U64 = (q * np.sign(np.diag(r))).astype(np.float32).astype(np.float64)
        code, signs, U = tp.TPLA_U_DENSE, None, torch.from_numpy(U64.astype(np.float32)).cuda()
    else:
        U64, code, signs, U = np.eye(d_c), tp.TPLA_U_IDENTITY, None, None
    a, b = pl.transform_weights(shape, code, signs, U, pl.to_device(W_UK, dtype), pl.to_device(W_UV, dtype))
    ra, rb = orc.reparameterize_weights(wl.as_f64(W_UK, dtype), wl.as_f64(W_UV, dtype), U64)
    ga = wl.as_f64(pl.from_device_bits(a), dtype); gb = wl.as_f64(pl.from_device_bits(b), dtype)
    if mode == "identity":
        assert np.array_equal(ga, ra) and np.array_equal(gb, rb)
    else:
        tol = 1e-5 if dtype == "f32" else 2.0 ** -8
        assert rel_err(ga, ra) <= tol and rel_err(gb, rb) <= tol
    # inverse undoes the transform (U U^T = I)
    back = torch.empty_like(a)
    tp.tpla_transform_latent(shape, code, 1, signs, U, a, back, H * d_n, 1)
    torch.cuda.synchronize()
    assert rel_err(wl.as_f64(pl.from_device_bits(back), dtype), wl.as_f64(W_UK, dtype)) <= (1e-5 if dtype == "f32" else 2e-2)


@pytest.mark.parametrize("dtype,d_c,g,d_r,pt", [
    ("bf16", 512, 2, 64, 64), ("bf16", 512, 4, 64, 64), ("f32", 64, 2, 16, 64), ("bf16", 96, 2, 16, 64),
    # matrix-core Hadamard pass: narrow slices, short / odd-sized pages, other RoPE widths, d_c = 256;
    # then shapes it declines (d_c = 1024, pages of 6 tokens, float storage at d_c = 512)
    ("bf16", 512, 8, 128, 16), ("bf16", 512, 1, 32, 20), ("bf16", 256, 2, 64, 128), ("bf16", 256, 4, 8, 4),
    ("bf16", 128, 2, 64, 64), ("bf16", 128, 1, 16, 192),
    ("bf16", 1024, 2, 64, 16), ("bf16", 512, 2, 64, 6), ("f32", 512, 2, 64, 16)])
def test_transform_latent_paged(dtype, d_c, g, d_r, pt):
    _say(f"transform_latent_paged {dtype} d_c={d_c} g={g} d_r={d_r} page_tokens={pt}")
    P = 7
    rng = np.random.default_rng(31)
    shape = tp.TplaShape(1, 16, d_c, g, d_r, 8, 8, pt, tp.TPLA_F32 if dtype == "f32" else tp.TPLA_BF16, 1.0)
    pool_np = wl.to_storage(rng.standard_normal((P, pt, d_c + d_r)), dtype)
    pool = pl.to_device(pool_np, dtype)
    ids_np = np.array([5, 0, 3], dtype=np.int32)
    ids = torch.from_numpy(ids_np).cuda()
    dl = d_c // g
    pow2 = (d_c & (d_c - 1)) == 0
    modes = [("identity", tp.TPLA_U_IDENTITY, None, None)]
    if pow2:
        modes.append(("hadamard", tp.TPLA_U_HADAMARD, rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d_c), None))
        modes.append(("hadamard", tp.TPLA_U_HADAMARD, None, None))       # no sign diagonal
    # dense orthogonal U (the PCA case): a random rotation, given in float
    modes.append(("dense", tp.TPLA_U_DENSE, None, np.linalg.qr(rng.standard_normal((d_c, d_c)))[0].astype(np.float32)))
    for name, code, signs_np, U_np in modes:
        outs = [torch.zeros((P, pt, dl + d_r), dtype=pl.torch_dtype(dtype), device="cuda") for _ in range(g)]
        signs = None if signs_np is None else torch.from_numpy(signs_np).cuda()
        U_dev = None if U_np is None else torch.from_numpy(U_np).cuda()
        tp.tpla_transform_latent_paged(shape, code, signs, U_dev, pool, outs, ids, len(ids_np))
        torch.cuda.synchronize()
        src64 = wl.as_f64(pool_np, dtype)
        if name == "identity":
            U64 = np.eye(d_c)
        elif name == "hadamard":
            U64 = orc.hadamard_U(d_c, signs_np)
        else:
            U64 = U_np.astype(np.float64)
        for i in range(g):
            got_bits = pl.from_device_bits(outs[i])
            got = wl.as_f64(got_bits, dtype)
            untouched = np.setdiff1d(np.arange(P), ids_np)
            assert np.all(got[untouched] == 0)                                  # only listed pages are written
            assert np.array_equal(got_bits[ids_np][:, :, dl:], pool_np[ids_np][:, :, d_c:])   # k_pe copied bit-exactly
            ref = orc.transform_latent(src64[ids_np][:, :, :d_c], U64)[:, :, i * dl:(i + 1) * dl]
            lat = got[ids_np][:, :, :dl]
            if name == "identity":
                assert np.array_equal(lat, ref)
            elif dtype == "f32":
                assert rel_err(lat, ref) <= 1e-5
            else:
                rr = orc.round_to_bf16(ref)
                diff = lat != rr
                if name == "dense":
                    # U's float entries enter the matrix cores as bf16 hi + lo: every product carries a
                    # relative 2^-17, so the float sum is within 2^-16 sum_k |x_k U_kj| of the exact one
                    # (accumulation included), and the stored value within half a bf16 step of that.
                    slack = (np.abs(src64[ids_np][:, :, :d_c]) @ np.abs(U64))[:, :, i * dl:(i + 1) * dl] * 2.0 ** -16
                    mag = np.maximum(np.maximum(np.abs(rr), np.abs(ref)), 1e-300)
                    half_step = 2.0 ** (np.floor(np.log2(mag)) - 8)
                    assert np.all(np.abs(lat - ref) <= half_step + slack)
                    assert diff.mean() <= 3e-2
                else:
                    # one rounding of the float64 result; float butterflies may land on
                    # the other side of a tie for a tiny fraction of elements (1 ulp)
                    assert diff.mean() <= 1e-3
                    assert np.all(np.abs(lat - rr)[diff] <= np.abs(rr[diff]) * 2.0 ** -7 + 1e-30)


def test_write_mla_cache():
    _say("write_mla_cache")
    for dtype in ("f32", "bf16"):
        d_c, d_r, pt, P, T = 512, 64, 64, 5, 150
        rng = np.random.default_rng(41)
        shape = tp.TplaShape(1, 16, d_c, 2, d_r, 8, 8, pt, tp.TPLA_F32 if dtype == "f32" else tp.TPLA_BF16, 1.0)
        c = wl.to_storage(rng.standard_normal((T, d_c)) * np.exp(rng.uniform(-2, 2, size=(T, 1))), dtype)
        k = wl.to_storage(rng.standard_normal((T, d_r)), dtype)
        slots_np = rng.permutation(P * pt)[:T].astype(np.int32)
        slots_np[7] = -1                                     # skipped token
        pool = torch.zeros((P, pt, d_c + d_r), dtype=pl.torch_dtype(dtype), device="cuda")
        for eps in (1e-6, -1.0):
            pool.zero_()
            tp.tpla_write_mla_cache(shape, pl.to_device(c, dtype), pl.to_device(k, dtype),
                                    torch.from_numpy(slots_np).cuda(), T, eps, pool)
            torch.cuda.synchronize()
            got = wl.as_f64(pl.from_device_bits(pool), dtype).reshape(P * pt, d_c + d_r)
            c64, k64 = wl.as_f64(c, dtype), wl.as_f64(k, dtype)
            ref = orc.mla_cache_rows(c64, k64, eps) if eps >= 0 else np.concatenate([c64, k64], axis=1)
            keep = slots_np >= 0
            assert np.array_equal(got[slots_np[keep]][:, d_c:], ref[keep][:, d_c:])
            tol = 1e-6 if dtype == "f32" else 2.0 ** -8
            assert np.all(np.abs(got[slots_np[keep]][:, :d_c] - ref[keep][:, :d_c]) <= tol * np.abs(ref[keep][:, :d_c]) + 1e-30)
            written = np.zeros(P * pt, dtype=bool); written[slots_np[keep]] = True
            assert np.all(got[~written] == 0)


def test_append_token_sliced():
    _say("append_token_sliced")
    for dtype, d_c, g, d_r in (("bf16", 512, 2, 64), ("bf16", 512, 4, 64), ("f32", 64, 2, 16)):
        Bn, pt, P = 9, 64, 4
        rng = np.random.default_rng(61)
        shape = tp.TplaShape(Bn, 16, d_c, g, d_r, 8, 8, pt, tp.TPLA_F32 if dtype == "f32" else tp.TPLA_BF16, 1.0)
        c = wl.to_storage(rng.standard_normal((Bn, d_c)) * np.exp(rng.uniform(-2, 2, size=(Bn, 1))), dtype)
        k = wl.to_storage(rng.standard_normal((Bn, d_r)), dtype)
        slots_np = rng.permutation(P * pt)[:Bn].astype(np.int32)
        slots_np[3] = -1
        dl = d_c // g
        for alpha in (None, list(rng.uniform(1.0, 3.0, size=g))):
            pools = [torch.zeros((P, pt, dl + d_r), dtype=pl.torch_dtype(dtype), device="cuda") for _ in range(g)]
            tp.tpla_append_token_sliced(shape, pl.to_device(c, dtype), pl.to_device(k, dtype), alpha, 1e-6,
                                        torch.from_numpy(slots_np).cuda(), pools)
            torch.cuda.synchronize()
            a64 = None if alpha is None else np.asarray(alpha, dtype=np.float32).astype(np.float64)
            ref = orc.sliced_rms_rows(wl.as_f64(c, dtype), wl.as_f64(k, dtype), g, a64, 1e-6)
            keep = slots_np >= 0
            for i in range(g):
                got = wl.as_f64(pl.from_device_bits(pools[i]), dtype).reshape(P * pt, dl + d_r)
                assert np.array_equal(got[slots_np[keep]][:, dl:], ref[i][keep][:, dl:])       # k_pe bit-exact
                tol = 1e-6 if dtype == "f32" else 2.0 ** -8
                lat, r = got[slots_np[keep]][:, :dl], ref[i][keep][:, :dl]
                assert np.all(np.abs(lat - r) <= tol * np.abs(r) + 1e-30)
                written = np.zeros(P * pt, dtype=bool); written[slots_np[keep]] = True
                assert np.all(got[~written] == 0)


# ------------------------------------------------------------ absorb / combine
@pytest.mark.parametrize("dtype,Bn,H,g", [("bf16", 5, 64, 2), ("bf16", 17, 32, 4), ("f32", 3, 4, 2),
                                          # batches whose blocks of 16 sequences are dealt over 2, 5 and 8 workgroups
                                          # per (head, column block) of the absorb kernel, ragged last block
                                          ("bf16", 37, 16, 2), ("bf16", 130, 16, 1), ("bf16", 300, 16, 4)])
def test_absorb_and_combine(dtype, Bn, H, g):
    _say(f"absorb/combine {dtype} B={Bn} H={H} g={g}")
    d_c, d_n, d_v, d_r = (512, 128, 128, 64) if dtype == "bf16" else (64, 32, 32, 16)
    rng = np.random.default_rng(51)
    shape = tp.TplaShape(Bn, H, d_c, g, d_r, d_n, d_v, 64, tp.TPLA_F32 if dtype == "f32" else tp.TPLA_BF16, 1.0)
    q = wl.to_storage(rng.standard_normal((Bn, H, d_n)), dtype)
    Wk = wl.to_storage(rng.standard_normal((H, d_n, d_c)) * 0.05, dtype)
    Wv = wl.to_storage(rng.standard_normal((H, d_c, d_v)) * 0.05, dtype)
    mu = list(rng.uniform(0.5, 2.5, size=g))
    dl = d_c // g
    q_lat = torch.empty((g, Bn, H, dl), dtype=pl.torch_dtype(dtype), device="cuda")
    tp.tpla_absorb_query(shape, pl.to_device(q, dtype), pl.to_device(Wk, dtype), mu, q_lat)
    ref = orc.absorb_query(wl.as_f64(q, dtype), wl.as_f64(Wk, dtype), g, np.asarray(mu, dtype=np.float32).astype(np.float64))
    torch.cuda.synchronize()
    assert rel_err(wl.as_f64(pl.from_device_bits(q_lat), dtype), ref) <= (1e-5 if dtype == "f32" else 2.0 ** -8)
    o_lat_np = rng.standard_normal((g, Bn, H, dl)).astype(np.float32)
    o = torch.empty((Bn, H, d_v), dtype=torch.float32, device="cuda")
    tp.tpla_combine_shards(shape, torch.from_numpy(o_lat_np).cuda(), pl.to_device(Wv, dtype), o)
    torch.cuda.synchronize()
    assert rel_err(o.cpu().numpy(), orc.combine_shards(o_lat_np.astype(np.float64), wl.as_f64(Wv, dtype))) <= 1e-5


@pytest.mark.parametrize("dtype,Bn,H,d_v,D", [("bf16", 32, 64, 128, 7168), ("bf16", 5, 32, 128, 1024), ("bf16", 40, 16, 64, 320),
                                              ("f32", 3, 4, 32, 96), ("bf16", 2, 5, 16, 100),
                                              # matrix-core path: three passes over the batch; 32, 3 and 6 chunks per k-range
                                              ("bf16", 70, 64, 128, 7168), ("bf16", 33, 24, 128, 2048), ("bf16", 8, 24, 128, 4096),
                                              ("bf16", 4, 2, 64, 4096)])     # one chunk per k-range
def test_output_projection(dtype, Bn, H, d_v, D):
    _say(f"output_projection {dtype} B={Bn} H={H} d_v={d_v} D={D}")
    rng = np.random.default_rng(71)
    shape = tp.TplaShape(Bn, H, 64, 2, 16, 8, d_v, 64, tp.TPLA_F32 if dtype == "f32" else tp.TPLA_BF16, 1.0)
    o_np = rng.standard_normal((Bn, H, d_v)).astype(np.float32)
    W = wl.to_storage(rng.standard_normal((H * d_v, D)) * 0.02, dtype)
    ws_b = tp.tpla_output_projection_workspace_bytes(shape, D)
    ws = torch.empty(max(ws_b, 16), dtype=torch.uint8, device="cuda")
    out = torch.full((Bn, D), float("nan"), dtype=torch.float32, device="cuda")
    tp.tpla_output_projection(shape, torch.from_numpy(o_np).cuda(), pl.to_device(W, dtype), D, ws, ws_b, out)
    torch.cuda.synchronize()
    ref = orc.output_projection(o_np.astype(np.float64), wl.as_f64(W, dtype))
    assert rel_err(out.cpu().numpy(), ref) <= 1e-5


ATTN_BLOCK_CASES = [
    ("dsv3_ragged", DSV3, [700, 64, 0, 1500, 129], 1024, (0, 3)),
    ("g4_hadamard_shape", wl.scaled(wl.CONFIGS["ragged_g4"], H=16), [300, 65], 512, (0,)),
    ("generic_f32", wl.Workload("odd", B=3, H=5, d_c=80, g=2, d_r=24, d_n=16, d_v=16, dtype="f32", seed=11), [200, 0, 65], 96, (0, 2)),
]


@pytest.mark.parametrize("name,w,lens,D,splits", ATTN_BLOCK_CASES, ids=[c[0] for c in ATTN_BLOCK_CASES])
def test_decode_shards_project_matches_oracle_in_float_and_bf16(name, w, lens, D, splits):
    """The attention block's output in one call (decode of all slices, merge, value up-projection and
    sum over slices, then W_O) against the oracle's combine_shards + output_projection, with float
    and with bfloat16 outputs, and bit for bit against the separate calls."""
    lens = np.asarray(lens, dtype=np.int32)
    Bn = len(lens)
    w = wl.scaled(w, B=Bn)
    dt = w.dtype
    probs = [build_shard_problem(w, lens, rng_extra=i) for i in range(w.g)]
    shape = pl.make_shape(w)
    dev = "cuda"
    q_lat = pl.to_device(np.stack([p["q_lat"] for p in probs]), dt)
    q_pe = pl.to_device(probs[0]["q_pe"], dt)
    pools = []
    for i in range(w.g):
        pool = probs[0]["pool"].copy()
        for b in range(Bn):
            for j in range((int(lens[b]) + w.page_tokens - 1) // w.page_tokens):
                pool[probs[0]["bt"][b, j], :, :w.dl] = probs[i]["pool"][probs[i]["bt"][b, j], :, :w.dl]
        pools.append(pl.to_device(pool, dt))
    bt = torch.from_numpy(probs[0]["bt"]).to(dev)
    ln = torch.from_numpy(lens).to(dev)
    mp = probs[0]["max_pages"]
    rng = np.random.default_rng(977)
    Wv = wl.to_storage(rng.standard_normal((w.H, w.d_c, w.d_v)) * 0.05, dt)
    Wo = wl.to_storage(rng.standard_normal((w.H * w.d_v, D)) * 0.05, dt)
    Wv_d, Wo_d = pl.to_device(Wv, dt), pl.to_device(Wo, dt)
    kpe = [r[:, w.dl:] for r in probs[0]["rows64"]]
    ref_lat = np.stack([orc.shard_attention(wl.as_f64(probs[i]["q_lat"], dt), wl.as_f64(probs[0]["q_pe"], dt),
                                            [r[:, :w.dl] for r in probs[i]["rows64"]], kpe, w.sm_scale)[0] for i in range(w.g)])
    ref_o = orc.combine_shards(ref_lat, wl.as_f64(Wv, dt))
    ref_out = orc.output_projection(ref_o, wl.as_f64(Wo, dt))
    nan = float("nan")
    for n_splits in splits:
        _say(f"decode_shards_project {name} B={Bn} D={D} n_splits={n_splits}")
        ws_b = tp.tpla_attention_block_workspace_bytes(shape, mp, n_splits, D)
        assert ws_b >= tp.tpla_workspace_bytes_all(shape, mp, n_splits) and ws_b >= tp.tpla_output_projection_workspace_bytes(shape, D)
        ws = torch.empty(ws_b, dtype=torch.uint8, device=dev)
        o = torch.full((Bn, w.H, w.d_v), nan, dtype=torch.float32, device=dev)
        o_lat = torch.full((w.g, Bn, w.H, w.dl), nan, dtype=torch.float32, device=dev)
        out32 = torch.full((Bn, D), nan, dtype=torch.float32, device=dev)
        out16 = torch.full((Bn, D), nan, dtype=torch.bfloat16, device=dev)
        tp.tpla_decode_shards_project(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, Wv_d, Wo_d, D,
                                      out32, tp.TPLA_F32, o, o_lat, None)
        tp.tpla_decode_shards_project(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, Wv_d, Wo_d, D,
                                      out16, tp.TPLA_BF16, o, o_lat, None)
        torch.cuda.synchronize()
        assert rel_err(o.cpu().numpy(), ref_o) <= TOL[dt]
        assert rel_err(out32.cpu().numpy(), ref_out) <= TOL[dt]
        # bfloat16 output: one rounding (2^-9 relative) on top
        got16 = wl.as_f64(pl.from_device_bits(out16), "bf16")
        assert rel_err(got16, ref_out) <= max(TOL[dt], 2.0 ** -8)
        assert np.array_equal(pl.from_device_bits(out16), wl.f32_to_bf16_bits(out32.cpu().numpy()))
        # the separate calls give the same bits
        o2 = torch.full_like(o, nan); o_lat2 = torch.full_like(o_lat, nan); out2 = torch.full_like(out32, nan)
        tp.tpla_decode_shards_combine(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, Wv_d, o2, o_lat2, None)
        tp.tpla_output_projection(shape, o2, Wo_d, D, ws, ws_b, out2)
        torch.cuda.synchronize()
        assert torch.equal(out2, out32) and torch.equal(o2, o)
        # o itself as bfloat16 from the fused decode + combine call and from the combine alone
        ob = torch.full((Bn, w.H, w.d_v), nan, dtype=torch.bfloat16, device=dev)
        tp.tpla_decode_shards_combine_to(shape, q_lat, q_pe, pools, bt, mp, ln, n_splits, ws, ws_b, Wv_d, ob, tp.TPLA_BF16,
                                         o_lat2, None)
        oc = torch.full_like(ob, nan)
        tp.tpla_combine_shards_to(shape, o_lat, Wv_d, oc, tp.TPLA_BF16)
        of = torch.full_like(o, nan)
        tp.tpla_combine_shards(shape, o_lat, Wv_d, of)
        torch.cuda.synchronize()
        assert np.array_equal(pl.from_device_bits(ob), wl.f32_to_bf16_bits(o.cpu().numpy()))
        assert np.array_equal(pl.from_device_bits(oc), wl.f32_to_bf16_bits(of.cpu().numpy()))
        assert rel_err(wl.as_f64(pl.from_device_bits(oc), "bf16"), ref_o) <= max(TOL[dt], 2.0 ** -8)


def test_layer_step_as_hip_graph_replays_like_eager():
    """The step captured in a HIP graph: several replays, eager work and synchronisations between
    them, new inputs written into the same tensors; every replay equals the eager result bit for bit."""
    _say("layer step as HIP graph")
    w = wl.scaled(wl.CONFIGS["dsv3_4k"], B=3, H=16, context=0)
    lens = [200, 64, 1000]
    dev = "cuda"
    rng = np.random.default_rng(5)
    shape = pl.make_shape(w)
    pages = (np.asarray(lens) + 63) // 64
    P = int(pages.sum())
    bt = np.zeros((w.B, int(pages.max())), dtype=np.int32); k = 0
    for b in range(w.B):
        bt[b, :pages[b]] = np.arange(k, k + pages[b]); k += pages[b]
    pools = [torch.randn((P, 64, w.dl + w.d_r), device=dev).to(torch.bfloat16) for _ in range(w.g)]
    W_UK_t = (torch.randn((w.H, w.d_n, w.d_c), device=dev) * 0.02).to(torch.bfloat16)
    W_UV_t = (torch.randn((w.H, w.d_c, w.d_v), device=dev) * 0.02).to(torch.bfloat16)
    q_nope = torch.randn((w.B, w.H, w.d_n), device=dev).to(torch.bfloat16)
    q_pe = torch.randn((w.B, w.H, w.d_r), device=dev).to(torch.bfloat16)
    bt_t, lens_t = torch.from_numpy(bt).to(dev), torch.tensor(lens, dtype=torch.int32, device=dev)
    mu = [2.0, 2.0]
    step = pl.DecodeStep(shape, int(pages.max()))
    graph = step.capture(q_nope, q_pe, W_UK_t, W_UV_t, pools, bt_t, lens_t, mu)
    eager = pl.DecodeStep(shape, int(pages.max()))
    for it in range(4):
        if it:      # new queries and a shorter third sequence, written into the captured tensors
            q_nope.copy_(torch.randn_like(q_nope, dtype=torch.float32).to(torch.bfloat16))
            q_pe.copy_(torch.randn_like(q_pe, dtype=torch.float32).to(torch.bfloat16))
            lens_t.copy_(torch.tensor([200, 64, 1000 - 100 * it], dtype=torch.int32))
        ref = eager.run(q_nope, q_pe, W_UK_t, W_UV_t, pools, bt_t, lens_t, mu).clone()
        torch.cuda.synchronize()
        step.o.fill_(float("nan")); step.o_lat.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(step.o, ref), it
        assert torch.equal(step.o_lat, eager.o_lat) and torch.equal(step.lse, eager.lse)


# ------------------------------------------------------------ PCA calibration (Sec. 4.3.2)
@pytest.mark.parametrize("dtype,d_c,d_r,pt,P", [("bf16", 512, 64, 64, 40), ("bf16", 256, 64, 16, 9), ("bf16", 128, 8, 64, 3),
                                                ("bf16", 1024, 64, 32, 6), ("bf16", 384, 64, 64, 5),
                                                ("bf16", 96, 16, 8, 5), ("f32", 64, 16, 64, 4)])
def test_latent_moments(dtype, d_c, d_r, pt, P):
    _say(f"latent_moments {dtype} d_c={d_c} d_r={d_r} page_tokens={pt} pages={P}")
    rng = np.random.default_rng(91)
    shape = tp.TplaShape(1, 16, d_c, 1, d_r, 8, 8, pt, tp.TPLA_F32 if dtype == "f32" else tp.TPLA_BF16, 1.0)
    F = wl.draw_anisotropic_latents(d_c, P * pt, d_c)
    rows = wl.to_storage(np.concatenate([F, rng.standard_normal((P * pt, d_r)).astype(np.float32)], axis=1), dtype)
    # listed pages in a shuffled order inside a larger pool; partly filled, one empty; the rest is NaN
    n_pool = P + 3
    ids_np = rng.permutation(n_pool)[:P].astype(np.int32)
    fill_np = rng.integers(1, pt + 1, size=P).astype(np.int32)
    fill_np[0] = pt
    if P > 2:
        fill_np[1] = 0
    pool_np = wl.nan_fill((n_pool, pt, d_c + d_r), dtype)
    valid = []
    for k in range(P):
        pool_np[ids_np[k], :fill_np[k]] = rows[k * pt:k * pt + fill_np[k]]
        valid.append(rows[k * pt:k * pt + fill_np[k], :d_c])
    ref_s, ref_G = orc.latent_moments(wl.as_f64(np.concatenate(valid), dtype))
    pool = pl.to_device(pool_np, dtype)
    ws_b = tp.tpla_latent_moments_workspace_bytes(shape, P)
    for fill in (fill_np, None):
        ws = torch.full((ws_b,), 0xFF, dtype=torch.uint8, device="cuda")
        s = torch.full((d_c,), float("nan"), dtype=torch.float64, device="cuda")
        G = torch.full((d_c, d_c), float("nan"), dtype=torch.float64, device="cuda")
        if fill is None:       # every page full: a pool without NaNs, all rows count
            full_np = wl.to_storage(rng.standard_normal((n_pool, pt, d_c + d_r)), dtype)
            pool = pl.to_device(full_np, dtype)
            ref_s, ref_G = orc.latent_moments(wl.as_f64(full_np[ids_np][:, :, :d_c].reshape(-1, d_c), dtype))
        tp.tpla_latent_moments(shape, pool, torch.from_numpy(ids_np).cuda(),
                               None if fill is None else torch.from_numpy(fill).cuda(), P, ws, ws_b, s, G)
        torch.cuda.synchronize()
        s, G = s.cpu().numpy(), G.cpu().numpy()
        assert np.array_equal(G, G.T)
        assert rel_err(G, ref_G) <= 1e-5 and rel_err(s, ref_s) <= 1e-5
    with pytest.raises(tp.TplaError):
        tp.tpla_latent_moments(shape, pool, None, None, P, ws, ws_b - 16, torch.empty(d_c, dtype=torch.float64, device="cuda"),
                               torch.empty((d_c, d_c), dtype=torch.float64, device="cuda"))


def test_pca_whole_path_bf16():
    """Cache written in MLA form -> PCA basis from the cached latents (GPU moments + host
    eigen-solver) -> weights and cache turned into that basis -> TPLA decode, against the
    oracle doing the same from its own eigen-decomposition.  Eigenvectors are unique up to
    sign only; every compared quantity is invariant to those signs."""
    _say("pca whole path bf16")
    w = wl.scaled(wl.CONFIGS["dsv3_4k"], B=3, H=16, d_c=256, g=2, context=0, seed=17)
    lens = [700, 90, 333]
    pt, dev = 64, "cuda"
    m = wl.draw_model_side(wl.scaled(w, context=max(lens)))
    pages = (np.asarray(lens) + pt - 1) // pt
    P = int(pages.sum()) + 2
    order = np.random.default_rng([w.seed, 5]).permutation(P)
    bt = np.zeros((w.B, int(pages.max())), dtype=np.int32); k = 0
    for b in range(w.B):
        bt[b, :pages[b]] = order[k:k + pages[b]]; k += pages[b]
    shape = pl.make_shape(w)
    F = wl.draw_anisotropic_latents(w.seed, sum(lens), w.d_c, decay=4.0)
    c64, k64, used, fill = [], [], [], []
    mla_pool = torch.full((P, pt, w.d_c + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev)
    t0 = 0
    for b in range(w.B):
        _, kp = wl.draw_sequence(w, b, lens[b])
        c = wl.to_storage(F[t0:t0 + lens[b]], "bf16"); t0 += lens[b]
        slots = torch.from_numpy(wl.slot_mapping(bt[b, :pages[b]], lens[b], pt)).to(dev)
        tp.tpla_write_mla_cache(shape, pl.to_device(c, "bf16"), pl.to_device(kp, "bf16"), slots, lens[b], -1.0, mla_pool)
        c64.append(wl.as_f64(c, "bf16")); k64.append(wl.as_f64(kp, "bf16"))
        used += list(bt[b, :pages[b]])
        fill += [pt] * (pages[b] - 1) + [lens[b] - pt * (pages[b] - 1)]
    used_t = torch.tensor(used, dtype=torch.int32, device=dev)
    U, eig, frac = pl.pca_calibrate(shape, mla_pool, used_t, torch.tensor(fill, dtype=torch.int32, device=dev), sum(lens))
    U_ref, lam = orc.pca_U(np.concatenate(c64))
    assert np.max(np.abs(eig - lam)) <= 1e-5 * lam[0]
    assert np.allclose(frac, orc.variance_fractions(lam, w.g), rtol=1e-5)
    assert np.max(np.abs(np.abs(U.cpu().numpy().astype(np.float64).T @ U_ref) - np.eye(w.d_c))) <= 2e-3
    mu = [1.0 / f for f in frac]                       # score factors from the variance shares
    mu_ref = list(orc.default_mu(w.g, lam))
    W_UK_t, W_UV_t = pl.transform_weights(shape, tp.TPLA_U_DENSE, None, U, pl.to_device(m["W_UK"], "bf16"), pl.to_device(m["W_UV"], "bf16"))
    pools = [torch.full((P, pt, w.dl + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev) for _ in range(w.g)]
    tp.tpla_transform_latent_paged(shape, tp.TPLA_U_DENSE, None, U, mla_pool, pools, used_t, len(used))
    step = pl.DecodeStep(shape, int(pages.max()))
    o = step.run(pl.to_device(m["q_nope"], "bf16"), pl.to_device(m["q_pe"], "bf16"), W_UK_t, W_UV_t, pools,
                 torch.from_numpy(bt).to(dev), torch.tensor(lens, dtype=torch.int32, device=dev), mu)
    torch.cuda.synchronize()
    ref = orc.tpla_decode(wl.as_f64(m["q_nope"], "bf16"), wl.as_f64(m["q_pe"], "bf16"), wl.as_f64(m["W_UK"], "bf16"),
                          wl.as_f64(m["W_UV"], "bf16"), c64, k64, w.g, w.sm_scale, U=U_ref, mu=mu_ref)
    assert rel_err(o.cpu().numpy(), ref["o"]) <= TOL["bf16"]
    # lse: absolute 1e-2 as everywhere, plus what the score factors add here: mu_i = 1 / share_i reaches
    # ~55 on the low-variance slice and multiplies the bf16 rounding of q_lat and of the stored cache (and
    # the 2e-3 the two eigen-decompositions may differ by) into the scores
    lse_err = float(np.max(np.abs(step.lse.cpu().numpy() - ref["lse"])))
    print("  lse err %.3g, mu %s" % (lse_err, ["%.3g" % x for x in mu]), flush=True)
    assert lse_err <= 1e-2 + 5e-4 * max(mu)
    # sign-invariant view of the latent-space tensors
    assert rel_err(np.abs(step.o_lat.cpu().numpy()), np.abs(ref["O_lat"])) <= TOL["bf16"]


# ------------------------------------------------------------ prefill (un-absorbed MLA, causal, packed)
def _prefill_problem(seed, lens, H, d_c):
    rng = np.random.default_rng([seed, 41])
    T = int(sum(lens))
    q_nope = wl.to_storage(rng.standard_normal((T, H, 128)), "bf16")
    q_pe = wl.to_storage(rng.standard_normal((T, H, 64)), "bf16")
    c = wl.to_storage(rng.standard_normal((T, d_c)), "bf16")
    k_pe = wl.to_storage(rng.standard_normal((T, 64)), "bf16")
    W_UK = wl.to_storage(rng.standard_normal((H, 128, d_c)) * 0.02, "bf16")
    W_UV = wl.to_storage(rng.standard_normal((H, d_c, 128)) * 0.02, "bf16")
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return {"q_nope": q_nope, "q_pe": q_pe, "c": c, "k_pe": k_pe, "W_UK": W_UK, "W_UV": W_UV, "cu": cu, "T": T}


def _run_prefill(p, H, d_c, B, max_len):
    shape = tp.TplaShape(B, H, d_c, 1, 64, 128, 128, 64, tp.TPLA_BF16, 1.0 / np.sqrt(192.0))
    ws_b = tp.tpla_prefill_workspace_bytes(shape, p["T"])
    ws = torch.full((ws_b,), 0xFF, dtype=torch.uint8, device="cuda")
    o = torch.full((p["T"], H, 128), float("nan"), dtype=torch.float32, device="cuda")
    dev = {k: pl.to_device(p[k], "bf16") for k in ("q_nope", "q_pe", "c", "k_pe", "W_UK", "W_UV")}
    tp.tpla_prefill_attention(shape, dev["q_nope"], dev["q_pe"], dev["c"], dev["k_pe"], dev["W_UK"], dev["W_UV"],
                              torch.from_numpy(p["cu"]).cuda(), p["T"], max_len, ws, ws_b, o)
    torch.cuda.synchronize()
    return o.cpu().numpy(), shape


@pytest.mark.parametrize("lens,H,d_c", [([1], 1, 128), ([37, 1, 128, 0, 300, 129], 4, 512), ([700], 3, 256),
                                        ([31, 32, 33, 127, 128, 129, 255, 257], 2, 512)])
def test_prefill_attention_matches_oracle(lens, H, d_c):
    _say(f"prefill_attention lens={lens} H={H} d_c={d_c}")
    p = _prefill_problem(len(lens) * 100 + H, lens, H, d_c)
    f64 = {k: wl.as_f64(p[k], "bf16") for k in ("q_nope", "q_pe", "c", "k_pe", "W_UK", "W_UV")}
    ref = orc.mla_prefill(f64["q_nope"], f64["q_pe"], f64["W_UK"], f64["W_UV"], f64["c"], f64["k_pe"], p["cu"],
                          1.0 / np.sqrt(192.0))
    for max_len in (max(lens), max(lens) + 200):            # a loose bound only adds idle workgroups
        o, _ = _run_prefill(p, H, d_c, len(lens), max_len)
        assert np.all(np.isfinite(o))                        # every row written, nothing leaks from the padding
        assert rel_err(o, ref) <= TOL["bf16"]
        # per-token check as well: early tokens have few keys and large outputs, late ones small
        den = np.max(np.abs(ref), axis=(1, 2), keepdims=True)
        assert np.max(np.abs(o - ref) / den) <= 2e-2


def test_prefill_attention_random_shapes():
    """Seeded random batches over the supported widths and odd head counts (groups of 8, 4, 2, 1 heads)."""
    rng = np.random.default_rng(2025)
    for trial, (H, d_c) in enumerate([(8, 384), (24, 128), (5, 512), (6, 256), (16, 384)]):
        B = int(rng.integers(1, 5))
        lens = [int(x) for x in rng.integers(0, 400, size=B)]
        if sum(lens) == 0:
            lens[0] = 17
        _say(f"prefill random trial {trial}: H={H} d_c={d_c} lens={lens}")
        p = _prefill_problem(1000 + trial, lens, H, d_c)
        f64 = {k: wl.as_f64(p[k], "bf16") for k in ("q_nope", "q_pe", "c", "k_pe", "W_UK", "W_UV")}
        ref = orc.mla_prefill(f64["q_nope"], f64["q_pe"], f64["W_UK"], f64["W_UV"], f64["c"], f64["k_pe"], p["cu"],
                              1.0 / np.sqrt(192.0))
        o, _ = _run_prefill(p, H, d_c, B, max(lens))
        assert np.all(np.isfinite(o)) and rel_err(o, ref) <= TOL["bf16"]


def test_prefill_attention_rejects_what_it_does_not_implement():
    p = _prefill_problem(1, [8], 1, 128)
    A = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    for kw in ({"d_n": 64}, {"d_r": 32}, {"dtype": tp.TPLA_F32}, {"d_c": 1024}):
        f = dict(B=1, H=1, d_c=128, g=1, d_r=64, d_n=128, d_v=128, page_tokens=64, dtype=tp.TPLA_BF16, sm_scale=0.1)
        f.update(kw)
        shape = tp.TplaShape(f["B"], f["H"], f["d_c"], f["g"], f["d_r"], f["d_n"], f["d_v"], f["page_tokens"], f["dtype"], f["sm_scale"])
        with pytest.raises(tp.TplaError) as e:
            tp.tpla_prefill_attention(shape, A, A, A, A, A, A, A, 8, 8, A, 1 << 30, A)
        assert e.value.code == -7


# ------------------------------------------------------------ whole path, bf16, model-shaped
@pytest.mark.parametrize("name,lens", [("dsv3_4k", [300, 1100, 64]), ("kimi_32k", [257, 900]), ("ragged_g4", [1500, 70, 640])])
def test_whole_path_bf16_scaled_configs(name, lens):
    w0 = wl.CONFIGS[name]
    _say(f"whole path bf16 {name} lens={lens}")
    w = wl.scaled(w0, B=len(lens), context=0, ragged=())
    m = wl.draw_model_side(wl.scaled(w, context=max(lens)))
    m["seq_lens"] = np.asarray(lens, dtype=np.int32)
    # rebuild the page table for the ragged lengths (permuted pool with spare pages)
    r = np.random.default_rng([w.seed, 5])
    pages = (np.asarray(lens) + 63) // 64
    P = int(pages.sum()) + 4
    order = r.permutation(P)
    bt = np.zeros((w.B, int(pages.max())), dtype=np.int32); k = 0
    for b in range(w.B):
        bt[b, :pages[b]] = order[k:k + pages[b]]; k += pages[b]
    m["block_table"], m["max_pages"], m["n_pool_pages"] = bt, int(pages.max()), P
    dev = "cuda"
    shape = pl.make_shape(w)
    c64, k64 = [], []
    mla_pool = torch.full((P, 64, w.d_c + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev)
    for b in range(w.B):
        c, kp = wl.draw_sequence(w, b, lens[b], heavy=m["heavy"])
        slots = torch.from_numpy(wl.slot_mapping(bt[b, :pages[b]], lens[b], 64)).to(dev)
        eps = 1e-6 if w.rms_prefill else -1.0
        tp.tpla_write_mla_cache(shape, pl.to_device(c, "bf16"), pl.to_device(kp, "bf16"), slots, lens[b], eps, mla_pool)
        cc = wl.as_f64(c, "bf16")
        # the cache stores bf16: the oracle rounds where the data is stored
        c64.append(orc.round_to_bf16(orc.rms_norm_unit(cc, eps)) if w.rms_prefill else cc)
        k64.append(wl.as_f64(kp, "bf16"))
    hadamard = w.transform == "hadamard"
    signs_np = m["signs"] if hadamard else None
    U64 = orc.hadamard_U(w.d_c, signs_np) if hadamard else None
    code = tp.TPLA_U_HADAMARD if hadamard else tp.TPLA_U_IDENTITY
    signs = torch.from_numpy(signs_np).to(dev) if hadamard else None
    W_UK_t, W_UV_t = pl.transform_weights(shape, code, signs, None, pl.to_device(m["W_UK"], "bf16"), pl.to_device(m["W_UV"], "bf16"))
    pools = [torch.full((P, 64, w.dl + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev) for _ in range(w.g)]
    used = torch.from_numpy(np.unique(np.concatenate([bt[b, :pages[b]] for b in range(w.B)])).astype(np.int32)).to(dev)
    tp.tpla_transform_latent_paged(shape, code, signs, None, mla_pool, pools, used, used.numel())
    step = pl.DecodeStep(shape, m["max_pages"])
    mu = [float(w.g)] * w.g
    o = step.run(pl.to_device(m["q_nope"], "bf16"), pl.to_device(m["q_pe"], "bf16"), W_UK_t, W_UV_t, pools,
                 torch.from_numpy(bt).to(dev), torch.from_numpy(m["seq_lens"]).to(dev), mu)
    torch.cuda.synchronize()
    ref = orc.tpla_decode(wl.as_f64(m["q_nope"], "bf16"), wl.as_f64(m["q_pe"], "bf16"), wl.as_f64(m["W_UK"], "bf16"),
                          wl.as_f64(m["W_UV"], "bf16"), c64, k64, w.g, w.sm_scale, U=U64, mu=mu)
    assert rel_err(wl.as_f64(pl.from_device_bits(step.q_lat), "bf16"), ref["Q_lat"]) <= TOL["bf16"]
    assert rel_err(step.o_lat.cpu().numpy(), ref["O_lat"]) <= TOL["bf16"]
    assert rel_err(o.cpu().numpy(), ref["o"]) <= TOL["bf16"]
    print("  lse err %.3g" % np.max(np.abs(step.lse.cpu().numpy() - ref["lse"])), flush=True)
    assert np.max(np.abs(step.lse.cpu().numpy() - ref["lse"])) <= 1e-2


def test_tpla_vs_mla_gap_matches_the_oracles_gap():
    """TPLA (g = 2) is not MLA: its per-slice softmaxes see only part of the score.  The size of
    that difference, with the cache in its own basis and in the Hadamard basis, measured through
    the library equals the one the oracle finds (heavy-channel latents as in the Kimi-shaped config)."""
    _say("TPLA vs MLA output gap")
    w = wl.scaled(wl.CONFIGS["kimi_32k"], B=3, context=0)
    lens = [500, 130, 64]
    dev = "cuda"
    m = wl.draw_model_side(wl.scaled(w, context=max(lens)))
    pages = (np.asarray(lens) + 63) // 64
    P = int(pages.sum())
    bt = np.zeros((w.B, int(pages.max())), dtype=np.int32); k = 0
    for b in range(w.B):
        bt[b, :pages[b]] = np.arange(k, k + pages[b]); k += pages[b]
    shape, shape1 = pl.make_shape(w), pl.make_shape(wl.scaled(w, g=1))
    mla_pool = torch.full((P, 64, w.d_c + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev)
    c64, k64 = [], []
    for b in range(w.B):
        c, kp = wl.draw_sequence(w, b, lens[b], heavy=m["heavy"])
        slots = torch.from_numpy(wl.slot_mapping(bt[b, :pages[b]], lens[b], 64)).to(dev)
        tp.tpla_write_mla_cache(shape, pl.to_device(c, "bf16"), pl.to_device(kp, "bf16"), slots, lens[b], -1.0, mla_pool)
        c64.append(wl.as_f64(c, "bf16")); k64.append(wl.as_f64(kp, "bf16"))
    q_nope, q_pe = pl.to_device(m["q_nope"], "bf16"), pl.to_device(m["q_pe"], "bf16")
    W_UK, W_UV = pl.to_device(m["W_UK"], "bf16"), pl.to_device(m["W_UV"], "bf16")
    bt_t, lens_t = torch.from_numpy(bt).to(dev), torch.tensor(lens, dtype=torch.int32, device=dev)
    used = torch.arange(P, dtype=torch.int32, device=dev)
    step1 = pl.DecodeStep(shape1, int(pages.max()))
    step1.absorb(q_nope, W_UK, None); step1.decode(0, q_pe, mla_pool, bt_t, lens_t); step1.combine(W_UV)
    o_mla = step1.o.double().cpu().numpy()
    f64 = {k_: wl.as_f64(m[k_], "bf16") for k_ in ("q_nope", "q_pe", "W_UK", "W_UV")}
    ref_mla = orc.mla_absorbed(f64["q_nope"], f64["q_pe"], f64["W_UK"], f64["W_UV"], c64, k64, w.sm_scale)
    assert rel_err(o_mla, ref_mla) <= TOL["bf16"]
    mu = [2.0, 2.0]
    gaps = {}
    for name, code, signs_np in (("identity", tp.TPLA_U_IDENTITY, None), ("hadamard", tp.TPLA_U_HADAMARD, m["signs"])):
        signs = None if signs_np is None else torch.from_numpy(signs_np).to(dev)
        Wk, Wv = pl.transform_weights(shape, code, signs, None, W_UK, W_UV)
        pools = [torch.full((P, 64, w.dl + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev) for _ in range(w.g)]
        tp.tpla_transform_latent_paged(shape, code, signs, None, mla_pool, pools, used, P)
        o = pl.DecodeStep(shape, int(pages.max())).run(q_nope, q_pe, Wk, Wv, pools, bt_t, lens_t, mu).double().cpu().numpy()
        U64 = None if signs_np is None else orc.hadamard_U(w.d_c, signs_np)
        ref = orc.tpla_decode(f64["q_nope"], f64["q_pe"], f64["W_UK"], f64["W_UV"], c64, k64, w.g, w.sm_scale, U=U64, mu=mu)["o"]
        got_gap = np.linalg.norm(o - o_mla) / np.linalg.norm(o_mla)
        ref_gap = np.linalg.norm(ref - ref_mla) / np.linalg.norm(ref_mla)
        gaps[name] = (got_gap, ref_gap)
        assert abs(got_gap - ref_gap) <= 0.05 * ref_gap + 5e-3, (name, got_gap, ref_gap)
    print("  gap (library, oracle):", gaps, flush=True)


def test_prefill_then_decode_end_to_end():
    """The two phases of Sec. 4.5 in sequence, every stage through the library: prompt latents
    normalised and written to the MLA cache, causal MLA prefill over the prompts, the cache turned
    into the Hadamard basis and sliced, the first generated token appended with the per-slice
    RMSNorm, one TPLA decode step and the output projection -- against the oracle doing the same
    (it rounds to bf16 wherever the library stores bf16)."""
    _say("prefill -> cache -> transform -> append -> decode -> W_O, end to end")
    w = wl.scaled(wl.CONFIGS["dsv3_32k"], B=2, H=16, context=0, rms_prefill=True, d_model=256)
    lens, pt, dev, eps = [150, 70], 64, "cuda", 1e-6
    m = wl.draw_model_side(wl.scaled(w, context=max(lens) + 1))
    shape = pl.make_shape(w)
    rng = np.random.default_rng([w.seed, 77])
    pages = (np.asarray(lens) + 1 + pt - 1) // pt                      # room for one more token
    P = int(pages.sum())
    bt = np.zeros((w.B, int(pages.max())), dtype=np.int32); k = 0
    for b in range(w.B):
        bt[b, :pages[b]] = np.arange(k, k + pages[b]); k += pages[b]
    # ---- prompt: raw latents -> MLA cache (global RMSNorm), packed normalised rows for the prefill
    mla_pool = torch.full((P, pt, w.d_c + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev)
    packed_c, packed_k, c64, k64, all_slots = [], [], [], [], []
    for b in range(w.B):
        c_raw, kp = wl.draw_sequence(w, b, lens[b])
        slots = wl.slot_mapping(bt[b, :pages[b]], lens[b], pt)
        tp.tpla_write_mla_cache(shape, pl.to_device(c_raw, "bf16"), pl.to_device(kp, "bf16"),
                                torch.from_numpy(slots).to(dev), lens[b], eps, mla_pool)
        c64.append(orc.round_to_bf16(orc.rms_norm_unit(wl.as_f64(c_raw, "bf16"), eps)))
        k64.append(wl.as_f64(kp, "bf16"))
        all_slots.append(slots)
    torch.cuda.synchronize()
    flat = mla_pool.view(P * pt, w.d_c + w.d_r)[torch.from_numpy(np.concatenate(all_slots)).long().to(dev)]
    got_c, ref_c = wl.as_f64(pl.from_device_bits(flat[:, :w.d_c].contiguous()), "bf16"), np.concatenate(c64)
    assert np.all(np.abs(got_c - ref_c) <= 2.0 ** -8 * np.abs(ref_c))          # float RMSNorm vs float64: at most one bf16 step
    T = sum(lens)
    qn_p = wl.to_storage(rng.standard_normal((T, w.H, w.d_n)), "bf16")
    qp_p = wl.to_storage(rng.standard_normal((T, w.H, w.d_r)), "bf16")
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    shape_p = pl.make_shape(wl.scaled(w, g=1))
    ws_b = tp.tpla_prefill_workspace_bytes(shape_p, T)
    ws = torch.empty(ws_b, dtype=torch.uint8, device=dev)
    o_p = torch.full((T, w.H, w.d_v), float("nan"), dtype=torch.float32, device=dev)
    W_UK, W_UV = pl.to_device(m["W_UK"], "bf16"), pl.to_device(m["W_UV"], "bf16")
    tp.tpla_prefill_attention(shape_p, pl.to_device(qn_p, "bf16"), pl.to_device(qp_p, "bf16"), flat[:, :w.d_c].contiguous(),
                              flat[:, w.d_c:].contiguous(), W_UK, W_UV, torch.from_numpy(cu).to(dev), T, max(lens), ws, ws_b, o_p)
    f64 = {k_: wl.as_f64(m[k_], "bf16") for k_ in ("W_UK", "W_UV", "q_nope", "q_pe")}
    ref_p = orc.mla_prefill(wl.as_f64(qn_p, "bf16"), wl.as_f64(qp_p, "bf16"), f64["W_UK"], f64["W_UV"],
                            np.concatenate(c64), np.concatenate(k64), cu, w.sm_scale)
    torch.cuda.synchronize()
    assert rel_err(o_p.cpu().numpy(), ref_p) <= TOL["bf16"]
    # ---- hand-over to decode: Hadamard basis, slices, one appended token per sequence
    signs_np = m["signs"]
    signs = torch.from_numpy(signs_np).to(dev)
    U64 = orc.hadamard_U(w.d_c, signs_np)
    W_UK_t, W_UV_t = pl.transform_weights(shape, tp.TPLA_U_HADAMARD, signs, None, W_UK, W_UV)
    pools = [torch.full((P, pt, w.dl + w.d_r), float("nan"), dtype=torch.bfloat16, device=dev) for _ in range(w.g)]
    used = torch.arange(P, dtype=torch.int32, device=dev)
    tp.tpla_transform_latent_paged(shape, tp.TPLA_U_HADAMARD, signs, None, mla_pool, pools, used, P)
    c_new = wl.to_storage(rng.standard_normal((w.B, w.d_c)) * 3.0, "bf16")        # already in the U basis, unnormalised
    k_new = wl.to_storage(rng.standard_normal((w.B, w.d_r)), "bf16")
    new_slots = np.array([bt[b, lens[b] // pt] * pt + lens[b] % pt for b in range(w.B)], dtype=np.int32)
    tp.tpla_append_token_sliced(shape, pl.to_device(c_new, "bf16"), pl.to_device(k_new, "bf16"), None, eps,
                                torch.from_numpy(new_slots).to(dev), pools)
    new_rows = orc.sliced_rms_rows(wl.as_f64(c_new, "bf16"), wl.as_f64(k_new, "bf16"), w.g, None, eps)
    step = pl.DecodeStep(shape, int(pages.max()))
    mu = [float(w.g)] * w.g
    o = step.run(pl.to_device(m["q_nope"], "bf16"), pl.to_device(m["q_pe"], "bf16"), W_UK_t, W_UV_t, pools,
                 torch.from_numpy(bt).to(dev), torch.tensor([L + 1 for L in lens], dtype=torch.int32, device=dev), mu)
    W_O = wl.draw_output_weight(w)
    wo_b = tp.tpla_output_projection_workspace_bytes(shape, w.d_model)
    wo_ws = torch.empty(max(wo_b, 16), dtype=torch.uint8, device=dev)
    y = torch.full((w.B, w.d_model), float("nan"), dtype=torch.float32, device=dev)
    tp.tpla_output_projection(shape, o, pl.to_device(W_O, "bf16"), w.d_model, wo_ws, wo_b, y)
    torch.cuda.synchronize()
    # oracle: transformed + rounded prompt rows, then the appended row (its slices, rounded), in the U basis
    c_dec, k_dec = [], []
    for b in range(w.B):
        prompt_t = orc.round_to_bf16(orc.transform_latent(c64[b], U64))
        app = orc.round_to_bf16(np.concatenate([new_rows[i][b, :w.dl] for i in range(w.g)]))
        c_dec.append(np.vstack([prompt_t, app[None, :]]))
        k_dec.append(np.vstack([k64[b], wl.as_f64(k_new, "bf16")[b][None, :]]))
    Wk_t, Wv_t = orc.reparameterize_weights(f64["W_UK"], f64["W_UV"], U64)
    Wk_t, Wv_t = orc.round_to_bf16(Wk_t), orc.round_to_bf16(Wv_t)
    ref = orc.tpla_decode(f64["q_nope"], f64["q_pe"], Wk_t, Wv_t, c_dec, k_dec, w.g, w.sm_scale, U=None, mu=mu)
    assert rel_err(o.cpu().numpy(), ref["o"]) <= TOL["bf16"]
    ref_y = orc.output_projection(ref["o"], wl.as_f64(W_O, "bf16"))
    assert rel_err(y.cpu().numpy(), ref_y) <= TOL["bf16"]
