"""tpla_decode_shards_combine_static (the entry point that takes no workspace: its partial
results live in a device array built into the library) against tpla_decode_shards_combine
and the float64 oracle, on two calls in a row, the second with a smaller input that must
not see what the first left in the array."""
import numpy as np
import pytest
import torch

import paper_2508_15881_amd as tp
from paper_2508_15881_amd import pipeline as pl
from paper_2508_15881_amd import workloads as wl
from oracle import tpla_oracle as orc
from gpu_common import TOL, build_shard_problem, rel_err

pytestmark = pytest.mark.gpu

DSV3 = wl.CONFIGS["dsv3_32k"]


def _problem(w, lens):
    """Inputs of all g slices over one page table, plus the oracle's o_lat, lse, o."""
    lens = np.asarray(lens, dtype=np.int32)
    Bn = len(lens)
    w = wl.scaled(w, B=Bn)
    dt = w.dtype
    probs = [build_shard_problem(w, lens, rng_extra=i) for i in range(w.g)]
    pools_np = []
    for i in range(w.g):
        pool = probs[0]["pool"].copy()
        for b in range(Bn):
            for j in range((int(lens[b]) + w.page_tokens - 1) // w.page_tokens):
                pool[probs[0]["bt"][b, j], :, :w.dl] = probs[i]["pool"][probs[i]["bt"][b, j], :, :w.dl]
        pools_np.append(pool)
    Wv = wl.to_storage(np.random.default_rng(99).standard_normal((w.H, w.d_c, w.d_v)) * 0.05, dt)
    kpe = [r[:, w.dl:] for r in probs[0]["rows64"]]
    ref_lat, ref_lse = [], []
    for i in range(w.g):
        c = [r[:, :w.dl] for r in probs[i]["rows64"]]
        o_i, l_i = orc.shard_attention(wl.as_f64(probs[i]["q_lat"], dt), wl.as_f64(probs[0]["q_pe"], dt), c, kpe, w.sm_scale)
        ref_lat.append(o_i); ref_lse.append(l_i)
    ref_lat = np.stack(ref_lat)
    return {
        "w": w, "shape": pl.make_shape(w), "mp": probs[0]["max_pages"], "lens": lens,
        "q_lat": pl.to_device(np.stack([p["q_lat"] for p in probs]), dt), "q_pe": pl.to_device(probs[0]["q_pe"], dt),
        "pools": [pl.to_device(p, dt) for p in pools_np], "bt": torch.from_numpy(probs[0]["bt"]).cuda(),
        "ln": torch.from_numpy(lens).cuda(), "Wv": pl.to_device(Wv, dt),
        "ref_lat": ref_lat, "ref_lse": np.stack(ref_lse), "ref_o": orc.combine_shards(ref_lat, wl.as_f64(Wv, dt)),
    }


def _outputs(p):
    w, nan = p["w"], float("nan")
    return (torch.full((w.B, w.H, w.d_v), nan, dtype=torch.float32, device="cuda"),
            torch.full((w.g, w.B, w.H, w.dl), nan, dtype=torch.float32, device="cuda"),
            torch.full((w.g, w.B, w.H), nan, dtype=torch.float32, device="cuda"))


def _check_call(p, n_splits):
    """One call of the static entry point; compares with the workspace entry point bit for bit
    (same kernels, same plan) and with the oracle at the decode tolerance."""
    o, o_lat, lse = _outputs(p)
    tp.tpla_decode_shards_combine_static(p["shape"], p["q_lat"], p["q_pe"], p["pools"], p["bt"], p["mp"], p["ln"],
                                         n_splits, p["Wv"], o, o_lat, lse)
    torch.cuda.synchronize()
    ws_b = tp.tpla_workspace_bytes_all(p["shape"], p["mp"], n_splits)
    assert 0 < ws_b <= (64 << 20)
    ws = torch.empty(ws_b, dtype=torch.uint8, device="cuda")
    o2, o_lat2, lse2 = _outputs(p)
    tp.tpla_decode_shards_combine(p["shape"], p["q_lat"], p["q_pe"], p["pools"], p["bt"], p["mp"], p["ln"], n_splits,
                                  ws, ws_b, p["Wv"], o2, o_lat2, lse2)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(o_lat, o_lat2) and torch.equal(lse, lse2)
    dt, nz = p["w"].dtype, p["lens"] > 0
    assert rel_err(o_lat.cpu().numpy(), p["ref_lat"]) <= TOL[dt]
    assert rel_err(o.cpu().numpy(), p["ref_o"]) <= TOL[dt]
    assert np.max(np.abs(lse.cpu().numpy()[:, nz] - p["ref_lse"][:, nz])) <= 1e-2


def test_static_scratch_entry_point_two_calls_the_second_smaller():
    big = _problem(DSV3, [3000, 700, 64, 0, 1500, 129])
    small = _problem(DSV3, [200, 65])
    for n_splits in (0, 5):
        print(f"static scratch: n_splits={n_splits} big then small", flush=True)
        _check_call(big, n_splits)
        _check_call(small, n_splits)
    # the generic (float) kernels go through the same scratch
    odd = wl.Workload("odd", B=3, H=5, d_c=80, g=2, d_r=24, d_n=16, d_v=16, dtype="f32", seed=11)
    print("static scratch: float path", flush=True)
    _check_call(_problem(odd, [300, 0, 65]), 0)
    _check_call(_problem(odd, [40]), 2)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    # 1024 chunks of 32 x 64 heads x 258 floats per slice: 4.3 GB of partial results
    w = wl.scaled(DSV3, B=32)
    shape = pl.make_shape(w)
    assert tp.tpla_workspace_bytes_all(shape, 2048, 1024) > (64 << 20)
    a = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(tp.TplaError) as e:
        tp.tpla_decode_shards_combine_static(shape, a, a, [a, a], a, 2048, a, 1024, a, a, a, None)
    assert e.value.code == -4 and "scratch" in tp.tpla_last_error()
