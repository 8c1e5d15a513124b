"""Parity at the full sizes of the benchmark configurations, in the launch
configurations bench.py times (automatic split plan; all slices in one launch
with the merge-and-combine kernel, and one slice per launch with separate
merge and combine), on sampled outputs: the oracle recomputes whole sequences
picked from the batch, every head of them, and one head of every other
sequence, so that no (slice, sequence) range of the plan goes unchecked."""
import numpy as np
import pytest
import torch

import paper_2508_15881_amd as tp
from paper_2508_15881_amd import pipeline as pl
from paper_2508_15881_amd import workloads as wl
from oracle import tpla_oracle as orc
from gpu_common import TOL, rel_err

pytestmark = pytest.mark.gpu


def _run_config(name, sample, w=None):
    w = wl.CONFIGS[name] if w is None else w
    print(f"full-size {name}: B={w.B} tokens~{w.B * (w.context or 26800)} sample={sample}", flush=True)
    dev = "cuda"
    shape = pl.make_shape(w)
    m = wl.draw_model_side(w)
    lens = m["seq_lens"]
    pt = w.page_tokens
    P = m["n_pool_pages"]
    pages = (lens.astype(np.int64) + pt - 1) // pt
    assert m["block_table"].max() < P and int(lens.max()) <= m["max_pages"] * pt
    tdt = pl.torch_dtype(w.dtype)
    mla_pool = torch.full((P, pt, w.d_c + w.d_r), float("nan"), dtype=tdt, device=dev)
    eps = 1e-6 if w.rms_prefill else -1.0
    hadamard = w.transform == "hadamard"
    U64 = orc.hadamard_U(w.d_c, m["signs"]) if hadamard else None
    q_nope, q_pe = wl.as_f64(m["q_nope"], w.dtype), wl.as_f64(m["q_pe"], w.dtype)
    W_UK, W_UV = wl.as_f64(m["W_UK"], w.dtype), wl.as_f64(m["W_UV"], w.dtype)
    mu = [float(w.g)] * w.g

    def reference(b, c, k, heads):
        c64 = wl.as_f64(c, w.dtype)
        if w.rms_prefill:
            c64 = orc.round_to_bf16(orc.rms_norm_unit(c64, eps))   # the cache stores bf16
        return orc.tpla_decode(q_nope[b:b + 1, heads], q_pe[b:b + 1, heads], W_UK[heads], W_UV[heads], [c64],
                               [wl.as_f64(k, w.dtype)], w.g, w.sm_scale, U=U64, mu=mu)

    refs = {}
    for b in range(w.B):
        L = int(lens[b])
        c, k = wl.draw_sequence(w, b, L, heavy=m["heavy"])
        slots = torch.from_numpy(wl.slot_mapping(m["block_table"][b, :pages[b]], L, pt)).to(dev)
        tp.tpla_write_mla_cache(shape, pl.to_device(c, w.dtype), pl.to_device(k, w.dtype), slots, L, eps, mla_pool)
        # the oracle works while the GPU writes: every head of the sampled sequences, one head of the others
        heads = slice(0, w.H) if b in sample else slice((7 * b + 3) % w.H, (7 * b + 3) % w.H + 1)
        refs[b] = (heads, reference(b, c, k, heads))
        if b % 16 == 15:
            print(f"  {b + 1} sequences written and recomputed", flush=True)
    torch.cuda.synchronize()
    print("  cache written", flush=True)
    code = tp.TPLA_U_HADAMARD if hadamard else tp.TPLA_U_IDENTITY
    signs = torch.from_numpy(m["signs"]).to(dev) if hadamard else None
    W_UK_t, W_UV_t = pl.transform_weights(shape, code, signs, None, pl.to_device(m["W_UK"], w.dtype),
                                          pl.to_device(m["W_UV"], w.dtype))
    pools = [torch.full((P, pt, w.dl + w.d_r), float("nan"), dtype=tdt, device=dev) for _ in range(w.g)]
    used_np = np.unique(np.concatenate([m["block_table"][b, :pages[b]] for b in range(w.B)])).astype(np.int32)
    tp.tpla_transform_latent_paged(shape, code, signs, None, mla_pool, pools, torch.from_numpy(used_np).to(dev), len(used_np))
    del mla_pool
    step = pl.DecodeStep(shape, m["max_pages"], 0)
    for fused in (True, False):
        path = "all slices per launch, merge-and-combine" if fused else "one slice per launch, merge, combine"
        step.o.fill_(float("nan")); step.o_lat.fill_(float("nan")); step.lse.fill_(float("nan"))
        o = step.run(pl.to_device(m["q_nope"], w.dtype), pl.to_device(m["q_pe"], w.dtype), W_UK_t, W_UV_t, pools,
                     torch.from_numpy(m["block_table"]).to(dev), torch.from_numpy(lens).to(dev), mu, fused=fused)
        torch.cuda.synchronize()
        print(f"  step done ({path})", flush=True)
        o = o.cpu().numpy(); o_lat = step.o_lat.cpu().numpy(); lse = step.lse.cpu().numpy()
        assert np.all(np.isfinite(o)) and np.all(np.isfinite(o_lat)) and np.all(np.isfinite(lse))
        worst = [0.0, 0.0, 0.0]
        for b in range(w.B):
            heads, ref = refs[b]
            e_lat = rel_err(o_lat[:, b:b + 1, heads], ref["O_lat"])
            e_o = rel_err(o[b:b + 1, heads], ref["o"])
            e_lse = float(np.max(np.abs(lse[:, b:b + 1, heads] - ref["lse"])))
            assert e_lat <= TOL[w.dtype] and e_o <= TOL[w.dtype] and e_lse <= 1e-2, (name, path, b, e_lat, e_o, e_lse)
            worst = [max(worst[0], e_lat), max(worst[1], e_o), max(worst[2], e_lse)]
            if b in sample:
                print(f"  sequence {b} (L={int(lens[b])}), every head: lse err {e_lse:.3g}, "
                      f"max |lse| {float(np.max(np.abs(ref['lse']))):.3g}", flush=True)
        print(f"  all {w.B} sequences ok: worst o_lat {worst[0]:.2e}, o {worst[1]:.2e}, lse {worst[2]:.3g}", flush=True)


@pytest.mark.timeout(300)
def test_full_size_dsv3_4k():
    _run_config("dsv3_4k", [0, 9, 15])


@pytest.mark.timeout(300)
def test_full_size_dsv3_32k():
    _run_config("dsv3_32k", [0, 17, 31])


@pytest.mark.timeout(400)
def test_full_size_mla_shaped_g1():
    """576-wide rows (one device of head-split MLA): 64 heads as pairs of waves, work items of 32 tiles."""
    _run_config("dsv3_32k with g = 1, B = 8", [0, 7], wl.scaled(wl.CONFIGS["dsv3_32k"], g=1, B=8))


@pytest.mark.timeout(600)
def test_full_size_kimi_32k():
    _run_config("kimi_32k", [3, 63])


@pytest.mark.timeout(900)
def test_full_size_ragged_g4():
    w = wl.CONFIGS["ragged_g4"]
    lens = wl.draw_model_side(w)["seq_lens"]
    order = np.argsort(lens)
    _run_config("ragged_g4", [int(order[0]), int(order[len(order) // 2]), int(order[-1])])


def test_full_size_prefill_32k_sampled_tokens():
    """One 32768-token sequence at 64 heads (the DeepSeek-V3 per-device shape), checked on
    sampled (token, head) outputs: the oracle's prefill row for a token equals its decode over the
    prefix, which it can afford for a handful of tokens."""
    L, H, d_c = 32768, 64, 512
    print(f"full-size prefill: L={L} H={H}", flush=True)
    dev = "cuda"
    rng = np.random.default_rng([7, 41])
    shape = tp.TplaShape(1, H, d_c, 1, 64, 128, 128, 64, tp.TPLA_BF16, 1.0 / np.sqrt(192.0))
    c = wl.to_storage(rng.standard_normal((L, d_c), dtype=np.float32), "bf16")
    k_pe = wl.to_storage(rng.standard_normal((L, 64), dtype=np.float32), "bf16")
    W_UK = wl.to_storage(rng.standard_normal((H, 128, d_c)) * 0.02, "bf16")
    W_UV = wl.to_storage(rng.standard_normal((H, d_c, 128)) * 0.02, "bf16")
    gen = torch.Generator(device=dev); gen.manual_seed(7)
    q_nope = torch.randn((L, H, 128), device=dev, dtype=torch.bfloat16, generator=gen)
    q_pe = torch.randn((L, H, 64), device=dev, dtype=torch.bfloat16, generator=gen)
    ws_b = tp.tpla_prefill_workspace_bytes(shape, L)
    ws = torch.empty(ws_b, dtype=torch.uint8, device=dev)
    o = torch.full((L, H, 128), float("nan"), dtype=torch.float32, device=dev)
    tp.tpla_prefill_attention(shape, q_nope, q_pe, pl.to_device(c, "bf16"), pl.to_device(k_pe, "bf16"),
                              pl.to_device(W_UK, "bf16"), pl.to_device(W_UV, "bf16"),
                              torch.tensor([0, L], dtype=torch.int32, device=dev), L, L, ws, ws_b, o)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(o).all())
    print("  kernel done", flush=True)
    c64, k64 = wl.as_f64(c, "bf16"), wl.as_f64(k_pe, "bf16")
    heads = [0, 21, 63]
    Wk, Wv = wl.as_f64(W_UK, "bf16")[heads], wl.as_f64(W_UV, "bf16")[heads]
    for t in (0, 1, 127, 128, 4097, 20000, L - 1):
        qn = q_nope[t, heads].double().cpu().numpy()[None]
        qp = q_pe[t, heads].double().cpu().numpy()[None]
        ref = orc.mla_naive(qn, qp, Wk, Wv, [c64[:t + 1]], [k64[:t + 1]], 1.0 / np.sqrt(192.0))[0]
        got = o[t, heads].cpu().numpy()
        assert rel_err(got, ref) <= TOL["bf16"], t
        print(f"  token {t}: rel err {rel_err(got, ref):.2e}", flush=True)
