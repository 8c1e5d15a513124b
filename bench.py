#!/usr/bin/env python3
"""Benchmark of the TPLA shard-decode path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dsv3_32k]
    python bench.py --traffic-calibration        (copy of known size, for scaling rocprofv3's byte counters)
    python bench.py --wg-timeline [--workload W] (per-workgroup timeline; library built with -DTPLA_WG_TIMELINE)

A step is one decode layer-step over one batch that is already resident in
HBM: absorb the query, run the attention of all g latent slices one after the
other on this GPU, and sum the slices through the value up-projection (the
stand-in for the all-reduce).  The cache transform that produces the shard
pools runs once before the timed region (it is cache-write-side work; its own
rate is reported as `transform`).  Before the W warm-up steps the GPU is held
under the same step until the kernel time has settled (`settle`): the chip
runs this step at its power limit and the first few hundred milliseconds of
load are a clock transient.  After the headline workload the other
model-shaped workloads run the same way and are reported under
`other_workloads`.  Prints ONE JSON line.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
OTHER_WORKLOADS = ("kimi_32k", "dsv3_4k", "ragged_g4")
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "decode_split_kernel_hbm_traffic.txt")


def kernel_source_digest():
    """Digest of the sources that decide the split kernel's memory traffic.  The measured-traffic
    figures under profiles/ carry the digest they were measured at; bench.py only quotes them
    while it still matches."""
    h = hashlib.sha256()
    for name in ("decode_mfma.hip", "lds_tile.h", "tpla_internal.h", "api.hip"):
        with open(os.path.join(ROOT, "paper_2508_15881_amd", "csrc", name), "r") as f:
            text = f.read()
        # comments and layout do not change the kernel: the digest is over the code alone
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def measured_traffic(workload, launch):
    """HBM bytes per launch of the split kernel from the rocprofv3 counter summary under profiles/
    (`launch` = "all_slices" | "one_slice"), or None when there is no figure for this workload or
    the kernel sources have changed since it was taken."""
    try:
        text = open(TRAFFIC_SUMMARY).read()
    except OSError:
        return None
    m = re.search(r"^sources_digest\s*=\s*(\w+)", text, flags=re.M)
    if not m or m.group(1) != kernel_source_digest():
        return None
    m = re.search(r"^traffic_bytes_per_launch\[%s,%s\]\s*=\s*(\d+)" % (re.escape(workload), launch), text, flags=re.M)
    return float(m.group(1)) if m else None


def cpu_baseline(w, model, budget_s=12.0):
    """The float64 oracle, as it stands, on a bounded sample of the same workload:
    whole sequences of the batch, one at a time, until the time budget is used."""
    from oracle import tpla_oracle as orc
    from paper_2508_15881_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    U = orc.hadamard_U(w.d_c, model["signs"]) if w.transform == "hadamard" else None
    W_UK = wl.as_f64(model["W_UK"], w.dtype)
    W_UV = wl.as_f64(model["W_UV"], w.dtype)
    q_nope = wl.as_f64(model["q_nope"], w.dtype)
    q_pe = wl.as_f64(model["q_pe"], w.dtype)
    mu = [float(w.g)] * w.g
    done_tokens, n_seq, t_total = 0, 0, 0.0
    for b in range(w.B):
        L = int(model["seq_lens"][b])
        c, k = wl.draw_sequence(w, b, L, heavy=model["heavy"])
        c64, k64 = wl.as_f64(c, w.dtype), wl.as_f64(k, w.dtype)
        if w.rms_prefill:
            c64 = orc.rms_norm_unit(c64, 1e-6)
        t0 = time.perf_counter()
        orc.tpla_decode(q_nope[b:b + 1], q_pe[b:b + 1], W_UK, W_UV, [c64], [k64], w.g, w.sm_scale, U=U, mu=mu)
        t_total += time.perf_counter() - t0
        done_tokens += L
        n_seq += 1
        if t_total >= budget_s:
            break
    esz = 4 if w.dtype == "f32" else 2
    gbs = done_tokens * w.g * (w.dl + w.d_r) * esz / t_total / 1e9
    return {"value": gbs, "unit": "GB/s", "cores": int(threads), "host_cpu_count": os.cpu_count(), "kind": "oracle",
            "sample": "%d of %d sequences (%d tokens), whole oracle step incl. its dense U products, %.1f s"
                      % (n_seq, w.B, done_tokens, t_total)}


def _under_profiler():
    """True when rocprofv3 (or another tool that preloads a GPU library into every child) runs this process."""
    return "rocprof" in os.environ.get("LD_PRELOAD", "").lower() or any(k.startswith("ROCPROF") for k in os.environ)


def _shader_clock_mhz():
    """Current shader clock from rocm-smi (None if the tool is missing or says nothing)."""
    import subprocess
    try:
        out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=10).stdout
    except Exception:
        return None
    m = re.search(r"sclk clock level:.*?\((\d+)Mhz\)", out)
    return int(m.group(1)) if m else None


def _socket_power_w():
    """Current socket power from amd-smi (None if the tool is missing or says nothing)."""
    import subprocess
    try:
        out = subprocess.run(["amd-smi", "metric", "-p"], capture_output=True, text=True, timeout=10).stdout
    except Exception:
        return None
    m = re.search(r"SOCKET_POWER:\s*(\d+)\s*W", out)
    return int(m.group(1)) if m else None


def _clock_while(fn, seconds=2.0, samples=3, burst=800):
    """Keeps the GPU busy with fn() for about `seconds`; samples (shader clock MHz, socket power W) meanwhile."""
    import torch
    clocks, t0 = [], time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(max(1, burst // 16)):
            fn()
        if (time.perf_counter() - t0) > seconds * (len(clocks) + 1) / (samples + 1) and len(clocks) < samples:
            for _ in range(burst):
                fn()                      # the queue holds work for the time the tools take
            clocks.append((_shader_clock_mhz(), _socket_power_w()))
    torch.cuda.synchronize()
    return clocks


class Prepared:
    """One workload resident in HBM: MLA pool written through S6, shard pools through S1, weights in
    the U basis, queries, page table, and the DecodeStep buffers."""

    def __init__(self, w, n_splits, dev="cuda"):
        import numpy as np
        import torch
        import paper_2508_15881_amd as tp
        from paper_2508_15881_amd import pipeline as pl
        from paper_2508_15881_amd import workloads as wl
        self.w = w
        self.shape = pl.make_shape(w)
        self.model = model = wl.draw_model_side(w)
        self.lens_np = lens_np = model["seq_lens"]
        P, pt = model["n_pool_pages"], w.page_tokens
        tdt = pl.torch_dtype(w.dtype)
        self.mla_pool = torch.full((P, pt, w.d_c + w.d_r), float("nan"), dtype=tdt, device=dev)

        def draw(b):
            return wl.draw_sequence(w, b, int(lens_np[b]), heavy=model["heavy"])

        # the host draws dominate the set-up: a few sequences at a time on worker threads
        with ThreadPoolExecutor(max_workers=6) as ex:
            for b0 in range(0, w.B, 6):
                for b, (c, k) in zip(range(b0, min(b0 + 6, w.B)), ex.map(draw, range(b0, min(b0 + 6, w.B)))):
                    L = int(lens_np[b])
                    n = (L + pt - 1) // pt
                    slots = torch.from_numpy(wl.slot_mapping(model["block_table"][b, :n], L, pt)).to(dev)
                    tp.tpla_write_mla_cache(self.shape, pl.to_device(c, w.dtype), pl.to_device(k, w.dtype), slots, L,
                                            1e-6 if w.rms_prefill else -1.0, self.mla_pool)
        hadamard = w.transform == "hadamard"
        self.code = tp.TPLA_U_HADAMARD if hadamard else tp.TPLA_U_IDENTITY
        self.signs = torch.from_numpy(model["signs"]).to(dev) if hadamard else None
        self.W_UK_t, self.W_UV_t = pl.transform_weights(self.shape, self.code, self.signs, None,
                                                        pl.to_device(model["W_UK"], w.dtype),
                                                        pl.to_device(model["W_UV"], w.dtype))
        self.pools = [torch.full((P, pt, w.dl + w.d_r), float("nan"), dtype=tdt, device=dev) for _ in range(w.g)]
        pages = (lens_np.astype(np.int64) + pt - 1) // pt
        self.used_np = np.unique(np.concatenate([model["block_table"][b, :pages[b]] for b in range(w.B)])).astype(np.int32)
        self.used = torch.from_numpy(self.used_np).to(dev)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_tr = []
        for _ in range(4):
            ev0.record()
            tp.tpla_transform_latent_paged(self.shape, self.code, self.signs, None, self.mla_pool, self.pools, self.used,
                                           len(self.used_np))
            ev1.record()
            torch.cuda.synchronize()
            t_tr.append(ev0.elapsed_time(ev1))
        self.esz = esz = 4 if w.dtype == "f32" else 2
        tr_bytes = len(self.used_np) * pt * ((w.d_c + w.d_r) + w.g * (w.dl + w.d_r)) * esz
        self.transform = {"us": min(t_tr) * 1e3, "GB/s_read_plus_write": tr_bytes / (min(t_tr) * 1e-3) / 1e9}
        self.q_nope = pl.to_device(model["q_nope"], w.dtype)
        self.q_pe = pl.to_device(model["q_pe"], w.dtype)
        self.bt = torch.from_numpy(model["block_table"]).to(dev)
        self.lens = torch.from_numpy(lens_np).to(dev)
        self.mu = [float(w.g)] * w.g
        self.step = pl.DecodeStep(self.shape, model["max_pages"], n_splits)
        # A cache that fits the 256 MB last-level cache would be re-read from there step after step:
        # small workloads rotate over enough copies of the pools (>= 8, >= 2 GiB in all) that every
        # step reads from HBM; the cache-resident figure is reported beside it.
        pool_bytes = sum(p.numel() * p.element_size() for p in self.pools)
        self.n_sets = 1 if pool_bytes >= (1 << 30) else max(8, -(-(2 << 30) // pool_bytes))
        self.pool_sets = [self.pools] + [[p.clone() for p in self.pools] for _ in range(self.n_sets - 1)]
        self.shard_bytes = wl.algorithmic_bytes_per_shard(w, lens_np)
        self._i = 0

    def run_step(self, pools=None):
        """One layer-step; rotates over the pool copies unless `pools` pins one."""
        if pools is None:
            pools = self.pool_sets[self._i % self.n_sets]
            self._i += 1
        self.step.run(self.q_nope, self.q_pe, self.W_UK_t, self.W_UV_t, pools, self.bt, self.lens, self.mu)


def settle(p, min_s, max_s, batch=40, keep_events_for=0):
    """Holds the GPU under the decode step until the split kernel's time has settled: batches of
    `batch` event-timed steps, at least min_s, until three batch means in a row agree to 2 %
    (at most max_s).  Returns what happened; nothing of it enters the timed region.
    keep_events_for = N leaves event pairs for N launches in place, so that the timed region can follow
    without the pause that creating them would be (the first launches after a pause run slower)."""
    import numpy as np
    import torch
    import paper_2508_15881_amd as tp
    cap = max(batch, keep_events_for)
    tp.tpla_profile_enable(cap)
    means, t0 = [], time.perf_counter()
    while True:
        for _ in range(batch):
            p.run_step()
        torch.cuda.synchronize()
        means.append(float(np.mean(tp.tpla_profile_collect(cap)[:batch])) * 1e3)
        el = time.perf_counter() - t0
        agreed = len(means) >= 3 and max(means[-3:]) <= 1.02 * min(means[-3:])
        if (el >= min_s and agreed) or el >= max_s:
            break
    if not keep_events_for:
        tp.tpla_profile_enable(0)
    return {"settle_s": el, "steps": batch * len(means), "agreed_to_2pct": bool(agreed),
            "launch_us_first_batch": means[0], "launch_us_slowest_batch": max(means), "launch_us_last_batch": means[-1]}


def timed_region(p, warmup, steps, pools=None, events_ready=False):
    """W untimed warm-up steps, then exactly K steps between two synchronisations, the split kernel of
    every step bracketed by HIP events on the launch stream (the warm-up steps carry events too and
    their readings are dropped: the events exist before the first step, so nothing but the
    synchronisation separates warm-up and timed steps).  Returns (ms_per_step, kernel ms list)."""
    import torch
    import paper_2508_15881_amd as tp
    if not events_ready:
        tp.tpla_profile_enable(warmup + steps)
    for _ in range(warmup):
        p.run_step(pools)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        p.run_step(pools)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kern_ms = tp.tpla_profile_collect(warmup + steps)[warmup:]
    tp.tpla_profile_enable(0)
    return (t1 - t0) * 1e3 / steps, kern_ms


def launch_stats(kern_ms):
    import numpy as np
    k = np.asarray(kern_ms, dtype=np.float64) * 1e3
    return {"launch_us": float(k.mean()), "launches": int(len(k)), "launch_us_min": float(k.min()),
            "launch_us_median": float(np.median(k)), "launch_us_first10": float(k[:10].mean()),
            "launch_us_last10": float(k[-10:].mean())}


def one_slice_launches(p, n):
    """The same kernel on one device's share: one slice per launch (tpla_decode_shard), event-timed."""
    import torch
    import paper_2508_15881_amd as tp
    w = p.w
    tp.tpla_profile_enable(n * w.g)
    for _ in range(n):
        for i in range(w.g):
            p.step.decode(i, p.q_pe, p.pools[i], p.bt, p.lens)
    torch.cuda.synchronize()
    ms = tp.tpla_profile_collect(n * w.g)
    tp.tpla_profile_enable(0)
    return ms


def measure_other(name, args):
    """Settle + warm-up + timed steps of another model-shaped workload."""
    import numpy as np
    from paper_2508_15881_amd import workloads as wl
    w = wl.CONFIGS[name]
    p = Prepared(w, 0)
    steps = max(args.steps, 50)
    st = settle(p, min(args.settle_s, 0.5), max(1.5, args.settle_s), keep_events_for=args.warmup + steps)
    ms_per_step, kern_ms = timed_region(p, args.warmup, steps, events_ready=True)
    ls = launch_stats(kern_ms)
    launch_bytes = w.g * p.shard_bytes
    achieved = launch_bytes / (ls["launch_us"] * 1e-6) / 1e9
    one = one_slice_launches(p, 30)
    one_us = float(np.mean(one)) * 1e3
    out = {"config": {"B": w.B, "H": w.H, "d_c": w.d_c, "g": w.g, "context_max": int(p.lens_np.max()),
                      "tokens": int(p.lens_np.sum()), "transform": w.transform, "pages_permuted": bool(w.permute_pages)},
           "ms_per_step": ms_per_step, "value_GB/s": launch_bytes / (ms_per_step * 1e-3) / 1e9,
           "steps": steps, "settle": st, "pool_copies_rotated": p.n_sets,
           "roofline": dict({"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": achieved / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": launch_bytes,
                             "traffic": measured_traffic(name, "all_slices")}, **ls),
           "one_slice": {"launch_us": one_us, "frac": p.shard_bytes / (one_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
           "transform_GB/s_read_plus_write": p.transform["GB/s_read_plus_write"]}
    return out


def traffic_calibration():
    """Kernels of known HBM traffic, for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE readings:
    five identity-mode tpla_transform_latent calls that copy 1 GiB each (read 1 GiB, write 1 GiB)
    and five tpla_stream_read calls over the same 1 GiB (read only)."""
    import torch
    import paper_2508_15881_amd as tp
    tp.load_library()
    d_c, n_rows = 512, (1 << 30) // (512 * 2)
    shape = tp.TplaShape(1, 1, d_c, 1, 64, 128, 128, 64, tp.TPLA_BF16, 1.0)
    src = torch.ones((n_rows, d_c), dtype=torch.bfloat16, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    for _ in range(5):
        tp.tpla_transform_latent(shape, tp.TPLA_U_IDENTITY, 0, None, None, src, dst, n_rows, 1)
    for _ in range(5):
        tp.tpla_stream_read(src, src.numel() * 2, sink)
    torch.cuda.synchronize()
    print(json.dumps({"copied_bytes_per_transform_axis_launch": src.numel() * 2,
                      "read_bytes_per_stream_read_launch": src.numel() * 2 - (src.numel() * 2) % 20480, "launches_each": 5}))


def wg_timeline(args):
    """Per-workgroup timeline of the split kernel (needs a library built with
    TPLA_EXTRA_HIPCC_FLAGS=-DTPLA_WG_TIMELINE): start skew, time to the first tile, end of the tile
    loop and end of the workgroup, and how the workgroups' durations differ by placement round
    (workgroup id / compute units) and by XCC, over several settled launches."""
    import ctypes
    import numpy as np
    import torch
    import paper_2508_15881_amd as tp
    from paper_2508_15881_amd import workloads as wl
    lib = tp.load_library()
    if not hasattr(lib, "tpla_debug_wg_timeline"):
        print("bench.py --wg-timeline: build the library with TPLA_EXTRA_HIPCC_FLAGS=-DTPLA_WG_TIMELINE first", file=sys.stderr)
        sys.exit(1)
    hip = ctypes.CDLL("libamdhip64.so")
    p_t, p_w, p_p = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    assert lib.tpla_debug_wg_timeline(ctypes.byref(p_t), ctypes.byref(p_w), ctypes.byref(p_p)) == 0
    w = wl.CONFIGS[args.workload]
    if args.set:
        w = wl.scaled(w, **{k: int(v) for k, v in (kv.split("=") for kv in args.set)})
    p = Prepared(w, args.n_splits)
    n_wg = p.step.ws_bytes // (w.H * (w.dl + 2) * 4) - w.g * w.B if args.n_splits == 0 else 0
    assert 0 < n_wg <= 4096, "the timeline covers balanced launches of at most 4096 workgroups"
    run = lambda: p.step.decode_all(p.q_pe, p.pools, p.bt, p.lens)
    p.step.absorb(p.q_nope, p.W_UK_t, p.mu)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < max(args.settle_s, 0.5):
        for _ in range(50):
            run()
        torch.cuda.synchronize()
    durs, firsts, loops, starts, kern = [], [], [], [], []
    for _ in range(12):
        tp.tpla_profile_enable(20)
        for _ in range(20):
            run()
        torch.cuda.synchronize()
        kern.append(float(np.mean(tp.tpla_profile_collect(20))) * 1e3)
        buf = np.zeros(4096 * 4, dtype=np.uint64)
        assert hip.hipMemcpy(buf.ctypes.data_as(ctypes.c_void_p), p_t, buf.nbytes, 2) == 0
        t = buf.reshape(-1, 4)[:n_wg].astype(np.float64) * 0.01       # microseconds
        t -= t[:, 0].min()
        starts.append(t[:, 0]); firsts.append(t[:, 1] - t[:, 0]); loops.append(t[:, 2]); durs.append(t[:, 3] - t[:, 0])
    tp.tpla_profile_enable(0)
    where = np.zeros(4096 * 2, dtype=np.uint32)
    assert hip.hipMemcpy(where.ctypes.data_as(ctypes.c_void_p), p_w, where.nbytes, 2) == 0
    xcc = (where.reshape(-1, 2)[:n_wg, 0] & 15).astype(int)
    D = np.array(durs)
    rel = (D / D.mean(axis=1, keepdims=True)).mean(axis=0)           # systematic part, relative to the launch mean
    z = (D - D.mean(axis=1, keepdims=True)) / D.std(axis=1, keepdims=True)
    cc = np.corrcoef(z)
    pct = lambda x: [round(float(v), 2) for v in np.percentile(np.concatenate(x), [0, 10, 50, 90, 100])]
    try:
        cus = torch.cuda.get_device_properties(0).multi_processor_count
    except Exception:
        cus = 256
    rounds = np.arange(n_wg) // cus
    # phase clocks (only the 32-heads-per-wave instances record them), from the last launch
    ph = np.zeros(4096 * 5, dtype=np.uint64)
    assert hip.hipMemcpy(ph.ctypes.data_as(ctypes.c_void_p), p_p, ph.nbytes, 2) == 0
    ph = ph.reshape(-1, 5)[:n_wg].astype(np.float64)
    phase = None
    if ph[:, 4].sum() > 0:
        n_items = max(1.0, float(np.count_nonzero(ph[:, 4])))
        phase = {"what": "shader clocks per 32-token tile of wave 0, mean over the workgroups of the last launch",
                 "plain_score_product_of_an_items_first_tile": float(ph[:, 0].sum() / n_items),
                 "wait_barrier_and_tile_requests": float(ph[:, 1].sum() / ph[:, 4].sum()),
                 "score_mfmas_with_previous_tiles_softmax_between_them": float(ph[:, 2].sum() / ph[:, 4].sum()),
                 "output_mfmas": float(ph[:, 3].sum() / ph[:, 4].sum())}
    print(json.dumps({
        "workload": w.name, "workgroups": int(n_wg), "launches": 12 * 20, "kernel_us_mean_with_timeline_code": float(np.mean(kern)),
        "percentiles": "min, 10 %, median, 90 %, max over workgroups and 12 sampled launches, microseconds",
        "workgroup_start_after_first": pct(starts), "first_tile_landed_after_start": pct(firsts),
        "tile_loop_done_after_first_start": pct(loops), "workgroup_duration": pct(durs),
        "duration_max_over_mean_per_launch": [round(float(d.max() / d.mean()), 3) for d in D],
        "same_workgroups_slow_every_launch_correlation": round(float((cc.sum() - len(cc)) / (len(cc) * (len(cc) - 1))), 3),
        "relative_duration_by_placement_round": {str(r): round(float(rel[rounds == r].mean()), 3) for r in sorted(set(rounds.tolist()))},
        "relative_duration_by_xcc": {str(x): round(float(rel[xcc == x].mean()), 3) for x in sorted(set(xcc.tolist()))},
        # how the last sampled launch was dealt to the XCCs: workgroup w ran on XCC (w + offset) % 8 for one offset?
        "xcc_of_workgroups_0_to_15": xcc[:16].tolist(),
        "workgroups_on_xcc_w_plus_offset_mod_8": {str(o): int(np.sum((np.arange(n_wg) + o) % 8 == xcc)) for o in range(8)
                                                  if np.sum((np.arange(n_wg) + o) % 8 == xcc) > 0},
        "phase_clocks_32_heads_per_wave": phase,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="dsv3_32k")
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--settle-s", type=float, default=1.0,
                    help="hold the GPU under the decode step for at least this long before the warm-up steps "
                         "(until the kernel time has settled, at most three times as long); 0 = off")
    ap.add_argument("--others", default=",".join(OTHER_WORKLOADS),
                    help="comma-separated workloads reported under other_workloads after the headline ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--set", action="append", default=[], metavar="FIELD=VALUE",
                    help="override an integer field of the workload, e.g. --set H=128 --set B=16")
    ap.add_argument("--skip-extras", action="store_true",
                    help="only the timed steps: no one-slice loop, stage timings, MLA reference or other workloads "
                         "(keeps every launch of the decode kernel in a profile identical)")
    ap.add_argument("--traffic-calibration", action="store_true")
    ap.add_argument("--wg-timeline", action="store_true",
                    help="per-workgroup timeline of the split kernel (library built with -DTPLA_WG_TIMELINE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (all g latent slices are computed on it and "
              "summed locally, no collective); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2508_15881_amd as tp
    from paper_2508_15881_amd import pipeline as pl
    from paper_2508_15881_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    tp.load_library()           # fails loudly when the HIP library is not built
    if args.traffic_calibration:
        traffic_calibration()
        return
    if args.wg_timeline:
        wg_timeline(args)
        return
    dev = "cuda"
    w = wl.CONFIGS[args.workload]
    if args.set:
        w = wl.scaled(w, name=w.name + "(" + ",".join(args.set) + ")",
                      **{k: int(v) for k, v in (kv.split("=") for kv in args.set)})

    # ---- inputs into HBM (untimed): MLA-style pool, then the shard pools --------
    p = Prepared(w, args.n_splits)
    shape, model, lens_np, pt, tdt, esz = p.shape, p.model, p.lens_np, w.page_tokens, pl.torch_dtype(w.dtype), p.esz
    mla_pool, pools, used, used_np = p.mla_pool, p.pools, p.used, p.used_np
    q_nope, q_pe, W_UK_t, W_UV_t, bt, lens, mu, step = p.q_nope, p.q_pe, p.W_UK_t, p.W_UV_t, p.bt, p.lens, p.mu, p.step
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    # ---- settle, W warm-up steps, then the timed region: exactly K steps ----------
    n_sets_rotated = p.n_sets
    settled = (settle(p, args.settle_s, 3.0 * args.settle_s, keep_events_for=args.warmup + args.steps)
               if args.settle_s > 0 else None)
    ms_per_step, kern_ms = timed_region(p, args.warmup, args.steps, events_ready=settled is not None)

    cache_resident = None
    if p.n_sets > 1:
        ms_c, kc = timed_region(p, 0, args.steps, pools)
        cache_resident = {"ms_per_step": ms_c, "split_kernel_us": float(np.mean(kc)) * 1e3,
                          "note": "same step re-reading one copy of the pools (it fits the last-level cache)"}
        del p.pool_sets[1:]
        p.n_sets = 1

    # one device's share: the same kernel launched for one slice at a time
    one_ms = one_slice_launches(p, min(args.steps, 200)) if not args.skip_extras else [float("nan")]

    # the other model-shaped workloads, one after the other, each with its own pools -- before the extra
    # stages below, of which the prefill and the PCA passes leave the GPU hot enough to cost the kernels that
    # follow them several per cent
    others = None
    if not args.skip_extras and args.others:
        others = {name: measure_other(name, args) for name in args.others.split(",") if name != w.name}

    shard_bytes = p.shard_bytes
    value = w.g * shard_bytes / (ms_per_step * 1e-3) / 1e9
    ls = launch_stats(kern_ms)
    kern_avg_ms = ls["launch_us"] * 1e-3
    launch_bytes = w.g * shard_bytes
    achieved = launch_bytes / (kern_avg_ms * 1e-3) / 1e9
    one_avg_ms = float(np.mean(one_ms))
    one_achieved = shard_bytes / (one_avg_ms * 1e-3) / 1e9

    # what this machine delivers to a kernel that only reads (same pool, 128-bit streaming loads):
    # boxes differ by several per cent, and so does this ceiling
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    nb0 = pools[0].numel() * pools[0].element_size()
    ceil_ms = []
    if not args.skip_extras:
        for i in range(12):
            ev0.record(); tp.tpla_stream_read(pools[i % w.g], nb0, sink); ev1.record()
            torch.cuda.synchronize()
            if i >= 2:
                ceil_ms.append(ev0.elapsed_time(ev1))
    ceiling = nb0 / (float(np.median(ceil_ms)) * 1e-3) / 1e9 if ceil_ms else None

    # modelled traffic of one split launch beyond the cache rows: queries, page table, lengths
    # (read by every workgroup's item) and the float partial results (written once)
    n_items = step.ws_bytes // (w.H * (w.dl + 2) * 4)          # partial-result slots of the plan
    all_traffic = launch_bytes + n_items * w.H * ((w.dl + w.d_r) * esz + (w.dl + 2) * 4) + w.g * w.B * model["max_pages"] * 4

    # stage breakdown (untimed region, events on torch's current stream = the launch stream)
    def timed(fn, reps=20, warm=1):
        if args.skip_extras:
            return float("nan")
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            fn()
        ev1.record(); torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps * 1e3
    us_absorb = timed(lambda: step.absorb(q_nope, W_UK_t, mu))
    # the long stages get enough launches for the clocks to settle after the short ones
    us_decode = timed(lambda: step.decode(0, q_pe, pools[0], bt, lens), reps=100, warm=30)
    us_decode_all = timed(lambda: step.decode_all(q_pe, pools, bt, lens), reps=100, warm=30)
    us_combine = timed(lambda: step.combine(W_UV_t))
    us_decode_combine = timed(lambda: step.decode_all_combine(q_pe, pools, bt, lens, W_UV_t), reps=100, warm=30)

    def separate_step():
        step.absorb(q_nope, W_UK_t, mu)
        step.decode_all(q_pe, pools, bt, lens)
        step.combine(W_UV_t)
    us_step_separate = timed(separate_step, reps=100, warm=30)
    us_wo = us_block = float("nan")
    if not args.skip_extras:
        # block output o W_O (after the timed step's last stage; weight-streaming GEMM)
        W_O = pl.to_device(wl.draw_output_weight(w), w.dtype)
        wo_ws_b = tp.tpla_output_projection_workspace_bytes(shape, w.d_model)
        wo_ws = torch.empty(max(wo_ws_b, 16), dtype=torch.uint8, device=dev)
        wo_out = torch.empty((w.B, w.d_model), dtype=torch.float32, device=dev)
        us_wo = timed(lambda: tp.tpla_output_projection(shape, step.o, W_O, w.d_model, wo_ws, wo_ws_b, wo_out))
        # the whole attention block after the query projections: absorb + one tpla_decode_shards_project call
        step_p = pl.DecodeStep(shape, model["max_pages"], args.n_splits, d_model=w.d_model)

        def block_step():
            step_p.absorb(q_nope, W_UK_t, mu)
            step_p.decode_all_project(q_pe, pools, bt, lens, W_UV_t, W_O)
        us_block = timed(block_step, reps=100, warm=30)
        del step_p

    # the same step replayed from a HIP graph (launch overhead of its kernels removed);
    # informational: the timed region above launches eagerly so that its kernels can be bracketed
    us_graph = float("nan")
    if not args.skip_extras:
        graph = step.capture(q_nope, q_pe, W_UK_t, W_UV_t, pools, bt, lens, mu)
        for _ in range(20):
            graph.replay()
        torch.cuda.synchronize()
        n_rep = min(max(args.steps, 100), 300)
        tg = time.perf_counter()
        for _ in range(n_rep):
            graph.replay()
        torch.cuda.synchronize()
        us_graph = (time.perf_counter() - tg) * 1e6 / n_rep
        del graph

    # PCA calibration path (Sec. 4.3.2), not part of the step: moments of the cached latents on
    # the GPU, eigen-solve on the host, cache turned into the dense basis on the matrix cores
    pca = None
    if not args.skip_extras and w.dtype == "bf16":
        n_used = len(used_np)
        ws_b = tp.tpla_latent_moments_workspace_bytes(shape, n_used)
        ws_m = torch.empty(max(ws_b, 16), dtype=torch.uint8, device=dev)
        m_sum = torch.empty(w.d_c, dtype=torch.float64, device=dev)
        m_gram = torch.empty((w.d_c, w.d_c), dtype=torch.float64, device=dev)
        us_mom = timed(lambda: tp.tpla_latent_moments(shape, mla_pool, used, None, n_used, ws_m, ws_b, m_sum, m_gram), reps=5)
        tcpu = time.perf_counter()
        U_np, eig, frac = tp.tpla_pca_basis(w.d_c, w.g, n_used * pt, m_sum.cpu().numpy(), m_gram.cpu().numpy())
        eig_s = time.perf_counter() - tcpu
        U_dev = torch.from_numpy(U_np).to(dev)
        scratch_pools = [torch.empty_like(q) for q in pools]
        us_dense = timed(lambda: tp.tpla_transform_latent_paged(shape, tp.TPLA_U_DENSE, None, U_dev, mla_pool,
                                                                scratch_pools, used, n_used), reps=3)
        del scratch_pools, ws_m
        pca = {"latent_moments_us": us_mom, "eigen_solve_host_s": eig_s, "dense_transform_us": us_dense,
               "dense_transform_TFLOPs_hi_lo": 4.0 * n_used * pt * w.d_c * w.d_c / (us_dense * 1e-6) / 1e12,
               "variance_fractions": [float(f) for f in frac]}

    # Prefill of one context-length sequence with un-absorbed MLA (the other phase of Sec. 4.5;
    # MFMA-bound, not part of the decode step): key/value up-projection + causal attention
    prefill, prefill_fn = None, None
    if not args.skip_extras and w.dtype == "bf16" and w.d_n == 128 and w.d_v == 128 and w.d_r == 64:
        Lp = int(lens_np.max())
        shape_p = pl.make_shape(wl.scaled(w, B=1, g=1))
        gen = torch.Generator(device=dev); gen.manual_seed(w.seed)
        pq_nope = torch.randn((Lp, w.H, w.d_n), device=dev, dtype=tdt, generator=gen)
        pq_pe = torch.randn((Lp, w.H, w.d_r), device=dev, dtype=tdt, generator=gen)
        pc = torch.randn((Lp, w.d_c), device=dev, dtype=tdt, generator=gen)
        pk = torch.randn((Lp, w.d_r), device=dev, dtype=tdt, generator=gen)
        pcu = torch.tensor([0, Lp], dtype=torch.int32, device=dev)
        pws_b = tp.tpla_prefill_workspace_bytes(shape_p, Lp)
        pws = torch.empty(pws_b, dtype=torch.uint8, device=dev)
        po = torch.empty((Lp, w.H, w.d_v), dtype=torch.float32, device=dev)
        W_UK0, W_UV0 = pl.to_device(model["W_UK"], w.dtype), pl.to_device(model["W_UV"], w.dtype)

        def prefill_fn():
            tp.tpla_prefill_attention(shape_p, pq_nope, pq_pe, pc, pk, W_UK0, W_UV0, pcu, Lp, Lp, pws, pws_b, po)
        us_pf = timed(prefill_fn, reps=3)
        flop = 2.0 * (w.d_n + w.d_r + w.d_v) * w.H * (Lp * (Lp + 1) / 2) + 2.0 * Lp * w.d_c * w.H * (w.d_n + w.d_v)
        prefill = {"tokens": Lp, "heads": w.H, "ms": us_pf * 1e-3, "TFLOP/s": flop / (us_pf * 1e-6) / 1e12,
                   "bound": "mfma", "peak_TFLOP/s": 2500.0, "frac": flop / (us_pf * 1e-6) / 1e12 / 2500.0,
                   "flop_counted": "causal half of QK^T and PV plus the key/value up-projection"}

    # shader clock and socket power under load: the decode step runs at the chip's power limit, the pure reader does not
    power_state = None
    if not args.skip_extras and _under_profiler():
        power_state = {"skipped": "a profiler is attached to this process: the two tools are scripts whose interpreter "
                                  "would be started from a process the profiler's library has already put on the GPU"}
    elif not args.skip_extras:
        power_state = {
            "what": "[shader clock MHz (rocm-smi), socket power W (amd-smi)] sampled while the GPU runs the named work back to back",
            "decode_steps": _clock_while(lambda: p.run_step(pools)),
            "pure_reader": _clock_while(lambda: tp.tpla_stream_read(pools[0], nb0, sink)),
        }
        if prefill_fn is not None:
            power_state["prefill_attention"] = _clock_while(prefill_fn, burst=8)
    if prefill_fn is not None:
        del pq_nope, pq_pe, pws, po, prefill_fn

    # MLA under head-split tensor parallelism, one device's share: the same H heads
    # over the unsliced 576-wide cache (the MLA pool is exactly the g = 1 layout).
    # Its time against one TPLA slice is this box's counterpart of the paper's ratio.
    w1 = wl.scaled(w, g=1)
    shape1 = pl.make_shape(w1)
    step1 = pl.DecodeStep(shape1, model["max_pages"], 0)
    step1.absorb(q_nope, W_UK_t, None)
    n_mla = 0 if args.skip_extras else min(max(args.steps, 100), 200)
    mla_ms = float("nan")
    if n_mla:
        for _ in range(100):
            step1.decode(0, q_pe, mla_pool, bt, lens)
        tp.tpla_profile_enable(n_mla)
        for _ in range(n_mla):
            step1.decode(0, q_pe, mla_pool, bt, lens)
        torch.cuda.synchronize()
        mla_ms = float(np.mean(tp.tpla_profile_collect(n_mla)))
        tp.tpla_profile_enable(0)
    mla_bytes = wl.algorithmic_bytes_per_shard(w1, lens_np)

    # How far TPLA's per-slice softmaxes move the block output away from MLA's (Sec. 4.2: the
    # slices' scores only approximate the global ones), with the cache left in its own basis and
    # in the Hadamard basis (Sec. 4.3.1).  Information only: the paper gives no per-tensor figure.
    gap = None
    if not args.skip_extras and w.g > 1 and (w.d_c & (w.d_c - 1)) == 0:
        W_UK0, W_UV0 = pl.to_device(model["W_UK"], w.dtype), pl.to_device(model["W_UV"], w.dtype)
        step1.absorb(q_nope, W_UK0, None)
        step1.decode(0, q_pe, mla_pool, bt, lens)
        step1.combine(W_UV0)
        o_mla = step1.o.double()
        scratch = [torch.empty_like(q) for q in pools]
        stepx = pl.DecodeStep(shape, model["max_pages"], 0)
        gap = {"what": "|o_TPLA - o_MLA|_F / |o_MLA|_F over the batch, mu_i = g"}
        sg = torch.from_numpy(model["signs"]).to(dev)
        for name, codex, sx in (("identity", tp.TPLA_U_IDENTITY, None), ("hadamard", tp.TPLA_U_HADAMARD, sg)):
            Wk, Wv = pl.transform_weights(shape, codex, sx, None, W_UK0, W_UV0)
            tp.tpla_transform_latent_paged(shape, codex, sx, None, mla_pool, scratch, used, len(used_np))
            ox = stepx.run(q_nope, q_pe, Wk, Wv, scratch, bt, lens, mu).double()
            gap[name] = float(torch.linalg.norm(ox - o_mla) / torch.linalg.norm(o_mla))
        del scratch, stepx

    out = {
        "metric": "latent-KV decode GB/s and % HBM roofline; µs per layer-step at 32K ctx",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "d_c": w.d_c, "g": w.g, "d_r": w.d_r,
                   "context": int(lens_np.max()), "tokens": int(lens_np.sum()), "page_tokens": pt,
                   "transform": w.transform, "n_splits": args.n_splits,
                   "step": "absorb + decode of all g slices (one split launch) + split merge and combine (one kernel), on one GPU"},
        "us_per_layer_step": ms_per_step * 1e3,
        "pct_hbm_roofline_step": 100.0 * value / HBM_PEAK_GBS,
        "settle": settled,
        "stages_us": {"absorb": us_absorb, "decode_shards(all slices, split+merge)": us_decode_all,
                      "decode_shard(one slice, split+merge)": us_decode, "combine": us_combine,
                      "decode_shards_combine(all slices, split + merge-and-combine kernel)": us_decode_combine,
                      "layer_step_with_separate_merge_and_combine": us_step_separate,
                      "output_projection(W_O, not in the step)": us_wo,
                      "layer_step_with_output_projection(absorb + tpla_decode_shards_project, bf16 block output)": us_block,
                      "one_device_share": us_absorb / w.g + us_decode + us_combine,
                      "layer_step_replayed_from_hip_graph": us_graph},
        "pool_copies_rotated": n_sets_rotated, "cache_resident": cache_resident,
        "tpla_vs_mla_output_gap": gap,
        "power_state": power_state,
        "pca_calibration": pca,
        "prefill_mla": prefill,
        "transform": p.transform,
        "roofline": dict({"bound": "hbm", "kernel": "decode split kernel, all g slices in one launch (tpla_decode_shards)",
                          "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name, "all_slices"),
                          "traffic_source": "profiles/decode_split_kernel_hbm_traffic.txt (quoted only while the kernel sources match the digest recorded there)",
                          "algorithmic_bytes_per_launch": launch_bytes, "modelled_all_traffic_bytes": all_traffic,
                          "streaming_read_ceiling_GB/s": ceiling,
                          "frac_of_streaming_read_ceiling": (achieved / ceiling) if ceiling else None}, **ls),
        "roofline_one_slice": {"bound": "hbm", "kernel": "decode split kernel, one slice per launch (tpla_decode_shard)",
                               "achieved": one_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": one_achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name, "one_slice"),
                               "launch_us": one_avg_ms * 1e3, "launches": len(one_ms),
                               "algorithmic_bytes_per_launch": shard_bytes},
        "mla_tp_reference": {"what": "same kernel, g=1: H heads over the unsliced (d_c + d_r)-wide cache = one device of MLA with head-split TP",
                             "launch_us": mla_ms * 1e3, "GB/s": mla_bytes / (mla_ms * 1e-3) / 1e9,
                             "frac": mla_bytes / (mla_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "time_ratio_mla_over_tpla_slice": mla_ms / one_avg_ms,
                             "bytes_ratio": mla_bytes / shard_bytes},
        "paper_context": "paper reports only ratios: TPLA vs MLA decode 1.79x (DeepSeek-V3) / 1.93x (Kimi-K2) at 32K, "
                         "2 GPUs of an unnamed model, BF16, FlashAttention-3, MoE removed (Sec. 5.4.1)",
    }
    if others is not None:
        out["other_workloads"] = others
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, model)
    print(json.dumps(out).replace("NaN", "null"))


if __name__ == "__main__":
    main()
