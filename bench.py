#!/usr/bin/env python3
"""Benchmark of the fused FlatQuant transform + INT4 quantization kernel on one MI355X.

A step is one pass of the whole online path (load tile, both contractions, absmax,
clip, round, pack, store) over one batch: one flatquant_transform_quant launch on the
LLaMA-2-7B prefill shape (T=2048 tokens, n=4096 = 64 x 64).  Inputs are resident in
HBM before the timed region; launches rotate over enough distinct input/output sets
that no launch finds its data in the 256 MB last-level cache ("cold", the headline),
and the same is repeated on a single set ("warm").  One rotation counter runs through warm-up and every timed region, so
no timed launch touches a set that any of the last ~1.2 GB of traffic touched.  The headline is the median of REPS
regions of --steps launches each (HIP events on the launch stream).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 MFMA, published
REPS = 5                       # timed regions per figure; the median is reported


def alg_bytes_per_token(n: int, per_token_clip: bool = True) -> int:
    """fp16 row in + packed codes out + fp16 step out (+ fp32 clip in)."""
    return 2 * n + n // 2 + 2 + (4 if per_token_clip else 0)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary shapes (decode, 70B, KV cache)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing and the parity check")
    ap.add_argument("--no-wide", action="store_true", help="skip the n=28672 (112 x 256) shape, which is MFMA-bound and needs 1.2 GB")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; the path shards over tokens without any exchange "
              "so no multi-GPU figure is produced. Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2410_09426_amd import binding as fq
    from paper_2410_09426_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    fq.lib()

    def dev(a):
        if a.dtype == np.float16:
            return torch.from_numpy(a.view(np.uint16).copy()).view(torch.float16).cuda()
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def time_region(fn, steps, warmup):
        """fn(i) enqueues step i on the current stream. Returns ms per step (events on that stream)."""
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for i in range(steps):
            fn(i)
        e1.record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return e0.elapsed_time(e1) / steps, wall_ms / steps

    class Rotation:
        """A step function over `nsets` buffer sets whose set index keeps counting through warm-up and all timed regions."""
        def __init__(self, launch, nsets):
            self.launch, self.nsets, self.count = launch, nsets, 0

        def __call__(self, _i=0):
            self.launch(self.count % self.nsets)
            self.count += 1

    def median_regions(fn, steps, warmup, reps=None):
        """Median over several regions of `steps` launches (REPS of them, 21 when a region is shorter than 200 launches: a
        short region carries its first launch on an idle stream and its last kernel's drain, several us in all, and
        scatters more).  The warm-up runs once, before the first region."""
        if reps is None:
            reps = REPS if steps >= 200 else 21
        ms, wall = [], []
        for r in range(reps):
            m, w = time_region(fn, steps, warmup if r == 0 else 0)
            ms.append(m)
            wall.append(w)
        return float(np.median(ms)), float(np.median(wall)), [float(v) for v in ms]

    def single_launch_us(fn, n=41):
        """One launch between two events, stream idle before it: launch latency + kernel, median of n."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        v = []
        for _ in range(n):
            torch.cuda.synchronize()
            e0.record(stream)
            fn()
            e1.record(stream)
            torch.cuda.synchronize()
            v.append(e0.elapsed_time(e1) * 1e3)
        return float(np.median(v))

    # ------------------------------------------------------------------ headline: prefill 7B
    c = synth.prefill_7b()
    T, n, n1, n2 = c.T, c.n, c.n1, c.n2
    P1, P2, clip = dev(c.P1), dev(c.P2), dev(c.clip)
    bytes_per_launch = T * alg_bytes_per_token(n)
    nsets = max(2, int(np.ceil(1.25e9 / bytes_per_launch)))          # > 1 GB of distinct lines in rotation
    x0 = dev(c.x)
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    codes = [torch.empty((T, n // 2), dtype=torch.uint8, device="cuda") for _ in range(nsets)]
    scales = [torch.empty((T,), dtype=torch.float16, device="cuda") for _ in range(nsets)]
    clips = [clip] + [clip.clone() for _ in range(nsets - 1)]

    # Device addresses are taken once: the host has to enqueue a launch in less time than the kernel runs (6 us), and
    # marshalling six tensors per call costs about 1 us of that in a short region (the binding takes plain addresses too).
    xa, ca, oa, sa = ([t.data_ptr() for t in v] for v in (xs, clips, codes, scales))
    p1a, p2a, st = P1.data_ptr(), P2.data_ptr(), stream.cuda_stream

    def launch_cold(k, s=st):
        fq.flatquant_transform_quant(xa[k], p1a, p2a, ca[k], 1, T, n1, n2, n, oa[k], sa[k], stream=s)

    def launch_probe(k, s=st):
        fq.flatquant_stream_probe(xa[k], T, n, n, oa[k], stream=s)

    step_cold = Rotation(launch_cold, nsets)
    step_warm = Rotation(lambda k: launch_cold(0), 1)
    # the same buffers and the same rotation without the arithmetic: what a copy-like launch of this size reaches on this
    # box.  Three launch shapes of the probe are timed; the fastest is the ceiling.
    step_probe = Rotation(launch_probe, nsets)

    def rotation_graph_us(launch, replays=9):
        """One launch per buffer set, all sets in order, captured in a HIP graph and replayed: us per launch with the host
        out of the loop (cold data as in the eager rotation).  None if capture is not available."""
        try:
            gs = torch.cuda.Stream()
            gs.wait_stream(stream)
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.stream(gs):
                launch(0, gs.cuda_stream)
                gs.synchronize()
                with torch.cuda.graph(gr, stream=gs):
                    for k in range(nsets):
                        launch(k, gs.cuda_stream)
                gr.replay()
                v = []
                for _ in range(replays):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(gs)
                    gr.replay()
                    e1.record(gs)
                    gs.synchronize()
                    v.append(e0.elapsed_time(e1) / nsets * 1e3)
            stream.wait_stream(gs)
            return float(np.median(v))
        except Exception as ex:   # a measurement nicety only
            print(f"bench.py: graph replay of the rotation skipped ({type(ex).__name__})", file=sys.stderr)
            return None
    probe_us = {}
    for shape, label in ((0, "persistent_two_wave_workgroups"), (1, "wave_per_row_nontemporal"), (2, "wave_per_row_plain_loads")):
        fq.fq_set_tuning("FLATQUANT_PROBE_SHAPE", shape)
        probe_us[label] = median_regions(step_probe, args.steps, args.warmup)[0] * 1e3
    fq.fq_set_tuning("FLATQUANT_PROBE_SHAPE", min(range(3), key=lambda i: list(probe_us.values())[i]))
    us_graph_probe = rotation_graph_us(launch_probe)   # (the probe writes into the code buffers: it runs before the kernel)
    fq.fq_set_tuning("FLATQUANT_PROBE_SHAPE", None)
    ms_probe = min(probe_us.values()) * 1e-3

    # The long regions run first: a chip that has just come out of idle takes a few hundred launches to settle (the
    # first regions of a fresh process measure 0.4 - 0.8 us per launch more than the later ones), and the K-launch
    # regions are meant to measure the kernel, not that transient.
    ms_cold_long = median_regions(step_cold, 1000, args.warmup, reps=3)[0]   # steady state, whatever --steps is
    ms_cold, wall_cold, cold_regions = median_regions(step_cold, args.steps, args.warmup)
    us_single_cold = single_launch_us(step_cold)
    ms_warm, _, _ = median_regions(step_warm, args.steps, args.warmup)
    us_graph_cold = rotation_graph_us(launch_cold)
    used = min(nsets, step_cold.count)
    for k in range(1, used):    # every rotation set that was used produced the same bytes
        assert torch.equal(codes[k], codes[0]) and torch.equal(scales[k].view(torch.int16), scales[0].view(torch.int16))

    tokens_per_s = T / (ms_cold * 1e-3)
    achieved = bytes_per_launch / (ms_cold * 1e-3) / 1e9
    flops_min = 2 * n * (n1 + n2) * T
    # HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counters: not measured in this run (a counter run is a run of
    # its own under rocprofv3), read from the committed summary of the same command
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "tq_prefill_7b_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("hbm_bytes_per_launch")
        traffic_source = "profiles/tq_prefill_7b_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the copy probe; not measured in this run)"

    out = {
        "metric": "fused transform+INT4-quant tokens/s (n=4096, T=2048)",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "repetitions": len(cold_regions),
        "ms_per_step": ms_cold,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "LLaMA-2-7B prefill shape: T=2048, n=4096 (n1=n2=64), per-token clip, fp16 in, INT4 codes + fp16 step out",
                   "cache": f"cold: rotation over {nsets} input/output sets ({nsets * bytes_per_launch / 1e9:.2f} GB)"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "frac_of_copy_probe": ms_probe / ms_cold},
        "detail": {
            "algorithmic_bytes_per_launch": bytes_per_launch,
            "us_per_call_cold": ms_cold * 1e3, "us_per_call_cold_regions": [v * 1e3 for v in cold_regions], "us_per_call_warm": ms_warm * 1e3,
            "us_single_launch_cold_idle_stream": us_single_cold, "us_per_call_cold_1000_step_regions": ms_cold_long * 1e3,
            "host_wall_us_per_call_cold": wall_cold * 1e3,
            "us_per_call_cold_graph_replay": us_graph_cold, "stream_probe_us_per_call_cold_graph_replay": us_graph_probe,
            "stream_probe_us_per_call_cold": ms_probe * 1e3, "stream_probe_us_by_shape": probe_us,
            "stream_probe_gbs": T * (2 * n + n // 2) / (ms_probe * 1e-3) / 1e9,
            "tokens_per_s_warm": T / (ms_warm * 1e-3),
            "gbs_warm": bytes_per_launch / (ms_warm * 1e-3) / 1e9,
            "mfma_tflops_min_count": flops_min / (ms_cold * 1e-3) / 1e12,
            "mfma_frac_of_f16_peak_min_count": flops_min / (ms_cold * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS,
        },
    }

    # ------------------------------------------------------------------ reference point: what a plain copy reaches on this machine
    src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")       # 1 GB: far larger than the 256 MB last-level cache
    dst = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
    ms_copy, _ = time_region(lambda i: dst.copy_(src), 20, 3)
    out["detail"]["torch_copy_1GB_gbs_read_plus_write"] = 2 * dst.numel() / (ms_copy * 1e-3) / 1e9
    del src, dst

    # ------------------------------------------------------------------ secondary shapes
    if not args.no_extras:
        extras = {}

        def graph_replay_us(name, launch, per_graph=20, replays=25):
            """`launch(s)` enqueues one step on stream s; 20 of them are captured in a HIP graph and replayed. us per step."""
            try:
                gs = torch.cuda.Stream()
                gs.wait_stream(stream)
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.stream(gs):
                    launch(gs)
                    gs.synchronize()
                    with torch.cuda.graph(gr, stream=gs):
                        for _ in range(per_graph):
                            launch(gs)
                    for _ in range(3):
                        gr.replay()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(gs)
                    for _ in range(replays):
                        gr.replay()
                    e1.record(gs)
                    gs.synchronize()
                stream.wait_stream(gs)
                return e0.elapsed_time(e1) / (replays * per_graph) * 1e3
            except Exception as ex:   # a measurement nicety only
                print(f"bench.py: graph replay for {name} skipped ({type(ex).__name__})", file=sys.stderr)
                return None

        def time_shape(name, Tn, a, b, steps, warmup, cold_sets=1, use_p1=True, use_p2=True):
            nn = a * b
            g = torch.Generator(device="cuda").manual_seed(1234 + nn)
            col = torch.ones(nn, device="cuda")
            idx = torch.randperm(nn, generator=g, device="cuda")[: max(1, nn // 100)]
            col[idx] = torch.empty(idx.numel(), device="cuda").uniform_(20, 100, generator=g)
            xsets = []
            for _ in range(cold_sets):
                xx = torch.empty((Tn, nn), dtype=torch.float16, device="cuda")
                for r0 in range(0, Tn, 2048):
                    r1 = min(Tn, r0 + 2048)
                    blk = torch.randn((r1 - r0, nn), generator=g, device="cuda") * col
                    xx[r0:r1] = blk.clamp_(-30000, 30000).half()
                xsets.append(xx)
            p1 = (torch.eye(a, device="cuda") + 0.05 * torch.randn((a, a), generator=g, device="cuda")).half()
            p2 = (torch.eye(b, device="cuda") + 0.05 * torch.randn((b, b), generator=g, device="cuda")).half()
            cl = torch.sigmoid(torch.empty(Tn, device="cuda").uniform_(1.5, 3.0, generator=g)).float()
            oc = [torch.empty((Tn, nn // 2), dtype=torch.uint8, device="cuda") for _ in range(cold_sets)]
            os_ = [torch.empty((Tn,), dtype=torch.float16, device="cuda") for _ in range(cold_sets)]

            st = Rotation(lambda k: fq.flatquant_transform_quant(xsets[k], p1 if use_p1 else None, p2 if use_p2 else None, cl, 1, Tn, a, b, nn,
                                                                 oc[k], os_[k], stream=stream), cold_sets)
            ms = median_regions(st, steps, warmup)[0]
            by = Tn * alg_bytes_per_token(nn)
            pad32 = 32 * ((a + 31) // 32)
            graph_us = None
            if Tn <= 256:   # launch-bound shapes: also replay the launches from a HIP graph, which takes the host out of the figure
                graph_us = graph_replay_us(name, lambda gs: fq.flatquant_transform_quant(
                    xsets[0], p1 if use_p1 else None, p2 if use_p2 else None, cl, 1, Tn, a, b, nn, oc[0], os_[0], stream=gs))
            extras[name] = {"T": Tn, "n1": a, "n2": b, "us_per_call": ms * 1e3, "us_per_call_graph_replay": graph_us, "tokens_per_s": Tn / (ms * 1e-3),
                            "gbs": by / (ms * 1e-3) / 1e9, "hbm_frac": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "mfma_tflops_min_count": 2 * nn * (a + b) * Tn / (ms * 1e-3) / 1e12,
                            # MFMA work as issued: row tiles padded to 32, K of the second contraction padded to 16 and doubled (hi + lo)
                            "mfma_frac_of_f16_peak_as_issued": (2 * pad32 * b * b + 4 * b * pad32 * 16 * ((a + 15) // 16)) * Tn / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS}
            del xsets, oc, os_

        time_shape("decode_4096", 64, 64, 64, 500, 50)
        time_shape("decode_11008", 64, 86, 128, 500, 50)
        time_shape("prefill_70b_8192", 16384, 64, 128, 20, 4, cold_sets=4)
        # the batch-64 row of the paper's kernel table (Table "kernel speedup"): 64 x 2048 tokens of 4096 channels, 1.3 GB per launch
        time_shape("prefill_7b_batch64", 131072, 64, 64, 6, 2, cold_sets=1)
        # online part of P_o for LLaMA-2-7B: 32 heads x 128, left factor only (the per-head factor is fused offline)
        time_shape("p_o_left_only_32x128", 2048, 32, 128, 200, 20, cold_sets=60, use_p2=False)
        if not args.no_wide:
            time_shape("prefill_70b_28672", 16384, 112, 256, 5, 1, cold_sets=1)

        # MXFP4 output on the headline shape (2n + n/2 + n/32 bytes per token + clip), cold rotation like the headline
        mxs = [torch.empty((T, n // 32), dtype=torch.uint8, device="cuda") for _ in range(nsets)]
        mxc = [torch.empty((T, n // 2), dtype=torch.uint8, device="cuda") for _ in range(nsets)]

        st_mx = Rotation(lambda k: fq.flatquant_transform_mxfp4(xs[k], P1, P2, clips[k], 1, T, n1, n2, n, mxc[k], mxs[k], stream=stream), nsets)
        ms = median_regions(st_mx, 200, 20)[0]
        by = T * (2 * n + n // 2 + n // 32 + 4)
        extras["mxfp4_prefill_7b"] = {"T": T, "n1": n1, "n2": n2, "us_per_call": ms * 1e3, "tokens_per_s": T / (ms * 1e-3),
                                      "gbs": by / (ms * 1e-3) / 1e9, "hbm_frac": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del mxs, mxc

        # KV-cache variant: 32768 tokens x 8 heads x 128, K and V alternate (two distinct 67 MB inputs + more sets for cold)
        Tk, H, D = 32768, 8, 128
        g = torch.Generator(device="cuda").manual_seed(99)
        kvsets = [torch.randn((Tk, H, D), generator=g, device="cuda").half() for _ in range(8)]
        Pk = (torch.eye(D, device="cuda").expand(H, D, D) + 0.05 * torch.randn((H, D, D), generator=g, device="cuda")).half().contiguous()
        kc = [torch.empty((Tk * H, D // 2), dtype=torch.uint8, device="cuda") for _ in range(8)]
        ks = [torch.empty((Tk * H,), dtype=torch.float16, device="cuda") for _ in range(8)]
        kz = [torch.empty((Tk * H,), dtype=torch.float16, device="cuda") for _ in range(8)]

        st_kv = Rotation(lambda k: fq.flatquant_kv_transform_quant(kvsets[k], Pk, H, 0.95, Tk, H, D, kc[k], ks[k], kz[k], stream=stream), 8)
        ms = median_regions(st_kv, 40, 8)[0]
        by = Tk * H * (2 * D + D // 2 + 4)
        extras["kv_cache"] = {"T": Tk, "H": H, "D": D, "us_per_call": ms * 1e3, "groups_per_s": Tk * H / (ms * 1e-3),
                              "gbs": by / (ms * 1e-3) / 1e9, "hbm_frac": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        Pshared = Pk[:1].contiguous()                     # the paper's setting: one P_h per layer, shared by the heads

        st_kvs = Rotation(lambda k: fq.flatquant_kv_transform_quant(kvsets[k], Pshared, 1, 0.95, Tk, H, D, kc[k], ks[k], kz[k], stream=stream), 8)
        ms_s = median_regions(st_kvs, 40, 8)[0]
        extras["kv_cache_shared_matrix"] = {"T": Tk, "H": H, "D": D, "us_per_call": ms_s * 1e3, "groups_per_s": Tk * H / (ms_s * 1e-3),
                                            "gbs": by / (ms_s * 1e-3) / 1e9, "hbm_frac": by / (ms_s * 1e-3) / 1e9 / HBM_PEAK_GBS}
        for bits in (3, 2):   # lower-bit caches: same kernel, D * bits / 8 code bytes per group (into the same buffers)
            st_kvb = Rotation(lambda k, bits=bits: fq.flatquant_kv_transform_quant_bits(kvsets[k], Pk, H, 0.95, bits, Tk, H, D, kc[k], ks[k], kz[k], stream=stream), 8)
            ms = median_regions(st_kvb, 40, 8)[0]
            by = Tk * H * (2 * D + D * bits // 8 + 4)
            extras[f"kv_cache_{bits}bit"] = {"T": Tk, "H": H, "D": D, "us_per_call": ms * 1e3, "groups_per_s": Tk * H / (ms * 1e-3),
                                            "gbs": by / (ms * 1e-3) / 1e9, "hbm_frac": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        # a decode step's share of the cache: 64 new tokens x 32 heads (one launch each for K and V in a layer)
        Td, Hd = 64, 32
        kvd = torch.randn((Td, Hd, D), generator=g, device="cuda").half()
        Pd = (torch.eye(D, device="cuda").expand(Hd, D, D) + 0.05 * torch.randn((Hd, D, D), generator=g, device="cuda")).half().contiguous()

        def st_kvd(i, s_=None):
            fq.flatquant_kv_transform_quant(kvd, Pd, Hd, 0.95, Td, Hd, D, kc[0], ks[0], kz[0], stream=s_ or stream)
        ms = median_regions(st_kvd, 200, 20)[0]
        extras["kv_cache_decode"] = {"T": Td, "H": Hd, "D": D, "us_per_call": ms * 1e3,
                                     "us_per_call_graph_replay": graph_replay_us("kv_cache_decode", lambda gs: st_kvd(0, gs))}
        # query side: per-head transform, fp16 out (same tensors, 2 x 2D bytes per group)
        qo = [torch.empty((Tk, H, D), dtype=torch.float16, device="cuda") for _ in range(4)]

        st_q = Rotation(lambda k: fq.flatquant_head_transform(kvsets[k], Pk, H, Tk, H, D, qo[k % 4], stream=stream), 8)
        ms = median_regions(st_q, 40, 8)[0]
        by = Tk * H * 4 * D
        extras["head_transform_fp16"] = {"T": Tk, "H": H, "D": D, "us_per_call": ms * 1e3, "gbs": by / (ms * 1e-3) / 1e9,
                                         "hbm_frac": by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del kvsets, kc, ks, kz, qo
        # ---- the consumer: W4A4 matrix product on int8 MFMA, and the whole quantized linear layer (transform + quantization of
        # the activations, then the product with pre-quantized weights), as fractions of the MFMA peak of its data type
        INT8_PEAK_TOPS = 5000.0

        def weight_copies(Tn, nbytes):   # prefill: one copy (the product is compute-bound); decode: 320 MB worth, past L2 + Infinity Cache
            return 1 if Tn > 128 else max(2, -(-320_000_000 // nbytes))

        def time_layer(name, Tn, mo, a, b, steps, warmup):
            nn = a * b
            g = torch.Generator(device="cuda").manual_seed(77 + mo + nn + Tn)
            x = (torch.randn((Tn, nn), generator=g, device="cuda")).half()
            p1 = (torch.eye(a, device="cuda") + 0.05 * torch.randn((a, a), generator=g, device="cuda")).half()
            p2 = (torch.eye(b, device="cuda") + 0.05 * torch.randn((b, b), generator=g, device="cuda")).half()
            cl = torch.full((Tn,), 0.9, device="cuda")
            xc = torch.empty((Tn, nn // 2), dtype=torch.uint8, device="cuda")
            xs_ = torch.empty((Tn,), dtype=torch.float16, device="cuda")
            # few tokens: the weights are the traffic, so they rotate through more copies than the caches hold (a decode
            # step reads every layer's weights from HBM); the FP16 weights beside them likewise
            nwc = weight_copies(Tn, mo * nn // 2)
            wcs = [torch.randint(0, 256, (mo, nn // 2), generator=g, dtype=torch.uint8, device="cuda") for _ in range(nwc)]
            wc = wcs[0]
            ws = (torch.rand((mo,), generator=g, device="cuda") * 1e-3 + 1e-4).half()
            y = torch.empty((Tn, mo), dtype=torch.float16, device="cuda")
            st_gemm = Rotation(lambda k: fq.flatquant_w4a4_gemm(xc, xs_, wcs[k], ws, Tn, mo, nn, y, mo, stream=stream), nwc)

            def layer(k):
                fq.flatquant_transform_quant(x, p1, p2, cl, 1, Tn, a, b, nn, xc, xs_, stream=stream)
                fq.flatquant_w4a4_gemm(xc, xs_, wcs[k], ws, Tn, mo, nn, y, mo, stream=stream)
            st_layer = Rotation(layer, nwc)
            st_layer()
            ms_g, ms_l = median_regions(st_gemm, steps, warmup)[0], median_regions(st_layer, steps, warmup)[0]
            ops = 2.0 * Tn * mo * nn
            layer_graph = None
            if Tn <= 256:
                def one_layer(gs):
                    fq.flatquant_transform_quant(x, p1, p2, cl, 1, Tn, a, b, nn, xc, xs_, stream=gs)
                    fq.flatquant_w4a4_gemm(xc, xs_, wc, ws, Tn, mo, nn, y, mo, stream=gs)
                layer_graph = graph_replay_us(name, one_layer)
            extras[name] = {"T": Tn, "m": mo, "n": nn, "weight_copies_rotated": nwc, "layer_us_graph_replay_weights_cached": layer_graph, "gemm_us": ms_g * 1e3, "gemm_tops": ops / (ms_g * 1e-3) / 1e12,
                            "gemm_frac_of_int8_mfma_peak": ops / (ms_g * 1e-3) / 1e12 / INT8_PEAK_TOPS,
                            "layer_us_transform_quant_plus_gemm": ms_l * 1e3}

        def time_mx_layer(name, Tn, mo, a, b, steps, warmup):   # the same layer with MXFP4 on both factors (scaled FP4 MFMA)
            nn = a * b
            g = torch.Generator(device="cuda").manual_seed(177 + mo + nn + Tn)
            x = (torch.randn((Tn, nn), generator=g, device="cuda")).half()
            p1 = (torch.eye(a, device="cuda") + 0.05 * torch.randn((a, a), generator=g, device="cuda")).half()
            p2 = (torch.eye(b, device="cuda") + 0.05 * torch.randn((b, b), generator=g, device="cuda")).half()
            cl = torch.full((Tn,), 0.9, device="cuda")
            xc = torch.empty((Tn, nn // 2), dtype=torch.uint8, device="cuda")
            xe = torch.empty((fq.fq_mxfp4_tiled_scale_bytes(Tn, nn),), dtype=torch.uint8, device="cuda")
            nwc = weight_copies(Tn, mo * nn // 2)
            wcs = [torch.randint(0, 256, (mo, nn // 2), generator=g, dtype=torch.uint8, device="cuda") for _ in range(nwc)]
            we = torch.randint(112, 118, (fq.fq_mxfp4_tiled_scale_bytes(mo, nn),), generator=g, dtype=torch.uint8, device="cuda")
            y = torch.empty((Tn, mo), dtype=torch.float16, device="cuda")
            st_gemm = Rotation(lambda k: fq.flatquant_mxfp4_gemm(xc, xe, wcs[k], we, Tn, mo, nn, y, mo, stream=stream), nwc)

            def layer(k):
                fq.flatquant_transform_mxfp4_tiled(x, p1, p2, cl, 1, Tn, a, b, nn, xc, xe, stream=stream)
                fq.flatquant_mxfp4_gemm(xc, xe, wcs[k], we, Tn, mo, nn, y, mo, stream=stream)
            st_layer = Rotation(layer, nwc)
            st_layer()
            ms_g, ms_l = median_regions(st_gemm, steps, warmup)[0], median_regions(st_layer, steps, warmup)[0]
            ops = 2.0 * Tn * mo * nn
            extras[name] = {"T": Tn, "m": mo, "n": nn, "weight_copies_rotated": nwc, "gemm_us": ms_g * 1e3, "gemm_tflops": ops / (ms_g * 1e-3) / 1e12,
                            "gemm_frac_of_fp4_mfma_peak": ops / (ms_g * 1e-3) / 1e12 / 10100.0,
                            "layer_us_transform_quant_plus_gemm": ms_l * 1e3}

        time_mx_layer("mxfp4_layer_prefill_qkvo_7b", 2048, 4096, 64, 64, 50, 5)
        time_mx_layer("mxfp4_layer_prefill_down_7b", 2048, 4096, 86, 128, 30, 5)
        time_layer("w4a4_layer_prefill_qkvo_7b", 2048, 4096, 64, 64, 50, 5)
        time_layer("w4a4_layer_prefill_down_7b", 2048, 4096, 86, 128, 30, 5)
        time_layer("w4a4_layer_decode_qkvo_7b", 64, 4096, 64, 64, 200, 20)
        time_layer("w4a4_layer_decode_down_7b", 64, 4096, 86, 128, 200, 20)
        time_layer("w4a4_layer_decode_batch1_qkvo_7b", 1, 4096, 64, 64, 200, 20)
        time_mx_layer("mxfp4_layer_decode_qkvo_7b", 64, 4096, 64, 64, 200, 20)
        time_mx_layer("mxfp4_layer_decode_down_7b", 64, 4096, 86, 128, 200, 20)
        time_mx_layer("mxfp4_layer_decode_batch1_qkvo_7b", 1, 4096, 64, 64, 200, 20)
        out["extras"] = extras

    # ------------------------------------------------------------------ CPU oracle: baseline timing + parity of the timed buffers
    if not args.no_cpu:
        from oracle import flatquant_oracle as fo
        from oracle import parity
        cores = len(os.sched_getaffinity(0))     # the cores this process may run on
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            blas_threads = None
        t0 = time.perf_counter()
        P = fo.kron_dense(c.P1, c.P2)
        t_kron = time.perf_counter() - t0
        reps, t_run = 0, 0.0
        while reps < 3 or (t_run < 10.0 and reps < 400):
            t0 = time.perf_counter()
            res = fo.transform_quant(c.x, c.P1, c.P2, c.clip, P=P)
            t_run += time.perf_counter() - t0
            reps += 1
        out["cpu_baseline"] = {"value": T * reps / t_run, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"all {T} tokens of the headline workload, {reps} passes of the fp64 dense-Kronecker oracle "
                                         f"(numpy + its BLAS, thread pool of {blas_threads}); building the {n}x{n} matrix once took {t_kron:.2f} s and is not in the rate"}
        # a second CPU line: the same oracle through the factored form of Eq. (2) (two small contractions per token)
        reps_f, t_f = 0, 0.0
        while reps_f < 2 or (t_f < 5.0 and reps_f < 400):
            t0 = time.perf_counter()
            yf = fo.affine_transform_factored(c.x, c.P1, c.P2)
            fo.quantize_sym_int4(yf, c.clip)
            t_f += time.perf_counter() - t0
            reps_f += 1
        out["detail"]["cpu_oracle_factored_form_tokens_per_s"] = T * reps_f / t_f
        rep = parity.check_sym(res["y"], c.clip, codes[0].cpu().numpy(),
                               scales[0].cpu().view(torch.int16).numpy().view(np.float16))
        out["detail"]["parity_on_timed_buffers"] = rep

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
