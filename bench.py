#!/usr/bin/env python3
"""Benchmark of the KVmix hot path on one MI355X.

One "step" = one decode step of the whole hot path over all layers of the workload: per layer,
kvmix_decode_step appends the new token's K/V to the fp16 window (flushing 32 aged tokens through
quantize-and-pack when the window overflows) and runs the fused mixed-bit decode attention. Inputs are synthetic
(kvmix_synth) and resident in HBM before the timed region.

Prints ONE JSON line: throughput in decode tokens/s of the headline workload, the HBM roofline of the attention kernel
(algorithmic bytes per launch / average launch duration, measured with events on the launch stream over an
attention-only timed region), a load-only pass of the same launch shape and size timed in the same run
(`stream_ceiling_gbs`), the CPU oracle timed on a bounded sample, and short runs of the other benchmark
configurations under `other_configs`.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import kvmix_synth as synth  # noqa: E402

HBM_PEAK_GBS = 8000.0
HEADLINE = "cfg2_llama2_7b"
# HBM bytes per attention launch of the headline workload from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# command (summary under profiles/), valid for the kernel source whose hash is recorded with it; a bench run on any
# other kernel source reports null.
TRAFFIC_RECORD = os.path.join(ROOT, "paper_2506_08018_amd", "measured_traffic.json")


def kernel_source_hash():
    h = hashlib.sha256()
    for name in ("kvmix_attn.hip", "kvmix_common.hpp"):
        h.update(open(os.path.join(ROOT, "paper_2506_08018_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(config):
    try:
        rec = json.load(open(TRAFFIC_RECORD))
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_sha256_16") != kernel_source_hash():
        return None
    return rec.get("bytes_per_launch", {}).get(config)


def algorithmic_bytes(units, n_q, n_w, kb, vb):
    """Bytes the method itself must move for one layer's decode attention (D = 128, group 32):
    packed token: 16*bK + 16*bV code bytes + 32 bytes of fp16 scale/min; window token: 512 bytes."""
    return units * (n_q * (16 * kb + 16 * vb + 32) + n_w * 512)


def build_layers(cfg, device, seed):
    import torch
    import paper_2506_08018_amd as kv
    L, B, Hq, Hkv, T, W = cfg["L"], cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["T"], cfg["W"]
    kbits, vbits = synth.bit_table(L, seed)
    if cfg["bits"] == "2/2":
        kbits[:], vbits[:] = 2, 2
    shape = kv.Shape(B, Hq, Hkv)
    # start 8 tokens short of T with 24 tokens above the window length, so that a flush of 32 aged tokens
    # falls inside a short run and the context is T right after it
    n_w0 = W + 24
    n_q0 = T - 8 - n_w0
    assert n_q0 % 32 == 0 and n_q0 >= 0
    layers = []
    prefill_s = 0.0
    # the first launch of a kernel instance loads its code object: one tiny launch per bit pair keeps that out of
    # the timed prefill launches below
    for kb, vb in sorted(set(zip(kbits.tolist(), vbits.tolist()))):
        wshape, wlc = kv.Shape(1, Hq // Hkv, 1), kv.LayerCfg(int(kb), int(vb), W)
        wcache = kv.LayerCache(wshape, wlc, T_cap=64, W_cap=W + 32, device=device)
        wk = torch.zeros((1, 1, 32, 128), dtype=torch.float16, device=device)
        kv.quantize_pack(wshape, wlc, wk, wk.clone(), wcache)
    torch.cuda.synchronize()
    for l in range(L):
        lc = kv.LayerCfg(int(kbits[l]), int(vbits[l]), W)
        cache = kv.LayerCache(shape, lc, T_cap=T + synth.GEN_ROOM, W_cap=W + 32, device=device)
        q, k, v = synth.gen_layer_torch(device, seed, l, B, Hq, Hkv, n_q0 + n_w0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        kv.quantize_pack(shape, lc, k[:, :, :n_q0], v[:, :, :n_q0], cache)
        e1.record()
        cache.set_window(k[:, :, n_q0:], v[:, :, n_q0:])
        torch.cuda.synchronize()
        prefill_s += e0.elapsed_time(e1) * 1e-3
        layers.append(dict(cfg=lc, cache=cache, q=q, out=torch.zeros_like(q)))
        del k, v
    torch.cuda.synchronize()
    # the prefill quantize-and-pack of the n_q0 aged tokens, one launch per layer: 2 B read per element of K and V,
    # (b + 1) / 8 B written per element (codes + fp16 scale and minimum per group of 32)
    elems = B * Hkv * n_q0 * 128
    moved = sum(elems * (4 + (int(kb) + int(vb) + 2) / 8.0) for kb, vb in zip(kbits, vbits))
    prefill = {"tokens": n_q0, "ms_all_layers": prefill_s * 1e3, "hbm_gbs": moved / prefill_s / 1e9,
               "frac_of_peak": moved / prefill_s / 1e9 / HBM_PEAK_GBS, "bytes_moved": moved}
    return shape, layers, kbits, vbits, prefill


def cpu_baseline(cfg, seed, kbits, vbits, target_s=12.0):
    """The oracle's decode attention (and quantize-pack) timed on the host cores for a bounded sample:
    whole kv heads of layer 0 (same recipe, numpy stream), scaled linearly to the full workload
    (units are independent)."""
    from oracle import kvmix_ref
    from oracle.kvmix_ref import RefCache
    L, B, Hq, Hkv, T, W = cfg["L"], cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["T"], cfg["W"]
    G = Hq // Hkv
    threads = kvmix_ref.num_threads()
    n_units = max(threads, 8)
    total_units = L * B * Hkv
    Hs = min(Hkv, n_units)
    Bs = max(1, min(B, n_units // Hs))
    n_q = (T - W) // 32 * 32
    q, k, v = synth.gen_layer_numpy(seed, 0, Bs, Hs * G, Hs, T)
    u16 = lambda a: np.ascontiguousarray(a).view(np.uint16)
    t_attn, t_qp, reps = 0.0, 0.0, 0
    while t_attn < target_s and reps < 1000:
        rc = RefCache(Bs, Hs * G, Hs, int(kbits[0]), int(vbits[0]), W, n_q, W + 32)
        t0 = time.perf_counter()
        rc.quantize_pack(u16(k[:, :, :n_q]), u16(v[:, :, :n_q]))
        t1 = time.perf_counter()
        rc.set_window(u16(k[:, :, n_q:]), u16(v[:, :, n_q:]))
        t2 = time.perf_counter()
        st, _ = rc.decode_attn(u16(q))
        t3 = time.perf_counter()
        assert st == 0
        t_qp += t1 - t0
        t_attn += t3 - t2
        reps += 1
    per_unit = t_attn / (reps * Bs * Hs)
    step_s = per_unit * total_units
    out = {
        "value": B / step_s, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": f"decode attention of {Bs * Hs} of {total_units} (layer,batch,kv-head) units (layer 0 bits "
                  f"K{int(kbits[0])}/V{int(vbits[0])}, context {T}), {reps} repetitions, {t_attn:.1f} s of CPU time, scaled "
                  f"linearly to all units; OpenMP over units",
        "quantize_pack_tokens_per_s": (reps * Bs * Hs * n_q) / t_qp,
    }
    if target_s >= 10.0:
        # the same attention on one thread, one unit, a few seconds
        kvmix_ref.set_num_threads(1)
        rc1 = RefCache(1, G, 1, int(kbits[0]), int(vbits[0]), W, n_q, W + 32)
        rc1.quantize_pack(u16(k[:1, :1, :n_q]), u16(v[:1, :1, :n_q]))
        rc1.set_window(u16(k[:1, :1, n_q:]), u16(v[:1, :1, n_q:]))
        t1, r1 = 0.0, 0
        while t1 < 3.0 and r1 < 1000:
            t0 = time.perf_counter()
            rc1.decode_attn(u16(q[:1, :G]))
            t1 += time.perf_counter() - t0
            r1 += 1
        kvmix_ref.set_num_threads(threads)
        out["one_thread_value"] = B / (t1 / r1 * total_units)
    return out


def measure(name, steps, warmup, seed, n_splits, device, cpu_s):
    """Builds the workload `name` in HBM, times `steps` decode steps after `warmup`, then an attention-only region and
    a load-only pass of the same launch shape; returns the figures of one configuration."""
    import torch
    import paper_2506_08018_amd as kv
    cfg = synth.CONFIGS[name]
    L, B, Hq, Hkv = cfg["L"], cfg["B"], cfg["Hq"], cfg["Hkv"]
    units = B * Hkv
    shape, layers, kbits, vbits, prefill = build_layers(cfg, device, seed)
    ws = torch.zeros(kv.workspace_bytes(shape, cfg["T"] + synth.GEN_ROOM), dtype=torch.uint8, device=device)
    g = torch.Generator(device=device)
    g.manual_seed(seed + 77)
    n_new = steps + warmup + 1
    k_new = torch.randn((n_new, L, B, Hkv, 128), generator=g, device=device, dtype=torch.float32).to(torch.float16)
    v_new = torch.randn((n_new, L, B, Hkv, 128), generator=g, device=device, dtype=torch.float32).to(torch.float16)

    # host side kept lean (tensor views and the stream handle are made once): the launches must be issued
    # faster than the GPU runs them
    hstream = torch.cuda.current_stream().cuda_stream
    new_views = [[(k_new[i, l], v_new[i, l]) for l in range(L)] for i in range(n_new)]

    def step(i):
        for ly, (kn, vn) in zip(layers, new_views[i]):
            kv.decode_step(shape, ly["cfg"], kn, vn, ly["q"], ly["cache"], ly["out"], ws, n_splits=n_splits, stream=hstream)

    def layer_bytes():
        return [algorithmic_bytes(units, ly["cache"].n_q, ly["cache"].n_w, ly["cfg"].k_bits, ly["cfg"].v_bits) for ly in layers]

    def attn_only():
        for ly in layers:
            kv.decode_attn(shape, ly["cfg"], ly["q"], ly["cache"], ly["out"], ws, n_splits=n_splits, stream=hstream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    total_bytes = 0
    marks[0].record()
    for i in range(warmup, warmup + steps):
        step(i)
        marks[i - warmup + 1].record()
        total_bytes += sum(layer_bytes())
    host_elapsed = time.perf_counter() - t0
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]

    # attention-only timed region: average launch duration of the dominant kernel, events on the launch stream
    attn_only()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(steps, 10)
    e0.record()
    for _ in range(reps):
        attn_only()
    e1.record()
    torch.cuda.synchronize()
    attn_ms = e0.elapsed_time(e1) / reps
    launch_us = attn_ms * 1e3 / L
    lb = layer_bytes()
    bytes_per_launch = float(np.mean(lb))
    achieved = bytes_per_launch / (launch_us * 1e-6) / 1e9

    # load-only pass: per layer the same number of bytes from that layer's own cache buffer, in the attention
    # launch's shape (as many workgroups of 768 threads), timed the same way
    n_wg = units * max(1, min(256 // units, 64)) if n_splits == 0 else units * n_splits
    sink = torch.zeros(4, dtype=torch.int32, device=device)

    def stream_only():
        for ly, nb in zip(layers, lb):
            buf = ly["cache"].packed
            kv.stream_read(buf, n_wg, 768, nbytes=min(nb, buf.numel()) // 16 * 16, sink=sink, stream=hstream)

    stream_only()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        stream_only()
    e1.record()
    torch.cuda.synchronize()
    stream_bytes = float(np.mean([min(nb, ly["cache"].packed.numel()) // 16 * 16 for ly, nb in zip(layers, lb)]))
    stream_us = e0.elapsed_time(e1) / reps * 1e3 / L
    stream_gbs = stream_bytes / (stream_us * 1e-6) / 1e9

    res = {
        "workload": name, "steps": steps, "warmup": warmup,
        "tokens_per_s": B * steps / elapsed, "ms_per_step": elapsed / steps * 1e3,
        "ms_per_step_event_median": float(np.median(per_step_ms)), "ms_per_step_event_min": float(np.min(per_step_ms)),
        "step_hbm_gbs": total_bytes / elapsed / 1e9, "step_frac_of_peak": total_bytes / elapsed / 1e9 / HBM_PEAK_GBS,
        "host_issue_ms_per_step": host_elapsed / steps * 1e3,
        "attn_only_ms_per_step": attn_ms, "attn_only_tokens_per_s": B / (attn_ms * 1e-3),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(name),
                     "kernel": "decode_attn_kernel", "bytes_per_launch": bytes_per_launch, "launch_us": launch_us,
                     "launches_timed": reps * L,
                     "stream_ceiling_gbs": stream_gbs, "stream_ceiling_launch_us": stream_us,
                     "stream_ceiling_note": "load-only kernel, same grid and bytes per launch, same run"},
        "prefill_quantize_pack": prefill,
        "packed_cache_bytes": int(sum(ly["cache"].nbytes() for ly in layers)),
        "layers": L, "batch": B, "q_heads": Hq, "kv_heads": Hkv, "context": cfg["T"], "window": cfg["W"],
        "mean_k_bits": float(np.mean(kbits)), "mean_v_bits": float(np.mean(vbits)),
    }
    if cpu_s > 0:
        res["cpu_baseline"] = cpu_baseline(cfg, seed, kbits, vbits, cpu_s)
    del layers, ws, k_new, v_new, new_views
    torch.cuda.empty_cache()
    return res


def widened_rows(device, seed):
    """Short timings of the calls beyond the headline step, one layer each at the headline's batch and context:
    multi-query attention (71 query heads padded to 72 on one kv head), a 4096-token chunk through kvmix_append_tokens,
    and attention on a cache whose Keys and Values age at fronts of their own."""
    import torch
    import paper_2506_08018_amd as kv
    out = {}
    hstream = torch.cuda.current_stream().cuda_stream

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3      # microseconds per call

    c2 = synth.CONFIGS[HEADLINE]
    T, W = c2["T"], c2["W"]
    # -- multi-query attention: B = 32 sequences, 72 query heads on 1 kv head, 4 layers in rotation
    B, Hq, Hkv = 32, 72, 1
    shape, lc = kv.Shape(B, Hq, Hkv), kv.LayerCfg(2, 2, W)
    n_w, n_q = W + 24, T - 8 - (W + 24)
    caches = []
    for l in range(4):
        c = kv.LayerCache(shape, lc, T + synth.GEN_ROOM, W + 32, device=device)
        q, k, v = synth.gen_layer_torch(device, seed, 100 + l, B, Hq, Hkv, n_q + n_w)
        kv.quantize_pack(shape, lc, k[:, :, :n_q], v[:, :, :n_q], c)
        c.set_window(k[:, :, n_q:], v[:, :, n_q:])
        caches.append(c)
        del k, v
    o = torch.zeros_like(q)
    ws = torch.zeros(kv.workspace_bytes(shape, T + synth.GEN_ROOM), dtype=torch.uint8, device=device)
    state = {"i": 0}

    def mqa():
        kv.decode_attn(shape, lc, q, caches[state["i"] % 4], o, ws, stream=hstream)
        state["i"] += 1
    us = timed(mqa, 80)
    nb = algorithmic_bytes(B * Hkv, n_q, n_w, 2, 2)
    out["mqa_72_heads_1_kv_head"] = {"batch": B, "q_heads": Hq, "kv_heads": Hkv, "context": n_q + n_w, "bits": "2/2", "launch_us": us,
                                      "bytes_per_launch": nb, "hbm_gbs": nb / us / 1e3, "frac_of_peak": nb / us / 1e3 / HBM_PEAK_GBS,
                                      "note": "9 head blocks per unit read the same records: bytes counted once"}
    del caches, ws
    # -- one 4096-token chunk of new tokens through kvmix_append_tokens (chunked prefill) at the headline shape
    B, Hq, Hkv = c2["B"], c2["Hq"], c2["Hkv"]
    shape, lc = kv.Shape(B, Hq, Hkv), kv.LayerCfg(2, 2, W)
    n_chunk = 4096
    c = kv.LayerCache(shape, lc, 2 * n_chunk + 64, W + 32, device=device)
    _, k, v = synth.gen_layer_torch(device, seed, 200, B, Hq, Hkv, n_chunk)

    def chunk():
        c.c.n_q, c.c.n_w, c.c.w0 = 0, 0, 0
        kv.append_tokens(shape, lc, k, v, c)
    us = timed(chunk, 10)
    elems = B * Hkv * n_chunk * 128
    moved = elems * (4 + (2 + 2 + 2) / 8.0)
    out["append_tokens_4096_chunk"] = {"batch": B, "kv_heads": Hkv, "tokens": n_chunk, "bits": "2/2", "launches": 2, "ms": us / 1e3,
                                        "hbm_gbs": moved / us / 1e3, "frac_of_peak": moved / us / 1e3 / HBM_PEAK_GBS}
    del c, k, v
    # -- attention with the Value front ahead of the Key front (Sec. 3.3 ratios 20 % / 10 %): 4 layers in rotation
    lc = kv.LayerCfg(3, 2, -1)
    caches = []
    Wc = 1024
    for l in range(4):
        c = kv.LayerCache(shape, lc, T + synth.GEN_ROOM, Wc, device=device)
        q, k, v = synth.gen_layer_torch(device, seed, 300 + l, B, Hq, Hkv, T)
        head_len = T - Wc + 32
        kv.quantize_pack(shape, lc, k[:, :, :head_len], v[:, :, :head_len], c)
        kv.append_tokens(shape, lc, k[:, :, head_len:], v[:, :, head_len:], c)
        keep_k, keep_v = kv.rpc_next(0.2, 0.1, T, T)
        kv.flush(shape, lc, c, keep_k, keep_v)
        caches.append(c)
        del k, v
    o = torch.zeros_like(q)
    ws = torch.zeros(kv.workspace_bytes(shape, T + synth.GEN_ROOM), dtype=torch.uint8, device=device)
    state["i"] = 0

    def fronts():
        kv.decode_attn(shape, lc, q, caches[state["i"] % 4], o, ws, stream=hstream)
        state["i"] += 1
    us = timed(fronts, 80)
    c = caches[0]
    units = B * Hkv
    nb = units * (c.n_q * (16 * 3 + 16) + c.n_qv * (16 * 2 + 16) + (c.n - c.n_q) * 256 + (c.n - c.n_qv) * 256)
    out["fronts_apart_r_0.2_0.1"] = {"batch": B, "kv_heads": Hkv, "context": c.n, "bits": "3/2", "key_front": c.n_q, "value_front": c.n_qv,
                                      "launches": 2, "us_per_call": us, "bytes_per_call": nb, "hbm_gbs": nb / us / 1e3,
                                      "frac_of_peak": nb / us / 1e3 / HBM_PEAK_GBS}
    del caches, ws
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the caches start 8 steps before a flush, so steps 40..71 hold exactly one flush step in 32 (its natural
    # rate); 40 warmup steps (30 ms) because the first steps after the set-up run measurably slower (5 warmup steps:
    # 0.78 ms per step, 40: 0.73 ms)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", default=HEADLINE, choices=sorted(synth.CONFIGS))
    ap.add_argument("--seed", type=int, default=synth.BASE_SEED)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short runs of the other benchmark configurations")
    ap.add_argument("--n-splits", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known size) so that rocprofv3 FETCH_SIZE / WRITE_SIZE "
                         "readings of the attention kernel can be scaled by what the same counters read for it")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (every unit = (layer, batch, kv head) is independent and "
                 "would shard by kv head, batch or layer without any exchange). Use --gpus 1.")

    import torch
    import paper_2506_08018_amd as kv
    kv.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    device = torch.device("cuda:0")
    torch.cuda.set_device(device)

    head = measure(args.config, args.steps, args.warmup, args.seed, args.n_splits, device, 0.0 if args.no_cpu_baseline else 12.0)

    others = {}
    if not args.no_other_configs and args.config == HEADLINE:
        # short runs of the other workloads (parity-test cases, not bench lines): each long enough to contain the flush
        plan = {"cfg1_single_layer": (64, 40), "cfg3_mistral_7b_gqa": (32, 40), "cfg4_llama3_8b_long": (32, 40), "cfg5_70b_stress": (16, 24)}
        for name, (st, wu) in plan.items():
            try:
                r = measure(name, st, wu, args.seed, 0, device, 0.0 if args.no_cpu_baseline else 3.0)
                if name == "cfg1_single_layer":
                    r["note"] = "3.6 MB per launch: cache-resident, launch-bound; not an HBM figure"
                others[name] = r
            except Exception as e:  # noqa: BLE001  (a failing side run must not take the headline down)
                others[name] = {"error": f"{type(e).__name__}: {e}"}

    if not args.no_other_configs and args.config == HEADLINE:
        try:
            others["widened"] = widened_rows(device, args.seed)
        except Exception as e:  # noqa: BLE001
            others["widened"] = {"error": f"{type(e).__name__}: {e}"}

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=device)   # 1 GiB read, 1 GiB written per call
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)       # an elementwise kernel (a plain copy_ would be a DMA transfer)
        torch.cuda.synchronize()
        del src, dst

    cfg = synth.CONFIGS[args.config]
    result = {
        "metric": "decode-attn tokens/s over mixed-bit KV; achieved HBM GB/s vs MI355X peak",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 in / f32 accumulate (2-4 bit integer codes)", "data": "synthetic",
        "config": {"workload": args.config, "layers": cfg["L"], "batch": cfg["B"], "q_heads": cfg["Hq"], "kv_heads": cfg["Hkv"],
                   "head_dim": 128, "context": cfg["T"], "window": cfg["W"], "group": 32,
                   "mean_k_bits": head["mean_k_bits"], "mean_v_bits": head["mean_v_bits"], "seed": args.seed,
                   "step": "per layer: kvmix_decode_step = append of 1 token (flush of 32 aged tokens when due) + decode attention",
                   "packed_cache_bytes": head["packed_cache_bytes"]},
        "ms_per_step_event_median": head["ms_per_step_event_median"],
        "step_hbm_gbs": head["step_hbm_gbs"], "step_frac_of_peak": head["step_frac_of_peak"],
        "host_issue_ms_per_step": head["host_issue_ms_per_step"],
        "attn_only_ms_per_step": head["attn_only_ms_per_step"],
        "attn_only_tokens_per_s": head["attn_only_tokens_per_s"],
        "roofline": head["roofline"],
        "prefill_quantize_pack": head["prefill_quantize_pack"],
    }
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    if others:
        result["other_configs"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
