#!/usr/bin/env python3
"""Benchmark of the KSA hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input resident in HBM:
  prefill of the 128K workload (batch 1, 32/8 heads, head_dim 128, 131072 text tokens, chunks of 64 with
  8 summary tokens each) followed by one decode step of the 128K-context workload (batch 64, 16376 visible
  summary rows + 128 text rows per KV head).  The layout / tile schedule depends on shapes only and is built
  once before the timed region (its build time is reported separately).

Prints one JSON line.  `value` is the prefill throughput in live TFLOP/s (4*d FLOPs per visible (q, k)
pair, nothing else counted); the decode bandwidth, both rooflines and the CPU oracle baseline ride along.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E


def live_pairs(n, c, m, C):
    """Visible (query, key) pairs per head of the KSA mask (closed form from Eq. 1 / Eq. 3)."""
    J = n // c
    text = sum(min(j, C) * c * c + c * (c + 1) // 2 + max(0, j - C) * m * c for j in range(J))
    return text + J * (m * c + m * (m + 1) // 2)


def measured_traffic(which):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a
    copy kernel of known size); the numbers live in profiles/hbm_traffic.txt as `<which>_traffic_bytes: N`."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith(which + "_traffic_bytes:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def kernel_source_digest():
    """sha256 over the sources of the prefill and decode kernels and of the schedule they walk: profiles/hbm_traffic.txt
    records the digest it was measured with, and a measurement taken with other sources is not reported."""
    import hashlib
    here = os.path.dirname(os.path.abspath(__file__))
    h = hashlib.sha256()
    for name in ("ksa_prefill.hip", "ksa_decode.hip", "ksa_layout.cpp", "ksa_schedule.h", "ksa_device.h"):
        h.update(open(os.path.join(here, "paper_2604_24432_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic_checked(which):
    """(bytes or None, note): the measured HBM traffic if profiles/hbm_traffic.txt was taken with the present sources."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.txt")
    digest, commit = None, None
    try:
        for line in open(path):
            if line.startswith("kernel_source_digest:"):
                digest = line.split(":")[1].strip()
            if line.startswith("measured_at_commit:"):
                commit = line.split(":")[1].strip()
    except OSError:
        return None, "profiles/hbm_traffic.txt missing"
    if digest != kernel_source_digest():
        return None, f"profiles/hbm_traffic.txt was measured with other kernel sources (commit {commit}): not reported"
    return measured_traffic(which), f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE at commit {commit} (profiles/hbm_traffic.txt)"


def achievable_rates(read_buffer):
    """The two 'achievable' figures beside the nominal peaks, measured now on this machine by libksa_probe.so: a loop of
    nothing but the prefill kernel's MFMA instruction on every SIMD (one wave per SIMD, as the prefill kernel runs), and
    a streaming read of the decode cache with the decode kernel's access pattern."""
    import ctypes as C
    here = os.path.dirname(os.path.abspath(__file__))
    lib = C.CDLL(os.path.join(here, "paper_2604_24432_amd", "libksa_probe.so"))
    lib.ksa_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.ksa_probe_read.argtypes = [C.c_void_p, C.c_longlong, C.c_int, C.POINTER(C.c_float)]
    out = {}
    for waves in (1, 2):
        tf, mhz = C.c_float(), C.c_float()
        # 20000 rounds x 8 MFMAs x 32 clocks = 5.1 M clocks per launch, 100 launches: about a quarter of a second
        rc = lib.ksa_probe_mfma(0, waves, 20000, 100, C.byref(tf), C.byref(mhz))
        if rc != 0:
            raise RuntimeError(f"ksa_probe_mfma failed ({rc})")
        out[f"mfma_only_tflops_{waves}_wave_per_simd"] = round(tf.value, 1)
        out[f"mfma_only_core_mhz_{waves}_wave_per_simd"] = round(mhz.value, 0)
    gbs = C.c_float()
    nbytes = read_buffer.numel() * read_buffer.element_size() // 16 * 16
    rc = lib.ksa_probe_read(C.c_void_p(read_buffer.data_ptr()), nbytes, 5, C.byref(gbs))
    if rc != 0:
        raise RuntimeError(f"ksa_probe_read failed ({rc})")
    out["stream_read_gbs"] = round(gbs.value, 1)
    out["stream_read_bytes"] = nbytes
    out["note"] = ("mfma_only: v_mfma_f32_32x32x16_bf16 back to back on all SIMDs, bf16 operands of magnitude 0.25 - 4 that "
                   "differ per lane, no memory traffic; the core clock is the kernel's own cycle counter against the "
                   "100 MHz wall counter.  stream_read: 16-byte non-temporal loads over the decode K cache")
    return out


def time_events(fn, steps):
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    return [e0.elapsed_time(e1) for e0, e1 in evs]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--hot-path-only", action="store_true",
                    help="skip everything outside the timed step (cache lifecycle timings, dense reference, CPU baseline): "
                         "for profiler runs, whose per-kernel statistics then cover the benchmark launches only")
    ap.add_argument("--no-full-attention", action="store_true",
                    help="skip the dense-causal reference run at the same length (about half a second of GPU time)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--backward-only", action="store_true",
                    help="one forward call, then only the prefill backward --steps times (for profiler runs of its kernels)")
    ap.add_argument("--decode-splits", type=int, default=0)
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy (reference dispatch for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--power-probe", type=float, default=0.0, metavar="SECONDS",
                    help="loop the 128K prefill, an MFMA-only kernel and the 128K backward for this long each while "
                         "sampling the board's power and clocks with amd-smi; print the samples as one JSON line and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_24432_amd as K
    from paper_2604_24432_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    # ---- prefill 128K -----------------------------------------------------------------------------
    cfg = synth.CONFIGS["prefill_128k"]
    t0 = time.perf_counter()
    p = K.make_params(cfg.batch, cfg.n_text, cfg.chunk_len, cfg.n_summary, cfg.window_chunks, cfg.n_q_heads,
                      cfg.n_kv_heads, cfg.head_dim)
    lay = K.ksa_build_layout(p)
    lay.upload()
    layout_ms = (time.perf_counter() - t0) * 1e3
    q, k, v = synth.make_prefill_inputs(cfg, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty((cfg.batch, cfg.n_q_heads, cfg.aug_len), dtype=torch.float32, device="cuda")
    pws = torch.empty(K.prefill_workspace_bytes(lay), dtype=torch.uint8, device="cuda")

    # ---- decode on a 128K context --------------------------------------------------------------------
    dcfg = synth.CONFIGS["decode_128k"]
    pos = dcfg.decode_pos
    n_cap = (pos // dcfg.chunk_len + 1) * dcfg.chunk_len
    dp = K.make_params(dcfg.batch, n_cap, dcfg.chunk_len, dcfg.n_summary, dcfg.window_chunks, dcfg.n_q_heads,
                       dcfg.n_kv_heads, dcfg.head_dim)
    s_cap, rows = K.cache_geometry(dp)
    W = (dcfg.window_chunks + 1) * dcfg.chunk_len
    base = (pos // dcfg.chunk_len - dcfg.window_chunks) * dcfg.chunk_len
    dq, k_sum, v_sum, k_txt, v_txt = synth.make_decode_inputs(dcfg, s_cap, W, device="cuda")
    k_cache, v_cache = K.pack_cache(dp, k_sum, v_sum, k_txt, v_txt, base)
    del k_sum, v_sum
    pos_t = torch.full((dcfg.batch,), pos, dtype=torch.int32, device="cuda")
    do = torch.empty_like(dq)
    dlse = torch.empty((dcfg.batch, dcfg.n_q_heads), dtype=torch.float32, device="cuda")
    ws = torch.empty(K.decode_workspace_bytes(dp, args.decode_splits), dtype=torch.uint8, device="cuda")
    rg = K.ksa_decode_ranges(dp, pos)
    vis_rows = int(rg[1] + rg[3] + rg[5])

    def prefill():
        K.ksa_prefill_fwd(lay, q, k, v, o=o, lse=lse, workspace=pws)

    def relayout():
        K.ksa_prefill_relayout_v(lay, v, pws)

    def decode():
        K.ksa_decode_fwd(dp, dq, k_cache, v_cache, pos_t, o=do, lse=dlse, workspace=ws, n_splits=args.decode_splits)

    def step():
        prefill()
        decode()

    if args.power_probe > 0:
        res = {"prefill_128k": power_probe(prefill, args.power_probe)}
        import ctypes as C
        plib = C.CDLL(os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2604_24432_amd", "libksa_probe.so"))
        plib.ksa_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        tf, mhz = C.c_float(), C.c_float()
        # one call = 41 launches of about 2.8 ms: the same board state as the prefill loop, but nothing except MFMAs
        res["mfma_only_loop"] = power_probe(lambda: plib.ksa_probe_mfma(0, 1, 20000, 4, C.byref(tf), C.byref(mhz)),
                                            args.power_probe)
        res["mfma_only_loop"]["tflops_last_call"] = round(tf.value, 1)
        res["mfma_only_loop"]["core_mhz_last_call"] = round(mhz.value, 0)
        prefill()
        g = synth.make_upstream_gradient(cfg, device="cuda")
        gq, gk, gv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        bws = torch.empty(K.prefill_bwd_workspace_bytes(lay), dtype=torch.uint8, device="cuda")
        res["prefill_backward_128k"] = power_probe(
            lambda: K.ksa_prefill_bwd(lay, q, k, v, o, lse, g, dq=gq, dk=gk, dv=gv, workspace=bws), args.power_probe)
        print(json.dumps(res), flush=True)
        return

    if args.traffic_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # 1 GiB read + 1 GiB written by one copy kernel
        torch.cuda.synchronize()
        del src, dst
    if args.backward_only:
        prefill()
        print(json.dumps({"prefill_backward": prefill_backward(cfg, lay, q, k, v, o, lse, max(args.steps, 1))}), flush=True)
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel durations with events on the launch stream, over the same number of steps
    pre_ms = time_events(prefill, args.steps)
    vt_ms = time_events(relayout, args.steps)
    dec_ms = time_events(decode, args.steps)
    pre_avg, dec_avg, vt_avg = float(np.mean(pre_ms)), float(np.mean(dec_ms)), float(np.mean(vt_ms))
    # ksa_prefill_fwd launches two kernels: the key-major copy of V (timed alone just above) and the attention
    # kernel, whose duration is the difference
    attn_avg = pre_avg - vt_avg

    live = live_pairs(cfg.n_text, cfg.chunk_len, cfg.n_summary, cfg.window_chunks)
    live_flops = 4.0 * cfg.head_dim * cfg.batch * cfg.n_q_heads * live
    pre_tflops = live_flops / (pre_avg * 1e-3) / 1e12      # whole call (both kernels): the reported value
    attn_tflops = live_flops / (attn_avg * 1e-3) / 1e12    # attention kernel alone: the roofline figure
    dec_bytes = 2.0 * dcfg.batch * dcfg.n_kv_heads * vis_rows * dcfg.head_dim * 2 \
        + 2.0 * dcfg.batch * dcfg.n_q_heads * dcfg.head_dim * 2
    dec_gbs = dec_bytes / (dec_avg * 1e-3) / 1e9

    tp = lay.tile_pairs()
    issued_pairs = int((tp["q_count"].astype(np.int64) * tp["k_count"]).sum())   # per (batch, head): padded tile area
    issued_flops = 4.0 * cfg.head_dim * cfg.batch * cfg.n_q_heads * issued_pairs
    pre_traffic, pre_traffic_note = measured_traffic_checked("prefill")
    dec_traffic, _ = measured_traffic_checked("decode")
    ach = achievable_rates(k_cache)

    out = {
        "metric": "KSA prefill live-TFLOP/s + %MFMA peak @128K; decode HBM GB/s + %peak",
        "value": round(pre_tflops, 2),
        "unit": "TFLOP/s (live bf16 FLOPs, 128K prefill)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "prefill_128k (B1 Hq32 Hkv8 d128 n131072 c64 m8 C1, L=147456) + decode_128k "
                               "(B64 Hq32 Hkv8 d128 pos 131135: 16376 summary + 128 text rows per KV head)",
                   "layout_build_ms": round(layout_ms, 2), "build": K.build_info()},
        "prefill": {"ms": round(pre_avg, 4), "ms_min": round(float(np.min(pre_ms)), 4), "live_flops": live_flops,
                    "live_tflops": round(pre_tflops, 2), "frac_mfma_peak": round(pre_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                    "preparation_pass_ms": round(vt_avg, 4), "attention_kernel_ms": round(attn_avg, 4),
                    "tile_issued_flops": issued_flops, "issued_over_live": round(issued_flops / live_flops, 4),
                    "heads_per_workgroup": lay.heads_per_workgroup, "q_tile_rows": lay.q_tile_rows},
        "decode": {"ms": round(dec_avg, 5), "ms_min": round(float(np.min(dec_ms)), 5), "bytes": dec_bytes,
                   "gbs": round(dec_gbs, 1), "frac_hbm_peak": round(dec_gbs / HBM_PEAK_GBS, 4),
                   "visible_rows_per_kv_head": vis_rows},
        "roofline": {"bound": "mfma", "kernel": "ksa_prefill_kernel<128, true>", "achieved": round(attn_tflops, 2),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": pre_traffic,
                     "traffic_source": pre_traffic_note,
                     "frac_of_mfma_only_loop": round(attn_tflops / ach["mfma_only_tflops_1_wave_per_simd"], 4)},
        "roofline_decode": {"bound": "hbm", "kernel": "ksa_decode_split_kernel<128,4>", "achieved": round(dec_gbs, 1),
                            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dec_gbs / HBM_PEAK_GBS, 4),
                            "traffic": dec_traffic,
                            "frac_of_stream_read": round(dec_gbs / ach["stream_read_gbs"], 4)},
        "achievable": ach,
    }

    if args.hot_path_only:
        print(json.dumps(out), flush=True)
        return
    out["prefill_backward"] = prefill_backward(cfg, lay, q, k, v, o, lse, 5)
    out["cache_lifecycle"] = cache_lifecycle(cfg, p, k, v, dcfg, dp, dq, k_cache, v_cache, ws, args)
    if not args.no_full_attention:
        del k_cache, v_cache
        out["full_attention_reference"] = full_attention_reference(cfg, q, k, v, pre_avg)
        out["paper_shape_reference"] = paper_shape_reference(cfg)
        out["sca_reference"] = sca_reference(cfg)
        out["swa_reference"] = swa_reference(cfg)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, q, k, v, o, live_flops / live)
    print(json.dumps(out), flush=True)


def power_probe(launch, seconds):
    """Keeps the GPU busy with `launch` for `seconds` while a thread samples `amd-smi metric -p -c` (a read-only
    query: socket power and the core clock of every XCD); returns the samples taken after the first second (the
    clocks need a moment to settle)."""
    import subprocess
    import threading
    import torch
    samples, stop = [], threading.Event()

    def sampler():
        t0 = time.perf_counter()
        while not stop.is_set():
            rec = {"t": round(time.perf_counter() - t0, 2)}
            try:
                txt = subprocess.run(["amd-smi", "metric", "-g", "0", "-p", "-c", "--json"], capture_output=True, text=True,
                                     timeout=20).stdout
                data = json.loads(txt)
                gpu = (data["gpu_data"] if isinstance(data, dict) else data)[0]
                rec["socket_power_w"] = gpu["power"]["socket_power"]["value"]
                clks = [v["clk"]["value"] for k, v in gpu["clock"].items() if k.startswith("gfx_") and isinstance(v, dict)
                        and isinstance(v.get("clk"), dict) and isinstance(v["clk"].get("value"), (int, float))]
                if clks:
                    rec["gfx_clk_mhz_mean"] = round(sum(clks) / len(clks), 1)
                    rec["gfx_clk_mhz_min"], rec["gfx_clk_mhz_max"] = min(clks), max(clks)
                    rec["gfx_max_clk_mhz"] = gpu["clock"]["gfx_0"]["max_clk"]["value"]
            except Exception as e:       # the probe must not take the benchmark down
                rec["error"] = f"{type(e).__name__}: {e}"
                samples.append(rec)
                break
            samples.append(rec)
            time.sleep(0.2)

    th = threading.Thread(target=sampler)
    th.start()
    t0, n = time.perf_counter(), 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            launch()
        torch.cuda.synchronize()
        n += 10
    busy = time.perf_counter() - t0
    stop.set()
    th.join()
    kept = [s for s in samples if s.get("t", 0) >= 1.0 and s.get("t", 0) <= busy]
    return {"launches": n, "busy_seconds": round(busy, 2), "ms_per_launch": round(busy * 1e3 / n, 3), "samples": kept}


def prefill_backward(cfg, lay, q, k, v, o, lse, steps):
    """Not part of the timed step: dQ, dK, dV of the same 128K prefill (ksa_prefill_bwd on the forward's O and
    log-sum-exp, N(0,1) upstream gradient).  FLOPs: five products of 2 d per live (query, key) pair (S, dP, dV, dQ, dK);
    the two kernels recompute S and dP once each, which is not counted."""
    import torch
    import paper_2604_24432_amd as K
    from paper_2604_24432_amd import synth
    g = synth.make_upstream_gradient(cfg, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(K.prefill_bwd_workspace_bytes(lay), dtype=torch.uint8, device="cuda")

    def bwd():
        K.ksa_prefill_bwd(lay, q, k, v, o, lse, g, dq=dq, dk=dk, dv=dv, workspace=ws)

    bwd()
    ms = time_events(bwd, steps)
    avg = float(np.mean(ms))
    flops = 10.0 * cfg.head_dim * cfg.batch * cfg.n_q_heads * live_pairs(cfg.n_text, cfg.chunk_len, cfg.n_summary,
                                                                         cfg.window_chunks)
    tf = flops / (avg * 1e-3) / 1e12
    return {"ms": round(avg, 3), "ms_min": round(float(np.min(ms)), 3), "live_flops": flops, "live_tflops": round(tf, 1),
            "frac_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
            "kernels": "ksa_bwd_delta_kernel, ksa_bwd_dq_kernel, ksa_bwd_dkv_kernel (split in profiles/)"}


def backward_of(lay, q, k, v, o, lse, seed, calls=2):
    """ms per ksa_prefill_bwd call for tensors already on the GPU (N(0,1) upstream gradient drawn here)."""
    import torch
    import paper_2604_24432_amd as K
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    g = torch.randn(o.shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(K.prefill_bwd_workspace_bytes(lay), dtype=torch.uint8, device="cuda")

    def bwd():
        K.ksa_prefill_bwd(lay, q, k, v, o, lse, g, dq=dq, dk=dk, dv=dv, workspace=ws)

    bwd()
    return float(np.mean(time_events(bwd, calls)))


def full_attention_reference(cfg, q, k, v, ksa_ms):
    """Not part of the timed step: dense causal attention over the same number of text tokens through the same
    library (no summaries, every earlier chunk in the window), i.e. what the summary mask saves at this length."""
    import torch
    import paper_2604_24432_amd as K
    n, c = cfg.n_text, cfg.chunk_len
    p = K.make_params(cfg.batch, n, c, 0, n // c, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    lay = K.ksa_build_layout(p)
    lay.upload()
    qd, kd, vd = q[:, :n], k[:, :n], v[:, :n]     # the first n rows of the synthetic tensors serve as the text tokens
    od = torch.empty_like(qd)
    ld = torch.empty((cfg.batch, cfg.n_q_heads, n), dtype=torch.float32, device="cuda")
    ws = torch.empty(K.prefill_workspace_bytes(lay), dtype=torch.uint8, device="cuda")
    K.ksa_prefill_fwd(lay, qd, kd, vd, o=od, lse=ld, workspace=ws)
    ms = float(np.mean(time_events(lambda: K.ksa_prefill_fwd(lay, qd, kd, vd, o=od, lse=ld, workspace=ws), 3)))
    flops = 4.0 * cfg.head_dim * cfg.batch * cfg.n_q_heads * live_pairs(n, c, 0, n // c)
    bwd_ms = backward_of(lay, qd, kd, vd, od, ld, cfg.seed + 60, calls=1)
    return {"workload": f"dense causal, B{cfg.batch} Hq{cfg.n_q_heads} Hkv{cfg.n_kv_heads} d{cfg.head_dim} n{n}",
            "ms": round(ms, 3), "live_tflops": round(flops / (ms * 1e-3) / 1e12, 1),
            "frac_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "ksa_prefill_speedup": round(ms / ksa_ms, 2),
            "backward_ms": round(bwd_ms, 2),
            "backward_frac_mfma_peak": round(2.5 * flops / (bwd_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}


def mask_reference(cfg, label, c, m, C, note, with_backward=True, heads=None):
    """Not part of the timed step: another mask of the paper at the benchmark's length and heads (or `heads` =
    (query heads, KV heads)) through the same library (seeded N(0,1) inputs of that shape)."""
    import torch
    import paper_2604_24432_amd as K
    from paper_2604_24432_amd import synth
    hq, hkv = heads if heads else (cfg.n_q_heads, cfg.n_kv_heads)
    pc = synth.KsaConfig(label, cfg.batch, hq, hkv, cfg.head_dim, cfg.n_text, c, m, C, seed=cfg.seed + 50 + c + C)
    p = K.make_params(pc.batch, pc.n_text, pc.chunk_len, pc.n_summary, pc.window_chunks, pc.n_q_heads, pc.n_kv_heads,
                      pc.head_dim)
    lay = K.ksa_build_layout(p)
    lay.upload()
    q, k, v = synth.make_prefill_inputs(pc, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty((pc.batch, pc.n_q_heads, pc.aug_len), dtype=torch.float32, device="cuda")
    ws = torch.empty(K.prefill_workspace_bytes(lay), dtype=torch.uint8, device="cuda")
    K.ksa_prefill_fwd(lay, q, k, v, o=o, lse=lse, workspace=ws)
    ms = float(np.mean(time_events(lambda: K.ksa_prefill_fwd(lay, q, k, v, o=o, lse=lse, workspace=ws), 5)))
    flops = 4.0 * pc.head_dim * pc.batch * pc.n_q_heads * live_pairs(pc.n_text, pc.chunk_len, pc.n_summary, pc.window_chunks)
    out = {"workload": f"{note}: B{pc.batch} Hq{pc.n_q_heads} Hkv{pc.n_kv_heads} d{pc.head_dim} n{pc.n_text} c{c} m{m} C{C}, "
                       f"L={pc.aug_len}",
           "ms": round(ms, 3), "live_flops": flops, "live_tflops": round(flops / (ms * 1e-3) / 1e12, 1),
           "frac_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    if with_backward:
        bwd_ms = backward_of(lay, q, k, v, o, lse, pc.seed + 7)
        out["backward_ms"] = round(bwd_ms, 2)
        out["backward_frac_mfma_peak"] = round(2.5 * flops / (bwd_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)
    return out


def paper_shape_reference(cfg):
    """The paper's own chunk form (one summary per chunk of 8 text tokens, 128 chunks of sliding window: table of model
    hyper-parameters)."""
    out = mask_reference(cfg, "paper_shape_128k", 8, 1, 128, "KSA in the paper's own form")
    # the same mask with the head layout of the paper's other model (16 query heads, 16 KV heads: no grouping)
    mha = mask_reference(cfg, "paper_shape_128k_h16", 8, 1, 128, "the same with 16 / 16 heads", with_backward=False, heads=(16, 16))
    out["heads16_16"] = {k: mha[k] for k in ("workload", "ms", "live_tflops", "frac_mfma_peak")}
    return out


def sca_reference(cfg):
    """Sliding Chunk Attention alone (Eq. 2: the paper's Hybrid-SCA baseline layers), chunks of 8, 128 sliding chunks."""
    return mask_reference(cfg, "sca_128k", 8, 0, 128, "sliding chunk attention, no summaries (Eq. 2)", with_backward=False)


def swa_reference(cfg):
    """Token-level sliding window attention (the paper's Hybrid-SWA baseline layers) of the same span, 1024 tokens:
    chunks of one token, 1023 previous ones visible."""
    return mask_reference(cfg, "swa_128k", 1, 0, 1023, "token-level sliding window of 1024 tokens", with_backward=False)


def cache_lifecycle(cfg, p, k, v, dcfg, dp, dq, k_cache, v_cache, ws, args):
    """Not part of the timed step: the data-movement entry points of the decode loop and its summary-token step,
    timed with events at the benchmark shapes (hand-off of the 128K prefill; one insert and one summary step of
    the B = 64 decode workload)."""
    import torch
    import paper_2604_24432_amd as K
    s_cap, rows = K.cache_geometry(p)
    hk = torch.empty((cfg.batch, cfg.n_kv_heads, rows, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    hv = torch.empty_like(hk)
    fill_ms = time_events(lambda: K.ksa_cache_from_prefill(p, cfg.n_text, k, v, hk, hv), args.steps)
    moved_rows = s_cap + min(cfg.n_text // cfg.chunk_len, cfg.window_chunks + 1) * cfg.chunk_len
    fill_bytes = 2.0 * 2.0 * cfg.batch * cfg.n_kv_heads * moved_rows * cfg.head_dim * 2   # K and V, read + written
    k_new = torch.randn((dcfg.batch, dcfg.n_kv_heads, dcfg.head_dim), device="cuda").to(torch.bfloat16)
    v_new = torch.randn_like(k_new)
    d_s_cap, _ = K.cache_geometry(dp)
    pos_t = torch.full((dcfg.batch,), dcfg.decode_pos, dtype=torch.int32, device="cuda")
    ord_t = torch.full((dcfg.batch,), d_s_cap - 1, dtype=torch.int32, device="cuda")
    do = torch.empty_like(dq)
    app_ms = time_events(lambda: K.ksa_cache_append(dp, K.KSA_ROW_TEXT, k_new, v_new, pos_t, k_cache, v_cache), args.steps)
    sum_ms = time_events(lambda: K.ksa_decode_summary_fwd(dp, dq, k_cache, v_cache, ord_t, o=do, return_lse=False,
                                                           workspace=ws, n_splits=args.decode_splits), args.steps)
    fill_avg = float(np.mean(fill_ms))
    return {"cache_from_prefill_ms": round(fill_avg, 5), "cache_from_prefill_bytes": fill_bytes,
            "cache_from_prefill_gbs": round(fill_bytes / (fill_avg * 1e-3) / 1e9, 1),
            "cache_append_ms": round(float(np.mean(app_ms)), 5),
            "decode_summary_fwd_ms": round(float(np.mean(sum_ms)), 5),
            "note": "hand-off of the 128K prefill (B1); insert and summary step at the decode shape (B64)"}


def cpu_baseline(cfg, q, k, v, o_gpu, flops_per_pair_all_heads):
    """The oracle as it stands, on the host cores, over a bounded sample of the same prefill workload:
    a seeded set of query rows for all heads.  Also checks the GPU output on those rows."""
    import torch
    from oracle import ksa_oracle as O
    gen = np.random.default_rng(12345)
    rows = np.sort(gen.choice(cfg.aug_len, size=2400, replace=False)).astype(np.int64)
    qf, kf, vf = (x.float().cpu().numpy() for x in (q, k, v))
    t0 = time.perf_counter()
    o_ref, _ = O.prefill(qf, kf, vf, cfg.n_text, cfg.chunk_len, cfg.n_summary, cfg.window_chunks, rows=rows)
    secs = time.perf_counter() - t0
    pairs = 0
    for a in rows:
        pairs += int(O.mask_row(int(a), cfg.n_text, cfg.chunk_len, cfg.n_summary, cfg.window_chunks).sum())
    flops = flops_per_pair_all_heads * pairs
    err = np.abs(o_gpu[:, torch.from_numpy(rows).cuda()].float().cpu().numpy() - o_ref)
    cores = O.num_threads()
    return {"value": round(flops / secs / 1e12, 6), "unit": "TFLOP/s (live, fp64 oracle)", "cores": cores,
            "kind": "oracle", "seconds": round(secs, 2),
            "sample": f"{len(rows)} seeded query rows x {cfg.n_q_heads} heads of the 128K prefill workload "
                      f"({pairs} visible pairs per head)",
            "gpu_vs_oracle_max_abs_on_sample": float(err.max()), "gpu_vs_oracle_mean_abs_on_sample": float(err.mean())}


if __name__ == "__main__":
    main()
