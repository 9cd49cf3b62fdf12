#!/usr/bin/env python3
"""Benchmark of the KVLinC 2-bit decode hot path on one MI355X.

One step = one pass of the whole hot path over one batch: kvlinc_append_quantize of one new token per sequence
(rotation, window write, and -- when a window is full -- the group flush with its state update) followed by
kvlinc_decode_attention over the whole cache.  Workload: the Llama-3-8B-shaped layer (batch 16, 32 query / 8 KV
heads, head_dim 128, context 8192, 2-bit keys per channel and rotated values per token at group 128, 128-token fp16
window, linear correction on).  Steps cycle over several distinct layer caches so that every step reads HBM and
not the 256 MB Infinity Cache, like the layers of a model do.  Inputs are resident in HBM before timing starts.

Prints ONE JSON line; see the design notes for the byte accounting behind "roofline".
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
WORKLOAD = 2  # index into kvlinc_synth.CONFIGS
# Decode launches of the timed region that carry dispatch events: 4 to 16 of them, evenly spaced.  (A launch with
# events costs the stream about 10 us over a plain one, so timing every 4th launch of 256 took 8 % off the throughput.)
def timed_steps(K):
    n = max(4, min(16, K // 16))
    return sorted(set(min(K - 1, int((i + 0.5) * K / n)) for i in range(n))) if K > 0 else []
KERNEL_SOURCES = ("kvlinc_decode.hip", "kvlinc_mfma.h", "kvlinc_internal.h")  # what the decode kernel is compiled from


def kernel_source_sha1():
    import hashlib
    h = hashlib.sha1()
    for name in KERNEL_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2510_05373_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload_name):
    """HBM bytes one decode launch of this workload moved (read + written) according to the FETCH_SIZE and WRITE_SIZE
    counters, each scaled by what the same counter reports for a plain copy of known size: read from the tracked
    rocprofv3 summary of this workload.  (bytes, file, note); bytes is None when there is no summary or when the
    summary was taken at another state of the kernel's sources (it records their SHA-1)."""
    rel = os.path.join("profiles", "decode_main_kernel_%s_hbm_traffic.txt" % workload_name)
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None, "no tracked counter summary for this workload"
    fields = {}
    for line in open(path):
        if ":" in line:
            k, v = line.split(":", 1)
            fields[k.strip()] = v.strip()
    sha_now = kernel_source_sha1()
    if fields.get("kernel_source_sha1") != sha_now:
        return None, rel, "summary taken at kernel sources %s, now %s" % (fields.get("kernel_source_sha1"), sha_now)
    return float(fields["traffic_bytes_per_launch"]), rel, "kernel sources %s" % sha_now


def read_only_ceiling(caches, B, H_kv, H_q, counts, n_res, reps, hip, new_event):
    """Mean duration (s) and bytes of a launch that only reads what one decode launch reads: the live group records
    of every (sequence, KV head), the fp16 window, the 16-bit state, P and W_q.  Equal lengths only."""
    import ctypes
    import torch
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2510_05373_amd", "libkvlinc_probe.so"))
    lib.kvlinc_probe_read_only.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_longlong),
                                           ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(ctypes.c_longlong), ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    n_wg = 512  # measured best for one launch of this size (256 .. 4096 tried)
    sink = torch.empty(n_wg * 256, dtype=torch.int32, device=caches[0].groups.device)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    args = []
    total = 0
    for c in caches:
        rec_bytes = c.groups.shape[-1] * 4  # one group record
        segs = [(c.groups, counts * rec_bytes, c.max_groups * rec_bytes, B * H_kv),
                (c.k_res, n_res * 256, c.R * 256, B * H_kv), (c.v_res, -(-n_res // 4) * 1024, c.R * 256, B * H_kv),
                (c.S16, B * H_kv * 65536, 0, 1), (c.P, B * H_kv * 1024, 0, 1), (c.Wq, H_q * 65536, 0, 1)]
        n = len(segs)
        ptr = (ctypes.c_void_p * n)(*[t.data_ptr() for t, _, _, _ in segs])
        nbytes = (ctypes.c_longlong * n)(*[b for _, b, _, _ in segs])
        stride = (ctypes.c_longlong * n)(*[s for _, _, s, _ in segs])
        runs = (ctypes.c_longlong * n)(*[r for _, _, _, r in segs])
        args.append((ptr, nbytes, stride, runs, n))
        total = sum(b * r for _, b, _, r in segs)
    events = []
    for i in range(8 + reps):
        a = args[i % len(args)]
        ev = (new_event(), new_event()) if i >= 8 else (None, None)
        rc = lib.kvlinc_probe_read_only(a[0], a[1], a[2], a[3], a[4], ctypes.c_void_p(sink.data_ptr()), n_wg, stream, ev[0], ev[1])
        assert rc == 0, "read-only probe rejected its arguments"
        if i >= 8:
            events.append(ev)
    torch.cuda.synchronize()
    ms = []
    for a, b in events:
        t = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(t), a, b) == 0
        ms.append(t.value)
        hip.hipEventDestroy(a)
        hip.hipEventDestroy(b)
    return float(np.mean(ms)) * 1e-3, total


def algorithmic_bytes(B, H_q, H_kv, n_quant, n_res, correction=True, bits=2):
    """Bytes one decode call must move: 2-bit codes (64 B per token and KV head; twice that at 4 bits), fp16 scale + zero-point (8 B),
    the fp16 window (512 B per window token and KV head), the 16-bit state S and the fp32 P once per (sequence, KV
    head), W_q once, q and out.  Split partials are an implementation choice and are not counted."""
    groups = sum(-(-int(n) // 128) for n in n_quant)
    total = groups * H_kv * (2 * 2048 * bits + 2 * 512)
    total += int(sum(n_res)) * H_kv * 512
    if correction:
        total += B * H_kv * (256 * 128 * 2 + 256 * 4) + H_q * 2 * 128 * 128 * 2
    total += B * H_q * 128 * 2 * 2
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--layers", type=int, default=None,
                    help="distinct layer caches cycled through (default: 8; 4 for the two largest workloads)")
    ap.add_argument("--workload", type=int, default=WORKLOAD, choices=[2, 3, 4, 5, 6, 7],
                    help="index into kvlinc_synth.CONFIGS; the default is the workload the metric is quoted on, the "
                         "others run on device-generated N(0, 1) data without the oracle leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run 4 plain device copies of 256 MiB, the known-size reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    ap.add_argument("--variant", default="default", choices=["default", "sliding-values", "state16", "alg1-literal", "bits4"],
                    help="measure one of the variants of the path (descriptor flags / 16-bit state storage / 4-bit codes); the "
                         "default line is the one the metric is quoted on")
    ap.add_argument("--no-events", action="store_true", help="diagnosis: no per-launch events (roofline is then void)")
    args = ap.parse_args()
    if args.variant != "default":
        args.no_cpu_baseline = True  # the oracle leg (timing and parity sample) belongs to the default path
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path shards by sequence / "
              "KV head without communication)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    import kvlinc_synth as synth
    import paper_2510_05373_amd as kv

    wl = args.workload
    bits = 4 if args.variant == "bits4" else 2
    cfg = synth.CONFIGS[wl]
    B, H_q, H_kv = cfg["B"], cfg["H_q"], cfg["H_kv"]
    L = args.layers if args.layers else (4 if wl in (4, 5) else 8)
    K_steps, W = args.steps, args.warmup
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if wl == 5:
        base_len = synth.ragged_lengths(wl, B, cfg["n_min"], cfg["n_max"]).astype(np.int64)
    else:
        base_len = np.full(B, cfg["n"], dtype=np.int64)
    n0 = int(base_len.max())
    pad = 0 if wl == 5 else 128  # equal lengths: the layers start between n0 and n0 + 127 tokens (see below)
    n_hist = n0 + pad

    # ---- inputs: one seeded K/V history copied into L distinct caches.  For the default workload it is generated
    # on the host (the oracle leg needs it); the other workloads take device-generated N(0, 1) data.
    t0 = time.time()
    Wq_h, Wk_h = synth.adapters_q(wl, H_q), synth.adapters_k(wl, H_kv)
    Wq, Wk = torch.from_numpy(Wq_h).to(dev), torch.from_numpy(Wk_h).to(dev)
    if wl == WORKLOAD:
        Kh = np.empty((B, H_kv, n_hist, 128), dtype=np.float16)
        Vh = np.empty_like(Kh)
        for b in range(B):
            for g in range(H_kv):
                Kh[b, g] = synth.keys(wl, b, g, n_hist)
                Vh[b, g] = synth.values(wl, b, g, n_hist)
        Kd, Vd = torch.from_numpy(Kh).to(dev), torch.from_numpy(Vh).to(dev)
    else:
        g0 = torch.Generator(device=dev)
        g0.manual_seed(synth.BASE_SEED + wl)
        Kd = torch.empty(B, H_kv, n_hist, 128, dtype=torch.float16, device=dev)
        Vd = torch.empty_like(Kd)
        for b in range(B):  # per sequence, to bound the fp32 temporaries
            Kd[b] = torch.randn(H_kv, n_hist, 128, device=dev, generator=g0).half()
            Vd[b] = torch.randn(H_kv, n_hist, 128, device=dev, generator=g0).half()
    total_steps = W + K_steps
    per_layer = -(-total_steps // L)
    # Windows flush once per 128 appends of a layer, i.e. with L layers taking turns some layer flushes every 128
    # steps on average.  With equal lengths the layers start between the nominal context and 127 tokens above it, with
    # windows that fill up at evenly spaced steps (128 / L appends apart, in the layer order 0, 4, 1, 5, ...), the
    # first of them a few steps into the timed region whatever the warm-up: a run of 256 steps has 2 steps with a
    # flush (its natural rate), a short run has one.  Ragged lengths are staggered by themselves.
    caches, start_len = [], []
    for j in range(L):
        if wl != 5:
            pos = (j % 4) * ((L + 3) // 4) + j // 4                # place of the layer in the order of the flushes
            short = (W // L + 3 + (128 // L) * pos) % 128          # its window fills up after `short` appends and the
            n_start = base_len + pad - max(short, 1)               # next append flushes it
        else:
            n_start = base_len
        c = kv.KVLincCache(B, H_q, H_kv, n_hist + per_layer + 256, Wq=Wq, Wk=Wk,
                           state_storage="fp16" if args.variant == "state16" else "fp32",
                           flags={"sliding-values": kv.KVLINC_FLAG_SLIDING_VALUES, "alg1-literal": kv.KVLINC_FLAG_ALG1_LITERAL}.get(args.variant, 0),
                           bits=bits)
        t_max = int(n_start.max())
        c.append(Kd[:, :, :t_max].contiguous(), Vd[:, :, :t_max].contiguous(),
                 n_new=torch.from_numpy(n_start.astype(np.int32)).to(dev))
        caches.append(c)
        start_len.append(n_start.copy())
    if wl != WORKLOAD:
        del Kd, Vd
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED)
    k_new = torch.randn(total_steps, B, H_kv, 1, 128, device=dev, generator=gen).half()
    v_new = torch.randn(total_steps, B, H_kv, 1, 128, device=dev, generator=gen).half()
    q_all = torch.randn(total_steps, B, H_q, 128, device=dev, generator=gen).half()
    out = torch.empty(B, H_q, 128, dtype=torch.float16, device=dev)
    max_ctx = n_hist + per_layer + 1
    for c in caches:
        c.workspace(max_ctx)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    # Argument marshalling done once per (step, layer): the timed loop only calls the C ABI.
    import ctypes
    from paper_2510_05373_amd import binding as kb
    stream = torch.cuda.current_stream()
    s_ptr = ctypes.c_void_p(stream.cuda_stream)
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    ws = [c.workspace(max_ctx) for c in caches]
    app_args = [(ctypes.byref(caches[i % L].struct), vp(k_new[i]), vp(v_new[i]), None, 1, 0, s_ptr)
                for i in range(total_steps)]
    dec_args = [(ctypes.byref(caches[i % L].struct), vp(q_all[i]), vp(out), vp(ws[i % L]), ws[i % L].numel() * 4,
                 max_ctx, s_ptr) for i in range(total_steps)]
    f_app, f_dec = kb.lib.kvlinc_append_quantize, kb.lib.kvlinc_decode_attention

    hip = ctypes.CDLL("libamdhip64.so")  # the copy torch has already loaded
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def new_event():
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        return e

    use_events = not args.no_events
    f_dec_t = kb.lib.kvlinc_decode_attention_timed

    for i in range(W):
        assert f_app(*app_args[i]) == 0
        if i == 0 and use_events:  # the single cold call: the first decode launch of the process
            cold_b, cold_c = new_event(), new_event()
            assert f_dec_t(*dec_args[i], cold_b, cold_c) == 0
        else:
            assert f_dec(*dec_args[i]) == 0
    torch.cuda.synchronize()
    first_call_ms = None
    if W > 0 and use_events:
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), cold_b, cold_c) == 0
        first_call_ms = ms.value
    lens = [start_len[j] + sum(1 for i in range(W) if i % L == j) for j in range(L)]  # per layer: [B] lengths

    # ---- timed region: exactly K steps.  A few evenly spaced decode launches (timed_steps) carry a start and a stop event
    # attached to its own dispatch on the launch stream (kvlinc_decode_attention_timed), so the kernel's duration is
    # measured inside the timed region without extra packets between the kernels (such a launch costs the host
    # about 25 us, so timing every launch would make the loop host-bound).
    timed = timed_steps(K_steps) if use_events else []
    ev_b = {s: new_event() for s in timed}
    ev_c = {s: new_event() for s in timed}
    rc = 0
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(K_steps):
        i = W + s
        rc |= f_app(*app_args[i])
        if s in ev_b:
            rc |= f_dec_t(*dec_args[i], ev_b[s], ev_c[s])
        else:
            rc |= f_dec(*dec_args[i])
    t_cpu_done = time.perf_counter()
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    assert rc == 0, "a library call was rejected"
    for c in caches:
        assert int(c.status.item()) == 0, "device status word set"
    elapsed = t_end - t_start
    tokens = 0
    alg_bytes = []
    flush_steps = 0  # steps of the timed region whose append flushed the window of at least one sequence
    for s in range(K_steps):
        j = (W + s) % L
        flush_steps += int(((lens[j] >= 128) & (lens[j] % 128 == 0)).any())
        lens[j] = lens[j] + 1
        n = lens[j]
        tokens += int(n.sum())
        n_res = (n - 1) % 128 + 1
        alg_bytes.append(algorithmic_bytes(B, H_q, H_kv, n - n_res, n_res, bits=bits))
    if use_events:
        decode_ms = np.empty(len(timed))
        for k, s in enumerate(timed):
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), ev_b[s], ev_c[s]) == 0
            decode_ms[k] = ms.value
            hip.hipEventDestroy(ev_b[s])
            hip.hipEventDestroy(ev_c[s])
        alg_bytes = [alg_bytes[s] for s in timed]
    else:
        decode_ms = np.array([float("nan")])
    decode_avg_s = float(decode_ms.mean()) * 1e-3
    achieved = float(np.mean(alg_bytes)) / decode_avg_s / 1e9
    traffic, traffic_file, traffic_note = measured_traffic(cfg["name"]) if args.variant == "default" else (None, None, "not collected for variants")
    # the practical ceiling: a launch that only reads the same bytes (windows full, as in most steps)
    ceiling = None
    if wl != 5 and not args.no_events:
        n_now = int(lens[0][0])
        n_res_now = (n_now - 1) % 128 + 1
        t_read, read_bytes = read_only_ceiling(caches, B, H_kv, H_q, (n_now - n_res_now) // 128, n_res_now, 32, hip, new_event)
        ceiling = {"read_only_launch_us": t_read * 1e6, "read_only_bytes": read_bytes,
                   "read_only_gbs": read_bytes / t_read / 1e9, "frac_of_peak": read_bytes / t_read / 1e9 / PEAK_HBM_GBS}

    result = {
        "metric": "decode-attention KV tokens/s at 2-bit (achieved HBM GB/s and % of peak under roofline)",
        "value": tokens / elapsed,
        "unit": "KV tokens/s",
        "n_gpus": 1, "steps": K_steps, "warmup": W,
        "ms_per_step": elapsed / K_steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u%d codes, f16 operands, f32 accumulate" % bits,
        "data": "synthetic",
        "config": {"workload": cfg["name"] + ("" if args.variant == "default" else " [variant: %s]" % args.variant), "batch": B, "q_heads": H_q, "kv_heads": H_kv, "head_dim": 128,
                   "context": n0 if wl != 5 else "%d..%d" % (int(base_len.min()), n0),
                   "context_of_the_layer_caches": "%d..%d" % (min(int(x.min()) for x in lens), max(int(x.max()) for x in lens)), "window": 128, "group": 128, "bits": bits, "correction_rank": 256,
                   "layer_caches_cycled": L, "step": "append 1 token/sequence + decode attention",
                   "steps_with_a_window_flush": flush_steps,
                   "decode_ms_median": float(np.median(decode_ms)), "decode_ms_mean": float(decode_ms.mean()),
                   "decode_ms_first_call": first_call_ms,
                   "launch_loop_cpu_ms_per_step": (t_cpu_done - t_start) / K_steps * 1e3, "setup_s": setup_s},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS, "traffic": traffic,
                     "traffic_source": traffic_file, "traffic_note": traffic_note,
                     "read_ceiling_frac": None if ceiling is None else ceiling["frac_of_peak"],
                     "read_ceiling": ceiling,
                     "frac_of_read_ceiling": None if ceiling is None else achieved / ceiling["read_only_gbs"],
                     "kernel": "decode_main_kernel (the one launch of kvlinc_decode_attention)",
                     "algorithmic_bytes_per_launch": float(np.mean(alg_bytes)),
                     "avg_launch_us": decode_avg_s * 1e6, "launches_timed": len(decode_ms)},
    }

    if args.pmc_calibration:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the oracle beside it: same decode step, bounded sample, host cores ----------------------------------
    if wl != WORKLOAD:
        result["cpu_baseline"] = None  # the oracle leg runs on the default workload only
    elif not args.no_cpu_baseline:
        from oracle import attention as o_attn
        from oracle import kvcache as o_cache
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        # parity of the bench configuration on the sample + timing of the oracle's decode of the same rows
        i_chk = W + K_steps - 1
        j = i_chk % L
        n = int(lens[j][0])  # equal lengths in this workload
        s0 = int(start_len[j][0])
        nq, nr = o_cache.window_split(n)
        n_app = n - s0
        idx = [i for i in range(W + K_steps) if i % L == j]
        k_app = k_new[idx][:, :, :, 0].cpu().numpy()  # [n_app, B, H_kv, 128]
        v_app = v_new[idx][:, :, :, 0].cpu().numpy()
        q_chk = q_all[i_chk].cpu().numpy()
        got = out.cpu().numpy().astype(np.float64)
        pairs = [(0, 0), (B - 1, H_kv - 1), (B // 2, 3)]
        gq = H_q // H_kv
        refs = []
        for (b, g) in pairs:
            Kf = np.concatenate([Kh[b, g, :s0], k_app[:n_app, b, g]])
            Vf = np.concatenate([Vh[b, g, :s0], v_app[:n_app, b, g]])
            refs.append(o_cache.build_cache(Kf, Vf, nq, Wk=Wk_h[g]))
        t_cpu, rows, reps = 0.0, 0, 0
        err_num = err_den = 0.0
        while t_cpu < 12.0:
            for (b, g), ref in zip(pairs, refs):
                t1 = time.perf_counter()
                ys = [o_attn.decode(q_chk[b, h], ref, Wq_h[h]) for h in range(g * gq, (g + 1) * gq)]
                t_cpu += time.perf_counter() - t1
                rows += 1
                if reps == 0:
                    for h, y in zip(range(g * gq, (g + 1) * gq), ys):
                        err_num += float(((got[b, h] - y) ** 2).sum())
                        err_den += float((y ** 2).sum())
                        assert np.abs(got[b, h] - y).max() <= 1e-2, "bench output off the oracle"
            reps += 1
        rel_l2 = (err_num / err_den) ** 0.5
        assert rel_l2 <= 2e-3, "bench output off the oracle (rel-L2 %g)" % rel_l2
        result["cpu_baseline"] = {
            "value": n * rows / t_cpu / H_kv, "unit": "KV tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "oracle decode (dense fp64 operands, Eq. 5) of %d (sequence, KV head) pairs x %d query heads "
                      "at context %d, %d repetitions, %.1f s; scaled to whole-layer tokens (one token = all %d KV "
                      "heads); the oracle's cache build is not timed" % (len(pairs), gq, n, reps, t_cpu, H_kv),
            "parity_rel_l2_on_sample": rel_l2,
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
