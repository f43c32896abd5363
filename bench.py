#!/usr/bin/env python3
"""Benchmark of the EchoKV decode hot path on one MI355X.

One step = one pass of the whole hot path of one target layer over one batch:
append the step's new token to the anchor and target caches
(echokv_cache_append x2), then echokv_decode_attn over every decode sequence
(retained-head streaming kernel, fused reconstruct+attend kernel, split-K
merge) and, where the configuration has one, the causal prefill chunk
(echokv_prefill_attn).  Inputs are synthetic, seeded, and resident in HBM
before the timed region.  Prints ONE JSON line.

The default workload is configuration 4, the largest one that fits one GPU:
32 ragged decode sequences (log-uniform 1 K .. 64 K tokens) plus one
8192-query causal prefill chunk in the same step.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--unfused] ...
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def kernel_source_sha(names=None):
    """Identifies the kernel sources a counter summary under profiles/ was taken with: a hash over
    the named files of csrc/ (all of them if none are named)."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2603_22910_amd", "csrc")
    for name in sorted(names or [n for n in os.listdir(csrc) if n.endswith((".h", ".hip"))]):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def read_traffic(workload_name):
    """L2-miss bytes (HBM or Infinity Cache) per launch of the dominant kernel from the committed
    rocprofv3 counter summary (profiles/traffic_<workload>.txt, `key = value` lines).
    Returns (bytes or None, note).  The summary names the source files of the kernel it measured
    (`kernel_sources`) and their hash (`kernel_source_sha`); if the files in the tree hash
    differently the summary is reported as stale and its figure is kept out of `traffic`."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload_name}.txt")
    if not os.path.exists(path):
        return None, "no counter summary committed for this workload"
    vals = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            vals[k.strip()] = v.strip()
    try:
        traffic = float(vals["hbm_bytes_per_launch"])
    except (KeyError, ValueError):
        return None, "counter summary has no hbm_bytes_per_launch"
    names = vals.get("kernel_sources", "").split() or None
    try:
        now = kernel_source_sha(names)
    except OSError:
        now = "unreadable"
    sha = vals.get("kernel_source_sha")
    if sha != now:
        return None, (f"stale: summary taken with kernel sources {sha}, tree has {now} "
                      f"(stored figure {traffic:.4g} B)")
    return traffic, f"profiles/{os.path.basename(path)} at commit {vals.get('commit', '?')}"


def cpu_baseline(inp, min_s=12.0):
    """The fp64 oracle, as it stands, timed on this host over a bounded sample
    (whole decode sequences of the same workload, shortest first so that the
    sample holds several) -> context tokens/s."""
    from oracle import echokv_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    w = inp.w
    f64 = lambda t: t.double().numpy()
    W_K, W_V = f64(inp.W_K), f64(inp.W_V)
    order = sorted(range(inp.n_decode), key=lambda b: inp.seq_len[b])
    tokens, seqs, t0 = 0, 0, time.perf_counter()
    while time.perf_counter() - t0 < min_s:       # whole sequences, wrapping round the batch
        b = order[seqs % inp.n_decode]
        r = inp.rows(b)
        orc.echokv_decode(f64(inp.q[b]), f64(inp.K_a[r]), f64(inp.V_a[r]), f64(inp.K_r[r]),
                          f64(inp.V_r[r]), W_K, W_V, w.n_kv_heads)
        tokens += inp.seq_len[b]; seqs += 1
    dt = time.perf_counter() - t0
    return {"value": tokens / dt, "unit": "context tokens/s/layer", "cores": int(threads),
            "kind": "oracle",
            "sample": f"{seqs} whole decode sequences, shortest first ({tokens} context tokens) of "
                      f"{w.name}, fp64 NumPy oracle, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration index (0-4)")
    ap.add_argument("--ramp-seconds", type=float, default=3.0,
                    help="untimed steps for this much wall time before the warm-up, so that the "
                         "timed steps run at the clocks the chip settles at under this load")
    ap.add_argument("--unfused", action="store_true", help="time the unfused comparison path")
    ap.add_argument("--packed-weights", action="store_true",
                    help="lay W_K/W_V out once with echokv_pack_weights before the timed region")
    ap.add_argument("--absorbed", action="store_true",
                    help="time the weight-absorbed decode (same output, other association "
                         "order, HBM-bound) instead of the fused reconstruct-then-attend kernel")
    ap.add_argument("--absorb-v", action="store_true",
                    help="time the value-absorbed decode (keys through the fused predictor product, "
                         "values in the other association order); combines with --rope-window")
    ap.add_argument("--rope-window", action="store_true",
                    help="time the paper-faithful decode instead: rotary embedding applied to the "
                         "rebuilt keys and 4 sink + 128 recent tokens attended uncompressed")
    ap.add_argument("--mlp-hidden", type=int, default=0,
                    help="time decode with the one-hidden-layer predictor of this hidden width (ReLU) "
                         "instead of the linear one")
    ap.add_argument("--no-absorbed", action="store_true",
                    help="skip the extra timing of the weight-absorbed mode after the headline run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain 1 GiB device copies (known HBM traffic) so a counter "
                         "run of this command can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_22910_amd import binding as ek
    from paper_2603_22910_amd import synth
    from paper_2603_22910_amd.harness import DeviceWorkload

    t_gen = time.perf_counter()
    w = synth.CONFIGS[args.config]
    inp = synth.generate(w)
    t_gen = time.perf_counter() - t_gen
    flags = (ek.FLAG_UNFUSED if args.unfused else ek.FLAG_ABSORBED if args.absorbed
             else ek.FLAG_ABSORB_V if args.absorb_v else 0)
    # the default run also times the weight-absorbed mode afterwards (reported beside the
    # headline, never as `value`): size the workspace for both
    also_absorbed = (not args.unfused and not args.absorbed and not args.packed_weights
                     and w.dtype == "bf16" and not args.no_absorbed and not args.rope_window
                     and not args.mlp_hidden and not args.absorb_v)
    dw = DeviceWorkload(inp, flags=flags | (ek.FLAG_ABSORBED if also_absorbed else 0))
    dw.set_flags(flags)
    if args.packed_weights:
        dw.pack_weights()
    dev = dw.dev
    B = inp.n_decode
    dec_tokens = inp.total_decode_tokens

    # the step's new token: the last cached row of every sequence, re-appended
    # each step (lengths are wound back by one on the host, so every step sees
    # exactly the configured context lengths)
    last_rows = torch.tensor([inp.seq_start[b] + inp.seq_len[b] - 1 for b in range(B)], device=dev)
    ka_new, va_new = dw.K_a[last_rows].contiguous(), dw.V_a[last_rows].contiguous()
    kt_new = torch.zeros(B, w.D, dtype=w.torch_dtype, device=dev)
    vt_new = torch.zeros(B, w.D, dtype=w.torch_dtype, device=dev)
    if w.n_retained:
        kt_new[:, :w.n_retained] = dw.K_r[last_rows]
        vt_new[:, :w.n_retained] = dw.V_r[last_rows]
    ones = [1] * B
    full_len = dw.anchor.seq_len.copy()

    extras = None
    if args.rope_window:
        rope = tuple(t.to(dev) for t in synth.rope_tables(w.head_dim, max(inp.seq_len) + 1))
        wk, wv = synth.window_rows(inp, 4, 128)
        extras = (rope, (wk.to(dev), wv.to(dev), 4, 128))

    mlp = None
    if args.mlp_hidden:
        mlp = tuple(t.to(dev) for t in synth.mlp_weights(w, args.mlp_hidden))

    has_prefill = inp.q_prefill is not None

    def step():
        dw.anchor.seq_len[:] = full_len - 1
        ek.cache_append(dw.shape, dw.anchor, ka_new, va_new, ones)
        dw.target.seq_len[:] = full_len - 1
        ek.cache_append(dw.shape, dw.target, kt_new, vt_new, ones)
        if mlp is not None:
            dw.decode_mlp(mlp, args.mlp_hidden, ek.ACT_RELU)
        elif extras is None:
            dw.decode()
        else:
            dw.decode_ex(*extras)
        if has_prefill:            # the configuration's causal prefill chunk rides in the same step
            if extras is None:
                dw.prefill()
            else:                  # the chunk with the rotary embedding (a chunk reads no window)
                dw.prefill_ex(extras[0])

    def clock_ramp():
        # untimed: run the step until the wall time is up (a fresh chip runs its first tens of
        # milliseconds of a heavy load at clocks it does not keep)
        t0, n = time.perf_counter(), 0
        while time.perf_counter() - t0 < args.ramp_seconds:
            step(); n += 1
            torch.cuda.synchronize()
        return time.perf_counter() - t0, n

    def timed_run():
        """Times exactly args.steps steps after args.warmup untimed ones.  Returns the wall time and,
        per profiler channel, (summed kernel ms by HIP events on the launch stream, launches)."""
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        ek.profile_enable(True)
        for ch in range(3):
            ek.profile_read(ch)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = [ek.profile_read(ch) for ch in range(3)]
        ek.profile_enable(False)
        return dt, prof

    ramp_s, ramp_steps = clock_ramp() if args.ramp_seconds > 0 else (0.0, 0)
    dt, prof = timed_run()
    kern_ms, launches = prof[0]
    tokens = dec_tokens
    if has_prefill:
        tokens += inp.seq_len[inp.n_decode]      # the chunk's context counts as processed tokens

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = dt * 1e3 / args.steps
    value = tokens / (dt / args.steps)

    # roofline of the dominant kernel (the fused predictor product + attention):
    # algorithmic work = 4 * d_in * d_out flop per cached token (K and V products)
    flops = 4.0 * w.d_in * w.d_out * dec_tokens
    if args.mlp_hidden:      # two layers, for keys and for values
        flops = 4.0 * args.mlp_hidden * (w.d_in + w.d_out) * dec_tokens
    bytes_alg = dec_tokens * 2.0 * w.d_in * w.elem_size + 2.0 * w.d_in * w.d_out * w.elem_size
    stream_ceiling = None

    def measured_stream_read():
        # what a plain streaming-read kernel gets out of this GPU's memory, over the anchor K cache
        # (or a scratch buffer when that is small): context for the nominal 8 TB/s
        nonlocal stream_ceiling
        if stream_ceiling is None:
            buf = dw.K_a if dw.K_a.numel() * dw.K_a.element_size() >= (1 << 29) else \
                torch.ones(1 << 29, dtype=torch.uint8, device=dev)
            stream_ceiling = ek.profile_stream_read(buf, 5)
        return stream_ceiling

    def absorbed_roofline(kern_ms, launches):
        # the absorbed path's kernels together read every cache row and both weight matrices once
        k_s = kern_ms / launches * 1e-3
        ach = bytes_alg / k_s / 1e9
        traffic, note = read_traffic(w.name + "_absorbed")
        return {"bound": "hbm", "kernel": "absorbed decode (all kernels of the call)",
                "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                "traffic": traffic, "traffic_source": note, "kernel_ms": k_s * 1e3,
                "algorithmic_bytes": bytes_alg, "measured_stream_read_GBs": measured_stream_read()}

    roofline = None
    if args.absorb_v and launches > 0 and kern_ms > 0:
        # keys: the predictor product as it is; values: absorbed -> half of the dense matrix work
        k_s = kern_ms / launches * 1e-3
        ach = 0.5 * flops / k_s / 1e12
        roofline = {"bound": "mfma", "kernel": "fused_kscores_kernel + value-side absorbed kernels",
                    "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / PEAK_BF16_TFLOPS, "traffic": None, "kernel_ms": k_s * 1e3,
                    "algorithmic_flop": 0.5 * flops, "algorithmic_bytes": bytes_alg}
    elif args.absorbed and launches > 0 and kern_ms > 0:
        roofline = absorbed_roofline(kern_ms, launches)
    elif launches > 0 and kern_ms > 0:
        k_s = kern_ms / launches * 1e-3
        ach = flops / k_s / 1e12
        peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS
        plain = not (args.mlp_hidden or args.rope_window or args.unfused or args.packed_weights)
        traffic, note = read_traffic(w.name) if plain else (None, "counter summaries cover the plain fused kernel only")
        roofline = {"bound": "mfma",
                    "kernel": "recon_mfma_kernel + fused_decode_kernel" if args.mlp_hidden else "fused_decode_kernel",
                    "achieved": ach,
                    "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                    "traffic": traffic, "traffic_source": note,
                    "kernel_ms": k_s * 1e3, "launches_timed": launches,
                    "algorithmic_flop": flops, "algorithmic_bytes": bytes_alg,
                    "hbm_frac_of_algorithmic_bytes": bytes_alg / k_s / 1e9 / PEAK_HBM_GBS}

    # second roofline object: the prefill chunk (predictor product over the chunk's visible context
    # + causal attention), both on the matrix cores
    roofline_prefill = None
    if has_prefill and w.dtype == "bf16" and prof[1][1] > 0 and prof[2][1] > 0:
        Lp = inp.seq_len[inp.n_decode]
        Tq, q0 = int(inp.q_prefill.shape[0]), inp.q_pos0
        recon_flop = 4.0 * w.d_in * w.d_out * Lp
        # causal scores + weighted sum: 4 * d flop per (query, visible key, query head)
        pairs = sum(q0 + i + 1 for i in range(Tq))
        attn_flop = 4.0 * w.head_dim * w.n_q_heads * pairs
        r_ms = prof[1][0] / prof[1][1]
        a_ms = prof[2][0] / prof[2][1]
        ach = (recon_flop + attn_flop) / ((r_ms + a_ms) * 1e-3) / 1e12
        traffic, note = read_traffic(w.name + "_prefill")
        roofline_prefill = {
            "bound": "mfma", "kernel": "recon_mfma_kernel + prefill_attn_dma_kernel (one chunk)",
            "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
            "traffic": traffic, "traffic_source": note,
            "kernel_ms": r_ms + a_ms, "algorithmic_flop": recon_flop + attn_flop,
            "predictor_product": {"kernel_ms": r_ms, "algorithmic_flop": recon_flop,
                                  "frac": recon_flop / (r_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
            "attention": {"kernel_ms": a_ms, "algorithmic_flop": attn_flop,
                          "frac": attn_flop / (a_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
            "chunk": {"queries": Tq, "q_pos0": q0, "context": Lp}}

    out = {
        "metric": "context tokens/s/layer for fused reconstruct+decode-attn; % MFMA & HBM peak",
        "value": value, "unit": "context tokens/s/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "context_tokens": tokens,
                   "decode_tokens": dec_tokens,
                   "prefill_chunk_tokens": inp.seq_len[inp.n_decode] if has_prefill else 0,
                   "H_q": w.n_q_heads, "H_kv": w.n_kv_heads, "head_dim": w.head_dim,
                   "n_retained": w.n_retained, "d_in": w.d_in, "d_out": w.d_out,
                   "path": ("unfused" if args.unfused else "absorbed" if args.absorbed
                            else "value-absorbed" if args.absorb_v else "fused"),
                   "extras": "rope + 4 sink + 128 recent window" if args.rope_window else None,
                   "predictor": f"one hidden layer of {args.mlp_hidden}, ReLU" if args.mlp_hidden else "linear",
                   "weights": "packed [d_out,d_in]" if args.packed_weights else "row-major [d_in,d_out]",
                   "step": "cache_append(anchor)+cache_append(target)+decode_attn"
                           + ("+prefill_attn" if has_prefill else "")},
        "clock_ramp": {"seconds": ramp_s, "untimed_steps": ramp_steps},
        "input_generation_s": t_gen,
        "roofline": roofline,
    }
    if roofline_prefill is not None:
        out["roofline_prefill"] = roofline_prefill
    if also_absorbed:
        # same step, same inputs, decode in the other association order (Eq. 3 is linear)
        dw.set_flags(ek.FLAG_ABSORBED)
        dt2, prof2 = timed_run()
        k2, l2 = prof2[0]
        out["absorbed_mode"] = {"value": tokens / (dt2 / args.steps), "unit": "context tokens/s/layer",
                                "ms_per_step": dt2 * 1e3 / args.steps,
                                "roofline": absorbed_roofline(k2, l2) if l2 > 0 and k2 > 0 else None}
        dw.set_flags(flags)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
