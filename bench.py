#!/usr/bin/env python3
"""Benchmark of the block-span server path on one MI355X.

A "step" is one batched decode step: one span_forward call that advances every session of
the workload by one token through all blocks of the span (norms, projections, rotary /
ALiBi, paged attention over the server-held cache, MLP).  Before the timed steps the
sessions' caches are built by cache replay (span_replay over the stored prefix inputs),
which is timed on its own and reported as replay tokens/s.

Prints ONE JSON line.  `value` = decode steps/s with all inputs resident in HBM.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate


def device_weights(shape, seed, device):
    """Seeded random-init weights drawn on the device (bench only; the parity tests use the
    numpy recipe of workloads/).  Same distributions: matrices 0.02*N(0,1), gains 1+0.02*N(0,1)."""
    import torch
    from workloads import tensor_shapes
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    out = []
    for _ in range(shape.n_blocks):
        blk = {}
        for name, dims in tensor_shapes(shape).items():
            t = torch.randn(dims, generator=g, device=device, dtype=torch.float32) * 0.02
            if name.endswith("_g"):
                t += 1.0
            blk[name] = t.to(torch.bfloat16)
        out.append(blk)
    return out


def library_source_sha() -> str:
    """Hash of the HIP sources the loaded library is built from (kernels and launch code)."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2312_08361_amd", "csrc", "*.h*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def recorded_traffic(workload: str, kernel: str):
    """HBM bytes per launch from the rocprofv3 --pmc runs summarised under profiles/ (FETCH_SIZE and WRITE_SIZE
    need runs of their own, so this figure is recorded, not measured by this run).  Returned only when the
    record was made with the kernel sources this run uses; otherwise (None, why)."""
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(tpath):
        return None, "no profiles/traffic.json"
    rec = json.load(open(tpath))
    src = rec.get("_source", {})
    if src.get("csrc_sha") != library_source_sha():
        return None, f"profiles/traffic.json was recorded with other kernel sources (sha {src.get('csrc_sha')}): dropped"
    val = rec.get(workload, {}).get(kernel)
    return val, f"recorded: profiles/traffic.json, rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of these kernel sources ({src.get('summary', 'profiles/')})"


def launch_stream(stream: int):
    """torch's handle of the HIP stream the library launches on, for recording events in order with its kernels.
    The library is given torch's current stream, which here is the null stream: that one must be addressed as
    torch's own current stream -- torch.cuda.ExternalStream(0) is not the null stream, and events recorded on it
    are stamped when the host enqueues them (measured: 2.00 ms per step against 2.30 by the wall clock and by
    events on the current stream)."""
    import torch
    cur = torch.cuda.current_stream()
    return cur if cur.cuda_stream == stream else torch.cuda.ExternalStream(stream)


def cpu_baseline(wl, decode_len, sample_tokens=256):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample:
    one block of the span (the blocks are identical in cost), fp32 arithmetic."""
    import numpy as np
    from oracle import span_oracle as so
    from workloads import SpanWeights, draw_hidden
    nproc = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas_threads = nproc
    cores = min(blas_threads, nproc)          # the oracle's time is in numpy's BLAS calls: the threads it actually used
    shape = wl.shape
    one = shape.with_blocks(1)
    w = {k: np.asarray(v, dtype=np.float32) for k, v in SpanWeights(one, seed=wl.seed)[0].items()}
    rng = np.random.default_rng(7)
    # decode: every session attends over a cache of `decode_len` tokens (contents do not affect time)
    past_k = rng.standard_normal((decode_len, shape.n_kv_heads, shape.head_dim), dtype=np.float32)
    past_v = rng.standard_normal((decode_len, shape.n_kv_heads, shape.head_dim), dtype=np.float32)
    xs = draw_hidden(shape, wl.seed, 0, wl.n_sessions)
    t0 = time.perf_counter()
    for b in range(wl.n_sessions):
        so.block_forward(one, w, xs[b:b + 1], past_k, past_v, dtype=np.float32)
    t_dec = (time.perf_counter() - t0) * shape.n_blocks            # whole span, all sessions
    # replay: sample_tokens of one session through one block
    xr = draw_hidden(shape, wl.seed, 1, sample_tokens)
    e = np.zeros((0, shape.n_kv_heads, shape.head_dim), np.float32)
    t0 = time.perf_counter()
    so.block_forward(one, w, xr, e, e, dtype=np.float32, matrix_attention=True)
    t_rep = (time.perf_counter() - t0) * shape.n_blocks
    return {"value": 1.0 / t_dec, "unit": "steps/s", "cores": int(cores), "nproc": int(nproc), "blas_threads": int(blas_threads),
            "kind": "oracle",
            "replay_tokens_per_s": sample_tokens / t_rep,
            "sample": f"fp32 oracle, 1 of {shape.n_blocks} blocks (x{shape.n_blocks} extrapolated): decode = "
                      f"{wl.n_sessions} sessions x 1 token over a {decode_len}-token cache; replay = "
                      f"{sample_tokens} tokens of one session"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama70b")
    ap.add_argument("--replay-reps", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-profile", action="store_true")
    ap.add_argument("--weight-bits", type=int, default=16, choices=[16, 8, 4],
                    help="compressed weights (Section 3.1 of the paper); 16 = the bf16 configuration of the headline metric")
    ap.add_argument("--hidden-codec", action="store_true",
                    help="also time the 8-bit block-wise codec of hidden states on the replay's output rows")
    ap.add_argument("--beam-reorder", action="store_true",
                    help="also time cache reordering of the decode batch used as a beam")
    ap.add_argument("--mixed-call", action="store_true",
                    help="also time one call in which all sessions but one decode while the last one replays its prefix")
    ap.add_argument("--training", action="store_true",
                    help="also time the training-time passes (Section 3.3): forward, and forward + backward w.r.t. the "
                         "input activations, on batches of 128-token sequences")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device copy (known HBM bytes) so that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2312_08361_amd import binding as B
    from paper_2312_08361_amd.server import SpanServer, config_for
    from workloads import WORKLOADS, normal_levels16
    from workloads import accounting as acc

    wl = WORKLOADS[args.workload]
    shape = wl.shape
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    K, W = args.steps, args.warmup
    n_sess = wl.n_sessions
    prefix = list(wl.prefix_lens)
    total_prefix = sum(prefix)
    prof_steps = 0 if args.no_kernel_profile else min(K, 16)
    max_len = max(prefix) + W + K + prof_steps + 1
    pages = sum((p + W + K + prof_steps + 1 + 15) // 16 for p in prefix)
    cfg = config_for(shape, max_pages=pages + 8, max_sessions=n_sess, max_session_tokens=max_len,
                     max_batch_tokens=min(total_prefix, 16384), io_f32=False,
                     weight_bits=0 if args.weight_bits == 16 else args.weight_bits,
                     levels=normal_levels16() if args.weight_bits == 4 else None)
    t_setup = time.perf_counter()
    srv = SpanServer(cfg, device_weights(shape, wl.seed, dev), dev, keep_canonical=args.training)
    torch.cuda.synchronize()
    stream = srv.stream

    g = torch.Generator(device=dev)
    g.manual_seed(1234)
    x_past = torch.randn((total_prefix, shape.d_model), generator=g, device=dev).to(torch.bfloat16)
    y_past = torch.empty_like(x_past)
    n_dec = W + K + prof_steps
    x_dec = torch.randn((n_dec, n_sess, shape.d_model), generator=g, device=dev).to(torch.bfloat16)
    y_dec = torch.empty_like(x_dec[0])
    setup_s = time.perf_counter() - t_setup

    # ---- cache replay (prefill), timed on fresh sessions -----------------------------------
    replay_ms = []
    sessions = []
    for rep in range(args.replay_reps + 1):                 # first repetition is the warm-up
        for s in sessions:
            srv.close(s)
        sessions = [srv.open(max_len) for _ in range(n_sess)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.span_replay(srv.span, sessions, prefix, x_past, y_past, stream)
        torch.cuda.synchronize()
        if rep > 0:
            replay_ms.append((time.perf_counter() - t0) * 1e3)
    replay_ms_med = float(np.median(replay_ms))
    replay_tok_s = total_prefix / (replay_ms_med * 1e-3)
    replay_flops = acc.prefill_flops(shape, prefix)

    # ---- decode steps ----------------------------------------------------------------------
    ones = [1] * n_sess
    for i in range(W):
        B.span_forward(srv.span, sessions, ones, x_dec[i], y_dec, stream)
    torch.cuda.synchronize()
    ext = launch_stream(stream)                        # the stream the library launches on
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(ext)
    for i in range(W, W + K):
        B.span_forward(srv.span, sessions, ones, x_dec[i], y_dec, stream)
    ev1.record(ext)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step_events = ev0.elapsed_time(ev1) / K
    ms_per_step = dt / K * 1e3
    steps_per_s = K / dt
    mean_past = [p + W + (K - 1) / 2.0 for p in prefix]
    step_bytes = acc.decode_step_bytes(shape, mean_past, args.weight_bits)

    # ---- per-kernel durations with HIP events (separate pass: events perturb step time) ----
    roofline = None
    kernels = {}
    roofline_replay = None
    if prof_steps:
        B.span_debug_profile(srv.span, 1)
        for i in range(W + K, W + K + prof_steps):
            B.span_forward(srv.span, sessions, ones, x_dec[i], y_dec, stream)
        torch.cuda.synchronize()
        names = {B.SPAN_K_NORM: "norm", B.SPAN_K_SKINNY: "gemv_kernel", B.SPAN_K_ATTN_DECODE: "attn_kernel<decode>",
                 B.SPAN_K_ATTN_MERGE: "attn_merge_kernel"}
        raw = {}
        for cls, name in names.items():
            n, ms = B.span_debug_profile_read(srv.span, cls)
            if n:
                raw[name] = (n, ms)
        # An event bracket around every launch keeps the next launch from being set up while
        # the current kernel drains, so every bracketed duration carries a constant extra.  The
        # timed region above has no brackets and (kernel trace) no gaps between kernels, so
        # the extra per launch is (sum of bracketed durations per step - un-bracketed step
        # time) / launches per step; it is subtracted from every average below.
        launches_per_step = sum(n for n, _ in raw.values()) / prof_steps
        bracketed_step_us = sum(ms for _, ms in raw.values()) / prof_steps * 1e3
        overhead_us = max(0.0, (bracketed_step_us - ms_per_step * 1e3) / launches_per_step)
        for name, (n, ms) in raw.items():
            kernels[name] = {"launches_per_step": n / prof_steps, "avg_us": ms / n * 1e3 - overhead_us,
                             "avg_us_bracketed": ms / n * 1e3,
                             "us_per_step": (ms / n * 1e3 - overhead_us) * n / prof_steps}
        n, ms = raw["gemv_kernel"]
        # the weight-streaming projection is launched 4x per block; together the launches of one
        # step read every weight of the span exactly once
        wbytes = acc.weight_bytes(shape) if args.weight_bits == 16 else acc.compressed_weight_bytes(shape, args.weight_bits)
        bytes_per_launch = wbytes / (4 * shape.n_blocks)
        avg_s = (ms / n * 1e3 - overhead_us) * 1e-6
        achieved = bytes_per_launch / avg_s / 1e9
        traffic, traffic_source = recorded_traffic(args.workload, "gemv_kernel")
        if args.weight_bits != 16:
            traffic, traffic_source = None, "not recorded for compressed weights"
        roofline = {"kernel": "gemv_kernel" if args.weight_bits == 16 else f"gemvq_kernel ({args.weight_bits}-bit weights)", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                    "bytes_per_launch": bytes_per_launch, "avg_launch_us": avg_s * 1e6,
                    "avg_launch_us_bracketed": ms / n * 1e3, "bracket_overhead_us": overhead_us}
        # replay: the tiled MFMA projection
        for s in sessions:
            srv.close(s)
        sessions = [srv.open(max_len) for _ in range(n_sess)]
        B.span_debug_profile(srv.span, 1)
        B.span_replay(srv.span, sessions, prefix, x_past, y_past, stream)
        torch.cuda.synchronize()
        n, ms = B.span_debug_profile_read(srv.span, B.SPAN_K_TILED)
        n_at, ms_at = B.span_debug_profile_read(srv.span, B.SPAN_K_ATTN_PREFILL)
        if n:
            flops_per_launch = 2.0 * acc.params_per_block(shape, False) * total_prefix / 4
            # chunked replay launches each projection once per chunk; scale to the launches seen
            flops_per_launch *= (4 * shape.n_blocks) / n
            avg_s = ms / n * 1e-3
            tf = flops_per_launch / avg_s / 1e12
            tr, tr_source = recorded_traffic(args.workload, "gemmd_kernel")
            roofline_replay = {"kernel": "gemmd_kernel", "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                               "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": tr, "traffic_source": tr_source,
                               "flops_per_launch": flops_per_launch, "avg_launch_us": avg_s * 1e6,
                               "attn_prefill_ms_total": ms_at, "gemm_ms_total": ms}
        B.span_debug_profile(srv.span, 0)

    # ---- optional: 8-bit codec of the hidden states that leave the span (replay output, decode output) ----
    codec = None
    if args.hidden_codec:
        from workloads import dynamic_levels256
        lv = dynamic_levels256()
        d = shape.d_model
        res = {}
        for name, src in (("replay_rows", y_past), ("decode_rows", y_dec)):
            Mrows = src.shape[0]
            codes = torch.empty((Mrows, d), dtype=torch.uint8, device=dev)
            amax = torch.empty((Mrows, d // 64), dtype=torch.float32, device=dev)
            back = torch.empty_like(src)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            for rep in range(3):
                with torch.cuda.stream(launch_stream(stream)):
                    ev[0].record()
                    B.span_hidden_encode(src, 0, Mrows, d, 64, lv, codes, amax, stream)
                    ev[1].record()
                    B.span_hidden_decode(codes, amax, Mrows, d, 64, lv, 0, back, stream)
                    ev[2].record()
                torch.cuda.synchronize()
            enc_us, dec_us = ev[0].elapsed_time(ev[1]) * 1e3, ev[1].elapsed_time(ev[2]) * 1e3
            byt = Mrows * d * 3 + Mrows * d // 64 * 4                      # bf16 rows + codes + block maxima
            res[name] = {"rows": Mrows, "encode_us": enc_us, "decode_us": dec_us,
                         "encode_gbs": byt / enc_us / 1e3, "decode_gbs": byt / dec_us / 1e3}
        codec = res

    # ---- optional: cache reordering of the batch taken as one beam (after the decode steps) ----
    beam = None
    if args.beam_reorder:
        lens0 = [B.span_session_length(srv.span, s) for s in sessions]
        hypo = [(i * 5 + 1) % n_sess if i % 3 else i for i in range(n_sess)]      # clones, moves, keeps and drops
        times = []
        for rep in range(12):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.span_reorder(srv.span, sessions, hypo, stream)
            torch.cuda.synchronize()
            if rep >= 2:
                times.append((time.perf_counter() - t0) * 1e6)
        page_bytes = 2 * shape.n_kv_heads * 16 * shape.head_dim * 2 * shape.n_blocks
        beam = {"beam": n_sess, "cached_tokens": lens0[0], "hypo_ids": hypo, "us_per_reorder": float(np.median(times)),
                "bytes_copied_at_most": (n_sess - 1) * page_bytes,
                "bytes_a_contiguous_cache_would_move":
                    2 * acc.kv_cache_bytes(shape.n_blocks, shape.n_kv_heads * shape.head_dim, sum(lens0))}
        for s in sessions:
            srv.close(s)
        sessions = [srv.open(max_len) for _ in range(n_sess)]

    # ---- optional: continuous batching, one call = (n_sess - 1) decode tokens + one session's replay ----
    mixed = None
    if args.mixed_call:
        for s in sessions:
            srv.close(s)
        sessions = [srv.open(max_len) for _ in range(n_sess)]
        B.span_replay(srv.span, sessions[:-1], prefix[:-1], x_past[:total_prefix - prefix[-1]], y_past, stream)
        x_mix = torch.cat([x_dec[0][:n_sess - 1], x_past[total_prefix - prefix[-1]:]])
        y_mix = torch.empty_like(x_mix)
        counts = [1] * (n_sess - 1) + [prefix[-1]]
        times = []
        for rep in range(4):                                    # first repetition is the warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.span_forward(srv.span, sessions, counts, x_mix, y_mix, stream)
            torch.cuda.synchronize()
            if rep:
                times.append((time.perf_counter() - t0) * 1e3)
            srv.close(sessions[-1])
            sessions[-1] = srv.open(max_len)
        t_mix = float(np.median(times))
        # the same work as two calls: the newcomer's replay alone, then the decode step of the others
        sep = []
        for rep in range(4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            B.span_replay(srv.span, sessions[-1:], prefix[-1:], x_mix[n_sess - 1:], y_mix[n_sess - 1:], stream)
            B.span_forward(srv.span, sessions[:-1], [1] * (n_sess - 1), x_mix[:n_sess - 1], y_mix[:n_sess - 1], stream)
            torch.cuda.synchronize()
            if rep:
                sep.append((time.perf_counter() - t0) * 1e3)
            srv.close(sessions[-1])
            sessions[-1] = srv.open(max_len)
        mixed = {"call": f"{n_sess - 1} sessions x 1 token (past {prefix[0]}+) + 1 session x {prefix[-1]} replayed tokens",
                 "ms": t_mix, "tokens": sum(counts), "tokens_per_s": sum(counts) / (t_mix * 1e-3),
                 "same_work_as_two_calls_ms": float(np.median(sep))}

    # ---- optional: training-time passes on batches of 128-token sequences (no sessions, no cache) ----
    training = None
    if args.training:
        for s in sessions:
            srv.close(s)
        sessions = []
        cap = min(4096, cfg.max_batch_tokens) // 128 * 128
        srv.attach_training(cap)
        res = {}
        for n_seq in sorted({8, cap // 128}):
            if n_seq * 128 > cap or n_seq > 64:
                continue
            lens = [128] * n_seq
            ntok = 128 * n_seq
            xt, gt = x_past[:ntok], x_past[ntok:2 * ntok] if total_prefix >= 2 * ntok else x_past[:ntok]
            yt, gx = torch.empty_like(xt), torch.empty_like(xt)
            tf, tb = [], []
            for rep in range(4):                                # first repetition is the warm-up
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                B.span_train_forward(srv.span, 0, shape.n_blocks, lens, xt, yt, stream)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                B.span_backward(srv.span, 0, shape.n_blocks, lens, xt, gt, gx, None, stream)
                torch.cuda.synchronize()
                t2 = time.perf_counter()
                if rep:
                    tf.append((t1 - t0) * 1e3)
                    tb.append((t2 - t1) * 1e3)
            f_ms, b_ms = float(np.median(tf)), float(np.median(tb))
            lin = 2.0 * acc.params_per_block(shape, False) * shape.n_blocks * ntok      # projections of one forward
            # the projections of one backward call on their own (HIP events around every projection launch)
            B.span_debug_profile(srv.span, 1)
            B.span_backward(srv.span, 0, shape.n_blocks, lens, xt, gt, gx, None, stream)
            torch.cuda.synchronize()
            n_t, ms_t = B.span_debug_profile_read(srv.span, B.SPAN_K_TILED)
            B.span_debug_profile(srv.span, 0)
            # forward sweep without the last block's down projection + the four transposed projections of every block
            proj_flops = 2 * lin - 2.0 * shape.d_model * shape.d_ff * ntok
            roof = None if not n_t else {"kernel": "gemmd_kernel / gemm_kernel (all projections of one backward call)",
                                         "bound": "mfma", "achieved": proj_flops / (ms_t * 1e-3) / 1e12,
                                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                         "frac": proj_flops / (ms_t * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                         "launches": n_t, "projection_ms_total": ms_t}
            res[f"{n_seq}x128"] = {
                "tokens": ntok, "forward_ms": f_ms, "forward_tokens_per_s": ntok / (f_ms * 1e-3),
                "backward_call_ms": b_ms, "backward_call_tokens_per_s": ntok / (b_ms * 1e-3),
                "forward_projection_tflops": lin / (f_ms * 1e-3) / 1e12,
                # a backward call = forward sweep (without the last down projection) + the four transposed projections
                "backward_call_projection_tflops": 2 * lin / (b_ms * 1e-3) / 1e12,
                "roofline_backward_projections": roof}
        training = {"note": "span_train_forward; span_backward = forward sweep + backward sweep in one call (the request "
                            "carries the inputs again, the server keeps nothing between requests)",
                    "extra_bytes": {"transposed_weights": srv.train_sizes[0], "scratch": srv.train_sizes[1]}, **res}

    # ---- practical ceilings of this device, beside the published peaks ----
    ceil_buf = torch.randn(1 << 29, device=dev, dtype=torch.float32).to(torch.bfloat16)      # 1 GiB of random bf16
    ceil_out = torch.empty(1 << 16, dtype=torch.float32, device=dev)
    read_gbs, mfma_tf = B.span_debug_ceilings(ceil_buf, ceil_buf.numel() * 2, ceil_out, stream)
    del ceil_buf, ceil_out
    ceilings = {"stream_read_gbs": read_gbs, "mfma_loop_tflops_random_bf16_operands": mfma_tf,
                "note": "pure read of 1 GiB; register-only 32x32x16 bf16 MFMA loop on N(0,1) operands",
                # the same rates against what this very device sustains (the matrix-loop figure differs by 10 % and more
                # between devices of one model: it is the clock their power management allows under that load)
                "decode_frac_of_stream_read": step_bytes / (ms_per_step * 1e-3) / 1e9 / read_gbs if read_gbs > 0 else None,
                "replay_frac_of_mfma_loop": replay_flops / (replay_ms_med * 1e-3) / 1e12 / mfma_tf if mfma_tf > 0 else None}

    out = {
        "metric": "70B-span decode steps/s + HBM GB/s %peak; cache-replay prefill tokens/s",
        "value": steps_per_s, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "ms_per_step_hip_events": ms_per_step_events, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if args.weight_bits == 16 else f"bf16 x {args.weight_bits}-bit block-quantised weights", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {shape.n_blocks} blocks, d_model {shape.d_model}, "
                               f"{shape.n_q_heads}/{shape.n_kv_heads} heads x {shape.head_dim}, d_ff {shape.d_ff}, "
                               f"{n_sess} sessions, prefix {min(prefix)}..{max(prefix)} tokens, 16-token KV pages",
                   "sessions": n_sess, "decode_start_len": max(prefix) + W, "arch": shape.arch},
        "session_tokens_per_s": steps_per_s * n_sess,
        "decode_algorithmic_bytes_per_step": step_bytes,
        "decode_hbm_gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "decode_hbm_frac_of_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "replay_tokens_per_s": replay_tok_s, "replay_ms": replay_ms_med, "replay_ms_runs": replay_ms, "replay_tokens": total_prefix,
        "replay_tflops": replay_flops / (replay_ms_med * 1e-3) / 1e12,
        "replay_mfma_frac_of_peak": replay_flops / (replay_ms_med * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "roofline": roofline, "roofline_replay": roofline_replay, "kernels_per_decode_step": kernels,
        "setup_s": setup_s, "ceilings": ceilings,
    }
    if mixed:
        out["mixed_call"] = mixed
    if beam:
        out["beam_reorder"] = beam
    if codec:
        out["hidden_codec"] = codec
    if training:
        out["training_passes"] = training
    srv.destroy()
    del srv
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, max(prefix))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
