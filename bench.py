#!/usr/bin/env python3
"""Throughput of block-denoising decode on one MI355X (synthetic, random-init, batch 1).

Workload = the headline configuration: Qwen2.5-VL-3B-shaped bf16 backbone, prefix of 1024 (768 synthetic
visual embeddings + 256 random text ids), blocks of B=32 with a fixed schedule of 4 unmasks per step.
One "step" of this benchmark is one whole block: the autoregressive seed, 8 denoising forwards with their
LM-head/confidence/unmask, and the causal commit forward (9 weight passes, 32 tokens).  Inputs are resident
in HBM before the timed region; the prefill is not timed.

Prints ONE JSON line (see the keys below).  `roofline` prices the dominant kernel class (by time) against
the 8 TB/s HBM peak using HIP events recorded around every launch in a second pass over the same steps;
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK = 2.5e15      # dense bf16 MFMA, FLOP/s
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "streaming_forward_config1_hbm_traffic.txt")


def measured_traffic(weights, layers, prefix, block):
    """HBM bytes one launch of the layers kernel moves on the default workload, from the hardware counters summarised in
    profiles/streaming_forward_config1_hbm_traffic.txt (FETCH_SIZE and WRITE_SIZE, scaled by a reference copy): its line
    'traffic_bytes_per_launch layers <bytes>'.  None for any other workload, or when the file is not there."""
    if (weights, layers, prefix, block) != ("bf16", 36, 1024, 32):
        return None
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == "layers":
                return float(f[2])
    except OSError:
        pass
    return None


def phase_timeline(ctx, n_layers):
    """Per-phase time line of the last forward from the kernel's own 100 MHz stamps (bd_k_trace): for every phase the
    time from the first workgroup's start to the last arrival at the barrier that ends it, the median workgroup's time
    in the phase, and the barrier's cost from the last arrival to the last release; averaged over layers 1..L-1."""
    import numpy as np
    t = ctx.bd_k_trace_read().astype(np.int64)
    t = (t - t[:, 0].min()) / 100.0                      # microseconds
    rows = []
    for e, name in enumerate(["qkv", "attention", "o", "gate/up", "down"]):
        span, med, bar = [], [], []
        for l in range(1, n_layers):
            start, arrive, release = t[:, l * 10 + 2 * e], t[:, 1 + l * 10 + 2 * e], t[:, 2 + l * 10 + 2 * e]
            span.append(arrive.max() - start.min())
            med.append(np.median(arrive - start))
            bar.append(release.max() - arrive.max())
        rows.append((name, float(np.mean(span)), float(np.mean(med)), float(np.mean(bar))))
    return rows, float(t.max())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8, help="blocks of 32 tokens to time (8 = 256 tokens)")
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layers", type=int, default=36, help="debug only: fewer layers (result is then not the metric)")
    ap.add_argument("--prefix", type=int, default=None, help="committed prefix length (default 1024; 2048 with --weights fp8)")
    ap.add_argument("--weights", choices=["bf16", "fp8"], default="bf16",
                    help="fp8 = configs[4]: e4m3 decoder linears with per-output-channel scales (seed 2), prefix 2048; "
                         "not the headline metric")
    ap.add_argument("--block", type=int, default=32)
    ap.add_argument("--fixed-k", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-pass", action="store_true")
    ap.add_argument("--verify", action="store_true",
                    help="also time the speculative verify pass (configs[3]): B drafted ids, one causal forward + accept")
    ap.add_argument("--speculative", type=int, default=0, metavar="N",
                    help="also time N iterations of the linear self-speculative loop (Alg. 1: draft + verify + accept "
                         "per call); with random weights nearly every draft is rejected, so this is ~2 forwards per token")
    ap.add_argument("--quadratic", type=int, default=0, metavar="B",
                    help="also time 8 iterations of the quadratic speculative loop (Alg. 2) with block size B "
                         "(B*(B+1) <= 64 rows, one forward per iteration)")
    ap.add_argument("--timeline", action="store_true",
                    help="instead of the benchmark: print the per-phase time line of one denoising forward (in-kernel "
                         "timestamps) at this prefix, as text")
    ap.add_argument("--flags", type=int, default=0, help="bd_config.flags of the context (alternative code paths, see include/bd.h)")
    ap.add_argument("--shuffle-pages", action="store_true",
                    help="hand the cache pages out in a shuffled order (the kernels then follow the page table)")
    ap.add_argument("--floors", action="store_true",
                    help="bound the layers kernel instead of benchmarking: its time with no weight requests (fixed cost of "
                         "hand-overs, barriers and arithmetic) and the time of its weight stream alone")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy kernel (reference for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU path (batch-1 decode); run with --gpus 1. "
              "Independent requests per GPU are the multi-GPU form and need no communication.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_06832_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    B, K = args.block, args.fixed_k
    fp8 = args.weights == "fp8"
    if args.prefix is None:
        args.prefix = 2048 if fp8 else 1024
    shape = inputs.QWEN3B.with_layers(args.layers)
    threads = min(16, os.cpu_count() or 8)

    t0 = time.time()
    w = inputs.make_weights(shape, 2 if fp8 else 0, args.weights, threads=threads)
    n_embed = args.prefix * 3 // 4
    emb, ids = inputs.make_prompt(shape, n_embed, args.prefix - n_embed, seed=104 if fp8 else 101)
    print(f"[bench] weights generated in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    blocks = args.warmup + args.steps
    max_seq = args.prefix + (max(blocks, args.steps) + 1) * B
    if args.quadratic > 0:        # eight iterations of at most qB accepted tokens, and the forward's qB (qB + 1) parked rows
        max_seq = max(max_seq, args.prefix + 8 * args.quadratic + args.quadratic * (args.quadratic + 1))
    ctx = binding.Context(shape, max_seq=max_seq, max_block=64,
                          weight_dtype=binding.BD_FP8_E4M3 if fp8 else binding.BD_BF16, flags=args.flags)
    if args.shuffle_pages:
        n_pages = -(-max_seq // 32)
        ctx.bd_kv_page_order(np.random.default_rng(5).permutation(n_pages).astype(np.int32))
    t0 = time.time()
    ctx.load_model(w)
    print(f"[bench] weights uploaded in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)
    d_emb = torch.from_numpy(emb).cuda()
    d_ids = torch.from_numpy(ids).cuda()
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    msk = torch.empty(B, dtype=torch.uint8, device="cuda")
    n_den = -(-(B - 1) // K)                     # denoising forwards per block

    def decode_block():
        tok.fill_(shape.mask_token_id)
        msk.fill_(1)
        for _ in range(n_den):
            ctx.bd_denoise_step(tok, msk, 0.9, K)
        ctx.bd_commit_block(tok)

    prefill_s = []
    block_ms = []                                # per-block latency of the last run, from events on the stream

    def run(n_blocks, after_prefill=None):
        tp = time.perf_counter()
        ctx.bd_prefill(d_emb, d_ids)
        torch.cuda.synchronize()
        prefill_s.append(time.perf_counter() - tp)
        if after_prefill is not None:
            after_prefill()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_blocks + 1)]
        t = time.perf_counter()
        ev[0].record()
        for i in range(n_blocks):
            decode_block()
            ev[i + 1].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        block_ms[:] = [ev[i].elapsed_time(ev[i + 1]) for i in range(n_blocks)]
        return dt

    if args.calibrate_copy:
        # a plain copy of known size: 2^28 fp32 read + written once (1 GiB each way), for scaling FETCH_SIZE / WRITE_SIZE
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.floors:
        def layers_us(c):
            c.bd_prefill(d_emb, d_ids)
            tok.fill_(shape.mask_token_id)
            msk.fill_(1)
            for _ in range(3):
                c.bd_denoise_step(tok, msk, 0.9, 1)
            c.bd_status()
            c.bd_k_profile(True)
            for _ in range(10):
                c.bd_denoise_step(tok, msk, 0.9, 1)
            c.bd_status()
            ms, cnt, _ = c.bd_k_profile_read()["layers"]
            c.bd_k_profile(False)
            return ms / cnt * 1e3
        full = layers_us(ctx)
        floor_ms, floor_bytes = ctx.bd_k_stream_floor(10)
        ctx.close()
        ctx2 = binding.Context(shape, max_seq=args.prefix + 2 * B, max_block=64,
                               weight_dtype=binding.BD_FP8_E4M3 if fp8 else binding.BD_BF16,
                               flags=binding.BD_FLAG_MEASURE_NO_WEIGHTS)
        ctx2.load_model(w)
        fixed = layers_us(ctx2)
        ctx2.close()
        L = shape.n_layers
        print(f"bounds of the layers kernel: {args.weights} weights, {L} layers, prefix {args.prefix}, B={B} (mean of 10 forwards, HIP events)")
        print(f"layers kernel as it runs                          {full:8.0f} us  {full / L:6.1f} us per layer")
        print(f"no weight requests (hand-overs, barriers, MFMAs)  {fixed:8.0f} us  {fixed / L:6.1f} us per layer   [results are wrong by construction]")
        print(f"weight stream alone ({floor_bytes / 1e9:.3f} GB, no consumer)       {floor_ms * 1e3:8.0f} us  {floor_ms * 1e3 / L:6.1f} us per layer   "
              f"= {floor_bytes / floor_ms / 1e6:.0f} GB/s")
        print(f"fixed + stream = {fixed + floor_ms * 1e3:.0f} us; the kernel overlaps {fixed + floor_ms * 1e3 - full:.0f} us of the two")
        return

    if args.timeline:
        ctx.bd_prefill(d_emb, d_ids)
        tok.fill_(shape.mask_token_id)
        msk.fill_(1)
        for _ in range(3):
            ctx.bd_denoise_step(tok, msk, 0.9, 1)
        ctx.bd_status()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            ctx.bd_denoise_step(tok, msk, 0.9, 1)
        e1.record()
        torch.cuda.synchronize()
        ctx.bd_k_trace(True)
        ctx.bd_denoise_step(tok, msk, 0.9, 1)
        ctx.bd_status()
        rows, span = phase_timeline(ctx, shape.n_layers)
        ctx.bd_k_trace(False)
        print(f"phase time line of one denoising forward: {args.weights} weights, {shape.n_layers} layers, prefix {args.prefix}, B={B}")
        print(f"forward (layers kernel + LM head + unmask), mean of 10 untraced: {e0.elapsed_time(e1) * 100:.0f} us; "
              f"traced layers kernel: {span:.0f} us")
        print(f"{'phase':10s} {'first start -> last arrival':>28s} {'median workgroup':>18s} {'barrier (last arrival -> last release)':>40s}   [us, mean over layers 1..L-1]")
        for name, sp, md, br in rows:
            print(f"{name:10s} {sp:28.2f} {md:18.2f} {br:40.2f}")
        print(f"{'sum':10s} {sum(r[1] for r in rows):28.2f} {'':18s} {sum(r[3] for r in rows):40.2f}   -> {sum(r[1] + r[3] for r in rows):.1f} us per layer")
        ctx.close()
        return

    run(args.warmup)                              # untimed warm-up blocks, then the prompt is prefilled afresh
    elapsed = run(args.steps)
    lat = sorted(block_ms)
    pct = lambda q: lat[min(len(lat) - 1, int(round(q * (len(lat) - 1))))] if lat else None
    step_latency = {"unit": "ms per block", "median": round(pct(0.5), 4), "p10": round(pct(0.1), 4), "p90": round(pct(0.9), 4),
                    "per_forward_median": round(pct(0.5) / (n_den + 1), 4)}
    assert int(msk.sum().item()) == 0 and ctx.bd_cache_len() == args.prefix + args.steps * B
    tokens = args.steps * B
    forwards = args.steps * (n_den + 1)
    ms_fwd = elapsed * 1e3 / forwards
    # algorithmic bytes of the whole run: weights once per forward + cached K/V at each block's length
    kv_pos_bytes = shape.n_layers * 2 * shape.kv_dim * 2
    w_bytes = 2 * shape.weight_elements()
    if fp8:   # one byte per decoder weight + 4 bytes per output channel; LM head stays bf16
        lm = shape.vocab * shape.hidden
        rows = shape.q_dim + 2 * shape.kv_dim + 2 * shape.hidden + 2 * shape.ffn
        w_bytes = (shape.weight_elements() - lm) + 2 * lm + 4 * rows * shape.n_layers
    total_bytes = sum((n_den + 1) * (w_bytes + kv_pos_bytes * (args.prefix + b * B)) for b in range(args.steps))
    step_frac = total_bytes / elapsed / 1e9 / HBM_PEAK_GBS

    verify_ms = None
    if args.verify:
        draft = torch.randint(0, shape.vocab - 1, (B,), dtype=torch.int32, device="cuda")
        pred = torch.zeros(B, dtype=torch.int32, device="cuda")
        nacc = torch.zeros(1, dtype=torch.int32, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ctx.bd_verify_block(draft, False, pred, nacc)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            ctx.bd_verify_block(draft, False, pred, nacc)
        e1.record()
        torch.cuda.synchronize()
        verify_ms = e0.elapsed_time(e1) / 10

    spec = None
    if args.speculative > 0:
        n_it = min(args.speculative, args.steps)            # the cache was sized for `steps` blocks
        ctx.bd_prefill(d_emb, d_ids)
        outp = torch.zeros(B, dtype=torch.int32, device="cuda")
        ctx.bd_speculative_step(B, outp)
        ctx.bd_prefill(d_emb, d_ids)
        torch.cuda.synchronize()
        t = time.perf_counter()
        emitted = 0
        for _ in range(n_it):
            emitted += ctx.bd_speculative_step(B, outp)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        spec = {"iterations": n_it, "tokens": emitted, "tokens_per_s": round(emitted / dt, 1),
                "ms_per_iteration": round(dt * 1e3 / n_it, 4), "forwards_per_iteration": 2 if B > 1 else 1}

    quad = None
    if args.quadratic > 0:
        qB = args.quadratic
        ctx.bd_prefill(d_emb, d_ids)
        dq = torch.zeros(qB, dtype=torch.int32, device="cuda")
        nq = torch.zeros(qB, dtype=torch.int32, device="cuda")
        ctx.bd_quad_draft(qB, dq)
        ctx.bd_quad_step(qB, dq, nq)
        ctx.bd_prefill(d_emb, d_ids)
        ctx.bd_quad_draft(qB, dq)
        torch.cuda.synchronize()
        t = time.perf_counter()
        emitted = 0
        for _ in range(8):
            emitted += ctx.bd_quad_step(qB, dq, nq)
            dq, nq = nq, dq
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        quad = {"block": qB, "rows_per_forward": qB * (qB + 1), "iterations": 8, "tokens": emitted,
                "tokens_per_s": round(emitted / dt, 1), "ms_per_iteration": round(dt * 1e3 / 8, 4)}

    roofline = None
    if not args.no_kernel_pass:
        run(args.steps, after_prefill=lambda: ctx.bd_k_profile(True))   # events around the decode launches only
        prof = ctx.bd_k_profile_read()
        ctx.bd_k_profile(False)
        stream = {k: v for k, v in prof.items() if v[2] > 0 and v[1] > 0}
        dom = max(stream, key=lambda k: stream[k][0])
        ms, cnt, nbytes = stream[dom]
        achieved = nbytes / (ms / cnt * 1e-3) / 1e9
        # which roofline bounds the dominant kernel is decided by measurement: its fraction of the HBM peak on the
        # algorithmic bytes against its fraction of the dense bf16 MFMA peak on the linears' flops for B rows
        mfma_flops = 2.0 * B * (shape.weight_elements() - shape.vocab * shape.hidden)
        mfma_frac = mfma_flops / (ms / cnt * 1e-3) / MFMA_BF16_PEAK if dom == "layers" else 0.0
        roofline = {"bound": "hbm" if achieved / HBM_PEAK_GBS >= mfma_frac else "mfma", "kernel": dom, "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "mfma_frac": round(mfma_frac, 4),
                    "traffic": measured_traffic(args.weights, args.layers, args.prefix, B) if dom == "layers" else None,
                    "avg_kernel_us": round(ms / cnt * 1e3, 2), "launches": cnt,
                    "classes": {k: {"avg_us": round(v[0] / v[1] * 1e3, 2), "launches": v[1],
                                    "GBps": round(v[2] / (v[0] / v[1] * 1e-3) / 1e9, 1) if v[2] else None}
                                for k, v in prof.items() if v[1] > 0}}

    cpu = None
    if not args.no_cpu_baseline:
        # the oracle as it stands, in float32, on the workload itself: the prompt is prefilled (not timed, as for the
        # GPU), then three denoising forwards and the commit forward of the first block are timed and extrapolated over
        # the block's schedule (n_den denoising forwards + 1 commit)
        from oracle.bd_oracle import BlockDiffusionOracle
        ctx.close()
        del ctx
        torch.cuda.empty_cache()
        o = BlockDiffusionOracle(shape, w, dtype=np.float32)
        tp = time.perf_counter()
        o.prefill(emb, ids, chunk=256)
        t_prefill = time.perf_counter() - tp
        t = np.full(B, shape.mask_token_id, np.int32)
        m = np.ones(B, bool)
        n_f = min(3, n_den)
        t1 = time.perf_counter()
        for _ in range(n_f):
            o.denoise_step(t, m, 0.9, K)
        t_den = (time.perf_counter() - t1) / max(n_f, 1)
        t[m] = 0                                   # (a block is committed complete: the timing does not depend on the ids)
        t1 = time.perf_counter()
        o.commit_block(t)
        t_com = time.perf_counter() - t1
        cpu = {"value": round(B / (n_den * t_den + t_com), 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
               "sample": f"float32 numpy oracle on {threads} host threads, same workload (prefix {args.prefix}, B={B}, {K} reveals/step): "
                         f"{n_f} denoising forwards ({t_den:.2f} s each) + the commit forward ({t_com:.2f} s) of the first block, "
                         f"extrapolated over its {n_den}+1 forwards; prompt pass {t_prefill:.1f} s, not counted"}
        ctx = None

    out = {
        "metric": f"decoded tokens/s at batch 1, 3B-shaped bf16, B={B}; % HBM roofline per step" if not fp8 else
                  f"decoded tokens/s at batch 1, 3B-shaped e4m3 weights (bf16 arithmetic), B={B}; % HBM roofline per step",
        "value": round(tokens / elapsed, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed * 1e3 / args.steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"configs[{4 if fp8 else {1024: 1, 8192: 2, 2048: 3}.get(args.prefix, 1)}]: 3B-shaped {'e4m3-weight' if fp8 else 'bf16'} ({shape.n_layers} layers), prefix {args.prefix} "
                               f"({n_embed} visual embeddings + {args.prefix - n_embed} ids), B={B}, "
                               f"fixed {K} unmasks/step, {tokens} tokens",
                   "block": B, "fixed_k": K, "prefix": args.prefix, "forwards_per_block": n_den + 1},
        "ms_per_forward": round(ms_fwd, 4), "hbm_roofline_frac_step": round(step_frac, 4), "step_latency": step_latency,
        **({"speculative": spec} if spec is not None else {}),
        **({"quadratic": quad} if quad is not None else {}),
        # the prompt pass (not part of `value`): large-M kernels for all but its last rows; linears only in the flop count
        "prefill": {"ms": round(min(prefill_s) * 1e3, 3), "tokens_per_s": round(args.prefix / min(prefill_s), 1),
                    "TFLOPs": round(2.0 * args.prefix * (shape.weight_elements() - shape.vocab * shape.hidden)
                                    / min(prefill_s) / 1e12, 1)},
        "algorithmic_GB_per_forward": round(total_bytes / forwards / 1e9, 4),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if verify_ms is not None:
        out["verify_pass_ms"] = round(verify_ms, 4)
    print(json.dumps(out), flush=True)
    if ctx is not None:
        ctx.close()


if __name__ == "__main__":
    main()
