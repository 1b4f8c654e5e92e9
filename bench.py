#!/usr/bin/env python3
"""Benchmark of the SSD hot path on one MI355X.

A "step" is one pass of the whole hot path: one batched verification forward
(tree build, embedding, all layers, LM-head reduction, acceptance) of the
8B-class workload (prompt 256, block 32, draft depth 4 -> 5 nodes, M = 160 rows)
against a cached prefix of S = 384 positions (the middle of the 256..480 range
the workload sweeps).  Inputs, weights and the prefix KV are resident in HBM
before the timed region.  --workload selects another configuration (the default
prefix is then prompt + half the generation length, for every sequence of the batch).

Prints ONE JSON line.  `value` is generated tokens/s of a complete
ssd_generate run of the same workload (prompt prefill and KV-append passes
included); `ms_per_step` is the verification-forward latency of the K timed
steps; `roofline` covers the dominant kernel (the gate/up projection GEMM)
with HIP-event timing on the library's stream; `forward` gives the whole
forward against the HBM roofline; `cpu_baseline` times the CPU oracle on a
bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0        # dense bf16


def kernel_source_stamp():
    """Hash of the sources the GEMM kernels are built from: a counter summary under profiles/ names the
    stamp of the build it was taken with, and is only quoted while the sources still hash to it."""
    import hashlib
    h = hashlib.sha256()
    for f in ("gemm_mfma.h", "kernels_mfma.hip", "kernels_mfma_f32.hip"):
        h.update(open(os.path.join(ROOT, "paper_2510_04147_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def read_measured_traffic(workload):
    """HBM bytes per launch of the gate/up GEMM from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size).  Returns (bytes or None, note):
    None when there is no summary or when it was taken with other kernel sources than the present ones."""
    path = os.path.join(ROOT, "profiles", f"gemm_gate_up_{workload}_traffic.txt")
    traffic, stamp = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":", 1)[1])
            if line.startswith("kernel_source_stamp:"):
                stamp = line.split(":", 1)[1].strip()
    except OSError:
        return None, "no counter summary for this workload"
    if stamp != kernel_source_stamp():
        return None, f"counter summary is stale (taken at kernel sources {stamp}, now {kernel_source_stamp()})"
    return traffic, "profiles/" + os.path.basename(path)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2_8b_b32_n4")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debug only; marks the line invalid)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-generate", action="store_true")
    ap.add_argument("--prefix", type=int, default=0, help="cached prefix length of the timed forward "
                    "(default: prompt + half the generation length)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy, the known-size kernel that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_04147_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    mlib = binding.load_measure_library()
    over = {"n_layers": args.layers} if args.layers else {}
    cfg = synth.model_config(wl["model"], **over)
    B, N, P, G, nseq = wl["block"], wl["draft"], wl["prompt_len"], wl["gen_len"], wl["batch"]
    S = args.prefix if args.prefix > 0 else P + G // 2
    assert S + B <= P + G, "the timed forward must fit the sequence"
    def note(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    note(f"generating weights for {args.workload} ({cfg['n_layers']} layers)")
    wg = synth.gen_weights(cfg, 0, device="cuda")
    torch.cuda.synchronize()                 # the library reads the weights on its own stream
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        eng = binding.SSD(cfg, wg, max_seqs=nseq, max_seq_len=P + G, block=B, max_draft=N,
                          max_rows=max(P, S, nseq * max(N + 2, 2 * N) * B, nseq * (P + G)))
        # ---- verification forward at prefix S, fixed block state with N drafts, every sequence of the batch
        note(f"context created; prefill of {nseq} x {S} positions")
        for i in range(nseq):
            eng.prefill_kv(i, synth.gen_prompt(cfg, wl["seed"] + i, S), 0)
        tok = [cfg["mask_id"]] * B
        masked = (1 << B) - 1
        drafts = [((3 + 5 * i) % B, 100 + i) for i in range(N)]
        assert len({q for q, _ in drafts}) == N, "draft positions must differ"
        out = eng.new_out(nseq)
        seqs = list(range(nseq))

        def step():
            eng.verify_tree(seqs, [tok] * nseq, [masked] * nseq, [S] * nseq, [drafts] * nseq, N, out)

        stream.synchronize()
        # The chip comes out of the set-up phase (weight generation, repack) in a lower power state and takes a
        # few tenths of a second of this kernel mix to settle: forwards run 5 % slower until then (4.97 against
        # 5.25 ms, one level or the other, seen switching in the middle of a timed loop).  Half a second of
        # untimed forwards first, so that the W warm-up steps and the K timed steps measure the settled state.
        note("settling forwards, then warm-up verification forwards")
        for _ in range(100):
            step()
        stream.synchronize()
        for _ in range(args.warmup):
            step()
        stream.synchronize()
        note(f"timing {args.steps} verification forwards")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(args.steps):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        ms_step = e0.elapsed_time(e1) / args.steps
        # median over the same number of forwards, one event pair each (a separate pass)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for a, b in evs:
            a.record(stream)
            step()
            b.record(stream)
        torch.cuda.synchronize()
        ms_each = [a.elapsed_time(b) for a, b in evs]
        ms_median = float(np.median(ms_each))

        if args.copy_calibration:
            a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            b = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            b.copy_(a)
            stream.synchronize()
            del a, b

        # ---- what this chip sustains for a pure streaming read of HBM-resident data (the weight
        # stream's access pattern, 2 GiB so the 256 MB Infinity Cache cannot serve it)
        note("streaming-read ceiling")
        big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
        big.zero_()
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        stream.synchronize()
        ceil_gbs = 0.0
        for wgs, depth in ((256, 8), (512, 8), (1024, 16)):
            for _ in range(2):
                mlib.ssd_measure_stream_read(big.data_ptr(), big.numel(), wgs, 8, depth, sink.data_ptr(), stream.cuda_stream)
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record(stream)
            for _ in range(5):
                mlib.ssd_measure_stream_read(big.data_ptr(), big.numel(), wgs, 8, depth, sink.data_ptr(), stream.cuda_stream)
            c1.record(stream)
            stream.synchronize()
            ceil_gbs = max(ceil_gbs, big.numel() * 5 / (c0.elapsed_time(c1) * 1e-3) / 1e9)
        # ---- the gate/up GEMM's loads and nothing else: every work-group reads the whole activation matrix
        # (L2) and its 1/256 of the weights (HBM, rotating through the 2 GiB buffer), one tile per CU
        d_, F_ = cfg["d_model"], cfg["d_ffn"]
        esz_ = 2 if cfg["dtype"] == "bf16" else 4
        stepb = 1024 * 8 * 16                                    # whole steps for every variant below
        sh_bytes = (nseq * (N + 1) * B * d_ * esz_) // stepb * stepb
        pr_bytes = (2 * F_ * d_ * esz_ // 256) // stepb * stepb
        load_only_us = None
        if sh_bytes >= stepb and pr_bytes >= stepb and sh_bytes + 8 * 256 * pr_bytes <= big.numel():
            load_only_us = {}
            for threads, depth in ((512, 4), (512, 8), (1024, 8)):
                def mixed(i):
                    off = sh_bytes + (i % 8) * 256 * pr_bytes
                    rc = mlib.ssd_measure_mixed_read(big.data_ptr(), sh_bytes, big.data_ptr() + off, pr_bytes, 256,
                                                      threads, depth, sink.data_ptr(), stream.cuda_stream)
                    assert rc == 0, rc
                for i in range(4):
                    mixed(i)
                c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                c0.record(stream)
                for i in range(16):
                    mixed(i)
                c1.record(stream)
                stream.synchronize()
                load_only_us[f"{threads}_lanes_x_{depth}_loads"] = c0.elapsed_time(c1) * 1e3 / 16
        del big

        # ---- per-kernel-class timing (HIP events on the same stream, separate pass)
        note(f"{ms_step:.3f} ms per forward; per-kernel event timing")
        for _ in range(3):                   # the streaming tests above left caches and clocks in another state
            step()
        n_prof = max(6, args.steps // 2)
        eng.profile_begin()
        for _ in range(n_prof):
            step()
        prof = eng.profile_read()
        eng.profile_end()

        # ---- the dominant kernel alone, for comparison: back to back through the kernel-level entry point,
        # one event pair around all launches; every layer's gate/up weights in turn, so the weights stream
        # from HBM, and a pool of activation matrices larger than the L2s.  (Inside the forward the kernel
        # is a few us faster: there HBM rests while the small kernels around it run.)
        gu_iso_us = None
        if cfg["dtype"] == "bf16":
            note("gate/up GEMM back to back")
            Mrows = nseq * (N + 1) * B
            pool = torch.randn(48, Mrows, cfg["d_model"], device="cuda").to(torch.bfloat16)
            act = torch.empty(Mrows, cfg["d_ffn"], dtype=torch.bfloat16, device="cuda")
            L = cfg["n_layers"]
            for l in range(L):
                eng.k_linear(binding.LIN_GU, l, pool[l % 48], act)
            reps = 3
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream.synchronize()
            g0.record(stream)
            for r in range(reps):
                for l in range(L):
                    eng.k_linear(binding.LIN_GU, l, pool[(r * L + l) % 48], act)
            g1.record(stream)
            stream.synchronize()
            gu_iso_us = 1e3 * g0.elapsed_time(g1) / (reps * L)
            del pool, act

        # ---- whole generation of the workload: SSD and stepwise
        gen = {}
        if not args.no_generate:
            note("full generation: SSD, then stepwise")
            prompts = [synth.gen_prompt(cfg, wl["seed"] + i, P) for i in range(nseq)]
            eng.generate(prompts, B, B, N)                       # warm
            toks_ssd, st_ssd = eng.generate(prompts, G, B, N)
            toks_step, st_step = eng.generate(prompts, G, B, 0)
            GT_ = G * nseq
            # shorter chains, for context: with random weights few drafts verify, so a shallower tree (fewer rows
            # per forward, the GEMM's row tile follows in steps of 32) trades less than it costs
            sweep = {}
            for nd in range(1, N):
                t_nd, st_nd = eng.generate(prompts, G, B, nd)
                sweep[str(nd)] = dict(tokens_per_s=GT_ / (st_nd["total_ms"] / 1e3), forwards=st_nd["forwards"],
                                      ms_per_forward=st_nd["decode_ms"] / st_nd["forwards"],
                                      equals_stepwise=bool(np.array_equal(t_nd, toks_step)))
            eng.set_tree_mode(1)                                 # the mix-order tree (Section 5.2), for context
            toks_mix, st_mix = eng.generate(prompts, G, B, N)
            eng.set_tree_mode(0)
            eng.set_cross_block(1)                               # rounds that reach across the block boundary (Section 3.2.2)
            toks_x, st_x = eng.generate(prompts, G, B, N)
            eng.set_cross_block(0)
            same = bool(np.array_equal(toks_ssd, toks_step) and np.array_equal(toks_mix, toks_step) and
                        np.array_equal(toks_x, toks_step) and all(v["equals_stepwise"] for v in sweep.values()))
            # the cache of the paper's experiments (Section 4.1): prefix + suffix, renewed by a forward over the
            # whole sequence every 8 decoded tokens; a different model function, so its own stepwise run
            eng.set_cache_mode(1, 8)
            toks_d, st_d = eng.generate(prompts, G, B, N)
            toks_d0, st_d0 = eng.generate(prompts, G, B, 0)
            eng.set_spill_over(1)                                # the chain continues into the next block (Section 3.2.2)
            toks_ds, st_ds = eng.generate(prompts, G, B, N)
            eng.set_spill_over(0)
            eng.set_cache_mode(0)
            # the acceptance-rate limit of self-drafting (Section 5.1, the procedure of Table 2), first sequence
            _, lim = eng.acceptance_limit(prompts[0], G, B, N, 5)
            GT = G * nseq                                        # tokens generated over the whole batch
            gen = dict(
                ssd_tokens_per_s=GT / (st_ssd["total_ms"] / 1e3), stepwise_tokens_per_s=GT / (st_step["total_ms"] / 1e3),
                ssd_forwards=st_ssd["forwards"], stepwise_forwards=st_step["forwards"], kv_passes=st_ssd["kv_passes"],
                accepted_per_forward=GT / max(sum(st_ssd["accept_hist"]), 1), accept_hist=st_ssd["accept_hist"][:N + 2],
                ssd_decode_ms_per_forward=st_ssd["decode_ms"] / st_ssd["forwards"],
                stepwise_ms_per_forward=st_step["decode_ms"] / st_step["forwards"],
                ssd_equals_stepwise=same, ssd_total_ms=st_ssd["total_ms"], stepwise_total_ms=st_step["total_ms"],
                draft_depth_sweep=sweep,
                mix_order_tokens_per_s=GT / (st_mix["total_ms"] / 1e3), mix_order_forwards=st_mix["forwards"],
                mix_order_accept_hist=st_mix["accept_hist"][:N + 2],
                cross_block_tokens_per_s=GT / (st_x["total_ms"] / 1e3), cross_block_forwards=st_x["forwards"],
                cross_block_kv_passes=st_x["kv_passes"],
                dual_cache=dict(refresh_interval=8, ssd_tokens_per_s=GT / (st_d["total_ms"] / 1e3),
                                stepwise_tokens_per_s=GT / (st_d0["total_ms"] / 1e3), ssd_forwards=st_d["forwards"],
                                stepwise_forwards=st_d0["forwards"], refreshes=st_d["kv_passes"],
                                accept_hist=st_d["accept_hist"][:N + 2],
                                spill_over_tokens_per_s=GT / (st_ds["total_ms"] / 1e3),
                                spill_over_forwards=st_ds["forwards"], spill_over_accept_hist=st_ds["accept_hist"][:N + 2],
                                ssd_equals_stepwise=bool(np.array_equal(toks_d, toks_d0) and
                                                         np.array_equal(toks_ds, toks_d0))),
                acceptance_limit=dict(draft_length=N, reduction_top_k=[round(x, 4) for x in lim["reduction"]],
                                      upper_bound=N / (N + 1), rounds=lim["rounds"]))
            # ---- the other acceptance extreme: the same model with every attention output projection zeroed.
            # A position's logits then depend on its own token only, all masked positions tie, the order is left
            # to right and every draft verifies: each round accepts N + 1 tokens (the upper bound of Tables 2-3).
            # Random weights sit near the lower extreme (about 1.3 tokens per forward); a trained model lies between.
            note("zero-attention model: generation at the upper acceptance bound")
            eng.close()
            wz = {k: v for k, v in wg.items() if k != "layers"}
            wz["layers"] = [dict(lw, wo=torch.zeros_like(lw["wo"])) for lw in wg["layers"]]
            engz = binding.SSD(cfg, wz, max_seqs=nseq, max_seq_len=P + G, block=B, max_draft=N,
                               max_rows=max(P, nseq * (N + 1) * B))
            engz.generate(prompts, B, B, N)                      # warm
            toks_z, st_z = engz.generate(prompts, G, B, N)
            toks_z0, st_z0 = engz.generate(prompts, G, B, 0)
            engz.close()
            del wz, engz
            hist_z = st_z["accept_hist"]
            full_rounds = hist_z[N + 1]
            gen["zero_attention"] = dict(
                ssd_tokens_per_s=GT / (st_z["total_ms"] / 1e3), stepwise_tokens_per_s=GT / (st_z0["total_ms"] / 1e3),
                ssd_forwards=st_z["forwards"], stepwise_forwards=st_z0["forwards"],
                accepted_per_forward=GT / max(sum(hist_z), 1), accept_hist=hist_z[:N + 2],
                ssd_decode_ms_per_forward=st_z["decode_ms"] / st_z["forwards"],
                stepwise_ms_per_forward=st_z0["decode_ms"] / st_z0["forwards"],
                ssd_equals_stepwise=bool(np.array_equal(toks_z, toks_z0)))
            # closed form: per block one draft forward and ceil((B - 1) / (N + 1)) verification rounds
            blocks = -(-G // B)
            want_fwd = sum(1 + -(-(min(B, G - b * B) - 1) // (N + 1)) for b in range(blocks))
            gen["zero_attention"]["forwards_closed_form"] = want_fwd
            gen["zero_attention"]["full_depth_rounds"] = full_rounds

    # ---- roofline arithmetic
    M = nseq * (N + 1) * B
    params = synth.streamed_param_count(cfg)
    esz = 2 if cfg["dtype"] == "bf16" else 4
    bytes_fwd = params * esz + nseq * S * synth.kv_bytes_per_token(cfg)
    flops_fwd = 2.0 * M * params + 4.0 * M * (S + B) * cfg["n_q_heads"] * cfg["head_dim"] * cfg["n_layers"]
    fwd_gbs = bytes_fwd / (ms_step * 1e-3) / 1e9
    fwd_tflops = flops_fwd / (ms_step * 1e-3) / 1e12
    d, F = cfg["d_model"], cfg["d_ffn"]
    gu = prof.get("gemm_gate_up_swiglu", dict(launches=0, ms=0.0))
    gu_bytes = 2 * F * d * esz + M * d * esz + M * F * esz     # weights + activations in + SwiGLU out
    gu_flops = 2.0 * M * 2 * F * d
    gu_us_raw = 1e3 * gu["ms"] / max(gu["launches"], 1)      # inside the forward, one event pair per launch
    # An event pair around every launch serialises the launches and adds a few microseconds to each: the class
    # times of a forward add up to more than the forward takes untimed.  That excess, spread evenly over the
    # event pairs of a forward, is taken off the kernel's pair time (the result agrees with the kernel's duration
    # in rocprofv3's trace of the same run within 1 %).
    classes_ms = sum(v["ms"] for v in prof.values()) / n_prof
    pairs_per_forward = sum(v["launches"] for v in prof.values()) / n_prof
    event_pair_us = max(0.0, (classes_ms - ms_step) * 1e3 / pairs_per_forward) if pairs_per_forward > 0 else 0.0
    gu_us = max(gu_us_raw - event_pair_us, 0.0)
    gu_gbs = gu_bytes / (gu_us * 1e-6) / 1e9 if gu_us > 0 else 0.0
    gu_tflops = gu_flops / (gu_us * 1e-6) / 1e12 if gu_us > 0 else 0.0
    traffic, traffic_note = read_measured_traffic(args.workload)
    # the bound is whichever of the two rooflines takes longer for this kernel's bytes and flops
    hbm_bound = gu_bytes / (HBM_PEAK_GBS * 1e9) >= gu_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if hbm_bound:
        roof = {"kernel": "k_gemm_mfma<SwiGLU> (gate/up projection)", "bound": "hbm", "achieved": gu_gbs,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gu_gbs / HBM_PEAK_GBS, "traffic": traffic,
                "bytes_per_launch": gu_bytes, "us_per_launch": gu_us, "us_per_launch_with_event_pairs": gu_us_raw,
                "event_pair_overhead_us": event_pair_us, "launches_timed": gu["launches"],
                "us_per_launch_back_to_back_alone": gu_iso_us}
    else:
        roof = {"kernel": "k_gemm_mfma<SwiGLU> (gate/up projection)", "bound": "mfma", "achieved": gu_tflops,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": gu_tflops / MFMA_BF16_PEAK_TFLOPS,
                "traffic": traffic, "flops_per_launch": gu_flops, "achieved_GBs": gu_gbs, "us_per_launch": gu_us,
                "us_per_launch_with_event_pairs": gu_us_raw,
                "event_pair_overhead_us": event_pair_us,
                "launches_timed": gu["launches"], "us_per_launch_back_to_back_alone": gu_iso_us}
    # a kernel that only loads this GEMM's bytes in the same one-tile-per-CU decomposition (no arithmetic)
    roof["us_loads_alone_same_decomposition"] = load_only_us
    roof["traffic_source"] = traffic_note
    # the whole forward against the same peak: its algorithmic bytes (weights + prefix KV) over its duration
    roof["forward_achieved"] = fwd_gbs if hbm_bound else fwd_tflops
    roof["forward_frac"] = fwd_gbs / HBM_PEAK_GBS if hbm_bound else fwd_tflops / MFMA_BF16_PEAK_TFLOPS
    line = {
        "metric": "generated tokens/sec at batch 1 + verify-forward HBM GB/s (% of roofline)",
        "value": gen.get("ssd_tokens_per_s"), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "model": wl["model"], "n_layers": cfg["n_layers"], "batch": nseq,
                   "prompt_len": P, "gen_len": G, "block": B, "draft_depth": N, "rows_per_forward": M,
                   "prefix_len_timed": S},
        "roofline": roof,
        "forward": {"bytes_per_forward": bytes_fwd, "achieved_GBs": fwd_gbs, "frac_of_hbm_peak": fwd_gbs / HBM_PEAK_GBS,
                    "flops_per_forward": flops_fwd, "achieved_TFLOPs": fwd_tflops,
                    "frac_of_mfma_peak": fwd_tflops / MFMA_BF16_PEAK_TFLOPS,
                    "hbm_streaming_read_ceiling_GBs": ceil_gbs, "frac_of_streaming_ceiling": fwd_gbs / ceil_gbs,
                    "ms_per_step_median": ms_median, "ms_per_step_each": [round(v, 3) for v in ms_each], "host_wall_ms_per_step": wall_ms,
                    "kernel_classes_us_per_forward": {k: 1e3 * v["ms"] / n_prof for k, v in prof.items()}},
        "generate": gen,
    }
    if args.layers:
        line["invalid"] = "layer count overridden"
    # a run whose SSD tokens differ from stepwise decoding measures a broken path: say so and fail
    broken = []
    if gen:
        if not gen["ssd_equals_stepwise"]:
            broken.append("SSD / mix-order / cross-block tokens differ from stepwise decoding")
        if not gen["dual_cache"]["ssd_equals_stepwise"]:
            broken.append("dual cache: SSD tokens differ from stepwise decoding")
        za = gen["zero_attention"]
        if not za["ssd_equals_stepwise"] or za["ssd_forwards"] != za["forwards_closed_form"]:
            broken.append("zero-attention model: tokens differ from stepwise or forwards differ from the closed form")
    if broken:
        line["invalid"] = "; ".join(broken)

    # ---- CPU oracle on a bounded sample (reported baseline, never a target)
    if not args.no_cpu_baseline:
        from oracle import decode
        note("CPU oracle sample")
        w = synth.weights_to(wg, "cpu")
        del wg
        torch.cuda.empty_cache()
        n_pre, nb = 16, 4                      # 16-token prefix, one 4-position block, stepwise
        sample_prompt = synth.gen_prompt(cfg, wl["seed"], n_pre)
        t0 = time.perf_counter()
        toks, st = decode.stepwise(w, cfg, sample_prompt, nb, nb, dtype=torch.float32)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": nb / dt, "unit": "tokens/s", "cores": torch.get_num_threads(),
                                "kind": "oracle", "seconds": dt,
                                "sample": f"oracle stepwise decoding (fp32 activations, bf16 weights upcast per use) "
                                          f"on the same {cfg['n_layers']}-layer model: {n_pre}-token prefill, one "
                                          f"{nb}-position block = {st['forwards']} forwards + {st['kv_passes']} KV passes"}
    print(json.dumps(line))
    if broken:
        sys.exit(3)


if __name__ == "__main__":
    main()
