"""Throughput of the ragged encoder hot path on one MI355X.

A step is one wf_encode_batch call over one synthetic batch (pack + hush append, conv stem, all
transformer blocks, final LayerNorm) with the log-mel input already resident in HBM.  Prints ONE
JSON line: encoded audio-seconds per second (payload audio, hush excluded), plus tokens/s, the
fraction of the bf16 MFMA peak, the roofline of the dominant kernel (HIP-event durations measured
here, on the launch stream) and the CPU oracle timed on a bounded sample of the same workload.
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

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0


def algorithmic_flops(shape, hush_frames, n_frames):
    d, f, N, C = shape.d_model, shape.d_mlp, shape.n_layers, shape.n_mels
    total = 0.0
    for T in n_frames:
        Tp = T + hush_frames
        L = (Tp + 1) // 2
        total += 2.0 * Tp * 3 * C * d                      # conv1: one d x 3C product per frame
        total += 2.0 * L * 3 * d * d                       # conv2
        total += N * (2.0 * L * d * (3 * d + d + 2 * f) + 4.0 * L * L * d)
    return total


def cpu_baseline(wl, weights, hush, mels, budget_flops=6e12):
    """The oracle as it stands, timed on a bounded sample of the workload's streams."""
    import numpy as np
    from oracle import encoder_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    order = sorted(range(len(mels)), key=lambda i: len(mels[i]))
    picks, fl = [], 0.0
    for q in (0.125, 0.375, 0.625, 0.875, 0.25, 0.5, 0.75):      # spread over the length distribution
        i = order[min(len(order) - 1, int(q * len(order)))]
        if i in picks:
            continue
        fi = algorithmic_flops(wl.shape, wl.hush_frames, [len(mels[i])])
        if picks and fl + fi > budget_flops:
            continue
        picks.append(i)
        fl += fi
    t0 = time.perf_counter()
    O.encode_batch(weights, wl.shape.n_heads, [mels[i] for i in picks], hush if wl.hush_frames > 0 else None)
    dt = time.perf_counter() - t0
    audio_s = sum(len(mels[i]) for i in picks) / 100.0
    return {"value": audio_s / dt, "unit": "audio-s/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(picks)} of {len(mels)} streams of {wl.name} ({[len(mels[i]) for i in picks]} frames), "
                      f"NumPy fp64 oracle, {dt:.1f} s wall, {fl / dt / 1e9:.1f} GFLOP/s"}


def bench_small_config(name, steps, warmup):
    """One of the other benchmark configurations through the same entry point: median of per-call HIP-event times
    (these calls are short, so the wall clock over a loop would mostly measure the host)."""
    import torch
    from paper_2412_11272_amd import binding as wf
    from paper_2412_11272_amd import synth
    wl = synth.workload(name)
    weights, hush, mels = synth.materialize(wl)
    enc = wf.encoder_for_workload(wl, weights, hush, wf.WF_PRECISION_BF16)
    flat, offs, nf = wf.pack_mels(mels)
    mel = torch.from_numpy(flat).cuda()
    cu, total_frames, M = wf.plan_batch(enc.cfg, nf)
    out = torch.empty((M, wl.shape.d_model), device="cuda", dtype=torch.bfloat16)
    stream = torch.cuda.current_stream().cuda_stream

    def timed():
        for _ in range(warmup):
            enc.encode(mel, offs, nf, out=out, stream=stream)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for e0, e1 in evs:
            e0.record()
            enc.encode(mel, offs, nf, out=out, stream=stream)
            e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps * 1e3
        per_call = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        return per_call[len(per_call) // 2], wall

    ms, wall = timed()
    ms_graph = None
    if enc.get_lanes() >= 1 and M < 8192:          # one-lane batches can be replayed from a captured graph (opt-in)
        enc.set_graphs(True)
        ms_graph, _ = timed()
        if enc.graph_stats()["replays"] == 0:
            ms_graph = None
        enc.set_graphs(False)
    enc.close()
    flops = algorithmic_flops(wl.shape, wl.hush_frames, nf)
    payload = float(sum(wl.n_frames)) / synth.FRAMES_PER_SECOND          # seeded audio only: the padding of cfg4a is not payload
    return {"streams": len(nf), "tokens": int(M), "ms": round(ms, 4), "ms_wall_mean": round(wall, 4),
            "ms_graph_replay": None if ms_graph is None else round(ms_graph, 4),
            "tokens_per_s": round(M / ms * 1e3, 1), "audio_s_per_s": round(payload / ms * 1e3, 1),
            "algorithmic_gflop": round(flops / 1e9, 2),
            "pct_bf16_mfma_peak": round(100.0 * flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 2)}


def bench_configs(steps, warmup):
    """Every benchmark configuration besides the headline one, plus the tokens-saved speed-up of the truncated
    buffer over the padded 30 s window (same 8 streams, same payload)."""
    res = {}
    for name in ("cfg1", "cfg2-2s", "cfg2-4s", "cfg2-8s", "cfg3", "cfg4a", "cfg4b"):
        res[name] = bench_small_config(name, max(steps, 30) if name < "cfg4" else steps, warmup)
    a, b = res["cfg4a"], res["cfg4b"]
    res["cfg4_padded_over_truncated"] = {"time_ratio_t4a_over_t4b": round(a["ms"] / b["ms"], 2),
                                         "flop_ratio": round(a["algorithmic_gflop"] / b["algorithmic_gflop"], 2),
                                         "token_ratio": round(a["tokens"] / b["tokens"], 2)}
    return res


def bench_frontend(wl, n_frames, steps, warmup):
    """Raw 16 kHz audio of the workload's lengths + the 8000-sample hush word -> packed log-mel (not part of `value`)."""
    import numpy as np
    import torch
    from paper_2412_11272_amd import binding as wf
    from paper_2412_11272_amd import synth
    lens = [int(t) * synth.SAMPLES_PER_FRAME for t in n_frames]
    audios = synth.make_audios([int(t) for t in n_frames], wl.seeds["mel"])
    hush = synth.make_hush_audio(wl.seeds["hush"])
    fe = wf.Frontend(wl.shape.n_mels, hush, len(lens), sum(lens) + len(lens) * len(hush))
    audio = torch.from_numpy(np.concatenate(audios)).cuda()
    offs = np.concatenate([[0], np.cumsum(lens)[:-1]])
    frames = sum(fe.n_frames(lens))
    out = torch.empty((frames, wl.shape.n_mels), device="cuda", dtype=torch.float32)
    for _ in range(warmup):
        fe.logmel(audio, offs, lens, out=out)
    torch.cuda.synchronize()
    # one event pair per call and the median over calls: the HIP runtime stalls the host once for tens of
    # milliseconds after a few dozen back-to-back sub-millisecond calls, which says nothing about the kernels
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in evs:
        e0.record()
        fe.logmel(audio, offs, lens, out=out)
        e1.record()
    torch.cuda.synchronize()
    per_call = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    ms = per_call[len(per_call) // 2]
    ms_mean = sum(per_call) / len(per_call)
    fe.close()
    flops = frames * (2.0 * 2 * 400 * 201)                     # the DFT contraction; the mel filters are a few % of it
    return {"ms": round(ms, 4), "ms_mean": round(ms_mean, 4), "timing": "median of per-call HIP-event times", "frames": int(frames), "audio_s_per_s": round(sum(lens) / 16000.0 / (ms / 1e3), 1),
            "dft_tflops": round(flops / ms / 1e9, 2), "peak_fp32_mfma_tflops": 157.3,
            "frac": round(flops / ms / 1e9 / 157.3, 4), "dtype": "f32"}


def bench_prefill(wl, states, cu, steps, warmup):
    """Decoder-side consumers of the encoder states of the same batch: per-layer cross-attention K/V
    projection, then ~100 prompt tokens per stream through the decoder (reported separately, not part of `value`)."""
    import numpy as np
    import torch
    from paper_2412_11272_amd import binding as wf
    from paper_2412_11272_amd import synth
    name = next(k for k, v in synth.SHAPES.items() if v == wl.shape)
    shape = synth.DEC_SHAPES[name]
    B, M, P = len(cu) - 1, int(cu[-1]), synth.PROMPT_TOKENS
    w = synth.make_decoder_weights(shape, wl.seeds["weights"] + 6)
    prompts = synth.make_prompts([P] * B, shape.n_vocab, wl.seeds["weights"] + 7)
    dec = wf.Decoder(shape, w, B, M, P * B, wf.WF_PRECISION_BF16)
    del w
    kv = torch.empty((shape.n_layers, M, 2 * shape.d_model), device="cuda", dtype=torch.bfloat16)
    hidden = torch.empty((P * B, shape.d_model), device="cuda", dtype=torch.bfloat16)
    logits = torch.empty((B, shape.n_vocab), device="cuda", dtype=torch.float32)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    ms_kv = timed(lambda: dec.cross_kv(states, out=kv))
    ms_pf = timed(lambda: dec.prefill(prompts, cu, kv, hidden=hidden, logits=logits))
    dec.set_profiling(True)
    dec.cross_kv(states, out=kv)
    dec.prefill(prompts, cu, kv, hidden=hidden, logits=logits)
    torch.cuda.synchronize()
    stats = dec.kernel_stats()
    dec.close()
    d, f, N = shape.d_model, shape.d_mlp, shape.n_layers
    fl_kv = 2.0 * M * d * 2 * d * N
    Pt = P * B
    fl_pf = N * (2.0 * Pt * d * (3 * d + d + d + d + 2 * f) + 2.0 * B * P * (P + 1) * d + 4.0 * P * M * d) + 2.0 * B * d * shape.n_vocab
    kern = {s["name"]: {"launches": s["launches"], "avg_ms": round(s["total_ms"] / s["launches"], 4),
                        "tflops": round(s["flops"] / s["total_ms"] / 1e9, 1) if s["flops"] else None}
            for s in stats if s["launches"]}
    return {"decoder": f"{name}: {N} layers, {P} prompt tokens x {B} streams, {M} encoder tokens",
            "cross_kv_ms": round(ms_kv, 3), "cross_kv_tflops": round(fl_kv / ms_kv / 1e9, 1),
            "prefill_ms": round(ms_pf, 3), "prefill_tflops": round(fl_pf / ms_pf / 1e9, 1), "dtype": "bf16", "kernels": kern}


def bench_rounds(wl, weights, hush, n_rounds):
    """Processing rounds over the workload's streams (Section "Operations"; step length and best effort,
    Section "Key Implementation Details"): every stream ingests audio in real time, each round encodes the
    current buffers as one ragged batch; virtual time advances by the measured round time.  Reported per
    step length, with the padded-30 s-window baseline next to it (not part of `value`)."""
    import numpy as np
    import torch
    from paper_2412_11272_amd import binding as wf
    from paper_2412_11272_amd import synth
    S, H, MAXF, TRACK = len(wl.n_frames), wl.hush_frames, 3000, 6016
    rng = np.random.default_rng(wl.seeds["lengths"] + 100)
    starts = [int(x) for x in rng.integers(0, 15_000_000, size=S)]        # streams out of phase by up to 15 s
    tracks = torch.from_numpy(np.clip(rng.normal(-0.3, 0.4, size=(S, TRACK, wl.shape.n_mels)), -1, 1).astype(np.float32)).cuda().bfloat16()
    out = torch.empty((S * (MAXF + H + 1) // 2, wl.shape.d_model), device="cuda", dtype=torch.bfloat16)
    res = []
    for mode in ("ragged+hush", "padded-30s"):
        pad = 0 if mode == "ragged+hush" else MAXF
        hf = H if pad == 0 else 0
        cfg = wf.make_config(wl.shape, hf, S, S * (MAXF + hf), MAXF + hf, wf.WF_PRECISION_BF16)
        enc = wf.Encoder(cfg, weights, hush if hf else None)
        for step_s in (0.01, 0.5, 1.0, 2.0):
            sim = wf.Rounds(starts, int(step_s * 1e6), 1500, 100, MAXF)
            while True:                                   # host-only fast-forward to t = 20 s: buffers in steady state
                s, _, _ = sim.begin()
                sim.end(1000)
                if s >= 20_000_000:
                    break
            sim.run(enc, tracks, 2, out, pad_to_frames=pad)
            sim.reset_stats()
            rec = sim.run(enc, tracks, n_rounds, out, pad_to_frames=pad)
            st = sim.stats()
            sim.close()
            span = (rec[-1]["end_us"] - rec[0]["start_us"]) / 1e6
            res.append({"mode": mode, "step_s": step_s, "rounds": n_rounds,
                        "round_ms_mean": round(st["mean_proc_us"] / 1e3, 2), "round_ms_max": round(st["max_proc_us"] / 1e3, 2),
                        "tokens_per_round": round(sum(r["tokens"] for r in rec) / n_rounds, 1),
                        "streams_per_round": round(sum(r["n_active"] for r in rec) / n_rounds, 1),
                        "word_latency_s": round(st["mean_latency_us"] / 1e6, 4),
                        "gpu_busy_frac": round(sum(r["proc_us"] for r in rec) / 1e6 / span, 4)})
        enc.close()
    return {"streams": S, "buffer_trim_s": 15.0, "runs": res}


def bench_beam(n_sessions):
    """Beam-pruning state machine on synthetic decoding sessions (host only; reported separately)."""
    from paper_2412_11272_amd import binding as wf
    from paper_2412_11272_amd import synth
    sessions = synth.make_beam_sessions(n_sessions, synth.BASE_SEED + 90)
    res = {"sessions": n_sessions, "original_beam": synth.BEAM_SIZE,
           "paper_table": "reduce ratio 53.8-68.6 %, average beam 2.26-2.85 of 5 (its data and models; context only)"}
    # both readings of the selective-matching rule: exempt tokens also left out of the reference (the library's
    # default), and the paper's literal rule (only the current best token is exempt)
    for key, filt in (("filtered_reference", True), ("literal_reference", False)):
        bp = wf.BeamPruner(synth.BEAM_SIZE, [], synth.TEXT_VOCAB, synth.PUNCT_IDS, filter_reference=filt)
        steps = reduced = beam_sum = 0
        t0 = time.perf_counter()
        for ref, cur in sessions:
            bp.reset(ref)
            beams, _ = bp.session(cur)
            steps += len(beams)
            reduced += int((beams < synth.BEAM_SIZE).sum())
            beam_sum += int(beams.sum())
        dt = time.perf_counter() - t0
        bp.close()
        res[key] = {"decoding_steps": steps, "reduce_ratio": round(reduced / steps, 4), "avg_beam": round(beam_sum / steps, 3),
                    "steps_per_s_one_core_incl_binding": round(steps / dt, 1)}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--lanes", type=int, default=0,
                    help="lanes of the encoder in the timed region (0 = the library's default); per-kernel durations are "
                         "always measured with one lane, i.e. with kernels running one at a time")
    ap.add_argument("--graphs", action="store_true", help="replay one-lane batches from captured HIP graphs (wf_encoder_set_graphs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--encoder-only", action="store_true",
                    help="time the encoder hot path only; by default the legs of the other rows (front end, decoder-side "
                         "steps, round driver, beam pruning) run after it and are reported in objects of their own")
    ap.add_argument("--frontend", action="store_true",
                    help="with --encoder-only: also time the raw-audio log-mel front end on audio of the same lengths")
    ap.add_argument("--prefill", action="store_true",
                    help="with --encoder-only: also time the decoder-side steps on the encoder states of the same batch")
    ap.add_argument("--rounds", type=int, default=-1,
                    help="processing rounds per step length through the round driver (default 8; 0 with --encoder-only)")
    ap.add_argument("--beam-sessions", type=int, default=-1,
                    help="synthetic decoding sessions for the beam-pruning state machine, host only (default 2000; 0 with --encoder-only)")
    ap.add_argument("--configs", action="store_true",
                    help="with --encoder-only: also time the other benchmark configurations (cfg1 .. cfg4b); on by default otherwise")
    ap.add_argument("--copy-calib-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (known traffic, to scale rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    legs = not args.encoder_only and args.workload == "cfg5"
    args.frontend = args.frontend or legs
    args.configs = args.configs or legs
    args.prefill = args.prefill or legs
    if args.rounds < 0:
        args.rounds = 8 if legs else 0
    if args.beam_sessions < 0:
        args.beam_sessions = 2000 if legs else 0
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (streams shard across GPUs without collectives; "
              "no multi-GPU path is built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2412_11272_amd import binding as wf
    from paper_2412_11272_amd import synth

    torch.cuda.set_device(0)
    prop = torch.cuda.get_device_properties(0)
    # dense bf16 MFMA peak = CUs x 4096 flop per clock x clock; the published 2.5 PFLOP/s is 256 CUs at 2.4 GHz and is
    # what every fraction here is quoted against, whatever the device reports
    khz = wf.device_info()["clock_khz"]
    peak_note = {"used_tflops": PEAK_BF16_TFLOPS, "device": prop.name, "compute_units": int(prop.multi_processor_count),
                 "max_clock_ghz": round(khz / 1e6, 3),
                 "from_device_tflops": round(prop.multi_processor_count * 4096 * khz * 1e3 / 1e12, 1)}
    wl = synth.workload(args.workload)
    weights, hush, mels = synth.materialize(wl)
    enc = wf.encoder_for_workload(wl, weights, hush, wf.WF_PRECISION_BF16)
    if args.lanes > 0:
        enc.set_lanes(args.lanes)
    if args.graphs:
        enc.set_graphs(True)
    lanes_timed = enc.get_lanes()
    flat, offs, nf = wf.pack_mels(mels)
    mel = torch.from_numpy(flat).cuda()
    cu, total_frames, M = wf.plan_batch(enc.cfg, nf)
    out = torch.empty((M, wl.shape.d_model), device="cuda", dtype=torch.bfloat16)
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        enc.encode(mel, offs, nf, out=out, stream=stream)

    if args.copy_calib_mib > 0:
        src = torch.ones(args.copy_calib_mib * 262144, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps

    # the same call timed one by one with an event pair each (median: robust against a host hiccup in the loop)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_call = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    ms_median = per_call[len(per_call) // 2]

    # same steps again with every launch bracketed by HIP events on the launch stream, on ONE lane so that a
    # kernel's duration is its own: with more lanes kernels of different groups overlap
    enc.set_lanes(1)
    enc.set_profiling(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_prof = (time.perf_counter() - t0) / args.steps
    stats = enc.kernel_stats()
    enc.set_profiling(False)

    payload_audio_s = float(sum(nf)) / synth.FRAMES_PER_SECOND
    flops = algorithmic_flops(wl.shape, wl.hush_frames, nf)
    kernels = {}
    for s in stats:
        if s["launches"] == 0:
            continue
        ms = s["total_ms"] / s["launches"]
        kernels[s["name"]] = {"launches_per_step": s["launches"] // args.steps, "avg_ms": round(ms, 4),
                              "share": round(s["total_ms"] / args.steps / (dt_prof * 1e3), 4),
                              "tflops": round(s["flops"] / s["total_ms"] / 1e9, 1) if s["flops"] else None,
                              "gbs": round(s["bytes"] / s["total_ms"] / 1e6, 1)}
    mfma = [s for s in stats if s["flops"] > 0 and s["launches"] > 0]
    dom = max(mfma, key=lambda s: s["total_ms"])
    achieved = dom["flops"] / dom["total_ms"] / 1e9          # TFLOP/s
    # HBM-side bytes cannot be counted from inside this process: the figure is the one recorded by the rocprofv3 --pmc
    # runs of this same command (profiles/traffic.json, with the commit it was taken at), not a measurement of this run
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            traffic = tj.get(args.workload, {}).get(dom["name"], {}).get("total_bytes")
            traffic_src = f"profiles/traffic.json ({tj.get('_recorded_at', 'commit not recorded')})"
        except Exception:
            traffic = None
    roofline = {"kernel": dom["name"], "bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_unit": "bytes per launch (L2 fill + write-back, rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE, calibrated)",
                "traffic_source": traffic_src,
                "algorithmic_bytes_per_launch": dom["bytes"] / dom["launches"],
                "avg_launch_ms": round(dom["total_ms"] / dom["launches"], 4),
                "flops_per_launch": dom["flops"] / dom["launches"],
                "ms_per_step_profiled": round(dt_prof * 1e3, 3),
                "measured_with": "one lane (kernels one at a time), every launch bracketed by HIP events"}

    result = {
        "metric": "encoded audio-sec/sec & tokens/sec per GPU; % of bf16 MFMA peak",
        "value": round(payload_audio_s / dt, 1), "unit": "audio-s/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt * 1e3, 3),
        "ms_per_step_median_of_event_timed_calls": round(ms_median, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{wl.name}: large-v3-shaped encoder, 64 ragged streams" if wl.name == "cfg5" else wl.name,
                   "streams": len(nf), "tokens": int(M), "frames_incl_hush": int(total_frames),
                   "payload_audio_s": payload_audio_s, "d_model": wl.shape.d_model, "n_layers": wl.shape.n_layers,
                   "lanes": lanes_timed},
        "tokens_per_s": round(M / dt, 1),
        "audio_s_per_s_incl_hush": round(total_frames / synth.FRAMES_PER_SECOND / dt, 1),
        "algorithmic_tflops": round(flops / dt / 1e12, 1),
        "pct_bf16_mfma_peak": round(100.0 * flops / dt / 1e12 / PEAK_BF16_TFLOPS, 2),
        "peak": peak_note,
        "roofline": roofline,
        "kernels": kernels,
    }
    if args.frontend:
        result["frontend"] = bench_frontend(wl, nf, args.steps, args.warmup)
    enc.close()
    if args.configs:
        del mel
        mel = None
        torch.cuda.empty_cache()
        result["configs"] = bench_configs(args.steps, args.warmup)
    if args.prefill:
        result["prefill"] = bench_prefill(wl, out, cu, args.steps, args.warmup)
    del mel, out
    if args.beam_sessions > 0:
        result["beam_pruning"] = bench_beam(args.beam_sessions)
    if args.rounds > 0:
        torch.cuda.empty_cache()
        result["rounds"] = bench_rounds(wl, weights, hush, args.rounds)
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, weights, hush, mels)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
