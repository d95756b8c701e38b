#!/usr/bin/env python3
"""Training-throughput benchmark of the RNNLM hot path on one MI355X.

A "step" is one training window of the whole hot path (stream indexing, gather, recurrent forward,
output layer, softmax/cross-entropy gradient, BPTT, all SGD updates) on seeded synthetic Zipf
streams that are already resident in HBM.  Prints ONE JSON line:

  value            training words/s = steps * B * T / seconds
  roofline         dense-MFMA roofline of the dominant kernel (the slowest of the three output-layer
                   contractions, found during warm-up), timed live inside the timed region with HIP events
                   on the kernel's stream; the other contractions ("gemm_ms") are timed in a short pass after
                   the region, because every bracketing event costs the stream several microseconds
  cpu_baseline     the fp64 oracle timed on a bounded sample of the same workload on the host cores

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--config all|cfg3|cfg4|cfg5] [--stages]
                       [--criterion softmax|nce|score] [--noise K] [--optimizer sgd|rmsprop] [--arch plain|compressed]

--config all (the default, full softmax + SGD only): the headline line is cfg5, the largest single-GPU
configuration; the same line carries the objects "cfg3" and "cfg4" with the same measurements of the two
other configurations the metric's target names (each timed with the same --steps / --warmup).

--criterion nce times the same window with the noise-contrastive output layer (the "next" row after the
headline path): K shared noise words per window drawn from the smoothed unigram of the token array.
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

PEAK_BF16_TFLOPS = 2516.6   # MI355X published dense bf16 MFMA peak
PEAK_FP32_TFLOPS = 157.3    # MI355X published fp32 matrix peak
PEAK_HBM_GBS = 8000.0       # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="all",
                    help="all: headline cfg5 plus sub-objects cfg3 and cfg4; or one configuration of synth.CONFIGS")
    ap.add_argument("--stages", action="store_true", help="also time every stage (adds event overhead)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--criterion", choices=["softmax", "nce", "score"], default="softmax",
                    help="softmax: training with the full normalised output (headline metric); nce: training with "
                         "noise-contrastive estimation; score: forward-only unnormalised scoring of given next words")
    ap.add_argument("--optimizer", choices=["sgd", "rmsprop"], default="sgd",
                    help="sgd: the fused plain SGD step (headline metric); rmsprop: the rmsprop-scaled step "
                         "(smoothing 0.9995, one statistic per word for E and Wo), full softmax only")
    ap.add_argument("--arch", choices=["plain", "compressed"], default="plain",
                    help="compressed: the architecture of Sec. 5.4 (512-unit layers below and above the state, tied "
                         "word matrix) on its word-prediction shape (config wp10k), full softmax + SGD")
    ap.add_argument("--streams", type=int, default=0, help="override the number of parallel streams B (scoring)")
    ap.add_argument("--noise", type=int, default=1024, help="noise words per window for --criterion nce")
    ap.add_argument("--shortlist", type=int, default=0,
                    help="--criterion score: score this many candidate words per position (Sec. 5.4 ranks a shortlist "
                         "of 100) instead of the one given next word")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three 256 MiB device-to-device copies (counter calibration for profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    comp = args.arch == "compressed"
    if comp and (args.criterion == "nce" or args.optimizer != "sgd"):
        print("bench.py: --arch compressed runs with the full softmax and plain SGD, or --criterion score",
              file=sys.stderr)
        return 2
    if args.optimizer == "rmsprop" and args.criterion == "score":
        print("bench.py: --criterion score has no optimiser", file=sys.stderr)
        return 2
    plain_headline = not comp and args.criterion == "softmax" and args.optimizer == "sgd"
    if args.config == "all":
        args.config = "cfg5" if plain_headline else ("wp10k" if comp else "cfg3")
        others = ["cfg3", "cfg4"] if plain_headline else []
    else:
        others = []
    res = run_config(args, args.config, headline=True)
    for name in others:
        sub = run_config(args, name, headline=False)
        res[name] = {k: sub[k] for k in ("value", "unit", "ms_per_step", "whole_path_mfma_frac", "output_gemms_mfma_frac",
                                         "gemm_ms", "roofline", "loss_first_last", "config")}
    print(json.dumps(res), flush=True)
    return 0


def run_config(args, config_name, headline):
    """Times args.steps training windows of one configuration (after args.warmup untimed ones) and returns
    the result object; headline = False skips the CPU baseline and the peak measurement."""
    import numpy as np
    import torch
    from paper_1502_00512_amd import binding, synth

    comp = args.arch == "compressed"
    cfg = synth.CONFIGS[config_name]
    V, H, B, T = cfg.V, cfg.H, (args.streams or cfg.B), cfg.T
    P = synth.COMPRESSED_P if comp else 0
    M = B * T
    precision = binding.RNNLM_BF16_FP32MASTER if cfg.precision == "bf16" else binding.RNNLM_FP32
    total_steps = args.steps + args.warmup
    # tokens: the data-offset scheme spreads the B read cursors over the whole corpus
    need = total_steps * T
    L_full = (cfg.N - 1) // B
    N = cfg.N if need <= L_full else need * B + 1
    t0 = time.time()
    tok = synth.make_tokens(cfg, N)
    if comp:
        E, A_, U, C_, b = synth.make_compressed_weights(V, H, P, cfg.init, cfg.init_scale, cfg.weight_seed)
        Wo = None
    else:
        E, U, Wo, b = synth.make_weights(V, H, cfg.init, cfg.init_scale, cfg.weight_seed)
    log(f"[bench] {cfg.name}: V={V} H={H} B={B} T={T} N={N} inputs generated in {time.time() - t0:.1f}s "
        f"tokens sha256 {synth.sha256_of(tok)[:16]}")

    nce = args.criterion == "nce"
    score = args.criterion == "score"
    rms = args.optimizer == "rmsprop"
    if comp:
        g = binding.Rnnlm(E, U, None, b, B, T, precision, A=A_, C_=C_)
    else:
        g = binding.Rnnlm(E, U, Wo, b, B, T, precision, K_max=args.noise if nce else 0, rmsprop=rms, r_init=1e-4)
    rms_lr, rms_rho, rms_eps = cfg.lr * 1e-2, 0.9995, 1e-4
    dtok = torch.as_tensor(tok).cuda()
    if nce:
        # noise distribution = smoothed unigram of the corpus; the draws of every window, generated up front
        lnq, thr = synth.unigram_noise(tok, V)
        dlnq = torch.as_tensor(lnq).cuda()
        dnoise = torch.as_tensor(np.stack([synth.noise_words(thr, args.noise, cfg.data_seed + 7, k)
                                           for k in range(total_steps)])).cuda()
        lnZ = float(np.log(V))  # scores start near 0: a constant normaliser of ln V makes them near-normalised
    x = torch.empty(T, B, dtype=torch.int32, device="cuda")
    y = torch.empty(T, B, dtype=torch.int32, device="cuda")
    sum_logp = torch.zeros(1, dtype=torch.float64, device="cuda")
    scores = torch.empty(T, B, dtype=torch.float32, device="cuda")
    if args.shortlist:
        # candidates: seeded uniform ids (which words are on the list does not change the work)
        cand = torch.as_tensor(np.random.default_rng(cfg.data_seed).integers(0, V, (T, B, args.shortlist)).astype(np.int32)).cuda()
        scores = torch.empty(T, B, args.shortlist, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step(k):
        g.rnnlm_stream_chunk(dtok, k, T, x, y, stream)
        if nce and rms:
            g.rnnlm_nce_train_chunk_rmsprop(x, y, dnoise[k % total_steps], dlnq, lnZ, rms_lr, rms_rho, rms_eps, None,
                                            sum_logp, stream)
        elif nce:
            g.rnnlm_nce_train_chunk(x, y, dnoise[k % total_steps], dlnq, lnZ, cfg.lr, None, sum_logp, stream)
        elif score and args.shortlist:
            g.rnnlm_forward_score_shortlist(x, cand, float(np.log(V)), scores, stream)
        elif score:
            g.rnnlm_forward_score(x, y, float(np.log(V)), scores, stream)
        elif rms:
            g.rnnlm_train_chunk_rmsprop(x, y, rms_lr, rms_rho, rms_eps, None, sum_logp, stream)
        else:
            g.rnnlm_train_chunk(x, y, cfg.lr, None, sum_logp, stream)

    stage_ids = {n: i for i, n in enumerate(binding.STAGES)}
    gemm_stages = ["rnn_fwd", "rnn_bwd", "nce_update"] if nce else ["out_fwd", "out_bwd_h", "out_bwd_w"]
    if score:
        gemm_stages = ["prep", "rnn_fwd", "nce_score"]
    if rms and not nce:
        gemm_stages = ["out_fwd", "out_bwd_h", "out_bwd_w", "rmsprop"]
    if comp and not score:
        gemm_stages = ["rnn_fwd", "rnn_bwd", "out_fwd", "out_bwd_h", "out_bwd_w", "proj"]

    # The contraction stages are bracketed by HIP events.  An event costs the stream several microseconds (3 % of
    # cfg3's window for six of them), so inside the timed region only the dominant stage is bracketed: the one the
    # roofline object reports, found during warm-up.  The other stages are timed in a short pass after the region.
    mask = sum(1 << stage_ids[n] for n in gemm_stages)

    def read_stages(names, nsteps):
        out = {}
        for n in names:
            ms, cnt = g.rnnlm_profile_read(stage_ids[n])
            out[n] = ms / max(cnt, 1) if n != "proj" else ms / nsteps   # proj: six launches per step, summed
        return out

    g.rnnlm_profile_enable(mask if args.warmup else 0)
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    timed_stages = list(gemm_stages)
    if args.warmup:
        warm = read_stages(gemm_stages, args.warmup)
        timed_stages = ["rnn_fwd"] if score else [max((n for n in gemm_stages if n not in ("proj", "rmsprop")), key=warm.get)]
    sign = 1.0 if nce else -1.0  # noise-contrastive calls return the loss itself, the others log-probabilities
    first_loss = sign * sum_logp.item() / M if args.warmup else float("nan")

    # timed region: K steps
    g.rnnlm_profile_enable(sum(1 << stage_ids[n] for n in timed_stages))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.warmup, total_steps):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    g.rnnlm_check()
    last_loss = sign * sum_logp.item() / M
    gemm_ms = read_stages(timed_stages, args.steps)
    rest = [n for n in gemm_stages if n not in timed_stages]
    if rest:
        g.rnnlm_profile_enable(mask)
        nrest = min(args.steps, 20)
        for k in range(nrest):
            step(k)
        torch.cuda.synchronize()
        later = read_stages(gemm_stages, nrest)
        gemm_ms.update({n: later[n] for n in rest})
        gemm_ms = {n: gemm_ms[n] for n in gemm_stages}
    g.rnnlm_profile_enable(0)

    stage_ms = None
    if args.stages:
        g.rnnlm_profile_enable((1 << len(binding.STAGES)) - 1)
        nst = min(args.steps, 50)
        for k in range(nst):
            step(k)
        torch.cuda.synchronize()
        stage_ms = {}
        for n, i in stage_ids.items():
            ms, cnt = g.rnnlm_profile_read(i)
            stage_ms[n] = round(ms / nst, 4)
        g.rnnlm_profile_enable(0)
        log("[bench] per-stage ms per step:", json.dumps(stage_ms))

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # what the box sustains (for context next to the published peaks)
    measured = g.rnnlm_measure_peaks(stream) if headline else None

    words_per_s = args.steps * M / dt
    peak = PEAK_BF16_TFLOPS if cfg.precision == "bf16" else PEAK_FP32_TFLOPS
    live = timed_stages[0] if len(timed_stages) == 1 else None  # the stage bracketed inside the timed region
    dominant = live or max(gemm_ms, key=gemm_ms.get)
    extra = {"timed_live": live or "all stages"}
    if score:
        flops_word = 2.0 * H * (H + 1)
        achieved = 2.0 * H * H * M / (gemm_ms["rnn_fwd"] * 1e-3) / 1e12
        dominant = "rnn_fwd"
        roofline = {"bound": "mfma", "kernel": "rnn_fwd", "achieved": round(achieved, 2), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None}
        extra["stage_ms_timed"] = {k: round(v, 4) for k, v in gemm_ms.items()}
        criterion = "forward-only unnormalised scoring of the given next words"
        metric = "scored words/sec (forward only, unnormalised output) at 1 MI355X"
        if args.shortlist:
            criterion = f"forward-only unnormalised scoring of a shortlist of {args.shortlist} candidate words per position"
            metric = "positions/sec (forward only, shortlist of candidates scored per position) at 1 MI355X"
        if comp:
            criterion = f"compressed architecture (P={P}), " + criterion
    elif comp and not score:
        flops_word = 6.0 * (V * P + 2.0 * P * H + H * H)
        # algorithmic flops per launch: recurrent kernels 2 H^2 per position, output contractions 2 V P per position
        work = {"rnn_fwd": 2.0 * H * H * M, "rnn_bwd": 2.0 * H * H * (M - B), "out_fwd": 2.0 * V * P * M,
                "out_bwd_h": 2.0 * V * P * M, "out_bwd_w": 2.0 * V * P * M}
        proj_ms = gemm_ms.pop("proj")
        dominant = live or max(gemm_ms, key=gemm_ms.get)
        achieved = work[dominant] / (gemm_ms[dominant] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None}
        extra["stage_ms_timed"] = {k: round(v, 4) for k, v in gemm_ms.items()}
        extra["stage_ms_timed"]["proj (six contractions through the inserted layers)"] = round(proj_ms, 4)
        extra["P"] = P
        criterion = f"compressed architecture (layers of {P} units below and above the state, tied word matrix), full softmax"
        metric = "training words/sec (fwd+BPTT+SGD, compressed architecture) at 1 MI355X"
    elif nce:
        Kn = args.noise
        flops_word = 6.0 * H * (Kn + 1 + H)  # K+1 scored words per position instead of V
        # algorithmic work per launch of the three longest stages: the recurrent kernels are contractions
        # (2 H^2 per position and direction), the row update moves the touched rows (4 B per element read from
        # the gradient panel or hidden states, 10 B per element for the fp32 master read-modify-write and the
        # bf16 copy, one row per list entry)
        work = {"rnn_fwd": ("mfma", 2.0 * H * H * M), "rnn_bwd": ("mfma", 2.0 * H * H * (M - B)),
                "nce_update": ("hbm", (Kn + M) * H * 14.0)}
        bound, amount = work[dominant]
        if bound == "mfma":
            achieved = amount / (gemm_ms[dominant] * 1e-3) / 1e12
            roofline = {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": peak,
                        "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None}
        else:
            achieved = amount / (gemm_ms[dominant] * 1e-3) / 1e9
            roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                        "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None}
        extra["stage_ms_timed"] = {k: round(v, 4) for k, v in gemm_ms.items()}
        extra["noise_words"] = Kn
        criterion = f"noise-contrastive output ({Kn} shared noise words per window, lnZ = ln V)"
        metric = "training words/sec (fwd+BPTT+SGD, noise-contrastive criterion) at 1 MI355X"
        if rms:
            criterion += ", rmsprop (0.9995, one statistic per word for E and Wo)"
            metric = "training words/sec (fwd+BPTT+rmsprop-scaled SGD, noise-contrastive criterion) at 1 MI355X"
    else:
        flops_word = 6.0 * H * (V + H)
        gemm_flops = 2.0 * H * V * M  # algorithmic flops of each output-layer contraction per window
        rms_ms = gemm_ms.pop("rmsprop", None)
        dominant = live or max(gemm_ms, key=gemm_ms.get)
        achieved = gemm_flops / (gemm_ms[dominant] * 1e-3) / 1e12
        out_gemm_frac = 3 * gemm_flops / (sum(gemm_ms.values()) * 1e-3) / 1e12 / peak
        if rms_ms is not None:
            # the apply pass reads the gradient (4 B) and read-modify-writes the fp32 master (8 B) + bf16 copy (2 B)
            extra["rmsprop_apply"] = {"ms": round(rms_ms, 4), "algorithmic_GBps":
                                      round(14.0 * (V * H + H * H) / (rms_ms * 1e-3) / 1e9, 1), "peak_GBps": PEAK_HBM_GBS}
        roofline = {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                    "traffic": measured_traffic(cfg.name, dominant)}
        extra["output_gemms_mfma_frac"] = round(out_gemm_frac, 4)
        extra["gemm_ms"] = {k: round(v, 4) for k, v in gemm_ms.items()}
        criterion = "full softmax"
        metric = "training words/sec (fwd+BPTT+SGD) at 1 MI355X"
        if rms:
            criterion = "full softmax, rmsprop (0.9995, one statistic per word for E and Wo)"
            metric = "training words/sec (fwd+BPTT+rmsprop-scaled SGD) at 1 MI355X"

    cpu = None
    if not headline:
        pass
    elif comp and not score and not args.no_cpu_baseline:
        cpu = cpu_baseline_compressed(cfg, E, A_, U, C_, b, tok)
    elif not args.no_cpu_baseline and not score and not rms:
        cpu = cpu_baseline(cfg, E, U, Wo, b, tok,
                           (synth.noise_words(thr, args.noise, cfg.data_seed + 7, 0), lnq, lnZ) if nce else None)

    res = {
        "metric": metric,
        "value": round(words_per_s, 1),
        "unit": "words/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(dt / args.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.precision if cfg.precision == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: Elman RNNLM V={V} H={H}, {B} streams x BPTT {T}, Zipf({cfg.zipf_s}) tokens, "
                               f"{criterion}" + ("" if score else f" + SGD lr={rms_lr if rms else cfg.lr}"), "V": V, "H": H, "B": B, "T": T, "tokens": int(N)},
        "whole_path_mfma_frac": round(words_per_s * flops_word / (peak * 1e12), 4),
        "loss_first_last": [round(first_loss, 4), round(last_loss, 4)],
        "roofline": roofline,
        "cpu_baseline": cpu,
        "measured_peaks": {k: round(v, 1) for k, v in measured.items()} if measured else None,
    }
    res.update(extra)
    if stage_ms is not None:
        res["stage_ms"] = stage_ms
    g.close()
    del g, dtok
    torch.cuda.empty_cache()
    return res


def measured_traffic(workload, kernel):
    """HBM bytes per launch of the kernel, from the committed counter summary (profiles/hbm_traffic.json:
    rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a device copy of known size); None if not measured."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            return json.load(f)[workload][kernel]["bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline_compressed(cfg, E, A, U, C, b, tok):
    """The numpy fp64 oracle of the compressed architecture on whole training windows (about 10 s)."""
    import numpy as np
    from oracle import compressed as Cq
    from oracle import oracle as O
    B, T = cfg.B, cfg.T
    x, y = O.stream_chunk(tok, B, T, 0)
    m = Cq.CompressedModel(*(np.asarray(a, np.float64).copy() for a in (E, A, U, C, b)), np.zeros((B, cfg.H)))
    total, reps = 0.0, 0
    while total < 10.0 and reps < 64:
        t0 = time.perf_counter()
        Cq.train_chunk(m, x.astype(np.int64), y.astype(np.int64), cfg.lr)
        total += time.perf_counter() - t0
        reps += 1
    return {"value": round(reps * B * T / total, 2), "unit": "words/s", "cores": os.cpu_count(), "kind": "oracle",
            "sample": f"{reps} x one training window of {B} streams x {T} timesteps ({reps * B * T} words, {total:.1f} s; "
                      "numpy fp64, its library's threads)"}


def cpu_baseline(cfg, E, U, Wo, b, tok, nce=None):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: the first window cut
    to as many leading timesteps as fit about 10-30 s of CPU work.  nce = (noise, lnq, lnZ) times the
    noise-contrastive step instead of the normalised one."""
    import numpy as np
    from oracle import oracle as O
    V, H, B, T = cfg.V, cfg.H, cfg.B, cfg.T
    x, y = O.stream_chunk(tok, B, T, 0)

    def timed(Ts):
        m = O.Model.from_weights(E, U, Wo, b, B)
        xs, ys = np.ascontiguousarray(x[:Ts]), np.ascontiguousarray(y[:Ts])
        t0 = time.perf_counter()
        if nce is None:
            O.train_chunk(m, xs, ys, cfg.lr)
        else:
            O.nce_train_chunk(m, xs, ys, nce[0], nce[1].astype(np.float64), nce[2], cfg.lr)
        return time.perf_counter() - t0

    Ts, dt = 1, timed(1)          # calibration: one timestep of the window
    if dt < 5.0 and T > 1:        # then as many timesteps as fit about 15 s
        Ts = int(max(2, min(T, 15.0 // dt)))
        dt = timed(Ts)
    words, total, reps = B * Ts, dt, 1
    while Ts == T and total < 10.0 and reps < 8:   # a whole window is short: repeat it up to about 10 s
        total += timed(Ts)
        words += B * Ts
        reps += 1
    return {"value": round(words / total, 2), "unit": "words/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"{reps} x one training window of {B} streams x {Ts} of {T} timesteps ({words} words, {total:.1f} s)"}


if __name__ == "__main__":
    sys.exit(main())
