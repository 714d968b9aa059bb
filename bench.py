#!/usr/bin/env python3
"""Benchmark of the KV-Prediction time-to-first-token path on one MI355X.

A step is one pass of the whole path (auxiliary prefill -> predictor -> one base step ->
greedy first token) over one batch of synthetic prompts, inputs resident in HBM.
Prints ONE JSON line: TTFT (ms_per_step: each step is one call, timed from before the call
to its first tokens on the host), prompt tokens/s (value), the roofline of the dominant kernel
class, all per-class rooflines, the chip's achievable peaks measured by plain probe kernels,
and the CPU oracle timed beside it.  Without --config the workload is the largest benchmark
configuration (config 4: 8B-class base, batch 4, 8192-token prompts).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu-baseline]

    python bench.py --peaks                   # only the achievable-peak probes

    python bench.py --sweep --config 2        # the three systems over prompt lengths at batch 8

    python bench.py --reference base|aux [--config C] ...
times, on the same kernels, ordinary inference of the base model (or of the auxiliary model
alone) to its first token: the two reference points of the paper's timing experiments
(Sec. 6.3 "Timing Experiments").  That line is context for the headline number, not the headline metric.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
PEAK_FP32_VECTOR_TFLOPS = 157.3


def workload_name(cfg, B, T):
    """The configuration's name, or that name with the overridden batch / prompt length spelled out."""
    if (B, T) == (cfg.batch, cfg.seq_len):
        return cfg.name
    return f"{cfg.name}_shapes_at_b{B}_t{T}"


def layerwise_variant(cfg):
    """The configuration with OpenELM-style layer-wise scaling (the models of the paper's experiments,
    Sec. 4.2 "Architectural Details") and query / key normalisation: key/value heads grow linearly
    from half the configuration's count to its full count (4 query heads each), feed-forward widths
    from half to one and a half times the configuration's width (same mean), both stacks."""
    import kvp_synth as S

    def widths(m):
        out = []
        for l in range(m.n_layers):
            t = l / max(1, m.n_layers - 1)
            nkv = max(1, round(m.n_kv_heads * (0.5 + 0.5 * t)))
            f = int(round(m.ffn_dim * (0.5 + t) / 64.0)) * 64
            out.append((nkv * (m.n_q_heads // m.n_kv_heads), nkv, f))
        return out

    return cfg.with_(name=cfg.name + "_layerwise_qknorm", qk_norm=True,
                     base=S.with_layer_widths(cfg.base, widths(cfg.base)), aux=S.with_layer_widths(cfg.aux, widths(cfg.aux)))


def algorithmic_work(cfg, B, T):
    """Algorithmic FLOPs and bytes per step for every kernel class (what the path must do,
    not what a particular kernel happens to move)."""
    a, b = cfg.aux, cfg.base
    es = 4 if cfg.dtype == "fp32" else 2
    N = B * T
    hd_a, hd_b = a.head_dim, b.head_dim
    # per layer (the widths are the same for every layer unless the stack has layer-wise widths)
    aux_gemm_flops = aux_attn_flops = 0
    for l in range(a.n_layers):
        nq, nkv, f = a.widths(l)
        if l == a.n_layers - 1:                          # last auxiliary layer: K and V projections only
            aux_gemm_flops += N * 2 * (a.d_model * 2 * nkv * hd_a)
        else:
            aux_gemm_flops += N * 2 * (a.d_model * (nq + 2 * nkv) * hd_a + nq * hd_a * a.d_model + 3 * a.d_model * f)
            aux_attn_flops += 2 * nq * hd_a * T * (T + 1) * B
    pred_flops = pred_bytes = gemv_w = dec_bytes = dec_flops = 0
    for i in range(b.n_layers):
        nq, nkv, f = b.widths(i)
        Ka, Kb = a.widths(cfg.layer_map[i])[1] * hd_a, nkv * hd_b
        pred_flops += 4 * Ka * Kb * N
        pred_bytes += 2 * Kb * es * N + 2 * Ka * Kb * es
        gemv_w += 2 * b.d_model * nq * hd_b + 3 * b.d_model * f + 2 * b.d_model
        dec_bytes += 2 * B * T * Kb * es
        dec_flops += 4 * nq * hd_b * T * B
    pred_bytes += sum(2 * a.widths(l)[1] * hd_a * es * N for l in range(a.n_layers))   # auxiliary cache read once
    gemv_bytes = es * (gemv_w + cfg.vocab * b.d_model + b.d_model)
    gemv_flops = 2 * B * (gemv_w + cfg.vocab * b.d_model)
    norm_bytes = (a.n_layers * 2 - 1) * N * a.d_model * (4 + es)
    return {
        "aux_gemm": {"bound": "mfma" if cfg.dtype == "bf16" else "alu", "flops": aux_gemm_flops},
        "aux_attn": {"bound": "mfma" if cfg.dtype == "bf16" else "alu", "flops": aux_attn_flops},
        "predictor": {"bound": "hbm", "flops": pred_flops, "bytes": pred_bytes},
        "base_gemv": {"bound": "hbm", "flops": gemv_flops, "bytes": gemv_bytes},
        "decode_attn": {"bound": "hbm", "flops": dec_flops, "bytes": dec_bytes},
        "embed_norm": {"bound": "hbm", "bytes": norm_bytes},
        "argmax": {"bound": "hbm", "bytes": B * cfg.vocab * 4},
    }


def roofline_entry(work, ms, launches, dtype):
    if not launches or ms <= 0:
        return None
    sec = ms / 1e3
    if work["bound"] == "hbm":
        ach = work["bytes"] / sec / 1e9
        e = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}
    else:
        peak = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_FP32_VECTOR_TFLOPS
        ach = work["flops"] / sec / 1e12
        e = {"bound": work["bound"], "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak}
    if "flops" in work and work["bound"] == "hbm":
        e["tflops"] = work["flops"] / sec / 1e12
    e["ms_per_step"] = ms
    e["launches_per_step"] = launches
    e["traffic"] = None
    return e


def kernel_sources_sha256():
    """Fingerprint of the kernel sources (every file under csrc/, in name order): measured traffic
    figures are only quoted while the kernels they were measured on are the ones that run."""
    d = os.path.join(ROOT, "paper_2410_08391_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()


def load_traffic(workload):
    """Measured HBM traffic per kernel class in bytes per step for `workload` (two rocprofv3 --pmc
    runs, FETCH_SIZE and WRITE_SIZE, each scaled by what the counter reads for a 256 MiB device
    copy; summarised under profiles/).  Each entry of profiles/traffic.json carries the fingerprint
    of the kernel sources it was measured on; an entry measured on other sources is stale and is
    not quoted.  Returns (bytes per class, note)."""
    p = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(p):
        return {}, "no profiles/traffic.json"
    with open(p) as f:
        data = json.load(f)
    if workload not in data:
        return {}, "not measured for this workload"
    stamp = data.get(workload + "__sources_sha256")
    if stamp != kernel_sources_sha256():
        return {}, "stale: measured on other kernel sources (sha256 %s...)" % (stamp or "unstamped")[:12]
    return data[workload], "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, see profiles/"


def cpu_baseline(cfg, store, tokens):
    """The CPU oracle as it stands, on a bounded sample of the same workload: ONE WHOLE sequence
    of the batch (sequences are independent, so a whole sequence is exact for what it covers;
    a prefix would flatter the oracle on long prompts, attention being quadratic)."""
    from oracle import kvp_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    B, T = tokens.shape
    sample = tokens[:1]
    t0 = time.time()
    O.kvp_prefill_predict(cfg, store.f64, sample)
    dt = time.time() - t0
    return {"value": T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 whole sequence of {T} tokens out of the workload's {B} x {T}, whole path incl. base step, {dt:.1f} s",
            "seconds": dt}


def achievable_peaks(K, torch, nbytes=1 << 30, reps=5):
    """What the chip sustains on the two roofs, from the library's probe kernels (kernels_probe.hip):
    a register-resident bf16 MFMA loop, a streaming read, a copy and a fill over 1 GiB, each the best
    of `reps` launches timed with HIP events on the launch stream."""
    stream = torch.cuda.current_stream()
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    a.random_(0, 256)
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")

    def best(fn):
        t = []
        for _ in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            torch.cuda.synchronize()
            t.append(e0.elapsed_time(e1))
        return min(t[1:])

    flops = [0.0]
    def mfma():
        flops[0] = K.kvp_probe_mfma(sink, 20000, stream.cuda_stream)
    ms = best(mfma)
    out = {"mfma_bf16_tflops": flops[0] / (ms / 1e3) / 1e12, "mfma_probe_ms": ms}
    out["read_gbs"] = nbytes / (best(lambda: K.kvp_probe_stream(0, a, b, nbytes, stream.cuda_stream)) / 1e3) / 1e9
    out["copy_gbs"] = 2 * nbytes / (best(lambda: K.kvp_probe_stream(1, a, b, nbytes, stream.cuda_stream)) / 1e3) / 1e9
    out["fill_gbs"] = nbytes / (best(lambda: K.kvp_probe_stream(2, a, b, nbytes, stream.cuda_stream)) / 1e3) / 1e9
    out["note"] = ("probe kernels of the library: register-resident v_mfma_f32_32x32x16_bf16 loop (no memory traffic); "
                   "streaming read / copy (read + written bytes) / fill over 1 GiB")
    return out


def reference_main(args):
    """TTFT of ordinary inference of one model alone (kvp_reference_prefill)."""
    import torch
    import kvp_synth as S
    import paper_2410_08391_amd as K

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    side = args.reference
    cfg = S.CONFIGS[args.config]
    B, T = args.batch or cfg.batch, args.prompt_tokens or cfg.seq_len
    m_shape = cfg.base if side == "base" else cfg.aux
    model = K.MODEL_BASE if side == "base" else K.MODEL_AUX
    store = S.WeightStore(cfg, device="cuda" if cfg.gen_device == "cuda" else "cpu")
    names = sorted(set(S.hot_path_tensor_names(cfg)) | set(S.reference_tensor_names(cfg, side)))
    store.prefetch(names)
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    tokens = S.draw_tokens(cfg, batch=B, seq_len=T)
    tok = torch.from_numpy(tokens).to("cuda")
    m = K.KVP(cfg, dev, max_batch=B, max_seq=T)
    dt = torch.float32 if cfg.dtype == "fp32" else torch.bfloat16
    kc = torch.zeros((m_shape.n_layers, B, m_shape.n_kv_heads, T, m_shape.head_dim), dtype=dt, device="cuda")
    vc = torch.zeros_like(kc)
    ws = torch.empty(K.kvp_reference_workspace_bytes(m.handle, model, B, T) + 256, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def step():   # the model's own cache is written in cache layout, as ordinary inference must
        K.kvp_reference_prefill(m.handle, model, tok, B, T, kc, vc, T, m.logits, m.argmax, ws, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    first = m.argmax[:B].cpu().tolist()
    m.profile(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = m.profile_read()
    m.profile(False)
    N = B * T
    a = m_shape
    gemm_flops = N * a.n_layers * 2 * (a.d_model * (a.q_dim + 2 * a.kv_dim) + a.q_dim * a.d_model + 3 * a.d_model * a.ffn_dim)
    attn_flops = 2 * a.n_q_heads * a.head_dim * T * (T + 1) * B * a.n_layers
    bound = "mfma" if cfg.dtype == "bf16" else "alu"
    roofs = {}
    for cls, wk in (("aux_gemm", {"bound": bound, "flops": gemm_flops}), ("aux_attn", {"bound": bound, "flops": attn_flops})):
        e = roofline_entry(wk, prof[cls]["ms"] / args.steps, prof[cls]["launches"] / args.steps, cfg.dtype)
        if e:
            roofs["prefill_gemm" if cls == "aux_gemm" else "prefill_attn"] = e
    dominant = max(roofs, key=lambda c: roofs[c]["ms_per_step"])
    roof = dict(roofs[dominant]); roof["kernel_class"] = dominant
    print(json.dumps({
        "metric": f"prompt_tokens_per_s (reference: ordinary inference of the {side} model alone, prefill + first token)",
        "value": B * T / (ms / 1e3), "unit": "tokens/s", "ttft_ms": ms,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload_name(cfg, B, T), "reference": side, "batch": B, "prompt_tokens": T, "layers": a.n_layers,
                   "d_model": a.d_model, "first_tokens": first[:8]},
        "roofline": roof, "rooflines": roofs,
        "class_ms": {c: prof[c]["ms"] / args.steps for c in prof if prof[c]["launches"]},
    }))


def sweep_main(args):
    """Times to first token over prompt lengths at the configuration's batch size, for the three
    systems of the paper's timing experiments (Sec. 6.3 "Timing Experiments": base model alone,
    KV Prediction, auxiliary model alone), all on this library's kernels.  One JSON line."""
    import torch
    import kvp_synth as S
    import paper_2410_08391_amd as K

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cfg = S.CONFIGS[args.config]
    B, Tmax = cfg.batch, cfg.seq_len
    store = S.WeightStore(cfg, device="cuda" if cfg.gen_device == "cuda" else "cpu")
    names = sorted(set(S.hot_path_tensor_names(cfg)) | set(S.reference_tensor_names(cfg, "base"))
                   | set(S.reference_tensor_names(cfg, "aux")))
    store.prefetch(names)
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    tok_all = torch.from_numpy(S.draw_tokens(cfg)).to("cuda")
    m = K.KVP(cfg, dev)
    dt = torch.float32 if cfg.dtype == "fp32" else torch.bfloat16
    stream = torch.cuda.current_stream().cuda_stream
    ref = {}
    for side, model, shape in (("base", K.MODEL_BASE, cfg.base), ("aux", K.MODEL_AUX, cfg.aux)):
        kc = torch.zeros((shape.n_layers, B, shape.n_kv_heads, Tmax, shape.head_dim), dtype=dt, device="cuda")
        ws = torch.empty(K.kvp_reference_workspace_bytes(m.handle, model, B, Tmax) + 256, dtype=torch.uint8, device="cuda")
        ref[side] = (model, kc, torch.zeros_like(kc), ws)

    def timed(fn, steps):
        for _ in range(max(1, args.warmup)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    rows = []
    T = 64
    lengths = []
    while T < Tmax:
        lengths.append(T)
        T *= 2
    lengths.append(Tmax)
    for T in lengths:
        tok = tok_all[:, :T].contiguous()
        steps = max(3, min(args.steps, int(args.steps * 1024 / (B * T)) + 3))
        row = {"prompt_tokens": T, "steps": steps}
        row["kv_prediction_ms"] = timed(lambda: m.run(tok), steps)
        for side in ("base", "aux"):
            model, kc, vc, ws = ref[side]
            row[side + "_alone_ms"] = timed(
                lambda: K.kvp_reference_prefill(m.handle, model, tok, B, T, kc, vc, Tmax, m.logits, m.argmax, ws, stream),
                max(3, steps // 2))
        row["speedup_over_base"] = row["base_alone_ms"] / row["kv_prediction_ms"]
        row["overhead_over_aux"] = row["kv_prediction_ms"] / row["aux_alone_ms"] - 1.0
        rows.append(row)
        print(f"# T={T}: base {row['base_alone_ms']:.3f} ms, KV Prediction {row['kv_prediction_ms']:.3f} ms, "
              f"aux {row['aux_alone_ms']:.3f} ms", file=sys.stderr, flush=True)
    print(json.dumps({
        "metric": "ttft_ms over prompt length (base alone / KV Prediction / auxiliary alone)",
        "unit": "ms", "n_gpus": 1, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + "_length_sweep", "batch": B, "lengths": lengths},
        "sweep": rows,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4,
                    help="benchmark configuration 0..4 (default 4: the largest, 8B-class base, batch 4, 8192-token prompts)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--peaks", action="store_true", help="run only the achievable-peak probes and print them as one JSON line")
    ap.add_argument("--no-peaks", action="store_true", help="skip the achievable-peak probes")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also run one plain 256 MiB device copy, so a rocprofv3 --pmc run of this command "
                         "holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--generate", type=int, default=0, metavar="N",
                    help="after the timed region also time N passes of the generation loop that follows the first "
                         "token (base model alone, own keys / values appended) and report the TTFT / step ratio")
    ap.add_argument("--reference", choices=["base", "aux"], default=None,
                    help="time ordinary inference of that model alone instead of the KV Prediction path")
    ap.add_argument("--batch", type=int, default=0, help="override the configuration's batch size (context runs; "
                    "the workload name in the JSON line then carries the override)")
    ap.add_argument("--prompt-tokens", type=int, default=0, help="override the configuration's prompt length")
    ap.add_argument("--layerwise", action="store_true",
                    help="context run: the configuration with OpenELM-style per-layer widths and query / key norm")
    ap.add_argument("--absorbed", action="store_true",
                    help="context run: also time the path with the predictor absorbed into the base step's attention "
                         "(first token from the auxiliary cache; predicted cache written beside the last base layers)")
    ap.add_argument("--sweep", action="store_true",
                    help="time the three systems (base alone, KV Prediction, auxiliary alone) over prompt lengths "
                         "64 .. the configuration's length at its batch size (use with --config 2: batch 8)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (sequences are independent, so more GPUs would "
                 "each run this same path on their share of the batch); use --gpus 1")

    if args.sweep:
        return sweep_main(args)
    if args.reference:
        return reference_main(args)

    import numpy as np
    import torch
    import kvp_synth as S
    import paper_2410_08391_amd as K

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.peaks:
        print(json.dumps({"metric": "achievable peaks (probe kernels)", "n_gpus": 1, "data": "synthetic",
                          "published": {"mfma_bf16_tflops": PEAK_BF16_TFLOPS, "hbm_gbs": PEAK_HBM_GBS},
                          "achievable": achievable_peaks(K, torch)}))
        return
    cfg = S.CONFIGS[args.config]
    if args.layerwise:
        cfg = layerwise_variant(cfg)
    B, T = args.batch or cfg.batch, args.prompt_tokens or cfg.seq_len
    store = S.WeightStore(cfg, device="cuda" if cfg.gen_device == "cuda" else "cpu")
    names = S.hot_path_tensor_names(cfg)
    if args.generate > 0:      # the generation loop needs the base model's own key / value projections
        names = sorted(set(names) | set(S.reference_tensor_names(cfg, "base")))
    store.prefetch(names)
    dev = {n: store.get(n).to("cuda").contiguous() for n in names}
    tokens = S.draw_tokens(cfg, batch=B, seq_len=T)
    tok = torch.from_numpy(tokens).to("cuda")
    m = K.KVP(cfg, dev, max_batch=B, max_seq=T + args.generate, T_cap=T + args.generate)

    for _ in range(args.warmup):
        m.run(tok)
    torch.cuda.synchronize()
    # The timed region: K steps, each ONE call as a caller sees it -- from just before the call to after
    # the stream has drained and the first tokens are on the host.  ms_per_step is the mean over the K
    # steps (the region is bracketed by synchronisation on both sides), ttft_ms their median.
    lat = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        t1 = time.perf_counter()
        m.run(tok)
        first = m.argmax[:B].cpu().tolist()          # blocks until the call's work is done
        lat.append((time.perf_counter() - t1) * 1e3)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    lat.sort()
    pct = lambda q: lat[min(len(lat) - 1, int(q * len(lat)))]
    ttft = pct(0.50)

    # For comparison: the same K calls queued back to back (the host's launch work of call i+1 hides
    # behind the device work of call i); not what a single caller sees, so not the headline.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        m.run(tok)
    torch.cuda.synchronize()
    ms_pipelined = (time.perf_counter() - t0) * 1e3 / args.steps

    # Device time per stage: one HIP event between the stages, on the stream the kernels run on
    # (three events per step perturb nothing measurable).
    stream = torch.cuda.current_stream()
    stage_ms = {"aux": 0.0, "predict": 0.0, "base": 0.0}
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for k in range(args.steps):
        evs[k][0].record(stream)
        m.run(tok, K.STAGE_AUX); evs[k][1].record(stream)
        m.run(tok, K.STAGE_PREDICT); evs[k][2].record(stream)
        m.run(tok, K.STAGE_BASE); evs[k][3].record(stream)
    torch.cuda.synchronize()
    for k in range(args.steps):
        for i, name in enumerate(("aux", "predict", "base")):
            stage_ms[name] += evs[k][i].elapsed_time(evs[k][i + 1]) / args.steps
    # Split of each stage over its kernel classes: a further pass with one HIP event after every
    # launch (kvp_profile_*).  An event between two microsecond-scale kernels costs about as much
    # as the kernels themselves, so only the *shares* within a stage are taken from this pass and
    # applied to the stage times measured above.
    m.profile(True)
    for _ in range(args.steps):
        m.run(tok)
    torch.cuda.synchronize()
    prof = m.profile_read()
    m.profile(False)
    stage_of = {"embed_norm": "aux", "aux_gemm": "aux", "aux_attn": "aux", "predictor": "predict",
                "base_gemv": "base", "decode_attn": "base", "argmax": "base"}
    chain_sum = {st: sum(prof[c]["ms"] for c in stage_of if stage_of[c] == st) for st in stage_ms}
    class_ms = {c: (stage_ms[stage_of[c]] * prof[c]["ms"] / chain_sum[stage_of[c]] if chain_sum[stage_of[c]] > 0 else 0.0)
                for c in stage_of}

    work = algorithmic_work(cfg, B, T)
    traffic, traffic_note = load_traffic(workload_name(cfg, B, T))
    roofs = {}
    for cls, wk in work.items():
        e = roofline_entry(wk, class_ms[cls], prof[cls]["launches"] / args.steps, cfg.dtype)
        if e:
            # per launch, like `achieved`
            e["traffic"] = traffic[cls] / e["launches_per_step"] if cls in traffic else None
            roofs[cls] = e
    dominant = max(roofs, key=lambda c: roofs[c]["ms_per_step"])
    roof = dict(roofs[dominant])
    roof["kernel_class"] = dominant
    # per-launch figures for the dominant class
    roof["avg_launch_us"] = roof["ms_per_step"] / roof["launches_per_step"] * 1e3

    out = {
        "metric": "prompt_tokens_per_s (TTFT path: aux prefill + KV predictor + 1 base step)",
        "value": B * T / (ms / 1e3),
        "unit": "tokens/s",
        "ttft_ms": ttft,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload_name(cfg, B, T), "batch": B, "prompt_tokens": T, "vocab": cfg.vocab,
                   "path": "mfma" if cfg.dtype == "bf16" else "fp32", "first_tokens": first[:8]},
        "roofline": roof,
        "rooflines": roofs,
        "ttft_single_call_ms": {"p10": pct(0.10), "p50": pct(0.50), "p90": pct(0.90), "mean": ms,
                                "note": "the timed steps: one call at a time, host wall time from before the call to first tokens on the host"},
        "pipelined_ms_per_step": ms_pipelined,
        "ttft_note": "ms_per_step / value: mean of the K timed steps, each a single call of the whole path as the library "
                     "schedules it (auxiliary chain and predictor + base chain overlapped on two streams) up to its first "
                     "tokens on the host; ttft_ms: their median; pipelined_ms_per_step: K calls queued back to back; "
                     "stage_ms: the stages run one after another",
        "traffic_note": traffic_note,
        "stage_ms": stage_ms,
        "event_chain_ms_sum": sum(prof[c]["ms"] for c in prof) / args.steps,
    }
    if args.absorbed:
        # The same step with the predictor absorbed into the attention (linear maps, Sec. 4.2): logits from the
        # auxiliary cache.  Three timings, each over args.steps calls between two events.
        def timed(stages):
            for _ in range(2):
                m.run(tok, stages)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(args.steps):
                m.run(tok, stages)
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps
        ab = K.STAGE_BASE_ABSORBED
        ref_logits = m.logits[:B].clone()
        t_first = timed(K.STAGE_AUX | ab)
        t_all = timed(K.STAGE_AUX | K.STAGE_PREDICT | ab)
        m.run(tok, K.STAGE_AUX)
        t_base = timed(ab)
        t_base_plain = timed(K.STAGE_BASE)
        m.run(tok, K.STAGE_AUX | ab)
        torch.cuda.synchronize()
        dl = (m.logits[:B] - ref_logits).abs().max().item() / ref_logits.abs().max().item()
        out["absorbed"] = {"first_token_ms": t_first, "first_token_and_cache_ms": t_all, "base_step_absorbed_ms": t_base,
                           "base_step_over_cache_ms": t_base_plain, "ttft_ms_default_path": ms,
                           "first_tokens_agree": m.argmax[:B].cpu().tolist() == first,
                           "logits_vs_default_path_rel": dl,
                           "note": "first_token_ms: auxiliary prefill + absorbed base step, no predicted cache; "
                                   "first_token_and_cache_ms: the same call also writes the predicted cache for the "
                                   "generation loop, on the caller's stream beside the last base layers"}
    if args.generate > 0:
        # Algorithm "KV Prediction Inference", the loop after the first token: feed the previous greedy
        # choice, append the base model's own key / value, attend over T + s entries.
        fed = m.argmax[:B].clone()
        m.generation_step(fed, T)            # warm-up of the generation kernels (slot T is rewritten below)
        torch.cuda.synchronize()
        fed.copy_(torch.tensor(first, dtype=torch.int32))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for sidx in range(args.generate):
            m.generation_step(fed, T + sidx)
            fed.copy_(m.argmax[:B])
        e1.record(stream)
        torch.cuda.synchronize()
        gen_ms = e0.elapsed_time(e1) / args.generate
        out["generation"] = {"steps": args.generate, "ms_per_step": gen_ms, "ttft_over_generation_step": ms / gen_ms,
                             "tokens_per_s": B / (gen_ms / 1e3),
                             "note": "base model alone, one token per sequence per step, cache of T + s entries"}
    if args.pmc_calibrate:
        src = torch.zeros(256 * 1024 * 1024 // 2, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["pmc_calibration"] = {"kernel": "torch device copy", "bytes_read": 256 * 1024 * 1024, "bytes_written": 256 * 1024 * 1024}
    if not args.no_peaks:
        del m
        torch.cuda.empty_cache()
        out["achievable"] = achievable_peaks(K, torch)
        ach = out["achievable"]
        for e in list(roofs.values()) + [roof]:       # every fraction also against the measured peak
            e["frac_of_achievable"] = e["achieved"] / (ach["read_gbs"] if e["bound"] == "hbm" else ach["mfma_bf16_tflops"]) \
                if cfg.dtype == "bf16" or e["bound"] == "hbm" else None
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, store, tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
