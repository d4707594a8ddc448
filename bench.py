#!/usr/bin/env python3
"""Throughput of one decoder-layer training step (forward + backward) on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 8b|1b|small|tiny]

A step is dlayer_forward + dlayer_backward over one batch of seeded synthetic bf16 inputs that are
resident in HBM before the timed region starts.  Prints ONE JSON line: whole-step TFLOP/s
(algorithmic FLOPs: 3 x forward, causal attention counted as half of the dense S^2 products, no
credit for recomputation), tokens/s, the roofline figure of the dominant kernel (the bf16 MFMA GEMM,
timed per launch with events on the launch stream) and the fp64 oracle timed on the host cores on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published: 2.5 PFLOP/s)

# HBM bytes per launch of the dominant kernel (mean over the replayed launches of the seven projection
# shapes of the 8B-shaped layer), from rocprofv3 FETCH_SIZE / WRITE_SIZE runs scaled by a plain 1 GiB copy in the same
# run (factors 2.0 and 1.0; profiles/layer_8b_hbm_traffic.txt).  Only valid for the GEMM source the
# counters were taken on: reported as null when gemm.hip has changed since.
GEMM_TRAFFIC = {"config": "8b", "gemm_hip_sha256": "f94e8db7edcbef10e1afe77c4e421204cea0725d8f7e95c0786bbaca67d9b716",
                "fetch_bytes": 1.496e+09, "write_bytes": 2.013e+08}


def _gemm_traffic(config_name):
    import hashlib
    src = os.path.join(ROOT, "paper_2602_08387_amd", "csrc", "gemm.hip")
    try:
        same = hashlib.sha256(open(src, "rb").read()).hexdigest() == GEMM_TRAFFIC["gemm_hip_sha256"]
    except OSError:
        same = False
    if not same or config_name != GEMM_TRAFFIC["config"]:
        return None
    return GEMM_TRAFFIC["fetch_bytes"] + GEMM_TRAFFIC["write_bytes"]


def _describe(cfg):
    return (f"decoder layer B{cfg.batch} S{cfg.seq} D{cfg.d_model} {cfg.n_q_heads}q/{cfg.n_kv_heads}kv x"
            f"{cfg.head_dim} F{cfg.d_ff} rope_base {cfg.rope_base:g}, fwd+bwd")


def cpu_baseline(cfg, budget_tokens, whole=False):
    """The fp64 oracle, as it stands, on a bounded sample: the same layer (same weights and widths)
    on one batch row cut to `budget_tokens` positions; whole=True: on the whole workload."""
    import numpy as np
    from oracle import decoder_layer as odl
    from synth import inputs as si
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    sub = cfg if whole else cfg.with_(batch=1, seq=min(cfg.seq, budget_tokens))
    inp = si.to_f64(si.make_layer_inputs(sub, seed=0))
    x, dy = inp.pop("x"), inp.pop("dy")
    t0 = time.perf_counter()
    f = odl.layer_forward(sub, x, inp)
    odl.layer_backward(sub, x, inp, dy, f)
    dt = time.perf_counter() - t0
    flops = si.layer_fwd_bwd_flops(sub)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "seconds": dt, "tokens_per_s": sub.tokens / dt,
            "sample": ("the whole workload" if whole else f"same layer and weights, 1 batch row cut to {sub.seq} positions") +
                      f" ({sub.tokens} of {cfg.tokens} tokens), fp64 NumPy, fwd+bwd"}


def bench_stack(args, torch, K, si, dev_bf16):
    """The stack workload (not the headline line): embedding -> 4 8B-shaped layers at B1 S8192 -> final
    RMSNorm -> LM head (V = 128256) -> mean cross-entropy, and back to the embedding gradients; one step =
    the whole forward and backward.  Pointer plumbing only; every arithmetic step is a library call."""
    cfg, L, V = si.CONFIGS["8b_stack_layer"], 4, 128256
    T, D = cfg.tokens, cfg.d_model
    raw = si.make_stack_inputs(cfg, L, V, seed=0)
    ids = torch.from_numpy(raw["ids"].reshape(-1)).cuda()
    tgt = torch.from_numpy(raw["targets"].reshape(-1)).cuda()
    E, w_lm, g_f = dev_bf16(raw["embed"]), dev_bf16(raw["w_lm"]), dev_bf16(raw["g_final"])
    W = [{n: dev_bf16(w[n]) for n in si.WEIGHT_NAMES} for w in raw["layers"]]
    del raw
    bf = lambda *s: torch.empty(*s, dtype=torch.bfloat16, device="cuda")
    u8 = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device="cuda")
    xs = [bf(T, D) for _ in range(L + 1)]
    saved = [u8(K.dlayer_saved_bytes(cfg)) for _ in range(L)]
    ws = u8(K.dlayer_workspace_bytes(cfg))
    h_f, rstd_f = bf(T, D), torch.empty(T, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    dh_f, dw_lm, dg_f, dE = bf(T, D), bf(V, D), bf(D), bf(V, D)
    dxa, dxb = bf(T, D), bf(T, D)
    dW = [{n: torch.empty_like(t) for n, t in W[l].items()} for l in range(L)]
    ws_head = u8(K.lm_head_ce_workspace_bytes(T, D, V, 0))
    ws_norm = u8(K.rmsnorm_backward_workspace_bytes(T, D))
    ws_emb = u8(K.embed_backward_workspace_bytes(T, V))

    def step():
        K.embed_forward(E, ids, T, V, D, xs[0])
        for l in range(L):
            K.dlayer_forward(cfg, xs[l], W[l], xs[l + 1], saved[l], ws)
        K.rmsnorm_forward(xs[L], g_f, T, D, cfg.rms_eps, h_f, rstd_f)
        K.lm_head_ce_fwd_bwd(h_f, w_lm, tgt, T, D, V, 1.0, 0, loss, dh_f, dw_lm, 0, ws_head)
        K.rmsnorm_backward(xs[L], g_f, rstd_f, dh_f, None, T, D, dxa, dg_f, 0, ws_norm)
        a, b = dxa, dxb
        for l in reversed(range(L)):
            K.dlayer_backward(cfg, xs[l], W[l], a, saved[l], b, dW[l], 0, ws)
            a, b = b, a
        K.embed_backward(a, ids, T, V, D, dE, ws_emb)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    flops = L * si.layer_fwd_bwd_flops(cfg) + 6.0 * T * D * V
    print(json.dumps({
        "metric": "4-layer stack fwd+bwd TFLOP/s (embedding, 4 layers, final norm, LM head, cross-entropy)",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"stack: B1 S8192, {L} x (D4096 32q/8kv x128 F14336), V {V}", "name": "stack",
                   "tokens_per_step": T, "flops_per_step": flops},
        "tokens_per_s": T / (ms * 1e-3), "frac_of_bf16_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "loss": float(loss.item())}))


def time_components(torch, K, si, cfg, x, w, reps):
    """The pieces of one step, each launched on its own through the building-block entry point that
    dlayer_forward / dlayer_backward use for it (same kernels, same shapes), one event pair per launch
    on the launch stream.  Returns a list of rows: name, kernel, ms, algorithmic TFLOP (or GB for the
    HBM-bound ones), achieved rate and its fraction of the bf16 MFMA peak (or of 8 TB/s)."""
    B, S, T, D, F = cfg.batch, cfg.seq, cfg.tokens, cfg.d_model, cfg.d_ff
    Hq, Hkv, dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    QD, KD = Hq * dh, Hkv * dh
    bf = lambda *shape: torch.empty(*shape, dtype=torch.bfloat16, device="cuda").normal_()
    u8 = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device="cuda")
    h, q, k, v, o = bf(T, D), bf(T, QD), bf(T, KD), bf(T, KD), bf(T, QD)
    g, u, a, y = bf(T, F), bf(T, F), bf(T, F), bf(T, D)
    dq, dk, dv, dg, du = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v), torch.empty_like(g), torch.empty_like(u)
    dx = torch.empty_like(h)
    lse = torch.empty(B, Hq, S, dtype=torch.float32, device="cuda")
    rstd = torch.empty(T, dtype=torch.float32, device="cuda")
    dgam = torch.empty(D, dtype=torch.bfloat16, device="cuda")
    dws = {n: torch.empty_like(t) for n, t in w.items() if t.dim() == 2}
    ws_rope, ws_attn = u8(K.qkv_rope_workspace_bytes(S, dh)), u8(K.attention_backward_workspace_bytes(B, S, Hq, Hkv, dh))
    ws_sw, ws_norm = u8(K.linear_swiglu_backward_workspace_bytes(T, D, F)), u8(K.rmsnorm_backward_workspace_bytes(T, D))
    ws_lin = u8(K.linear_backward_workspace_bytes(T, F, D))
    attn = 2.0 * B * Hq * float(S) ** 2 * dh
    wg = [("w_down", x, a, D, F), ("w_gate", dg, h, F, D), ("w_up", du, h, F, D), ("wo", x, o, D, QD),
          ("wq", dq, h, QD, D), ("wk", dk, h, KD, D), ("wv", dv, h, KD, D)]
    K.attention_forward(q, k, v, B, S, Hq, Hkv, dh, o, lse)     # a valid lse for the backward launches
    rows = [
        ("q, k, v projections + RoPE", "gemm_group_rope_kernel", 2.0 * T * D * (QD + 2 * KD),
         lambda: K.qkv_rope_forward(h, w["wq"], w["wk"], w["wv"], B, S, D, Hq, Hkv, dh, cfg.rope_base, cfg.rope_layout, q, k, v, ws_rope)),
        ("attention forward", "attn_fwd_kernel", attn, lambda: K.attention_forward(q, k, v, B, S, Hq, Hkv, dh, o, lse)),
        ("o projection + residual", "gemm_kernel<k,k>", 2.0 * T * QD * D, lambda: K.linear_forward(o, w["wo"], x, T, QD, D, y)),
        ("gate/up projections + SwiGLU", "gemm_swiglu_kernel<1>", 4.0 * T * D * F,
         lambda: K.linear_swiglu_forward(h, w["w_gate"], w["w_up"], T, D, F, g, u, a)),
        ("down projection + residual", "gemm_kernel<k,k>", 2.0 * T * F * D, lambda: K.linear_forward(a, w["w_down"], x, T, F, D, y)),
        ("down input gradient + SwiGLU gradient (+ W_down transpose)", "gemm_swiglu_kernel<2>", 2.0 * T * D * F,
         lambda: K.linear_swiglu_backward(x, w["w_down"], g, u, T, D, F, dg, du, ws_sw)),
        ("gate input gradient (+ W_gate transpose)", "gemm_kernel<k,k>", 2.0 * T * D * F,
         lambda: K.linear_backward(h, w["w_gate"], dg, T, D, F, dx, None, 0, ws_lin)),
        ("o input gradient (+ W_o transpose)", "gemm_kernel<k,k>", 2.0 * T * QD * D,
         lambda: K.linear_backward(o, w["wo"], x, T, QD, D, dq, None, 0, ws_lin)),
        ("attention backward (delta, dK+dV, dQ)", "attn_delta + attn_bwd_dkdv (stores dS) + attn_bwd_dq_from_ds", 2.0 * attn,
         lambda: K.attention_backward(q, k, v, o, dq, lse, B, S, Hq, Hkv, dh, dq, dk, dv, ws_attn)),
        ("seven weight gradients, one launch", "gemm_group_kernel<mn,mn>", sum(2.0 * T * N * Kd for _, _, _, N, Kd in wg),
         lambda: K.linear_wgrad_group([d for _, d, _, _, _ in wg], [xx for _, _, xx, _, _ in wg], [N for *_, N, _ in wg],
                                      [Kd for *_, Kd in wg], T, [dws[n] for n, *_ in wg], 0)),
    ]
    hbm = [
        ("RMSNorm forward", "rmsnorm_fwd_kernel", 4.0 * T * D, lambda: K.rmsnorm_forward(x, w["g_attn"], T, D, cfg.rms_eps, h, rstd)),
        ("RMSNorm backward + residual gradient", "rmsnorm_bwd_kernel", 10.0 * T * D,
         lambda: K.rmsnorm_backward(x, w["g_attn"], rstd, h, y, T, D, dx, dgam, 0, ws_norm)),
    ]
    K.rmsnorm_forward(x, w["g_attn"], T, D, cfg.rms_eps, h, rstd)
    out = []
    for kind, table in (("mfma", rows), ("hbm", hbm)):
        for name, kernel, work, fn in table:
            fn()
            evs = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(); fn(); e1.record()
                evs.append((e0, e1))
            torch.cuda.synchronize()
            ms = sum(p.elapsed_time(q_) for p, q_ in evs) / reps
            if kind == "mfma":
                rate = work / (ms * 1e-3) / 1e12
                out.append({"name": name, "kernel": kernel, "bound": "mfma", "ms": ms, "tflop": work / 1e12, "tflops": rate,
                            "frac": rate / PEAK_BF16_TFLOPS})
            else:
                rate = work / (ms * 1e-3) / 1e9
                out.append({"name": name, "kernel": kernel, "bound": "hbm", "ms": ms, "gb": work / 1e9, "gbps": rate, "frac": rate / 8000.0})
    return out


def bench_optimizer(args, torch, K, si):
    """The optimizer step of one 8B-shaped layer (not the headline line): global-norm clipping and AdamW
    over the layer's nine parameter tensors (218 M bf16 parameters, fp32 moments).  Both kernels are
    bound by HBM: 2 bytes per element for the norm, 22 for the update."""
    cfg = si.CONFIGS["8b"]
    shapes = si.weight_shapes(cfg)
    P = [torch.empty(shapes[n], dtype=torch.bfloat16, device="cuda").normal_(0, 0.02) for n in si.WEIGHT_NAMES]
    G = [torch.empty_like(p).normal_(0, 1e-3) for p in P]
    M = [torch.zeros(p.shape, dtype=torch.float32, device="cuda") for p in P]
    V = [torch.zeros(p.shape, dtype=torch.float32, device="cuda") for p in P]
    sq = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(K.grad_sq_norm_workspace_bytes(G), 256), dtype=torch.uint8, device="cuda")
    n = sum(p.numel() for p in P)
    state = {"t": 0}

    def step():
        state["t"] += 1
        K.grad_sq_norm(G, sq, 0, ws)
        K.adamw_step(P, G, M, V, state["t"], 3e-4, 0.9, 0.95, 1e-8, 0.1, 1.0, sq)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    nbytes = 24.0 * n
    print(json.dumps({
        "metric": "optimizer step (global-norm clip + AdamW) GB/s of algorithmic HBM bytes", "value": nbytes / (ms * 1e-3) / 1e9,
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"clip + AdamW over the 9 parameter tensors of one 8B-shaped layer ({n} parameters)", "name": "optimizer",
                   "bytes_per_step": nbytes},
        "roofline": {"bound": "hbm", "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                     "frac": nbytes / (ms * 1e-3) / 1e9 / 8000.0, "traffic": None}}))


def bench_tokenize(args):
    """The data pipeline's tokenization stage (host only, no GPU): indexation + producer-consumer
    tokenization of a synthetic JSONL corpus into a token file.  A step is one pass over the corpus."""
    import tempfile
    from synth import text as st
    from paper_2602_08387_amd import tokpipe as tp
    workers = args.tok_workers or min(16, os.cpu_count() or 1)
    merges = st.train_merges(0, 2000, 4000)
    eod = 256 + len(merges)
    with tempfile.TemporaryDirectory(prefix="tokbench_") as tmp:
        src, idx, out = (os.path.join(tmp, n) for n in ("corpus.jsonl", "corpus.idx", "corpus.tok"))
        with open(src, "wb") as f:           # distinct documents, made in parts to bound memory
            part, size = 0, 0
            while size < args.tok_megabytes * 1e6:
                chunk = st.make_jsonl(1000 + part, 1500, n_words=20000)
                f.write(chunk if chunk.endswith(b"\n") else chunk + b"\n")
                size += len(chunk) + 1
                part += 1
        t_index = []
        runs = []
        for it in range(args.warmup + args.steps):
            t0 = time.perf_counter()
            n_docs = tp.index_jsonl(src, idx, workers)
            t1 = time.perf_counter()
            stats = tp.tokenize(src, idx, out, merges, "text", eod, workers, args.tok_batch, 4 * workers)
            t2 = time.perf_counter()
            if it >= args.warmup:
                t_index.append(t1 - t0)
                runs.append((t2 - t0, stats.n_tokens, stats.bytes_read, stats.cache_hits, stats.cache_misses))
        sec = sum(r[0] for r in runs) / len(runs)
        tokens, nbytes = runs[-1][1], runs[-1][2]
        rec = {"metric": "tokenization throughput, indexation included", "value": tokens / sec, "unit": "tokens/s", "n_gpus": 1,
               "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak",
               "vs_baseline": None, "dtype": "u8", "data": "synthetic",
               "config": {"workload": f"JSONL -> token file: {n_docs} synthetic documents, {nbytes / 1e6:.0f} MB, byte-level BPE with "
                                      f"{len(merges)} merges; 1 reader, {workers} tokenizer workers, 1 writer, batches of {args.tok_batch} documents",
                          "name": "tokenize", "tokens": int(tokens), "documents": int(n_docs), "index_ms": 1e3 * sum(t_index) / len(t_index),
                          "megabytes_per_s": nbytes / sec / 1e6, "piece_cache_hit_rate": runs[-1][3] / max(1, runs[-1][3] + runs[-1][4])},
               "roofline": None, "note": "host-only workload: no GPU kernel runs, so no GPU roofline applies"}
        if not args.no_cpu_baseline:
            from oracle import tokenize as ot
            sample = open(src, "rb").read(int(args.tok_oracle_megabytes * 1e6))
            sample = sample[:sample.rfind(b"\n") + 1]
            t0 = time.perf_counter()
            docs = ot.tokenize_jsonl(sample, merges, "text", eod)
            dt = time.perf_counter() - t0
            rec["cpu_baseline"] = {"value": sum(map(len, docs)) / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle", "seconds": dt,
                                   "sample": f"the first {len(sample) / 1e6:.1f} MB of the same corpus ({len(docs)} documents), sequential Python"}
    print(json.dumps(rec))


PROBES = (
    # family, variant, label; one block = 16 MFMAs 32x32x16 (family 0) or 8 MFMAs 16x16x32 (family 1)
    (0, 0, "32x32x16 MFMAs alone"),
    (0, 1, "softmax-like VALU work alone (16 exp + 64 fma per block)"),
    (0, 2, "both, evenly interleaved (MFMA, 1 exp, 4 fma) x 16"),
    (0, 3, "both, two regions: (MFMA, 1 fma) x 8 then (MFMA, 2 exp, 7 fma) x 8"),
    (1, 0, "16x16x32 MFMAs, operands in registers"),
    (1, 1, "  with 2 ds_read_b128 per 8 MFMAs (128x128 wave tile)"),
    (1, 2, "  with 3 ds_read_b128 per 8 MFMAs (128x64 wave tile)"),
    (1, 3, "  with 3 pairs of ds_read_b64_tr_b16 per 8 MFMAs (128x64, transposed operands)"),
    # about a second of back-to-back launches each, pseudo-random operands: the rate at the clock the power limit allows
    (3, 0, "sustained, random operands: 16x16x32 MFMAs, operands in registers"),
    (3, 1, "sustained, random operands:   with 2 ds_read_b128 per 8 MFMAs"),
    (3, 2, "sustained, random operands:   with 3 ds_read_b128 per 8 MFMAs"),
    (3, 3, "sustained, random operands: 32x32x16 MFMAs, operands in registers"),
)


def run_probes(K):
    """Synthetic issue-rate measurements (C-ABI issue_rate_probe); flop rates count the MFMAs only."""
    rows = []
    for fam, var, label in PROBES:
        for wps in (1, 2):
            cyc, ms, ghz, _ = K.issue_rate_probe(fam, var, wps)
            big = fam == 0 or (fam, var) == (3, 3)     # blocks of 16 MFMAs 32x32x16, else 2 x 8 MFMAs 16x16x32 per iteration
            mfmas = 0 if (fam, var) == (0, 1) else 256 * 4 * wps * 2000 * (16 if big else 8 * 2)
            flop = mfmas * (32768.0 if big else 16384.0)
            rows.append({"probe": label, "waves_per_simd": wps, "cycles_per_block_per_simd": round(cyc, 1),
                         "ms": round(ms, 3), "shader_ghz": round(ghz, 2), "mfma_tflops": round(flop / ms / 1e9, 0)})
    for var, label in ((0, "MFMA waves alone"), (1, "VALU waves alone"), (2, "MFMA waves and VALU waves side by side")):
        cyc, ms, ghz, other = K.issue_rate_probe(2, var, 2)
        rows.append({"probe": "neighbouring waves: " + label, "cycles_per_mfma": round(cyc, 1), "cycles_per_fma": round(other, 2),
                     "ms": round(ms, 3), "shader_ghz": round(ghz, 2)})
    print(json.dumps({"probes": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="8b", choices=["tiny", "small", "1b", "8b", "70b_width", "stack", "optimizer", "tokenize"])
    ap.add_argument("--tok-megabytes", type=float, default=120.0, help="--config tokenize: size of the synthetic corpus")
    ap.add_argument("--tok-workers", type=int, default=0, help="--config tokenize: tokenizer threads (default: host cores, at most 16)")
    ap.add_argument("--tok-batch", type=int, default=64, help="--config tokenize: documents per queue entry")
    ap.add_argument("--tok-oracle-megabytes", type=float, default=6.0, help="--config tokenize: corpus prefix the oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=4096)
    ap.add_argument("--cpu-full", action="store_true",
                    help="also run the oracle once over the whole workload (about two minutes of host time at the 8B shape)")
    ap.add_argument("--no-components", action="store_true", help="skip the per-piece timing table")
    ap.add_argument("--recompute", type=int, default=0,
                    help="dlayer_cfg.recompute bits (1: rebuild h1, h2 in the backward; 2: rebuild the SwiGLU output); 0 is the timed default")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (the known-size dispatch that HBM byte "
                         "counters of a profiler run are scaled by)")
    ap.add_argument("--probes", action="store_true",
                    help="instead of the step: run the library's synthetic issue-rate probes (matrix pipe next to "
                         "VALU work, LDS operand feed, neighbouring waves) and print their table as one JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU decoder-layer step; this library has no multi-GPU path "
              "(no collectives, no sharding): run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.config == "tokenize":
        return bench_tokenize(args)

    import torch
    import paper_2602_08387_amd as K   # raises if the HIP library is not built: no fallback
    from synth import inputs as si
    from synth.device import dev_bf16

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.probes:
        return run_probes(K)
    if args.config == "stack":
        return bench_stack(args, torch, K, si, dev_bf16)
    if args.config == "optimizer":
        return bench_optimizer(args, torch, K, si)
    cfg = si.CONFIGS[args.config].with_(recompute=args.recompute)
    inp = si.make_layer_inputs(cfg, seed=0)
    x, dy = dev_bf16(inp["x"]), dev_bf16(inp["dy"])
    w = {n: dev_bf16(inp[n]) for n in si.WEIGHT_NAMES}
    del inp
    dw = {n: torch.empty_like(t) for n, t in w.items()}
    y, dx = torch.empty_like(x), torch.empty_like(x)
    saved = torch.empty(K.dlayer_saved_bytes(cfg), dtype=torch.uint8, device="cuda")
    ws = torch.empty(K.dlayer_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")

    def step():
        K.dlayer_forward(cfg, x, w, y, saved, ws)
        K.dlayer_backward(cfg, x, w, dy, saved, dx, dw, 0, ws)

    for _ in range(args.warmup):
        step()
    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)           # reads 1 GiB, writes 1 GiB
        del src, dst
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms = e0.elapsed_time(e1) / args.steps
    ms = max(ms, wall_ms) if abs(ms - wall_ms) > 0.2 * wall_ms else ms
    flops = si.layer_fwd_bwd_flops(cfg)
    tflops = flops / (ms * 1e-3) / 1e12

    # Forward and backward separately (informational).
    def timed(fn, n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n
    n_sub = max(3, args.steps // 2)
    # per-step spread (informational): one event pair per step
    evs = []
    for _ in range(max(5, args.steps)):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        step()
        b.record()
        evs.append((a, b))
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in evs)
    step_median_ms, step_min_ms = per_step[len(per_step) // 2], per_step[0]
    fwd_ms = timed(lambda: K.dlayer_forward(cfg, x, w, y, saved, ws), n_sub)
    bwd_ms = timed(lambda: K.dlayer_backward(cfg, x, w, dy, saved, dx, dw, 0, ws), n_sub)

    # Dominant kernel: the k-major x k-major bf16 MFMA GEMM.  The q, k, v, o and down projections and
    # every input-gradient product of the step run on it, the gate/up pair and the down-projection
    # input gradient on variants of it with the SwiGLU in the epilogue.  Launch it at the layer's
    # seven projection shapes, one event pair per launch on the launch stream, and compare algorithmic
    # FLOPs with the summed durations.
    T, D, F = cfg.tokens, cfg.d_model, cfg.d_ff
    QD, KD = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    acts = {D: x.view(T, D), QD: torch.empty(T, QD, dtype=torch.bfloat16, device="cuda").normal_(),
            F: torch.empty(T, F, dtype=torch.bfloat16, device="cuda").normal_()}
    launches = [("wq", D, QD), ("wk", D, KD), ("wv", D, KD), ("wo", QD, D), ("w_gate", D, F), ("w_up", D, F),
                ("w_down", F, D)]
    outs = {n: torch.empty(T, N, dtype=torch.bfloat16, device="cuda") for n, _, N in launches}
    reps = max(3, min(10, args.steps))
    dur_ms, gemm_flops = [], 0.0
    for r in range(reps + 1):
        for n, Kd, N in launches:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            K.linear_forward(acts[Kd], w[n], None, T, Kd, N, outs[n])
            b.record()
            if r > 0:
                dur_ms.append((a, b))
                gemm_flops += 2.0 * T * Kd * N
    torch.cuda.synchronize()
    total_ms = sum(a.elapsed_time(b) for a, b in dur_ms)
    achieved = gemm_flops / (total_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "gemm_kernel<256,256,2,4,k-major,k-major> (the layer's 7 projection shapes)",
                "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                "avg_launch_ms": total_ms / len(dur_ms), "launches_timed": len(dur_ms),
                "traffic": _gemm_traffic(args.config), "traffic_unit": "HBM bytes per launch (fetched + written)",
                "algorithmic_bytes_per_launch": sum(2.0 * (T * Kd + N * Kd + T * N * (2 if n in ("wo", "w_down") else 1))
                                                    for n, Kd, N in launches) / len(launches)}

    out = {
        "metric": "decoder-layer fwd+bwd TFLOP/s", "value": tflops, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": _describe(cfg), "name": args.config, "tokens_per_step": cfg.tokens,
                   "flops_per_step": flops, "recompute": cfg.recompute, "saved_bytes": K.dlayer_saved_bytes(cfg)},
        "tokens_per_s": cfg.tokens / (ms * 1e-3), "frac_of_bf16_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "peak_tflops": PEAK_BF16_TFLOPS, "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
        "ms_per_step_median": step_median_ms, "ms_per_step_min": step_min_ms,
        "paper_throughput": "not reported in the paper's text (Fig. 2b is an image; 8B Llama-3, Leonardo)",
        "roofline": roofline,
    }
    if not args.no_components:
        # every piece of the step on its own: which kernel is dominant in the step, which one is furthest
        # from its roofline
        comps = time_components(torch, K, si, cfg, x.view(T, D), w, max(3, min(10, args.steps)))
        mf = [c for c in comps if c["bound"] == "mfma"]
        roofline["in_step"] = comps
        roofline["in_step_sum_ms"] = sum(c["ms"] for c in comps)
        roofline["in_step_dominant"] = max(mf, key=lambda c: c["ms"])["name"]
        roofline["in_step_worst"] = min(mf, key=lambda c: c["frac"])["name"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_tokens)
        if args.cpu_full:
            out["cpu_baseline_full"] = cpu_baseline(cfg, cfg.seq, whole=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
