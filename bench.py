#!/usr/bin/env python3
"""Benchmark of the verification hot path on one MI355X.

One "step" = one vl_verify_prefill call over the whole synthetic batch: teacher-forced causal prefill of
every sequence, comparison of the recomputed hidden states at the committed layers, LM head + argmax +
token check, flags and summary.  Inputs (weights, tokens, commitments) are resident in HBM before the
timed region starts.  Prints ONE JSON line on stdout; progress goes to stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1] [--no-cpu-baseline] [--no-decode]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def attention_flops(model, lengths):
    """Causal attention at its triangular cost: QK^T and PV, 2 flops per multiply-add."""
    tri = sum(t * (t + 1) / 2 for t in lengths)
    return 4.0 * model.n_q_heads * model.head_dim * tri * model.n_layers


# Bytes moved between L2 and the memory side by ONE launch of the gate/up GEMM at the default workload, from two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE; KiB per dispatch), each scaled by what the same counter reads for a plain
# 1 GiB -> 1 GiB elementwise kernel (0.500 and 1.000 on MI355X); the commands and raw figures are in profiles/.  The
# figure belongs to one version of the kernel source: any edit of that file makes it unknown again.
GATEUP_TRAFFIC = {
    "source": "paper_2509_24257_amd/csrc/kernels_gemm_mfma.hip",
    "sha256": "c6c7b874d529d72db5c027c2a6b5b7933eaa85b94f15b464a8383235da091dc3",
    "workload": "cfg1-8b-b8x1024",
    "bytes_per_launch": (1376925 / 0.500 + 229376 / 1.000) * 1024,
}


def measured_traffic(wl):
    import hashlib
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), GATEUP_TRAFFIC["source"])
    try:
        with open(path, "rb") as f:
            same = hashlib.sha256(f.read()).hexdigest() == GATEUP_TRAFFIC["sha256"]
    except OSError:
        same = False
    if not same or wl.name != GATEUP_TRAFFIC["workload"]:
        return None
    return round(GATEUP_TRAFFIC["bytes_per_launch"])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=1, help="index into the five evaluation workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="commitments from vl_prefill_commit instead of vl_decode_commit")
    ap.add_argument("--cpu-sample-tokens", type=int, default=64)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, a reference of known size for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2509_24257_amd as P
    import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    wl = synth.workload(args.workload)
    m = wl.model
    n, c = wl.n_tokens, len(wl.commit_layers)
    bf = wl.hidden_dtype == "bf16"
    log(f"[bench] workload {wl.name}: N={n} tokens, B={len(wl.lengths)}, commit layers {wl.commit_layers}")

    cfg = P.ModelCfg(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab, m.rms_eps,
                     m.rope_base, P.VL_BF16 if m.dtype == "bf16" else P.VL_F32, n, len(wl.lengths), max(wl.lengths))
    t0 = time.time()
    ctx = P.Context(cfg, 0, 0)
    keep_host = (not args.no_cpu_baseline) and m.n_params() * 2 < 40e9      # keep the drawn weights for the oracle leg
    host_w = {}
    for kind in synth.GLOBAL_KINDS:
        w = np.ascontiguousarray(synth.weight(m, kind, 0, 16))
        ctx.vl_load_weights(kind, 0, w.ctypes.data, w.nbytes)
        if keep_host:
            host_w[(kind, 0)] = w
    for l in range(m.n_layers):
        for kind in synth.PER_LAYER_KINDS:
            w = np.ascontiguousarray(synth.weight(m, kind, l, 16))
            ctx.vl_load_weights(kind, l, w.ctypes.data, w.nbytes)
            if keep_host:
                host_w[(kind, l)] = w
        if l % 8 == 7:
            log(f"[bench] weights: layer {l + 1}/{m.n_layers} loaded ({time.time() - t0:.0f} s)")
    log(f"[bench] {m.n_params() / 1e9:.2f} B parameters drawn and uploaded in {time.time() - t0:.1f} s")

    x = synth.tokens(wl)
    d_tok = torch.from_numpy(x).to(dev)
    hd_code = P.VL_BF16 if bf else P.VL_F32
    d_com = torch.zeros((max(c, 1), n, m.d_model), dtype=torch.int16 if bf else torch.float32, device=dev)
    d_cam = torch.zeros(n, dtype=torch.int32, device=dev)

    # ---- commitments of an honest inferencer (also the decode side of the verify/decode cost ratio)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if args.no_decode:
        ctx.vl_prefill_commit(d_tok.data_ptr(), wl.lengths, wl.commit_layers, d_com.data_ptr(), hd_code, d_cam.data_ptr())
    else:
        ctx.vl_decode_commit(d_tok.data_ptr(), wl.lengths, wl.prompt_lens, wl.commit_layers, d_com.data_ptr(), hd_code,
                             d_cam.data_ptr())
    torch.cuda.synchronize()
    t_commit = time.perf_counter() - t0
    log(f"[bench] commitments by {'prefill' if args.no_decode else 'prefill(prompt)+token-by-token decode'}: {t_commit:.2f} s")

    # ---- the commitment step that follows in the protocol: Merkle roots over the committed states (not part of `value`)
    merkle = None
    if c:
        d_roots = torch.zeros((c * n, 32), dtype=torch.uint8, device=dev)
        ctx.vl_op_merkle_roots(d_com.data_ptr(), hd_code, c * n, d_roots.data_ptr())          # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.vl_op_merkle_roots(d_com.data_ptr(), hd_code, c * n, d_roots.data_ptr())
        torch.cuda.synchronize()
        t_mk = time.perf_counter() - t0
        merkle = {"roots": c * n, "scalars_per_root": m.d_model, "ms": round(t_mk * 1e3, 3),
                  "ns_per_scalar": round(t_mk / (c * n * m.d_model) * 1e9, 4)}
        log(f"[bench] Merkle roots of the {c} x {n} committed states: {t_mk * 1e3:.1f} ms")

    # ---- tamper (host side, from the seeded generator), back to HBM
    pos = synth.tamper_positions(wl)
    if bf:
        com_host = synth.bf16_bits_to_f32(d_com.cpu().numpy().view(np.uint16))
    else:
        com_host = d_com.cpu().numpy()
    com_t = synth.tamper_hidden(wl, com_host[:c], pos) if c else com_host[:0]
    cam_host = d_cam.cpu().numpy()
    cam_t, _ = synth.tamper_argmax(wl, cam_host, pos)
    if c:
        st = synth.f32_to_bf16_bits(com_t).view(np.int16) if bf else com_t
        d_com[:c].copy_(torch.from_numpy(st).to(dev))
    d_cam.copy_(torch.from_numpy(cam_t).to(dev))
    d_flags = torch.zeros(n, dtype=torch.uint8, device=dev)
    tol = P.Tol(wl.tol_rel_l2, wl.tol_max_abs, wl.tol_logit_margin)
    cam_ptr = d_cam.data_ptr() if wl.check_argmax else 0

    def step():
        return ctx.vl_verify_prefill(d_tok.data_ptr(), wl.lengths, wl.commit_layers, d_com.data_ptr(), hd_code, cam_ptr, tol,
                                     d_flags.data_ptr())

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                      # the runtime's device-to-device copy: reads 1 GiB, writes 1 GiB
        torch.mul(src, 1.0, out=dst)        # a plain elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        sm = step()
    expect = np.ones(n, np.uint8)
    expect[pos] = 0
    flags_ok = bool((d_flags.cpu().numpy() == expect).all())
    log(f"[bench] warm-up done; flags equal the planted tamper mask: {flags_ok}; rejected {sm.n_rejected}/{n}")

    # ---- timed region: exactly K steps, event pairs around the dominant kernel (gate/up GEMM) on the library's stream
    ctx.vl_profile_enable(1)
    ctx.vl_profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    dev_ms = 0.0
    for _ in range(args.steps):
        sm = step()
        dev_ms += sm.ms_forward
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ctx.vl_profile_read()
    gu_ms, gu_launches = prof["gateup_gemm"]
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = n * args.steps / elapsed

    # ---- one extra untimed step with every stage bracketed, for the breakdown
    ctx.vl_profile_enable(2)
    step()
    stages = {k: round(v[0], 3) for k, v in ctx.vl_profile_read().items() if v[1] > 0}
    ctx.vl_profile_enable(0)

    gemm_flops = m.gemm_flops_per_token() * n
    if not wl.check_argmax:
        gemm_flops -= 2.0 * m.vocab * m.d_model * n
    attn_flops = attention_flops(m, wl.lengths)
    mfma_tflops = (gemm_flops + attn_flops) / (ms_per_step * 1e-3) / 1e12
    gu_flops = 2.0 * n * (2 * m.d_ffn) * m.d_model
    gu_avg_ms = gu_ms / max(gu_launches, 1)
    gu_tflops = gu_flops / (gu_avg_ms * 1e-3) / 1e12 if gu_launches else 0.0
    compare_bytes = c * n * m.d_model * (4 + (2 if bf else 4))
    compare_gbs = compare_bytes / (stages.get("compare", 0) * 1e-3) / 1e9 if stages.get("compare") else None
    # the argmax over the vocabulary is the epilogue of the LM-head GEMM (no logits in memory); the "argmax" stage is
    # the reduction of its per-part maxima: vocab / 128 (value, index) pairs per token
    argmax_gbs = n * ((m.vocab + 127) // 128) * 8 / (stages.get("argmax", 0) * 1e-3) / 1e9 if stages.get("argmax") else None

    out = {
        "metric": "verified tokens/s (8B-shape bf16 prefill+compare, 1 GPU); MFMA util %",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if m.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "model_shape": m.name, "layers": m.n_layers, "d_model": m.d_model,
                   "tokens": n, "sequences": len(wl.lengths), "commit_layers": list(wl.commit_layers),
                   "argmax_check": wl.check_argmax, "tampered_positions": int(len(pos))},
        "mfma_util_pct": round(100.0 * mfma_tflops / PEAK_BF16_TFLOPS, 2),
        "achieved_tflops_whole_path": round(mfma_tflops, 1),
        "device_ms_per_step": round(dev_ms / args.steps, 3),
        "flags_match_tamper_mask": flags_ok,
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma_kernel<SWIGLU> (gate/up GEMM, M=%d N=%d K=%d)" % (n, 2 * m.d_ffn, m.d_model),
                     "achieved": round(gu_tflops, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(gu_tflops / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(wl),
                     "avg_launch_ms": round(gu_avg_ms, 4), "launches": gu_launches},
        "stages_ms": stages,
        "compare_stage": {"achieved_GBps": round(compare_gbs, 1) if compare_gbs else None,
                          "argmax_GBps": round(argmax_gbs, 1) if argmax_gbs else None, "peak_GBps": PEAK_HBM_GBS},
        "commit_seconds": round(t_commit, 3),
        "verify_over_commit_cost": round((ms_per_step * 1e-3) / t_commit, 5),
        "commit_kind": "prefill" if args.no_decode else "prefill(prompt)+decode",
        "merkle_commit": merkle,
    }
    if not args.no_decode:
        # the inferencer's side: every decode step streams all weights once (the embedding table is only gathered from)
        steps_dec = max(t - pl for t, pl in zip(wl.lengths, wl.prompt_lens))
        w_bytes = (m.n_params() - m.vocab * m.d_model) * 2
        ms_dec = t_commit * 1e3 / max(steps_dec, 1)
        out["decode_commit"] = {"steps": int(steps_dec), "ms_per_step_incl_prompt_prefill": round(ms_dec, 3),
                                 "weight_bytes_per_step": int(w_bytes), "bound": "hbm",
                                 "achieved_GBps": round(w_bytes / (ms_dec * 1e-3) / 1e9, 1), "peak_GBps": PEAK_HBM_GBS,
                                 "frac": round(w_bytes / (ms_dec * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}

    # ---- CPU baseline: the oracle, untuned, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import verillm_oracle as O

        ts = min(args.cpu_sample_tokens, wl.lengths[0])
        log(f"[bench] CPU oracle on the first {ts} tokens of sequence 0 (all {m.n_layers} layers, LM head, compare) ...")

        def wfn(kind, layer):
            w = host_w.get((kind, layer))
            return w if w is not None else synth.weight(m, kind, layer, 16)

        om = O.Model(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab, m.rms_eps,
                     m.rope_base, wfn)
        com_s = (synth.f32_to_bf16_bits(com_t[:, :ts]) if bf else com_t[:, :ts]) if c else np.zeros((0, ts, m.d_model), np.float32)
        t0 = time.perf_counter()
        ref = O.verify(om, x[:ts], [ts], wl.commit_layers, com_s, cam_t[:ts] if wl.check_argmax else None, wl.tol_rel_l2,
                       wl.tol_max_abs, wl.tol_logit_margin)
        t_cpu = time.perf_counter() - t0
        same = bool((ref["flags"] == d_flags.cpu().numpy()[:ts]).all())
        log(f"[bench] oracle: {ts} tokens in {t_cpu:.1f} s; its flags equal the GPU's on the sample: {same}")
        try:
            cores = len(os.sched_getaffinity(0))
        except Exception:
            cores = os.cpu_count()
        omp = os.environ.get("OMP_NUM_THREADS")
        if omp:
            cores = min(cores, int(omp))
        out["cpu_baseline"] = {"value": round(ts / t_cpu, 3), "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "sample": "first %d tokens of sequence 0, all %d layers + LM head + compare, float64 numpy; "
                                         "weights already drawn, their upcast to float64 included" % (ts, m.n_layers),
                               "flags_equal_gpu_on_sample": same}
    ctx.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
