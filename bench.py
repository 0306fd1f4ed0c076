"""Benchmark of the GSA hot path on one MI355X.

A step is one forward + backward of the operator over the 1.3B-layer batch
(B=8, T=2048, H=4, d_k=d_v=512, m=64, bf16, 16384 tokens), inputs resident in HBM.
Prints ONE JSON line: throughput, the roofline of the dominant kernel (measured with
HIP events inside the library on the launch stream), the decode step's bandwidth, and
the fp64 CPU oracle timed on the host cores as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def per_token_bytes(cfg, esz):
    """Compulsory HBM bytes per token (all H heads) of forward and backward: every input read
    once, every output written once; chunk memories and other workspace traffic not counted."""
    H, dk, dv, m = cfg.H, cfg.d_k, cfg.d_v, cfg.m
    fwd = H * ((2 * dk + dv) * esz + m * 4 + dv * esz + m * 4)             # q,k,v,g -> o,z
    bwd = H * ((2 * dk + 2 * dv) * esz + 2 * m * 4 + (2 * dk + dv) * esz + m * 4)   # q,k,v,dO,g,z -> dq,dk,dv,dg
    return fwd, bwd


def per_token_head_flops(cfg, C=64):
    """Matrix-core FLOPs per (token, head) at chunk size C.

    nominal: the count of the chunkwise scheme as written (Appendix A; Algorithm 1), every C x C product in
             full: forward 2C(d_k+d_v) + 4Cm + 4m(d_k+d_v); backward (recompute, dp/dz, reverse scan,
             gradients) 5C(d_k+d_v) + 10Cm + 10m(d_k+d_v).
    executed: what the kernels issue.  The chunk kernels skip the 16 x 16 blocks above the diagonal of every
             causally masked C x C product (10 of 16 blocks at C = 64); the wide contractions (apply kernel)
             multiply the masked matrices in full.  This is the number the MFMA fraction is quoted on.
    algorithmic: the chunk-free recurrent form, 4m(d_k+d_v) forward and 8m(d_k+d_v) backward."""
    dk, dv, m = cfg.d_k, cfg.d_v, cfg.m
    D = dk + dv
    nb = C // 16
    tri = (nb * (nb + 1) // 2) / float(nb * nb)
    nominal = (2 * C * D + 4 * C * m + 4 * m * D, 5 * C * D + 10 * C * m + 10 * m * D)
    fwd = (2 * m * D                                             # scan
           + 2 * C * dk * tri + 2 * m * dk + 4 * C * m * tri     # QK^T, Q Kt^T, gated intra scores, pair weights A2
           + 2 * C * dv + 2 * m * dv)                            # o
    bwd = (2 * m * D                                             # recomputed scan
           + 2 * C * dv * tri + 2 * m * dv + 2 * C * m * tri     # dO V^T, dO Vt^T, gated intra part of dp
           + 2 * m * D                                           # reverse scan
           + 2 * C * dk * tri + 2 * m * D + 8 * C * m * tri      # QK^T, [K|V] E^T, intra part of ds (2x), Bm, A2
           + 2 * C * (2 * dk + dv) + 2 * m * (2 * dk + dv))      # dq, dk, dv
    return dict(executed=(fwd, bwd), nominal=nominal, algorithmic=(4 * m * D, 8 * m * D))


def prefill_decode(args):
    """Generation workload (the shape of the paper's Figure 4c measurement): batch 1, 24 layers of
    H=4, m=64, d=512; a 2048-token prefix through gsa_fwd, whose final memories seed a token-by-token
    gsa_decode_step loop over the layers.  One decode token = 24 dependent launches of 4 memories each,
    a latency-bound regime, so the loop is also replayed from a HIP graph."""
    import torch
    import paper_2409_07146_amd as gsa
    from paper_2409_07146_amd import synth
    dev = torch.device("cuda:0")
    L, T, ntok = 24, 2048, args.decode_steps
    cfg = synth.GsaConfig("prefill", B=1, T=T, H=4, d_k=512, d_v=512, m=64, dtype="bf16", seed=41)
    x = synth.make_inputs(cfg)
    q, k, v, g = (x[n].to(dev) for n in ("q", "k", "v", "g"))
    prob = gsa.make_problem(q, v, g, 1.0, None)
    ws = gsa.alloc_workspace(prob, False, dev)

    def prefill():
        return [gsa.gsa_fwd(q, k, v, g, save_z=False, final_state=True, workspace=ws)[2:] for _ in range(L)]

    states = prefill()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        states = prefill()
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - t0) / 3 * 1e3
    d = synth.make_decode_inputs(1, 4, 512, 512, 64, 4, seed=42)
    dq_, dk_, dv_, dg_ = (d[n].to(dev) for n in ("q", "k", "v", "g"))
    out = torch.empty_like(dv_[0])
    dws = gsa.alloc_decode_workspace(1, 4, 512, 512, 64, dev) if not args.decode_one_workgroup else None

    def token(i):
        for KT, VT in states:
            gsa.gsa_decode_step(dq_[i % 4], dk_[i % 4], dv_[i % 4], dg_[i % 4], KT, VT, out=out, workspace=dws)

    for i in range(8):
        token(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(ntok):
        token(i)
    torch.cuda.synchronize()
    eager_us = (time.perf_counter() - t0) / ntok * 1e6
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        token(0)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        token(0)
    for _ in range(8):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(ntok):
        graph.replay()
    torch.cuda.synchronize()
    graph_us = (time.perf_counter() - t0) / ntok * 1e6
    state_bytes = 2 * 4 * L * 4 * 64 * 1024
    print(json.dumps({
        "metric": "gsa_decode_tokens_per_s_batch1", "value": round(1e6 / graph_us, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": ntok, "warmup": 8, "ms_per_step": round(graph_us * 1e-3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "prefill_decode: batch 1, 24 layers x (H=4 m=64 d_k=d_v=512), 2048-token prefix "
                               "(bf16) then one %s per layer and token (fp32 memories), HIP graph over the 24 layers"
                               % ("gsa_decode_step" if dws is None else "gsa_decode_step_ws")},
        "decode_token_us": {"hip_graph": round(graph_us, 2), "eager_launches": round(eager_us, 2),
                            "per_layer_step_graph": round(graph_us / L, 2)},
        "state_GB_per_s": round(state_bytes / graph_us / 1e3, 1),
        "prefill": {"ms_24_layers": round(prefill_ms, 3), "tokens_per_s": round(T / (prefill_ms * 1e-3), 1)},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="layer_1p3b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-steps", type=int, default=512)
    ap.add_argument("--readout", default="softmax", choices=["softmax", "identity", "swish", "relu", "relu2"],
                    help="read-out variant (gsa_fwd_ex / gsa_bwd_ex); the headline is softmax")
    ap.add_argument("--given-intensity", action="store_true",
                    help="write intensities as an input of their own (gsa_fwd_ex / gsa_bwd_ex)")
    ap.add_argument("--feature-map", default="none", choices=["none", "swish"],
                    help="q, k, v as raw projections with the Swish feature map applied inside the kernels; also "
                         "times the same work with the feature map as element-wise passes of their own")
    ap.add_argument("--epilogue", action="store_true",
                    help="also time the forward with the layer's output epilogue fused in (gsa_fwd_act) against the "
                         "forward followed by the same work as element-wise passes of their own")
    ap.add_argument("--decode-one-workgroup", action="store_true",
                    help="prefill_decode: use gsa_decode_step (one workgroup per memory) instead of gsa_decode_step_ws")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the operator has no cross-GPU path); "
              "--gpus %d with WORLD_SIZE=%s is not supported" % (args.gpus, os.environ.get("WORLD_SIZE", "1")),
              file=sys.stderr)
        sys.exit(2)

    if args.workload == "prefill_decode":
        return prefill_decode(args)

    import torch
    import paper_2409_07146_amd as gsa
    from paper_2409_07146_amd import synth

    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.workload] if args.workload in synth.CONFIGS else synth.VARIANTS[args.workload]
    x = synth.make_inputs(cfg)
    put = lambda t: None if t is None else t.to(dev)
    q, k, v, g, dO, cu = (put(x[n]) for n in ("q", "k", "v", "g", "dO", "cu_seqlens"))
    prob = gsa.make_problem(q, v, g, 1.0, cu)
    ws = gsa.alloc_workspace(prob, True, dev)

    s_in = (-torch.expm1(g)).contiguous() if args.given_intensity else None
    var = dict(s=s_in, readout=args.readout, feature_map=args.feature_map)

    def step():
        o, z, _, _ = gsa.gsa_fwd(q, k, v, g, cu_seqlens=cu, workspace=ws, **var)
        return gsa.gsa_bwd(q, k, v, g, z, dO, cu_seqlens=cu, workspace=ws, **var)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tokens = cfg.tokens
    tok_s = tokens / (dt / args.steps)
    # the same steps again, each bracketed by a pair of events on the launch stream (the library enqueues on
    # torch's current stream, so torch's events see its kernels): median and spread of single steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(args.steps, 50))]
    for a, b in evs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    ev_ms = sorted(a.elapsed_time(b) for a, b in evs)
    ev_median, ev_min, ev_p90 = ev_ms[len(ev_ms) // 2], ev_ms[0], ev_ms[(9 * len(ev_ms)) // 10]

    # "GSA w/o recomp." (Section 4, Efficiency): the forward keeps the per-chunk memories for the backward.
    # A second figure beside the headline one, which recomputes them as the paper's default does.
    prob_k = gsa.make_problem(q, v, g, 1.0, cu, keep_states=True)
    ws_k = gsa.alloc_workspace(prob_k, True, dev)

    def step_keep():
        o, z, _, _ = gsa.gsa_fwd(q, k, v, g, cu_seqlens=cu, workspace=ws_k, keep_states=True, **var)
        return gsa.gsa_bwd(q, k, v, g, z, dO, cu_seqlens=cu, workspace=ws_k, keep_states=True, **var)

    for _ in range(args.warmup):
        step_keep()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_keep()
    torch.cuda.synchronize()
    keep_ms = (time.perf_counter() - t0) / args.steps * 1e3
    esz_k = 2 if cfg.dtype == "bf16" else 4
    chunk_k = 64 if cfg.dtype == "bf16" else 32
    kept_bytes = (tokens // chunk_k) * cfg.H * cfg.m * (cfg.d_k + cfg.d_v) * esz_k
    del ws_k

    # the same work with the feature map outside the operator: three element-wise passes before the
    # forward, three through the slope after the backward (torch's kernels; a comparison leg only)
    outside_ms = None
    if args.feature_map != "none":
        var0 = dict(var, feature_map="none")
        F = torch.nn.functional

        def step_outside():
            pq, pk, pv = F.silu(q), F.silu(k), F.silu(v)
            o, z, _, _ = gsa.gsa_fwd(pq, pk, pv, g, cu_seqlens=cu, workspace=ws, **var0)
            r = gsa.gsa_bwd(pq, pk, pv, g, z, dO, cu_seqlens=cu, workspace=ws, **var0)
            return (torch.ops.aten.silu_backward(r[0], q), torch.ops.aten.silu_backward(r[1], k),
                    torch.ops.aten.silu_backward(r[2], v))

        for _ in range(args.warmup):
            step_outside()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_outside()
        torch.cuda.synchronize()
        outside_ms = (time.perf_counter() - t0) / args.steps * 1e3

    # the layer's output epilogue (Swish(o), sums of squares for the RMS norm): fused into the kernel that
    # writes o against torch's element-wise kernels after it (a comparison leg only; forward calls)
    epilogue = None
    if args.epilogue:
        def timed(fn):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / args.steps * 1e3

        def outside():
            o = gsa.gsa_fwd(q, k, v, g, cu_seqlens=cu, workspace=ws, **var)[0]
            y = torch.nn.functional.silu(o)
            return y, y.float().pow(2).sum(-1)

        epilogue = {"fwd_ms": round(timed(lambda: gsa.gsa_fwd(q, k, v, g, cu_seqlens=cu, workspace=ws, **var)), 4),
                    "fwd_act_fused_ms": round(timed(lambda: gsa.gsa_fwd_act(q, k, v, g, cu_seqlens=cu, workspace=ws,
                                                                            **var)), 4),
                    "fwd_act_fused_without_o_ms": round(timed(lambda: gsa.gsa_fwd_act(q, k, v, g, cu_seqlens=cu,
                                                                                      workspace=ws, want_o=False,
                                                                                      **var)), 4),
                    "fwd_then_elementwise_passes_ms": round(timed(outside), 4)}

    # per-kernel durations, HIP events on the launch stream (second pass, same work)
    gsa.gsa_profile_reset()
    gsa.gsa_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    # yardstick: a plain device copy of 256 MiB (512 MiB of traffic) through the library's probe kernel
    prof = gsa.gsa_profile_read()
    cp_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    cp_dst = torch.empty_like(cp_src)
    for _ in range(3):
        gsa.gsa_profile_copy(cp_dst, cp_src)      # first touches of the destination
    torch.cuda.synchronize()
    gsa.gsa_profile_reset()
    for _ in range(10):
        gsa.gsa_profile_copy(cp_dst, cp_src)
    torch.cuda.synchronize()
    prof["copy_probe_kernel"] = gsa.gsa_profile_read()["copy_probe_kernel"]
    gsa.gsa_profile_enable(False)
    del cp_src, cp_dst
    kern_ms = {n: ms / max(cnt, 1) for n, (ms, cnt) in prof.items() if cnt}
    esz = 2 if cfg.dtype == "bf16" else 4
    fwd_b, bwd_b = per_token_bytes(cfg, esz)
    # algorithmic bytes of each kernel per launch: the API tensors it must read or write once
    # (workspace traffic -- chunk memories, small per-chunk matrices -- is not counted)
    H, dk, dv, m = cfg.H, cfg.d_k, cfg.d_v, cfg.m
    per_tok = {
        "scan_fwd_kernel": H * (dk + dv) * esz,
        "chunk_fwd_kernel": H * (2 * dk * esz + 8 * m),
        "apply_fwd_kernel": H * 2 * dv * esz,
        "chunk_dz_kernel": H * (2 * dv * esz + 8 * m),
        "scan_bwd_kernel": H * (dk + dv) * esz,
        "chunk_intra_kernel": H * ((2 * dk + dv) * esz + 12 * m),
        "apply_bwd_kernel": H * 2 * (2 * dk + dv) * esz,
    }
    alg_bytes = {n: b * tokens for n, b in per_tok.items()}
    dom = max((n for n in kern_ms if n in alg_bytes), key=lambda n: kern_ms[n])
    achieved = alg_bytes[dom] / (kern_ms[dom] * 1e-3) / 1e9
    fl = per_token_head_flops(cfg)
    exec_flops = sum(fl["executed"]) * tokens * cfg.H
    nominal_flops = sum(fl["nominal"]) * tokens * cfg.H
    # HBM traffic per launch of that kernel, from hardware counters collected in separate profiler
    # runs of this same command (stored next to their summaries); None when no such record exists
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.json" % cfg.name)
    if os.path.exists(tpath):
        with open(tpath) as f:
            rec = json.load(f).get("kernels", {}).get(dom)
        if rec:
            traffic = int(rec["fetch_bytes"] + rec["write_bytes"])
    step_bytes = (fwd_b + bwd_b) * tokens
    roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "avg_launch_ms": round(kern_ms[dom], 4),
                "algorithmic_bytes_per_launch": alg_bytes[dom],
                # the per-kernel figure credits a kernel with every API tensor it touches, and several kernels
                # touch the same tensor; the whole step against every API tensor counted ONCE is the honest total
                "whole_step": {"compulsory_bytes": step_bytes,
                               "GB_per_s": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                               "frac": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                               "note": "per-kernel algorithmic bytes overlap across kernels"}}

    # decode step: 512 steps at batch 64 (one state set, then rotating over 8 state sets)
    dd = synth.DECODE
    di = synth.make_decode_inputs(dd["B"], dd["H"], dd["d_k"], dd["d_v"], dd["m"], 4, state_std=dd["state_std"],
                                  seed=dd["seed"])
    nsets = 8
    Ks = [di["K"].to(dev).clone() for _ in range(nsets)]
    Vs = [di["V"].to(dev).clone() for _ in range(nsets)]
    dq_, dk_, dv_, dg_ = (di[n].to(dev) for n in ("q", "k", "v", "g"))
    od = torch.empty_like(dv_[0])
    state_bytes = 2 * 4 * dd["B"] * dd["H"] * dd["m"] * (dd["d_k"] + dd["d_v"])
    dec = {}
    for label, sets, w in (("one_state_set", 1, None), ("rotating_8_state_sets", nsets, None)):
        for i in range(20):
            gsa.gsa_decode_step(dq_[i % 4], dk_[i % 4], dv_[i % 4], dg_[i % 4], Ks[i % sets], Vs[i % sets], out=od,
                                workspace=w)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.decode_steps):
            gsa.gsa_decode_step(dq_[i % 4], dk_[i % 4], dv_[i % 4], dg_[i % 4], Ks[i % sets], Vs[i % sets], out=od,
                                workspace=w)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / args.decode_steps * 1e6
        dec[label] = {"entry": "gsa_decode_step" if w is None else "gsa_decode_step_ws", "us_per_step": round(us, 2),
                      "GB_per_s": round(state_bytes / us / 1e3, 1),
                      "frac_hbm_peak": round(state_bytes / us / 1e3 / HBM_PEAK_GBS, 4)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import build as obuild
        obuild.build(force=False)
        from oracle import gsa_oracle
        f64 = lambda t: None if t is None else t.double().numpy()
        cun = None if x["cu_seqlens"] is None else x["cu_seqlens"].numpy()
        qn, kn, vn, gn, dn = (f64(x[n]) for n in ("q", "k", "v", "g", "dO"))
        reps, cdt = 0, 0.0
        t0 = time.perf_counter()
        while cdt < 10.0 and reps < 64:      # a bounded sample: whole batches until about 10 s of CPU work
            gsa_oracle.fwd(qn, kn, vn, gn, cu_seqlens=cun)
            gsa_oracle.bwd(qn, kn, vn, gn, dn, cu_seqlens=cun)
            reps += 1
            cdt = time.perf_counter() - t0
        cpu = {"value": round(reps * tokens / cdt, 1), "unit": "tokens/s", "cores": gsa_oracle.num_threads(),
               "kind": "oracle", "sample": "the whole %s batch (%d tokens), fp64 forward + backward, %d repetitions, "
               "%.1f s" % (cfg.name, tokens, reps, cdt)}

    out = {
        "metric": "gsa_layer_fwd_bwd_tokens_per_s", "value": round(tok_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "%s: B=%d T=%d H=%d d_k=%d d_v=%d m=%d fwd+bwd%s" % (
            cfg.name, cfg.B, cfg.T, cfg.H, cfg.d_k, cfg.d_v, cfg.m,
            "" if cfg.cu_seqlens is None else " packed %s" % (list(cfg.cu_seqlens),)),
            "tokens_per_step": tokens, "chunk": 64, "readout": args.readout,
            "write_intensity": "given" if args.given_intensity else "1 - exp(g)",
            "feature_map": args.feature_map},
        **({} if outside_ms is None else {"feature_map_outside_ms_per_step": round(outside_ms, 4)}),
        **({} if epilogue is None else {"epilogue": epilogue}),
        "roofline": roofline,
        "timing": {"wall_mean_ms": round(ms_per_step, 4), "event_median_ms": round(ev_median, 4),
                   "event_min_ms": round(ev_min, 4), "event_p90_ms": round(ev_p90, 4), "event_steps": len(ev_ms)},
        "path": {"executed_gflop_per_step": round(exec_flops / 1e9, 2),
                 "nominal_gflop_per_step": round(nominal_flops / 1e9, 2),
                 "executed_tflops": round(exec_flops / (ms_per_step * 1e-3) / 1e12, 2),
                 "frac_mfma_bf16_peak": round(exec_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                 "algorithmic_GB_per_s": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                 "frac_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                 "kernel_ms": {n: round(ms, 4) for n, ms in kern_ms.items()}},
        "without_recompute": {"entry": "gsa_fwd/gsa_bwd with gsa_problem.keep_states", "ms_per_step": round(keep_ms, 4),
                              "tokens_per_s": round(tokens / (keep_ms * 1e-3), 1),
                              "memories_kept_bytes": kept_bytes},
        "decode": dec,
        "copy_probe": {"bytes_moved": 2 * (256 << 20), "us": round(kern_ms["copy_probe_kernel"] * 1e3, 2),
                       "GB_per_s": round(2 * (256 << 20) / (kern_ms["copy_probe_kernel"] * 1e-3) / 1e9, 1)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
