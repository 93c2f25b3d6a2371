"""Benchmark of the QaRL low-bit MoE hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras] [--no-cpu]

A step is one pass of the decode-shaped W4A16 MoE layer (route -> gate_up GEMM with SiLU*mul ->
down GEMM -> weighted combine; the GEMMs take the router's ids directly) over one batch of 256 synthetic tokens with
Qwen3-30B-A3B expert shapes (128 experts, hidden 2048, intermediate 768, top-8), every input
already resident in HBM.  The quantized weights rotate over several distinct copies so that the
256 MB last-level cache cannot serve a 311 MB layer twice.  Prints ONE JSON line: the decode
figure as `value` (algorithmic GB/s), the roofline of the dominant kernel, the oracle timed on
the host cores, and under `extra` the other rows of the path (prefill TFLOP/s, quantize GB/s,
FP8, LM-head log-prob, the 48-layer sweep).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TF = 2500.0
MFMA_FP8_PEAK_TF = 5000.0
# HBM bytes per gate_up launch of the headline step from two counter runs (2.000 x FETCH_SIZE + 1.000 x WRITE_SIZE,
# the factors a plain copy kernel of known size gives).  Counters cannot be read from inside this process, so the
# figure is stored with the summary it comes from; it belongs to the 256-token workload and to the kernel as it
# stood when that summary was taken: 217 302 647 B read + 3 146 985 B written (an earlier measurement of the same
# launch, profiles/qgemm_stream_decode256_hbm_traffic.txt, gave 220 271 616 B).
GATE_UP_TRAFFIC_BYTES = 220449632
GATE_UP_TRAFFIC_SOURCE = "profiles/qgemm_all_formats_hbm_traffic.txt"
MIN_EVENT_LAUNCHES = 32   # gate_up launches bracketed by events, whatever --steps is


def weight_bytes_w4a16(E, N, K):
    return E * N * (K // 2 + K // 128 * 2)


def weight_bytes_fp8(E, N, K):
    return E * N * (K + 4)


def weight_bytes_fp4(E, N, K):
    return E * N * (K // 2 + 4)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--copies", type=int, default=4, help="distinct weight copies the steps rotate over")
    ap.add_argument("--settle", type=int, default=1000,
                    help="untimed steps at the end of the set-up, before the W warm-up steps: the clocks and the memory "
                         "system reach the steady state of a running decode loop (a step measured 2 %% slower right "
                         "after the set-up kernels)")
    ap.add_argument("--event-every", type=int, default=8,
                    help="bracket the dominant launch with HIP events on every N-th timed step")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--extras", default="all",
                    help="comma-separated subset of the other rows to time: quantize, prefill (with the LM head and the "
                         "sequence objective), backward, dense, fp8, stack; default all")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--sweep-layers", type=int, default=48)
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 256 MiB -> 256 MiB elementwise copy a few times, the known-size kernel "
                         "that FETCH_SIZE / WRITE_SIZE readings of a counter run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not "
                 "supported, run with --gpus 1" % args.gpus)

    import numpy as np
    import torch
    from paper_2604_07853_amd import binding as q
    from paper_2604_07853_amd import synth

    q.lib()
    torch.cuda.set_device(0)
    dev = "cuda"
    E, H, I, TOPK = synth.E, synth.H, synth.I, synth.TOPK
    T = 256
    M = T * TOPK

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def timed(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters  # ms

    def rotate(items):
        """A callable that returns the next of `items` at every call: GEMM launches timed on their own alternate
        between copies of the weights, so that a tensor smaller than the 256 MB last-level cache is not served
        from it (inside a layer the other launches evict it)."""
        state = [0]

        def nxt():
            state[0] += 1
            return items[state[0] % len(items)]
        return nxt

    def clone_qw(w):
        c = q.QWeight.empty(w.fmt, w.E, w.N, w.K, dev)
        c.codes.copy_(w.codes)
        c.scales.copy_(w.scales)
        return c

    # ---- weights: `copies` independently drawn layers, quantized by the library's own kernel
    layers = []
    masters0 = None
    for c in range(args.copies):
        gu, dn = synth.expert_weights(E, H, I, seed=1000 + 2 * c, device=dev)
        qgu = q.qarl_quantize_weights(gu)
        qdn = q.qarl_quantize_weights(dn)
        if c == 0:
            masters0 = (gu, dn)
        else:
            del gu, dn
        layers.append(q.MoELayer(qgu, qdn, T, TOPK, q.QARL_PATH_DECODE, dev))
    xs = [synth.normal_bf16((T, H), 1.0, seed=10 + i, device=dev) for i in range(4)]
    lgs = [synth.router_logits(T, E, seed=20 + i, device=dev) for i in range(4)]
    torch.cuda.synchronize()

    state = {"i": 0}
    gu_events = []

    # One step = the whole hot path of a decode-sized batch: router, gate_up (SiLU*mul), down + combine.  At this
    # size the GEMMs take the router's ids directly (qarl_qgemm_routed), so no grouping pass runs.  The dominant
    # launch (gate_up) is bracketed by HIP events on every EVENT_EVERY-th step of the timed region: an event pair
    # costs the stream a few microseconds, and the step time is the headline.
    EVENT_EVERY = max(1, args.event_every)

    def step(record=False):
        i = state["i"]
        state["i"] += 1
        layer = layers[i % len(layers)]
        x, lg = xs[i % 4], lgs[i % 4]
        r = q.qarl_moe_route(lg, TOPK, True, out=layer.routing, group=False)
        if record:
            a, b = ev(), ev()
            a.record()
        q.qarl_qgemm_routed(layer.gu, x, r.ids, T, TOPK, True, epilogue=q.QARL_EPI_SILU_MUL, out=layer.a, ws=layer.ws)
        if record:
            b.record()
            gu_events.append((a, b))
        q.qarl_qgemm_routed(layer.dn, layer.a, r.ids, T, TOPK, False, epilogue=q.QARL_EPI_COMBINE, combine_w=r.w,
                            out=layer.out, ws=layer.ws)

    for _ in range(args.settle):   # set-up, not part of the contract's W warm-up steps
        step()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0, t1 = ev(), ev()
    t0.record()
    for k in range(args.steps):
        step(record=(k % EVENT_EVERY == min(EVENT_EVERY // 2, args.steps - 1)))
    t1.record()
    torch.cuda.synchronize()
    ms_step = t0.elapsed_time(t1) / args.steps
    timed_in_region = len(gu_events)
    k = 0
    while len(gu_events) < MIN_EVENT_LAUNCHES:      # a short run: further bracketed launches behind the timed region,
        step(record=(k % 2 == 1))                   # every other step, in the same rotation over the weight copies
        k += 1
    torch.cuda.synchronize()
    if args.calibrate:
        ca = torch.ones((64 << 20,), dtype=torch.float32, device=dev)
        cb = torch.empty_like(ca)
        for _ in range(5):
            torch.mul(ca, 1.0, out=cb)
        torch.cuda.synchronize()
        del ca, cb
    gu_times = np.array([a.elapsed_time(b) for a, b in gu_events])
    ms_gu = float(gu_times.mean())

    # algorithmic bytes of a step: every expert's codes + scales once, logits, x, a (written + read), out
    active = int(torch.unique(layers[0].routing.ids).numel())
    w_gu = weight_bytes_w4a16(E, 2 * I, H) * active // E
    w_dn = weight_bytes_w4a16(E, H, I) * active // E
    act = T * E * 2 + T * H * 2 + 2 * M * I * 2 + T * H * 2
    step_bytes = w_gu + w_dn + act
    gu_bytes = w_gu + T * H * 2 + M * I * 2
    value = step_bytes / (ms_step * 1e-3) / 1e9
    gu_gbs = gu_bytes / (ms_gu * 1e-3) / 1e9

    result = {
        "metric": "MoE quant GEMM: decode HBM GB/s + prefill TFLOP/s, % of MI355X roofline",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 weights x bf16 activations, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "moe_decode_w4a16: 256 tokens, 128 experts x (gate_up [1536,2048] + down [2048,768]) "
                               "int4 g128, top-8, bf16 out", "tokens": T, "experts": E, "active_experts": active,
                   "weight_copies": args.copies, "settle_steps": args.settle, "step_bytes": step_bytes,
                   "step_flop": synth.flops_moe(T)},
        "roofline": {"bound": "hbm", "kernel": "qgemm_stream_w4_kernel<SILU_MUL> (gate_up)",
                     "achieved": round(gu_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gu_gbs / HBM_PEAK_GBS, 4), "traffic": GATE_UP_TRAFFIC_BYTES,
                     "traffic_source": GATE_UP_TRAFFIC_SOURCE,
                     "bytes_per_launch": gu_bytes, "ms_per_launch": round(ms_gu, 5),
                     "ms_per_launch_median": round(float(np.median(gu_times)), 5), "launches_timed": len(gu_events),
                     "launches_timed_inside_region": timed_in_region,
                     "note": "event brackets add about 3 us to a launch; the kernel trace under profiles/ has the "
                             "kernel's own duration",
                     "step_frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4)},
    }

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    if not args.no_cpu:
        import oracle
        gu, dn = masters0
        n_steps_cpu = 4
        guc, gus = oracle.quantize_int4(synth.bits(gu))
        dnc, dns = oracle.quantize_int4(synth.bits(dn))
        xb = [synth.bits(x) for x in xs[:n_steps_cpu]]
        lb = [synth.bits(l) for l in lgs[:n_steps_cpu]]
        c0 = time.perf_counter()
        for i in range(n_steps_cpu):
            oracle.moe_ffn_w4a16(xb[i], lb[i], guc, gus, dnc, dns, TOPK)
        cpu_s = (time.perf_counter() - c0) / n_steps_cpu
        result["cpu_baseline"] = {"value": round(step_bytes / cpu_s / 1e9, 4), "unit": "GB/s", "cores": oracle.cores(),
                                  "kind": "oracle", "sample": "%d full steps of the same layer (256 tokens, all 128 "
                                  "experts), %.2f s per step" % (n_steps_cpu, cpu_s)}
    del masters0

    # ---- the other rows of the path, each timed on its own
    if not args.no_extras:
        extra = {}
        want = set(args.extras.split(","))
        on = lambda name: "all" in want or name in want
        # (a1) int4 re-quantization of one layer's masters (the fp8 copies below feed the fp8 rows)
        gu, dn = synth.expert_weights(E, H, I, seed=5000, device=dev)
        outq = q.QWeight.empty(q.QARL_W4A16_G128, E, 2 * I, H, dev)
        ms = timed(lambda: q.qarl_quantize_weights(gu, out=outq), 20, 3)
        qb = gu.numel() * 2 + weight_bytes_w4a16(E, 2 * I, H)
        extra["quantize_int4_gate_up"] = {"ms": round(ms, 4), "GB/s": round(qb / ms / 1e6, 1),
                                          "frac_hbm": round(qb / ms / 1e6 / HBM_PEAK_GBS, 4), "bytes": qb}
        outf = q.QWeight.empty(q.QARL_FP8_E4M3_CH, E, 2 * I, H, dev)
        ms = timed(lambda: q.qarl_quantize_weights(gu, q.QARL_FP8_E4M3_CH, out=outf), 20, 3)
        qb8 = gu.numel() * 2 + weight_bytes_fp8(E, 2 * I, H)
        extra["quantize_fp8_gate_up"] = {"ms": round(ms, 4), "GB/s": round(qb8 / ms / 1e6, 1),
                                         "frac_hbm": round(qb8 / ms / 1e6 / HBM_PEAK_GBS, 4), "bytes": qb8}
        qdn8 = q.qarl_quantize_weights(dn, q.QARL_FP8_E4M3_CH)
        lowbit = [("fp8", outf, qdn8, weight_bytes_fp8(E, 2 * I, H) + weight_bytes_fp8(E, H, I))]
        if on("fp8"):   # the two 4-bit-weight x e4m3-activation formats ride along in the fp8 rows
            outf4 = q.QWeight.empty(q.QARL_FP4_E2M1_CH, E, 2 * I, H, dev)
            ms = timed(lambda: q.qarl_quantize_weights(gu, q.QARL_FP4_E2M1_CH, out=outf4), 20, 3)
            qb4 = gu.numel() * 2 + weight_bytes_fp4(E, 2 * I, H)
            extra["quantize_fp4_gate_up"] = {"ms": round(ms, 4), "GB/s": round(qb4 / ms / 1e6, 1),
                                             "frac_hbm": round(qb4 / ms / 1e6 / HBM_PEAK_GBS, 4), "bytes": qb4}
            lowbit.append(("fp4", outf4, q.qarl_quantize_weights(dn, q.QARL_FP4_E2M1_CH),
                           weight_bytes_fp4(E, 2 * I, H) + weight_bytes_fp4(E, H, I)))
            lowbit.append(("w4a8", q.qarl_quantize_weights(gu, q.QARL_W4A8_G128), q.qarl_quantize_weights(dn, q.QARL_W4A8_G128),
                           weight_bytes_w4a16(E, 2 * I, H) + weight_bytes_w4a16(E, H, I)))
        del gu, dn

        if on("prefill"):
            # (a6-a9) prefill / training-forward shape, W4A16: 8 x 2048 tokens, Zipf-skewed router
            Tp = 16384
            xp = synth.normal_bf16((Tp, H), 1.0, seed=30, device=dev)
            lgp = synth.router_logits(Tp, E, seed=31, device=dev, zipf_s=1.1)
            lp_layer = q.MoELayer(layers[0].gu, layers[0].dn, Tp, TOPK, q.QARL_PATH_PREFILL, dev)
            ms_all = timed(lambda: lp_layer.forward(xp, lgp), 10, 2)
            r = lp_layer.routing
            Mp = Tp * TOPK
            next_gu, next_dn = rotate([l.gu for l in layers]), rotate([l.dn for l in layers])
            ms_gu_p = timed(lambda: q.qarl_qgemm_grouped(next_gu(), xp, r.offsets, Mp, row_map=r.tokens,
                                                         epilogue=q.QARL_EPI_SILU_MUL, out=lp_layer.a,
                                                         path=q.QARL_PATH_PREFILL, ws=lp_layer.ws), 12, 2)
            ybuf = torch.empty((Mp, H), dtype=torch.float32, device=dev)
            ms_dn_p = timed(lambda: q.qarl_qgemm_grouped(next_dn(), lp_layer.a, r.offsets, Mp, out=ybuf,
                                                         out_dtype=q.QARL_OUT_F32, path=q.QARL_PATH_PREFILL,
                                                         ws=lp_layer.ws), 12, 2)
            del ybuf
            fl_gu, fl_dn = 2 * Mp * 2 * I * H, 2 * Mp * H * I
            extra["prefill_w4a16_16384tok_zipf"] = {
                "layer_ms": round(ms_all, 4), "gate_up_ms": round(ms_gu_p, 4), "down_ms": round(ms_dn_p, 4),
                "gemm_TFLOP/s": round((fl_gu + fl_dn) / (ms_gu_p + ms_dn_p) / 1e9, 1),
                "gemm_frac_mfma_bf16": round((fl_gu + fl_dn) / (ms_gu_p + ms_dn_p) / 1e9 / MFMA_BF16_PEAK_TF, 4),
                "layer_TFLOP/s": round((fl_gu + fl_dn) / ms_all / 1e9, 1),
                "max_expert_rows": int(r.counts.max()), "min_expert_rows": int(r.counts.min())}
            lgu = synth.router_logits(Tp, E, seed=32, device=dev)
            ms_all_u = timed(lambda: lp_layer.forward(xp, lgu), 10, 2)
            extra["prefill_w4a16_16384tok_uniform"] = {"layer_ms": round(ms_all_u, 4),
                                                       "layer_TFLOP/s": round((fl_gu + fl_dn) / ms_all_u / 1e9, 1)}

            # (a10, a11) LM head + log-prob on the layer's output
            V = synth.V
            wlm = synth.normal_bf16((V, H), 0.02, seed=40, device=dev)
            tg = synth.targets(Tp, V, seed=41, device=dev)
            ws = torch.empty((q.qarl_logprob_workspace_bytes(Tp, H, V),), dtype=torch.uint8, device=dev)
            hh = lp_layer.out
            ms_lp = timed(lambda: q.qarl_token_logprob(hh, wlm, tg, ws=ws), 3, 1)
            fl_lp = 2 * Tp * H * V
            extra["lm_head_logprob_16384x151936"] = {"ms": round(ms_lp, 3), "TFLOP/s": round(fl_lp / ms_lp / 1e9, 1),
                                                     "frac_mfma_bf16": round(fl_lp / ms_lp / 1e9 / MFMA_BF16_PEAK_TF, 4)}
            # sequence-level surrogate (section 3.2) on the log-probs of that configuration: 8 responses x 2048 tokens.
            # Two small launches over 0.26 MB: launch-bound, reported as time per call.
            Sq, Lq = 8, Tp // 8
            g = torch.Generator(device=dev)
            g.manual_seed(60)
            lp_o = -torch.rand((Tp,), generator=g, device=dev) * 5 - 0.01
            lp_c = lp_o + torch.randn((Tp,), generator=g, device=dev) * 1e-3
            lp_s = lp_o + torch.randn((Tp,), generator=g, device=dev) * 0.05
            so = torch.arange(Sq + 1, dtype=torch.int32, device=dev) * Lq
            adv = torch.randn((Sq,), generator=g, device=dev)
            tb_out = q.qarl_tbpo_objective(lp_c, lp_o, lp_s, so, adv, 1.0, 0.0004, 0.0003, 0.0007, 2.0)
            ms_tb = timed(lambda: q.qarl_tbpo_objective(lp_c, lp_o, lp_s, so, adv, 1.0, 0.0004, 0.0003, 0.0007, 2.0,
                                                        out=tb_out), 50, 5)
            tb_bytes = 4 * Tp * 4
            extra["tbpo_objective_8x2048"] = {"ms": round(ms_tb, 4), "GB/s": round(tb_bytes / ms_tb / 1e6, 1),
                                              "bytes": tb_bytes, "launches": 2}
            del wlm, ws, lp_layer, xp

        if on("backward"):
            # straight-through backward of the gate_up projection at the training-forward shape (16 384 tokens, Zipf):
            # dX = dY What (128 x 128 tiles, 16-bit operands) and dW = dY^T X (256 x 256 tiles)
            Tb = 16384
            Mb = Tb * TOPK
            lgb = synth.router_logits(Tb, E, seed=31, device=dev, zipf_s=1.1)
            rb = q.qarl_moe_route(lgb, TOPK)
            xb = synth.normal_bf16((Tb, H), 1.0, seed=33, device=dev)
            dyb = synth.normal_bf16((Mb, 2 * I), 1.0, seed=34, device=dev)
            dxb = torch.empty((Mb, H), dtype=torch.bfloat16, device=dev)
            dwb = torch.empty((E, 2 * I, H), dtype=torch.bfloat16, device=dev)
            ms_dx = timed(lambda: q.qarl_qgemm_grouped_dx(layers[0].gu, dyb, rb.offsets, Mb, out=dxb), 5, 1)
            ms_dw = timed(lambda: q.qarl_grouped_dw(dyb, xb, rb.offsets, E, row_map=rb.tokens, out=dwb), 5, 1)
            fl_b = 2 * Mb * 2 * I * H
            extra["backward_gate_up_16384tok_zipf"] = {
                "dx_ms": round(ms_dx, 4), "dx_TFLOP/s": round(fl_b / ms_dx / 1e9, 1),
                "dx_frac_mfma_bf16": round(fl_b / ms_dx / 1e9 / MFMA_BF16_PEAK_TF, 4),
                "dw_ms": round(ms_dw, 4), "dw_TFLOP/s": round(fl_b / ms_dw / 1e9, 1),
                "dw_frac_mfma_bf16": round(fl_b / ms_dw / 1e9 / MFMA_BF16_PEAK_TF, 4)}
            del xb, dyb, dxb, dwb, rb

        if on("dense"):
            # a dense SiLU-gated MLP of a second model shape (hidden 4096, intermediate 12288) through the same calls
            Hd, Id, Td = 4096, 12288, 4096
            gud = synth.normal_bf16((1, 2 * Id, Hd), 0.02, seed=70, device=dev)
            dnd = synth.normal_bf16((1, Hd, Id), 0.02, seed=71, device=dev)
            qgud, qdnd = q.qarl_quantize_weights(gud), q.qarl_quantize_weights(dnd)
            del gud, dnd
            xd = synth.normal_bf16((Td, Hd), 1.0, seed=72, device=dev)
            offd = torch.tensor([0, Td], dtype=torch.int32, device=dev)
            ad = torch.empty((Td, Id), dtype=torch.bfloat16, device=dev)
            yd = torch.empty((Td, Hd), dtype=torch.bfloat16, device=dev)
            wsd = torch.empty((max(q.qarl_qgemm_workspace_bytes(qgud, Td, Td, q.QARL_EPI_SILU_MUL),
                                   q.qarl_qgemm_workspace_bytes(qdnd, Td, Td, q.QARL_EPI_NONE), 16),), dtype=torch.uint8, device=dev)
            ms_gud = timed(lambda: q.qarl_qgemm_grouped(qgud, xd, offd, Td, epilogue=q.QARL_EPI_SILU_MUL, out=ad,
                                                        path=q.QARL_PATH_PREFILL, ws=wsd), 10, 2)
            ms_dnd = timed(lambda: q.qarl_qgemm_grouped(qdnd, ad, offd, Td, out=yd, path=q.QARL_PATH_PREFILL, ws=wsd), 10, 2)
            fl_d = 2 * Td * (2 * Id * Hd + Hd * Id)
            extra["dense_mlp_w4a16_4096x12288_4096tok"] = {
                "gate_up_ms": round(ms_gud, 4), "down_ms": round(ms_dnd, 4),
                "TFLOP/s": round(fl_d / (ms_gud + ms_dnd) / 1e9, 1),
                "frac_mfma_bf16": round(fl_d / (ms_gud + ms_dnd) / 1e9 / MFMA_BF16_PEAK_TF, 4)}
            # the same MLP at a decode batch of 64 tokens on the weight-streaming path: gate_up with K = 4096 as it is;
            # the K = 12288 down projection as six K-chunks of 2048, chunk c = expert c, every token listing all six,
            # the activations read as [6 T][2048], the combine (unit weights) adding the six fp32 partial products
            Tdd, KC = 64, 2048
            Cd = Id // KC
            dnd2 = synth.normal_bf16((1, Hd, Id), 0.02, seed=71, device=dev)
            qdnc = q.qarl_quantize_weights(dnd2.view(Hd, Cd, KC).permute(1, 0, 2).contiguous())
            del dnd2
            xdd = xd[:Tdd].contiguous()
            offdd = torch.tensor([0, Tdd], dtype=torch.int32, device=dev)
            add = torch.empty((Tdd, Id), dtype=torch.bfloat16, device=dev)
            ydd = torch.empty((Tdd, Hd), dtype=torch.bfloat16, device=dev)
            idsd = torch.arange(Cd, dtype=torch.int32, device=dev).repeat(Tdd, 1).contiguous()
            onesd = torch.ones((Tdd, Cd), dtype=torch.float32, device=dev)
            wsdd = torch.empty((max(q.qarl_qgemm_workspace_bytes(qdnc, Tdd * Cd, Tdd * Cd, q.QARL_EPI_COMBINE), 16),),
                               dtype=torch.uint8, device=dev)
            ms_gudd = timed(lambda: q.qarl_qgemm_grouped(qgud, xdd, offdd, Tdd, epilogue=q.QARL_EPI_SILU_MUL, out=add,
                                                         path=q.QARL_PATH_DECODE, ws=wsd), 20, 3)
            ms_dndd = timed(lambda: q.qarl_qgemm_routed(qdnc, add.view(Tdd * Cd, KC), idsd, Tdd, Cd, False,
                                                        epilogue=q.QARL_EPI_COMBINE, combine_w=onesd, out=ydd, ws=wsdd), 20, 3)
            wb_gu, wb_dn = weight_bytes_w4a16(1, 2 * Id, Hd), weight_bytes_w4a16(1, Hd, Id)
            extra["dense_mlp_w4a16_4096x12288_decode_64tok"] = {
                "gate_up_ms": round(ms_gudd, 4), "down_ms": round(ms_dndd, 4),
                "gate_up_weight_GB/s": round(wb_gu / ms_gudd / 1e6, 1), "down_weight_GB/s": round(wb_dn / ms_dndd / 1e6, 1),
                "frac_hbm": round((wb_gu + wb_dn) / (ms_gudd + ms_dndd) / 1e6 / HBM_PEAK_GBS, 4),
                "note": "down = 6 K-chunks as experts in routed mode + combine; both weights (75 MB) fit the last-level cache"}
            del qgud, qdnd, qdnc, xd, xdd, ad, add, yd, ydd, wsd, wsdd

        if on("fp8"):
            # FP8 W8A8 layer at 256 and 8192 tokens: the whole layer, and the two grouped GEMM launches on their own
            for (fname, qgu8, qdn8, b8), (T8, path, tag) in [(f, c) for f in lowbit for c in
                                                             ((256, q.QARL_PATH_DECODE, "decode"),
                                                              (8192, q.QARL_PATH_PREFILL, "prefill"))]:
                x8 = synth.normal_bf16((T8, H), 1.0, seed=50, device=dev)
                lg8 = synth.router_logits(T8, E, seed=51, device=dev)
                l8 = q.MoELayer(qgu8, qdn8, T8, TOPK, path, dev)
                ms8 = timed(lambda: l8.forward(x8, lg8), 20, 3)
                r8, M8 = l8.routing, T8 * TOPK
                def copies_of(w):   # enough copies that their codes exceed three times the last-level cache
                    n = max(2, -(-768 * 2 ** 20 // (w.codes.numel() * w.codes.element_size())))
                    return [w] + [clone_qw(w) for _ in range(n - 1)]
                gu_set, dn_set = copies_of(qgu8), copies_of(qdn8)
                next_gu, next_dn = rotate(gu_set), rotate(dn_set)
                if l8.routed:   # decode: the GEMMs read the router's ids and quantize the rows they gather
                    ms8_gu = timed(lambda: q.qarl_qgemm_routed(next_gu(), x8, r8.ids, T8, TOPK, True, epilogue=q.QARL_EPI_SILU_MUL,
                                                               out=l8.a, ws=l8.ws), 20, 3)
                    y8 = torch.empty((M8, H), dtype=torch.float32, device=dev)
                    ms8_dn = timed(lambda: q.qarl_qgemm_routed(next_dn(), l8.a, r8.ids, T8, TOPK, False, out=y8,
                                                               out_dtype=q.QARL_OUT_F32, ws=l8.ws), 20, 3)
                else:
                    ms8_gu = timed(lambda: q.qarl_qgemm_grouped(next_gu(), l8.xq, r8.offsets, M8, row_map=r8.tokens, x_scales=l8.sx,
                                                                epilogue=q.QARL_EPI_SILU_MUL, out=l8.a, path=path,
                                                                ws=l8.ws), 20, 3)
                    y8 = torch.empty((M8, H), dtype=torch.float32, device=dev)
                    ms8_dn = timed(lambda: q.qarl_qgemm_grouped(next_dn(), l8.aq, r8.offsets, M8, x_scales=l8.sa, out=y8,
                                                                out_dtype=q.QARL_OUT_F32, path=path, ws=l8.ws), 20, 3)
                del y8, gu_set, dn_set, next_gu, next_dn
                f8 = synth.flops_moe(T8)
                extra["%s_%s_%dtok" % (fname, tag, T8)] = {
                    "layer_ms": round(ms8, 4), "gate_up_ms": round(ms8_gu, 4), "down_ms": round(ms8_dn, 4),
                    "weight_GB/s": round(b8 / ms8 / 1e6, 1), "frac_hbm": round(b8 / ms8 / 1e6 / HBM_PEAK_GBS, 4),
                    "gemm_weight_GB/s": round(b8 / (ms8_gu + ms8_dn) / 1e6, 1),
                    "gemm_frac_hbm": round(b8 / (ms8_gu + ms8_dn) / 1e6 / HBM_PEAK_GBS, 4),
                    "TFLOP/s": round(f8 / ms8 / 1e9, 1), "frac_mfma_fp8": round(f8 / ms8 / 1e9 / MFMA_FP8_PEAK_TF, 4),
                    "gemm_TFLOP/s": round(f8 / (ms8_gu + ms8_dn) / 1e9, 1),
                    "gemm_frac_mfma_fp8": round(f8 / (ms8_gu + ms8_dn) / 1e9 / MFMA_FP8_PEAK_TF, 4)}
                del l8
        del lowbit, qdn8, outf, outq

        if on("stack"):
            # 48-layer stack: re-quantize every layer after a simulated update, then decode at 512 tokens
            L = args.sweep_layers
            if L > 0:
                T5 = 512
                masters, quant = [], []
                for l in range(L):
                    gu, dn = synth.expert_weights(E, H, I, seed=7000 + 2 * l, device=dev)
                    masters.append((gu, dn))
                    quant.append((q.QWeight.empty(q.QARL_W4A16_G128, E, 2 * I, H, dev),
                                  q.QWeight.empty(q.QARL_W4A16_G128, E, H, I, dev)))
                for l in range(L):   # the simulated update: w += N(0, 1e-4), rounded to bf16
                    masters[l] = (synth.perturb(masters[l][0], 1e-4, 8000 + l), synth.perturb(masters[l][1], 1e-4, 9000 + l))

                def requant():
                    for l in range(L):
                        q.qarl_quantize_weights(masters[l][0], out=quant[l][0])
                        q.qarl_quantize_weights(masters[l][1], out=quant[l][1])
                ms_rq = timed(requant, 3, 1)
                rq_bytes = L * (E * 3 * I * H * 2 + weight_bytes_w4a16(E, 2 * I, H) + weight_bytes_w4a16(E, H, I))
                del masters
                lay5 = [q.MoELayer(quant[l][0], quant[l][1], T5, TOPK, q.QARL_PATH_DECODE, dev) for l in range(L)]
                x5 = [synth.normal_bf16((T5, H), 1.0, seed=60 + l, device=dev) for l in range(4)]
                lg5 = [synth.router_logits(T5, E, seed=70 + l, device=dev) for l in range(4)]

                def sweep():
                    for l in range(L):
                        lay5[l].forward(x5[l % 4], lg5[l % 4])
                ms_sw = timed(sweep, 5, 1)

                # the two GEMM calls of the sweep on their own (ids of the last pass; down includes its combine launch)
                def sweep_gu():
                    for l in range(L):
                        ly = lay5[l]
                        q.qarl_qgemm_routed(ly.gu, x5[l % 4], ly.routing.ids, T5, TOPK, True,
                                            epilogue=q.QARL_EPI_SILU_MUL, out=ly.a, ws=ly.ws)

                def sweep_dn():
                    for l in range(L):
                        ly = lay5[l]
                        q.qarl_qgemm_routed(ly.dn, ly.a, ly.routing.ids, T5, TOPK, False, epilogue=q.QARL_EPI_COMBINE,
                                            combine_w=ly.routing.w, out=ly.out, ws=ly.ws)
                ms_sw_gu = timed(sweep_gu, 5, 1) / L
                ms_sw_dn = timed(sweep_dn, 5, 1) / L
                sw_bytes = L * (weight_bytes_w4a16(E, 2 * I, H) + weight_bytes_w4a16(E, H, I))
                extra["stack_requantize_%dlayers" % L] = {"ms": round(ms_rq, 3), "GB/s": round(rq_bytes / ms_rq / 1e6, 1),
                                                          "frac_hbm": round(rq_bytes / ms_rq / 1e6 / HBM_PEAK_GBS, 4)}
                extra["stack_decode_sweep_%dlayers_512tok" % L] = {
                    "ms": round(ms_sw, 3), "weight_GB/s": round(sw_bytes / ms_sw / 1e6, 1),
                    "frac_hbm": round(sw_bytes / ms_sw / 1e6 / HBM_PEAK_GBS, 4),
                    "TFLOP/s": round(L * synth.flops_moe(T5) / ms_sw / 1e9, 1),
                    "ms_per_layer": round(ms_sw / L, 5), "gate_up_ms_per_layer": round(ms_sw_gu, 5),
                    "down_combine_ms_per_layer": round(ms_sw_dn, 5)}
        result["extra"] = extra

    print(json.dumps(result))


if __name__ == "__main__":
    main()
