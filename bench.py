#!/usr/bin/env python3
"""Benchmark of the BitNet a4.8 quantized linears on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: the five
projections of a 7B block at prefill size (4 sequences x 4096 tokens = 16384 tokens), each as
"quantize activations, then ternary GEMM":
    qkv  4096 -> 12288  INT4 absmean                (W1.58A4)
    o    4096 ->  4096  top-50% + INT8 absmax       (sparse W1.58A8)
    gate 4096 -> 11008  INT4, up 4096 -> 11008 INT4 (W1.58A4)
    down 11008 -> 4096  top-50% + INT8              (sparse W1.58A8)
All inputs and packed weights are resident in HBM before the timed region.  `value` is
dense-equivalent int8 TOPS (2*M*N*K per projection) over the whole step, quantize kernels
included.  The roofline object covers the dominant kernel, the W1.58A4 prefill GEMM, timed
with events on the launch stream inside the timed region.  Decode-shape weight bandwidth
(packed-weight GB/s at 1/8/32/64 tokens) is reported in the same JSON line under "decode", and
the FP4 activation variant against the INT4 path at 3B-like shapes under "fp4_variant"; one
token through a whole FFN block, four calls against the gate-first form, under "decode_ffn_1token";
the per-head quantizer of the attention states (Section 4.2) at 7B width under "attention_states".
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

EPS = 1e-5
INT8_PEAK_TOPS = 5033.0      # MI355X dense int8 MFMA
FP6_FP4_PEAK_TOPS = 10066.0  # MI355X dense fp6 / fp4 MFMA (the INT4 GEMM runs on E3M2 x E2M1 operands)
HBM_PEAK_GBS = 8000.0
# Bytes between L2 and the memory fabric per launch of the W1.58A4 prefill GEMM at the benchmark
# shapes, from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in
# profiles/gemm_7b_prefill_hbm_traffic.txt (calibrated against a 1 GiB device copy):
# 490.2 MB fetched + 374.7 MB written (2-bit weights; 677.6 MB fetched with E2M1 nibbles).
A4_GEMM_TRAFFIC_BYTES = 864.9e6
HIDDEN, FFN = 4096, 11008


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-fp4", action="store_true")
    ap.add_argument("--a4-weights", choices=["mx2", "mx4"], default="mx2",
                    help="block-float weight form of the INT4 projections: 2-bit codes expanded in registers, or E2M1 nibbles")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for the HBM traffic counters)")
    return ap.parse_args()


def cpu_baseline(sample_tokens=128):
    """The oracle, as it stands, on a bounded sample: the qkv projection (INT4 quantize,
    integer matmul, rescale) for `sample_tokens` tokens at full N and K."""
    from oracle import bitnet_a48 as O
    from paper_2411_04965_amd import synth as S
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    N, K = 3 * HIDDEN, HIDDEN
    W = S.latent_weights(N, K, S.seed_for(3, 10))
    T, alpha = O.ternarize(W, EPS)
    X = S.heavy(sample_tokens, K, S.seed_for(3, 11))
    t0 = time.perf_counter()
    reps = 0
    while True:
        q, d = O.quant_int4(X, EPS)
        acc = O.matmul_int(q, T)
        O.rescale(acc, d, alpha, "bf16")
        reps += 1
        if time.perf_counter() - t0 > 10.0 or reps >= 20:
            break
    dt = (time.perf_counter() - t0) / reps
    tops = 2.0 * sample_tokens * N * K / dt / 1e12
    return {"value": tops, "unit": "TOPS", "cores": int(cores), "kind": "oracle",
            "sample": "qkv 4096->12288, %d tokens (quant_int4 + matmul_int + rescale), %d reps, %.3f s each"
                      % (sample_tokens, reps, dt)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU path exists.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2411_04965_amd import binding as B
    from paper_2411_04965_amd import synth as S

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    M = args.tokens
    bf16 = torch.bfloat16

    def to_dev(x):
        return torch.from_numpy(x).to(dev).to(bf16).contiguous()

    # ---- weights (packed once, offline step) and inputs, resident in HBM
    A4L = B.BL_W_MX2 if args.a4_weights == "mx2" else B.BL_W_MX4
    projs = S.projections(HIDDEN, FFN)
    W = {}
    for i, (name, N, K, kind) in enumerate(projs):
        w = torch.from_numpy(S.latent_weights(N, K, S.seed_for(3, 20 + i))).to(dev)
        # INT4 projections: block-float layout (E2M1 nibbles) for the 6-bit x 4-bit matrix instruction
        W[name] = B.pack_ternary(w, EPS, A4L if kind == "a4" else B.BL_W_GEMM)
        del w
    x_hidden = to_dev(S.heavy(M, HIDDEN, S.seed_for(3, 1)))
    x_attn = to_dev(S.heavy(M, HIDDEN, S.seed_for(3, 3)))
    x_down = to_dev(S.glu_like(M, FFN, S.seed_for(3, 2)))
    inputs = {"qkv": x_hidden, "o": x_attn, "gate": x_hidden, "up": x_hidden, "down": x_down}

    # preallocated outputs / code buffers (no allocation inside the timed region)
    bufs = {}
    for name, N, K, kind in projs:
        mode = B.BL_ACT_INT4_ABSMEAN_MX6 if kind == "a4" else B.BL_ACT_TOPK_INT8_ABSMAX
        L = B.lib()
        bufs[name] = dict(
            mode=mode, layout=A4L if kind == "a4" else B.BL_W_GEMM,
            q=torch.empty(L.quantize_act_bytes(mode, M, K), dtype=torch.uint8, device=dev),
            scale=torch.empty(M, dtype=torch.float32, device=dev),
            Y=torch.empty((M, N), dtype=bf16, device=dev),
            ws=B.workspace(mode, M, N, K, dev))
    stream = torch.cuda.current_stream().cuda_stream
    L = B.lib()

    gemm_events = {name: [] for name, *_ in projs}
    quant_events = {name: [] for name, *_ in projs}

    def step(record):
        for name, N, K, kind in projs:
            b = bufs[name]
            X = inputs[name]
            topk = K // 2 if kind == "a8s" else 0
            if record:
                e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
                e0.record()
            if name == "up":
                # gate and up read the same tensor: it is quantized once (by "gate") and used twice
                b = dict(b, q=bufs["gate"]["q"], scale=bufs["gate"]["scale"])
            else:
                rc = L.quantize_act(X.data_ptr(), B.BL_BF16, M, K, b["mode"], topk, EPS,
                                    b["q"].data_ptr(), b["scale"].data_ptr(), None, None, stream)
                assert rc == 0, rc
            if record:
                e1.record()
            rc = L.bitlinear_gemm(b["q"].data_ptr(), b["scale"].data_ptr(), b["mode"], M, K,
                                  W[name][0].data_ptr(), b["layout"], W[name][1].data_ptr(), N,
                                  b["Y"].data_ptr(), B.BL_BF16, None, b["ws"].data_ptr(),
                                  b["ws"].numel(), stream)
            assert rc == 0, rc
            if record:
                e2.record()
                quant_events[name].append((e0, e1))
                gemm_events[name].append((e1, e2))

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)              # 1 GiB read + 1 GiB written per launch
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ops_per_step = sum(2.0 * M * N * K for _, N, K, _ in projs)
    value = ops_per_step / (ms_per_step * 1e-3) / 1e12

    per_kernel = {}
    for name, N, K, kind in projs:
        g = float(np.mean([a.elapsed_time(b) for a, b in gemm_events[name]]))
        qd = float(np.mean([a.elapsed_time(b) for a, b in quant_events[name]]))
        in_b = M * K * 2
        out_b = M * bl_code_bytes(kind, K) + 4 * M
        per_kernel[name] = {"gemm_ms": round(g, 4), "gemm_tops": round(2.0 * M * N * K / g / 1e9, 1),
                            "quant_ms": round(qd, 4),
                            "quant_gbs": None if name == "up" else round((in_b + out_b) / qd / 1e6, 1)}
    # dominant kernel: the W1.58A4 prefill GEMM (qkv, gate, up launches)
    a4 = [(n_, N, K) for n_, N, K, kind in projs if kind == "a4"]
    a4_ops = sum(2.0 * M * N * K for _, N, K in a4)
    a4_ms = sum(per_kernel[n_]["gemm_ms"] for n_, _, _ in a4)
    achieved = a4_ops / (a4_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "gemm_a4_mx_kernel (qkv, gate, up): E3M2 x E2M1 block-float MFMA, weights "
                          + ("2-bit in HBM and LDS" if args.a4_weights == "mx2" else "E2M1 nibbles in HBM and LDS"),
                "achieved": round(achieved, 1), "peak": FP6_FP4_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(achieved / FP6_FP4_PEAK_TOPS, 4),
                "frac_of_int8_peak": round(achieved / INT8_PEAK_TOPS, 4),
                "traffic": A4_GEMM_TRAFFIC_BYTES if (M == 16384 and args.a4_weights == "mx2") else None,
                "algorithmic_bytes": round(sum(M * K * 3 / 4 + N * K / (4 if args.a4_weights == "mx2" else 2) + 2 * M * N
                                               for _, N, K in a4) / len(a4)),
                "avg_launch_ms": round(a4_ms / len(a4), 4)}

    out = {
        "metric": "W1.58A4 linear TOPS (prefill) & packed-weight GB/s (decode), 7B shapes",
        "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8+fp6xfp4",
        "data": "synthetic (seeded; N(0,1) + heavy-tailed outlier channels, bf16)",
        "config": {"workload": "7B prefill block: %d tokens x {qkv 4096->12288 A4, o 4096->4096 A8s, "
                               "gate/up 4096->11008 A4 (one shared quantized input), down 11008->4096 A8s}, "
                               "quantize + GEMM" % M,
                   "tokens": M},
        "roofline": roofline,
        "kernels": per_kernel,
    }
    if not args.no_decode:
        out["decode"] = decode_bench(B, S, torch, dev)
        out["decode_ffn_1token"] = decode_ffn_bench(B, S, torch, dev)
    if not args.no_fp4:
        out["fp4_variant"] = fp4_compare(B, S, torch, dev)
    out["attention_states"] = heads_bench(B, S, torch, dev, M)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


def decode_ffn_bench(B, S, torch, dev, layers=8, replays=20):
    """One token through the FFN's three linears and its glue at 7B width, from HIP-graph replays of
    `layers` distinct weight sets: gate, up, ReLU^2 GLU, down as four calls against the gate-first
    form (gate, then the up projection only where the gate is open with the GLU inside, then down)."""
    bf16 = torch.bfloat16
    X = torch.from_numpy(S.heavy(1, HIDDEN, S.seed_for(2, 900))).to(dev).to(bf16)
    sets = []
    for l in range(layers):
        ws_ = []
        for i, (N, K) in enumerate(((FFN, HIDDEN), (FFN, HIDDEN), (HIDDEN, FFN))):
            w = torch.from_numpy(S.latent_weights(N, K, S.seed_for(2, 2000 + 10 * l + i))).to(dev)
            ws_.append(B.pack_ternary(w, EPS, B.BL_W_GEMM))
            if i == 1:
                ws_.append(B.pack_ternary(w, EPS, B.BL_W_ROWS))
            del w
        sets.append(ws_)
    ws4 = B.workspace(B.BL_ACT_INT4_ABSMEAN, 1, FFN, HIDDEN, dev)
    ws8 = B.workspace(B.BL_ACT_TOPK_INT8_ABSMAX, 1, HIDDEN, FFN, dev)
    G = torch.empty((1, FFN), dtype=torch.float32, device=dev)
    U = torch.empty((1, FFN), dtype=torch.float32, device=dev)
    Y = torch.empty((1, HIDDEN), dtype=bf16, device=dev)

    def dense(l):
        (pg, ag), (pu, au), _, (pd, ad) = sets[l]
        B.bitlinear_a4(X, pg, ag, FFN, EPS, ws=ws4, out=G)
        B.bitlinear_a4(X, pu, au, FFN, EPS, ws=ws4, out=U)
        Hh = B.relu2_glu(G, U)
        B.bitlinear_a8_sparse(Hh, FFN // 2, pd, ad, HIDDEN, EPS, ws=ws8, out=Y)

    def gate_first(l):
        (pg, ag), _, (pr, ar), (pd, ad) = sets[l]
        B.bitlinear_a4(X, pg, ag, FFN, EPS, ws=ws4, out=G)
        Hh = B.bitlinear_a4_up_gated(X, pr, ar, FFN, G, EPS)
        B.bitlinear_a8_sparse(Hh, FFN // 2, pd, ad, HIDDEN, EPS, ws=ws8, out=Y)

    res = {}
    side = torch.cuda.Stream()
    for name, fn in (("four_calls", dense), ("gate_first", gate_first)):
        for l in range(layers):
            fn(l)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for l in range(layers):
                    fn(l)
        g.replay()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        res[name + "_us"] = round(e0.elapsed_time(e1) / (replays * layers) * 1e3, 2)
        del g
    res["open_gate_fraction"] = round(float((G > 0).float().mean().item()), 3)
    return res


def heads_bench(B, S, torch, dev, T, H=32, D=128, iters=20):
    """Per-head absmax quantizer of the attention states (Section 4.2) on one projection's worth of
    heads at 7B width: T tokens x 32 heads x 128 channels of bfloat16, to 4 and to 3 bits.  GB/s over
    the algorithmic bytes (2 D in, D bits / 8 + 4 out per head).  The calls rotate over four input
    tensors (0.5 GB together) so that none of them is still in the 256 MB memory-side cache when
    its turn comes again."""
    Xs = [torch.from_numpy(S.heavy(T, H * D, S.seed_for(5, 1 + i))).to(dev).to(torch.bfloat16).reshape(T, H, D)
          for i in range(4)]
    res = {"tokens": T, "heads": H, "head_dim": D}
    for bits in (4, 3):
        for i in range(4):
            B.quantize_heads(Xs[i], bits, EPS)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            B.quantize_heads(Xs[i % 4], bits, EPS)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        nbytes = T * H * (2 * D + D * bits // 8 + 4)
        res["bits%d" % bits] = {"ms": round(ms, 4), "gbs": round(nbytes / ms / 1e6, 1),
                                "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 3)}
    return res


def fp4_compare(B, S, torch, dev, M=8192, hidden=3200, ffn=8640, iters=20):
    """The FP4 (E2M1 + E8M0 per 32 channels) activation variant against the INT4 path on identical
    seeded inputs at 3B-like shapes: quantizer + GEMM per projection, dense TOPS."""
    res = {"tokens": M}
    for name, N, K in (("qkv", 3 * hidden, hidden), ("gate", ffn, hidden)):
        w = torch.from_numpy(S.latent_weights(N, K, S.seed_for(4, 20 + len(name)))).to(dev)
        # each path with the weight form it runs fastest on (measured): 2-bit codes for INT4, E2M1
        # nibbles for FP4, whose scaled MFMA leaves less room for the expansion arithmetic
        packed = {lay: B.pack_ternary(w, EPS, lay) for lay in (B.BL_W_MX2, B.BL_W_MX4)}
        del w
        X = torch.from_numpy(S.heavy(M, K, S.seed_for(4, 21))).to(dev).to(torch.bfloat16)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        row = {}
        for label, fp4, mode, lay in (("fp4", True, B.BL_ACT_FP4_E2M1_B32_MX, B.BL_W_MX4),
                                      ("int4", False, B.BL_ACT_INT4_ABSMEAN_MX6, B.BL_W_MX2)):
            p, a = packed[lay]
            ws = B.workspace(mode, M, N, K, dev)
            for _ in range(3):
                B.bitlinear_a4(X, p, a, N, EPS, act_fp4=fp4, ws=ws, out=Y, layout=lay)
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                B.bitlinear_a4(X, p, a, N, EPS, act_fp4=fp4, ws=ws, out=Y, layout=lay)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / iters
            row[label] = {"ms": round(ms, 4), "tops": round(2.0 * M * N * K / ms / 1e9, 1),
                          "weights": "mx4" if lay == B.BL_W_MX4 else "mx2"}
        res[name] = row
    return res


def bl_code_bytes(kind, K):
    Kp = (K + 255) // 256 * 256
    return Kp * 3 // 4 if kind == "a4" else Kp      # 6-bit codes / int8


def decode_bench(B, S, torch, dev, layers=8, replays=20):
    """Packed-weight bandwidth at decode shapes.  `layers` distinct weight sets per projection
    (more than the 256 MB last-level cache holds in total) are run back to back from one HIP
    graph per projection, so launch overhead of the Python binding is not in the timing."""
    res = {}
    bf16 = torch.bfloat16
    projs = S.projections(HIDDEN, FFN)
    packed = {}
    for i, (name, N, K, kind) in enumerate(projs):
        sets = []
        for l in range(layers):
            w = torch.from_numpy(S.latent_weights(N, K, S.seed_for(2, 1000 + 10 * l + i))).to(dev)
            sets.append(B.pack_ternary(w, EPS, B.BL_W_GEMM))
            del w
        packed[name] = sets
    side = torch.cuda.Stream()
    for M in (1, 8, 32, 64):
        row = {}
        tot_bytes, tot_ms = 0.0, 0.0
        for name, N, K, kind in projs:
            X = torch.from_numpy(S.glu_like(M, K, S.seed_for(2, 200 + M)) if name == "down"
                                 else S.heavy(M, K, S.seed_for(2, 100 + M))).to(dev).to(bf16)
            mode = B.BL_ACT_INT4_ABSMEAN if kind == "a4" else B.BL_ACT_TOPK_INT8_ABSMAX
            ws = B.workspace(mode, M, N, K, dev)
            Y = torch.empty((M, N), dtype=bf16, device=dev)

            def run(l):
                p, a = packed[name][l % layers]
                if kind == "a4":
                    B.bitlinear_a4(X, p, a, N, EPS, ws=ws, out=Y)
                else:
                    B.bitlinear_a8_sparse(X, K // 2, p, a, N, EPS, ws=ws, out=Y)
            for l in range(layers):
                run(l)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for l in range(layers):
                        run(l)
            g.replay()
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(replays):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / (replays * layers)
            wbytes = N * K / 4
            row[name] = {"us": round(ms * 1e3, 2), "weight_gbs": round(wbytes / ms / 1e6, 1)}
            tot_bytes += wbytes
            tot_ms += ms
            del g
        row["layer_weight_gbs"] = round(tot_bytes / tot_ms / 1e6, 1)
        row["frac_hbm_peak"] = round(tot_bytes / tot_ms / 1e6 / HBM_PEAK_GBS, 4)
        res["M%d" % M] = row
    return res


if __name__ == "__main__":
    main()
