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
BF16_PEAK_TFLOPS = 2516.0    # MI355X dense bfloat16 MFMA (the gradient GEMMs of the backward pass)
HIDDEN, FFN = 4096, 11008
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemm_7b_prefill_hbm_traffic.txt")


def measured_traffic_bytes():
    """Bytes between L2 and the memory fabric per launch of the W1.58A4 prefill GEMM at the
    benchmark's shapes, as the rocprofv3 FETCH_SIZE / WRITE_SIZE runs measured them (counters cannot
    be read from inside this process): the line `roofline_traffic_bytes_per_launch: <bytes>` of the
    committed summary of those runs, or None if the summary is absent."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("roofline_traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-prefill", action="store_true",
                    help="skip the timed prefill step (profiling the decode sweep alone); the line then has value 0")
    ap.add_argument("--decode-tokens", type=int, nargs="*", default=[1, 8, 32, 64])
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-fp4", action="store_true")
    ap.add_argument("--no-probe", action="store_true", help="skip the operand-data probe of the qkv GEMM")
    ap.add_argument("--step-only", action="store_true",
                    help="time the prefill step and nothing else (for counter runs: every launch of the process is then "
                         "one of the step's eight kernels)")
    ap.add_argument("--probe-only", action="store_true",
                    help="run only the operand-data probe (for a counter run: its launches are then the only "
                         "block-float GEMM launches of the process, 23 per operand setting, in order)")
    ap.add_argument("--a4-weights", choices=["mx2", "mx4"], default="mx2",
                    help="block-float weight form of the INT4 projections: 2-bit codes expanded in registers, or E2M1 nibbles")
    ap.add_argument("--ffn", choices=["fused", "separate"], default="fused",
                    help="gate and up projection as one GEMM with the ReLU^2 GLU in its epilogue (H written), or as two GEMMs (G and U written)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for the HBM traffic counters)")
    return ap.parse_args()


def cpu_baseline(sample_tokens=1024):
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
        if time.perf_counter() - t0 > 12.0 or reps >= 200:
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
    fused = args.ffn == "fused"
    H_ffn = torch.empty((M, FFN), dtype=bf16, device=dev)
    ws_gu = torch.empty(max(L.bitlinear_gate_up_workspace_bytes(M, FFN, HIDDEN, A4L), 16), dtype=torch.uint8, device=dev)
    # the step's launches: with the fused FFN front, gate and up are one entry (N = both widths)
    launches = ([("qkv", 3 * HIDDEN, HIDDEN, "a4"), ("o", HIDDEN, HIDDEN, "a8s"), ("gate_up", 2 * FFN, HIDDEN, "a4"),
                 ("down", HIDDEN, FFN, "a8s")] if fused else projs)

    # events of the timed steps exist before the timed region: recording one is all that is left in it
    n_timed = 0 if args.no_prefill else args.steps
    pool = [[tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in launches] for _ in range(n_timed)]
    gemm_events = {name: [] for name, *_ in launches}
    quant_events = {name: [] for name, *_ in launches}

    def step(record, it=0):
        for pi, (name, N, K, kind) in enumerate(launches):
            b = bufs["gate" if name == "gate_up" else name]
            X = inputs["gate" if name == "gate_up" else name]
            topk = K // 2 if kind == "a8s" else 0
            if record:
                e0, e1, e2 = pool[it][pi]
                e0.record()
            if name == "gate_up":
                # eq. 7 once, then one GEMM over both weight matrices whose epilogue applies eq. 5: H only
                rc = L.quantize_act(X.data_ptr(), B.BL_BF16, M, K, b["mode"], 0, EPS,
                                    b["q"].data_ptr(), b["scale"].data_ptr(), None, None, stream)
                assert rc == 0, rc
                if record:
                    e1.record()
                rc = B.gemm_a4_glu_prequantized(L, b["q"], b["scale"], M, K, W["gate"], W["up"], A4L, FFN, H_ffn, stream)
                assert rc == 0, rc
                if record:
                    e2.record()
                    quant_events[name].append((e0, e1))
                    gemm_events[name].append((e1, e2))
                continue
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

    if args.probe_only:
        b = bufs["qkv"]
        rc = L.quantize_act(x_hidden.data_ptr(), B.BL_BF16, M, HIDDEN, b["mode"], 0, EPS, b["q"].data_ptr(),
                            b["scale"].data_ptr(), None, None, stream)
        assert rc == 0, rc
        bo = bufs["o"]
        rc = L.quantize_act(x_attn.data_ptr(), B.BL_BF16, M, HIDDEN, bo["mode"], HIDDEN // 2, EPS, bo["q"].data_ptr(),
                            bo["scale"].data_ptr(), None, None, stream)
        assert rc == 0, rc
        print(json.dumps({"operand_data_probe": {
            "qkv_block_float_gemm": operand_data_probe(B, L, torch, M, 3 * HIDDEN, HIDDEN, b, W["qkv"], A4L, stream),
            "o_int8_gemm": operand_data_probe(B, L, torch, M, HIDDEN, HIDDEN, bo, W["o"], B.BL_W_GEMM, stream)}}))
        return

    if args.no_prefill:
        out = {"metric": "W1.58A4 linear TOPS (prefill) & packed-weight GB/s (decode), 7B shapes", "value": 0.0,
               "unit": "TOPS", "n_gpus": 1, "steps": 0, "warmup": 0, "ms_per_step": 0.0, "higher_is_better": True,
               "scaling": "weak", "vs_baseline": None, "dtype": "int8+fp6xfp4", "data": "synthetic",
               "config": {"workload": "decode sweep only (--no-prefill): not a benchmark result"}}
        out["decode"] = decode_bench(B, S, torch, dev, tokens=tuple(args.decode_tokens))
        print(json.dumps(out))
        return

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(args.steps):
        step(True, it)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ops_per_step = sum(2.0 * M * N * K for _, N, K, _ in projs)
    value = ops_per_step / (ms_per_step * 1e-3) / 1e12

    per_kernel = {}
    for name, N, K, kind in launches:
        g = float(np.mean([a.elapsed_time(b) for a, b in gemm_events[name]]))
        qd = float(np.mean([a.elapsed_time(b) for a, b in quant_events[name]]))
        in_b = M * K * 2
        out_b = M * bl_code_bytes(kind, K) + 4 * M
        per_kernel[name] = {"gemm_ms": round(g, 4), "gemm_tops": round(2.0 * M * N * K / g / 1e9, 1),
                            "quant_ms": round(qd, 4),
                            "quant_gbs": None if name == "up" else round((in_b + out_b) / qd / 1e6, 1)}
    # dominant kernel: the W1.58A4 prefill GEMM (qkv, gate, up launches; gate and up as one launch
    # with the GLU epilogue when fused)
    a4 = [(n_, N, K) for n_, N, K, kind in launches if kind == "a4"]
    a4_ops = sum(2.0 * M * N * K for _, N, K in a4)
    a4_ms = sum(per_kernel[n_]["gemm_ms"] for n_, _, _ in a4)
    achieved = a4_ops / (a4_ms * 1e-3) / 1e12
    def out_bytes(n_, N):                       # bf16 outputs: H alone for the fused gate/up launch
        return 2 * M * (N // 2 if n_ == "gate_up" else N)
    roofline = {"bound": "mfma", "kernel": "gemm_a4_mx_kernel (%s): E3M2 x E2M1 block-float MFMA, weights "
                          % ("qkv; gate + up with the GLU epilogue" if fused else "qkv, gate, up")
                          + ("2-bit in HBM and LDS" if args.a4_weights == "mx2" else "E2M1 nibbles in HBM and LDS"),
                "achieved": round(achieved, 1), "peak": FP6_FP4_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(achieved / FP6_FP4_PEAK_TOPS, 4),
                "frac_of_int8_peak": round(achieved / INT8_PEAK_TOPS, 4),
                "traffic": measured_traffic_bytes() if (M == 16384 and args.a4_weights == "mx2") else None,
                # what the method itself has to move per launch: 4-bit codes, 2-bit weights, bf16 outputs
                "algorithmic_bytes": round(sum(M * K / 2 + N * K / 4 + out_bytes(n_, N) for n_, N, K in a4) / len(a4)),
                # what this kernel's formats move: the INT4 levels travel as 6-bit E3M2 codes
                "format_bytes": round(sum(M * K * 3 / 4 + N * K / (4 if args.a4_weights == "mx2" else 2) + out_bytes(n_, N)
                                          for n_, N, K in a4) / len(a4)),
                "avg_launch_ms": round(a4_ms / len(a4), 4)}

    out = {
        "metric": "W1.58A4 linear TOPS (prefill) & packed-weight GB/s (decode), 7B shapes",
        "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8+fp6xfp4",
        "data": "synthetic (seeded; N(0,1) + heavy-tailed outlier channels, bf16)",
        "config": {"workload": "7B prefill block: %d tokens x {qkv 4096->12288 A4, o 4096->4096 A8s, "
                               "gate/up 4096->11008 A4 (one shared quantized input%s), down 11008->4096 A8s}, "
                               "quantize + GEMM" % (M, "; one GEMM, ReLU^2 GLU in its epilogue, H written" if fused else ""),
                   "tokens": M, "ffn_front": args.ffn},
        "roofline": roofline,
        "kernels": per_kernel,
    }
    if args.step_only:
        print(json.dumps(out))
        return
    out["ffn_front"] = ffn_front_bench(B, L, torch, M, x_hidden, bufs["gate"], W, A4L, H_ffn, stream)
    if not args.no_probe:
        out["operand_data_probe"] = {
            "qkv_block_float_gemm": operand_data_probe(B, L, torch, M, 3 * HIDDEN, HIDDEN, bufs["qkv"], W["qkv"], A4L, stream),
            "o_int8_gemm": operand_data_probe(B, L, torch, M, HIDDEN, HIDDEN, bufs["o"], W["o"], B.BL_W_GEMM, stream)}
    if not args.no_decode:
        out["decode"] = decode_bench(B, S, torch, dev, tokens=tuple(args.decode_tokens))
        out["decode_ffn_1token"] = decode_ffn_bench(B, S, torch, dev)
    if not args.no_fp4:
        out["fp4_variant"] = fp4_compare(B, S, torch, dev)
    out["attention_states"] = heads_bench(B, S, torch, dev, M)
    out["ste_backward"] = ste_backward_bench(B, S, torch, dev, M)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


def ffn_front_bench(B, L, torch, M, X, b, W, A4L, H, stream, iters=20):
    """From the input of an FFN block to the quantized input of its down projection, two ways on the same
    buffers: (a) gate GEMM, up GEMM (G and U written as bfloat16), then the Top_k + INT8 quantizer
    that forms eq. 5 while it loads G and U; (b) one GEMM over both weight matrices with eq. 5 in its
    epilogue (H written), then the Top_k + INT8 quantizer on H.  The INT4 quantizer of the input is
    common to both and left out."""
    dev = X.device
    G = torch.empty((M, FFN), dtype=torch.bfloat16, device=dev)
    U = torch.empty((M, FFN), dtype=torch.bfloat16, device=dev)
    q8 = torch.empty(L.quantize_act_bytes(B.BL_ACT_TOPK_INT8_ABSMAX, M, FFN), dtype=torch.uint8, device=dev)
    s8 = torch.empty(M, dtype=torch.float32, device=dev)
    rc = L.quantize_act(X.data_ptr(), B.BL_BF16, M, HIDDEN, b["mode"], 0, EPS, b["q"].data_ptr(),
                        b["scale"].data_ptr(), None, None, stream)
    assert rc == 0

    def three():
        for name, Y in (("gate", G), ("up", U)):
            rc = L.bitlinear_gemm(b["q"].data_ptr(), b["scale"].data_ptr(), b["mode"], M, HIDDEN, W[name][0].data_ptr(),
                                  A4L, W[name][1].data_ptr(), FFN, Y.data_ptr(), B.BL_BF16, None, None, 0, stream)
            assert rc == 0, rc
        rc = L.quantize_act_glu(G.data_ptr(), U.data_ptr(), B.BL_BF16, M, FFN, FFN // 2, EPS, q8.data_ptr(),
                                s8.data_ptr(), None, stream)
        assert rc == 0, rc

    def fused():
        rc = B.gemm_a4_glu_prequantized(L, b["q"], b["scale"], M, HIDDEN, W["gate"], W["up"], A4L, FFN, H, stream)
        assert rc == 0, rc
        rc = L.quantize_act(H.data_ptr(), B.BL_BF16, M, FFN, B.BL_ACT_TOPK_INT8_ABSMAX, FFN // 2, EPS, q8.data_ptr(),
                            s8.data_ptr(), None, None, stream)
        assert rc == 0, rc

    res = {}
    for label, fn in (("two_gemms_then_glu_quantizer_ms", three), ("glu_gemm_then_quantizer_ms", fused)):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[label] = round(e0.elapsed_time(e1) / iters, 4)
    res["bytes_written_and_reread_between"] = {"two_gemms": 2 * 2 * M * FFN * 2, "glu_gemm": 2 * M * FFN * 2}
    return res


def operand_data_probe(B, L, torch, M, N, K, b, Wq, layout, stream, iters=20):
    """One GEMM of the step timed on its real operands, then with the activation codes zeroed, then with
    the weights zeroed too.  The kernel executes the same instructions on the same addresses in all three
    (no branch depends on a code or a weight), so a shorter time can only come from a higher clock: the
    matrix units draw less power when their operands do not toggle."""
    q0 = b["q"].clone()
    w0 = Wq[0].clone()
    Y = b["Y"]

    def run(q, w):
        rc = L.bitlinear_gemm(q.data_ptr(), b["scale"].data_ptr(), b["mode"], M, K, w.data_ptr(), layout,
                              Wq[1].data_ptr(), N, Y.data_ptr(), B.BL_BF16, None, b["ws"].data_ptr(),
                              b["ws"].numel(), stream)
        assert rc == 0, rc

    res = {}
    for label, zq, zw in (("real_operands_ms", False, False), ("zero_codes_ms", True, False),
                          ("zero_codes_zero_weights_ms", True, True)):
        if zq:
            q0.zero_()
        if zw:
            w0.zero_()
        for _ in range(3):
            run(q0, w0)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            run(q0, w0)
        e1.record()
        torch.cuda.synchronize()
        res[label] = round(e0.elapsed_time(e1) / iters, 4)
    res["tops_real"] = round(2.0 * M * N * K / res["real_operands_ms"] / 1e9, 1)
    res["tops_zero"] = round(2.0 * M * N * K / res["zero_codes_zero_weights_ms"] / 1e9, 1)
    return res


def ste_backward_bench(B, S, torch, dev, M, iters=5):
    """Straight-through backward (Section 2.2) of the qkv projection at the step's token count: the two
    gradient GEMMs on bfloat16 operands with their operand preparation (weights expanded from 2 bits,
    dY scaled and transposed, codes transposed), timed apart."""
    N, K = 3 * HIDDEN, HIDDEN
    L = B.lib()
    w = torch.from_numpy(S.latent_weights(N, K, S.seed_for(3, 70))).to(dev)
    pk, ak = B.pack_ternary(w, EPS, B.BL_W_KMAJOR)
    del w
    X = torch.from_numpy(S.heavy(M, K, S.seed_for(3, 71))).to(dev).to(torch.bfloat16)
    qa = B.quantize_act(X, B.BL_ACT_INT4_ABSMEAN, 0, EPS)
    dY = (torch.randn((M, N), device=dev) * 0.01).to(torch.bfloat16)
    ws = torch.empty(L.bitlinear_backward_workspace_bytes(M, N, K), dtype=torch.uint8, device=dev)
    res = {"shape": "dY %d x %d, K = %d" % (M, N, K)}
    for label, dx, dw in (("dX", True, False), ("dW", False, True)):
        for _ in range(2):
            B.bitlinear_backward(dY, qa["q"], qa["scale"], B.BL_ACT_INT4_ABSMEAN, K, pk, ak, dx, dw, ws=ws)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            B.bitlinear_backward(dY, qa["q"], qa["scale"], B.BL_ACT_INT4_ABSMEAN, K, pk, ak, dx, dw, ws=ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        res[label + "_ms"] = round(ms, 3)
        res[label + "_tflops"] = round(2.0 * M * N * K / ms / 1e9, 1)
        res[label + "_frac_of_bf16_peak"] = round(2.0 * M * N * K / ms / 1e9 / BF16_PEAK_TFLOPS, 3)
    return res


def decode_ffn_bench(B, S, torch, dev, layers=8, replays=20):
    """One token through the FFN's three linears and its glue at 7B width, from HIP-graph replays of
    `layers` distinct weight sets: gate, up, ReLU^2 GLU, down as four calls; the gate-first form (gate,
    then the up projection only where the gate is open with the GLU inside, then down); and gate + up +
    GLU as one launch followed by down."""
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

    Hb = torch.empty((1, FFN), dtype=bf16, device=dev)
    ws_gu = torch.empty(max(B.lib().bitlinear_gate_up_workspace_bytes(1, FFN, HIDDEN, B.BL_W_GEMM), 16), dtype=torch.uint8,
                        device=dev)

    def one_launch_front(l):
        # gate, up and eq. 5 in one launch (H only), then down
        (pg, ag), (pu, au), _, (pd, ad) = sets[l]
        B.bitlinear_a4_gate_up(X, pg, ag, pu, au, FFN, EPS, B.BL_W_GEMM, want=("H",), ws=ws_gu, out={"H": Hb})
        B.bitlinear_a8_sparse(Hb, FFN // 2, pd, ad, HIDDEN, EPS, ws=ws8, out=Y)

    res = {}
    side = torch.cuda.Stream()
    for name, fn in (("four_calls", dense), ("gate_first", gate_first), ("gate_up_glu_then_down", one_launch_front)):
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


def _graph_time_us(torch, fn, n_calls, replays, side):
    """Capture `n_calls` invocations fn(0) .. fn(n_calls - 1) in one HIP graph on `side` and time
    `replays` replays with events on the current stream: microseconds per invocation."""
    for i in range(n_calls):
        fn(i)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for i in range(n_calls):
                fn(i)
    g.replay()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (replays * n_calls)
    del g
    return us


DECODE_LAYERS = 32            # distinct layers of the sweep: 32 x 50.6 MB = 1.6 GB of packed weights
DECODE_MIN_SET_BYTES = 640e6  # per-projection timing cycles at least this many bytes of distinct weights


def decode_bench(B, S, torch, dev, tokens=(1, 8, 32, 64), replays=5):
    """Packed-weight bandwidth at decode shapes, with the weights coming from HBM.

    Weights: DECODE_LAYERS distinct layers (five projections each, 1.6 GB in all), drawn on the
    device from a seeded generator and packed once.  Per token count:
      * `layer_sweep`: one HIP graph walks the projections of all layers in model order (qkv, o, the
        gate and up projection with their GLU behind one entry point, down), so every weight byte
        read is one of 1.6 GB read since its last use (the memory-side cache holds 256 MB);
        `layer_sweep_five_calls` is the same walk with gate and up as two calls;
      * per projection: a graph over enough distinct weight sets of that one shape that a replay
        touches at least DECODE_MIN_SET_BYTES (the o projection gets extra sets for that);
      * for the two top-K + INT8 projections at 1 and 8 tokens also the row-skipping path
        (BL_W_KMAJOR): microseconds, GB/s over the bytes it has to read (the rows of the channels
        kept by at least one token) and dense-equivalent GB/s (all N*K/4 bytes over the same time).
    `launch_floor_us` is the same graph timing of the library's empty kernel."""
    bf16 = torch.bfloat16
    projs = S.projections(HIDDEN, FFN)
    gen = torch.Generator(device=dev)
    gen.manual_seed(S.seed_for(2, 4000))

    def n_sets(nbytes):
        return max(DECODE_LAYERS, int(-(-DECODE_MIN_SET_BYTES // nbytes)))

    packed, packed_k = {}, {}
    for name, N, K, kind in projs:
        sets, sets_k = [], []
        for l in range(n_sets(N * K / 4)):
            w = torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02
            sets.append(B.pack_ternary(w, EPS, B.BL_W_GEMM))
            if kind == "a8s":
                sets_k.append(B.pack_ternary(w, EPS, B.BL_W_KMAJOR))
            del w
        packed[name] = sets
        packed_k[name] = sets_k
    side = torch.cuda.Stream()
    res = {"layers": DECODE_LAYERS,
           "weights_resident_mb": round(sum(p.numel() for v in list(packed.values()) + list(packed_k.values())
                                            for p, _ in v) / 1e6, 1),
           "launch_floor_us": round(_graph_time_us(torch, lambda i: B.noop(), 160, 20, side), 3)}
    for M in tokens:
        row = {}
        X, ws, Y = {}, {}, {}
        for name, N, K, kind in projs:
            X[name] = torch.from_numpy(S.glu_like(M, K, S.seed_for(2, 200 + M)) if name == "down"
                                       else S.heavy(M, K, S.seed_for(2, 100 + M))).to(dev).to(bf16)
            mode = B.BL_ACT_INT4_ABSMEAN if kind == "a4" else B.BL_ACT_TOPK_INT8_ABSMAX
            ws[name] = B.workspace(mode, M, N, K, dev)
            Y[name] = torch.empty((M, N), dtype=bf16, device=dev)

        def run(name, N, K, kind, l, kmajor=False):
            if kind == "a4":
                p, a = packed[name][l]
                B.bitlinear_a4(X[name], p, a, N, EPS, ws=ws[name], out=Y[name])
            elif kmajor:
                p, a = packed_k[name][l]
                B.bitlinear_a8_sparse(X[name], K // 2, p, a, N, EPS, layout=B.BL_W_KMAJOR, ws=ws[name], out=Y[name])
            else:
                p, a = packed[name][l]
                B.bitlinear_a8_sparse(X[name], K // 2, p, a, N, EPS, ws=ws[name], out=Y[name])

        for name, N, K, kind in projs:
            n = len(packed[name])
            us = _graph_time_us(torch, lambda l: run(name, N, K, kind, l), n, replays, side)
            wbytes = N * K / 4
            row[name] = {"us": round(us, 2), "weight_gbs": round(wbytes / us / 1e3, 1),
                         "frac_hbm_peak": round(wbytes / us / 1e3 / HBM_PEAK_GBS, 4), "weight_sets": n}
            if kind == "a8s" and M <= 8:
                qd = B.quantize_act(X[name], B.BL_ACT_TOPK_INT8_ABSMAX, topk=K // 2, eps=EPS)
                codes = B.unpack_act(qd["q"], B.BL_ACT_TOPK_INT8_ABSMAX, M, K)
                union = int((codes != 0).any(dim=0).sum().item())
                us_k = _graph_time_us(torch, lambda l: run(name, N, K, kind, l, True), n, replays, side)
                need = union * N / 4
                row[name]["row_skipping"] = {
                    "us": round(us_k, 2), "channels_read": union, "channels": K,
                    "required_gbs": round(need / us_k / 1e3, 1),
                    "frac_hbm_peak": round(need / us_k / 1e3 / HBM_PEAK_GBS, 4),
                    "dense_equivalent_gbs": round(wbytes / us_k / 1e3, 1)}

        # gate and up projection behind one entry point (one quantized input; one launch for up to 8
        # tokens), writing H = bf16(U * max(G, 0)^2) only
        Hbuf = {"H": torch.empty((M, FFN), dtype=bf16, device=dev)}
        ws_gu = torch.empty(max(B.lib().bitlinear_gate_up_workspace_bytes(M, FFN, HIDDEN, B.BL_W_GEMM), 16),
                            dtype=torch.uint8, device=dev)

        def gate_up(l):
            (pg, ag), (pu, au) = packed["gate"][l], packed["up"][l]
            B.bitlinear_a4_gate_up(X["gate"], pg, ag, pu, au, FFN, EPS, want=("H",), ws=ws_gu, out=Hbuf)
        n = len(packed["gate"])
        us = _graph_time_us(torch, gate_up, n, replays, side)
        wbytes = 2 * FFN * HIDDEN / 4
        row["gate_up_glu"] = {"us": round(us, 2), "weight_gbs": round(wbytes / us / 1e3, 1),
                              "frac_hbm_peak": round(wbytes / us / 1e3 / HBM_PEAK_GBS, 4), "weight_sets": n}

        lbytes = sum(N * K / 4 for _, N, K, _ in projs)

        def layer(i):
            for name, N, K, kind in projs:
                run(name, N, K, kind, i)
        us_layer = _graph_time_us(torch, layer, DECODE_LAYERS, replays, side)
        row["layer_sweep_five_calls"] = {"us_per_layer": round(us_layer, 2), "weight_gbs": round(lbytes / us_layer / 1e3, 1),
                                         "frac_hbm_peak": round(lbytes / us_layer / 1e3 / HBM_PEAK_GBS, 4)}

        def layer_fused(i):
            run("qkv", 3 * HIDDEN, HIDDEN, "a4", i)
            run("o", HIDDEN, HIDDEN, "a8s", i)
            gate_up(i)
            run("down", HIDDEN, FFN, "a8s", i)
        us_layer = _graph_time_us(torch, layer_fused, DECODE_LAYERS, replays, side)
        row["layer_sweep"] = {"us_per_layer": round(us_layer, 2), "weight_gbs": round(lbytes / us_layer / 1e3, 1),
                              "frac_hbm_peak": round(lbytes / us_layer / 1e3 / HBM_PEAK_GBS, 4),
                              "calls": "qkv, o, gate+up+GLU, down"}
        if M <= 8:
            def layer_k(i):
                for name, N, K, kind in projs:
                    run(name, N, K, kind, i, kmajor=(kind == "a8s"))
            us_lk = _graph_time_us(torch, layer_k, DECODE_LAYERS, replays, side)
            need = sum((row[name]["row_skipping"]["channels_read"] * N / 4) if kind == "a8s" else N * K / 4
                       for name, N, K, kind in projs)
            row["layer_sweep_row_skipping"] = {
                "us_per_layer": round(us_lk, 2), "required_gbs": round(need / us_lk / 1e3, 1),
                "frac_hbm_peak": round(need / us_lk / 1e3 / HBM_PEAK_GBS, 4),
                "dense_equivalent_gbs": round(lbytes / us_lk / 1e3, 1)}
        res["M%d" % M] = row
    return res


if __name__ == "__main__":
    main()
