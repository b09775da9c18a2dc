#!/usr/bin/env python3
"""Benchmark of the masked-layer hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input that
is already resident in HBM:
    dk_encode -> dk_conv_fwd | dk_linear_fwd -> dk_decode_verify -> dk_wgrad
(dk_decode_verify = dk_verify + dk_decode in one sweep over the encoded results).
The step is captured once into a HIP graph and replayed (--no-graph: eager).
--noise-vectors M uses the *_m entry points (M noise vectors per group);
--workload field1 | field2 | field3[.i] | field4[.i] | field5[.i] | fieldmbv2dw[.i] runs the finite-field
variant instead (dkf_quantize -> dkf_encode -> dkf_linear_fwd | dkf_conv_fwd ->
dkf_decode_verify -> dkf_wgrad).
Prints ONE JSON line: whole-path executed TFLOP/s (forward + weight gradient
on all K+2 encoded rows per group), decoded samples/s, the roofline record of
the dominant kernel (timed with events on the launch stream inside the timed
region) and the fp64 CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
MFMA_I8_PEAK_TOPS = 5000.0        # MI355X dense int8 matrix peak
HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E


def workload(name):
    import dk_inputs
    if name == "config1":
        return dk_inputs.config1(), "config1: dense 256->512, K=2, 1 group"
    if name == "config2":
        return dk_inputs.config2(), "config2: conv3x3 s1 p1 64->64 @32x32 NCHW, batch 256, K=4 (G=64, 384 encoded rows)"
    if name == "config2.ragged":
        # rows of odd length (63 channels of 31x31 pixels): no row but the first of a tensor starts on a
        # 16-byte boundary, so the mixing kernels move unaligned vectors and finish each row element-wise
        rng = np.random.default_rng(22)
        return (dk_inputs.masked_layer_inputs(rng, dk_inputs.conv(63, 63, 31, 31, 3), K=4, batch=256,
                                              noise_std=10.0, delta_std=0.1),
                "config2 with ragged rows: conv3x3 s1 p1 63->63 @31x31, batch 256, K=4")
    if name.startswith("config3."):
        i = int(name.split(".")[1])
        return dk_inputs.config3(index=i)[0], "config3 layer %d (VGG-16 conv stack @32x32, batch 128, K=4)" % i
    if name.startswith("config4."):
        i = int(name.split(".")[1])
        for k, (d, count) in enumerate(dk_inputs.config4()):
            if k == i:
                return d, "config4 shape %d x%d (ResNet-50 convs @224x224 input, batch 64, K=8)" % (i, count)
        raise SystemExit("config4 has 22 shapes")
    if name.startswith("config5."):
        i = int(name.split(".")[1])
        return dk_inputs.config5(index=i)[0], "config5 layer %d (VGG classifier, batch 1024, K=8)" % i
    if name.startswith("mbv2dw."):
        i = int(name.split(".")[1])
        d, count = dk_inputs.mobilenetv2_dw(index=i)[0]
        return d, "MobileNetV2 depthwise 3x3 layer %d x%d (224x224 input, batch 64, K=8)" % (i, count)
    raise SystemExit("unknown workload " + name)


def algorithmic_bytes(K, G, n, m, M=1):
    """HBM bytes each bandwidth-bound kernel must move (fp32), per launch."""
    S = K + M + 1
    return {
        "encode": 4 * G * n * (K + M + S),
        "decode_verify": 4 * G * m * (S + K),      # one read of ybar serves both
        "delta_mix": 4 * G * m * (K + S),
    }


def measured_traffic(workload_name, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc
    summary of this same command (profiles/traffic.json), or None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        rec = json.load(open(path)).get(workload_name, {}).get(kernel)
        return None if rec is None else rec["hbm_bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        return None


def cpu_baseline(d, budget_s=15.0):
    """The fp64 oracle's staged masked layer on the first few groups."""
    import oracle
    L, K, G = d["layer"], d["K"], d["G"]
    M = d.get("M", 1)
    S = K + M + 1
    flop_per_group = 2 * 2 * S * L.macs_per_row

    def run(ng):
        sl = slice(0, ng * K)
        t0 = time.perf_counter()
        if M == 1:
            oracle.masked_layer(d["W"], d["X"][sl], d["r"][:ng], d["delta"][sl], d["A"][:ng],
                                d["gamma"][:ng], stride=L.stride, pad=L.pad)
        else:
            oracle.masked_layer_m(d["W"], d["X"][sl], d["r"][:ng * M], d["delta"][sl], d["A"][:ng],
                                  d["gamma"][:ng], K, stride=L.stride, pad=L.pad)
        return time.perf_counter() - t0

    oracle.build()
    t1 = run(1)
    ng = int(max(1, min(G, budget_s / max(t1, 1e-3))))
    t = run(ng) if ng > 1 else t1
    return {
        "value": flop_per_group * ng / t / 1e12, "unit": "TFLOP/s",
        "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "staged fp64 oracle (encode, layer on encodings, verify, decode, masked wgrad) on the "
                  "first %d of %d groups, %.1f s" % (ng, G, t),
        "samples_per_s": ng * K / t,
    }


def pmc_calibration_copies(torch):
    """Three plain 1 GiB device copies: a transfer of known size against which
    rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled."""
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def field_workload(name):
    import dk_inputs
    if name == "field1":
        return dk_inputs.config1_field(), "config1 over F_p: dense 256->512, K=2, 1 group"
    if name == "field2":
        return dk_inputs.config2_field(), "config2 over F_p: conv3x3 s1 p1 64->64 @32x32 NCHW, batch 256, K=4"
    if name.startswith("field3."):
        i = int(name.split(".")[1])
        return dk_inputs.config3_field(index=i), "config3 layer %d over F_p (VGG-16 conv stack @32x32, batch 128, K=4)" % i
    if name.startswith("field4."):
        i = int(name.split(".")[1])
        d, count = dk_inputs.config4_field(index=i)
        return d, "config4 shape %d x%d over F_p (ResNet-50 convs @224x224 input, batch 64, K=8)" % (i, count)
    if name.startswith("field5."):
        i = int(name.split(".")[1])
        return (dk_inputs.config5_field(index=i)[0],
                "config5 layer %d over F_p, p=2^25-39, l=8 (VGG classifier, batch 1024, K=8)" % i)
    if name.startswith("fieldmbv2dw."):
        i = int(name.split(".")[1])
        d, count = dk_inputs.mobilenetv2_dw_field(index=i)
        return d, "MobileNetV2 depthwise 3x3 layer %d x%d over F_p (224x224 input, batch 64, K=8)" % (i, count)
    raise SystemExit("unknown workload " + name)


def field_cpu_baseline(d, budget_s=15.0):
    """The field oracle's staged layer on the first few groups."""
    from oracle import field as F
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    op_per_group = 2 * 2 * S * L.macs_per_row

    def run(ng):
        sl = slice(0, ng * K)
        t0 = time.perf_counter()
        layer = F.masked_dw_layer if L.kind == "dwconv" else F.masked_layer
        layer(d["W"], d["X"][sl], d["r"][:ng], d["delta"][sl], d["A"][:ng], d["gamma"][:ng],
              stride=L.stride, pad=L.pad)
        return time.perf_counter() - t0

    import oracle
    oracle.build()
    t1 = run(1)
    ng = int(max(1, min(G, budget_s / max(t1, 1e-3))))
    t = run(ng) if ng > 1 else t1
    return {
        "value": op_per_group * ng / t / 1e12, "unit": "TOP/s (one field multiply-add = 2)",
        "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "staged field oracle (quantise, encode, product on encodings, verify, decode, masked "
                  "wgrad, one remainder per operation) on the first %d of %d groups, %.1f s" % (ng, G, t),
        "samples_per_s": ng * K / t,
    }


def field_main(args):
    """The finite-field variant of a layer:
    dkf_encode -> dkf_linear_fwd_w | dkf_quantize(W), dkf_conv_fwd -> dkf_decode_verify -> dkf_wgrad."""
    import torch
    import paper_2207_00083_amd as dk
    dk.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.pmc_calibration:
        pmc_calibration_copies(torch)
    d, wname = field_workload(args.workload)
    L, K, G = d["layer"], d["K"], d["G"]
    S = K + 2
    R = G * S

    def dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int32) if a.dtype == np.uint32 else a).cuda()

    Ainv, nvec, B = dk.dkf_coeffs(d["A"], d["gamma"])
    W, X, r, delta = dev(d["W"]), dev(d["X"]), dev(d["r"]), dev(d["delta"])
    A_d, Ainv_d, nvec_d, B_d, gamma_d = dev(d["A"]), dev(Ainv), dev(nvec), dev(B), dev(d["gamma"])
    i32 = dict(dtype=torch.int32, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")
    conv = L.kind in ("conv", "dwconv")
    Wq = torch.empty(L.w_shape, **i32)
    xbar = torch.empty((R,) + L.in_shape, **i32)
    ybar = torch.empty((R,) + L.out_shape, **i32)
    y = torch.empty((G * K,) + L.out_shape, **f32)
    dW = torch.empty(L.w_shape, **f32)
    verdict = torch.empty(G, **i32)
    ws_f = torch.empty(dk.dkf_conv_fwd_workspace_bytes(L, R) if conv else dk.dkf_fwd_workspace_bytes(L.M, L.N, R),
                       dtype=torch.uint8, device="cuda")
    ws_w = torch.empty(dk.dkf_wgrad_workspace_bytes(L, G, K), dtype=torch.uint8, device="cuda")
    stages = ["quantize_w", "encode", "fwd", "decode_verify", "wgrad"]

    def step(ev=None):
        if ev: ev[0].record()
        if conv:
            dk.dkf_quantize(W, xq=Wq)
        if ev: ev[1].record()
        if args.rng_noise:
            dk.dkf_encode_rng(X, A_d, K, 20220701, xbar=xbar)
        else:
            dk.dkf_encode(X, r, A_d, K, xbar=xbar)
        if ev: ev[2].record()
        if conv:
            dk.dkf_conv_fwd(L, Wq, xbar, ybar=ybar, ws=ws_f)
        else:
            # dense layers: the weights are quantised where they are split into digits (no W_q round trip)
            dk.dkf_linear_fwd_w(W, xbar, ybar=ybar, ws=ws_f)
        if ev: ev[3].record()
        dk.dkf_decode_verify(ybar, Ainv_d, nvec_d, K, y=y, verdict=verdict)
        if ev: ev[4].record()
        dk.dkf_wgrad(L, delta, B_d, gamma_d, xbar, K, dW=dW, ws=ws_w)
        if ev: ev[5].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        ref = [t.clone() for t in (y, dW, verdict)]
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    step()
            torch.cuda.current_stream().wait_stream(side)
        except Exception as e:                      # noqa: BLE001 - capture refused: time eager launches
            sys.stderr.write("bench.py: HIP graph capture failed, timing eager launches (%s)\n" % e)
            graph = None
        torch.cuda.synchronize()
        if graph:
            # replays that differ from the eager results are an error, not a reason to fall back
            for _ in range(3):
                for t in (y, dW):
                    t.zero_()
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                if not all(torch.equal(a, b) for a, b in zip((y, dW, verdict), ref)):
                    raise RuntimeError("graph replay differs from the eager step")
        for _ in range(args.warmup):
            graph.replay() if graph else step()
        torch.cuda.synchronize()

    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay() if graph else step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    dk.dk_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dk.dk_profile_enable(False)
    kernels = dk.dk_profile_read()
    assert int(verdict.sum().item()) == 0, "clean synthetic data must verify"

    ms_per_step = wall / args.steps * 1e3
    stage_ms = {s: float(np.mean([e[i].elapsed_time(e[i + 1]) for e in events])) for i, s in enumerate(stages)}
    mac = float(R) * L.macs_per_row                # field multiply-adds per contraction
    op_step = 2.0 * 2.0 * mac                       # forward + weight gradient
    tops = op_step / (ms_per_step * 1e-3) / 1e12
    # The contraction kernel runs twice a step.  The forward multiplies 4 digit
    # planes of the encodings with the 2 non-zero planes of ordinary weights
    # (8 int8 products per field product; 4 when one plane holds them, see below),
    # the weight gradient 4 x 4 planes (16),
    # or three products of half against half (12) where the operands come with
    # digit-sum planes: dense layers, 1x1 and most stride-1 convolutions.  Executed products
    # are counted.  The roofline record is the longer of the two launches.
    # (the library's own choice, restated: the three-part form also serves
    # stride-1 filters whose output width grows by at most 1/7 when rounded up to 16)
    three_part = (L.kind == "linear" or L.kh * L.kw == 1 or
                  (L.stride == 1 and (L.Wo + 15) // 16 * 16 * 7 <= L.Wo * 8))
    n, m = dk.dk_layer_in_len(L), dk.dk_layer_out_len(L)
    if L.kind == "dwconv":
        # a few multiply-adds per element moved: both kernels read the encodings (or the mixed
        # gradients and the encodings) once and write (or reduce) once -- 4 R (n + m) bytes each
        dwk = {"f_dw_fwd": 4.0 * R * (n + m), "f_dw_wgrad": 4.0 * R * (n + m)}
        dom = max(dwk, key=lambda k: kernels[k][0])
        ach = dwk[dom] / (kernels[dom][0] * 1e-3) / 1e9
        roofline = {
            "kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": ach / HBM_PEAK_GBPS, "traffic": None, "avg_launch_ms": kernels[dom][0],
            "bytes_per_launch": dwk[dom],
            "other": {k: {"avg_launch_ms": kernels[k][0], "GBps": b / (kernels[k][0] * 1e-3) / 1e9}
                      for k, b in dwk.items() if k != dom},
            "timed": "HIP events around every launch of this kernel, %d eager steps after the timed region" % args.steps,
        }
    # Weights whose quantised values all lie in [-127, 127] fill one digit plane; the forward then
    # multiplies 4 x 1 planes (the library takes those steps for dense layers and for
    # convolutions with more than 64 output channels and a contraction of at least 512).
    wq = np.rint(np.asarray(d["W"], dtype=np.float64) * 2.0 ** 8)
    # (128-row tiles: the library takes 64-row tiles when the last 128 output channels are at most 64)
    wide_tiles = L.kind != "linear" and not (L.Co % 128 != 0 and L.Co % 128 <= 64)
    one_digit = bool(wq.min() >= -127 and wq.max() <= 127) and (
        L.kind == "linear" or (wide_tiles and L.Ci * L.kh * L.kw >= 512))
    gemm = {"f_gemm_fwd": 4 if one_digit else 8, "f_gemm_wgrad": 12 if three_part else 16}
    dom = max(gemm, key=lambda k: kernels[k][0]) if L.kind != "dwconv" else None
    gemm_ms = kernels[dom][0] if dom else 0.0
    int8_ops = 2.0 * mac * gemm[dom] if dom else 0.0
    ach = int8_ops / (gemm_ms * 1e-3) / 1e12 if dom else 0.0
    roofline = roofline if L.kind == "dwconv" else {
        "kernel": dom, "bound": "mfma", "achieved": ach, "peak": MFMA_I8_PEAK_TOPS, "unit": "TOP/s",
        "frac": ach / MFMA_I8_PEAK_TOPS, "traffic": measured_traffic(args.workload, dom),
        "avg_launch_ms": gemm_ms, "int8_op_per_launch": int8_ops,
        "digit_products_per_field_product": gemm,
        "field_top_per_s": 2.0 * mac / (gemm_ms * 1e-3) / 1e12,
        "other_contraction": {k: {"avg_launch_ms": kernels[k][0],
                                  "int8_TOPs": 2.0 * mac * c / (kernels[k][0] * 1e-3) / 1e12}
                              for k, c in gemm.items() if k != dom},
        "timed": "HIP events around every launch of this kernel, %d eager steps after the timed region" % args.steps,
    }
    ab = {"f_encode": 4 * G * n * (K + 1 + S), "f_decode_verify": 4 * G * m * (S + K),
          "f_delta_mix": 4 * G * m * (K + S)}
    hbm = {k: {"GBps": b / (kernels[k][0] * 1e-3) / 1e9, "frac": b / (kernels[k][0] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
               "bytes": b, "avg_launch_ms": kernels[k][0]} for k, b in ab.items() if k in kernels}
    out = {
        "metric": "masked-layer TOP/s over F_p (fwd+wgrad, one field multiply-add = 2, executed on all K+2 "
                  "encoded rows), whole hot path",
        "value": tops, "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 field elements, int8 digit MFMA", "data": "synthetic",
        "config": {"workload": wname, "K": K, "G": G, "layer": L.asdict(),
                   "launch": "HIP graph replay of one captured step" if graph else "eager"},
        "decoded_samples_per_s": G * K / (ms_per_step * 1e-3),
        "stage_ms": stage_ms,
        "fwd_stage_tops": 2.0 * mac / (stage_ms["fwd"] * 1e-3) / 1e12,
        "wgrad_stage_tops": 2.0 * mac / (stage_ms["wgrad"] * 1e-3) / 1e12,
        "roofline": roofline, "hbm_kernels": hbm,
        "kernel_ms": {k: v[0] for k, v in kernels.items()},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = field_cpu_baseline(d)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="config2")
    ap.add_argument("--noise-vectors", type=int, default=1, metavar="M",
                    help="noise vectors per group (M > 1: tolerate M colluding accelerators, K+M+1 encodings "
                         "per group; same layer shape, batch and K as the named workload)")
    ap.add_argument("--rng-noise", action="store_true",
                    help="draw the noise inside the encoding kernel (dk_encode_rng / dkf_encode_rng, one seed "
                         "per step) instead of reading noise rows from HBM")
    ap.add_argument("--with-dgrad", action="store_true",
                    help="also time the un-encoded data gradient of the layer (dk_dgrad on the K*G real "
                         "gradients); reported as dgrad_ms, not part of the masked path or of `value`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch every step eagerly")
    ap.add_argument("--fork", action="store_true",
                    help="capture the weight gradient on a second graph branch (it may then overlap the "
                         "forward chain; per-kernel profiler durations of overlapped kernels are inflated)")
    ap.add_argument("--fuse", choices=["never", "always", "auto"], default="auto",
                    help="fused kernels for 1x1 convolutions (forward + decode + verify in one kernel through "
                         "dk_conv_fwd_decode_verify; gradient mixing inside the weight gradient's loader): "
                         "never, wherever eligible, or the library's own choice by layer shape")
    ap.add_argument("--group-chunks", type=int, default=1, metavar="N",
                    help="run encode -> forward -> decode+verify on N runs of virtual batches one after the "
                         "other, so that a run's encoded results are still in the last-level cache when they "
                         "are decoded (separate kernels only: implies --fuse never)")
    ap.add_argument("--chunk-streams", type=int, default=1, choices=[1, 2],
                    help="with --group-chunks: put the runs alternately on two streams (two branches of the "
                         "captured graph), so that a run's encoding can overlap the previous run's forward")
    ap.add_argument("--rotate", type=int, default=0,
                    help="buffer sets every pass cycles through, so that no kernel finds the inputs of the "
                         "step before in the 256 MB last-level cache (1 = reuse one set; default: as many "
                         "sets, at least 3, as put 600 MB between two uses of a set)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="first run three plain 1 GiB device copies (a known-size reference for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--mfma-rate", action="store_true",
                    help="only measure what the matrix pipes sustain with constant and with random operands "
                         "(dkf_probe_mfma_rate: int8; dk_probe_mfma_rate: fp32) and print the rates")
    args = ap.parse_args()
    if args.mfma_rate:
        print(json.dumps(mfma_rate()))
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build covers the one-GPU hot path only; run with --gpus 1\n")
        raise SystemExit(2)

    subs = sub_workloads(args.workload)
    if subs:
        print(json.dumps(aggregate(args, subs)))
        return
    out = field_main(args) if args.workload.startswith("field") else layer_main(args)
    print(json.dumps(out))


def mfma_rate():
    """Operations per second of kernels that issue nothing but matrix instructions (int8 and fp32)."""
    import torch
    import paper_2207_00083_amd as dk
    dk.load()

    def rate(probe, kind):
        probe(kind, 2000)
        torch.cuda.synchronize()
        rates = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ops = probe(kind, 40000)
            e1.record()
            torch.cuda.synchronize()
            rates.append(ops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        return {"T_per_s": sum(rates) / len(rates), "min": min(rates), "max": max(rates)}

    out = {"metric": "matrix-instruction rate, operands in registers, one wave per SIMD",
           "int8": {"unit": "TOP/s", "peak": 5000.0}, "fp32": {"unit": "TFLOP/s", "peak": 157.3}}
    for name, kind in (("constant_operands", 0), ("random_bytes", 1), ("random_balanced_digits", 2)):
        out["int8"][name] = rate(dk.dkf_probe_mfma_rate, kind)
    for name, kind in (("constant_operands", 0), ("random_operands", 1)):
        out["fp32"][name] = rate(dk.dk_probe_mfma_rate, kind)
    return out


def sub_workloads(name):
    """(sub-workload, multiplicity) pairs of a whole-network workload name."""
    import dk_inputs
    if name == "config3":
        return [("config3.%d" % i, 1) for i in range(len(dk_inputs.config3_layers()))]
    if name == "config4":
        return [("config4.%d" % i, c) for i, (_, c) in enumerate(dk_inputs.resnet50_convs())]
    if name == "config5":
        return [("config5.%d" % i, 1) for i in range(len(dk_inputs.config5_layers()))]
    if name == "mbv2dw":
        return [("mbv2dw.%d" % i, c[3]) for i, c in enumerate(dk_inputs.MOBILENETV2_DW)]
    if name == "field5":
        return [("field5.%d" % i, 1) for i in range(len(dk_inputs.config5_layers()))]
    if name == "field3":
        return [("field3.%d" % i, 1) for i in range(len(dk_inputs.config3_layers()))]
    if name == "field4":
        return [("field4.%d" % i, c) for i, (_, c) in enumerate(dk_inputs.resnet50_convs())]
    if name == "fieldmbv2dw":
        return [("fieldmbv2dw.%d" % i, c[3]) for i, c in enumerate(dk_inputs.MOBILENETV2_DW)]
    return None


def aggregate(args, subs):
    """Every layer of a network workload, one after the other (each layer is
    its own masked-layer problem with its own inputs; the non-linear layers
    between them are not part of the path).  Times add up with the layers'
    multiplicities; the roofline record is that of the layer with the largest
    share of the time."""
    import copy
    name, layers, total_ms, total_op, batch, total_floor = args.workload, [], 0.0, 0.0, None, 0.0
    for sub, count in subs:
        a = copy.copy(args)
        a.workload, a.no_cpu_baseline = sub, True
        o = field_main(a) if sub.startswith("field") else layer_main(a)
        op = o["value"] * 1e12 * o["ms_per_step"] * 1e-3
        layers.append({"workload": sub, "count": count, "ms_per_step": o["ms_per_step"], "value": o["value"],
                       "roofline_kernel": o["roofline"]["kernel"], "roofline_bound": o["roofline"]["bound"],
                       "roofline_frac": o["roofline"]["frac"], "layer": o["config"].get("layer"),
                       "kernel_ms": o.get("kernel_ms")})
        if "roofline_floor_ms" in o:
            layers[-1].update(roofline_floor_ms=o["roofline_floor_ms"], step_frac=o["step_frac"],
                              step_bound=o["step_bound"])
            total_floor += count * o["roofline_floor_ms"]
        total_ms += count * o["ms_per_step"]
        total_op += count * op
        batch = o["config"]["K"] * o["config"]["G"]
        o["_share"] = count * o["ms_per_step"]
        layers[-1]["_o"] = o
    top = max(layers, key=lambda l: l["_o"]["_share"])["_o"]
    for l in layers:
        del l["_o"]
    out = {
        "metric": top["metric"] + ", all layers of the network in sequence",
        "value": total_op / (total_ms * 1e-3) / 1e12, "unit": top["unit"], "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": total_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": top["dtype"], "data": "synthetic",
        "config": {"workload": "%s: %d layer shapes, %d layers with multiplicity, batch %d"
                               % (name, len(subs), sum(c for _, c in subs), batch),
                   "launch": top["config"]["launch"]},
        "decoded_samples_per_s": batch / (total_ms * 1e-3),
        "roofline": top["roofline"],
        "layers": layers,
    }
    if total_floor > 0.0:
        out["roofline_floor_ms"] = total_floor
        out["step_frac"] = total_floor / total_ms
    if not args.no_cpu_baseline:
        a = copy.copy(args)
        a.workload = subs[0][0]
        d = (field_workload if a.workload.startswith("field") else workload)(a.workload)[0]
        out["cpu_baseline"] = (field_cpu_baseline if a.workload.startswith("field") else cpu_baseline)(d)
        out["cpu_baseline"]["sample"] = "layer %s only: %s" % (a.workload, out["cpu_baseline"]["sample"])
    return out


def layer_main(args):
    import torch
    import paper_2207_00083_amd as dk
    dk.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.pmc_calibration:
        pmc_calibration_copies(torch)

    d, wname = workload(args.workload)
    L, K, G = d["layer"], d["K"], d["G"]
    M = args.noise_vectors
    if M > 1:
        import dk_inputs
        d = dk_inputs.collusion_layer_inputs(np.random.default_rng([7, M]), L, K=K, M=M, batch=G * K)
        wname += ", %d noise vectors per group" % M
    S = K + M + 1
    n, m = dk.dk_layer_in_len(L), dk.dk_layer_out_len(L)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    Ainv, nvec, B = dk.dk_coeffs_m(d["A"], d["gamma"], K)
    W = dev(d["W"])
    A_d, Ainv_d, nvec_d, B_d, gamma_d = dev(d["A"]), dev(Ainv), dev(nvec), dev(B), dev(d["gamma"])
    f32 = dict(dtype=torch.float32, device="cuda")
    u8 = dict(dtype=torch.uint8, device="cuda")

    class Buffers:
        """One set of the per-step tensors (inputs, encodings, outputs, workspaces)."""
        def __init__(self):
            self.X, self.r, self.delta = dev(d["X"]), dev(d["r"]), dev(d["delta"])
            self.xbar = torch.empty((G * S,) + L.in_shape, **f32)
            self.ybar = torch.empty((G * S,) + L.out_shape, **f32)
            self.y = torch.empty((G * K,) + L.out_shape, **f32)
            self.dW = torch.empty(L.w_shape, **f32)
            self.verdict = torch.empty(G, dtype=torch.int32, device="cuda")
            self.resid = torch.empty(G, **f32)
            lib = dk.load()
            self.ws_fwd = torch.empty(lib.dk_fwd_workspace_bytes(C.byref(dk.DkLayer.of(L)), G * S), **u8)
            self.ws_wg = torch.empty(lib.dk_workspace_bytes_m(C.byref(dk.DkLayer.of(L)), dk.DK_OP_WGRAD, G, K, M), **u8)
            self.ws_vf = torch.empty(lib.dk_workspace_bytes_m(None, dk.DK_OP_VERIFY, G, K, M), **u8)
            if args.group_chunks > 1:
                # a run of virtual batches may need more forward workspace than the whole batch
                # (other slicing of the contraction); one workspace pair per stream
                nb = max(lib.dk_fwd_workspace_bytes(C.byref(dk.DkLayer.of(L)), (G * (c + 1) // args.group_chunks
                                                                               - G * c // args.group_chunks) * S)
                         for c in range(args.group_chunks))
                self.ws_fwd = [torch.empty(max(nb, self.ws_fwd.numel()), **u8) for _ in range(args.chunk_streams)]
                self.ws_vf = [torch.empty(self.ws_vf.numel(), **u8) for _ in range(args.chunk_streams)]
            if one_call:
                del self.ybar, self.ws_fwd, self.ws_vf
                self.ws_fdv = torch.empty(dk.dk_conv_fwd_decode_verify_workspace_bytes(L, G, K), **u8)

    # Every pass below cycles through `--rotate` sets of the per-step tensors.
    # Between two uses of a set the other sets push more than the last-level
    # cache's 256 MB through it, so no kernel finds the inputs of the step
    # before still cached -- as in training, where a layer's tensors come back
    # after the rest of the network has run.  What one kernel of a step leaves
    # behind for the next (the forward's output, read by decode + verify) stays:
    # the path runs that way.  The weights are shared by all sets.
    if args.group_chunks > 1:
        args.fuse = "never"
    fuse = {"never": dk.DK_FUSE_NEVER, "always": dk.DK_FUSE_ALWAYS, "auto": dk.DK_FUSE_AUTO}[args.fuse]
    dk.dk_set_option(dk.DK_OPT_FUSE_FWD, fuse)
    dk.dk_set_option(dk.DK_OPT_FUSE_WGRAD, fuse)
    # one call for forward + decode + verify (the library fuses it where it can and may)
    one_call = args.fuse != "never" and L.kind == "conv" and M == 1
    b0 = Buffers()
    one_set = sum(t.numel() * t.element_size() for v in vars(b0).values()
                  for t in (v if isinstance(v, list) else [v]))
    nsets = args.rotate if args.rotate >= 1 else int(min(16, max(3, -(-600e6 // one_set) + 1)))
    sets = [b0] + [Buffers() for _ in range(nsets - 1)]
    y, dW, verdict = b0.y, b0.dW, b0.verdict
    conv = L.kind in ("conv", "dwconv")

    stages = ["encode", "fwd", "decode_verify", "wgrad"]

    side2 = torch.cuda.Stream()

    def step(ev=None, fork=False, b=b0):
        """fork=True (graph capture only): the weight gradient needs nothing of
        the forward chain but the encodings, so it goes on a second stream and
        the two branches of the captured graph may overlap."""
        cur = torch.cuda.current_stream()
        if args.group_chunks > 1:
            # virtual batches in runs: a run's encodings and results stay cached between its kernels
            S_ = K + M + 1
            two = args.chunk_streams == 2
            if two:
                side2.wait_stream(cur)
            for c in range(args.group_chunks):
                g0, g1 = G * c // args.group_chunks, G * (c + 1) // args.group_chunks
                if g0 == g1:
                    continue
                si = c % 2 if two else 0
                with torch.cuda.stream(side2 if si else cur):
                    dk.dk_encode_m(b.X[g0 * K:g1 * K], b.r[g0 * M:g1 * M], A_d[g0:g1], K, M,
                                   xbar=b.xbar[g0 * S_:g1 * S_])
                    if conv:
                        dk.dk_conv_fwd(L, W, b.xbar[g0 * S_:g1 * S_], ybar=b.ybar[g0 * S_:g1 * S_], ws=b.ws_fwd[si])
                    else:
                        dk.dk_linear_fwd(W, b.xbar[g0 * S_:g1 * S_], ybar=b.ybar[g0 * S_:g1 * S_], ws=b.ws_fwd[si])
                    dk.dk_decode_verify_m(b.ybar[g0 * S_:g1 * S_], Ainv_d[g0:g1], nvec_d[g0:g1], K, M, tol=1e-3,
                                          y=b.y[g0 * K:g1 * K], verdict=b.verdict[g0:g1], resid=b.resid[g0:g1],
                                          ws=b.ws_vf[si])
            if two:
                cur.wait_stream(side2)
            if ev:
                for e_ in ev[:4]: e_.record()
            dk.dk_wgrad_m(L, b.delta, B_d, gamma_d, b.xbar, K, M, dW=b.dW, scale=1.0, ws=b.ws_wg)
            if ev: ev[4].record()
            return
        if ev: ev[0].record()
        if args.rng_noise:
            dk.dk_encode_rng(b.X, A_d, K, M, 20220701, 10.0, xbar=b.xbar)
        else:
            dk.dk_encode_m(b.X, b.r, A_d, K, M, xbar=b.xbar)
        if ev: ev[1].record()
        if fork:
            side2.wait_stream(cur)
            with torch.cuda.stream(side2):
                dk.dk_wgrad_m(L, b.delta, B_d, gamma_d, b.xbar, K, M, dW=b.dW, scale=1.0, ws=b.ws_wg)
        if one_call:
            if ev: ev[2].record()
            dk.dk_conv_fwd_decode_verify(L, W, b.xbar, Ainv_d, nvec_d, K, tol=1e-3, y=b.y, verdict=b.verdict,
                                         resid=b.resid, ws=b.ws_fdv)
        else:
            if conv:
                dk.dk_conv_fwd(L, W, b.xbar, ybar=b.ybar, ws=b.ws_fwd)
            else:
                dk.dk_linear_fwd(W, b.xbar, ybar=b.ybar, ws=b.ws_fwd)
            if ev: ev[2].record()
            dk.dk_decode_verify_m(b.ybar, Ainv_d, nvec_d, K, M, tol=1e-3, y=b.y, verdict=b.verdict, resid=b.resid,
                                  ws=b.ws_vf)
        if ev: ev[3].record()
        if fork:
            cur.wait_stream(side2)
        else:
            dk.dk_wgrad_m(L, b.delta, B_d, gamma_d, b.xbar, K, M, dW=b.dW, scale=1.0, ws=b.ws_wg)
        if ev: ev[4].record()

    for i in range(max(args.warmup, nsets)):
        step(b=sets[i % nsets])
    torch.cuda.synchronize()
    ref = [t.clone() for t in (y, dW, verdict)]

    # Capture one step per buffer set into a HIP graph (the library allocates
    # nothing and never synchronises, so its launches can be recorded).  Only a
    # failure to capture falls back to eager launches; replays that differ from
    # the eager results are an error.
    graphs = None
    if not args.no_graph:
        try:
            graphs = []
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for b in sets:
                    g_ = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g_, stream=side):
                        step(fork=args.fork, b=b)
                    graphs.append(g_)
            torch.cuda.current_stream().wait_stream(side)
        except Exception as e:                      # noqa: BLE001 - capture refused: time eager launches
            sys.stderr.write("bench.py: HIP graph capture failed, timing eager launches (%s)\n" % e)
            graphs = None
        torch.cuda.synchronize()
        if graphs:
            for rep in range(3):
                for b, g_ in zip(sets, graphs):
                    for t in (b.y, b.dW):
                        t.zero_()
                    torch.cuda.synchronize()
                    g_.replay()
                    torch.cuda.synchronize()
                    if not all(torch.equal(a, c) for a, c in zip((b.y, b.dW, b.verdict), ref)):
                        raise RuntimeError("graph replay %d differs from the eager step" % rep)
            for i in range(args.warmup):
                graphs[i % nsets].replay()
            torch.cuda.synchronize()

    def timed(nsteps, use_sets, use_graphs):
        t0 = time.perf_counter()
        for i in range(nsteps):
            if use_graphs:
                use_graphs[i % len(use_graphs)].replay()
            else:
                step(b=use_sets[i % len(use_sets)])
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / nsteps * 1e3

    ms_per_step = timed(args.steps, sets, graphs)
    # for context: the same steps on one buffer set (inputs of the step before still cached)
    warm_ms_per_step = timed(args.steps, sets[:1], graphs[:1] if graphs else None) if nsets > 1 else ms_per_step

    # Eager pass with an event between the entry points (stage times).
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(events[i], b=sets[i % nsets])
    torch.cuda.synchronize()

    # Pass over the same K steps with every kernel launch bracketed by HIP
    # events on its launch stream (the brackets cost a few microseconds per
    # launch, so this pass is not the one `value` is taken from).
    dk.dk_profile_enable(True)
    for i in range(args.steps):
        step(b=sets[i % nsets])
    torch.cuda.synchronize()
    dk.dk_profile_enable(False)
    kernels = dk.dk_profile_read()
    # and a few launches on one set only, to report what warm inputs are worth
    warm_kernels = kernels
    if nsets > 1:
        dk.dk_profile_enable(True)
        for i in range(min(5, args.steps)):
            step(b=b0)
        torch.cuda.synchronize()
        dk.dk_profile_enable(False)
        warm_kernels = dk.dk_profile_read()

    for b in sets:
        assert int(b.verdict.sum().item()) == 0, "clean synthetic data must verify"
        assert torch.equal(b.dW, dW) and torch.equal(b.y, y), "buffer sets disagree"
    set_bytes = sum(t.numel() * t.element_size() for v in vars(b0).values()
                    for t in (v if isinstance(v, list) else [v]))
    graph = graphs
    stage_ms = {s: float(np.mean([e[i].elapsed_time(e[i + 1]) for e in events]))
                for i, s in enumerate(stages)}

    flop_fwd = 2.0 * G * S * L.macs_per_row         # executed: all K+2 encoded rows
    flop_step = 2.0 * flop_fwd                      # forward + weight gradient
    tflops = flop_step / (ms_per_step * 1e-3) / 1e12
    ab = algorithmic_bytes(K, G, n, m, M)

    # Dominant kernel = the contraction kernel with the longest average launch
    # (forward and weight gradient execute the same FLOP count per launch).
    contraction = {k: v for k, v in kernels.items()
                   if k.startswith(("conv_", "contract_", "dw_", "fused1x1_"))
                   and v[1] in (args.steps, args.steps * args.group_chunks)}
    dom = max(contraction, key=lambda k: contraction[k][0])
    dom_ms = contraction[dom][0]
    dom_warm_ms = warm_kernels.get(dom, (dom_ms, 0))[0]
    dom_tflops = flop_fwd / (dom_ms * 1e-3) / 1e12
    # What a contraction must move at least: both operands read once, the result
    # written once (forward: encodings, weights -> results; weight gradient:
    # mixed gradients, encodings -> dW).  Where that takes longer at 8 TB/s than
    # the FLOP at the matrix peak (few channels, 1x1 filters on large images,
    # depthwise), the kernel's yardstick is HBM, not MFMA.
    w_elems = float(np.prod(L.w_shape))
    contr_bytes = 4.0 * (G * S * (n + m) + w_elems)
    timed_note = ("HIP events around every launch of this kernel, %d eager launches after the timed region, "
                  "cycling through %d buffer sets of %.0f MB (avg_launch_ms); warm_launch_ms: %d launches on "
                  "one set" % (args.steps, nsets, set_bytes / 1e6, min(5, args.steps)))
    if contr_bytes / HBM_PEAK_GBPS / 1e9 > flop_fwd / MFMA_F32_PEAK_TFLOPS / 1e12:
        gbps = contr_bytes / (dom_ms * 1e-3) / 1e9
        roofline = {
            "kernel": dom, "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": gbps / HBM_PEAK_GBPS, "traffic": measured_traffic(args.workload, dom),
            "avg_launch_ms": dom_ms, "warm_launch_ms": dom_warm_ms, "bytes_per_launch": contr_bytes,
            "timed": timed_note,
        }
    else:
        roofline = {
            "kernel": dom, "bound": "mfma", "achieved": dom_tflops, "peak": MFMA_F32_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": dom_tflops / MFMA_F32_PEAK_TFLOPS,
            "traffic": measured_traffic(args.workload, dom),
            "avg_launch_ms": dom_ms, "warm_launch_ms": dom_warm_ms, "flop_per_launch": flop_fwd,
            "timed": timed_note,
        }
    kname = {"encode": "encode_rng" if args.rng_noise else "encode", "decode_verify": "decode_verify",
             "delta_mix": "delta_mix"}
    if args.rng_noise:
        ab["encode"] -= 4 * G * M * n          # the noise rows are not read
    hbm = {}
    for k, label in kname.items():
        if label in kernels:
            ms = kernels[label][0]
            hbm[k] = {"GBps": ab[k] / (ms * 1e-3) / 1e9, "frac": ab[k] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                      "bytes": ab[k], "avg_launch_ms": ms}

    # Floor of the whole step: every kernel at the roofline that bounds it --
    # each contraction the longer of FLOP / matrix peak and bytes / HBM peak,
    # each mixing kernel its algorithmic bytes / HBM peak.
    # Where a fused kernel ran, its floor takes the place of the two it replaces:
    # forward + decode + verify reads the encodings and writes the K decoded rows;
    # the weight gradient with the mixing in its loader reads the K gradients.
    flop_ms = flop_fwd / MFMA_F32_PEAK_TFLOPS / 1e12 * 1e3
    hbm_ms = lambda nbytes: nbytes / HBM_PEAK_GBPS / 1e9 * 1e3
    fwd_bytes, wg_bytes, mix_bytes = contr_bytes, contr_bytes, dict(ab)
    if "fused1x1_fwd_decode_verify" in kernels:
        fwd_bytes = 4.0 * (G * S * n + w_elems + G * K * m)
        mix_bytes.pop("decode_verify")
    if "fused1x1_wgrad" in kernels:
        wg_bytes = 4.0 * (G * K * m + G * S * n + w_elems)
        mix_bytes.pop("delta_mix")
    mix_floor_ms = hbm_ms(sum(mix_bytes.values()))
    floor_ms = max(flop_ms, hbm_ms(fwd_bytes)) + max(flop_ms, hbm_ms(wg_bytes)) + mix_floor_ms
    hbm_part_ms = (mix_floor_ms + (hbm_ms(fwd_bytes) if hbm_ms(fwd_bytes) > flop_ms else 0.0)
                   + (hbm_ms(wg_bytes) if hbm_ms(wg_bytes) > flop_ms else 0.0))

    out = {
        "metric": "masked-layer TFLOP/s (fwd+wgrad, executed on all K+2 encoded rows), whole hot path",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wname + (", noise drawn in the encoding kernel" if args.rng_noise else ""),
                   "K": K, "G": G, "layer": L.asdict(),
                   "launch": ("HIP graph replay of one captured step"
                              + (", weight gradient on a second branch" if args.fork else "")) if graph else "eager"},
        "pct_mfma_peak": 100.0 * tflops / MFMA_F32_PEAK_TFLOPS,
        "decoded_samples_per_s": G * K / (ms_per_step * 1e-3),
        "decoded_samples_per_s_fwd_only": G * K / ((stage_ms["encode"] + stage_ms["fwd"]
                                                    + stage_ms["decode_verify"]) * 1e-3),
        "stage_note": ("fwd = 0, decode_verify = forward + decode + verify in one call"
                       if one_call else "one entry point per stage"),
        "effective_tflops": tflops * K / S,
        "stage_ms": stage_ms,
        "fwd_stage_tflops": flop_fwd / (stage_ms["fwd"] * 1e-3) / 1e12,
        "wgrad_stage_tflops": flop_fwd / (stage_ms["wgrad"] * 1e-3) / 1e12,
        "roofline": roofline,
        "hbm_kernels": hbm,
        "kernel_ms": {k: v[0] for k, v in kernels.items()},
        "kernel_ms_sum": float(sum(v[0] * v[1] for v in kernels.values()) / args.steps),
        "warm_ms_per_step": warm_ms_per_step,
        "roofline_floor_ms": floor_ms,
        "step_frac": floor_ms / ms_per_step,
        "step_bound": "hbm" if hbm_part_ms > 0.5 * floor_ms else "mfma",
        "buffers": "%d sets of %.0f MB used in turn in every pass (timed region included)" % (nsets, set_bytes / 1e6),
    }
    if args.with_dgrad:
        dx = torch.empty((G * K,) + L.in_shape, **f32)
        ws_dg = torch.empty(dk.load().dk_dgrad_workspace_bytes(C.byref(dk.DkLayer.of(L)), G * K), **u8)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for _ in range(3):
            dk.dk_dgrad(L, W, b0.delta, dx=dx, ws=ws_dg)
        ev[0].record()
        for _ in range(args.steps):
            dk.dk_dgrad(L, W, b0.delta, dx=dx, ws=ws_dg)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / args.steps
        out["dgrad_ms"] = ms
        out["dgrad_tflops"] = 2.0 * G * K * L.macs_per_row / (ms * 1e-3) / 1e12
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(d)
    return out


if __name__ == "__main__":
    main()
