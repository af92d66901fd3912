#!/usr/bin/env python3
"""Benchmark of the quantized matrix-product path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch that is
already resident in HBM: abs-max and quant_int of the activations, dot'_int on
the int8 matrix cores with the dequantize + bias + ReLU epilogue, re-quantization
of the intermediate, the second product (arxiv 1805.12096, Sections 4.2-4.3).
The default workload is the Transformer-base FFN block in int8 at M = 8192
tokens (the paper's GPU batch size, Section 2.3; widths from Table 1).  Parameter
preparation is memoized (Section 4.3) and therefore outside the timed region.

Prints ONE JSON line.  `value` is useful integer operations (2 M N K per
product) per second for the whole step.  Beside it: the roofline position of
the longest-running kernel (durations measured here with HIP events on the
launch stream), the greedy output-layer workload (tokens/s, GB/s), the int16
Transformer-big FFN, and the CPU oracle timed on this host on a bounded sample
of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file on the default workload
# (profiles/ffn_int8_hbm_counters.txt: FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 after calibration on a known copy).
MEASURED_TRAFFIC = {
    "gemm1 single pass: bias+relu -> max|H| -> quant_int(H)": 29.7e6,
    "(two-pass) gemm1 pass 1: bias+relu -> max|H|": 12.8e6,
    "(two-pass) gemm1 pass 2: bias+relu -> quant_int(H)": 29.6e6,
    "gemm2+bias": 41.6e6,
    "absmax+quant_int(A) [2 launches]": 21.2e6,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-extras", action="store_true", help="skip the output-layer and int16 side workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-graph", action="store_true", help="launch directly instead of replaying a HIP graph")
    ap.add_argument("--no-autotune", action="store_true", help="keep the shape heuristic instead of timing tile variants")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy, the known-size reference for scaling HBM counters")
    ap.add_argument("--no-parity", action="store_true",
                    help="skip the per-config parity / overflow report of the CPU leg")
    ap.add_argument("--cpu-rows", type=int, default=8192, help="token rows of the workload the oracle is timed on")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1805_12096_amd as mq
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    mq.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    QT = {8: torch.int8, 16: torch.int16}

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    def time_events(fn, iters, warm):
        """Average duration of fn in microseconds, HIP events on the launch stream."""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    def graphed(fn, reps=1):
        """Capture `reps` calls of fn into a HIP graph; returns a replay callable (or a plain loop)."""
        if args.no_graph:
            return (lambda: [fn() for _ in range(reps)])
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(reps):
                fn()
        return g.replay

    STEPS_PER_GRAPH = 10
    SPIN_UP_MS = 40.0

    def time_steps(fn, steps, warm):
        """Microseconds per step over EXACTLY `steps` steps after `warm` untimed ones.  Steps are replayed as HIP
        graphs of STEPS_PER_GRAPH consecutive steps (the remainder one step at a time): a graph launch costs
        several microseconds of its own, which a loop over batches would not pay once per batch."""
        one = graphed(fn, 1)
        many = graphed(fn, STEPS_PER_GRAPH) if steps >= STEPS_PER_GRAPH and not args.no_graph else None
        # The device needs some tens of milliseconds of steady work to settle at its working clock after the idle
        # gaps of set-up (the first of two identical measurements in a process came out 5 % slower): the step runs
        # untimed for SPIN_UP_MS before the warm-up steps.
        t_spin = time.perf_counter()
        while (time.perf_counter() - t_spin) * 1e3 < SPIN_UP_MS:
            for _ in range(8):
                (many or one)()
            torch.cuda.synchronize()
        for _ in range(warm):
            one()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        done = 0
        if many is not None:
            for _ in range(steps // STEPS_PER_GRAPH):
                many()
                done += STEPS_PER_GRAPH
        while done < steps:
            one()
            done += 1
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / steps

    def time_kernel(fn, reps=10, iters=20):
        """Average duration of one call of fn (us): `reps` back-to-back copies replayed as one graph, so
        that host launch overhead does not hide kernels of a few microseconds."""
        return time_events(graphed(fn, reps), iters, 3) / reps

    QWS = mq.mq_quantize_absmax_ws_bytes()     # workspace of the abs-max + quant_int call

    # ------------------------------------------------------------ FFN workloads
    class FFN:
        def __init__(self, c, bits):
            self.bits = bits
            self.A = to_dev(c["A"])
            self.M, self.d = self.A.shape
            self.f = c["W1t"].shape[0]
            self.p1 = mq.prepare_weight(to_dev(c["W1t"]), bits)
            self.p2 = mq.prepare_weight(to_dev(c["W2t"]), bits)
            self.b1, self.b2 = to_dev(c["b1"]), to_dev(c["b2"])
            M, d, f = self.M, self.d, self.f
            self.s1 = torch.empty(1, dtype=torch.float32, device=dev)
            self.s2 = torch.empty(1, dtype=torch.float32, device=dev)
            self.hmax = torch.zeros(1, dtype=torch.float32, device=dev)
            # activations live in the packed (fragment-order) layout the product kernels stream
            self.q1 = torch.empty(mq.mq_packed_bytes(bits, M, d), dtype=torch.uint8, device=dev)
            self.q2 = torch.empty(mq.mq_packed_bytes(bits, M, f), dtype=torch.uint8, device=dev)
            self.H = torch.empty((M, f), dtype=torch.float32, device=dev)
            self.Y = torch.empty((M, d), dtype=torch.float32, device=dev)
            self.ops = 2 * (2 * M * d * f)
            self.ws_bytes = mq.mq_ffn_ws_bytes(M, d, f) if bits == 8 else mq.mq_ffn_i16_ws_bytes(M, d, f)
            self.ws = torch.empty(max(self.ws_bytes, QWS), dtype=torch.uint8, device=dev)
            if bits == 8:
                # the timed block runs on a workspace of its own, prepared once (agreement words zeroed) and left
                # prepared by every call: nothing else may write to it
                self.ws_ffn = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
                mq.mq_ffn_ws_prepare(self.ws_ffn, self.ws_bytes, M, d, f)
            self.part_bytes = mq.mq_gemm_amax_ws_bytes(M, f)
            self.part = torch.empty(self.part_bytes, dtype=torch.uint8, device=dev)

        # the individual launches, so each can be timed alone
        def k_absmax(self):
            mq.mq_absmax_f32(self.A, self.A.numel(), self.s1)

        def k_scale1(self):
            mq.mq_scale_from_amax(self.s1, self.bits, self.s1)

        def k_quant1(self):
            mq.mq_quantize_pack_f32(self.A, self.M, self.d, self.bits, self.s1, self.q1)

        def k_gemm1(self):
            mq.mq_gemm_dequant_packed(self.q1, self.p1.packed, self.bits, self.M, self.f, self.d, self.s1,
                                      self.p1.scale, self.b1, True, self.H, self.hmax)

        def k_scale2(self):
            mq.mq_scale_from_amax(self.hmax, self.bits, self.s2)

        def k_quant2(self):
            mq.mq_quantize_pack_f32(self.H, self.M, self.f, self.bits, self.s2, self.q2)

        def k_gemm2(self):
            mq.mq_gemm_dequant_packed(self.q2, self.p2.packed, self.bits, self.M, self.d, self.f, self.s2,
                                      self.p2.scale, self.b2, False, self.Y, None)

        def fused_step(self):
            if self.bits == 16:
                mq.mq_ffn_i16_f32(self.A, self.M, self.d, self.f, self.p1.packed, self.p1.scale, self.b1,
                                  self.p2.packed, self.p2.scale, self.b2, self.Y, self.ws, self.ws_bytes)
                return
            mq.mq_ffn_i8_f32_prepared(self.A, self.M, self.d, self.f, self.p1.packed, self.p1.scale, self.b1,
                                      self.p2.packed, self.p2.scale, self.b2, self.Y, self.ws_ffn, self.ws_bytes)

        def plain_step(self):
            # the entry point that takes any workspace: one more launch, which zeroes the agreement words
            mq.mq_ffn_i8_f32(self.A, self.M, self.d, self.f, self.p1.packed, self.p1.scale, self.b1,
                             self.p2.packed, self.p2.scale, self.b2, self.Y, self.ws_ffn, self.ws_bytes)

        def step(self):
            self.k_absmax()
            self.k_scale1()
            self.k_quant1()
            self.hmax.zero_()
            self.k_gemm1()
            self.k_scale2()
            self.k_quant2()
            self.k_gemm2()

        # building blocks of the fused step, for per-kernel timing
        def k_absmax_quant1(self):
            mq.mq_quantize_absmax_pack_f32(self.A, self.M, self.d, self.bits, self.q1, self.s1, self.ws, QWS)

        def k_gemm1_amax(self):
            mq.mq_gemm_amax_packed(self.q1, self.p1.packed, self.M, self.f, self.d, self.s1, self.p1.scale,
                                   self.b1, True, self.part, self.part_bytes)

        def k_gemm1_requant(self):
            mq.mq_gemm_requant_packed(self.q1, self.p1.packed, self.M, self.f, self.d, self.s1, self.p1.scale,
                                      self.b1, True, self.part, self.part_bytes, self.s2, self.q2)

        def k_gemm1_single(self):
            mq.mq_gemm_requant_single_packed(self.q1, self.p1.packed, self.M, self.f, self.d, self.s1,
                                             self.p1.scale, self.b1, True, self.part, self.part_bytes,
                                             self.s2, self.q2)

        def k_clear(self):
            self.part[:8].zero_()       # stands in for the 1-block clear launch inside k_gemm1_single

        def kernel_table(self, fused):
            """name -> (callable, algorithmic HBM bytes, integer ops issued on the matrix cores)."""
            M, d, f, e = self.M, self.d, self.f, self.bits // 8
            mm = 2 * M * d * f * (4 if self.bits == 16 else 1)       # int16 = four int8 products
            if fused:
                return {
                    "absmax+quant_int(A) [2 launches]": (self.k_absmax_quant1, 2 * 4 * M * d + e * M * d, 0),
                    "gemm1 single pass: bias+relu -> max|H| -> quant_int(H)":
                        (self.k_gemm1_single, e * M * d + e * d * f + e * M * f, mm),
                    "gemm2+bias": (self.k_gemm2, e * M * f + e * d * f + 4 * M * d, mm),
                    # the two-pass form of gemm1, used when the result has more tiles than the chip holds
                    "(two-pass) gemm1 pass 1: bias+relu -> max|H|": (self.k_gemm1_amax, e * M * d + e * d * f, mm),
                    "(two-pass) gemm1 pass 2: bias+relu -> quant_int(H)":
                        (self.k_gemm1_requant, e * M * d + e * d * f + e * M * f, mm),
                }
            return {
                "absmax(A)": (self.k_absmax, 4 * M * d, 0),
                "quant_int(A)": (self.k_quant1, 4 * M * d + e * M * d, 0),
                "gemm1+bias+relu+amax": (self.k_gemm1, e * M * d + e * d * f + 4 * M * f, mm),
                "quant_int(H)": (self.k_quant2, 4 * M * f + e * M * f, 0),
                "gemm2+bias": (self.k_gemm2, e * M * f + e * d * f + 4 * M * d, mm),
            }

    def run_ffn(c, bits, steps, warmup, fused):
        w = FFN(c, bits)
        step = w.fused_step if fused else w.step
        step()
        torch.cuda.synchronize()
        us = time_steps(step, steps, warmup)
        if fused:
            w.step()            # leaves s2 / q2 of the unfused chain in place for the gemm2 timing
        per_kernel = {}
        for kname, (fn, nbytes, mops) in w.kernel_table(fused and bits == 8).items():
            kus = time_kernel(fn)
            if fn == w.k_gemm1_single:
                # the stand-alone entry point spends one extra tiny launch on clearing its two counters (inside
                # the block that is the first kernel's job); its share is measured the same way and taken off
                kus -= time_kernel(w.k_clear)
            per_kernel[kname] = {"us": round(kus, 2), "alg_bytes": nbytes, "GBps": round(nbytes / kus / 1e3, 1),
                                 "mfma_TOPS": round(mops / kus / 1e6, 1)}
        return w, us, per_kernel

    # Section 4.4 in miniature: time the tile variants once per product shape and freeze the fastest
    tuned = {}

    def autotune(bits, M_, N_, K_):
        if args.no_autotune:
            return
        nb_ = mq.mq_autotune_ws_bytes(bits, M_, N_, K_)
        ws_ = torch.empty(nb_, dtype=torch.uint8, device=dev)
        best, us_ = mq.mq_autotune_gemm(bits, M_, N_, K_, 20, ws_, nb_)
        tuned[f"i{bits} {M_}x{N_}x{K_}"] = {"variant": best, "us": round(us_, 2)}
        del ws_

    # ----------------------------------------------------------------- config 2
    autotune(8, 8192, 2048, 512)
    autotune(8, 8192, 512, 2048)
    c2 = workloads.config2()
    w2, us2, pk2 = run_ffn(c2, 8, args.steps, args.warmup, fused=True)
    tops2 = w2.ops / us2 / 1e6
    us2_chain = time_steps(w2.step, args.steps, args.warmup)     # the same block call by call, H in fp32
    us2_plain = time_steps(w2.plain_step, args.steps, args.warmup)

    # the dominant launch of the timed step: the single-pass first product (the longest one; the second product is
    # within a few percent of it, so the choice is fixed rather than left to run-to-run noise), else the longest
    single = [k for k in pk2 if k.startswith("gemm1 single pass")]
    dom = single[0] if single else max((k for k in pk2 if not k.startswith("(two-pass)") and "launches]" not in k),
                                       key=lambda k: pk2[k]["us"])
    dk = pk2[dom]
    hbm_frac = dk["GBps"] / PEAK_HBM_GBS
    mfma_frac = dk["mfma_TOPS"] / PEAK_INT8_TOPS
    # the roof that binds this kernel at its algorithmic traffic / op count
    t_hbm = dk["alg_bytes"] / (PEAK_HBM_GBS * 1e3)
    t_mfma = (dk["mfma_TOPS"] * dk["us"]) / PEAK_INT8_TOPS
    if t_hbm >= t_mfma:
        roofline = {"bound": "hbm", "achieved": dk["GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(hbm_frac, 4)}
    else:
        roofline = {"bound": "mfma", "achieved": dk["mfma_TOPS"], "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                    "frac": round(mfma_frac, 4)}
    roofline.update({"kernel": dom, "us": dk["us"], "traffic": MEASURED_TRAFFIC.get(dom)})

    result = {
        "metric": "int8 GEMM TOPS (useful 2MNK ops of the FFN block / step time)",
        "value": round(tops2, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us2 / 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i8", "data": "synthetic",
        "config": {"workload": "transformer-base FFN int8: [8192x512]x[512x2048]+bias+ReLU, requantize, "
                               "[8192x2048]x[2048x512]+bias; per-tensor abs-max scales",
                   "M": w2.M, "d": w2.d, "ffn": w2.f, "graph": not args.no_graph,
                   "steps_per_graph": 1 if args.no_graph else STEPS_PER_GRAPH,
                   "path": "mq_ffn_i8_f32_prepared (3 launches, H never stored in fp32; the workspace's agreement "
                           "words are zeroed once by mq_ffn_ws_prepare outside the timed region and left zero by "
                           "every call)"},
        "unfused_chain": {"us_per_step": round(us2_chain, 2), "TOPS": round(w2.ops / us2_chain / 1e6, 2),
                          "what": "abs-max, scale, quant_int, product(+max|H|), scale, quant_int, product as 9 launches, "
                                  "H stored and re-read in fp32"},
        "plain_entry": {"us_per_step": round(us2_plain, 2), "TOPS": round(w2.ops / us2_plain / 1e6, 2),
                        "what": "mq_ffn_i8_f32 on any workspace: 4 launches, the first one zeroes the agreement words"},
        "pct_int8_mfma_peak": round(100 * tops2 / PEAK_INT8_TOPS, 2),
        "roofline": roofline,
        "kernels": pk2,
    }

    if args.copy_calibration:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------- extras
    if not args.no_extras:
        extras = {}
        # greedy output layer (one decode step, 300 sentences, 36000-word tied embedding)
        c3 = workloads.config3()
        Hd = to_dev(c3["Hd"])
        M, d = Hd.shape
        V = c3["E"].shape[0]
        pe = mq.prepare_weight(to_dev(c3["E"]), 8)
        s = torch.empty(1, dtype=torch.float32, device=dev)
        q = torch.empty((M, d), dtype=torch.int8, device=dev)
        nws = mq.mq_argmax_ws_bytes(M, V)
        ws = torch.empty(nws, dtype=torch.uint8, device=dev)
        tok = torch.empty(M, dtype=torch.int32, device=dev)
        val = torch.empty(M, dtype=torch.float32, device=dev)

        qp = torch.empty(mq.mq_packed_bytes(8, M, d), dtype=torch.uint8, device=dev)
        qws = torch.empty(QWS, dtype=torch.uint8, device=dev)
        # the output layer's quantizer runs on a workspace of its own, prepared once (one kernel per call, which
        # leaves its agreement words zero); the other workloads below use the entry point that takes any workspace
        qws_out = torch.empty(QWS, dtype=torch.uint8, device=dev)
        mq.mq_quantize_absmax_ws_prepare(qws_out, QWS)

        def out_step():
            mq.mq_quantize_absmax_pack_f32_prepared(Hd, M, d, 8, qp, s, qws_out, QWS)
            mq.mq_gemm_argmax_packed(qp, pe.packed, M, V, d, s, pe.scale, tok, val, ws, nws)

        out_step()

        def warm_round():             # the same 16 steps as the cold round, on one embedding that stays cached
            for _ in range(16):
                out_step()

        us3 = time_events(graphed(warm_round), max(5, args.steps // 10), 2) / 16
        us3k = time_kernel(lambda: mq.mq_gemm_argmax_packed(qp, pe.packed, M, V, d, s, pe.scale, tok, val, ws, nws))
        # cold: 16 distinct embeddings (295 MB) in rotation, so the 256 MB last-level cache cannot hold them
        pes = [pe] + [mq.prepare_weight(torch.randn(V, d, device=dev) * 0.05, 8) for _ in range(15)]

        def cold_round():
            for q_ in pes:
                mq.mq_quantize_absmax_pack_f32_prepared(Hd, M, d, 8, qp, s, qws_out, QWS)
                mq.mq_gemm_argmax_packed(qp, q_.packed, M, V, d, s, q_.scale, tok, val, ws, nws)

        us3c = time_events(graphed(cold_round), max(5, args.steps // 10), 2) / len(pes)
        del pes
        alg3 = V * d + 4 * M * d + 8 * M
        extras["output_layer_argmax"] = {
            "workload": f"[{M}x{d}] hidden x tied embedding [{V}x{d}] int8, abs-max + quant_int (one kernel on a prepared workspace) + fused arg-max",
            "us_per_step_warm": round(us3, 2), "tokens_per_s_warm": round(M / us3 * 1e6, 0),
            "GBps_alg_warm": round(alg3 / us3 / 1e3, 1),
            "us_per_step_cold": round(us3c, 2), "tokens_per_s_cold": round(M / us3c * 1e6, 0),
            "GBps_alg_cold": round(alg3 / us3c / 1e3, 1), "pct_hbm_peak_cold": round(100 * alg3 / us3c / 1e3 / PEAK_HBM_GBS, 1),
            "TOPS_warm": round(2 * M * V * d / us3 / 1e6, 1), "argmax_product_only_us": round(us3k, 2)}
        # short-listed output layer: 100 most frequent ids + 100 candidates per source word of a 384-word batch
        rng = np.random.default_rng(workloads.BASE_SEED + 33)
        sl_host = np.unique(np.concatenate([np.arange(100), rng.integers(0, V, size=384 * 100 // 8)])).astype(np.int32)
        sl = to_dev(sl_host)
        us3s = time_kernel(lambda: mq.mq_gemm_argmax_shortlist(qp, pe.packed, sl, sl.numel(), M, V, d, s, pe.scale,
                                                                tok, val, ws, nws))
        extras["output_layer_shortlist"] = {"shortlist_rows": int(sl.numel()), "argmax_product_only_us": round(us3s, 2)}

        # beam search (Table 2, b = 2 / b = 4): 300 sentences x beam hypotheses, the k = beam best words per row with
        # log-probabilities (softmax normaliser fused into the streaming kernel)
        beam_out = {}
        for beam in (2, 4):
            rows_b = M * beam
            Hb = torch.randn(rows_b, d, device=dev)
            qb = torch.empty(mq.mq_packed_bytes(8, rows_b, d), dtype=torch.uint8, device=dev)
            sb = torch.empty(1, dtype=torch.float32, device=dev)
            mq.mq_quantize_absmax_pack_f32(Hb, rows_b, d, 8, qb, sb, qws, QWS)
            nwb = mq.mq_topk_ws_bytes(rows_b, V, beam)
            wsb = torch.empty(nwb, dtype=torch.uint8, device=dev)
            tokb = torch.empty((rows_b, beam), dtype=torch.int32, device=dev)
            lpb = torch.empty((rows_b, beam), dtype=torch.float32, device=dev)
            usb = time_kernel(lambda: mq.mq_gemm_topk_packed(qb, pe.packed, None, 0, rows_b, V, d, sb, pe.scale, beam,
                                                             tokb, lpb, wsb, nwb))
            beam_out[f"beam{beam}"] = {"rows": rows_b, "us": round(usb, 2),
                                       "TOPS": round(2 * rows_b * V * d / usb / 1e6, 1)}
            del Hb, qb, wsb
        extras["output_layer_beam_topk"] = beam_out

        # the same FFN block with the paper's fixed multipliers (127/2 on inputs clipped to [-2, 2]): no abs-max
        # pass, the intermediate is quantized in the first product's epilogue -> three launches
        sc = torch.full((1,), 63.5, dtype=torch.float32, device=dev)
        w2.p1f = mq.prepare_weight(to_dev(c2["W1t"] * np.float32(8)), 8, scale=sc)
        w2.p2f = mq.prepare_weight(to_dev(c2["W2t"] * np.float32(8)), 8, scale=sc)

        def fixed_step():
            mq.mq_quantize_pack_f32(w2.A, w2.M, w2.d, 8, sc, w2.q1)
            mq.mq_gemm_requant_fixed_packed(w2.q1, w2.p1f.packed, w2.M, w2.f, w2.d, sc, w2.p1f.scale, w2.b1, True, sc, w2.q2)
            mq.mq_gemm_dequant_packed(w2.q2, w2.p2f.packed, 8, w2.M, w2.d, w2.f, sc, w2.p2f.scale, w2.b2, False, w2.Y, None)

        fixed_step()
        usf = time_steps(fixed_step, args.steps, args.warmup)
        extras["ffn_base_int8_fixed_multipliers"] = {
            "what": "same block, multipliers fixed at 63.5 as in the paper (no abs-max), 3 launches",
            "us_per_step": round(usf, 2), "TOPS": round(w2.ops / usf / 1e6, 1)}

        # int16 Transformer-big FFN
        autotune(16, 8192, 4096, 1024)
        autotune(16, 8192, 1024, 4096)
        c4 = workloads.config4()
        w4, us4, pk4 = run_ffn(c4, 16, max(10, args.steps // 10), max(3, args.warmup // 5), fused=True)
        extras["ffn_big_int16"] = {
            "workload": "[8192x1024]x[1024x4096]+bias+ReLU, requantize, [8192x4096]x[4096x1024]+bias, int16, "
                        "one mq_ffn_i16_f32 call (5 launches); the kernel table times the call-by-call pieces",
            "us_per_step": round(us4, 1), "TOPS_useful": round(w4.ops / us4 / 1e6, 1),
            "pct_int8_mfma_peak_issued": round(100 * 4 * w4.ops / us4 / 1e6 / PEAK_INT8_TOPS, 2),
            "kernels": pk4}
        # the paper's 16-bit scheme (Section 4.2): every tensor times 2^10, no abs-max; the first product writes the
        # second one's packed 16-bit input from its epilogue, H is never stored in fp32
        sc16 = torch.full((1,), 1024.0, dtype=torch.float32, device=dev)
        p1x = mq.prepare_weight(to_dev(c4["W1t"]), 16, scale=sc16)
        p2x = mq.prepare_weight(to_dev(c4["W2t"]), 16, scale=sc16)

        def fixed16_step():
            mq.mq_quantize_pack_f32(w4.A, w4.M, w4.d, 16, sc16, w4.q1)
            mq.mq_gemm_requant_fixed_packed_i16(w4.q1, p1x.packed, w4.M, w4.f, w4.d, sc16, sc16, w4.b1, True, sc16, w4.q2)
            mq.mq_gemm_dequant_packed(w4.q2, p2x.packed, 16, w4.M, w4.d, w4.f, sc16, sc16, w4.b2, False, w4.Y, None)

        fixed16_step()
        usf16 = time_steps(fixed16_step, max(10, args.steps // 10), max(3, args.warmup // 5))
        extras["ffn_big_int16_fixed_multiplier"] = {
            "what": "same block, every multiplier 2^10 as in the paper (no abs-max, 4 launches, H written as packed int16)",
            "us_per_step": round(usf16, 1), "TOPS_useful": round(w4.ops / usf16 / 1e6, 1),
            "pct_int8_mfma_peak_issued": round(100 * 4 * w4.ops / usf16 / 1e6 / PEAK_INT8_TOPS, 2)}
        del w4, p1x, p2x

        # single int16 product of the 384-word CPU batch (latency case: reported in microseconds)
        c1 = workloads.config1()
        A1 = to_dev(c1["A"])
        p1_ = mq.prepare_weight(to_dev(c1["Wt"]), 16)
        b1_ = to_dev(c1["bias"])
        q1_ = torch.empty(mq.mq_packed_bytes(16, 384, 512), dtype=torch.uint8, device=dev)
        s1_ = torch.empty(1, dtype=torch.float32, device=dev)
        Y1_ = torch.empty((384, 512), dtype=torch.float32, device=dev)

        def c1_step():
            mq.mq_quantize_absmax_pack_f32(A1, 384, 512, 16, q1_, s1_, qws, QWS)
            mq.mq_gemm_dequant_packed(q1_, p1_.packed, 16, 384, 512, 512, s1_, p1_.scale, b1_, False, Y1_, None)

        c1_step()
        us1 = time_steps(c1_step, args.steps, args.warmup)
        extras["single_int16_product_384x512x512"] = {"us_per_call": round(us1, 2), "launches": 3,
                                                      "TOPS_useful": round(2 * 384 * 512 * 512 / us1 / 1e6, 2)}

        # all parameter products of one greedy decode step of the 6-layer base AAN decoder + output layer
        c5 = workloads.config5()
        g5 = []
        for g in c5["gemms"]:
            Ad = to_dev(g["A"])
            N5, K5 = g["Wt"].shape
            g5.append((Ad, mq.prepare_weight(to_dev(g["Wt"]), 8), to_dev(g["bias"]), bool(g["relu"]), N5, K5,
                       torch.empty((300, N5), dtype=torch.float32, device=dev)))
        nlw = max(mq.mq_linear_ws_bytes(8, 300, k_) for _, _, _, _, _, k_, _ in g5)
        lws = torch.empty(nlw, dtype=torch.uint8, device=dev)
        Hd5 = to_dev(c5["output"]["Hd"])
        pe5 = mq.prepare_weight(to_dev(c5["output"]["E"]), 8)

        def c5_step():
            for Ad, pw_, b_, relu_, N5, K5, Ybuf in g5:      # abs-max, quant_int, product, bias (+ReLU) per call
                mq.mq_linear_f32(Ad, 300, K5, None, pw_.packed, pw_.scale, 8, N5, b_, relu_, Ybuf, None, lws, nlw)
            mq.mq_quantize_absmax_pack_f32(Hd5, M, d, 8, qp, s, qws, QWS)
            mq.mq_gemm_argmax_packed(qp, pe5.packed, M, V, d, s, pe5.scale, tok, val, ws, nws)

        c5_step()
        us5 = time_events(graphed(c5_step), max(10, args.steps // 4), 3)
        ops5 = sum(2 * 300 * n_ * k_ for _, _, _, _, n_, k_, _ in g5) + 2 * M * V * d
        extras["aan_decode_step_products"] = {
            "workload": "42 int8 parameter products of a 6-layer base AAN decoder step (300 sentences) + greedy output layer",
            "us_per_step": round(us5, 1), "launches": sum(2 if k_ <= 1024 else 3 for _, _, _, _, _, k_, _ in g5) + 4, "tokens_per_s": round(300 / us5 * 1e6, 0),
            "TOPS_useful": round(ops5 / us5 / 1e6, 1)}
        del g5

        # the same decode step with its real dependencies: six chained decoder layers (running average, averaging
        # block's network and gate, source attention over 25 positions, feed-forward block, layer normalisations)
        # and the greedy output layer, as one HIP graph
        cc = workloads.config5_chained()
        Lc = []
        for Pl in cc["layers"]:
            prods = {n_: (mq.prepare_weight(to_dev(Pl[n_]["Wt"]), 8), to_dev(Pl[n_]["bias"]))
                     for n_ in ("aan_ffn1", "aan_ffn2", "aan_gate", "ctx_q", "ctx_o", "ffn1", "ffn2")}
            norms = {n_: (to_dev(Pl[n_]["gamma"]), to_dev(Pl[n_]["beta"])) for n_ in ("ln1", "ln2", "ln3")}
            Lc.append(mq.aan_layer(prods, norms, 512, 2048, 2048))
        KVc = [(to_dev(k_), to_dev(v_)) for k_, v_ in cc["KV"]]
        gpc = [to_dev(g_) for g_ in cc["g_prev"]]
        gnc = [torch.empty_like(g_) for g_ in gpc]
        xs = [to_dev(cc["x0"])] + [torch.empty((300, 512), dtype=torch.float32, device=dev) for _ in Lc]
        nwl = mq.mq_aan_layer_ws_bytes(300, 512, 2048, 2048)
        wsl = torch.empty(nwl, dtype=torch.uint8, device=dev)
        pec = mq.prepare_weight(to_dev(cc["E"]), 8)

        def chained_step():
            for l_, layer_ in enumerate(Lc):
                mq.mq_aan_layer_f32(layer_, xs[l_], gpc[l_], cc["t"], KVc[l_][0], KVc[l_][1], 300, 25, cc["heads"], True,
                                    True, 1e-6, xs[l_ + 1], gnc[l_], wsl, nwl)
            mq.mq_quantize_absmax_pack_f32(xs[-1], M, d, 8, qp, s, qws, QWS)
            mq.mq_gemm_argmax_packed(qp, pec.packed, M, V, d, s, pec.scale, tok, val, ws, nws)

        chained_step()
        usc = time_events(graphed(chained_step), max(10, args.steps // 4), 3)
        extras["aan_decode_step_chained"] = {
            "workload": "one greedy decode step of the 6-layer base AAN decoder for 300 sentences at position 20: "
                        "42 int8 products with their float glue (running average, gate, source attention over 25 "
                        "positions x 8 heads, layer normalisations) and the greedy output layer, one HIP graph",
            "us_per_step": round(usc, 1), "launches": 6 * 14 + 4, "tokens_per_s": round(300 / usc * 1e6, 0)}
        del Lc, KVc, wsl
        result["extras"] = extras
    if tuned:
        result["autotuned"] = tuned

    # ------------------------------------------------------------- CPU baseline
    if not args.no_cpu:
        import oracle
        rows = min(args.cpu_rows, c2["A"].shape[0])
        A = c2["A"][:rows]
        qW1, sW1 = oracle.quant_int_absmax(c2["W1t"], 8)      # memoized, not timed
        qW2, sW2 = oracle.quant_int_absmax(c2["W2t"], 8)
        t0 = time.perf_counter()
        qA, sA = oracle.quant_int_absmax(A, 8)
        Hh = oracle.dequant_bias(oracle.dot_int(qA, qW1), sA, sW1, c2["b1"], True)
        qH, sH = oracle.quant_int_absmax(Hh, 8)
        oracle.dequant_bias(oracle.dot_int(qH, qW2), sH, sW2, c2["b2"], False)
        dt = time.perf_counter() - t0
        ops = 2 * (2 * rows * w2.d * w2.f)
        result["cpu_baseline"] = {"value": round(ops / dt / 1e12, 5), "unit": "TOPS", "cores": oracle.num_threads(),
                                  "kind": "oracle", "seconds": round(dt, 2),
                                  "sample": f"first {rows} of {w2.M} token rows of the same FFN workload, "
                                            "weights pre-quantized (memoized)"}
        # the latency-bound configs on the oracle, all host threads and one thread (seconds per call)
        nthr = oracle.num_threads()
        c1o, c3o = workloads.config1(), workloads.config3()
        side = {}
        for label, n_ in (("all_threads", nthr), ("one_thread", 1)):
            oracle.set_num_threads(n_)
            t0 = time.perf_counter()
            oracle.linear(c1o["A"], c1o["Wt"], 16, c1o["bias"], False)
            t1 = time.perf_counter()
            oracle.greedy_output_layer(c3o["Hd"], c3o["E"])
            t2 = time.perf_counter()
            side[label] = {"config1_int16_product_s": round(t1 - t0, 4), "config3_output_layer_s": round(t2 - t1, 3)}
        oracle.set_num_threads(nthr)
        result["cpu_baseline"]["other_configs"] = side
        if not args.no_parity:
            result["cpu_baseline"]["parity"] = parity_report(mq, torch, dev, to_dev, oracle)
    print(json.dumps(result))


def parity_report(mq, torch, dev, to_dev, oracle):
    """Per benchmark config: does the GPU path reproduce the oracle (quantized tensors, 32-bit sums, float outputs,
    tokens), how many 32-bit sums wrapped, which seed.  Part of the CPU leg: the oracle recomputes everything."""
    import numpy as np
    import workloads
    QT = {8: torch.int8, 16: torch.int16}
    qws = torch.empty(mq.mq_quantize_absmax_ws_bytes(), dtype=torch.uint8, device=dev)

    def gpu_product(A, Wt, bias, bits, relu):
        M, K = A.shape
        N = Wt.shape[0]
        pw = mq.prepare_weight(to_dev(Wt), bits)
        qa = torch.empty(mq.mq_packed_bytes(bits, M, K), dtype=torch.uint8, device=dev)
        sa = torch.empty(1, dtype=torch.float32, device=dev)
        mq.mq_quantize_absmax_pack_f32(to_dev(A), M, K, bits, qa, sa, qws, qws.numel())
        q = torch.empty((M, K), dtype=QT[bits], device=dev)
        mq.mq_unpack_weight(qa, bits, M, K, q)
        C = torch.empty((M, N), dtype=torch.int32, device=dev)
        mq.mq_gemm_i32_packed(qa, pw.packed, bits, M, N, K, C)
        Y = torch.empty((M, N), dtype=torch.float32, device=dev)
        mq.mq_gemm_dequant_packed(qa, pw.packed, bits, M, N, K, sa, pw.scale, None if bias is None else to_dev(bias),
                                  relu, Y, None)
        return q.cpu().numpy(), C.cpu().numpy(), Y.cpu().numpy()

    def check_product(A, Wt, bias, bits, relu):
        o = oracle.linear(A, Wt, bits, bias, relu)
        q, C, Y = gpu_product(A, Wt, bias, bits, relu)
        return ({"quantized": bool(np.array_equal(q, o["qA"])), "acc": bool(np.array_equal(C, o["acc"])),
                 "out": bool(np.array_equal(Y, o["Y"])), "overflow_count": int(o["overflow_count"]),
                 "overflow_fraction": round(o["overflow_count"] / o["acc"].size, 4)}, o["Y"])

    def merge(parts):
        out = {k: all(p_[k] for p_ in parts) for k in ("quantized", "acc", "out")}
        out["overflow_count"] = [p_["overflow_count"] for p_ in parts]
        out["overflow_fraction"] = [p_["overflow_fraction"] for p_ in parts]
        return out

    report = {}
    c = workloads.config1()
    r, _ = check_product(c["A"], c["Wt"], c["bias"], 16, False)
    report["config1"] = dict(r, seed=workloads.BASE_SEED + 1)
    for name, cfg, bits in (("config2", workloads.config2(), 8), ("config4", workloads.config4(), 16)):
        r1, H = check_product(cfg["A"], cfg["W1t"], cfg["b1"], bits, True)
        r2, _ = check_product(H, cfg["W2t"], cfg["b2"], bits, False)
        report[name] = dict(merge([r1, r2]), seed=workloads.BASE_SEED + int(name[-1]))
    c = workloads.config3()
    o = oracle.greedy_output_layer(c["Hd"], c["E"])
    M, d = c["Hd"].shape
    V = c["E"].shape[0]
    pe = mq.prepare_weight(to_dev(c["E"]), 8)
    qa = torch.empty(mq.mq_packed_bytes(8, M, d), dtype=torch.uint8, device=dev)
    sa = torch.empty(1, dtype=torch.float32, device=dev)
    mq.mq_quantize_absmax_pack_f32(to_dev(c["Hd"]), M, d, 8, qa, sa, qws, qws.numel())
    nws = mq.mq_argmax_ws_bytes(M, V)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)
    tok = torch.empty(M, dtype=torch.int32, device=dev)
    val = torch.empty(M, dtype=torch.float32, device=dev)
    mq.mq_gemm_argmax_packed(qa, pe.packed, M, V, d, sa, pe.scale, tok, val, ws, nws)
    C = torch.empty((M, V), dtype=torch.int32, device=dev)
    mq.mq_gemm_i32_packed(qa, pe.packed, 8, M, V, d, C)
    report["config3"] = {"acc": bool(np.array_equal(C.cpu().numpy(), o["acc"])),
                         "tokens": bool(np.array_equal(tok.cpu().numpy(), o["tok"])),
                         "out": bool(np.array_equal(val.cpu().numpy(), o["maxlogit"])), "overflow_count": 0,
                         "seed": workloads.BASE_SEED + 3}
    c5 = workloads.config5()
    parts = [check_product(g["A"], g["Wt"], g["bias"], 8, bool(g["relu"]))[0] for g in c5["gemms"][:7]]
    report["config5"] = dict(merge(parts), what="the seven products of layer 0 (the other layers repeat their shapes)",
                             seed=workloads.BASE_SEED + 5)
    return report


if __name__ == "__main__":
    main()
