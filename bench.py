#!/usr/bin/env python3
"""Benchmark of the int8 conv2d hot path (layout rewrite -> int8 MFMA GEMM stage) on one MI355X.

    python bench.py [--gpus 1] [--steps 200] [--warmup 10] [--workload C4] [--no-extras]

A step is one pass of the whole path -- input rewrite, weight rewrite, GEMM stage, or for the
shapes where the library picks it the GEMM stage that applies the rewrite itself -- over the
headline workload, through the one-shot C-ABI call, inputs resident in HBM.  One JSON line is
printed; `value` is effective int8 TOPS = 2*N*K*P*Q*C*R*S / time with the unpadded op count.
`per_config` carries, for every benchmark configuration, the operator-only, transform-only
and combined times (the three columns of the paper's Table 3), `n_scaled` the same kernels at
a batch size large enough to reach steady state (supplementary).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_OPS = 5.0e15   # dense int8 MFMA, MI355X
PEAK_HBM_BPS = 8.0e12    # HBM3E

# HBM-side bytes per launch of the dominant kernel (the GEMM stage on C4a), from the two
# rocprofv3 counter runs summarised in profiles/conv2d_int8_C4_hbm_counters.txt (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a 256 MiB device copy).  They
# describe the kernel source whose hash is recorded here; for any other source `traffic` is null.
TRAFFIC = {
    "source": "paper_2104_04731_amd/csrc/band_mfma.hip",
    "sha256": "fca480ff4cc07f1c3ac0289a0f33ec7652b88cec35c838be8373bbbea4b59404",
    "fetch_bytes": 4642305,
    "write_bytes": 3211264,
}


def measured_traffic():
    import hashlib
    try:
        with open(os.path.join(ROOT, TRAFFIC["source"]), "rb") as f:
            h = hashlib.sha256(f.read()).hexdigest()
    except OSError:
        return None
    if TRAFFIC["sha256"] is None or h != TRAFFIC["sha256"] or TRAFFIC["fetch_bytes"] is None:
        return None
    return TRAFFIC["fetch_bytes"] + TRAFFIC["write_bytes"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C4", help="C1, C2, C3, C4 (= C4a + C4b), C4a, C4b, C5")
    ap.add_argument("--no-extras", action="store_true", help="headline only (for profiling runs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--n-scaled-only", action="store_true",
                    help="run only the supplementary steady-state section (for profiling runs)")
    ap.add_argument("--steady-gemm-only", action="store_true",
                    help="run only the GEMM stage of C4a at N=2048, a few launches (for counter runs)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a known-size reference for "
                         "scaling hardware byte counters in profiler runs)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: one GPU only (the path would shard over batch or output channels without any "
              "exchange, so several GPUs are several independent runs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2104_04731_amd import binding as lib
    from paper_2104_04731_amd.inputs import CONFIGS

    lib.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    def timed(fn, steps, warmup):
        """(wall ms per call, event ms per call) over `steps` back-to-back calls.

        The calls are captured once into a HIP graph and the graph is replayed, so that the
        timed region holds exactly `steps` passes of device work and no per-call host cost
        (the kernels here run for microseconds; a Python call costs more than that)."""
        for _ in range(max(warmup, 1)):
            fn()                                  # also sizes the library's cached workspace
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(steps):
                fn()
        graph.replay()                            # untimed replay: graph upload, caches warm
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps

    flush_buf = torch.empty(640 << 20, dtype=torch.int8, device=dev)   # larger than L2s + the 256 MB last-level cache

    def sampled(fn, n, cold):
        """Per-call device times (us) of `n` individually timed calls, each one replay of a graph that holds
        one call, between an event pair on the launch stream (Sec. 5.1's protocol: warm-up, then repeated
        measurements with their spread).  cold: every call is preceded by an untimed 640 MB fill, so that
        nothing it touches is left in any cache; warm: the same buffers every call, a memory-silent spin in between."""
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        for _ in range(3):
            g.replay()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for e0, e1 in ev:
            # either way the device is kept busy for ~100 us before each sample, so that the host has queued
            # the event pair and the replay before the device gets there (else a sample holds host launch time)
            if cold:
                flush_buf.fill_(1)
            else:
                torch.cuda._sleep(200000)
            e0.record()
            g.replay()
            e1.record()
        torch.cuda.synchronize()
        return [e0.elapsed_time(e1) * 1e3 for e0, e1 in ev]

    def stats(us):
        import statistics
        return {"n": len(us), "mean_us": round(statistics.fmean(us), 3), "median_us": round(statistics.median(us), 3),
                "sigma_us": round(statistics.pstdev(us), 3), "min_us": round(min(us), 3)}

    class Case:
        """Device buffers and closures for one convolution."""

        def __init__(self, cfg):
            self.cfg = cfg
            x, w = cfg.make()
            self.x = torch.from_numpy(x).to(dev)
            self.w = torch.from_numpy(w).to(dev)
            self.out = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=dev)
            self.layout, self.cb, _ = lib.select_layout(cfg.dims())
            self.tile, self.split = lib.query_tiling(cfg.dims(), self.layout, self.cb)
            if self.layout == lib.LAYOUT_IMPLICIT:   # no input rewrite exists: the GEMM stage reads NCHW
                self.xp = self.x
                self.rewrite = None
            elif self.layout == lib.LAYOUT_IM2COL:
                self.xp = lib.im2col_int8(self.x, cfg.R, cfg.S, cfg.stride, cfg.pad)
                self.rewrite = lambda: lib.im2col_int8(self.x, cfg.R, cfg.S, cfg.stride, cfg.pad, out=self.xp)
            else:
                self.xp = lib.pack_layout(self.x, self.cb, cfg.pad)
                self.rewrite = lambda: lib.pack_layout(self.x, self.cb, cfg.pad, out=self.xp)
            self.wp = lib.pack_weights(self.w, self.layout, self.cb)
            self.rewrite_w = lambda: lib.pack_weights(self.w, self.layout, self.cb, out=self.wp)
            self.op = lambda: lib.conv2d_int8_packed(cfg.dims(), self.layout, self.cb, self.xp, self.wp, self.out)
            self.combined = lambda: lib.conv2d_int8(self.x, self.w, cfg.stride, cfg.pad, out=self.out)
            # inference steady state: weights rewritten ahead of time, input rewrite + GEMM stage per call
            nb = lib.conv2d_int8_workspace_bytes(cfg.dims(), self.layout, self.cb, True)
            ws = torch.empty(nb + 256, dtype=torch.int8, device=dev)
            self.ws = ws[(-ws.data_ptr()) % 256:] if nb else None
            self.combined_prepacked = lambda: lib.conv2d_int8_ex(cfg.dims(), self.layout, self.cb, self.x, self.wp,
                                                                 self.out, self.ws, wt_is_packed=True)
            self.rewrite_bytes = self.x.numel() + self.xp.numel() if self.rewrite else 0   # read once + written once

        def report(self, steps, warmup):
            cfg = self.cfg
            _, op = timed(self.op, steps, warmup)
            tr = timed(self.rewrite, steps, warmup)[1] if self.rewrite else None
            _, trw = timed(self.rewrite_w, steps, warmup)
            wall, comb = timed(self.combined, steps, warmup)
            _, pre = timed(self.combined_prepacked, steps, warmup)
            o_mac = lib.layout_overheads(cfg.dims(), self.layout, self.cb)[0]   # multiply-accumulates on padding
            # Every candidate layout the library has for this shape, through the explicit entry point with a
            # caller workspace (input rewrite + weight rewrite + GEMM stage each call): what the selector's pick
            # costs against the fastest candidate (Sec. 4.4: the choice depends on operator, layout and metric).
            cands = []
            for lay, cb in ((lib.LAYOUT_PACKED, 64), (lib.LAYOUT_PACKED, 32), (lib.LAYOUT_PACKED, 16), (lib.LAYOUT_IM2COL, 0),
                            (lib.LAYOUT_PAD_ONLY, 0), (lib.LAYOUT_IMPLICIT, 0), (lib.LAYOUT_IMAGE_PACK, 0),
                            (lib.LAYOUT_IMAGE_PACK, 16), (lib.LAYOUT_IMAGE_PACK, 64)):
                if not lib.layout_applies(cfg.dims(), lay, cb):
                    continue
                nb = lib.conv2d_int8_workspace_bytes(cfg.dims(), lay, cb)
                wsb = torch.empty(nb + 256, dtype=torch.int8, device=dev)
                wsa = wsb[(-wsb.data_ptr()) % 256:] if nb else None
                _, t = timed(lambda: lib.conv2d_int8_ex(cfg.dims(), lay, cb, self.x, self.w, self.out, wsa), min(steps, 100), 3)
                cands.append({"layout": lib.LAYOUT_NAMES[lay], "cb": cb, "combined_us": round(t * 1e3, 3),
                              "picked": (lay, cb) == (self.layout, self.cb if lay != lib.LAYOUT_PAD_ONLY else 0)})
                del wsb
            fastest = min(c["combined_us"] for c in cands)
            picked = [c for c in cands if c["picked"]]
            regret = round(picked[0]["combined_us"] / fastest - 1.0, 4) if picked else None
            warm, cold = sampled(self.combined, 100, False), sampled(self.combined, 100, True)
            # the same convolution on NHWC tensors (Sec. 5.2): NHWC in, KCRS weights, NHWC result
            xh = self.x.permute(0, 2, 3, 1).contiguous()
            oh = torch.empty((cfg.N, cfg.P, cfg.Q, cfg.K), dtype=torch.int32, device=dev)
            _, nh = timed(lambda: lib.conv2d_int8_nhwc(xh, self.w, cfg.stride, cfg.pad, out=oh), steps, warmup)
            del xh, oh
            if self.tile >= 0:
                rows, cols = lib.tile_info(self.tile)[:2]
            elif self.tile == lib.TILE_BAND:
                rows, cols = "band 32", "rows of one image"
            else:
                rows, cols = min(64, -(-cfg.K // 32) * 32), 128
            return {
                "name": cfg.name, "layout": lib.LAYOUT_NAMES[self.layout], "cb": self.cb,
                "tile": f"{rows}x{cols}", "split_k": self.split, "ops": cfg.ops,
                "op_us": round(op * 1e3, 3), "transf_in_us": round(tr * 1e3, 3) if tr else None,
                "transf_wt_us": round(trw * 1e3, 3), "combined_us": round(comb * 1e3, 3),
                "combined_weights_prepacked_us": round(pre * 1e3, 3),
                "tops_op": round(cfg.ops / (op * 1e-3) / 1e12, 3),
                "issued_tops_op": round((cfg.ops + 2 * o_mac) / (op * 1e-3) / 1e12, 3),
                "tops_combined": round(cfg.ops / (comb * 1e-3) / 1e12, 3),
                "pct_mfma_peak_op": round(100 * cfg.ops / (op * 1e-3) / PEAK_INT8_OPS, 3),
                "transf_in_GBps": round(self.rewrite_bytes / (tr * 1e-3) / 1e9, 1) if tr else None,
                "pct_hbm_peak_transf": round(100 * self.rewrite_bytes / (tr * 1e-3) / PEAK_HBM_BPS, 2) if tr else None,
                "combined_GBps": round((self.x.numel() + self.w.numel() + 4 * self.out.numel()) / (comb * 1e-3) / 1e9, 1),
                "combined_single_calls_warm": stats(warm), "combined_single_calls_cold": stats(cold),
                "nhwc_one_shot_us": round(nh * 1e3, 3),
                "candidates": cands, "selector_regret": regret,
            }

    if args.calibration_copy:
        src = torch.zeros(256 << 20, dtype=torch.int8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.n_scaled_only:
        print(json.dumps({"n_scaled": n_scaled(lib, timed, CONFIGS, dev)}), flush=True)
        return

    if args.steady_gemm_only:
        # the steady-state GEMM stage on its own (for counter runs): random operands, all-zero operands (what the
        # time owes to switching activity), and the register-resident MFMA probe under the same conditions
        cfg = CONFIGS["C4a"].scaled(2048)
        x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
        w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=dev)
        xp = lib.pack_layout(x, 64, cfg.pad)
        wp = lib.pack_weights(w, lib.LAYOUT_PACKED, 64)
        o = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=dev)
        _, ms = timed(lambda: lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_PACKED, 64, xp, wp, o), 10, 3)
        xz, wz = torch.zeros_like(xp), torch.zeros_like(wp)
        _, ms_z = timed(lambda: lib.conv2d_int8_packed(cfg.dims(), lib.LAYOUT_PACKED, 64, xz, wz, o), 10, 3)
        blocks, iters = 256 * 8, 4096
        buf = torch.empty(blocks * 256, dtype=torch.int32, device=dev)
        _, ms_p = timed(lambda: lib.mfma_probe_int8(blocks, iters, out=buf), 5, 2)
        probe_ops = 2 * 32768 * 16 * iters * blocks
        def eager_ms(fn, n=5):
            for _ in range(2):
                fn()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for _ in range(n):
                fn()
            ev1.record()
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) / n

        # for scale: the vendor library's int8 GEMM (torch._int_mm = hipBLASLt) on matrices of the same sizes, and both
        # on a square 8192^3 problem (ours as a 1x1 convolution over 8 images of 32x32 pixels, 8192 -> 8192 channels)
        vendor = {}
        try:
            gm, gk, gn = cfg.N * cfg.P * cfg.Q, cfg.C * cfg.R * cfg.S, cfg.K
            ga = torch.randint(-128, 128, (gm, gk), dtype=torch.int8, device=dev)
            gb = torch.randint(-128, 128, (gn, gk), dtype=torch.int8, device=dev).t()
            vendor["same_sizes_tops"] = round(2.0 * gm * gk * gn / (eager_ms(lambda: torch._int_mm(ga, gb)) * 1e-3) / 1e12, 1)
            ga.zero_()
            gbz = torch.zeros((gn, gk), dtype=torch.int8, device=dev).t()
            vendor["same_sizes_zero_tops"] = round(2.0 * gm * gk * gn / (eager_ms(lambda: torch._int_mm(ga, gbz)) * 1e-3) / 1e12, 1)
            del ga, gb, gbz
            sq = 8192
            sa = torch.randint(-128, 128, (sq, sq), dtype=torch.int8, device=dev)
            sb = torch.randint(-128, 128, (sq, sq), dtype=torch.int8, device=dev).t()
            vendor["square_8192_tops"] = round(2.0 * sq ** 3 / (eager_ms(lambda: torch._int_mm(sa, sb)) * 1e-3) / 1e12, 1)
            sa.zero_()
            sbz = torch.zeros((sq, sq), dtype=torch.int8, device=dev).t()
            vendor["square_8192_zero_tops"] = round(2.0 * sq ** 3 / (eager_ms(lambda: torch._int_mm(sa, sbz)) * 1e-3) / 1e12, 1)
            del sa, sb, sbz
        except Exception as e:  # not every build has the routine
            vendor["error"] = str(e)[:120]
        sdims = (8, 8192, 32, 32, 8192, 1, 1, 1, 0)
        sx = lib.pack_layout(torch.randint(-128, 128, (8, 8192, 32, 32), dtype=torch.int8, device=dev), 64, 0)
        sw = lib.pack_weights(torch.randint(-128, 128, (8192, 8192, 1, 1), dtype=torch.int8, device=dev), lib.LAYOUT_PACKED, 64)
        so = torch.empty((8, 8192, 32, 32), dtype=torch.int32, device=dev)
        ours_sq = 2.0 * 8192 ** 3 / (eager_ms(lambda: lib.conv2d_int8_packed(sdims, lib.LAYOUT_PACKED, 64, sx, sw, so)) * 1e-3) / 1e12
        sx.zero_()
        sw.zero_()
        ours_sq_z = 2.0 * 8192 ** 3 / (eager_ms(lambda: lib.conv2d_int8_packed(sdims, lib.LAYOUT_PACKED, 64, sx, sw, so)) * 1e-3) / 1e12
        del sx, sw, so
        print(json.dumps({"gemm_stage_C4a_N2048_us": round(ms * 1e3, 2), "tiling": lib.query_tiling(cfg.dims(), lib.LAYOUT_PACKED, 64),
                          "tile": "%dx%d, %d threads" % tuple(lib.tile_info(lib.query_tiling(cfg.dims(), lib.LAYOUT_PACKED, 64)[0])[:3]),
                          "vendor_gemm": vendor, "square_8192_tops": round(ours_sq, 1), "square_8192_zero_tops": round(ours_sq_z, 1),
                          "tops": round(cfg.ops / (ms * 1e-3) / 1e12, 2),
                          "all_zero_operands_us": round(ms_z * 1e3, 2), "all_zero_operands_tops": round(cfg.ops / (ms_z * 1e-3) / 1e12, 2),
                          "mfma_probe_us": round(ms_p * 1e3, 2), "mfma_probe_tops": round(probe_ops / (ms_p * 1e-3) / 1e12, 2)}), flush=True)
        return

    groups = {"C1": ["C1"], "C2": ["C2"], "C3": ["C3"], "C4": ["C4a", "C4b"], "C4a": ["C4a"], "C4b": ["C4b"],
              "C5": ["C5"]}
    if args.workload not in groups:
        print(f"unknown workload {args.workload}", file=sys.stderr)
        sys.exit(2)
    head = [Case(CONFIGS[n]) for n in groups[args.workload]]
    head_ops = sum(c.cfg.ops for c in head)

    def step():
        for c in head:
            c.combined()

    wall_ms, ev_ms = timed(step, args.steps, args.warmup)
    value = head_ops / (wall_ms * 1e-3) / 1e12
    # the same step one call at a time: median and spread, caches warm and cold (Sec. 5.1: mean of 200 with sigma)
    step_warm, step_cold = stats(sampled(step, args.steps, False)), stats(sampled(step, args.steps, True))

    # the same step with every convolution forced through stored rewrites (channel blocking, block 64,
    # caller workspace): input rewrite + weight rewrite, then the GEMM stage -- reported beside `value`
    two_stage = None
    if not args.no_extras and any(c.layout == lib.LAYOUT_IMPLICIT for c in head):
        ws = []
        for c in head:
            nb = lib.conv2d_int8_workspace_bytes(c.cfg.dims(), lib.LAYOUT_PACKED, 64)
            t = torch.empty(nb + 256, dtype=torch.int8, device=dev)
            ws.append(t[(-t.data_ptr()) % 256:])

        def step_two_stage():
            for c, w in zip(head, ws):
                lib.conv2d_int8_ex(c.cfg.dims(), lib.LAYOUT_PACKED, 64, c.x, c.w, c.out, w)

        ts_ms, _ = timed(step_two_stage, args.steps, args.warmup)
        two_stage = {"ms_per_step": round(ts_ms, 6), "value": round(head_ops / (ts_ms * 1e-3) / 1e12, 4),
                     "layouts": ["packed/cb64"] * len(head)}

    # config 4 read as a chain (the second layer consumes the first one's activated output): convolution,
    # activation + the next layer's channel blocking in one pass, weight rewrite, GEMM stage -- reported
    # beside `value`, which times the two layers on independent inputs
    chained = None
    if not args.no_extras and args.workload == "C4":
        a4, b4 = head
        xq = lib.requant_pack_layout(a4.out, 64, b4.cfg.pad, 9, True)
        wq = lib.pack_weights(b4.w, lib.LAYOUT_PACKED, 64)

        def step_chained():
            a4.combined()
            lib.requant_pack_layout(a4.out, 64, b4.cfg.pad, 9, True, out=xq)
            lib.pack_weights(b4.w, lib.LAYOUT_PACKED, 64, out=wq)
            lib.conv2d_int8_packed(b4.cfg.dims(), lib.LAYOUT_PACKED, 64, xq, wq, b4.out)

        ch_ms, _ = timed(step_chained, args.steps, args.warmup)
        chained = {"ms_per_step": round(ch_ms, 6), "value": round(head_ops / (ch_ms * 1e-3) / 1e12, 4),
                   "path": "conv2d_int8(C4a) -> requant_pack_layout(shift 9, relu) -> pack_weights -> GEMM stage(C4b)"}
        # the same chain with the activation in the first GEMM stage's epilogue: the int32 tensor between the
        # layers is never stored, and the rewrite of both layers' weights is hoisted (inference steady state)
        xq1 = lib.pack_layout(a4.x, 64, a4.cfg.pad)
        wq1 = lib.pack_weights(a4.w, lib.LAYOUT_PACKED, 64)

        def step_fused():
            lib.pack_layout(a4.x, 64, a4.cfg.pad, out=xq1)
            lib.conv2d_int8_packed_requant(a4.cfg.dims(), lib.LAYOUT_PACKED, 64, xq1, wq1, 64, b4.cfg.pad, 9, True, out=xq)
            lib.conv2d_int8_packed(b4.cfg.dims(), lib.LAYOUT_PACKED, 64, xq, wq, b4.out)

        def step_unfused_hoisted():
            lib.pack_layout(a4.x, 64, a4.cfg.pad, out=xq1)
            lib.conv2d_int8_packed(a4.cfg.dims(), lib.LAYOUT_PACKED, 64, xq1, wq1, a4.out)
            lib.requant_pack_layout(a4.out, 64, b4.cfg.pad, 9, True, out=xq)
            lib.conv2d_int8_packed(b4.cfg.dims(), lib.LAYOUT_PACKED, 64, xq, wq, b4.out)

        fu_ms, _ = timed(step_fused, args.steps, args.warmup)
        un_ms, _ = timed(step_unfused_hoisted, args.steps, args.warmup)
        chained["weights_hoisted"] = {
            "fused_epilogue_ms": round(fu_ms, 6), "separate_activation_ms": round(un_ms, 6),
            "fused_value": round(head_ops / (fu_ms * 1e-3) / 1e12, 4),
            "path": "pack_layout(C4a) -> GEMM stage with activation epilogue (C4a) -> GEMM stage (C4b)"}

    # dominant kernel of the step: the MFMA GEMM stage of the largest convolution
    dom = max(head, key=lambda c: c.cfg.ops)
    _, dom_ms = timed(dom.op, args.steps, args.warmup)
    if dom.layout == lib.LAYOUT_IMPLICIT:
        # the stencil-unrolling GEMM stage moves input + weights + int32 output once each and is bound by that
        nbytes = dom.x.numel() + dom.w.numel() + 4 * dom.out.numel()
        achieved = nbytes / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_BPS / 1e9, "unit": "GB/s",
                    "frac": round(achieved * 1e9 / PEAK_HBM_BPS, 5), "traffic": None,
                    "kernel": "conv_pointwise_*_kernel (the library picks among the 1x1 forms by grid size)" if (dom.cfg.R, dom.cfg.S) == (1, 1) and dom.cfg.C % 64 == 0
                    else "conv_window_kernel", "config": dom.cfg.name, "launch_us": round(dom_ms * 1e3, 3)}
    else:
        achieved = dom.cfg.ops / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_INT8_OPS / 1e12,
                    "unit": "TOP/s", "frac": round(achieved * 1e12 / PEAK_INT8_OPS, 5), "traffic": measured_traffic(),
                    "kernel": "conv_band_kernel" if dom.tile == lib.TILE_BAND else "igemm_i8_kernel", "config": dom.cfg.name,
                    "launch_us": round(dom_ms * 1e3, 3),
                    "launch_stats_warm": stats(sampled(dom.op, args.steps, False)),
                    "launch_stats_cold": stats(sampled(dom.op, args.steps, True))}

    result = {
        "metric": "int8 conv effective TOPS (2*N*K*P*Q*C*R*S / time), layout rewrite + MFMA GEMM stage",
        "value": round(value, 4), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms, 6), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "i8", "data": "synthetic",
        "config": {"workload": " + ".join(
            f"{c.cfg.name}: N={c.cfg.N} C={c.cfg.C} H={c.cfg.H} W={c.cfg.W} K={c.cfg.K} "
            f"{c.cfg.R}x{c.cfg.S} stride {c.cfg.stride} pad {c.cfg.pad}" for c in head),
            "path": "conv2d_int8 one-shot, layout picked per shape: input rewrite + weight rewrite + GEMM stage, "
                    "or (implicit) the rewrite applied inside the GEMM stage",
            "layouts": [lib.LAYOUT_NAMES[c.layout] + (f"/cb{c.cb}" if c.cb else "") for c in head]},
        "event_ms_per_step": round(ev_ms, 6),
        "timing": {"value_from": "mean over one graph of `steps` back-to-back steps (same buffers: operands in L2 / last-level cache)",
                   "single_steps_warm": step_warm, "single_steps_cold": step_cold,
                   "single_step_overhead_us": round(step_warm["median_us"] - wall_ms * 1e3, 3),
                   "cold_penalty_us": round(step_cold["median_us"] - step_warm["median_us"], 3),
                   "cold_value_estimate": round(head_ops / ((wall_ms * 1e3 + max(step_cold["median_us"] - step_warm["median_us"], 0.0)) * 1e-6) / 1e12, 4),
                   "note": "single steps: one graph replay per step between an event pair, after ~100 us of other device work "
                           "so that the host is ahead (warm: a memory-silent spin; cold: a 640 MB fill that evicts L2 and the "
                           "256 MB last-level cache).  A single replay between events carries a fixed overhead (single_step_overhead_us: "
                           "its warm median minus the back-to-back mean); cold_value_estimate = ops / (back-to-back mean + cold_penalty)"},
        "pct_mfma_peak": round(100 * value * 1e12 / PEAK_INT8_OPS, 3),
        "rewrite_then_gemm_only": two_stage,
        "chained_with_activation": chained,
        "roofline": roofline,
    }

    if not args.no_extras:
        steps = min(args.steps, 200)
        result["per_config"] = [Case(CONFIGS[n]).report(steps, args.warmup) for n in CONFIGS]
        result["n_scaled"] = n_scaled(lib, timed, CONFIGS, dev)

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline([c.cfg for c in head])

    print(json.dumps(result), flush=True)


def n_scaled(lib, timed, CONFIGS, dev):
    """Supplementary: the same kernels at batch sizes that reach steady state.  Layout kernels
    move >= 1 GiB (beyond the 256 MB Infinity Cache); the GEMM stage runs tens of waves of tiles."""
    import torch
    out = {}
    # GEMM stage of the deep 3x3 layer at N=2048 (operands pre-rewritten): 12.25 rounds of
    # 256x256 tiles on 256 CUs, so the partly filled last round costs 6 %
    cfg = CONFIGS["C4a"].scaled(2048)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
    w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=dev)
    lay, cb, _ = lib.select_layout(cfg.dims())
    xp = lib.pack_layout(x, cb, cfg.pad)
    wp = lib.pack_weights(w, lay, cb)
    o = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=dev)
    tile, split = lib.query_tiling(cfg.dims(), lay, cb)
    _, ms = timed(lambda: lib.conv2d_int8_packed(cfg.dims(), lay, cb, xp, wp, o), 20, 3)
    rows, cols = lib.tile_info(tile)[:2]
    out["gemm_stage_C4a_N2048"] = {"us": round(ms * 1e3, 2), "tops": round(cfg.ops / (ms * 1e-3) / 1e12, 2),
                                   "pct_mfma_peak": round(100 * cfg.ops / (ms * 1e-3) / PEAK_INT8_OPS, 2),
                                   "tile": f"{rows}x{cols}", "split_k": split}
    # the same stage with the other two epilogues: an NHWC int32 result (16-byte stores, 2 KB runs per pixel
    # instead of 128-byte runs per channel) and the activation (int8, the next layer's blocked input)
    onh = torch.empty((cfg.N, cfg.P, cfg.Q, cfg.K), dtype=torch.int32, device=dev)
    _, ms_n = timed(lambda: lib.conv2d_int8_packed_nhwc(cfg.dims(), lay, cb, xp, wp, onh), 20, 3)
    xact = lib.conv2d_int8_packed_requant(cfg.dims(), lay, cb, xp, wp, 64, 0, 9, True)
    _, ms_a = timed(lambda: lib.conv2d_int8_packed_requant(cfg.dims(), lay, cb, xp, wp, 64, 0, 9, True, out=xact), 20, 3)
    out["gemm_stage_C4a_N2048"]["nhwc_result_us"] = round(ms_n * 1e3, 2)
    out["gemm_stage_C4a_N2048"]["activation_epilogue_us"] = round(ms_a * 1e3, 2)
    del onh, xact
    _, ms = timed(lambda: lib.pack_layout(x, cb, cfg.pad, out=xp), 20, 3)
    b = x.numel() + xp.numel()
    out["pack_layout_C4a_N2048"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                    "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2),
                                    "note": "237 MB: fits the 256 MB last-level cache; see pack_layout_C4a_N8192"}
    big = CONFIGS["C4a"].scaled(8192)
    xb = torch.randint(-128, 128, (big.N, big.C, big.H, big.W), dtype=torch.int8, device=dev)
    xbp = lib.pack_layout(xb, cb, big.pad)
    _, ms = timed(lambda: lib.pack_layout(xb, cb, big.pad, out=xbp), 10, 2)
    b = xb.numel() + xbp.numel()
    out["pack_layout_C4a_N8192"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                    "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    del xb, xbp
    # unpacking the NKPQ result for an NHWC consumer (int32, read once + written once)
    oh = lib.unpack_nhwc_int32(o)
    _, ms = timed(lambda: lib.unpack_nhwc_int32(o, out=oh), 10, 2)
    b = 8 * o.numel()
    out["unpack_nhwc_C4a_N2048"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                    "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    # activation + the next layer's channel blocking in one pass (int32 read once, int8 blocks written once)
    xq = lib.requant_pack_layout(o, 64, 0, 9, True)
    _, ms = timed(lambda: lib.requant_pack_layout(o, 64, 0, 9, True, out=xq), 10, 2)
    b = 4 * o.numel() + xq.numel()
    out["requant_pack_C4a_N2048"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                     "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    del x, xp, o, oh, xq
    # pack_layout of the 64-channel 56x56 layer at N=2048 (~0.9 GiB moved)
    cfg = CONFIGS["C2"].scaled(2048)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
    xp = lib.pack_layout(x, 64, cfg.pad)
    _, ms = timed(lambda: lib.pack_layout(x, 64, cfg.pad, out=xp), 10, 2)
    b = x.numel() + xp.numel()
    out["pack_layout_C2_N2048"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                    "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    # the same rewrite from an NHWC source (the source-layout experiment of the paper's Sec. 5.2)
    xh = x.permute(0, 2, 3, 1).contiguous()
    _, ms = timed(lambda: lib.pack_layout_nhwc(xh, 64, cfg.pad, out=xp), 10, 2)
    out["pack_layout_nhwc_C2_N2048"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                         "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    del x, xp, xh
    # im2col of the 7x7 stem at N=512 (~1.3 GB moved)
    cfg = CONFIGS["C3"].scaled(512)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
    xp = lib.im2col_int8(x, cfg.R, cfg.S, cfg.stride, cfg.pad)
    _, ms = timed(lambda: lib.im2col_int8(x, cfg.R, cfg.S, cfg.stride, cfg.pad, out=xp), 10, 2)
    b = x.numel() + xp.numel()
    out["im2col_C3_N512"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                              "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    del x, xp
    # the stencil-unrolling GEMM stage (whole convolution through the one-shot entry point, no rewritten activations:
    # at these sizes the 7x7 stem's 9 KB of weights are rewritten by a small kernel first, the 1x1 layer is one
    # launch): the 7x7 stem at N=512 and the 1x1 layer at N=8192; bytes = input + weights + int32 output, each once
    for key, name, scale in (("implicit_conv_C3_N512", "C3", 512), ("implicit_conv_C4b_N8192", "C4b", 8192)):
        cfg = CONFIGS[name].scaled(scale)
        x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
        w = torch.randint(-128, 128, (cfg.K, cfg.C, cfg.R, cfg.S), dtype=torch.int8, device=dev)
        o = torch.empty((cfg.N, cfg.K, cfg.P, cfg.Q), dtype=torch.int32, device=dev)
        assert lib.select_layout(cfg.dims())[0] == lib.LAYOUT_IMPLICIT
        _, ms = timed(lambda: lib.conv2d_int8(x, w, cfg.stride, cfg.pad, out=o), 10, 2)
        b = x.numel() + w.numel() + 4 * o.numel()
        out[key] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                    "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2),
                    "tops": round(cfg.ops / (ms * 1e-3) / 1e12, 2)}
        del x, w, o
    # stencil unrolling of the 64-channel 3x3 layer from both source layouts (Sec. 5.2): from NHWC a tap's
    # channels are one contiguous run
    cfg = CONFIGS["C2"].scaled(512)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
    xh = x.permute(0, 2, 3, 1).contiguous()
    a1 = lib.im2col_int8(x, cfg.R, cfg.S, cfg.stride, cfg.pad)
    for key, fn in (("im2col_C2_N512", lambda: lib.im2col_int8(x, cfg.R, cfg.S, cfg.stride, cfg.pad, out=a1)),
                    ("im2col_nhwc_C2_N512", lambda: lib.im2col_nhwc_int8(xh, cfg.R, cfg.S, cfg.stride, cfg.pad, out=a1))):
        _, ms = timed(fn, 10, 2)
        b = x.numel() + a1.numel()
        out[key] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                    "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    del x, xh, a1
    # Image Pack of the same stem (stride phases to channels): bytes = input + packed image
    cfg = CONFIGS["C3"].scaled(4096)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
    x2 = lib.image_pack_int8(cfg.dims(), x)
    _, ms = timed(lambda: lib.image_pack_int8(cfg.dims(), x, out=x2), 10, 2)
    b = x.numel() + x2.numel()
    out["image_pack_C3_N4096"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                  "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
    del x, x2
    cfg = CONFIGS["C3"].scaled(512)
    x = torch.randint(-128, 128, (cfg.N, cfg.C, cfg.H, cfg.W), dtype=torch.int8, device=dev)
    xp = lib.im2col_int8(x, cfg.R, cfg.S, cfg.stride, cfg.pad)
    # Dilated 3x3 (dilation 2, "same" size) over 64 channels of 28x28: the packed route against the
    # paper's reference for it, the kernel spread out with zeros and run densely (Sec. 6.1); then its
    # two layout kernels at a batch that fills the chip.
    dil = 2
    for key, n in (("dilated_3x3_d2_N4", 4), ("dilated_3x3_d2_N4096", 4096)):
        dims = (n, 64, 28, 28, 64, 3, 3, 1, 2)
        xd = torch.randint(-128, 128, dims[:4], dtype=torch.int8, device=dev)
        wd = torch.randint(-128, 128, (64, 64, 3, 3), dtype=torch.int8, device=dev)
        wsp = torch.zeros((64, 64, 5, 5), dtype=torch.int8, device=dev)
        wsp[:, :, ::dil, ::dil] = wd
        od = torch.empty((n, 64, 28, 28), dtype=torch.int32, device=dev)
        need = lib.conv2d_int8_dilated_workspace_bytes(dims, dil)
        wsb = torch.empty(need + 256, dtype=torch.int8, device=dev)
        wsb = wsb[(-wsb.data_ptr()) % 256:]
        _, ms_p = timed(lambda: lib.conv2d_int8_dilated(dims, dil, xd, wd, out=od, workspace=wsb), 10, 2)
        _, ms_s = timed(lambda: lib.conv2d_int8(xd, wsp, 1, 2, out=od), 10, 2)
        # and with the dilation as an address multiplier of the GEMM stage (no Image Pack at all)
        nd = lib.conv2d_int8_workspace_bytes(dims, lib.LAYOUT_PACKED, 64)
        wsd = torch.empty(nd + 256, dtype=torch.int8, device=dev)
        wsd = wsd[(-wsd.data_ptr()) % 256:]
        _, ms_d = timed(lambda: lib.conv2d_int8_dilated_direct(dims, dil, xd, wd, 64, out=od, workspace=wsd), 10, 2)
        ops = 2 * n * 64 * 28 * 28 * 64 * 9
        entry = {"packed_us": round(ms_p * 1e3, 2), "spread_kernel_us": round(ms_s * 1e3, 2),
                 "address_multiplier_us": round(ms_d * 1e3, 2),
                 "packed_tops": round(ops / (ms_p * 1e-3) / 1e12, 2), "spread_kernel_tops": round(ops / (ms_s * 1e-3) / 1e12, 2),
                 "address_multiplier_tops": round(ops / (ms_d * 1e-3) / 1e12, 2)}
        del wsd
        if n > 4:
            x2 = lib.dilation_pack_int8(dims, dil, xd)
            _, ms = timed(lambda: lib.dilation_pack_int8(dims, dil, xd, out=x2), 10, 2)
            b = xd.numel() + x2.numel()
            entry["dilation_pack"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                      "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
            d2 = lib.dilated_desc(dims, dil)
            o2 = torch.empty((d2[0], 64, d2[2] - 2, d2[3] - 2), dtype=torch.int32, device=dev)
            _, ms = timed(lambda: lib.dilation_unpack_int32(dims, dil, o2, out=od), 10, 2)
            b = 4 * (o2.numel() + od.numel())
            entry["dilation_unpack"] = {"us": round(ms * 1e3, 2), "bytes": b, "GBps": round(b / (ms * 1e-3) / 1e9, 1),
                                        "pct_hbm_peak": round(100 * b / (ms * 1e-3) / PEAK_HBM_BPS, 2)}
            del x2, o2
        out[key] = entry
        del xd, wd, wsp, od, wsb
    # what the matrix cores sustain with register-resident operands and nothing else in the way
    blocks, iters = 256 * 8, 4096
    buf = torch.empty(blocks * 256, dtype=torch.int32, device=dev)
    _, ms = timed(lambda: lib.mfma_probe_int8(blocks, iters, out=buf), 5, 2)
    probe_ops = 2 * 32768 * 16 * iters * blocks
    out["mfma_probe"] = {"us": round(ms * 1e3, 2), "tops": round(probe_ops / (ms * 1e-3) / 1e12, 1),
                         "pct_mfma_peak": round(100 * probe_ops / (ms * 1e-3) / PEAK_INT8_OPS, 2),
                         "shape": f"{blocks} workgroups x 4 waves x {iters} x 4 v_mfma_i32_32x32x32_i8, pseudo-random operands"}
    out["gemm_stage_C4a_N2048"]["pct_of_mfma_probe"] = round(100 * out["gemm_stage_C4a_N2048"]["tops"] / out["mfma_probe"]["tops"], 2)
    # the vendor library's int8 GEMM on a matrix of the same sizes as that stage (M = N*P*Q rows of C*R*S bytes,
    # already unrolled and row-major, times K columns), for scale only: torch._int_mm, i.e. hipBLASLt
    try:
        c4 = CONFIGS["C4a"].scaled(2048)
        gm, gk, gn = c4.N * c4.P * c4.Q, c4.C * c4.R * c4.S, c4.K
        ga = torch.randint(-128, 128, (gm, gk), dtype=torch.int8, device=dev)
        gb = torch.randint(-128, 128, (gn, gk), dtype=torch.int8, device=dev).t()
        for _ in range(2):
            torch._int_mm(ga, gb)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()                      # eager calls: ~1 ms each, far above the launch cost
        for _ in range(5):
            torch._int_mm(ga, gb)
        ev1.record()
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / 5
        out["vendor_gemm_reference"] = {"us": round(ms * 1e3, 2), "tops": round(2.0 * gm * gk * gn / (ms * 1e-3) / 1e12, 1),
                                        "shape": f"torch._int_mm [{gm} x {gk}] x [{gk} x {gn}], second operand column-major"}
        del ga, gb
    except Exception as e:  # not every build has the routine
        out["vendor_gemm_reference"] = {"error": str(e)[:120]}
    # a plain device-to-device copy of the same size, for scale
    y = torch.empty_like(xp)
    _, ms = timed(lambda: y.copy_(xp), 10, 2)
    out["copy_reference"] = {"bytes": 2 * xp.numel(), "GBps": round(2 * xp.numel() / (ms * 1e-3) / 1e9, 1)}
    # every bandwidth figure also as a fraction of what that plain copy reaches on this machine
    def against_copy(entry):
        if isinstance(entry, dict):
            if "GBps" in entry and entry is not out["copy_reference"]:
                entry["pct_of_copy"] = round(100 * entry["GBps"] / out["copy_reference"]["GBps"], 1)
            for v in list(entry.values()):
                against_copy(v)
    against_copy(out)
    return out


def cpu_baseline(cfgs):
    """The CPU checker, as it stands, timed on the host cores over the headline workload."""
    from oracle import direct
    best = None
    ops = sum(c.ops for c in cfgs)
    data = [c.make() for c in cfgs]
    for _ in range(3):
        t0 = time.perf_counter()
        for c, (x, w) in zip(cfgs, data):
            direct.conv2d_int8(x, w, c.stride, c.pad)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    res = {"value": round(ops / best / 1e12, 6), "unit": "TOPS", "cores": direct.threads(), "cpu_model": model, "kind": "oracle",
           "sample": "whole headline workload (" + " + ".join(c.name for c in cfgs) + "), best of 3, "
                     f"{best * 1e3:.1f} ms"}
    # the two smallest configurations on one thread, for scale
    from paper_2104_04731_amd.inputs import CONFIGS
    cores = direct.threads()
    direct.set_threads(1)
    one = {}
    for name in ("C1", "C2"):
        c = CONFIGS[name]
        x, w = c.make()
        t0 = time.perf_counter()
        direct.conv2d_int8(x, w, c.stride, c.pad)
        one[name] = round((time.perf_counter() - t0) * 1e3, 3)
    direct.set_threads(cores)
    res["one_thread_ms"] = one
    return res


if __name__ == "__main__":
    main()
