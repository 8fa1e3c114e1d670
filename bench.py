"""Benchmark of the AllGather-GEMM hot path on one MI355X.

One step = signal_reset, the emulated producer on the producer stream and the signal-gated GEMM on the
consumer stream (the whole fused AG+GEMM of the 70B-MLP-shaped workload).  Prints ONE JSON line.
Inputs are synthetic, seeded, and resident in HBM before the timed region starts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published)
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E peak (published)
SETTLE_STEPS = 150          # untimed steps run before --warmup whatever its value: the chip needs about 0.1 s under this
                            # load before its clocks hold still (the first steps after an idle period run 10 % slow)


def _measured_traffic(workload: str, summary: str = "gemm_kernel_{}_hbm_traffic.txt"):
    """HBM bytes per kernel launch measured with rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, scaled by a copy of
    known size).  This run does not measure them: the figure is read from the committed summary of that measurement
    (returned with the file's name so that the output says where it comes from); (None, None) if there is none."""
    name = summary.format(workload)
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1].split()[0])), "profiles/" + name
    except OSError:
        pass
    return None, None


class HipEvents:
    """HIP events made without the system-scope fence that a default event adds when it completes (that fence
    flushes and invalidates the L2 between the kernels it sits between, which would be charged to the kernels
    being timed).  Plumbing for the measurement only."""

    def __init__(self):
        import ctypes
        self.C = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.live = []

    def new(self, timing: bool = True):
        ev = self.C.c_void_p()
        flags = 0x20000000 | (0 if timing else 0x2)      # hipEventDisableSystemFence | hipEventDisableTiming
        rc = self.hip.hipEventCreateWithFlags(self.C.byref(ev), self.C.c_uint(flags))
        if rc != 0:
            raise RuntimeError(f"hipEventCreateWithFlags failed ({rc})")
        self.live.append(ev)
        return ev

    def record(self, ev, stream: int):
        rc = self.hip.hipEventRecord(ev, self.C.c_void_p(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed ({rc})")

    def wait(self, stream: int, ev):
        rc = self.hip.hipStreamWaitEvent(self.C.c_void_p(stream), ev, self.C.c_uint(0))
        if rc != 0:
            raise RuntimeError(f"hipStreamWaitEvent failed ({rc})")

    def elapsed_ms(self, a, b) -> float:
        ms = self.C.c_float()
        rc = self.hip.hipEventElapsedTime(self.C.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def close(self):
        for ev in self.live:
            self.hip.hipEventDestroy(ev)
        self.live = []


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps first; the chip needs some tens of ms under load to settle its clocks")
    ap.add_argument("--workload", default="ag_gemm_70b_mlp")
    ap.add_argument("--tile", type=int, default=-1)
    ap.add_argument("--chunks", type=int, default=4, help="signals per shard")
    ap.add_argument("--producer-wgs", type=int, default=0)
    ap.add_argument("--wide-producer", action="store_true",
                    help="copy kernel with four waves per workgroup (default: one wave per workgroup: the same fused "
                         "time, for a quarter of the registers and issue slots the copy takes on every compute unit)")
    ap.add_argument("--t-local", action="store_true",
                    help="read the own shard from T like any other (default: in place, where the caller keeps it, "
                         "with the local copy into T done last)")
    ap.add_argument("--link-gbps", type=float, default=76.8,
                    help="rate of one emulated link of the full-mesh block (one direction of an xGMI link)")
    ap.add_argument("--cpu-rows", type=int, default=8192, help="rows of C the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="profiling aid for rocprofv3 --pmc runs: also run one plain 256 MiB device copy, the known-size "
                         "kernel that the FETCH_SIZE / WRITE_SIZE counters are scaled by, and launch producer and "
                         "consumer on one stream (counter collection runs kernels one at a time)")
    ap.add_argument("--no-extras", action="store_true", help="skip the reducer / serial / copy-only timings")
    ap.add_argument("--shape", default="", help="profiling aid: W,Ms,K,N of an ad-hoc AllGather-GEMM shape")
    ap.add_argument("--only-gemm", action="store_true",
                    help="profiling aid: deliver the shards once, then time the GEMM alone (prints a short line)")
    ap.add_argument("--only-reducer", action="store_true",
                    help="profiling aid: the ReduceScatter reducer alone at its full size (prints a short line); with "
                         "--pmc-calibration a 256 MiB copy of known size runs first")
    ap.add_argument("--only-moe", action="store_true",
                    help="profiling aid: routing + grouped GEMM of the MoE shape alone, tokens already gathered "
                         "(prints a short line); --pmc-calibration as for --only-reducer")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (peers are emulated on the same GPU); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2504_19442_amd as agg
    import workloads as wl
    from harness import AgGemmRun

    if (args.only_reducer or args.only_moe) and args.pmc_calibration:
        src = torch.ones(256 << 20, device="cuda", dtype=torch.uint8)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.only_moe:
        ms = wl.MOE_FULL
        gen = torch.Generator(device="cuda").manual_seed(4000)
        Xs = [(torch.rand((ms.tokens_per_rank, ms.K), device="cuda", generator=gen) * 2 - 1).to(torch.bfloat16)
              for _ in range(ms.W)]
        Wt = (torch.randn((ms.E, ms.N, ms.K), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        ids = torch.rand((ms.T, ms.E), device="cuda", generator=gen).argsort(dim=1)[:, : ms.topk].to(torch.int32).contiguous()
        mctx = agg.symm_alloc(ms.W, 0, ms.tokens_per_rank * ms.K * 2, ms.W * args.chunks)
        agg.agg_reserve_moe(mctx, ms.T, ms.topk, ms.E, ms.N)
        mp, mc = mctx.streams()
        mctx.set_tile_config(args.tile)
        Pm = ms.T * ms.topk
        Ym = torch.empty((Pm, ms.N), device="cuda", dtype=torch.bfloat16)
        tok = torch.empty((Pm,), device="cuda", dtype=torch.int32)
        seg = torch.empty((ms.E + 1,), device="cuda", dtype=torch.int32)
        agg.signal_reset(mctx)
        agg.ag_producer_emulate(mctx, Xs, None, agg.PRODUCER_KERNEL, 0, mp)
        torch.cuda.synchronize()

        def step_moe_only():
            agg.ag_moe_gemm(mctx, ms.T, ms.topk, ms.E, ms.N, ms.K, ids, Wt, tok, seg, Ym, ms.N, agg.BF16, mc)

        for _ in range(args.warmup):
            step_moe_only()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_moe_only()
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / args.steps
        assert agg.agg_status(mctx) == agg.OK
        mctx.free()
        moe_bytes = Wt.numel() * 2 + ms.T * ms.K * 2 + Pm * ms.N * 2
        print(json.dumps({"only_moe_ms": round(t * 1e3, 4), "tflops": round(ms.flops / t / 1e12, 1),
                          "algorithmic_bytes": moe_bytes, "algorithmic_GBps": round(moe_bytes / t / 1e9, 1),
                          "workload": ms.name, "tile_config": args.tile}), flush=True)
        return 0

    if args.only_reducer:
        rs = wl.RS_FULL
        slots = [torch.randn((rs.Ms, rs.N), device="cuda", dtype=torch.float32) for _ in range(rs.W)]
        R = torch.empty((rs.Ms, rs.N), device="cuda", dtype=torch.float32)
        rctx = agg.symm_alloc(rs.W, 0, 16, rs.W)
        _, rc_ = rctx.streams()
        agg.signal_reset(rctx)
        for w in range(rs.W):
            agg.signal_set(rctx, w, rc_)
        for _ in range(args.warmup):
            agg.rs_reduce(rctx, rs.Ms, rs.N, slots, R, rs.N, agg.F32, 0, rc_)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            agg.rs_reduce(rctx, rs.Ms, rs.N, slots, R, rs.N, agg.F32, 0, rc_)
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / args.steps
        assert agg.agg_status(rctx) == agg.OK
        rctx.free()
        print(json.dumps({"only_reducer_ms": round(t * 1e3, 4), "bytes": rs.reducer_bytes,
                          "achieved_GBps": round(rs.reducer_bytes / t / 1e9, 1),
                          "frac_of_hbm_peak": round(rs.reducer_bytes / t / 1e9 / PEAK_HBM_GBPS, 4),
                          "workload": rs.name}), flush=True)
        return 0

    if args.shape:
        W_, Ms_, K_, N_ = (int(x) for x in args.shape.split(","))
        shape = wl.AgGemmShape("adhoc_" + args.shape.replace(",", "x"), 99, W_, Ms_, K_, N_)
    else:
        shape = wl.AG_SHAPES[args.workload]
    rank = 0
    hev = HipEvents()

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    class AgProblem:
        """One AllGather-GEMM workload set up on the device, and the steps that are timed on it."""

        def __init__(self, shape):
            self.shape = shape
            self.inp = wl.make_ag_gemm(shape)
            self.run = AgGemmRun(self.inp, rank, chunks_per_shard=args.chunks)
            self.ctx = self.run.ctx
            self.ctx.set_tile_config(args.tile)
            # The copy kernel's workgroups: one wave each where the GEMM runs for several rounds of tiles (the copy then
            # takes a quarter of the registers and issue slots on the compute units it shares, and arrives in time all
            # the same), four waves where the GEMM is a single round and waits for the last shard to land
            rounds = ((shape.M + 255) // 256) * ((shape.N + 223) // 224) / 256.0
            self.narrow = (not args.wide_producer) and rounds >= 2.0
            self.local_flag = agg.PRODUCER_NARROW if self.narrow else 0
            if not args.t_local:
                self.ctx.set_local_shard(self.run.remote[rank])
                self.local_flag |= agg.PRODUCER_LOCAL_LAST
            self.C = torch.empty((shape.M, shape.N), device="cuda", dtype=torch.bfloat16)
            self.prod, self.cons = self.run.prod, self.run.cons
            self.prod_h, self.cons_h = self.prod.cuda_stream, self.cons.cuda_stream
            self.ev_cons_done = hev.new(timing=False)
            # Counter collection runs one kernel at a time, in the order the queues offer them: a consumer that gets
            # its turn before its producer would wait for signals that cannot come.  Under --pmc-calibration (the
            # counter runs) the producer therefore goes on the consumer's stream, ahead of the GEMM; per-kernel
            # counters are not affected.
            self.step_prod = self.cons if args.pmc_calibration else self.prod
            self.k = 0

        def gemm(self, stream=None):
            sh = self.shape
            agg.ag_gemm(self.ctx, sh.M, sh.N, sh.K, self.run.B_nk, sh.K, agg.B_NK, self.C, sh.N, agg.BF16,
                        stream or self.cons)

        def produce(self, stream, mode=None):
            flags = self.local_flag
            if mode is not None and mode != agg.PRODUCER_KERNEL:
                flags &= ~agg.PRODUCER_NARROW                 # (the narrow form exists for the copy kernel only)
            agg.ag_producer_emulate(self.ctx, self.run.remote, None, (agg.PRODUCER_KERNEL if mode is None else mode) | flags,
                                    args.producer_wgs, stream)

        def mark(self):
            hev.record(self.ev_cons_done, self.cons_h)

        def step_fused(self, ev_pairs=None, mode=None):
            agg.signal_reset(self.ctx)
            hev.wait(self.prod_h, self.ev_cons_done)     # T is shared: the next arrival waits for the last consumer
            self.produce(self.step_prod, mode)
            if ev_pairs is not None:
                e0, e1 = ev_pairs[self.k]
                self.k += 1
                hev.record(e0, self.cons_h)
            self.gemm()
            if ev_pairs is not None:
                hev.record(e1, self.cons_h)
            self.mark()

        def step_serial(self, mode=None):
            agg.signal_reset(self.ctx)
            self.produce(self.cons, mode)
            self.gemm()

        def overlap(self, n2, rounds):
            """GEMM alone (signals already set for this epoch), copy alone, serial copy-then-GEMM on one stream, fused:
            alternated over several rounds (clocks drift with load and temperature: taking them one after the other
            would bias the ratios); medians of the rounds are reported."""
            acc = {"fused": [], "gemm": [], "copy": [], "serial": []}
            for _ in range(rounds):
                self.mark()
                acc["fused"].append(timed(self.step_fused, n2, 10))
                agg.signal_reset(self.ctx)
                self.produce(self.prod)
                torch.cuda.synchronize()            # signals of this epoch are set: the GEMM alone does not wait
                acc["gemm"].append(timed(self.gemm, n2, 10))
                acc["copy"].append(timed(lambda: self.produce(self.prod), n2, 10))
                acc["serial"].append(timed(self.step_serial, n2, 10))
            assert agg.agg_status(self.ctx) == agg.OK
            t_fused, t_gemm, t_copy, t_serial = (float(np.median(acc[k])) for k in ("fused", "gemm", "copy", "serial"))
            fl = self.shape.flops
            return {
                "t_fused_ms": round(t_fused * 1e3, 4), "t_gemm_ms": round(t_gemm * 1e3, 4),
                "t_copy_ms": round(t_copy * 1e3, 4), "t_serial_ms": round(t_serial * 1e3, 4),
                "overlap_efficiency": round(t_serial / t_fused, 4),
                "hidden_fraction": round((t_serial - t_fused) / t_copy, 4),
                "fused_tflops": round(fl / t_fused / 1e12, 2),
                "fused_frac_of_bf16_peak": round(fl / t_fused / 1e12 / PEAK_BF16_TFLOPS, 4),
                "gemm_alone_tflops": round(fl / t_gemm / 1e12, 2),
                "gemm_alone_frac_of_bf16_peak": round(fl / t_gemm / 1e12 / PEAK_BF16_TFLOPS, 4),
                "fused_over_gemm": round(t_fused / t_gemm, 4),
                "protocol": f"medians of {rounds} alternating rounds of {n2} steps",
            }, t_gemm, t_copy

        def close(self):
            self.run.close()

    prob = AgProblem(shape)
    inp, run, ctx, C = prob.inp, prob.run, prob.ctx, prob.C
    M, N, K = shape.M, shape.N, shape.K
    prod, cons, prod_h, cons_h = prob.prod, prob.cons, prob.prod_h, prob.cons_h
    local_flag = prob.local_flag
    ev_cons_done = prob.ev_cons_done

    if args.only_gemm:
        agg.signal_reset(ctx)
        prob.produce(prod)
        torch.cuda.synchronize()
        t = timed(prob.gemm, args.steps, args.warmup)
        assert agg.agg_status(ctx) == agg.OK
        print(json.dumps({"only_gemm_ms": round(t * 1e3, 4), "tflops": round(shape.flops / t / 1e12, 1),
                          "workload": shape.name, "tile_config": args.tile}), flush=True)
        prob.close()
        return 0

    if args.pmc_calibration:
        src = torch.ones(256 << 20, device="cuda", dtype=torch.uint8)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    prob.mark()
    # ---- the headline: fused step.  First the settling phase (a fixed number of steps, whatever --warmup says), then
    # the --warmup steps, then exactly --steps timed ones.
    settle = 0 if args.pmc_calibration else SETTLE_STEPS
    for _ in range(settle + args.warmup):
        prob.step_fused()
    torch.cuda.synchronize()
    pairs = [(hev.new(), hev.new()) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for _ in range(args.steps):
        prob.step_fused(pairs)
    torch.cuda.synchronize()
    t_fused = (time.perf_counter() - t0) / args.steps
    assert agg.agg_status(ctx) == agg.OK, "a wait timed out during the bench"
    kern = [hev.elapsed_ms(a, b) for a, b in pairs]
    kern_ms = float(np.mean(kern))
    flops = shape.flops
    tflops = flops / t_fused / 1e12
    traffic, traffic_source = _measured_traffic(shape.name)

    out = {
        "metric": "AG-GEMM TFLOP/s (fraction of bf16 MFMA peak) + overlap efficiency vs serial",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": settle,
        "ms_per_step": round(t_fused * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": shape.name, "W": shape.W, "rank": rank, "M": M, "N": N, "K": K,
                   "signals_per_shard": args.chunks, "tile_config": args.tile, "out": "bf16",
                   "producer": "copy kernel on the producer stream, " + ("one wave" if prob.narrow else "four waves")
                               + " per workgroup, one workgroup per compute unit",
                   "own_shard": "from T" if args.t_local else "read in place, copied into T last"},
        "fraction_of_bf16_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": {"bound": "mfma", "achieved": round(flops / (kern_ms * 1e-3) / 1e12, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(flops / (kern_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "traffic_note": "HBM-side bytes per launch from an earlier rocprofv3 --pmc run (not measured by "
                                     "this run); algorithmic bytes are A + B + C once",
                     "algorithmic_bytes": shape.W * shape.Ms * K * 2 + K * N * 2 + M * N * 2,
                     "kernel": "gemm_kernel (signal-gated, fused run)",
                     "kernel_ms": round(kern_ms, 4), "kernel_ms_median": round(float(np.median(kern)), 4)},
        "targets": {"fraction_of_bf16_peak": 0.70, "hidden_fraction": 0.90,
                    "met": None},
    }

    if not args.no_extras:
        n2, rounds = max(5, args.steps // 5), 5
        out["overlap"], t_gemm, t_copy = prob.overlap(max(n2, 20), rounds)
        out["targets"]["met"] = bool(out["fraction_of_bf16_peak"] >= 0.70 and out["overlap"]["hidden_fraction"] >= 0.90)
        # the same with the other width of the copy kernel's workgroups, for comparison
        saved = prob.local_flag
        prob.local_flag ^= agg.PRODUCER_NARROW
        ov2, _, _ = prob.overlap(max(n2, 20), 3)
        prob.local_flag = saved
        out["overlap_other_producer_width"] = dict(ov2, producer=("four waves" if prob.narrow else "one wave")
                                                   + " per workgroup")

        # the 8B-MLP-shaped workload (256 tiles of 256x224: one round over the CUs), same protocol
        if not args.shape and shape.name != wl.AG_8B.name:
            p8 = AgProblem(wl.AG_8B)
            p8.mark()
            timed(p8.step_fused, 50, 100)
            pairs8 = [(hev.new(), hev.new()) for _ in range(100)]
            p8.k = 0
            t0 = time.perf_counter()
            for _ in range(100):
                p8.step_fused(pairs8)
            torch.cuda.synchronize()
            t8 = (time.perf_counter() - t0) / 100
            k8 = float(np.mean([hev.elapsed_ms(a, b) for a, b in pairs8]))
            ov8, _, _ = p8.overlap(40, 5)
            tr8, trs8 = _measured_traffic(wl.AG_8B.name)
            out["ag_gemm_8b_mlp"] = {
                "workload": wl.AG_8B.name, "M": wl.AG_8B.M, "N": wl.AG_8B.N, "K": wl.AG_8B.K,
                "ms_per_step": round(t8 * 1e3, 4), "tflops": round(wl.AG_8B.flops / t8 / 1e12, 2),
                "fraction_of_bf16_peak": round(wl.AG_8B.flops / t8 / 1e12 / PEAK_BF16_TFLOPS, 4),
                "roofline": {"bound": "mfma", "achieved": round(wl.AG_8B.flops / (k8 * 1e-3) / 1e12, 2),
                             "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                             "frac": round(wl.AG_8B.flops / (k8 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                             "kernel_ms": round(k8, 4), "traffic": tr8, "traffic_source": trs8},
                "overlap": ov8, "protocol": "100 timed steps after 150 untimed ones",
            }
            p8.close()
            del p8

        # measured ceilings beside the published peaks: the matrix pipes alone on the GEMM's register pattern (random
        # operands as in the workload, and constant operands), and the copy kernel alone for HBM
        def mfma_rate(constant):
            it = 2000
            agg.agg_mfma_ceiling(ctx, it, constant, cons)        # warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fl = 0.0
            for _ in range(100):                                 # about 0.1 s, like the timed region of the headline
                fl += agg.agg_mfma_ceiling(ctx, it, constant, cons)
            torch.cuda.synchronize()
            return fl / (time.perf_counter() - t0) / 1e12

        out["ceilings"] = {
            "mfma_loop_random_operands_tflops": round(mfma_rate(False), 1),
            "mfma_loop_constant_operands_tflops": round(mfma_rate(True), 1),
            "copy_kernel_GBps_read_plus_write": round(2.0 * shape.W * shape.Ms * K * 2 / t_copy / 1e9, 1),
            "note": "register-resident v_mfma_f32_16x16x32_bf16 loop, 224 accumulators per wave, no memory traffic",
        }
        out["roofline"]["frac_of_measured_mfma_ceiling"] = round(
            out["roofline"]["achieved"] / out["ceilings"]["mfma_loop_random_operands_tflops"], 4)

        # Full-mesh arrival at link rate (Section 3.7, the AMD case): all 7 peers at once, each on a link held to
        # `--link-gbps`, chunk by chunk; consumer in sub-chunk order, and in shard order for contrast
        ctx.set_link_rate(args.link_gbps)

        def step_mesh():
            agg.signal_reset(ctx)
            hev.wait(prod_h, ev_cons_done)
            agg.ag_producer_emulate(ctx, run.remote, None, agg.PRODUCER_LINKS | local_flag, args.producer_wgs, prod)
            agg.ag_gemm(ctx, M, N, K, run.B_nk, K, agg.B_NK, C, N, agg.BF16, cons)
            hev.record(ev_cons_done, cons_h)

        def step_mesh_copy():
            agg.ag_producer_emulate(ctx, run.remote, None, agg.PRODUCER_LINKS | local_flag, args.producer_wgs, prod)

        def step_mesh_serial():
            agg.signal_reset(ctx)
            agg.ag_producer_emulate(ctx, run.remote, None, agg.PRODUCER_LINKS | local_flag, args.producer_wgs, cons)
            agg.ag_gemm(ctx, M, N, K, run.B_nk, K, agg.B_NK, C, N, agg.BF16, cons)

        mesh = {"sub": [], "rot": [], "copy": [], "serial": []}
        n3 = max(10, args.steps // 10)
        for _ in range(3):
            hev.record(ev_cons_done, cons_h)
            ctx.set_tile_order(agg.ORDER_SUBCHUNK)
            mesh["sub"].append(timed(step_mesh, n3, 10))
            ctx.set_tile_order(agg.ORDER_ROTATED)
            mesh["rot"].append(timed(step_mesh, n3, 10))
            mesh["copy"].append(timed(step_mesh_copy, n3, 10))
            mesh["serial"].append(timed(step_mesh_serial, n3, 10))
        assert agg.agg_status(ctx) == agg.OK
        ctx.set_link_rate(0.0)
        m_sub, m_rot, m_copy, m_serial = (float(np.median(mesh[k])) for k in ("sub", "rot", "copy", "serial"))
        out["full_mesh"] = {
            "link_GBps": args.link_gbps, "links": shape.W - 1,
            "t_copy_ms": round(m_copy * 1e3, 4), "t_serial_ms": round(m_serial * 1e3, 4),
            "t_fused_subchunk_order_ms": round(m_sub * 1e3, 4), "t_fused_shard_order_ms": round(m_rot * 1e3, 4),
            "tflops_subchunk_order": round(flops / m_sub / 1e12, 2),
            "overlap_efficiency": round(m_serial / m_sub, 4),
            "hidden_fraction": round((m_serial - m_sub) / m_copy, 4),
            "hidden_fraction_shard_order": round((m_serial - m_rot) / m_copy, 4),
            "protocol": f"medians of 3 alternating rounds of {n3} steps",
        }

        # The same step with the copy engines as producer (Section 3.6: one transfer per chunk, another per signal),
        # for comparison with the copy kernel above: on one GPU an engine moves about 50 GB/s device to device
        def step_sdma():
            agg.signal_reset(ctx)
            hev.wait(prod_h, ev_cons_done)
            agg.ag_producer_emulate(ctx, run.remote, None, agg.PRODUCER_SDMA | local_flag, 0, prod)
            agg.ag_gemm(ctx, M, N, K, run.B_nk, K, agg.B_NK, C, N, agg.BF16, cons)
            hev.record(ev_cons_done, cons_h)

        def step_sdma_copy():
            agg.ag_producer_emulate(ctx, run.remote, None, agg.PRODUCER_SDMA | local_flag, 0, prod)

        hev.record(ev_cons_done, cons_h)
        s_fused = timed(step_sdma, 5, 2)
        s_copy = timed(step_sdma_copy, 5, 2)
        assert agg.agg_status(ctx) == agg.OK
        out["copy_engine_producer"] = {
            "t_copy_ms": round(s_copy * 1e3, 4), "t_fused_ms": round(s_fused * 1e3, 4),
            "copy_GBps": round(shape.W * shape.Ms * K * 2 / s_copy / 1e9, 1),
            "hidden_fraction": round((s_copy + t_gemm - s_fused) / s_copy, 4),
            "note": "one stream, shard after shard; serial time taken as copy alone + GEMM alone",
        }

        # The fused step recorded once in a HIP graph (the epoch kept on the device, so that every replay is a run
        # with fresh signals) and replayed: what a serving loop that cannot afford the launches would do
        ctx.set_device_epoch(True)
        s0 = torch.cuda.Stream()

        def enqueue_run():
            agg.signal_reset(ctx, s0)
            prod.wait_stream(s0)
            cons.wait_stream(s0)
            agg.ag_producer_emulate(ctx, run.remote, None, agg.PRODUCER_KERNEL | local_flag, args.producer_wgs, prod)
            agg.ag_gemm(ctx, M, N, K, run.B_nk, K, agg.B_NK, C, N, agg.BF16, cons)
            s0.wait_stream(prod)
            s0.wait_stream(cons)

        with torch.cuda.stream(s0):
            enqueue_run()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s0, capture_error_mode="thread_local"):
            enqueue_run()
        t_graph = timed(graph.replay, n2 * 2, 5)
        assert agg.agg_status(ctx) == agg.OK, "a wait timed out in a graph replay"
        ctx.set_device_epoch(False)
        out["graph_replay"] = {"ms_per_replay": round(t_graph * 1e3, 4), "tflops": round(flops / t_graph / 1e12, 2),
                               "note": "signal_reset + producer + gated GEMM + join as one HIP graph"}

        # the reducer of GEMM+ReduceScatter at its full size (all signals set: pure streaming reduction)
        rs = wl.RS_FULL
        slots = [torch.randn((rs.Ms, rs.N), device="cuda", dtype=torch.float32) for _ in range(rs.W)]
        R = torch.empty((rs.Ms, rs.N), device="cuda", dtype=torch.float32)
        rctx = agg.symm_alloc(rs.W, 0, 16, rs.W)
        rp, rc_ = rctx.streams()
        rcs = torch.cuda.ExternalStream(rc_)
        agg.signal_reset(rctx)
        for w in range(rs.W):
            agg.signal_set(rctx, w, rc_)

        def step_reduce():
            agg.rs_reduce(rctx, rs.Ms, rs.N, slots, R, rs.N, agg.F32, 0, rc_)

        t_red = timed(step_reduce, 100, 100)
        assert agg.agg_status(rctx) == agg.OK
        rctx.free()
        out["reducer"] = {"workload": rs.name, "bytes": rs.reducer_bytes, "ms": round(t_red * 1e3, 4),
                          "traffic": _measured_traffic(rs.name, "reduce_kernel_{}.txt"),
                          "achieved_GBps": round(rs.reducer_bytes / t_red / 1e9, 1),
                          "frac_of_hbm_peak": round(rs.reducer_bytes / t_red / 1e9 / PEAK_HBM_GBPS, 4)}

        # GEMM + ReduceScatter at its full size: one GEMM launch with the reducer on a second stream; the peers'
        # slots are signalled before the launch (values drawn on the device, same distributions).  Four variants,
        # alternated over three rounds after a common warm-up (the first thing timed after a pause runs slow).
        gen = torch.Generator(device="cuda").manual_seed(4000)
        A_loc = (torch.rand((rs.M, rs.Kl), device="cuda", generator=gen) * 2 - 1).to(torch.bfloat16)
        B_loc = (torch.randn((rs.N, rs.Kl), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        P_other = torch.empty((rs.M, rs.N), device="cuda", dtype=torch.float32)
        RS_K = 4
        gctx = agg.symm_alloc(rs.W, 0, 16, rs.W * RS_K)
        gp, gc = gctx.streams()

        def step_gemm_rs(own_last, chunks):
            def f():
                gctx.set_rs_own_slice_last(own_last)
                gctx.set_rs_chunks(chunks)
                agg.signal_reset(gctx)
                for w in range(1, rs.W):      # the peers' slots "arrive" on the reduce stream, ahead of the reducer
                    for c_ in range(chunks):
                        agg.signal_set(gctx, w * RS_K + c_, gc)
                agg.gemm_rs(gctx, rs.M, rs.N, rs.Kl, A_loc, rs.Kl, B_loc, rs.Kl, agg.B_NK, slots, P_other, R, rs.N,
                            agg.F32, gp, gc)
            return f

        def step_gemm_rs_gemm_only():        # the GEMM half alone: own slice into its slot, the rest into P_other
            agg.gemm_rs_scatter(gctx, rs.M, rs.N, rs.Kl, A_loc, rs.Kl, B_loc, rs.Kl, agg.B_NK,
                                [slots[0]] + [None] * (rs.W - 1), P_other, None, 0, gp)

        variants = {"default": step_gemm_rs(True, 1), "last4": step_gemm_rs(True, RS_K),
                    "first": step_gemm_rs(False, 1), "gemm": step_gemm_rs_gemm_only}
        timed(variants["default"], 100, 0)
        grs = {k: [] for k in variants}
        for _ in range(3):
            for k, fn in variants.items():
                grs[k].append(timed(fn, 20, 3))
        assert agg.agg_status(gctx) == agg.OK
        gctx.free()
        t_grs, t_grs_last, t_grs_first, t_grs_gemm = (float(np.median(grs[k])) for k in ("default", "last4", "first", "gemm"))
        out["gemm_rs"] = {"workload": rs.name, "ms": round(t_grs * 1e3, 4),
                          "ms_own_slice_last_4_chunks": round(t_grs_last * 1e3, 4),
                          "ms_own_slice_first": round(t_grs_first * 1e3, 4),
                          "ms_gemm_alone": round(t_grs_gemm * 1e3, 4),
                          "gemm_alone_tflops": round(2.0 * rs.M * rs.N * rs.Kl / t_grs_gemm / 1e12, 1),
                          "gemm_tflops": round(2.0 * rs.M * rs.N * rs.Kl / t_grs / 1e12, 1),
                          "protocol": "medians of 3 alternating rounds of 20 steps after 100 warm-up steps",
                          "note": "GEMM (fp32 out, 8192x8192x3584) + reducer on a second stream, per step; "
                                  "ms = the library's default (own slice last, one signal per slice)"}
        del A_loc, B_loc, P_other, slots, R

        # MoE AllGather grouped GEMM at the Table 4 shape: routing + gated grouped GEMM, producer beside it
        ms = wl.MOE_FULL
        Xs = [(torch.rand((ms.tokens_per_rank, ms.K), device="cuda", generator=gen) * 2 - 1).to(torch.bfloat16)
              for _ in range(ms.W)]
        Wt = (torch.randn((ms.E, ms.N, ms.K), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        keys = torch.rand((ms.T, ms.E), device="cuda", generator=gen)
        ids = keys.argsort(dim=1)[:, : ms.topk].to(torch.int32).contiguous()
        mctx = agg.symm_alloc(ms.W, 0, ms.tokens_per_rank * ms.K * 2, ms.W * args.chunks)
        agg.agg_reserve_moe(mctx, ms.T, ms.topk, ms.E, ms.N)
        mp, mc = mctx.streams()
        mps, mcs = torch.cuda.ExternalStream(mp), torch.cuda.ExternalStream(mc)
        Pm = ms.T * ms.topk
        Ym = torch.empty((Pm, ms.N), device="cuda", dtype=torch.bfloat16)
        tok = torch.empty((Pm,), device="cuda", dtype=torch.int32)
        seg = torch.empty((ms.E + 1,), device="cuda", dtype=torch.int32)
        ev_m = hev.new(timing=False)
        hev.record(ev_m, mc)

        def step_moe():
            agg.signal_reset(mctx)
            hev.wait(mp, ev_m)
            agg.ag_producer_emulate(mctx, Xs, None, agg.PRODUCER_KERNEL, 0, mp)
            agg.ag_moe_gemm(mctx, ms.T, ms.topk, ms.E, ms.N, ms.K, ids, Wt, tok, seg, Ym, ms.N, agg.BF16, mc)
            hev.record(ev_m, mc)

        t_moe = timed(step_moe, 30, 60)
        assert agg.agg_status(mctx) == agg.OK
        mctx.free()
        moe_bytes = Wt.numel() * 2 + ms.T * ms.K * 2 + Pm * ms.N * 2
        out["moe"] = {"workload": ms.name, "ms": round(t_moe * 1e3, 4), "tflops": round(ms.flops / t_moe / 1e12, 1),
                      "algorithmic_GBps": round(moe_bytes / t_moe / 1e9, 1),
                      "note": "routing + signal-gated grouped GEMM with the emulated gather beside it, per step"}
        del Xs, Wt, Ym

        # MoE + ReduceScatter at the Table 5 shape "MoE-RS-3": grouped GEMM, top-k reduction, reducer; peers pre-signalled
        mr = wl.MOE_RS_FULL
        Pr = mr.T * mr.topk
        Hh = (torch.rand((Pr, mr.Kl), device="cuda", generator=gen) * 2 - 1).to(torch.bfloat16)
        W2 = (torch.randn((mr.E, mr.N, mr.Kl), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        ids2 = torch.rand((mr.T, mr.E), device="cuda", generator=gen).argsort(dim=1)[:, : mr.topk].to(torch.int32).contiguous()
        g2 = torch.rand((mr.T, mr.topk), device="cuda", generator=gen) + 0.1
        g2 = (g2 / g2.sum(dim=1, keepdim=True)).contiguous()
        Yw = torch.empty((Pr, mr.N), device="cuda", dtype=torch.float32)
        tk2 = torch.empty((Pr,), device="cuda", dtype=torch.int32)
        sg2 = torch.empty((mr.E + 1,), device="cuda", dtype=torch.int32)
        pp2 = torch.empty((Pr,), device="cuda", dtype=torch.int32)
        sl2 = [torch.randn((mr.tokens_per_rank, mr.N), device="cuda", dtype=torch.float32) for _ in range(mr.W)]
        R2 = torch.empty((mr.tokens_per_rank, mr.N), device="cuda", dtype=torch.float32)
        qctx = agg.symm_alloc(mr.W, 0, 16, mr.W)
        agg.agg_reserve_moe(qctx, mr.T, mr.topk, mr.E, mr.N)
        qp, qc = qctx.streams()

        Zo = torch.empty((mr.T, mr.N), device="cuda", dtype=torch.float32)

        def step_moe_rs(z_other=Zo):
            agg.signal_reset(qctx)
            for w in range(1, mr.W):
                agg.signal_set(qctx, w, qc)
            agg.moe_rs(qctx, mr.T, mr.topk, mr.E, mr.N, mr.Kl, Hh, W2, ids2, g2, Yw, tk2, sg2, pp2, sl2, z_other, R2, mr.N,
                       agg.F32, qp, qc)

        # A rank of the real operation computes its K slice's partial sums for EVERY token and pushes seven eighths of
        # them to their owners: here they land in Z_other.  That is the step that is reported; the variant that
        # computes this rank's own tokens only (Z_other left out) is an eighth of that work and is listed beside it.
        t_mrs = timed(step_moe_rs, 50, 100)
        t_own = timed(lambda: step_moe_rs(None), 50, 50)
        assert agg.agg_status(qctx) == agg.OK
        qctx.free()
        # bytes that must move whatever the implementation: H and the weights once, the partial sums of the other
        # ranks' tokens written once (the pushes), the W slots read, R written.  The fp32 intermediate Y (written by the
        # grouped GEMM, read by the top-k reduction) is this implementation's own round trip, not compulsory traffic:
        # it is reported beside, not counted
        mrs_bytes = (Pr * mr.Kl * 2 + mr.E * mr.N * mr.Kl * 2 + (mr.T - mr.tokens_per_rank) * mr.N * 4
                     + (mr.W + 1) * mr.tokens_per_rank * mr.N * 4)
        out["moe_rs"] = {"workload": mr.name, "ms": round(t_mrs * 1e3, 4), "tflops": round(mr.flops / t_mrs / 1e12, 1),
                         "compulsory_bytes": mrs_bytes,
                         "compulsory_GBps": round(mrs_bytes / t_mrs / 1e9, 1),
                         "frac_of_hbm_peak": round(mrs_bytes / t_mrs / 1e9 / PEAK_HBM_GBPS, 4),
                         "intermediate_Y_round_trip_bytes": 2 * Pr * mr.N * 4,
                         "ms_own_tokens_only": round(t_own * 1e3, 4),
                         "note": "routing + grouped GEMM (K = 192 per rank, all tokens) + top-k reduction (all tokens; the "
                                 "other ranks' partial sums go to Z_other) + reducer, per step; ms_own_tokens_only = the "
                                 "same call without Z_other (an eighth of the GEMM's rows stored and reduced)"}
        del Zo
        del Hh, W2, Yw, sl2

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of rows of the same workload
    if args.cpu_rows > 0:
        import oracle
        rows = np.arange(0, M, max(1, M // args.cpu_rows), dtype=np.int64)[: args.cpu_rows]
        t0 = time.perf_counter()
        ref = oracle.ag_gemm(inp.shards, inp.B_kn, rank, rows=rows)
        dt = time.perf_counter() - t0
        got = C[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
        ok = bool(np.all(np.abs(got - ref) <= 0.5 * ulp + 1e-3 * np.sqrt(K) * 2.0**-8))
        out["cpu_baseline"] = {"value": round(2.0 * len(rows) * N * K / dt / 1e12, 5), "unit": "TFLOP/s",
                               "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"{len(rows)} evenly spaced rows of C (all {N} columns), {dt:.2f} s",
                               "gpu_matches_oracle_on_sample": ok}
    hev.close()
    prob.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
