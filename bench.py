"""Benchmark of liblg on one MI355X.

One "step" is one pass of the whole hot path: one launch of every op at every shape of the
benchmark configurations 0..4 (small matmul, reductions and transpose, matmul sweep, conv2d,
depthwise conv) on seeded synthetic inputs already resident in HBM, each op between two HIP
events on the launch stream.  Ops are ordered so that every operand was last touched more than
1 GiB of traffic earlier (cold in L2 and in the 256 MiB Infinity Cache) and so that every
memory-bound op follows a compute-bound contraction (no other kernel's write-back in its way).

Prints ONE JSON line.  `value` is the contraction throughput of the whole step (matmul + conv
FLOPs divided by the full step time, memory-bound ops included in the time); per-op figures
against their own rooflines are under `ops`; `roofline` describes the dominant kernel (the MFMA
GEMM tile the 8192^3 matmul runs on) and `cpu_baseline` the CPU oracle timed on a bounded sample.

Beside the in-step figure every memory-bound op carries `us_cold_rotating`: a batch of
back-to-back launches that rotates over distinct buffer sets adding up to at least 1 GiB, so no
launch finds its operands in a cache and no event or launch gap is charged to a 20-90 us kernel.
`ceilings` holds the measured HBM stream rates (read, write, copy probes of the library) taken
the same two ways, `extras` the ops outside the configurations (copy2d, transposed-operand
products, a large convolution, the accumulating shallow product).
"""
import argparse
import math
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_FP32_PEAK = 157.3e12      # 256 CU x 4 SIMD x 64 FLOP/clk x 2.4 GHz
HBM_PEAK = 8.0e12              # bytes/s


# HBM traffic of the dominant kernel per launch (average over its launches in one step), from two
# counter runs of this file (FETCH_SIZE, then WRITE_SIZE; commands, raw figures and the calibration
# against the copy kernel in profiles/bench_step_hbm_traffic.md).  Valid only for the kernel and
# planner sources and the launch plans the counters were taken with: anything else makes `traffic` null.
TRAFFIC = {
    "kernel": "gemm_128x128",
    "source_sha256": "1b3c26716e74f62ebfa50039e6ec355b3e034b5cbc07057b829dd2cfc912252d",
    # [block_m, block_n, k_splits] of the launches counted
    "plans": {"8192x8192x8192": [128, 128, 1], "4096x4096x4096": [128, 128, 1], "16384x512x2048": [128, 128, 1]},
    "fetch_bytes": 2513437818,       # 1227264.6 KiB read by FETCH_SIZE x 2.0 (copy-kernel calibration)
    "write_bytes": 123033203,        # 120149.6 KiB read by WRITE_SIZE x 1.0
}
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2202_03293_amd", "csrc", f)
                  for f in ("gemm_kernel.hpp", "gemm_plan.hpp", "gemm.hip")]


def kernel_source_sha256():
    import hashlib
    h = hashlib.sha256()
    for path in KERNEL_SOURCES:
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(kernel_name, plans):
    """The counted bytes, or None when the kernel, its sources or the plan of any of its launches
    differ from what the counters were taken with."""
    if TRAFFIC["source_sha256"] is None or TRAFFIC["kernel"] != kernel_name:
        return None
    if kernel_source_sha256() != TRAFFIC["source_sha256"] or TRAFFIC["plans"] != plans:
        return None
    return dict(fetch_bytes=TRAFFIC["fetch_bytes"], write_bytes=TRAFFIC["write_bytes"],
                total_bytes=TRAFFIC["fetch_bytes"] + TRAFFIC["write_bytes"])


class ClockSampler:
    """Samples the GPU's current engine and memory clocks (the starred line of the driver's
    pp_dpm_sclk / pp_dpm_mclk tables) from a thread while the timed region runs; reports nothing
    when the files are not there or not readable."""

    def __init__(self, period_s=0.1):
        import glob
        self.files = {k: sorted(glob.glob(f"/sys/class/drm/card*/device/pp_dpm_{k}"))[:1] for k in ("sclk", "mclk")}
        self.samples = {"sclk": [], "mclk": []}
        self.period_s = period_s
        self._stop = False
        self._thread = None

    def _read(self, kind):
        for path in self.files[kind]:
            try:
                with open(path) as f:
                    for line in f:
                        if line.rstrip().endswith("*"):
                            return float(line.split(":")[1].strip().split("M")[0])
            except (OSError, ValueError, IndexError):
                return None
        return None

    def _loop(self):
        while not self._stop:
            for kind in ("sclk", "mclk"):
                v = self._read(kind)
                if v is not None:
                    self.samples[kind].append(v)
            time.sleep(self.period_s)

    def __enter__(self):
        import threading
        self._thread = threading.Thread(target=self._loop, daemon=True)
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._thread.join()

    def summary(self):
        out = {}
        for kind, v in self.samples.items():
            out[kind + "_mhz"] = (dict(min=min(v), median=sorted(v)[len(v) // 2], max=max(v), samples=len(v))
                                  if v else None)
        return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults follow the paper's protocol (Section 4.3): 100 measurements per op after the warm-up,
    # reported as mean, median and quartiles; a step is ~9 ms, so this is ~1 s of GPU time
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the paper's batch-1 stride/dilation sweep (Sections 4.6.2, 4.7): launch-bound "
                         "problems, reported per launch from batches of back-to-back launches under `sweep`")
    ap.add_argument("--ceilings-sweep", action="store_true",
                    help="also sweep the HBM stream probes over workgroup size, words per lane and cache hints "
                         "(the table behind the quoted ceilings), reported under `ceilings.sweep`")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: liblg runs on ONE GPU only (it has no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2202_03293_amd as lg
    import seeded_inputs as si

    lg.lib()                                  # fail loudly when the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    def dev(a):
        return torch.from_numpy(a).cuda()

    def ws(nbytes):
        return torch.empty(nbytes // 4, device="cuda") if nbytes else None

    # ------------------------------------------------------------------ build the op list
    ops = []      # the step: dicts name, call, flops, bytes, bound, kernel
    extras = []   # ops outside the benchmark configurations, timed after the step

    def add(name, call, flops, nbytes, bound, kernel, to=None, rotate=None):
        (ops if to is None else to).append(dict(name=name, call=call, flops=float(flops), bytes=float(nbytes),
                                                bound=bound, kernel=kernel, rotate=rotate))

    def gemm_plan(M, N, K):
        return list(lg.lg_matmul_plan(M, N, K))

    def gemm_kernel_name(M, N, K):
        bm, bn, sp = gemm_plan(M, N, K)
        return (f"gemm_{bm}x{bn}" + (f"_splitk{sp}" if sp > 1 else "") +
                ("_tile_loop" if lg.lg_matmul_plan_tile_loop(M, N, K) else ""))

    host_keep = {}
    mm = {}
    sweep = [(2, case, shape) for case, shape in enumerate(si.MATMUL_SWEEP)] + [(0, 0, si.MATMUL_SMALL)]
    for seed, case, (M, N, K) in sweep:
        A, B = si.matmul_inputs(seed, M, N, K, case=case)
        if (M, N, K) == (8192, 8192, 8192):
            host_keep["mm8192"] = (A[:128].copy(), B)
        if (M, N, K) == si.MATMUL_SMALL:
            host_keep["mm256"] = (A, B)
        Ad, Bd = dev(A), dev(B)
        Cd = torch.zeros((M, N), device="cuda")
        w = ws(lg.lg_matmul_workspace_bytes(M, N, K))
        def mk_mm(Ad=Ad, Bd=Bd, M=M, N=N, K=K):
            a, b, c = Ad.clone(), Bd.clone(), torch.zeros((M, N), device="cuda")
            wk = ws(lg.lg_matmul_workspace_bytes(M, N, K))
            return lambda: lg.lg_matmul(a, b, c, workspace=wk)
        mm[(M, N, K)] = dict(name=f"matmul_{M}x{N}x{K}",
                             call=(lambda Ad=Ad, Bd=Bd, Cd=Cd, w=w: lg.lg_matmul(Ad, Bd, Cd, workspace=w)),
                             flops=2.0 * M * N * K, nbytes=4.0 * (M * K + K * N + M * N),
                             kernel=gemm_kernel_name(M, N, K), operands=(Ad, Bd), make=mk_mm)
        del A, B

    # the row and the column reduction get their own tensor of the configured shape, so the second
    # one cannot be served from what the first left in the 256 MiB Infinity Cache
    R, Cn = si.REDUCE_SHAPE
    x_rows = dev(si.uniform(1, 0, si.REDUCE_SHAPE, 0, 1))
    x_cols = dev(si.uniform(1, 2, si.REDUCE_SHAPE, 0, 1))
    out_rows = torch.empty(R, device="cuda")
    out_cols = torch.empty(Cn, device="cuda")
    ws_cols = ws(lg.lg_reduce_cols_workspace_bytes(R, Cn))
    x_tr = dev(si.uniform(1, 1, si.TRANSPOSE_SHAPE, 0, 1))
    y_tr = torch.empty((si.TRANSPOSE_SHAPE[1], si.TRANSPOSE_SHAPE[0]), device="cuda")
    x_cp = dev(si.uniform(1, 3, si.TRANSPOSE_SHAPE, 0, 1))
    y_cp = torch.empty_like(x_cp)

    n1, w1, c1, k1 = si.DWCONV1D_SHAPE
    I1h, K1h = si.dwconv1d_inputs(4, n1, w1, c1, k1)
    I1, K1 = dev(I1h), dev(K1h)
    O1 = torch.empty((n1, w1 - k1 + 1, c1), device="cuda")
    del I1h
    n2, h2, w2, c2, kh2, kw2 = si.DWCONV2D_SHAPE
    I2h, K2h = si.dwconv2d_inputs(4, n2, h2, w2, c2, kh2, kw2)
    I2, K2 = dev(I2h), dev(K2h)
    O2 = torch.empty((n2, h2 - kh2 + 1, w2 - kw2 + 1, c2), device="cuda")

    convs = []
    for case, (N, H, W, C, F, KH, KW, s) in enumerate(si.CONV2D_SHAPES + [si.CONV2D_LARGE]):
        Ih, Kh = si.conv2d_inputs(3, N, H, W, C, F, KH, KW, case=case)
        Id, Kd = dev(Ih), dev(Kh)
        OH, OW = (H - KH) // s + 1, (W - KW) // s + 1
        Od = torch.empty((N, OH, OW, F), device="cuda")
        w = ws(lg.lg_conv2d_workspace_bytes(N, H, W, C, KH, KW, F, s, s, 1, 1))
        # input elements that take part in at least one output (a 1x1 stride-2 filter skips 3/4)
        touched_in = N * OH * OW * C if (KH == 1 and KW == 1) else N * H * W * C
        def mk_conv(Id=Id, Kd=Kd, Od=Od, s=s, shape=(N, H, W, C, KH, KW, F)):
            i, k, o = Id.clone(), Kd.clone(), torch.empty_like(Od)
            n_, h_, w_, c_, kh_, kw_, f_ = shape
            wk = ws(lg.lg_conv2d_workspace_bytes(n_, h_, w_, c_, kh_, kw_, f_, s, s, 1, 1))
            return lambda: lg.lg_conv2d_nhwc_hwcf(i, k, o, stride=(s, s), workspace=wk)
        convs.append(dict(make=mk_conv, name=f"conv2d_n{N}h{H}c{C}f{F}k{KH}s{s}",
                          call=(lambda Id=Id, Kd=Kd, Od=Od, w=w, s=s:
                                lg.lg_conv2d_nhwc_hwcf(Id, Kd, Od, stride=(s, s), workspace=w)),
                          flops=2.0 * N * OH * OW * F * KH * KW * C,
                          nbytes=4.0 * (touched_in + KH * KW * C * F + N * OH * OW * F),
                          kernel="conv_" + gemm_kernel_name(N * OH * OW, F, KH * KW * C)))

    # the transposed-operand variants of the 4096^3 product (Section 4.6.1: A^T B, A B^T)
    Mt = Nt = Kt = 4096
    At_h, Bt_h = si.matmul_inputs(2, Mt, Nt, Kt, case=5)
    At_d = dev(np.ascontiguousarray(At_h.T))            # stored K x M
    Bn_d = dev(Bt_h)
    An_d = dev(At_h)
    Bt_d = dev(np.ascontiguousarray(Bt_h.T))            # stored N x K
    Ct_d = torch.zeros((Mt, Nt), device="cuda")
    wt = ws(lg.lg_matmul_workspace_bytes(Mt, Nt, Kt))
    del At_h, Bt_h

    # (the contractions of a few GFLOP get a rotating cold figure as well: `rotate`)
    def add_mm(shape, to=None, rotate=False):
        d = mm[shape]
        add(d["name"], d["call"], d["flops"], d["nbytes"], "mfma", d["kernel"], to=to,
            rotate=rotation(d["nbytes"], d["make"]) if rotate else None)

    def add_conv(c, to=None, rotate=False):
        add(c["name"], c["call"], c["flops"], c["nbytes"], "mfma", c["kernel"], to=to,
            rotate=rotation(c["nbytes"], c["make"]) if rotate else None)

    # Buffer sets for the rotating cold measurement of a memory-bound op: `make()` clones the op's
    # operands (same values, other addresses) and returns the call on the clone; at least four sets
    # and at least 2 GiB in all (eight times the Infinity Cache, so that nothing read by one launch
    # survives until its set comes round again, whichever hints keep the outputs out of the caches).
    def rotation(nbytes, make):
        return dict(sets=min(64, max(4, math.ceil((2 << 30) / nbytes))), make=make)

    tr_bytes, red_bytes = 8.0 * x_tr.numel(), 4.0 * (R * Cn)
    dw1_bytes = 4.0 * (O1.numel() + K1.numel() + I1.numel())
    dw2_bytes = 4.0 * (O2.numel() + K2.numel() + I2.numel())

    def mk_transpose():
        x, y = x_tr.clone(), torch.empty_like(y_tr)
        return lambda: lg.lg_transpose(x, y)

    def mk_copy():
        x, y = x_cp.clone(), torch.empty_like(y_cp)
        return lambda: lg.lg_copy2d(x, y)

    def mk_rows():
        x, y = x_rows.clone(), torch.empty_like(out_rows)
        return lambda: lg.lg_reduce_rows(x, y)

    def mk_cols():
        x, y, w = x_cols.clone(), torch.empty_like(out_cols), ws(lg.lg_reduce_cols_workspace_bytes(R, Cn))
        return lambda: lg.lg_reduce_cols(x, y, workspace=w)

    def mk_dw1():
        x, y = I1.clone(), torch.empty_like(O1)
        return lambda: lg.lg_dwconv1d_nwc_wc(x, K1, y)

    def mk_dw2():
        x, y = I2.clone(), torch.empty_like(O2)
        return lambda: lg.lg_dwconv2d_nhwc_hwc(x, K2, y)

    # Order.  What a kernel writes with ordinary stores lingers dirty in the 256 MiB Infinity Cache and
    # is paid for by whichever later kernel next allocates there (streaming loads and stores pass it
    # by).  Two ops leave their whole output behind, 256 MiB each (transpose, 1-D depthwise), so:
    # every memory-bound op directly follows a contraction and finds its operands cold (last touched a
    # whole step, > 1 GiB of traffic, ago); the transpose is followed by the 4096^3 and 16384 x 512 x
    # 2048 products (370 MB of distinct operands between them) and the 1-D depthwise op, last in the
    # step, by the 8192^3 product that opens the next one (805 MB), which flush what they left before
    # the next memory-bound op starts.
    add_mm((8192, 8192, 8192))
    add("transpose_8192x8192", lambda: lg.lg_transpose(x_tr, y_tr), 0, tr_bytes, "hbm", "transpose",
        rotate=rotation(tr_bytes, mk_transpose))
    add_mm((4096, 4096, 4096))
    add_mm((16384, 512, 2048))
    add("reduce_rows_4096x16384", lambda: lg.lg_reduce_rows(x_rows, out_rows), R * Cn, 4.0 * (R * Cn + R), "hbm",
        "reduce_rows", rotate=rotation(red_bytes, mk_rows))
    add_conv(convs[0], rotate=True)
    add("reduce_cols_4096x16384", lambda: lg.lg_reduce_cols(x_cols, out_cols, workspace=ws_cols), R * Cn,
        4.0 * (R * Cn + Cn), "hbm", "reduce_cols", rotate=rotation(red_bytes, mk_cols))
    add_conv(convs[1], rotate=True)
    add("dwconv2d_n8h114c96k3", lambda: lg.lg_dwconv2d_nhwc_hwc(I2, K2, O2), 2.0 * O2.numel() * kh2 * kw2,
        dw2_bytes, "hbm", "dwconv2d", rotate=rotation(dw2_bytes, mk_dw2))
    add_conv(convs[2], rotate=True)
    add_mm((1024, 1024, 1024), rotate=True)
    add_mm((4096, 4096, 64), rotate=True)
    add_mm(si.MATMUL_SMALL)          # configuration 0: 0.2 us of math, a launch-latency figure
    # depthwise bytes follow the paper's accounting: output written, filter read, input read once
    add("dwconv1d_n32w4098c512k3", lambda: lg.lg_dwconv1d_nwc_wc(I1, K1, O1), 2.0 * O1.numel() * k1,
        dw1_bytes, "hbm", "dwconv1d", rotate=rotation(dw1_bytes, mk_dw1))

    # Outside the configurations: the copy yardstick, the transposed-operand products, a convolution
    # large enough to fill the machine, and the shallow product accumulating into C (the output is
    # read as well as written, which halves the arithmetic intensity: the HBM side of the ridge).
    add_mm((4096, 4096, 4096), to=extras)      # predecessor of the copy, as in the step; not reported twice
    add("copy2d_8192x8192", lambda: lg.lg_copy2d(x_cp, y_cp), 0, 8.0 * x_cp.numel(), "hbm", "copy2d", to=extras,
        rotate=rotation(8.0 * x_cp.numel(), mk_copy))
    add_conv(convs[3], to=extras)
    add("matmul_AtB_4096x4096x4096", lambda: lg.lg_matmul_t(At_d, Bn_d, Ct_d, trans_a=True, workspace=wt),
        2.0 * Mt * Nt * Kt, 12.0 * Mt * Nt, "mfma", gemm_kernel_name(Mt, Nt, Kt) + "_tn", to=extras)
    add("matmul_ABt_4096x4096x4096", lambda: lg.lg_matmul_t(An_d, Bt_d, Ct_d, trans_b=True, workspace=wt),
        2.0 * Mt * Nt * Kt, 12.0 * Mt * Nt, "mfma", gemm_kernel_name(Mt, Nt, Kt) + "_nt", to=extras)
    d64 = mm[(4096, 4096, 64)]
    A64, B64 = d64["operands"]
    C64acc = torch.zeros((4096, 4096), device="cuda")
    add("matmul_4096x4096x64_accumulate", lambda: lg.lg_matmul(A64, B64, C64acc, accumulate=True), d64["flops"],
        4.0 * (2 * 4096 * 64 + 2 * 4096 * 4096), "mfma", d64["kernel"] + "_acc", to=extras)

    # ------------------------------------------------------------------ run
    def run_list(lst, events=None):
        for i, op in enumerate(lst):
            if events is not None:
                events[i][0].record(stream)
            op["call"]()
            if events is not None:
                events[i][1].record(stream)

    def event_grid(lst, n):
        return [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in lst]
                for _ in range(n)]

    for _ in range(args.warmup):
        run_list(ops)
    torch.cuda.synchronize()
    all_events = event_grid(ops, args.steps)
    torch.cuda.synchronize()
    clocks = ClockSampler()
    with clocks:
        t0 = time.perf_counter()
        for k in range(args.steps):
            run_list(ops, all_events[k])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    def op_records(lst, grid):
        recs = []
        for i, op in enumerate(lst):
            ts = np.array([a.elapsed_time(b) for a, b in (ev[i] for ev in grid)]) * 1e-3
            mean, med = float(ts.mean()), float(np.median(ts))
            rec = dict(op=op["name"], kernel=op["kernel"], bound=op["bound"], us_mean=mean * 1e6, us_median=med * 1e6,
                       us_p25=float(np.percentile(ts, 25)) * 1e6, us_p75=float(np.percentile(ts, 75)) * 1e6)
            if op["bound"] == "mfma":
                rec.update(gflops=op["flops"] / mean / 1e9, frac_mfma_peak=op["flops"] / mean / MFMA_FP32_PEAK,
                           gbps=op["bytes"] / mean / 1e9, frac_hbm_peak=op["bytes"] / mean / HBM_PEAK)
            else:
                rec.update(gbps=op["bytes"] / mean / 1e9, frac_hbm_peak=op["bytes"] / mean / HBM_PEAK,
                           gflops=op["flops"] / mean / 1e9)
            op["mean_s"] = mean
            recs.append(rec)
        return recs

    per_op = op_records(ops, all_events)

    # the ops outside the configurations, the same way (20 passes)
    for _ in range(3):
        run_list(extras)
    extra_events = event_grid(extras, 20)
    for k in range(20):
        run_list(extras, extra_events[k])
    torch.cuda.synchronize()
    per_extra = op_records(extras, extra_events)[1:]
    extras = extras[1:]

    # What the two events cost an op in the step: a pair with nothing between, and a pair around the
    # smallest launch there is (a copy of one row of four floats), each directly behind a 4096^3 product
    # like the ops of the step.
    tiny_x, tiny_y = torch.zeros((1, 4), device="cuda"), torch.zeros((1, 4), device="cuda")
    behind = next(op for op in ops if op["name"] == "matmul_4096x4096x4096")["call"]
    ev_pairs, ev_tiny = [], []
    for _ in range(30):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        behind()
        e[0].record(stream)
        e[1].record(stream)
        behind()
        e[2].record(stream)
        lg.lg_copy2d(tiny_x, tiny_y)
        e[3].record(stream)
        torch.cuda.synchronize()
        ev_pairs.append(e[0].elapsed_time(e[1]) * 1e3)
        ev_tiny.append(e[2].elapsed_time(e[3]) * 1e3)
    event_overhead = dict(us_between_two_events=float(np.median(ev_pairs)),
                          us_smallest_launch_between_events=float(np.median(ev_tiny)),
                          note="medians of 30; every in-step figure (us_mean ...) contains the second: marker, "
                               "dispatch of a kernel behind it, marker behind the kernel")

    # the measured ceiling for the contractions: a register-only MFMA issue loop, long enough (~14 ms
    # per launch) for the engine clock to settle -- a one-millisecond launch from idle reads 10 % low
    probe_out = torch.empty(lg.lg_mfma_probe_out_elems(), device="cuda")
    probe_iters = 64000
    lg.lg_mfma_probe(probe_out, probe_iters)
    torch.cuda.synchronize()
    probe_ts = []
    for _ in range(5):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        lg.lg_mfma_probe(probe_out, probe_iters)
        b.record(stream)
        torch.cuda.synchronize()
        probe_ts.append(a.elapsed_time(b) * 1e-3)
    mfma_measured = lg.lg_mfma_probe_flops(probe_iters) / float(np.median(probe_ts))
    for r in per_op + per_extra:
        if r["bound"] == "mfma":
            r["frac_mfma_measured"] = r["gflops"] * 1e9 / mfma_measured

    contraction_flops = sum(op["flops"] for op in ops if op["bound"] == "mfma")
    value = contraction_flops / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the GEMM tile the 8192^3 matmul runs on, averaged over ALL launches of a step
    # that share that kernel (a kernel-trace summary groups them the same way)
    dom_name = mm[(8192, 8192, 8192)]["kernel"]
    dom = [op for op in ops if op["kernel"] == dom_name]
    dom_flops = sum(op["flops"] for op in dom) / len(dom)
    dom_dur = sum(op["mean_s"] for op in dom) / len(dom)
    roofline = dict(bound="mfma", kernel=f"lg::gemm_kernel<{dom_name}, vec, matmul>",
                    launches_per_step=len(dom), ops=[op["name"] for op in dom],
                    flops_per_launch=dom_flops, avg_launch_us=dom_dur * 1e6,
                    achieved=dom_flops / dom_dur / 1e12, peak=MFMA_FP32_PEAK / 1e12, unit="TFLOP/s",
                    frac=dom_flops / dom_dur / MFMA_FP32_PEAK,
                    measured_ceiling=mfma_measured / 1e12, frac_of_measured_ceiling=dom_flops / dom_dur / mfma_measured)
    dom_plans = {op["name"].split("_", 1)[1]: gemm_plan(*[int(v) for v in op["name"].split("_", 1)[1].split("x")])
                 for op in dom}
    tr = measured_traffic(dom_name, dom_plans)
    # HBM bytes per launch as counted (null once the kernel or planner sources or the plan of one of the
    # launches differ from the counted ones), beside the operand bytes per launch; the excess is A/B
    # panels streamed once per block of output tiles
    roofline.update(traffic=tr["total_bytes"] if tr else None, traffic_unit="bytes per launch",
                    traffic_fetch_bytes=tr["fetch_bytes"] if tr else None,
                    traffic_write_bytes=tr["write_bytes"] if tr else None,
                    algorithmic_bytes=sum(op["bytes"] for op in dom) / len(dom), plans=dom_plans,
                    source_sha256=kernel_source_sha256())

    out = dict(metric="matmul/conv GFLOP/s (% fp32 MFMA peak); reduce/transpose GB/s (% HBM peak)",
               value=value, unit="GFLOP/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=ms_per_step, higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="f32", data="synthetic",
               config=dict(workload="configs[0..4]: matmul 256^3; reduce_rows, reduce_cols 4096x16384; transpose 8192^2; matmul "
                                    "sweep 1024^3, 4096^3, 8192^3, 16384x512x2048, 4096x4096x64; conv2d x3; dwconv1d; dwconv2d; "
                                    "one launch of each per step"),
               frac_mfma_peak=value * 1e9 / MFMA_FP32_PEAK, roofline=roofline, clocks=clocks.summary(), ops=per_op,
               extras=per_extra, event_overhead=event_overhead)

    # ------------------------------------------------------------------ cold, rotating buffer sets
    # A batch of back-to-back launches that walks over `sets` distinct copies of the operands (>= 1 GiB
    # in all, several times the 256 MiB Infinity Cache): every launch finds its operands cold, and no
    # event or launch gap is charged to it.  Beside it, the same launches one by one between events.
    def cold_rotating(calls, rounds=3, reps=5):
        for c in calls:
            c()
        torch.cuda.synchronize()
        # a batch lasts at least ~8 ms and follows ~30 ms of the same launches, so that a short op is timed at
        # the clocks sustained work runs at (2-3 ms batches of a 25 us kernel started from an idle GPU read
        # 10 % slower); more passes over the same >= 2 GiB of buffer sets stay cold
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for c in calls:
            c()
        b.record(stream)
        torch.cuda.synchronize()
        one_pass_ms = max(a.elapsed_time(b), 1e-3)
        rounds = max(rounds, min(40, math.ceil(8.0 / one_pass_ms)))
        for _ in range(min(200, math.ceil(30.0 / one_pass_ms))):   # ~30 ms of the same launches, untimed
            for c in calls:
                c()
        batch, single = [], []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(rounds):
                for c in calls:
                    c()
            b.record(stream)
            torch.cuda.synchronize()
            batch.append(a.elapsed_time(b) * 1e3 / (rounds * len(calls)))
        for r in range(max(15, len(calls))):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            calls[r % len(calls)]()
            b.record(stream)
            torch.cuda.synchronize()
            single.append(a.elapsed_time(b) * 1e3)
        return float(np.median(batch)), float(np.median(single))

    # HBM stream ceilings from the library's probes (lg_stream_probe), at 256 MiB per stream and at
    # the footprint of the small depthwise op, measured like the ops: rotating batch and one by one.
    def stream_ceiling(mode, nfloats, threads=256, unroll=1, hint=3):
        nbytes = 4.0 * nfloats * (2 if mode == "copy" else 1)
        sets = max(4, math.ceil((2 << 30) / nbytes))
        sink = torch.zeros(1024, device="cuda")
        calls = []
        for _ in range(sets):
            x = torch.ones(nfloats, device="cuda") if mode != "write" else None
            y = torch.empty(nfloats, device="cuda") if mode != "read" else sink
            calls.append(lambda x=x, y=y: lg.lg_stream_probe(mode, x, y, threads=threads, unroll=unroll, hint=hint))
        b, s1 = cold_rotating(calls)
        del calls
        torch.cuda.empty_cache()
        return dict(mode=mode, bytes=nbytes, threads=threads, words_per_lane=unroll, hint=hint,
                    us_cold_rotating=b, gbps_cold_rotating=nbytes / b / 1e3, frac_hbm_peak_cold_rotating=nbytes / b / 1e3 / (HBM_PEAK / 1e9),
                    us_single=s1, gbps_single=nbytes / s1 / 1e3, frac_hbm_peak_single=nbytes / s1 / 1e3 / (HBM_PEAK / 1e9))

    big = (256 << 20) // 4
    ceilings = dict(read=stream_ceiling("read", big), write=stream_ceiling("write", big), copy=stream_ceiling("copy", big),
                    copy_at_dwconv2d_size=stream_ceiling("copy", O2.numel()),
                    note="lg_stream_probe, 256 lanes x one 128-bit word per lane, non-temporal hints on both sides "
                         "(the best point of the sweep in profiles/hbm_ceilings.md); 256 MiB per stream, and a copy of "
                         "the 2-D depthwise output's size (its input is 3.6 % larger)")
    if args.ceilings_sweep:
        sw = []
        for mode in ("read", "write", "copy"):
            for threads in (256, 512, 1024):
                for unroll in (1, 2, 4, 8):
                    for hint in ((3, 0) if mode != "copy" else (3, 0, 1, 2)):
                        if mode == "copy" and unroll == 8:
                            continue     # 8 words per lane in flight both ways: an order of magnitude slower, says nothing
                        sw.append(stream_ceiling(mode, big, threads, unroll, hint))
        ceilings["sweep"] = sw
    out["ceilings"] = ceilings

    for op, rec in list(zip(ops, per_op)) + list(zip(extras, per_extra)):
        if op["rotate"] is None:
            continue
        calls = [op["rotate"]["make"]() for _ in range(op["rotate"]["sets"])]
        b, s1 = cold_rotating(calls)
        del calls
        torch.cuda.empty_cache()
        if op["bound"] == "mfma":
            rec.update(us_cold_rotating=b, gflops_cold_rotating=op["flops"] / b / 1e3,
                       frac_mfma_peak_cold_rotating=op["flops"] / b / 1e3 / (MFMA_FP32_PEAK / 1e9),
                       us_cold_single=s1, buffer_sets=op["rotate"]["sets"])
            continue
        ceil = ceilings["read"] if op["kernel"].startswith("reduce") else \
            ceilings["copy_at_dwconv2d_size"] if op["kernel"] == "dwconv2d" else ceilings["copy"]
        rec.update(us_cold_rotating=b, gbps_cold_rotating=op["bytes"] / b / 1e3,
                   frac_hbm_peak_cold_rotating=op["bytes"] / b / 1e3 / (HBM_PEAK / 1e9),
                   us_cold_single=s1, buffer_sets=op["rotate"]["sets"],
                   stream_ceiling=ceil["mode"] + ("" if ceil is not ceilings["copy_at_dwconv2d_size"] else " (same size)"),
                   frac_of_stream_ceiling_cold_rotating=(op["bytes"] / b) / (ceil["bytes"] / ceil["us_cold_rotating"]),
                   frac_of_stream_ceiling_in_step=(op["bytes"] / rec["us_mean"]) / (ceil["bytes"] / ceil["us_single"]))

    # The memory-bound ops and every op under 50 us once more, 10 / 20 launches back to back on the same buffers: "warm" figures
    # (part of a 256 MiB operand is still in the last-level cache, and no other kernel's write-back
    # is in the way), to set beside the cold figures of the step above.
    def back_to_back_us(call, batch=10, reps=5):
        call()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(batch):
                call()
            b.record(stream)
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3 / batch)
        return float(np.median(ts))

    for op, rec in list(zip(ops, per_op)) + list(zip(extras, per_extra)):
        if op["bound"] == "hbm" or rec["us_mean"] < 50.0:      # short launches too: event resolution, launch gaps
            rec["us_warm_back_to_back"] = back_to_back_us(op["call"], batch=10 if op["bound"] == "hbm" else 20)
            if op["bound"] == "hbm":
                rec["gbps_warm"] = op["bytes"] / rec["us_warm_back_to_back"] / 1e3
            else:
                rec["gflops_warm"] = op["flops"] / rec["us_warm_back_to_back"] / 1e3

    # ------------------------------------------------------------------ launch-bound problems
    def per_launch_us(call, batch=20, reps=7):
        """(eager, graph): microseconds per launch from batches of back-to-back launches, issued one
        by one through the Python binding and replayed from a HIP graph of the same batch."""
        for _ in range(batch):
            call()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(batch):
                call()

        def timed(run):
            ts = []
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                run()
                b.record(stream)
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b) * 1e3 / batch)
            return float(np.median(ts))

        def eager():
            for _ in range(batch):
                call()
        return timed(eager), timed(graph.replay)

    # configuration 0 is 34 MFLOP: inside the step above its figure is the cost of one launch issued
    # from Python between two events.  Back to back, and replayed from a graph, it is the kernel's own
    # latency on top of the dispatch floor (an empty-handed copy of one row, timed the same way).
    sm_call = mm[si.MATMUL_SMALL]["call"]
    sm_eager, sm_graph = per_launch_us(sm_call)
    tiny_in, tiny_out = torch.zeros((1, 64), device="cuda"), torch.zeros((1, 64), device="cuda")
    _, floor_graph = per_launch_us(lambda: lg.lg_copy2d(tiny_in, tiny_out))
    out["small_matmul"] = dict(shape=list(si.MATMUL_SMALL), kernel=mm[si.MATMUL_SMALL]["kernel"],
                               us_per_launch_eager=sm_eager, us_per_launch_graph=sm_graph,
                               us_dispatch_floor_graph=floor_graph,
                               gflops_graph=mm[si.MATMUL_SMALL]["flops"] / sm_graph / 1e3)

    # ------------------------------------------------------------------ the paper's small sweep
    if args.sweep:
        sweep = []
        for size in (16, 20, 32, 40, 55, 64, 128):
            for sd in ((1, 1), (2, 1), (1, 2), (2, 2)):
                st, dl = sd
                # (N, C, F, K_w) = (1, 32, 64, 3): conv1d over W = size, conv2d over H = W = size
                I1s = dev(si.uniform(5, 0, (1, size, 32), -1, 1)); K1s = dev(si.uniform(5, 1, (3, 32, 64), -1, 1))
                ow = lg.lg_conv_out_extent(size, 3, st, dl)
                if ow > 0:
                    O1s = torch.empty((1, ow, 64), device="cuda")
                    w1s = ws(lg.lg_conv1d_workspace_bytes(1, size, 32, 3, 64, st, dl))
                    us, ug = per_launch_us(lambda: lg.lg_conv1d_nwc_wcf(I1s, K1s, O1s, stride=st, dilation=dl, workspace=w1s))
                    sweep.append(dict(op="conv1d", size=size, stride=st, dilation=dl, us=us, us_graph=ug,
                                      gflops=2.0 * ow * 64 * 3 * 32 / ug / 1e3))
                    I2s = dev(si.uniform(5, 2, (1, size, size, 32), -1, 1)); K2s = dev(si.uniform(5, 3, (3, 3, 32, 64), -1, 1))
                    O2s = torch.empty((1, ow, ow, 64), device="cuda")
                    w2s = ws(lg.lg_conv2d_workspace_bytes(1, size, size, 32, 3, 3, 64, st, st, dl, dl))
                    us, ug = per_launch_us(lambda: lg.lg_conv2d_nhwc_hwcf(I2s, K2s, O2s, stride=(st, st), dilation=(dl, dl),
                                                                         workspace=w2s))
                    sweep.append(dict(op="conv2d", size=size, stride=st, dilation=dl, us=us, us_graph=ug,
                                      gflops=2.0 * ow * ow * 64 * 9 * 32 / ug / 1e3))
                    Kd = dev(si.uniform(5, 4, (3, 32), -1, 1)); Od = torch.empty((1, ow, 32), device="cuda")
                    us, ug = per_launch_us(lambda: lg.lg_dwconv1d_nwc_wc(I1s, Kd, Od, stride=st, dilation=dl))
                    sweep.append(dict(op="dwconv1d", size=size, stride=st, dilation=dl, us=us, us_graph=ug,
                                      gbps=4.0 * (ow * 32 + 3 * 32 + size * 32) / ug / 1e3))
        # 2-D depthwise at the batch-1 MobileNet layer sizes of Section 4.7 (output extent x channels)
        for size, C in ((112, 32), (112, 64), (56, 128), (28, 256), (14, 512), (7, 1024)):
            for st, dl in ((1, 1), (2, 1), (1, 2), (2, 2)):
                H = (size - 1) * st + 2 * dl + 1
                Id2 = dev(si.uniform(5, 5, (1, H, H, C), -1, 1)); Kd2 = dev(si.uniform(5, 6, (3, 3, C), -1, 1))
                Od2 = torch.empty((1, size, size, C), device="cuda")
                us, ug = per_launch_us(lambda: lg.lg_dwconv2d_nhwc_hwc(Id2, Kd2, Od2, stride=(st, st), dilation=(dl, dl)))
                g = math.gcd(st, dl)
                sweep.append(dict(op="dwconv2d", size=size, channels=C, stride=st, dilation=dl, us=us, us_graph=ug,
                                  gbps=4.0 * (size * size * C + 9 * C + H * H * C / (g * g)) / ug / 1e3))
        out["sweep"] = sweep

    # ------------------------------------------------------------------ CPU oracle baseline
    if not args.no_cpu_baseline:
        from oracle import lgo
        A128, B = host_keep["mm8192"]
        t = time.perf_counter()
        lgo.matmul(A128, B)
        dt = time.perf_counter() - t
        others = {}
        xs = si.uniform(1, 0, (1024, 16384), 0, 1)
        t = time.perf_counter(); lgo.reduce_rows(xs); d = time.perf_counter() - t
        others["reduce_rows_GBps"] = xs.nbytes / d / 1e9
        t = time.perf_counter(); lgo.reduce_cols(xs); d = time.perf_counter() - t
        others["reduce_cols_GBps"] = xs.nbytes / d / 1e9
        xt = si.uniform(1, 1, (2048, 8192), 0, 1)
        t = time.perf_counter(); lgo.transpose(xt); d = time.perf_counter() - t
        others["transpose_GBps"] = 2 * xt.nbytes / d / 1e9
        t = time.perf_counter(); lgo.dwconv2d_nhwc_hwc(I2h, K2h); d = time.perf_counter() - t
        others["dwconv2d_GBps"] = 4.0 * (O2.numel() + K2.numel() + I2.numel()) / d / 1e9
        A256, B256 = host_keep["mm256"]
        t = time.perf_counter(); lgo.matmul(A256, B256); d = time.perf_counter() - t
        others["matmul_256_all_threads_GFLOPs"] = 2.0 * 256 ** 3 / d / 1e9
        # the paper's own numbers are single-threaded: the same 256^3 product on one host thread, in a
        # child process that only loads the oracle (the thread count is fixed when OpenMP starts)
        import subprocess
        code = ("import sys, time; sys.path.insert(0, %r); import seeded_inputs as si; from oracle import lgo; "
                "A, B = si.matmul_inputs(0, 256, 256, 256, case=0); lgo.matmul(A, B); t = time.perf_counter(); "
                "lgo.matmul(A, B); print(2.0 * 256 ** 3 / (time.perf_counter() - t) / 1e9)" % ROOT)
        try:
            r = subprocess.run([sys.executable, "-c", code], env=dict(os.environ, OMP_NUM_THREADS="1"),
                               capture_output=True, text=True, timeout=120)
            others["matmul_256_one_thread_GFLOPs"] = float(r.stdout.strip().splitlines()[-1])
        except (subprocess.SubprocessError, ValueError, IndexError):
            others["matmul_256_one_thread_GFLOPs"] = None
        out["cpu_baseline"] = dict(value=2.0 * 128 * 8192 * 8192 / dt / 1e9, unit="GFLOP/s",
                                   cores=lgo.num_threads(), kind="oracle",
                                   sample="rows 0..127 of the 8192^3 matmul (naive fp64-accumulate loop nest, "
                                          f"{dt:.1f} s); other ops on slices: {json.dumps(others)}")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
