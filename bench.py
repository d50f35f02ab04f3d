#!/usr/bin/env python3
"""Benchmark of the FlattenQuant linear-layer hot path on one MI355X.

Workload (default): the metric's "M = 8192 LLaMA-7B shapes" — the INT4 FFN pair 4096->11008 and
11008->4096 plus the INT8 4096->4096 projection, all at M = 8192 tokens, synthetic outlier-bearing
bf16 activations (fq_workloads.py).  One step = one fq_linear call per layer: dynamic per-tensor
absmax, fused flatten-quantize, integer GEMM with the dequantize epilogue (bf16 out).
Inputs are resident in HBM before the timed region.

The 4-bit layers are timed as the task names them: packed two per byte in HBM and LDS, widened to int8 in
registers, multiplied on the int8 MFMA with int32 accumulation.  The same layers in the second storage
(E3M2 codes on the 6-bit MFMA; same integers, bit-identical accumulators) are measured beside it and
reported under "int4_storage", each storage with its own roofline; --e3m2 makes that one the timed path.

Prints ONE JSON line: whole-step throughput in TOPS (integer ops actually executed, 2*M*Kpad*N per
layer), the roofline of the dominant kernel (the 4-bit GEMM) from HIP-event timings taken in this
process, the ceilings measured on this GPU (MFMA-only loops on zero and on live operands, a plain copy,
the clock the GEMMs ran at), and the CPU oracle timed on a bounded sample.
"""
import argparse
import glob
import hashlib
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA peak (packed INT4 is widened to int8 on chip: same ceiling)
FP6_PEAK_TFLOPS = 10100.0    # dense 6-bit MFMA peak: the ceiling of the 4-bit layers in E3M2 storage
BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0
RAMP_MS = 150.0              # load applied before any timed region: the clock needs tens of ms to settle


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_sources_sha():
    """Hash of the kernel sources: a stored profile figure belongs to the binary built from exactly these."""
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2402_17985_amd", "csrc", "*"))):
        if os.path.isfile(f):
            h.update(os.path.basename(f).encode())
            h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(workload, path):
    """HBM-side bytes per launch of the dominant kernel from profiles/ (two rocprofv3 --pmc runs), or None when
    the stored figure was measured on other kernel sources than the ones in the tree."""
    fn = os.path.join(ROOT, "profiles", "traffic_dominant_kernel.json")
    try:
        rec = json.load(open(fn))
    except (OSError, ValueError):
        return None, "no stored profile"
    if rec.get("kernel_sources_sha") != kernel_sources_sha():
        return None, "stored profile is from other kernel sources (stale)"
    v = rec.get("bytes_per_launch", {}).get(f"{workload}:{path}")
    return v, ("profiles/traffic_dominant_kernel.json (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not this run)" if v else
               "no stored figure for this workload")


class PowerSampler:
    """Board power from the driver's sysfs node while a region runs (plain file reads on a helper thread)."""

    def __init__(self):
        self.files = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") + \
            glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")
        self.samples, self._stop, self._thr = [], threading.Event(), None

    def _run(self):
        while not self._stop.is_set():
            for f in self.files[:1]:
                try:
                    self.samples.append(int(open(f).read()) / 1e6)
                except (OSError, ValueError):
                    pass
            time.sleep(0.005)

    def __enter__(self):
        if self.files:
            self._thr = threading.Thread(target=self._run, daemon=True)
            self._thr.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self._thr:
            self._thr.join()

    def watts(self):
        s = sorted(self.samples)
        return None if not s else round(s[len(s) // 2], 0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--configs", default="cfg3,cfg3i8", help="comma-separated workload names from fq_workloads")
    ap.add_argument("--variant", type=int, default=-1, help="force a GEMM tile variant (fq_gemm_select)")
    ap.add_argument("--static", action="store_true", help="static activation scale a' = T (the paper's mode)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--sweep", action="store_true", help="also time every GEMM variant per layer (stderr table)")
    ap.add_argument("--align", type=int, default=0,
                    help="padding of the flattened width (0: 128 channels for INT8, 256 for INT4, so that rows start "
                         "on 128-byte boundaries; 32 is the paper's value)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and replay it instead of launching eagerly")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run one plain 1 GiB device copy at the end (the reference kernel for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--no-bmm", action="store_true", help="skip the attention-shaped batched-product rows")
    ap.add_argument("--fused", action="store_true",
                    help="also time fq_linear_fused_a_i8 against quantize-then-GEMM on the INT8 layers of cfg3i8 and cfg5")
    ap.add_argument("--e3m2", action="store_true",
                    help="time the 4-bit layers as E3M2 codes on the 6-bit MFMA instead of packed nibbles on the int8 MFMA")
    ap.add_argument("--no-alt", action="store_true", help="do not also measure the 4-bit storage that is not timed")
    ap.add_argument("--no-peak", action="store_true", help="skip the measured ceilings (MFMA-only loops, copy)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives or sharding are part of it); use --gpus 1")

    import numpy as np
    import torch

    import fq_workloads as WL
    import paper_2402_17985_amd as fq
    from paper_2402_17985_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    fq.lib()
    dev = "cuda:0"
    fq.fq_gemm_select(args.variant)
    E3 = B.FQ_BITS_I4_E3M2
    # storage of a layer's quantized tensors on the timed path / on the other path (None: no other)
    store_of = lambda bits: bits if (bits == 8 or not args.e3m2) else E3
    alt_of = lambda bits: None if (bits == 8 or args.no_alt) else (4 if args.e3m2 else E3)
    storage_name = {8: "int8", 4: "nibble", E3: "e3m2"}
    wall_khz = fq.fq_peak_wall_clock_khz() or 100000

    def event_time_ms(fn, iters, warmup=10):
        """Average duration of fn() over `iters` launches, HIP events on the current stream."""
        for _ in range(warmup):
            fn()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record()
        for _ in range(iters):
            fn()
        stop.record()
        stop.synchronize()
        return start.elapsed_time(stop) / iters

    ticks = torch.zeros(2, dtype=torch.int64, device=dev)

    def gemm_time_and_clock(fn, iters):
        """event_time_ms of a GEMM call with the kernels' clock probe on: (ms, average shader clock in MHz)."""
        fq.fq_peak_gemm_ticks(ticks)
        try:
            for _ in range(10):
                fn()
            ticks.zero_()
            ms = event_time_ms(fn, iters, warmup=0)
            t = ticks.cpu().numpy()
        finally:
            fq.fq_peak_gemm_ticks(None)
        mhz = float(t[0]) / float(t[1]) * wall_khz / 1e3 if t[1] > 0 else None
        return ms, mhz

    def ramp_and_time(run, steps, warmup):
        """Load until the clock has settled (at least RAMP_MS and `warmup` steps), then time exactly `steps` steps."""
        t0, n = time.perf_counter(), 0
        while n < warmup or (time.perf_counter() - t0) * 1e3 < RAMP_MS:
            run()
            n += 1
            if n % 16 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        with PowerSampler() as ps:
            t0 = time.perf_counter()
            for _ in range(steps):
                run()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) * 1e3 / steps
        return dt, ps.watts(), n

    # ---------------- build the layers (offline part: plan + weight quantization) ----------------
    layers = []
    for cname in args.configs.split(","):
        cfg = WL.CONFIGS[cname]
        for li in range(len(cfg.layers)):
            t0 = time.time()
            L = WL.make_layer(cfg, li)
            sp = L.spec

            def upload(store, dtype):
                if dtype == "bf16":
                    return torch.from_numpy(store.view(np.int16)).to(dev).view(torch.bfloat16)
                return torch.from_numpy(store).to(dev)
            Xd, Wd = upload(L.X_store, sp.x_dtype), upload(L.W_store, sp.w_dtype)
            lay = fq.FqLinear(Wd, L.chmax, L.T, store_of(sp.bits), device=dev, align=args.align)
            lay_alt = None
            if alt_of(sp.bits) is not None:
                lay_alt = fq.FqLinear(Wd, L.chmax, L.T, alt_of(sp.bits), device=dev, align=args.align)
                lay_alt.workspace(sp.M)
            Y = torch.empty((sp.M, sp.N), dtype=torch.bfloat16, device=dev)
            Ybf = torch.empty((sp.M, sp.N), dtype=torch.bfloat16, device=dev)
            a_static = torch.tensor([L.T], dtype=torch.float32, device=dev) if args.static else None
            lay.workspace(sp.M)
            # operands of the bf16 baseline GEMM (the tensors themselves when they already are bf16)
            Xb = Xd if Xd.dtype == torch.bfloat16 else Xd.to(torch.bfloat16)
            Wb = Wd if Wd.dtype == torch.bfloat16 else Wd.to(torch.bfloat16)
            # flattened width with the paper's padding to 32 channels (what the useful-work figure counts)
            _, _, kprime, _ = fq.fq_flatten_plan(L.chmax, L.T, 32)
            kpad32 = (kprime + 31) // 32 * 32
            layers.append(dict(name=f"{cname}.{sp.name}", spec=sp, L=L, X=Xd, W=Wd, Xb=Xb, Wb=Wb, lay=lay, lay_alt=lay_alt,
                               Y=Y, Ybf=Ybf, a_static=a_static, kpad32=kpad32))
            log(f"[setup] {cname}.{sp.name}: M={sp.M} K={sp.K} N={sp.N} bits={sp.bits} T={L.T:.4g} "
                f"Kprime={lay.Kprime} Kpad={lay.Kpad} (+{100.0 * (lay.Kpad - sp.K) / sp.K:.1f}%) "
                f"max n={int(lay.rep_host.max())} [{time.time() - t0:.1f}s]")
    torch.cuda.synchronize()

    def step():
        for d in layers:
            d["lay"].forward(d["X"], Y=d["Y"], absmax_in=d["a_static"])

    # --graph: one step (15 kernel launches) is captured once into a HIP graph and replayed, which
    # removes the host launch path from between the kernels; the library records no memset nodes (its
    # clears are fill kernels).
    run_step = step
    if args.graph:
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay

    # ---------------- the timed region: warm-up (clock ramp included), then exactly K steps ----------------
    t_step_ms, watts_step, n_warm = ramp_and_time(run_step, args.steps, args.warmup)

    # the same step with the 4-bit layers in the other storage (reported beside the timed path)
    t_alt_ms = None
    if any(d["lay_alt"] is not None for d in layers):
        def step_alt():
            for d in layers:
                (d["lay_alt"] or d["lay"]).forward(d["X"], Y=d["Y"], absmax_in=d["a_static"])
        t_alt_ms, _, _ = ramp_and_time(step_alt, args.steps, args.warmup)

    ops_hw = sum(2.0 * d["spec"].M * d["lay"].Kpad * d["spec"].N for d in layers)
    ops_eff = sum(2.0 * d["spec"].M * d["spec"].K * d["spec"].N for d in layers)
    ops_pad32 = sum(2.0 * d["spec"].M * d["kpad32"] * d["spec"].N for d in layers)
    value = ops_hw / (t_step_ms * 1e-3) / 1e12

    # ---------------- per-kernel breakdown (HIP events, same process) ----------------
    rows = []
    t_bf16_total = t_vendor_total = t_best_bf16_total = 0.0
    dom_bits = 4 if any(d["spec"].bits == 4 for d in layers) else 8
    # per storage of the dominant (4-bit, else 8-bit) GEMM: flops, ms, launches, time-weighted clock
    per_store = {}
    fqa = dict(bytes=0.0, ms=0.0)

    def kernels_of(d, lay):
        """(flatten-quantize call, GEMM call, bytes of Xq) of one layer in the storage of `lay`."""
        sp, Kpad, st = d["spec"], lay.Kpad, lay.bits
        if st == E3:
            Xq = torch.empty((Kpad // 128, sp.M, 96), dtype=torch.uint8, device=dev)
        else:
            Xq = torch.empty((sp.M, Kpad if st == 8 else Kpad // 2), dtype=torch.int8 if st == 8 else torch.uint8, device=dev)
        s_x = torch.empty(1, dtype=torch.float32, device=dev)
        ws = torch.empty(fq.fq_act_workspace_bytes(sp.K, Kpad), dtype=torch.uint8, device=dev)
        f_act = lambda: fq.fq_flatten_quant_act(d["X"], lay.src, lay.rep, st, Xq, s_x, ws, absmax_in=d["a_static"])
        if st == E3:
            f_gemm = lambda: fq.fq_gemm_i4_e3m2(Xq, lay.Wq, s_x, lay.s_w, None, d["Y"])
        else:
            gemm = fq.fq_gemm_i8 if st == 8 else fq.fq_gemm_i4
            f_gemm = lambda: gemm(Xq, lay.Wq, s_x, lay.s_w, d["Y"])
        return f_act, f_gemm, Xq.numel(), (Xq, s_x, ws)

    def measure(d, lay):
        sp = d["spec"]
        f_act, f_gemm, xq_bytes, keep = kernels_of(d, lay)
        t_act = event_time_ms(f_act, args.steps)
        t_gemm, mhz = gemm_time_and_clock(f_gemm, args.steps)
        t_lin = event_time_ms(lambda: lay.forward(d["X"], Y=d["Y"], absmax_in=d["a_static"]), args.steps)
        flops = 2.0 * sp.M * lay.Kpad * sp.N
        # algorithmic HBM bytes of flatten-quantize: X read once (static) or twice (dynamic), Xq written
        act_bytes = sp.M * sp.K * d["X"].element_size() * (1 if args.static else 2) + xq_bytes
        if sp.bits == dom_bits:
            ps = per_store.setdefault(lay.bits, dict(flops=0.0, ms=0.0, launches=0, mhz_ms=0.0))
            ps["flops"] += flops
            ps["ms"] += t_gemm
            ps["launches"] += 1
            ps["mhz_ms"] += (mhz or 0.0) * t_gemm
        peak = FP6_PEAK_TFLOPS if lay.bits == E3 else INT8_PEAK_TOPS
        res = dict(storage=storage_name[lay.bits], Kpad=lay.Kpad, ms_flatten_quant=round(t_act, 4), ms_gemm=round(t_gemm, 4),
                   ms_linear=round(t_lin, 4), gemm_tops=round(flops / t_gemm / 1e9, 1),
                   gemm_pct_of_own_peak=round(100 * flops / t_gemm / 1e9 / peak, 2),
                   gemm_pct_int8_peak=round(100 * flops / t_gemm / 1e9 / INT8_PEAK_TOPS, 2),
                   gemm_clock_mhz=None if mhz is None else round(mhz, 0),
                   flatten_quant_gbs=round(act_bytes / t_act / 1e6, 1),
                   linear_eff_tops=round(2.0 * sp.M * sp.K * sp.N / t_lin / 1e9, 1))
        return res, act_bytes, t_act, t_lin, f_gemm, keep

    for d in layers:
        sp, lay = d["spec"], d["lay"]
        res, act_bytes, t_act, t_lin, f_gemm, keep = measure(d, lay)
        f_bf = lambda: fq.fq_gemm_bf16(d["Xb"], d["Wb"], d["Ybf"])
        t_bf = event_time_ms(f_bf, args.steps)
        # reference only: the vendor library's bf16 GEMM (through torch.matmul) on the same operands
        t_vendor = event_time_ms(lambda: torch.matmul(d["Xb"], d["Wb"].t(), out=d["Ybf"]), args.steps)
        t_bf16_total += t_bf
        t_vendor_total += t_vendor
        t_best_bf16_total += min(t_bf, t_vendor)
        fqa["bytes"] += act_bytes
        fqa["ms"] += t_act
        row = dict(layer=d["name"], bits=sp.bits, M=sp.M, K=sp.K, N=sp.N, Kpad_at_32=d["kpad32"], **res,
                   ms_gemm_bf16=round(t_bf, 4), ms_vendor_bf16=round(t_vendor, 4),
                   bf16_tflops=round(2.0 * sp.M * sp.K * sp.N / t_bf / 1e9, 1),
                   vendor_bf16_tflops=round(2.0 * sp.M * sp.K * sp.N / t_vendor / 1e9, 1),
                   speedup_vs_bf16=round(min(t_bf, t_vendor) / t_lin, 3),
                   speedup_vs_inlibrary_bf16=round(t_bf / t_lin, 3), speedup_vs_vendor_bf16=round(t_vendor / t_lin, 3))
        if d["lay_alt"] is not None:
            res_alt, _, _, _, _, keep_alt = measure(d, d["lay_alt"])
            row["other_storage"] = res_alt
            del keep_alt
        rows.append(row)
        log("[kernel] " + json.dumps(row))
        if args.sweep:
            for v in (2, 6, 7, 10, 11):
                if v == 11 and lay.bits != 8:
                    continue
                fq.fq_gemm_select(v)
                tg = event_time_ms(f_gemm, max(5, args.steps // 2))
                log(f"[sweep] {d['name']} variant {v}: gemm {tg:.4f} ms = {2.0 * sp.M * lay.Kpad * sp.N / tg / 1e9:.0f} TOPS")
            fq.fq_gemm_select(args.variant)
        del keep

    def storage_roofline(st):
        ps = per_store.get(st)
        if not ps:
            return None
        avg_ms = ps["ms"] / ps["launches"]
        achieved = ps["flops"] / ps["launches"] / avg_ms / 1e9
        if st == E3:
            kernel, peak, unit = "gemm_f6_wide_kernel (4-bit values as E3M2 codes, 6-bit MFMA)", FP6_PEAK_TFLOPS, "TFLOP/s"
        else:
            kernel, peak, unit = f"int{dom_bits} GEMM on the int8 MFMA", INT8_PEAK_TOPS, "TOP/s"
        traffic, traffic_source = stored_traffic(args.configs, storage_name[st])
        return dict(bound="mfma", kernel=kernel, achieved=round(achieved, 1), peak=peak, unit=unit,
                    frac=round(achieved / peak, 4), traffic=traffic, traffic_source=traffic_source,
                    avg_launch_ms=round(avg_ms, 4), launches_per_step=ps["launches"],
                    frac_of_int8_peak=round(achieved / INT8_PEAK_TOPS, 4),
                    clock_mhz_during_kernel=round(ps["mhz_ms"] / ps["ms"], 0) if ps["mhz_ms"] else None)

    timed_store = store_of(dom_bits)
    roofline = storage_roofline(timed_store)
    int4_storage = None
    if dom_bits == 4:
        int4_storage = {}
        for st, t_ms in ((timed_store, t_step_ms), (alt_of(4), t_alt_ms)):
            if st is None or t_ms is None:
                continue
            lay_in = lambda d: d["lay"] if (d["lay"].bits == st or d["spec"].bits == 8) else d["lay_alt"]
            ops_st = sum(2.0 * d["spec"].M * lay_in(d).Kpad * d["spec"].N for d in layers)
            int4_storage[storage_name[st]] = dict(
                timed_path=(st == timed_store), ms_per_step=round(t_ms, 4), value=round(ops_st / (t_ms * 1e-3) / 1e12, 2),
                bytes_per_value=0.5 if st == 4 else 0.75, roofline=storage_roofline(st))
    flatten_roofline = dict(bound="hbm", kernel="colabsmax + scale + flatten_quant", achieved=round(fqa["bytes"] / fqa["ms"] / 1e6, 1),
                            peak=HBM_PEAK_GBS, unit="GB/s", frac=round(fqa["bytes"] / fqa["ms"] / 1e6 / HBM_PEAK_GBS, 4))

    # ---------------- ceilings measured on this GPU ----------------
    # MFMA-only loops (no memory traffic) per matrix-pipe format on all-zero operands and on live ones (the workload's
    # own quantized weights); each also reports the shader clock it ran at (s_memtime over s_memrealtime) and the
    # board power.  A plain 1 GiB copy.  These are the ceilings the nominal peaks above should be read with.
    measured_peak = None
    if not args.no_peak:
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        blocks = 2 * cus
        sink = torch.empty(blocks * 256, dtype=torch.float32, device=dev)
        pticks = torch.zeros(2 * blocks, dtype=torch.int64, device=dev)
        macs = {B.FQ_PEAK_I8: 32768, B.FQ_PEAK_BF16: 16384, B.FQ_PEAK_E3M2: 65536, B.FQ_PEAK_I8_NIBBLES: 32768}

        def live_operand(st):
            for d in layers:
                for lay in (d["lay"], d["lay_alt"]):
                    if lay is not None and lay.bits == st and lay.Wq.numel() >= 65536:
                        return lay.Wq
            return None

        def mfma_peak(kind, operands, iters):
            # ramp on the same loop first, then time one launch
            t0 = time.perf_counter()
            while (time.perf_counter() - t0) * 1e3 < RAMP_MS:
                fq.fq_peak_mfma(kind, operands, blocks, iters // 8, None, sink)
                torch.cuda.synchronize()
            with PowerSampler() as ps:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fq.fq_peak_mfma(kind, operands, blocks, iters, pticks, sink)
                e1.record()
                e1.synchronize()
            ms = e0.elapsed_time(e1)
            t = pticks.cpu().numpy().reshape(-1, 2).astype(np.float64)
            mhz = float((t[:, 0] / np.maximum(t[:, 1], 1.0)).mean()) * wall_khz / 1e3
            return dict(tops=round(blocks * 4 * iters * 16 * macs[kind] * 2 / ms / 1e9, 0), clock_mhz=round(mhz, 0),
                        board_watts=ps.watts())
        measured_peak = {"unit": "TOP/s (dense multiply-adds x 2)", "method": "fq_peak_mfma: 16 independent 32x32 MFMAs per "
                         "loop pass, operands in registers, 2 x CUs workgroups of 4 waves; live = the workload's quantized weights"}
        for name, kind, st, iters in (("int8", B.FQ_PEAK_I8, 8, 120000), ("int8_on_widened_nibbles", B.FQ_PEAK_I8_NIBBLES, 4, 120000),
                                      ("e3m2", B.FQ_PEAK_E3M2, E3, 60000), ("bf16", B.FQ_PEAK_BF16, "bf16", 120000)):
            ops_live = layers[0]["Wb"] if st == "bf16" else live_operand(st)
            entry = {}
            if kind != B.FQ_PEAK_I8_NIBBLES:
                entry["zeros"] = mfma_peak(kind, None, iters)
            if ops_live is not None:
                entry["live"] = mfma_peak(kind, ops_live, iters)
            measured_peak[name] = entry
        src_buf = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst_buf = torch.empty_like(src_buf)
        t_copy = event_time_ms(lambda: fq.fq_peak_copy(src_buf, dst_buf), 10, warmup=3)
        measured_peak["copy_1gib_gbs_read_plus_write"] = round(2.0 * src_buf.numel() * 4 / t_copy / 1e6, 0)
        del src_buf, dst_buf, sink, pticks
        log("[peak] " + json.dumps(measured_peak))
        # the dominant kernel against the live ceiling of its own pipe
        key = {4: "int8_on_widened_nibbles", 8: "int8", E3: "e3m2"}[timed_store]
        live = measured_peak.get(key, {}).get("live")
        if roofline and live:
            roofline["frac_of_measured_live_mfma_peak"] = round(roofline["achieved"] / live["tops"], 4)

    # ---------------- batched integer product on attention shapes (reported beside the step) ----------------
    # OPT-13B attention geometry (40 heads of 128) at 2048 tokens, 4 sequences: Q K^T [2048 x 2048 x 128] and
    # P V [2048 x 128 x 2048] per head, 160 heads; per-tensor scales, bf16 output.  Both are bound by HBM:
    # algorithmic bytes = operands read once + output written once.
    bmm_rows = []
    if not args.no_bmm:
        heads, S, dh = 160, 2048, 128
        gen = torch.Generator(device=dev)
        gen.manual_seed(1234)
        one = torch.ones(1, dtype=torch.float32, device=dev)
        for name, Mb, Nb, Kb in (("QK^T", S, S, dh), ("PV", S, dh, S)):
            for bits in (8, 4):
                rb = Kb if bits == 8 else Kb // 2
                Aq = torch.randint(-128, 128, (heads, Mb, rb), dtype=torch.int8, device=dev, generator=gen)
                Bq = torch.randint(-128, 128, (heads, Nb, rb), dtype=torch.int8, device=dev, generator=gen)
                if bits == 4:
                    Aq, Bq = Aq.view(torch.uint8), Bq.view(torch.uint8)
                Yb = torch.empty((heads, Mb, Nb), dtype=torch.bfloat16, device=dev)
                f = fq.fq_bmm_i8 if bits == 8 else fq.fq_bmm_i4
                t = event_time_ms(lambda: f(Aq, Bq, one, one, Yb), args.steps)
                nbytes = heads * ((Mb + Nb) * rb + Mb * Nb * 2)
                row = dict(op=f"bmm_i{bits} {name}", batch=heads, M=Mb, N=Nb, K=Kb, ms=round(t, 4),
                           gbs=round(nbytes / t / 1e6, 1), pct_hbm_peak=round(100 * nbytes / t / 1e6 / HBM_PEAK_GBS, 2),
                           tops=round(2.0 * heads * Mb * Nb * Kb / t / 1e9, 1))
                bmm_rows.append(row)
                log("[kernel] " + json.dumps(row))
                del Aq, Bq, Yb

    # ---------------- flatten + quantize fused into the GEMM's A-operand load (on request) ----------------
    # The INT8 layer three ways on the same inputs: the default path (quantize, then the large-problem GEMM), the same
    # two steps with the GEMM forced to the 128 x 128 register-staged kernel (the structure the fused kernel shares),
    # and fq_linear_fused_a_i8, which reads X in the GEMM.  Static and dynamic activation scale.
    fused_rows = []
    if args.fused:
        for cname, idx in (("cfg3i8", 0), ("cfg5", 1)):
            Lf = WL.make_layer(WL.CONFIGS[cname], idx)
            sp = Lf.spec
            layf = fq.FqLinear(torch.from_numpy(Lf.W_store.view(np.int16)).to(dev).view(torch.bfloat16), Lf.chmax, Lf.T, 8, device=dev)
            Xf = torch.from_numpy(Lf.X_store.view(np.int16)).to(dev).view(torch.bfloat16)
            Yf = torch.empty((sp.M, sp.N), dtype=torch.bfloat16, device=dev)
            Yg = torch.empty_like(Yf)
            wsf = torch.empty(fq.fq_linear_workspace_bytes(sp.M, sp.K, layf.Kpad, 8), dtype=torch.uint8, device=dev)
            for static in (False, True):
                a_in = torch.full((1,), float(Lf.T), dtype=torch.float32, device=dev) if static else None
                unfused = lambda: fq.fq_linear(Xf, layf.src, layf.rep, layf.Wq, layf.s_w, 8, Yf, wsf, absmax_in=a_in)
                fused = lambda: fq.fq_linear_fused_a_i8(Xf, layf.src, layf.rep, layf.Wq, layf.s_w, Yg, wsf, absmax_in=a_in)
                t_default = event_time_ms(unfused, args.steps)
                fq.fq_gemm_select(2)
                try:
                    t_same = event_time_ms(unfused, max(args.steps // 4, 5))
                finally:
                    fq.fq_gemm_select(args.variant)
                t_fused = event_time_ms(fused, max(args.steps // 4, 5))
                unfused()
                fused()
                torch.cuda.synchronize()
                row = dict(layer=f"{cname}.{sp.name}", M=sp.M, K=sp.K, N=sp.N, Kpad=layf.Kpad, scale="static" if static else "dynamic",
                           ms_quantize_then_gemm=round(t_default, 4), ms_quantize_then_gemm_same_tile=round(t_same, 4),
                           ms_fused=round(t_fused, 4), outputs_identical=bool(torch.equal(Yf.view(torch.int16), Yg.view(torch.int16))))
                fused_rows.append(row)
                log("[fused] " + json.dumps(row))
            del Lf, layf, Xf, Yf, Yg, wsf

    if args.copy_ref:
        src_buf = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst_buf = torch.empty_like(src_buf)
        for _ in range(3):
            fq.fq_peak_copy(src_buf, dst_buf)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src_buf, dst_buf

    # ---------------- CPU oracle on a bounded sample ----------------
    # The same step (fq_linear per layer) on the host cores, layers taken largest first; a layer that
    # would take longer than the budget is cut to its first rows.  About 20 s in total.
    cpu = None
    if not args.no_cpu:
        from oracle import fq_oracle as O
        budget, spent, ops, parts = 20.0, 0.0, 0.0, []
        for d in sorted(layers, key=lambda d: -(d["spec"].M * d["lay"].Kpad * d["spec"].N)):
            if spent >= 0.6 * budget:
                break
            L, sp, lay = d["L"], d["spec"], d["lay"]
            Wq_o, s_w_o = O.flatten_weights(L.W, lay.src_host, sp.bits)      # offline part, not timed
            a_st = np.float32(L.T) if args.static else None
            t0 = time.perf_counter()
            O.linear(L.X, lay.src_host, lay.rep_host, Wq_o, s_w_o, sp.bits, a_static=a_st, row0=0, rows=64)
            t_probe = time.perf_counter() - t0                                # includes the full-tensor absmax
            t0 = time.perf_counter()
            O.linear(L.X, lay.src_host, lay.rep_host, Wq_o, s_w_o, sp.bits, a_static=a_st, row0=0, rows=128)
            per_row = max((time.perf_counter() - t0 - t_probe) / 64.0, 1e-6)
            nrows = int(min(sp.M, max(64, (budget - spent) / per_row)))
            t0 = time.perf_counter()
            acc_o, y_o, s_x_o = O.linear(L.X, lay.src_host, lay.rep_host, Wq_o, s_w_o, sp.bits, a_static=a_st, row0=0, rows=nrows)
            dt = time.perf_counter() - t0
            spent += dt
            ops += 2.0 * nrows * lay.Kpad * sp.N
            parts.append(f"{d['name']}: first {nrows} of {sp.M} rows (Kpad={lay.Kpad}, N={sp.N}, INT{sp.bits}) {dt:.1f} s")
            # the sample doubles as a check of the timed call: the bf16 tensor that the timed launch configuration
            # stores (same buffers, same kernel instantiation) against the oracle's rounded output, bit for bit
            lay.forward(d["X"], Y=d["Y"], absmax_in=d["a_static"])
            torch.cuda.synchronize()
            got = d["Y"][:nrows].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            same = bool(np.array_equal(got, O.dequant_out(acc_o, s_x_o, s_w_o, "bf16")))
            log(f"[check] {d['name']}: the timed call's bf16 output equals the oracle's rounded output bit for bit on the "
                f"{nrows}-row sample: {same}")
            if not same:
                sys.exit("bench.py: GPU result differs from the oracle on the sampled rows")
            del got, acc_o, y_o
        cpu = dict(value=round(ops / spent / 1e12, 5), unit="TOPS", cores=O.num_threads(), kind="oracle",
                   sample="fq_linear (dynamic absmax over all rows, flatten-quantize, integer GEMM, dequantize) on "
                          + "; ".join(parts))

    out = {
        "metric": "fq_linear_tops_m8192_llama7b_shapes",
        "value": round(value, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(t_step_ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("int4 as e3m2 codes (6-bit MFMA, exact integer products, fp32 accumulate below 2^24) + int8 "
                  "(int8 MFMA, int32 accumulate); bf16 in/out" if args.e3m2 else
                  "int4 (packed nibbles widened to int8 on chip) + int8, int8 MFMA with int32 accumulation; bf16 in/out"),
        "data": "synthetic",
        "config": {"workload": "+".join(args.configs.split(",")) +
                               ": LLaMA-7B FFN pair 4096->11008->4096 INT4 and 4096->4096 INT8 projection, M=8192 tokens, "
                               "bf16 activations with 0.5% outlier channels x[10,100], <=15% of channels flattened",
                   "activation_scale": "static a'=T" if args.static else "dynamic per-tensor absmax",
                   "layers": [r["layer"] for r in rows], "gemm_variant": args.variant,
                   "launch": "one HIP graph per step, replayed" if args.graph else "eager",
                   "int4_storage": "E3M2 codes, k-blocked" if args.e3m2 else "packed nibbles, two per byte",
                   "kpad_align": args.align if args.align else ("128" if args.e3m2 else "128 (INT8) / 256 (INT4)"),
                   "warmup_steps_run": n_warm, "clock_ramp_ms": RAMP_MS},
        "pct_int8_mfma_peak": round(100.0 * value / INT8_PEAK_TOPS, 2),
        "effective_tops": round(ops_eff / (t_step_ms * 1e-3) / 1e12, 2),
        "tops_at_paper_padding_32": round(ops_pad32 / (t_step_ms * 1e-3) / 1e12, 2),
        "board_watts_during_timed_steps": watts_step,
        "speedup_vs_bf16": round(t_best_bf16_total / t_step_ms, 3),
        "speedup_vs_bf16_note": "against the faster of the in-library and the vendor bf16 GEMM, per layer",
        "speedup_vs_inlibrary_bf16": round(t_bf16_total / t_step_ms, 3),
        "ms_bf16_gemm_same_shapes": round(t_bf16_total, 4),
        "speedup_vs_vendor_bf16": round(t_vendor_total / t_step_ms, 3),
        "ms_vendor_bf16_gemm_same_shapes": round(t_vendor_total, 4),
        "roofline": roofline,
        "flatten_quant_roofline": flatten_roofline,
        "int4_storage": int4_storage,
        "measured_peak": measured_peak,
        "cpu_baseline": cpu,
        "layers": rows,
        "bmm": bmm_rows,
        "fused_a_operand": fused_rows,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
