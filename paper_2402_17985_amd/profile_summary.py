"""Turn rocprofv3 CSV output of `bench.py` into the short summaries kept under profiles/.

    python -m paper_2402_17985_amd.profile_summary stats   <dir> <out.txt>  "<command that made dir>"
    python -m paper_2402_17985_amd.profile_summary pmc     <dir> <out.txt>  "<command that made dir>"
    python -m paper_2402_17985_amd.profile_summary traffic <fetch dir> <write dir> <out.txt> <out.json> "<commands>"
    python -m paper_2402_17985_amd.profile_summary table   <out.txt> <bench line>.json [...] [--static <bench line>.json ...]
    python -m paper_2402_17985_amd.profile_summary fused   <out.txt> <bench line>.json   (a `bench.py --fused` run)

stats:   per-kernel call count, total and average duration from a `--kernel-trace --stats` run.
pmc:     per-kernel mean of every counter of a `--pmc` run.
traffic: HBM-side bytes per launch of the dominant GEMM kernel from a FETCH_SIZE run and a WRITE_SIZE run of
         `bench.py --copy-ref` (counters in KiB per dispatch), each scaled by what the same counter reads for the
         copy kernel of known size in the same run (1 GiB read, 1 GiB written per launch).  Writes the figures
         together with the hash of the kernel sources they belong to; bench.py reports them as roofline.traffic
         only while that hash matches the tree.

table:   one row per layer out of the JSON lines that `bench.py --configs <cfg>` printed (one file per run).

Only reads CSV / JSON files and writes text; runs nothing."""
import collections
import csv
import glob
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GIB = float(1 << 30)


def kernel_sources_sha():
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2402_17985_amd", "csrc", "*"))):
        if os.path.isfile(f):
            h.update(os.path.basename(f).encode())
            h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def _find(d, suffix):
    files = glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True)
    if not files:
        raise SystemExit(f"no *{suffix} under {d}")
    return files


def short(name, n=72):
    name = name.replace("fq::(anonymous namespace)::", "").replace("void ", "")
    return name[:n]


def kernel_durations(d):
    """{kernel: [durations in ns]} from the kernel trace."""
    out = collections.defaultdict(list)
    for f in _find(d, "kernel_trace.csv"):
        for r in csv.DictReader(open(f)):
            out[r["Kernel_Name"]].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return out


def counters(d):
    """{kernel: {counter: [values per dispatch]}}"""
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in _find(d, "counter_collection.csv"):
        for r in csv.DictReader(open(f)):
            out[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return out


def cmd_stats(d, out, command):
    dur = kernel_durations(d)
    total = sum(sum(v) for v in dur.values())
    lines = [f"# {command}", "# per kernel: calls, total ms, average us, share of GPU kernel time", ""]
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        if sum(v) < 0.002 * total:
            continue
        lines.append(f"{len(v):7d} {sum(v) / 1e6:10.3f} ms {sum(v) / len(v) / 1e3:10.2f} us {100.0 * sum(v) / total:6.2f} %  {short(k)}")
    open(out, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


def cmd_pmc(d, out, command):
    lines = [f"# {command}", "# per kernel: mean of each counter over its dispatches", ""]
    for k, c in sorted(counters(d).items()):
        n = max(len(v) for v in c.values())
        lines.append(f"{short(k)}  ({n} dispatches)")
        for name, v in sorted(c.items()):
            lines.append(f"    {name:34s} {sum(v) / len(v):16.5g}")
    open(out, "w").write("\n".join(lines) + "\n")
    print("\n".join(lines))


def _mean(c, kernel_substr, counter):
    vals = [x for k, cc in c.items() if kernel_substr in k for x in cc.get(counter, [])]
    return (sum(vals) / len(vals), len(vals)) if vals else (None, 0)


def cmd_traffic(fetch_dir, write_dir, out, out_json, command):
    cf, cw = counters(fetch_dir), counters(write_dir)
    copy_f, nf = _mean(cf, "copy_kernel", "FETCH_SIZE")
    copy_w, nw = _mean(cw, "copy_kernel", "WRITE_SIZE")
    if not copy_f or not copy_w:
        raise SystemExit("the runs hold no copy_kernel dispatches: run bench.py with --copy-ref")
    f_scale = GIB / (copy_f * 1024.0)
    w_scale = GIB / (copy_w * 1024.0)
    lines = [f"# {command}",
             f"# copy kernel of 1 GiB read + 1 GiB written: FETCH_SIZE reads {copy_f:.0f} KiB ({nf} launches) -> factor {f_scale:.3f};"
             f" WRITE_SIZE reads {copy_w:.0f} KiB ({nw} launches) -> factor {w_scale:.3f}", ""]
    rec = {"kernel_sources_sha": kernel_sources_sha(), "fetch_factor": round(f_scale, 4), "write_factor": round(w_scale, 4),
           "command": command, "bytes_per_launch": {}, "kernels": {}}
    for key, sub in (("cfg3,cfg3i8:nibble", "gemm_deep_kernel<1"), ("cfg3,cfg3i8:e3m2", "gemm_f6_wide_kernel"),
                     ("int8", "gemm_deep_kernel<0")):
        f, n1 = _mean(cf, sub, "FETCH_SIZE")
        w, n2 = _mean(cw, sub, "WRITE_SIZE")
        if f is None or w is None:
            continue
        fb, wb = f * 1024.0 * f_scale, w * 1024.0 * w_scale
        lines.append(f"{sub:24s} {n1:4d} launches: fetch {fb / 1e6:9.1f} MB  write {wb / 1e6:9.1f} MB  total {(fb + wb) / 1e6:9.1f} MB per launch")
        rec["kernels"][sub] = {"fetch_bytes": round(fb), "write_bytes": round(wb), "launches": n1}
        if ":" in key:
            rec["bytes_per_launch"][key] = round(fb + wb)
    open(out, "w").write("\n".join(lines) + "\n")
    json.dump(rec, open(out_json, "w"), indent=1)
    print("\n".join(lines))


def cmd_table(out, files, static_files):
    L = ["bench.py on the configurations of BASELINE.json (one MI355X; HIP-event timings inside bench.py; dynamic per-tensor",
         "activation scale unless marked static; bf16 output; Kpad padded to 128 channels (256 for packed nibbles)).",
         "4-bit layers as packed nibbles on the int8 MFMA; 'e3m2 us' / 'e3m2 TOPS' = the same layer's GEMM in E3M2 storage on the 6-bit MFMA.",
         "commands (from the repository root):  python3 bench.py --no-cpu --no-peak --configs <cfg> --steps 50 --warmup 30   [--static]",
         "gemm TOPS = 2*M*Kpad*N / t_gemm (%peak: of the 5.0 POP/s int8 MFMA peak); clk = shader clock during the GEMM (MHz);",
         "fq GB/s = algorithmic bytes of absmax + flatten-quantize / their time; lin = whole fq_linear; bf16 = in-library bf16 MFMA GEMM",
         "at the unflattened K; vendor = torch.matmul on the same operands; speedup = min(t bf16, t vendor) / t(fq_linear).", "",
         f"{'layer':20s} {'bits':>4s} {'M':>6s} {'K':>6s} {'N':>6s} {'Kpad':>6s} {'fq us':>8s} {'fq GB/s':>8s} {'gemm us':>8s} {'gemm TOPS':>9s} "
         f"{'%peak':>6s} {'clk':>5s} {'lin us':>8s} {'bf16 us':>8s} {'vendor us':>9s} {'speedup':>7s} {'e3m2 us':>8s} {'e3m2 TOPS':>9s}"]

    def rows(fn, tag=""):
        d = json.loads(open(fn).read().strip().split("\n")[-1])
        for r in d["layers"]:
            o = r.get("other_storage") or {}
            L.append(f"{r['layer'] + tag:20s} {r['bits']:4d} {r['M']:6d} {r['K']:6d} {r['N']:6d} {r['Kpad']:6d} "
                     f"{r['ms_flatten_quant'] * 1e3:8.1f} {r['flatten_quant_gbs']:8.0f} {r['ms_gemm'] * 1e3:8.1f} {r['gemm_tops']:9.0f} "
                     f"{r['gemm_pct_int8_peak']:6.1f} {r.get('gemm_clock_mhz', 0):5.0f} {r['ms_linear'] * 1e3:8.1f} {r['ms_gemm_bf16'] * 1e3:8.1f} "
                     f"{r.get('ms_vendor_bf16', 0) * 1e3:9.1f} {r['speedup_vs_bf16']:7.3f} {o.get('ms_gemm', 0) * 1e3:8.1f} {o.get('gemm_tops', 0):9.0f}")
        return d

    steps = []
    for fn in files:
        d = rows(fn)
        steps.append(f"  {d['config']['layers']}: {d['ms_per_step']:.4f} ms per step, {d['value']:.0f} TOPS executed, "
                     f"{d['effective_tops']:.0f} TOPS effective (unflattened K), speedup {d['speedup_vs_bf16']:.3f}")
    if static_files:
        L += ["", "static activation scale a' = T (the paper's mode: no absmax pass)"]
        for fn in static_files:
            rows(fn, " (static)")
    L += ["", "whole-step figures (value = sum of 2*M*Kpad*N over the run's layers / step time):"] + steps
    if any("cfgP" in ln for ln in L):
        L += ["", "cfgP is the shape of the paper's own operator measurement (Table 5: 8 x 2048 tokens, 4096 -> 4096, 1024 expanded channels).",
              "The paper's figures there, on one A100-80GB with library GEMMs and native INT4 tensor cores (context, another machine):",
              "flatten 0.19 ms; GEMM FP16 3.12 ms, INT8 2.35 ms, INT4 1.57 ms."]
    open(out, "w").write("\n".join(L) + "\n")
    print("\n".join(L))


def cmd_fused(out, fn):
    d = json.loads(open(fn).read().strip().split("\n")[-1])
    L = ["fq_linear_fused_a_i8 (flatten + quantize fused into the GEMM's A-operand load) against quantize-then-GEMM, INT8, bf16 in / out,",
         "one MI355X, HIP-event averages.  command:  python3 bench.py --no-cpu --no-peak --no-bmm --no-alt --fused --steps 40 --warmup 20",
         "default = fq_linear as dispatched (flatten-quantize kernel, then the large-problem GEMM); same tile = fq_linear with the GEMM forced",
         "to the 128 x 128 register-staged kernel whose structure the fused kernel shares; fused = fq_linear_fused_a_i8.", "",
         f"{'layer':14s} {'M':>6s} {'K':>6s} {'N':>6s} {'Kpad':>6s} {'scale':>8s} {'default us':>11s} {'same tile us':>13s} {'fused us':>9s} {'fused/default':>13s} {'fused/same tile':>15s} {'identical':>9s}"]
    for r in d["fused_a_operand"]:
        L.append(f"{r['layer']:14s} {r['M']:6d} {r['K']:6d} {r['N']:6d} {r['Kpad']:6d} {r['scale']:>8s} {r['ms_quantize_then_gemm'] * 1e3:11.1f} "
                 f"{r['ms_quantize_then_gemm_same_tile'] * 1e3:13.1f} {r['ms_fused'] * 1e3:9.1f} {r['ms_fused'] / r['ms_quantize_then_gemm']:13.2f} "
                 f"{r['ms_fused'] / r['ms_quantize_then_gemm_same_tile']:15.2f} {str(r['outputs_identical']):>9s}")
    open(out, "w").write("\n".join(L) + "\n")
    print("\n".join(L))


if __name__ == "__main__":
    a = sys.argv[1:]
    if len(a) == 4 and a[0] == "stats":
        cmd_stats(a[1], a[2], a[3])
    elif len(a) == 4 and a[0] == "pmc":
        cmd_pmc(a[1], a[2], a[3])
    elif len(a) == 6 and a[0] == "traffic":
        cmd_traffic(a[1], a[2], a[3], a[4], a[5])
    elif len(a) == 3 and a[0] == "fused":
        cmd_fused(a[1], a[2])
    elif len(a) >= 3 and a[0] == "table":
        rest = a[2:]
        k = rest.index("--static") if "--static" in rest else len(rest)
        cmd_table(a[1], rest[:k], rest[k + 1:])
    else:
        raise SystemExit(__doc__)
