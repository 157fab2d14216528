"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/.

The summaries are what the roofline figures of bench.py are checked against, so they must be
reproducible from the repository alone.  Every run below starts from /tmp on the GPU machine
(`cd /tmp && export TMPDIR=/tmp`), BENCH = `python3 <repo>/bench.py --config N --oracle-layers 0 --no-other-configs`:

  kernel trace   rocprofv3 --kernel-trace --stats -d DIR/trace -o t --output-format csv -- BENCH --steps 20 --warmup 3 > DIR/bench.json
  HBM reads      rocprofv3 --pmc FETCH_SIZE -d DIR/fetch -o f --output-format csv -- BENCH --steps 3 --warmup 1
  HBM writes     rocprofv3 --pmc WRITE_SIZE -d DIR/write -o w --output-format csv -- BENCH --steps 3 --warmup 1
  LDS            rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_INSTS_LDS SQ_ACTIVE_INST_LDS -d DIR/lds -o l --output-format csv -- BENCH --steps 3 --warmup 1
  calibration    rocprofv3 --pmc FETCH_SIZE -d DIR/cal_f -o f --output-format csv -- python3 <repo>/bench.py --copy-calibration
                 rocprofv3 --pmc WRITE_SIZE -d DIR/cal_w -o w --output-format csv -- python3 <repo>/bench.py --copy-calibration

then, anywhere the CSVs are:

  python -m paper_2510_17777_amd.profile_summary --config N --dir DIR --out profiles [--head GIT_REVISION]

writes profiles/decode_step_cfgN_kernel_trace.txt and profiles/decode_step_cfgN_traffic_and_lds.txt.

The kernels of `bench.py --variants` (attention-mass retrieval, encoder salience, packing; VBENCH =
`python3 <repo>/bench.py --variants --oracle-layers 0`) have summaries of their own:

  kernel trace   rocprofv3 --kernel-trace --stats -d DIR/vtrace -o v --output-format csv -- VBENCH > DIR/vbench.json
  SQ counters    rocprofv3 --pmc SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_ACTIVE_INST_VALU SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_WAIT_INST_LDS SQ_ACTIVE_INST_LDS -d DIR/vpmc1 -o m --output-format csv -- VBENCH --steps 5 --warmup 1
                 rocprofv3 --pmc SQ_WAIT_INST_ANY SQ_WAIT_ANY SQ_ACTIVE_INST_ANY SQ_INSTS_VALU_TRANS_F32 SQ_LDS_BANK_CONFLICT SQ_INSTS_LDS SQ_INSTS_SALU SQ_LDS_IDX_ACTIVE -d DIR/vpmc2 -o m --output-format csv -- VBENCH --steps 5 --warmup 1
                 rocprofv3 --pmc SQ_VALU_MFMA_COEXEC_CYCLES SQ_BUSY_CU_CYCLES -d DIR/vpmc3 -o m --output-format csv -- VBENCH --steps 5 --warmup 1

  python -m paper_2510_17777_amd.profile_summary --variants --dir DIR --out profiles [--head GIT_REVISION]

writes profiles/variants_cfg4_kernel_trace.txt, profiles/mass_retrieval_cfg4_sq_counters.txt and
profiles/salience_encoder_layers_sq_counters.txt.
The counters FETCH_SIZE / WRITE_SIZE are in KiB per dispatch; each is scaled by what the same counter reads
for the library's plain copy kernel of 1 GiB (the factor is printed in the summary).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

KERNELS = ("score_kernel", "scores_filter_kernel", "select_filtered_kernel", "select_single_kernel", "select_hist_kernel",
           "select_threshold_kernel", "select_emit_kernel", "attn_partial_flash_kernel", "attn_partial_mfma_kernel",
           "attn_partial_kernel", "attn_combine_kernel", "step_tail_kernel", "pack_kernel", "copy_kernel", "read_kernel",
           "mass_rowstat_kernel", "mass_colsum_kernel", "mass_lse_kernel", "salience_rowstat_kernel",
           "salience_colsum_kernel", "salience_final_kernel")


def short_name(mangled: str):
    """Readable kernel name from rocprofv3's (mangled or demangled) one; None for kernels that are not the library's."""
    hit = None
    for k in KERNELS:
        if re.search(r"(?<![a-z_])" + k + r"(?![a-z_])", mangled):
            hit = k
            break
    if hit is None:
        return None
    if hit == "score_kernel":
        # template <T, D, kStream, kFilter>: the last two bools are visible in both name forms
        if re.search(r"Lb1ELb1E|true, true", mangled):
            hit += "<stream,candidates>"
        elif re.search(r"Lb1ELb0E|true, false", mangled):
            hit += "<stream>"
    return hit


def _one(pattern: str) -> str:
    found = sorted(glob.glob(pattern, recursive=True))
    if not found:
        raise FileNotFoundError(pattern)
    return found[-1]


def kernel_stats(dirname: str):
    """{(kernel, work-items of the grid): (calls, avg_us, share of the traced time, min_us, max_us)} from the per-dispatch
    trace, so that the launches of the folded call and the 28-times-smaller per-layer launches stay apart."""
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(_one(os.path.join(dirname, "**", "*kernel_trace.csv")))):
        k = short_name(r["Kernel_Name"])
        if k:
            grid = int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"])
            acc[(k, grid)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in acc.values()) or 1.0
    rows = {key: (len(v), sum(v) / len(v), 100.0 * sum(v) / total, min(v), max(v)) for key, v in acc.items()}
    return collections.OrderedDict(sorted(rows.items(), key=lambda kv: -kv[1][0] * kv[1][1]))


def counters(dirname: str):
    """{(kernel, work-items of the grid): {counter: mean per dispatch}} from a --pmc run."""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_one(os.path.join(dirname, "**", "*counter_collection.csv")))):
        k = short_name(r["Kernel_Name"])
        if k:
            acc[(k, int(float(r["Grid_Size"])))][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in acc.items()}


def largest_grid(table, prefix: str):
    """Key of the launch of a kernel with the most work-items: the one of the folded call."""
    keys = [key for key in table if key[0].startswith(prefix)]
    return max(keys, key=lambda key: key[1]) if keys else None


def describe(w) -> str:
    return (f"cfg{w.cfg} ({w.name}: {w.layers} layer(s) x batch {w.batch} folded, {w.n_q_heads}q/{w.n_kv_heads}kv heads, "
            f"D={w.head_dim}, {w.dtype}, {w.n_vis} visual + {w.n_txt} text tokens, k={w.k})")


SQ_COUNTERS = ["SQ_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", "SQ_WAVE_CYCLES", "SQ_ACTIVE_INST_ANY", "SQ_ACTIVE_INST_VALU",
               "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_VALU_MFMA_COEXEC_CYCLES", "SQ_INSTS_VALU", "SQ_INSTS_MFMA",
               "SQ_INSTS_VALU_TRANS_F32", "SQ_INSTS_LDS", "SQ_INSTS_SALU", "SQ_WAIT_ANY", "SQ_WAIT_INST_ANY",
               "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_LDS", "SQ_LDS_IDX_ACTIVE", "SQ_LDS_BANK_CONFLICT"]
SQ_COMMANDS = """Commands (one counter group per run, from /tmp on the GPU box, TMPDIR=/tmp):
  rocprofv3 --pmc SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_ACTIVE_INST_VALU SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_WAIT_INST_LDS SQ_ACTIVE_INST_LDS \\
      -d out -o m --output-format csv -- python3 bench.py --variants --oracle-layers 0 --steps 5 --warmup 1
  rocprofv3 --pmc SQ_WAIT_INST_ANY SQ_WAIT_ANY SQ_ACTIVE_INST_ANY SQ_INSTS_VALU_TRANS_F32 SQ_LDS_BANK_CONFLICT SQ_INSTS_LDS SQ_INSTS_SALU SQ_LDS_IDX_ACTIVE \\
      -d out -o m --output-format csv -- python3 bench.py --variants --oracle-layers 0 --steps 5 --warmup 1
  rocprofv3 --pmc SQ_VALU_MFMA_COEXEC_CYCLES SQ_BUSY_CU_CYCLES \\
      -d out -o m --output-format csv -- python3 bench.py --variants --oracle-layers 0 --steps 5 --warmup 1
Values: mean per dispatch, summed over the chip (256 compute units, 1024 SIMDs).
"""


def _sq_table(C, keys, heads):
    o = ["%-28s" % "counter" + "".join("%26s" % h for h in heads)]
    for c in SQ_COUNTERS:
        o.append("%-28s" % c + "".join("%26.4g" % C[k].get(c, float("nan")) for k in keys))
    return "\n".join(o)


def _sq_reading(d, label):
    """What the counters of one kernel say about the two pipes: SQ_ACTIVE_INST_VALU counts issue slots of 4 cycles
    (1 per ordinary vector or matrix instruction, 2 per exponential); a matrix instruction keeps its pipe busy 16."""
    cu = d["SQ_BUSY_CU_CYCLES"] / 256
    el = d["SQ_INSTS_VALU_TRANS_F32"] / 1024
    mf, va, co = d["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024, d["SQ_ACTIVE_INST_VALU"] * 4 / 1024, d["SQ_VALU_MFMA_COEXEC_CYCLES"] / 1024
    return ("  %s: %.0f k cycles per compute unit; per SIMD the matrix pipe is busy %.0f k cycles (%.0f %%), vector issue %.0f k cycles\n"
            "      (%.0f %%), both at once %.0f k cycles: %.1f cycles per (row, key) element and lane; matrix %.1f + vector %.1f if the two pipes never\n"
            "      overlapped, %.1f if they overlapped fully."
            % (label, cu / 1e3, mf / 1e3, 100 * mf / cu, va / 1e3, 100 * va / cu, co / 1e3, cu / el, mf / el, va / el, max(mf, va) / el))


def variants_main(args):
    D = args.dir
    bj = json.loads([ln for ln in open(os.path.join(D, "vbench.json")) if ln.startswith("{")][-1])
    v = bj["variants"]
    src = bj.get("source_id", "unknown")
    head = f"git {args.head}, " if args.head else ""
    mine = ("mass_", "salience_", "pack_kernel", "scores_filter_kernel")
    st = collections.OrderedDict((k, x) for k, x in kernel_stats(os.path.join(D, "vtrace")).items() if k[0].startswith(mine))
    o = ["Kernel-trace summary of the variants measured beside the decode step (bench.py --variants), long-video workload",
         "(cfg4: 28 layers folded, 28q/4kv heads, D=128, fp16, 50176 visual + 1024 text tokens, k=2509), one MI355X.",
         f"source_id = {src}   ({head}hash of csrc/ and include/ as bench.py prints it)", "",
         "Command (from /tmp on the GPU box, TMPDIR=/tmp):",
         "  rocprofv3 --kernel-trace --stats -d out -o v --output-format csv -- python3 bench.py --variants --oracle-layers 0",
         "(the variants call sv_score_visual_mass with a 32-token question, sv_topk_select on its masses (scores_filter_kernel,",
         " then select_filtered_kernel), sv_pack_selected, sv_sparse_decode_attn gathered / packed / dense and over a keep-ratio",
         " sweep, and sv_salience_self on three encoder-shaped layers -- 256 frames x 729 tokens, one sequence of 16384 tokens and",
         " one of 100000 tokens, 16 heads, head dim padded to 96; rows are per (kernel, grid size in work-items), which keeps the",
         " three salience shapes apart; the attention and scoring kernels are listed in the decode-step summaries.)", "",
         "%-30s %10s %6s %10s %10s %10s" % ("kernel", "work-items", "calls", "avg_us", "min_us", "max_us")]
    for (k, grid), (calls, avg, pct, lo, hi) in st.items():
        o.append("%-30s %10d %6d %10.1f %10.1f %10.1f" % (k, grid, calls, avg, lo, hi))
    o += ["", "bench.py --variants of the same run (medians of event-timed calls, under the tracer): retrieval by attention mass,",
          "32-token question: %.0f us = %.0f TFLOP/s of QK^T on the matrix cores, %.0f G exponentials/s; sv_topk_select on the masses %.1f us;"
          % (v["retrieval_mass_32tok_us"], v["retrieval_mass_TFLOPs"], v["retrieval_mass_Gexp_per_s"], v["select_after_mass_us"]),
          "sv_pack_selected %.1f us; attention gathered %.1f us, packed %.1f us, dense %.1f us.  sv_salience_self:"
          % (v["pack_us"], v["attn_gathered_us"], v["attn_packed_us"], v["attn_dense_us"])]
    for e in v["encoder_salience"]:
        o.append("  %-40s %8.1f us = %.0f TFLOP/s of QK^T, %.0f G exponentials/s, %.3f of the vector-issue bound"
                 % (e["workload"], e["us"], e["QK_TFLOPs"], e["Gexp_per_s"], e["frac_of_vector_issue_peak"]))
    os.makedirs(args.out, exist_ok=True)
    open(os.path.join(args.out, "variants_cfg4_kernel_trace.txt"), "w").write("\n".join(o) + "\n")
    print("\n".join(o))

    C = {}
    for sub in ("vpmc1", "vpmc2", "vpmc3"):
        for key, d in counters(os.path.join(D, sub)).items():
            if "rowstat" in key[0] or "colsum" in key[0]:
                C.setdefault(key, {}).update(d)
    m_row, m_col = largest_grid(C, "mass_rowstat"), largest_grid(C, "mass_colsum")
    o = ["SQ counters of the attention-mass retrieval kernels (sv_score_visual_mass, 32-token question), long-video workload",
         "(cfg4: 28 layers folded, 28q/4kv heads -> 224 query rows per kv head, D=128, fp16, 50176 visual + 1024 text keys), one MI355X.",
         f"source_id = {src}   ({head}hash of csrc/ and include/ as bench.py prints it)", "", SQ_COMMANDS,
         _sq_table(C, [m_row, m_col], ["mass_rowstat_kernel<128>", "mass_colsum_kernel<128>"]), "",
         "Reading (SQ_ACTIVE_INST_VALU counts issue slots of 4 cycles: 1 per ordinary vector or matrix instruction, 2 per",
         "exponential; a matrix instruction keeps the matrix pipe busy for 16 cycles; both kernels at 3 wavefronts per SIMD):",
         _sq_reading(C[m_row], "rowstat"), _sq_reading(C[m_col], "colsum")]
    open(os.path.join(args.out, "mass_retrieval_cfg4_sq_counters.txt"), "w").write("\n".join(o) + "\n")
    print("\n".join(o[-3:]))

    sal = sorted((k for k in C if k[0].startswith("salience")), key=lambda k: (k[1], k[0]))
    # shapes by grid size: A = one sequence of 16384 tokens (3072 workgroups), B = 256 frames of 729 tokens (12288)
    want = {"A": 3072 * 256, "B": 12288 * 256}
    pick = [(tag, kern, next((k for k in sal if k[0] == kern and k[1] == grid), None))
            for tag, grid in want.items() for kern in ("salience_rowstat_kernel", "salience_colsum_kernel")]
    pick = [(tag, kern, k) for tag, kern, k in pick if k is not None]
    o = ["SQ counters of the query-agnostic salience kernels (sv_salience_self) on two of the encoder-shaped layers that",
         "bench.py --variants runs (synthetic q, k; 16 heads, head dim zero-padded to 96, fp16), one MI355X:",
         "  A: one sequence of 16384 tokens (grid of 786432 work-items = 3072 workgroups in both passes)",
         "  B: 256 frames of 729 tokens     (grid of 3145728 work-items = 12288 workgroups)",
         f"source_id = {src}   ({head}hash of csrc/ and include/ as bench.py prints it)", "", SQ_COMMANDS,
         _sq_table(C, [k for _, _, k in pick], ["%s %s<96>" % (tag, kern.split("_")[1]) for tag, kern, _ in pick]), "",
         "Reading (issue slots of 4 cycles: 1 per ordinary vector or matrix instruction, 2 per exponential; at head dim 96 an",
         "element takes three matrix instructions of 16 cycles per 4 elements, 12 cycles per element; 3 wavefronts per SIMD):"]
    o += [_sq_reading(C[k], "%s %s" % (tag, kern.split("_")[1])) for tag, kern, k in pick]
    open(os.path.join(args.out, "salience_encoder_layers_sq_counters.txt"), "w").write("\n".join(o) + "\n")
    print("\n".join(o[-4:]))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--variants", action="store_true", help="summarise the runs of bench.py --variants instead")
    ap.add_argument("--dir", required=True, help="directory holding trace/ fetch/ write/ lds/ cal_f/ cal_w/ and bench.json")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    ap.add_argument("--head", default="", help="git revision of the sources the runs were made with")
    args = ap.parse_args()
    if args.variants:
        return variants_main(args)
    import sv_inputs
    w = sv_inputs.workload(args.config)
    D = args.dir
    bj = json.loads([ln for ln in open(os.path.join(D, "bench.json")) if ln.startswith("{")][-1])
    src = bj.get("source_id", "unknown")
    head = f"git {args.head}, " if args.head else ""
    bench = f"python3 bench.py --config {w.cfg} --oracle-layers 0 --no-other-configs"

    st = kernel_stats(os.path.join(D, "trace"))
    o = [f"Kernel-trace summary of the sparse decode step, {describe(w)}, one MI355X.",
         f"source_id = {src}   ({head}hash of csrc/ and include/ as bench.py prints it)", "",
         "Command (from /tmp on the GPU box, TMPDIR=/tmp):",
         f"  rocprofv3 --kernel-trace --stats -d out -o t --output-format csv -- {bench} --steps 20 --warmup 3",
         "(bench.py runs the warm-up and the timed steps, the same steps again one by one between events, the scoring launch",
         " alone as sv_decode_step issues it, the read-stream probe, about 0.2 s of steps while it reads the clocks, and for",
         " layered workloads the per-layer modes, which launch the same kernels on one layer at a time: rows are therefore",
         " per (kernel, grid size in work-items); the largest grid of a kernel is the launch of the folded call.)", "",
         "%-36s %10s %7s %10s %8s %10s %10s" % ("kernel", "work-items", "calls", "avg_us", "pct", "min_us", "max_us")]
    for (k, grid), (calls, avg, pct, lo, hi) in st.items():
        o.append("%-36s %10d %7d %10.1f %8.2f %10.1f %10.1f" % (k, grid, calls, avg, pct, lo, hi))
    rf = bj["roofline"]
    ks = largest_grid(st, "score_kernel")
    o += ["", "bench.py line of the same run: step %.1f us (%.1f GB/s of algorithmic bytes, %.1f %% of 8 TB/s);"
          % (bj["value"], bj["step_achieved_GBps"], 100 * bj["step_hbm_frac"]),
          "scoring launch alone by HIP events: mean %.1f us over %d B -> %.1f GB/s = %.1f %% of 8 TB/s;"
          % (rf["mean_us"], rf["bytes_per_launch"], rf["achieved"], 100 * rf["frac"])]
    if ks:
        o.append("by the profiler's begin/end stamps of the same launches (%s, %d work-items): avg %.1f us -> %.1f GB/s = %.1f %% of 8 TB/s."
                 % (ks[0], ks[1], st[ks][1], rf["bytes_per_launch"] / st[ks][1] / 1e3, rf["bytes_per_launch"] / st[ks][1] / 1e3 / 80.0))
    o.append("(event-timed figures of a run under the tracer carry its cost per launch, a few microseconds: the step and mode")
    o.append(" times of an untraced run are lower; the begin/end stamps of the kernels above are not affected.)")
    for name, m in bj.get("modes", {}).items():
        o.append("mode %-32s %s" % (name, json.dumps(m)))
    os.makedirs(args.out, exist_ok=True)
    path = os.path.join(args.out, f"decode_step_cfg{w.cfg}_kernel_trace.txt")
    open(path, "w").write("\n".join(o) + "\n")
    print("\n".join(o))

    f, wr, l = counters(os.path.join(D, "fetch")), counters(os.path.join(D, "write")), counters(os.path.join(D, "lds"))
    cal_f = next(v for k, v in counters(os.path.join(D, "cal_f")).items() if k[0] == "copy_kernel")["FETCH_SIZE"]
    cal_w = next(v for k, v in counters(os.path.join(D, "cal_w")).items() if k[0] == "copy_kernel")["WRITE_SIZE"]
    ff, fw = 1048576.0 / cal_f, 1048576.0 / cal_w
    o = [f"HBM traffic and LDS counters per dispatch, {describe(w)}, one MI355X.",
         f"source_id = {src}   ({head}same build as decode_step_cfg{w.cfg}_kernel_trace.txt)", "",
         "Commands (one counter group per run, from /tmp on the GPU box, TMPDIR=/tmp):",
         f"  rocprofv3 --pmc FETCH_SIZE -d out -o f --output-format csv -- {bench} --steps 3 --warmup 1",
         f"  rocprofv3 --pmc WRITE_SIZE -d out -o w --output-format csv -- {bench} --steps 3 --warmup 1",
         f"  rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_INSTS_LDS SQ_ACTIVE_INST_LDS -d out -o l --output-format csv -- {bench} --steps 3 --warmup 1",
         "Calibration (plain copy kernel of the library, 1 GiB = 1048576 KiB read and written per launch):",
         "  rocprofv3 --pmc FETCH_SIZE -d out -o f --output-format csv -- python3 bench.py --copy-calibration   -> FETCH_SIZE %.0f => factor %.3f" % (cal_f, ff),
         "  rocprofv3 --pmc WRITE_SIZE -d out -o w --output-format csv -- python3 bench.py --copy-calibration   -> WRITE_SIZE %.0f => factor %.3f" % (cal_w, fw),
         "Rows are per (kernel, grid size in work-items), means over the dispatches of the run; the largest grid of a kernel",
         "is the launch of the folded call, the smaller ones belong to bench.py's per-layer modes.", "",
         "%-36s %10s %12s %12s %16s %16s" % ("kernel", "work-items", "FETCH_SIZE", "WRITE_SIZE", "fetched_bytes", "written_bytes")]
    for key in sorted(f, key=lambda key: (key[0], -key[1])):
        fs, ws = f[key].get("FETCH_SIZE", float("nan")), wr.get(key, {}).get("WRITE_SIZE", float("nan"))
        o.append("%-36s %10d %12.1f %12.1f %16.0f %16.0f" % (key[0], key[1], fs, ws, fs * 1024 * ff, ws * 1024 * fw))
    kb = rf["bytes_per_launch"]
    ks = largest_grid(f, "score_kernel")
    if ks and ks in wr:
        fb, wb = f[ks]["FETCH_SIZE"] * 1024 * ff, wr[ks]["WRITE_SIZE"] * 1024 * fw
        o += ["", "scoring launch inside sv_decode_step (%d work-items): algorithmic bytes per launch = all visual K = %d B;" % (ks[1], kb),
              "fetched %.0f B (x%.4f), written %.0f B." % (fb, fb / kb, wb), "traffic_bytes_per_launch = %d" % round(fb + wb)]
    ka = largest_grid(f, "attn_partial")
    if ka and ka in wr:
        ab = sv_inputs.algorithmic_bytes(w, *_lens(w, sv_inputs)) - kb
        fb, wb = f[ka]["FETCH_SIZE"] * 1024 * ff, wr[ka]["WRITE_SIZE"] * 1024 * fw
        o.append("attention launch (%d work-items): algorithmic bytes = K,V of text + kept rows = %d B; fetched %.0f B (x%.3f), written %.0f B."
                 % (ka[1], ab, fb, fb / ab, wb))
    o += ["", "LDS counters (sum over the chip, mean per dispatch):",
          "%-36s %10s %14s %14s %18s %16s" % ("kernel", "work-items", "SQ_INSTS_LDS", "LDS_IDX_ACTIVE", "LDS_BANK_CONFLICT", "conflict/active")]
    for key in sorted(l, key=lambda key: (key[0], -key[1])):
        c = l[key]
        a, cf, i = c.get("SQ_LDS_IDX_ACTIVE", 0.0), c.get("SQ_LDS_BANK_CONFLICT", 0.0), c.get("SQ_INSTS_LDS", 0.0)
        o.append("%-36s %10d %14.0f %14.0f %18.0f %16s" % (key[0], key[1], i, a, cf, ("%.3f" % (cf / a)) if a > 0 else "-"))
    path = os.path.join(args.out, f"decode_step_cfg{w.cfg}_traffic_and_lds.txt")
    open(path, "w").write("\n".join(o) + "\n")
    print("\n".join(o))


def _lens(w, sv_inputs):
    """Live lengths of the workload's batch entries (drawn for the ragged workload, the capacities otherwise)."""
    import numpy as np
    if w.structure == "ragged":
        inp = sv_inputs.make_layer(w, 0)
        return inp["vis_len"], inp["txt_len"]
    return np.full(w.B, w.n_vis), np.full(w.B, w.n_txt)


if __name__ == "__main__":
    main()
