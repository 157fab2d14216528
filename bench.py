#!/usr/bin/env python3
"""Benchmark of the sparse decode step (score -> top-k -> sparse attention) on one MI355X.

One "step" is one sv_decode_step over the whole workload: for the long-video config
that is all 28 independent layers folded into the batch dimension (one launch per
stage).  Inputs are synthetic, seeded, and resident in HBM before timing starts.

Prints ONE JSON line and exits 1 if the GPU result does not match the oracle.  Besides the step latency it carries
  other_configs (default run only) the other four workloads of the benchmark set, each with its step latency, its
                fraction of the roofline and a parity report on a bounded sample;
  modes         (layered workloads) beside the folded headline, what the same work costs when every layer is a
                call of its own, as a decoder must issue it: 28 sv_decode_step calls in a row, and the paper's own
                per-token loop -- one sv_sparse_decode_attn per layer on packed (or gathered) kept rows;
  roofline      the scoring kernel as sv_decode_step launches it (it moves ~88 % of the
                step's algorithmic bytes): bytes of visual K per launch / its mean duration
                measured with HIP events on the launch stream, against the 8 TB/s HBM peak;
  cpu_baseline  the CPU oracle (plain C, fp64, OpenMP over independent units) timed on
                a bounded sample of the same inputs on this host's cores;
  parity        index-set rule statistics (boundary tie counts) and output error of the
                GPU result against the oracle on that same sample.
"""
from __future__ import annotations

import argparse
import json
import os
import glob
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def measured_traffic(cfg: int):
    """HBM bytes per launch of the scoring kernel (FETCH_SIZE + WRITE_SIZE, calibrated against a plain copy).
    NOT measured by the run that prints it: hardware counters need runs of their own under rocprofv3 --pmc, so the
    figure is read from the committed summary of those runs, and the line names that file and the sources it was
    taken at.  Returns (bytes or None, source description or None)."""
    path = os.path.join(ROOT, "profiles", f"decode_step_cfg{cfg}_traffic_and_lds.txt")
    if not os.path.exists(path):
        return None, None
    val, src = None, ""
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            val = int(line.split("=")[1])
        if line.startswith("source_id"):
            src = line.split("=")[1].strip()
    rel = os.path.relpath(path, ROOT)
    return val, f"{rel} (rocprofv3 --pmc runs of this command, sources {src or 'unknown'}; not measured in this run)"


MFMA_FP16_PEAK_TFLOPS = 2500.0     # dense fp16 matrix-core peak of the device


def read_clocks_MHz():
    """Current shader and memory clock levels from sysfs (best effort; None where unreadable).  Read while work is
    queued on the device: starting another program from a process that holds the GPU is not an option."""
    clocks = {}
    try:
        for name in ("sclk", "mclk"):
            for path in sorted(glob.glob(f"/sys/class/drm/card*/device/pp_dpm_{name}")):
                cur = [ln for ln in open(path).read().splitlines() if ln.rstrip().endswith("*")]
                if cur:
                    clocks[f"{name}_MHz"] = int("".join(ch for ch in cur[0].split(":")[1] if ch.isdigit()))
                    break
    except Exception:   # noqa: BLE001 - files may be missing or unreadable
        return None
    return clocks or None


def sclk_under(torch, fn, seconds=0.15):
    """Shader clock (MHz) read while calls of fn are queued for about `seconds`; None if unreadable."""
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fn()
    torch.cuda.synchronize()
    one = max(time.perf_counter() - t0, 1e-6)
    for _ in range(max(2, int(seconds / one))):
        fn()
    c = read_clocks_MHz()
    torch.cuda.synchronize()
    return None if not c else c.get("sclk_MHz")


def issue_bound_fractions(rate_element_passes, sclk_MHz):
    """An (query, key, head) element-pass of the attention-mass kernels is a matrix instruction, a multiply-add, an
    exponential (two slots) and an add: five 4-cycle issue slots for 64 lanes per SIMD.  Fraction of that bound at the
    nominal 2.4 GHz and at the clock the device held under this very load."""
    out = {"frac_of_vector_issue_peak": round(rate_element_passes / VALU_ISSUE_PEAK_ELEMENT_PASSES, 3)}
    if sclk_MHz:
        out["sclk_MHz_under_this_load"] = sclk_MHz
        out["frac_of_vector_issue_bound_at_that_clock"] = round(
            rate_element_passes / (VALU_ISSUE_PEAK_ELEMENT_PASSES * sclk_MHz / 2400.0), 3)
    return out


def time_variants(sv, torch, w, d, shape, buf, reps):
    """Event-timed variants around the step (all on the workload's own tensors, idx/count as the step left them):
    gathered attention per decoded token, packing + attention on the packed rows (the paper's once-per-round
    retrieval, section 3.2), dense attention over the whole cache (the baseline of the paper's kernel-level
    comparison, section 4.5), and the whole step for a sweep of keep ratios."""
    dev = d["q"].device
    stream = torch.cuda.current_stream()

    def timed(fn):
        for _ in range(3):
            fn()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record(stream)
            fn()
            b.record(stream)
        torch.cuda.synchronize()
        return round(float(np.median([a.elapsed_time(b) * 1e3 for a, b in evs])), 2)

    out = {}
    out["attn_gathered_us"] = timed(lambda: sv.sv_sparse_decode_attn(
        shape, d["q"], d["k_vis"], d["v_vis"], d["k_txt"], d["v_txt"], buf.idx, buf.count, buf.out, buf.lse,
        buf.workspace))
    B, Hkv, D, k = shape.batch, shape.n_kv_heads, shape.head_dim, shape.k
    k_pack = torch.empty((B, Hkv, k, D), dtype=d["k_vis"].dtype, device=dev)
    v_pack = torch.empty_like(k_pack)
    out["pack_us"] = timed(lambda: sv.sv_pack_selected(shape, d["k_vis"], d["v_vis"], buf.idx, buf.count,
                                                       k_pack, v_pack))
    pshape = sv.make_shape(d["q"], k_pack, d["k_txt"], k, txt_len=shape.txt_len)
    pbuf = sv.DecodeBuffers(pshape, dev, with_scores=False)
    out["attn_packed_us"] = timed(lambda: sv.sv_sparse_decode_attn(
        pshape, d["q"], k_pack, v_pack, d["k_txt"], d["v_txt"], None, buf.count, pbuf.out, pbuf.lse, pbuf.workspace))
    out["packed_equals_gathered_max_abs"] = float((pbuf.out - buf.out).abs().max())
    if d["q"].dtype == torch.float16 and shape.n_txt_max >= 32:
        # once-per-round retrieval with a 32-token question (attention mass), then the unchanged selection
        Tq = 32
        g = torch.Generator(device=dev)
        g.manual_seed(20251017)
        qm = torch.randn((B, Tq, shape.n_q_heads, D), device=dev, dtype=torch.float32, generator=g).to(torch.float16)
        mscores = torch.empty((B, Hkv, shape.n_vis_max), dtype=torch.float32, device=dev)
        mshape = sv.make_shape(qm[:, 0], d["k_vis"], d["k_txt"], k, vis_len=shape.vis_len, txt_len=shape.txt_len)
        mws = sv.sv_score_visual_mass(mshape, qm, d["k_vis"], d["k_txt"], mscores)
        out["retrieval_mass_32tok_us"] = timed(lambda: sv.sv_score_visual_mass(mshape, qm, d["k_vis"], d["k_txt"],
                                                                               mscores, None, mws))
        rows = Tq * (shape.n_q_heads // Hkv)
        keys = int(shape.n_vis_max if shape.vis_len is None else shape.vis_len.sum().item() / B)
        flop = 2.0 * 2 * B * Hkv * rows * (keys + shape.n_txt_max) * D      # two passes of QK^T
        out["retrieval_mass_TFLOPs"] = round(flop / (out["retrieval_mass_32tok_us"] * 1e-6) / 1e12, 1)
        out["retrieval_mass_frac_of_fp16_mfma_peak"] = round(out["retrieval_mass_TFLOPs"] / MFMA_FP16_PEAK_TFLOPS, 3)
        rate = 2.0 * B * Hkv * rows * keys / (out["retrieval_mass_32tok_us"] * 1e-6)
        out["retrieval_mass_Gexp_per_s"] = round(rate / 1e9, 1)
        out["retrieval_mass_bounds"] = issue_bound_fractions(
            rate, sclk_under(torch, lambda: sv.sv_score_visual_mass(mshape, qm, d["k_vis"], d["k_txt"], mscores, None, mws)))
        out["select_after_mass_us"] = timed(lambda: sv.sv_topk_select(shape, mscores, buf.idx, buf.count, buf.workspace))
        # leave idx/count as the step produced them for whatever follows
        sv.sv_decode_step(shape, d["q"], d["k_vis"], d["v_vis"], d["k_txt"], d["v_txt"], None, buf.idx, buf.count,
                          buf.out, buf.lse, buf.workspace)
        torch.cuda.synchronize()
        del qm, mscores, mws
    if shape.vis_len is None:   # dense baseline and sweep: uniform visual length only
        Nv = shape.n_vis_max
        dshape = sv.make_shape(d["q"], d["k_vis"], d["k_txt"], Nv, txt_len=shape.txt_len)
        dbuf = sv.DecodeBuffers(dshape, dev, with_scores=False)
        dbuf.count.fill_(Nv)
        out["attn_dense_us"] = timed(lambda: sv.sv_sparse_decode_attn(
            dshape, d["q"], d["k_vis"], d["v_vis"], d["k_txt"], d["v_txt"], None, dbuf.count, dbuf.out, dbuf.lse,
            dbuf.workspace))
        del dbuf
        sweep = []
        for keep in (0.5, 0.25, 0.10, 0.05, 0.02):
            kk = max(1, int(round(Nv * keep)))
            s2 = sv.make_shape(d["q"], d["k_vis"], d["k_txt"], kk, txt_len=shape.txt_len)
            b2 = sv.DecodeBuffers(s2, dev, with_scores=False)
            step_us = timed(lambda: sv.sv_decode_step(s2, d["q"], d["k_vis"], d["v_vis"], d["k_txt"], d["v_txt"],
                                                      None, b2.idx, b2.count, b2.out, b2.lse, b2.workspace))
            attn_us = timed(lambda: sv.sv_sparse_decode_attn(s2, d["q"], d["k_vis"], d["v_vis"], d["k_txt"],
                                                             d["v_txt"], b2.idx, b2.count, b2.out, b2.lse,
                                                             b2.workspace))
            sweep.append({"keep": keep, "k": kk, "step_us": step_us, "attn_us": attn_us,
                          "dense_attn_over_sparse_attn": round(out["attn_dense_us"] / attn_us, 2)})
            del b2
        out["sweep"] = sweep
    return out


# Vector-issue bound of the two attention-mass computations: per (query, key, head) element and pass a wavefront issues a
# matrix instruction, a multiply-add, an exponential (two slots) and an add -- five 4-cycle issue slots for 64 lanes --
# on each of the 4 SIMDs of the 256 compute units at 2.4 GHz.
VALU_ISSUE_PEAK_ELEMENT_PASSES = 256 * 4 * 64 / (5 * 4) * 2.4e9


def time_encoder_salience(sv, torch, reps):
    """Query-agnostic salience of a vision-encoder layer (paper section 3.1; figure on the salience kernels, panel a):
    synthetic q, k ~ N(0, 1) in the shapes of the two encoder families the paper names, head dims zero-padded to 96."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(20251017)
    out = []
    for name, B, N, H, d_head in (("siglip_256_frames_x_729_tokens", 256, 729, 16, 72),
                                  ("qwenvl_one_sequence_of_16384_tokens", 1, 16384, 16, 80),
                                  ("qwenvl_one_sequence_of_100000_tokens", 1, 100000, 16, 80)):
        reps = reps if N < 50000 else min(reps, 3)    # 64 ms a call
        D = 96
        q = torch.zeros((B, N, H, D), dtype=torch.float16, device=dev)
        k = torch.zeros((B, H, N, D), dtype=torch.float16, device=dev)
        q[..., :d_head] = torch.randn((B, N, H, d_head), device=dev, dtype=torch.float32, generator=g).to(torch.float16)
        k[..., :d_head] = torch.randn((B, H, N, d_head), device=dev, dtype=torch.float32, generator=g).to(torch.float16)
        shape = sv.make_encoder_shape(q, k, scale=float(d_head) ** -0.5)
        sal = torch.empty((B, N), dtype=torch.float32, device=dev)
        ws = sv.sv_salience_self(shape, q, k, sal)
        for _ in range(2):
            sv.sv_salience_self(shape, q, k, sal, None, ws)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        stream = torch.cuda.current_stream()
        for a, b in evs:
            a.record(stream)
            sv.sv_salience_self(shape, q, k, sal, None, ws)
            b.record(stream)
        torch.cuda.synchronize()
        us = float(np.median([a.elapsed_time(b) * 1e3 for a, b in evs]))
        elements = float(B) * H * N * N
        rate = 2.0 * elements / (us * 1e-6)          # element-passes per second (two passes)
        tflops = 2 * 2 * elements * D / (us * 1e-6) / 1e12
        sclk = sclk_under(torch, lambda: sv.sv_salience_self(shape, q, k, sal, None, ws)) if N < 50000 else None
        out.append({"workload": name, "tokens": N, "batch": B, "heads": H, "head_dim": d_head, "padded_head_dim": D,
                    "us": round(us, 1), "QK_TFLOPs": round(tflops, 1),
                    "frac_of_fp16_mfma_peak": round(tflops / MFMA_FP16_PEAK_TFLOPS, 3),
                    "Gexp_per_s": round(rate / 1e9, 1), **issue_bound_fractions(rate, sclk),
                    "salience_sums_to_one_max_dev": float((sal.double().sum(dim=1) - 1.0).abs().max()),
                    "workspace_MB": round(ws.numel() / 1e6, 1)})
        del q, k, sal, ws
    return out


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload id (4 = long video, the graded one)")
    ap.add_argument("--seed", type=int, default=0, help="offset added to every input seed (another draw of the same workload)")
    ap.add_argument("--copies", type=int, default=0,
                    help="independent copies of the inputs the steps rotate over; 0 = 8 when the whole KV cache would "
                         "otherwise sit in the 256 MB last-level cache (configs 1, 2, 5), else 1")
    ap.add_argument("--oracle-layers", type=int, default=28,
                    help="how many leading layers the CPU oracle is timed and compared on (0 = skip)")
    ap.add_argument("--gen-workers", type=int, default=min(16, len(os.sched_getaffinity(0))))
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only launch the library's plain 1 GiB copy kernel 5 times (run under rocprofv3 --pmc "
                         "to learn what FETCH_SIZE / WRITE_SIZE report for a known size)")
    ap.add_argument("--keep-scores", action="store_true",
                    help="hand sv_decode_step a scores buffer (it then also stores all 22 MB of scores per step)")
    ap.add_argument("--variants", action="store_true",
                    help="also time, on the same inputs, the paper's retrieve-once use (pack the kept rows, then "
                         "attention on the packed buffers), the dense baseline and a sweep of keep ratios, and the "
                         "query-agnostic salience of two encoder-shaped layers; adds a \"variants\" object to the JSON line")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="config 4 only: skip the short measurement of the other four workloads (\"other_configs\")")
    ap.add_argument("--set", action="append", default=[], metavar="KNOB=VALUE",
                    help="launch-shape knob for sweeps, e.g. --set attn_batches=4")
    return ap.parse_args()


LLC_BYTES = 256 << 20     # last-level cache of the device


def source_id() -> str:
    """Hash of the kernel and C-ABI sources the loaded library was built from (names the build in the JSON line
    and in the profile summaries, where a git revision is not available on the GPU machine)."""
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2510_17777_amd", "csrc", "*")) +
                       [os.path.join(ROOT, "include", "sparsevila.h")]):
        h.update(open(path, "rb").read())
    return h.hexdigest()[:12]


class Problem:
    """One resident copy of the workload's tensors with its own output buffers."""

    def __init__(self, sv, torch, sv_inputs, w, dev, workers, keep_scores):
        t0 = time.time()
        self.w = w
        self.inp = sv_inputs.make_inputs(w, workers=workers)
        self.gen_s = time.time() - t0
        self.d = {n: torch.from_numpy(self.inp[n]).to(dev) for n in ("q", "k_vis", "v_vis", "k_txt", "v_txt")}
        self.ragged = w.structure == "ragged"
        self.vis_len = self.inp["vis_len"] if self.ragged else None
        self.txt_len = self.inp["txt_len"] if self.ragged else None
        self.shape = sv.make_shape(self.d["q"], self.d["k_vis"], self.d["k_txt"], w.k, vis_len=self.vis_len,
                                   txt_len=self.txt_len)
        self.buf = sv.DecodeBuffers(self.shape, dev, with_scores=keep_scores)
        self.queries = [self.d["q"]]
        for rnd in range(1, w.rounds):
            self.queries.append(torch.from_numpy(sv_inputs.round_query(w, rnd)).to(dev))
        self.sv = sv

    def step(self, rnd: int = 0):
        d, b = self.d, self.buf
        self.sv.sv_decode_step(self.shape, self.queries[rnd % len(self.queries)], d["k_vis"], d["v_vis"], d["k_txt"],
                               d["v_txt"], b.scores, b.idx, b.count, b.out, b.lse, b.workspace)


def event_times_us(torch, fn, reps, warm=3):
    """fn(i) called reps times, each call between two events on the current stream; microseconds per call."""
    stream = torch.cuda.current_stream()
    for i in range(warm):
        fn(i)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for i, (a, b) in enumerate(evs):
        a.record(stream)
        fn(i)
        b.record(stream)
    torch.cuda.synchronize()
    return np.array([a.elapsed_time(b) * 1e3 for a, b in evs])


def graph_replay_times_us(torch, fn, reps, warm=3):
    """fn(0) captured once into a HIP graph (the library only launches kernels: nothing allocates or synchronises),
    then reps replays, each between two events: what the same launches cost without the host's per-call work."""
    fn(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn(0)
    torch.cuda.synchronize()
    return event_times_us(torch, lambda _i: graph.replay(), reps, warm=warm)


def per_layer_modes(sv, torch, pr, reps):
    """The step as a decoder issues it: its layers depend on each other, so every layer is a call of its own.
    Each mode is timed twice: the calls issued from Python one by one (the host's per-call work, tens of microseconds
    through ctypes, can exceed what two short kernels take), and the same calls replayed from a HIP graph, which is
    what a native caller's launch rate looks like; the graph figure is the one reported as `us`.
    (a) 28 sv_decode_step calls, one after the other (retrieval at every step);
    (b) the paper's own decode loop, section 3.2 / 4.1: retrieval and packing once per round, then per decoded token
        and per layer one sv_sparse_decode_attn over the text rows and the packed kept rows (here: one token = the
        28 per-layer calls in a row), and the same with the rows gathered through idx instead of packed."""
    w, d, dev = pr.w, pr.d, pr.d["q"].device
    L, per = w.layers, pr.shape.batch // w.layers
    k, Hkv, D = w.k, w.n_kv_heads, w.head_dim
    es = w.elem_size
    layer_algo = sv_inputs_algorithmic_bytes(pr) // L
    attn_bytes_layer = per * Hkv * D * es * 2 * (min(k, w.n_vis) + w.n_txt)
    out = {}
    sls = [slice(l * per, (l + 1) * per) for l in range(L)]
    lshapes = [sv.make_shape(d["q"][sl], d["k_vis"][sl], d["k_txt"][sl], k) for sl in sls]
    # outputs of layer l go to slice l of a second set of buffers, so the two modes can be compared
    b2 = sv.DecodeBuffers(pr.shape, dev, with_scores=False)
    lws = torch.empty((sv.workspace_bytes(lshapes[0]),), dtype=torch.uint8, device=dev)

    def sequential(_i):
        for ls, sl in zip(lshapes, sls):
            sv.sv_decode_step(ls, d["q"][sl], d["k_vis"][sl], d["v_vis"][sl], d["k_txt"][sl], d["v_txt"][sl], None,
                              b2.idx[sl], b2.count[sl], b2.out[sl], b2.lse[sl], lws)
    t = event_times_us(torch, sequential, reps)
    us_eager = float(np.median(t))
    us = float(np.median(graph_replay_times_us(torch, sequential, reps)))
    out["sequential_per_layer_calls"] = {
        "calls": L, "us": round(us, 1), "us_per_layer": round(us / L, 2), "timed": "replay of a HIP graph of the calls",
        "us_eager_python_calls": round(us_eager, 1),
        "achieved_GBps": round(L * layer_algo / (us * 1e-6) / 1e9, 1),
        "hbm_frac": round(L * layer_algo / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "idx_equal_to_folded": bool(torch.equal(b2.idx, pr.buf.idx) and torch.equal(b2.count, pr.buf.count)),
        "out_max_abs_diff_to_folded": float((b2.out - pr.buf.out).abs().max())}

    k_pack = torch.empty((pr.shape.batch, Hkv, k, D), dtype=d["k_vis"].dtype, device=dev)
    v_pack = torch.empty_like(k_pack)
    sv.sv_pack_selected(pr.shape, d["k_vis"], d["v_vis"], pr.buf.idx, pr.buf.count, k_pack, v_pack)
    pshapes = [sv.make_shape(d["q"][sl], k_pack[sl], d["k_txt"][sl], k) for sl in sls]
    pws = torch.empty((sv.workspace_bytes(pshapes[0]),), dtype=torch.uint8, device=dev)

    def token_packed(_i):
        for ps, sl in zip(pshapes, sls):
            sv.sv_sparse_decode_attn(ps, d["q"][sl], k_pack[sl], v_pack[sl], d["k_txt"][sl], d["v_txt"][sl], None,
                                     pr.buf.count[sl], b2.out[sl], b2.lse[sl], pws)

    def token_gathered(_i):
        for ls, sl in zip(lshapes, sls):
            sv.sv_sparse_decode_attn(ls, d["q"][sl], d["k_vis"][sl], d["v_vis"][sl], d["k_txt"][sl], d["v_txt"][sl],
                                     pr.buf.idx[sl], pr.buf.count[sl], b2.out[sl], b2.lse[sl], lws)
    for name, fn in (("per_layer_attention_packed", token_packed), ("per_layer_attention_gathered", token_gathered)):
        us_eager = float(np.median(event_times_us(torch, fn, reps)))
        us = float(np.median(graph_replay_times_us(torch, fn, reps)))
        out[name] = {"calls": L, "us_per_token_all_layers": round(us, 1), "us_per_layer": round(us / L, 2),
                     "timed": "replay of a HIP graph of the calls", "us_eager_python_calls": round(us_eager, 1),
                     "bytes_per_layer": attn_bytes_layer,
                     "achieved_GBps": round(L * attn_bytes_layer / (us * 1e-6) / 1e9, 1),
                     "hbm_frac": round(L * attn_bytes_layer / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                     "out_max_abs_diff_to_folded": float((b2.out - pr.buf.out).abs().max())}
    return out


def sv_inputs_algorithmic_bytes(pr) -> int:
    import sv_inputs
    return sv_inputs.algorithmic_bytes(pr.w, pr.inp["vis_len"], pr.inp["txt_len"])


def measure_other_config(sv, torch, sv_inputs, args, cfg):
    """One of the other workloads of the benchmark set, measured the same way as the headline but without the
    per-kernel legs: W warm-up steps, K timed steps between two synchronisations, the same steps between events,
    and the parity report against the oracle on a bounded sample (at most four layers of a layered workload)."""
    dev = "cuda:0"
    w = sv_inputs.workload(cfg, seed_offset=args.seed)
    copies = 8 if sv_inputs.cache_bytes(w) <= 2 * LLC_BYTES else 1
    problems = [Problem(sv, torch, sv_inputs, sv_inputs.workload(cfg, seed_offset=args.seed + 7919 * c), dev,
                        args.gen_workers, False) for c in range(copies)]
    rounds = max(1, w.rounds)

    def step(i: int):
        problems[i % copies].step((i // copies) % rounds)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / args.steps * 1e6
    ev = event_times_us(torch, step, args.steps, warm=0)
    algo = float(np.mean([sv_inputs_algorithmic_bytes(p) for p in problems]))
    pr = problems[0]
    pr.step(0)
    torch.cuda.synchronize()
    out = {"workload": f"cfg{w.cfg}_{w.name}", "dtype": w.dtype, "value": round(us, 2), "unit": "us",
           "step_event_us_median": round(float(np.median(ev)), 2), "step_algorithmic_bytes": int(algo),
           "step_hbm_frac": round(algo / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4), "rotating_copies": copies,
           "working_set_cache_resident": bool(copies * sv_inputs.cache_bytes(w) <= LLC_BYTES)}
    if args.oracle_layers > 0:
        import oracle
        from oracle.compare import check_index_sets, out_tolerance
        nb = min(min(args.oracle_layers, 4) * w.batch, w.B)
        inp = pr.inp
        sub = {n: inp[n][:nb] for n in ("q", "k_vis", "v_vis", "k_txt", "v_txt")}
        vl = inp["vis_len"][:nb] if pr.ragged else None
        tl = inp["txt_len"][:nb] if pr.ragged else None
        ref = oracle.decode_step(sub["q"], sub["k_vis"], sub["v_vis"], sub["k_txt"], sub["v_txt"], w.k, vis_len=vl, txt_len=tl)
        idx, cnt = pr.buf.idx[:nb].cpu().numpy(), pr.buf.count[:nb].cpu().numpy()
        rep = check_index_sets(ref["scores"], w.k, vl, idx, cnt)
        ref_out, _, _ = oracle.sparse_decode_attn(sub["q"], sub["k_vis"], sub["v_vis"], sub["k_txt"], sub["v_txt"], idx, cnt,
                                                  txt_len=tl)
        err = float(np.abs(pr.buf.out[:nb].cpu().numpy() - ref_out).max())
        out["parity"] = dict(problems=rep.problems, equal_sets=rep.equal_sets, boundary_ties_total=rep.summary()["boundary_ties_total"],
                             failures=len(rep.failures), out_max_abs_err=err, out_tol=out_tolerance(w.np_dtype),
                             ok=bool(rep.ok and err <= out_tolerance(w.np_dtype)))
    del problems
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2510_17777_amd as sv
    import sv_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    sv.load_library()
    for item in args.set:
        name, val = item.split("=")
        sv.sv_set_tuning(name, int(val))

    if args.copy_calibration:
        n = 1 << 30
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            sv.sv_copy_bytes(dst, src, n)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n, "launches": 5}))
        return

    dev = "cuda:0"
    w = sv_inputs.workload(args.config, seed_offset=args.seed)
    # A cache that fits the last-level cache would be served from it on every step after the first: such
    # workloads rotate over independent copies (other seeds), so that every step reads its rows from HBM.
    copies = args.copies if args.copies > 0 else (8 if sv_inputs.cache_bytes(w) <= 2 * LLC_BYTES else 1)
    problems = [Problem(sv, torch, sv_inputs, sv_inputs.workload(args.config, seed_offset=args.seed + 7919 * c), dev,
                        args.gen_workers, args.keep_scores) for c in range(copies)]
    pr = problems[0]
    inp, d, shape, buf = pr.inp, pr.d, pr.shape, pr.buf
    t_gen = sum(p.gen_s for p in problems)
    rounds = max(1, w.rounds)

    def step(i: int):
        problems[i % copies].step((i // copies) % rounds)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    us_per_step = wall / args.steps * 1e6

    # Spread of single steps: the same steps again, each between two events on the launch stream.
    stream = torch.cuda.current_stream()
    step_ev_us = event_times_us(torch, step, args.steps, warm=0)

    # The dominant kernel alone: the scoring launch exactly as the step issues it.  The test build of the library
    # (the same kernel objects; its C-ABI layer knows the "step_stages" knob, the product's does not) makes
    # sv_decode_step return after that launch; it is bracketed by events on the stream it is launched on.
    with sv.test_hooks():
        for item in args.set:
            name, val = item.split("=")
            sv.sv_set_tuning(name, int(val))
        sv.sv_set_tuning("step_stages", 1)
        score_us = event_times_us(torch, step, args.steps, warm=2)

    # What a plain read stream reaches on this device: the same visual-K bytes read once by a kernel
    # that does nothing else (context for the roofline fraction; the peak stays the published 8 TB/s).
    sink = torch.zeros(sv.READ_SINK_BYTES // 4, dtype=torch.int32, device=dev)
    flats = [p.d["k_vis"].reshape(-1) for p in problems]
    probe_bytes = flats[0].numel() * flats[0].element_size() // 16 * 16
    probe_us = event_times_us(torch, lambda i: sv.sv_read_bytes(flats[i % copies], probe_bytes, sink), 10, warm=2)
    probe_gbps = probe_bytes / (float(probe_us.mean()) * 1e-6) / 1e9

    # Clocks while the device is busy with steps (best effort; the box decides power state and clocks).
    # Read from sysfs: starting another program from a process that holds the GPU is not an option.
    for i in range(max(200, int(0.2 / (us_per_step * 1e-6)))):
        step(i)
    clocks = read_clocks_MHz()
    torch.cuda.synchronize()

    # Leave the buffers of copy 0 holding the result of a step with query 0 for the parity report.
    pr.step(0)
    torch.cuda.synchronize()

    algo_bytes = float(np.mean([sv_inputs_algorithmic_bytes(p) for p in problems]))
    k_bytes = float(np.mean([w.n_kv_heads * w.head_dim * w.elem_size * p.inp["vis_len"].astype(np.int64).sum()
                             for p in problems]))
    step_gbps = algo_bytes / (us_per_step * 1e-6) / 1e9
    score_gbps = k_bytes / (float(score_us.mean()) * 1e-6) / 1e9
    traffic, traffic_src = measured_traffic(w.cfg)

    result = {
        "metric": "sparse_decode_step_latency", "value": round(us_per_step, 2), "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us_per_step / 1e3, 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"cfg{w.cfg}_{w.name}", "batch": w.batch, "layers_folded": w.layers,
                   "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "n_visual": w.n_vis, "n_text": w.n_txt, "k": w.k, "mode": "folded_layers_one_call",
                   "seed_offset": args.seed,
                   "score_rows_per_block": sv.sv_get_tuning("score_rows_per_block"),
                   "attn_batches": sv.sv_get_tuning("attn_batches") or "planned per call"},
        "source_id": source_id(),
        "kv_cache_bytes": sv_inputs.cache_bytes(w),
        "rotating_copies": copies,
        "working_set_cache_resident": bool(copies * sv_inputs.cache_bytes(w) <= LLC_BYTES),
        "step_algorithmic_bytes": int(algo_bytes),
        "step_achieved_GBps": round(step_gbps, 1),
        "step_hbm_frac": round(step_gbps / HBM_PEAK_GBPS, 4),
        "step_event_us": {"median": round(float(np.median(step_ev_us)), 2),
                          "p10": round(float(np.percentile(step_ev_us, 10)), 2),
                          "p90": round(float(np.percentile(step_ev_us, 90)), 2)},
        "roofline": {"bound": "hbm", "kernel": "score_kernel", "achieved": round(score_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(score_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "bytes_per_launch": int(k_bytes),
                     "mean_us": round(float(score_us.mean()), 2), "median_us": round(float(np.median(score_us)), 2),
                     "read_stream_probe_GBps": round(probe_gbps, 1),
                     "frac_of_read_stream_probe": round(score_gbps / probe_gbps, 4)},
        "clocks_under_load": clocks,
        "input_gen_s": round(t_gen, 1),
    }

    if w.layers > 1 and not pr.ragged:
        # side by side with the folded headline: what the same work costs when every layer is a call of its own
        result["modes"] = {"folded_layers_one_call": {"calls": 1, "us": round(float(np.median(step_ev_us)), 1),
                                                      "hbm_frac": round(algo_bytes / (float(np.median(step_ev_us)) * 1e-6) / 1e9
                                                                        / HBM_PEAK_GBPS, 4)}}
        result["modes"].update(per_layer_modes(sv, torch, pr, min(args.steps, 20)))
        pr.step(0)
        torch.cuda.synchronize()

    if args.variants:
        result["variants"] = time_variants(sv, torch, w, d, shape, buf, args.steps)
        result["variants"]["encoder_salience"] = time_encoder_salience(sv, torch, min(args.steps, 10))

    if args.oracle_layers > 0:
        import oracle
        from oracle.compare import check_index_sets, out_tolerance
        ragged = pr.ragged
        nb = min(args.oracle_layers * w.batch, w.B)
        sub = {n: inp[n][:nb] for n in ("q", "k_vis", "v_vis", "k_txt", "v_txt")}
        vl = inp["vis_len"][:nb] if ragged else None
        tl = inp["txt_len"][:nb] if ragged else None
        cores = len(os.sched_getaffinity(0))
        os.environ.setdefault("OMP_NUM_THREADS", str(cores))
        t0 = time.perf_counter()
        ref = oracle.decode_step(sub["q"], sub["k_vis"], sub["v_vis"], sub["k_txt"], sub["v_txt"], w.k,
                                 vis_len=vl, txt_len=tl)
        t_oracle = time.perf_counter() - t0
        threads = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
        result["cpu_baseline"] = {
            "value": round(t_oracle / nb * w.B * 1e6, 1), "unit": "us", "cores": threads, "kind": "oracle",
            "sample": f"first {nb} of {w.B} batch entries (layers) of the same inputs, one oracle step "
                      f"took {t_oracle:.2f} s; value = that time scaled by {w.B}/{nb}"}
        idx, cnt = buf.idx[:nb].cpu().numpy(), buf.count[:nb].cpu().numpy()
        rep = check_index_sets(ref["scores"], w.k, vl, idx, cnt)
        ref_out, _, _ = oracle.sparse_decode_attn(sub["q"], sub["k_vis"], sub["v_vis"], sub["k_txt"],
                                                  sub["v_txt"], idx, cnt, txt_len=tl)
        err = float(np.abs(buf.out[:nb].cpu().numpy() - ref_out).max())
        result["parity"] = dict(rep.summary(), out_max_abs_err=err, out_tol=out_tolerance(w.np_dtype),
                                ok=bool(rep.ok and err <= out_tolerance(w.np_dtype)))

    if args.config == 4 and not args.no_other_configs:
        # the other four workloads of the benchmark set, in the same line (the graded one stays the headline)
        del problems, pr, d, shape, buf, flats
        torch.cuda.empty_cache()
        result["other_configs"] = [measure_other_config(sv, torch, sv_inputs, args, c) for c in (1, 2, 3, 5)]

    print(json.dumps(result))
    bad = [o["workload"] for o in result.get("other_configs", []) if "parity" in o and not o["parity"]["ok"]]
    if bad:
        print(f"bench.py: the GPU result does not match the oracle on {bad}", file=sys.stderr)
        sys.exit(1)
    if "parity" in result and not result["parity"]["ok"]:
        print("bench.py: the GPU result does not match the oracle (see \"parity\")", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
