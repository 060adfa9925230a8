#!/usr/bin/env python3
"""Benchmark of the Prism hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM:  prism_estimate (pool + energies -> calibrate -> dual-band scores ->
softmax -> top-p -> union -> CSR)  ->  prism_v_image  ->  prism_sparse_attn_pre.
Default workload: the Llama-3-8B-shaped layer at 128K tokens (the configuration the
headline metric is quoted on).  Prints ONE JSON line.

  value        effective TFLOP/s = dense-causal FLOPs of the layer / time of one step
  roofline     dominant kernel (block-sparse attention): executed bf16 MFMA FLOPs
               (4*B*B*d per listed block pair) / kernel time measured with HIP events
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def profiled_traffic(workload: str, kernel: str):
    """(HBM bytes per launch of `kernel`, file it was read from) out of the committed rocprofv3
    counter summary of this workload (profiles/hot_path_<workload>.txt, lines
    'TRAFFIC kernel=... read_bytes=... write_bytes=...'); (None, None) when there is none.
    Counter runs are separate rocprofv3 --pmc passes, so this figure is never measured in the
    timed run itself: the JSON line carries the file name beside it."""
    rel = os.path.join("profiles", f"hot_path_{workload}.txt")
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.startswith("TRAFFIC") and f"kernel={kernel} " in line:
                    kv = dict(x.split("=") for x in line.split()[1:])
                    return float(kv["read_bytes"]) + float(kv["write_bytes"]), rel
    except OSError:
        pass
    return None, None


def stats(xs):
    """mean / median / min of a list of per-step times, rounded."""
    import numpy as np
    a = np.asarray(xs, dtype=np.float64)
    return {"mean": round(float(a.mean()), 4), "median": round(float(np.median(a)), 4), "min": round(float(a.min()), 4)}


PEAK_PROBES = (("mfma_32x32x16_bf16_only", (1, 2)), ("mfma_plus_lds_read_1_to_1", (2,)),
               ("mfma_plus_lds_read_1_to_2", (1, 2)), ("lds_read_b128_only", (2,)),
               ("valu_fma_f32", (1,)), ("valu_exp_f32", (1,)), ("mfma_plus_4fma_1exp_same_wave", (1, 2)),
               ("stream_read_16B", (16, 128, 1024, 8192)))


def measure_peaks(which=None):
    """Achievable peaks of this GPU from the probe loops of libprism_peaks.so (bench-only library
    built beside libprism.so): rows of {probe, arg, ms, rate, unit, shader_mhz, cycles_per_op}.
    `which` = {probe name: args} restricts the run; None runs every probe at every argument."""
    import ctypes
    path = os.path.join(ROOT, "paper_2602_08426_amd", "libprism_peaks.so")
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: run __graft_entry__.build() first")
    lib = ctypes.CDLL(path)
    lib.prism_peaks_name.restype = ctypes.c_char_p
    lib.prism_peaks_measure.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    index = {lib.prism_peaks_name(i).decode(): i for i in range(lib.prism_peaks_count())}
    rows = []
    for name, args in PEAK_PROBES:
        if which is not None:
            if name not in which:
                continue
            args = which[name]
        for arg in args:
            out = (ctypes.c_double * 4)()
            if lib.prism_peaks_measure(index[name], arg, out) != 0:
                raise RuntimeError(f"peak probe {name}({arg}) failed")
            ms, work = out[0], out[1]
            if name.startswith("mfma"):
                rate, unit = work / ms / 1e9, "TFLOP/s"
            elif name.startswith("valu"):
                rate, unit = work * 64 / ms / 1e9, "Tlane-op/s"
            else:
                rate, unit = work / ms / 1e6, "GB/s"
            rows.append({"probe": name, "arg": arg, "ms": round(ms, 4), "rate": round(rate, 1), "unit": unit,
                         "shader_mhz": round(out[2], 0), "cycles_per_op": round(out[3], 2)})
            log(f"peak {name}({arg}): {rate:.1f} {unit}, {out[2]:.0f} MHz, {out[3]:.2f} cycles/op")
    return rows


def measure_issue_patterns():
    """Cycles per repetition of short instruction patterns for one wave per SIMD (libprism_peaks.so)."""
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2602_08426_amd", "libprism_peaks.so"))
    lib.prism_peaks_name.restype = ctypes.c_char_p
    lib.prism_peaks_issue_pattern_name.restype = ctypes.c_char_p
    lib.prism_peaks_measure.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    probe = {lib.prism_peaks_name(i).decode(): i for i in range(lib.prism_peaks_count())}["issue_pattern"]
    rows = []
    for pat in range(lib.prism_peaks_issue_patterns()):
        out = (ctypes.c_double * 4)()
        if lib.prism_peaks_measure(probe, pat, out) != 0:
            raise RuntimeError(f"issue pattern {pat} failed")
        name = lib.prism_peaks_issue_pattern_name(pat).decode()
        rows.append({"pattern": name, "cycles_per_repetition": round(out[3], 2), "shader_mhz": round(out[2], 0)})
        log(f"issue pattern [{name}]: {out[3]:.2f} cycles, {out[2]:.0f} MHz")
    return rows


def peaks_main() -> int:
    rows = measure_peaks()
    print(json.dumps({"metric": "achievable peaks of this GPU (probe loops of libprism_peaks.so)",
                      "published": {"bf16_mfma_tflops": PEAK_BF16_TFLOPS, "hbm_gbs": PEAK_HBM_GBS},
                      "arg_meaning": "workgroups per CU for the on-chip probes, footprint in MiB for stream_read_16B",
                      "rows": rows,
                      "issue_patterns_one_wave_per_simd": measure_issue_patterns()}), flush=True)
    return 0


def cpu_baseline(w, Qb, Kb, Vb, mask, flop_dense: float, budget_rows: int = 2048):
    """Time the oracle (as it stands): the selection in full, kv group by kv group, and the
    block-masked attention on a seeded sample of (head, q-block) rows drawn over all heads and
    extrapolated by executed-block count."""
    import numpy as np
    from oracle import prism_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    g = w.group
    N, B = w.n_blocks, w.block
    t_sel = 0.0
    for kv in range(w.n_kv_heads):
        Qg = orc.bf16_to_f64(Qb[kv * g:(kv + 1) * g])
        Kg = orc.bf16_to_f64(Kb[kv:kv + 1])
        t0 = time.perf_counter()
        orc.prism_select(Qg, Kg, w.d_high, w.d_low, B, w.top_p)
        t_sel += time.perf_counter() - t0
    rng = np.random.default_rng(0)
    rows = sorted((int(rng.integers(w.n_q_heads)), int(rng.integers(N))) for _ in range(budget_rows))
    t_rows, blocks_sample = 0.0, 0
    for kv in sorted({hq // g for hq, _ in rows}):
        Qg = orc.bf16_to_f64(Qb[kv * g:(kv + 1) * g])
        Kg = orc.bf16_to_f64(Kb[kv:kv + 1])
        Vg = orc.bf16_to_f64(Vb[kv:kv + 1])
        mine = [(hq - kv * g, u) for hq, u in rows if hq // g == kv]
        t0 = time.perf_counter()
        orc.block_sparse_attention(Qg, Kg, Vg, mask[kv * g:(kv + 1) * g], B, mine)
        t_rows += time.perf_counter() - t0
        blocks_sample += sum(int(mask[kv * g + hq, u, :u + 1].sum()) for hq, u in mine)
    t_attn = t_rows * (float(mask.sum()) / max(blocks_sample, 1))
    total = t_sel + t_attn
    return {
        "value": flop_dense / total / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": (f"selection oracle timed in full (all {w.n_kv_heads} kv groups, {w.n_q_heads} q-heads); "
                   f"attention oracle on {budget_rows} seeded (head,q-block) rows over all heads ({blocks_sample} "
                   f"blocks, {t_rows:.1f} s), scaled by executed-block count to {int(mask.sum())} blocks"),
        "est_seconds": round(t_sel, 2), "attn_seconds_extrapolated": round(t_attn, 2),
    }


def estimate_curve(args) -> int:
    """prism_estimate latency at 8K..128K for B = 128 and 64 on the Llama-shaped layer."""
    import numpy as np
    import torch

    from paper_2602_08426_amd import binding as pb
    from paper_2602_08426_amd import workloads as wl

    base = wl.WORKLOADS["c4_llama_128k"]
    rows = []
    for L in (8192, 16384, 32768, 65536, 131072):
        w = wl.small_variant(base, L)
        Qb, Kb, _ = wl.generate(w, n_threads=args.gen_threads)
        q, k = pb.bf16_bits_to_device(Qb), pb.bf16_bits_to_device(Kb)
        for B in (128, 64):
            params = pb.make_params(w.n_q_heads, w.n_kv_heads, L, B, w.d_high, w.d_low, w.top_p)
            N = L // B
            pairs = w.n_q_heads * N * (N + 1) // 2
            mask_bits, row_ptr, col_idx, info = pb.alloc_estimate_outputs(params, pairs)
            ws = pb.alloc_workspace(pb.prism_estimate_workspace_bytes(params))
            for _ in range(3):
                pb.prism_estimate(params, q, k, mask_bits, row_ptr, col_idx, pairs, info, ws)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(10):
                pb.prism_estimate(params, q, k, mask_bits, row_ptr, col_idx, pairs, info, ws)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / 10
            dens = int(info.cpu()[0]) / pairs
            rows.append({"seq_len": L, "block": B, "ms_estimate": round(ms, 4), "block_density": round(dens, 4)})
            log(f"L={L} B={B}: estimate {ms:.3f} ms, density {dens:.3f}")
            del mask_bits, row_ptr, col_idx, info, ws
        del q, k
    print(json.dumps({"metric": "prism_estimate latency vs sequence length", "unit": "ms", "data": "synthetic",
                      "paper_context": "paper: ~9 ms (B=128) and ~22 ms (B=64) at 128K on its hardware",
                      "rows": rows}), flush=True)
    return 0


def occupancy_sweep() -> int:
    """Attention throughput per busy workgroup when only part of the chip works: uniform rows of 2048
    entries over 16 cache-resident blocks (B = 128, d = 128), from 16 rows (16 workgroups on 16 CUs) to
    8192 rows (512 persistent workgroups, two per CU), both attention kernels.  Separates what a workgroup
    can do at the clock of a lightly loaded chip from what the power limit leaves when all 256 CUs run."""
    import numpy as np
    import torch

    from paper_2602_08426_amd import binding as pb

    B, n = 128, 2048
    rows_out = []
    for h, L in ((1, 2048), (1, 8192), (4, 8192), (8, 8192), (16, 8192), (32, 32768)):
        hkv = 1 if h < 8 else h // 4
        N = L // B
        torch.manual_seed(0)
        q = torch.randn((h, L, 128), device="cuda").to(torch.bfloat16)
        k = torch.randn((hkv, L, 128), device="cuda").to(torch.bfloat16)
        v = torch.randn((hkv, L, 128), device="cuda").to(torch.bfloat16)
        lst = np.tile(np.arange(16, dtype=np.int32), n // 16)
        rp = torch.arange(0, (h * N + 1) * n, n, dtype=torch.int32, device="cuda")
        ci = torch.from_numpy(np.tile(lst, h * N)).cuda()
        for tag, fl in (("sparse_attn_kernel<128>", pb.PRISM_FLAG_GENERAL_KERNEL), ("sparse_attn_w64_kernel", 0)):
            params = pb.make_params(h, hkv, L, B, flags=fl | pb.PRISM_FLAG_BIDIRECTIONAL)
            img = pb.alloc_workspace(pb.prism_sparse_attn_workspace_bytes(params))
            pb.prism_v_image(params, v, img)
            out = torch.empty_like(q)
            pb.prism_sparse_attn_pre(params, q, k, img, rp, ci, ci.numel(), out, None)
            torch.cuda.synchronize()
            ts = []
            for _ in range(3):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                pb.prism_sparse_attn_pre(params, q, k, img, rp, ci, ci.numel(), out, None)
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            rows = h * N
            wgs = min(rows, 512)
            tf = 4.0 * B * B * 128 * ci.numel() / (min(ts) * 1e-3) / 1e12
            rows_out.append({"kernel": tag, "rows": rows, "workgroups": wgs, "ms": round(min(ts), 3),
                             "tflops": round(tf, 1), "tflops_per_workgroup": round(tf / wgs, 3)})
            log(f"rows {rows:5d} workgroups {wgs:3d} {tag}: {min(ts):.3f} ms, {tf:.1f} TFLOP/s, "
                f"{tf / wgs:.3f} per workgroup")
    print(json.dumps({"metric": "attention throughput vs number of busy workgroups (cache-resident uniform lists)",
                      "unit": "TFLOP/s", "rows": rows_out}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4_llama_128k")
    ap.add_argument("--dense-reps", type=int, default=2)
    ap.add_argument("--graph-reps", type=int, default=10,
                    help="replays of the step captured in a HIP graph (0 = skip)")
    ap.add_argument("--stream-reps", type=int, default=3,
                    help="repetitions of the attention kernel with its arithmetic left out (memory side alone)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gen-threads", type=int, default=16)
    ap.add_argument("--estimate-curve", action="store_true",
                    help="instead of the step benchmark: prism_estimate time vs sequence length for "
                         "B = 128 and B = 64 (the block-size study of the paper's App. E), one JSON line")
    ap.add_argument("--peaks", action="store_true",
                    help="instead of the step benchmark: run the machine-peak probes (MFMA-only loop, MFMA with "
                         "LDS operand reads, LDS reads, VALU, streaming reads over several footprints), one JSON line")
    ap.add_argument("--no-peaks", action="store_true", help="skip the two peak probes of the default run")
    ap.add_argument("--occupancy-sweep", action="store_true",
                    help="instead of the step benchmark: attention throughput per busy workgroup from 16 to 512 "
                         "workgroups on cache-resident lists (what the power limit costs), one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) for counter calibration")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2602_08426_amd import binding as pb
    from paper_2602_08426_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    pb._load()                                   # fails loudly if libprism.so is missing
    if args.estimate_curve:
        return estimate_curve(args)
    if args.peaks:
        return peaks_main()
    if args.occupancy_sweep:
        return occupancy_sweep()
    w = wl.WORKLOADS[args.workload]
    h, hkv, L, B, N, d = w.n_q_heads, w.n_kv_heads, w.seq_len, w.block, w.n_blocks, w.head_dim

    t0 = time.perf_counter()
    Qb, Kb, Vb = wl.generate(w, n_threads=args.gen_threads)
    log(f"generated {w.name} in {time.perf_counter() - t0:.1f}s")
    q, k, v = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    params = pb.make_params(h, hkv, L, B, w.d_high, w.d_low, w.top_p)
    pairs = h * N * (N + 1) // 2
    mask_bits, row_ptr, col_idx, info = pb.alloc_estimate_outputs(params, pairs)
    ws_est = pb.alloc_workspace(pb.prism_estimate_workspace_bytes(params))
    v_image = pb.alloc_workspace(pb.prism_sparse_attn_workspace_bytes(params))
    out = torch.empty_like(q)
    stream = torch.cuda.current_stream()

    def step(ev=None):
        if ev:
            ev[0].record(stream)
        pb.prism_estimate(params, q, k, mask_bits, row_ptr, col_idx, pairs, info, ws_est)
        if ev:
            ev[1].record(stream)
        pb.prism_v_image(params, v, v_image)
        if ev:
            ev[2].record(stream)
        # col_count = capacity: row_ptr never exceeds it, so no host sync is needed here
        pb.prism_sparse_attn_pre(params, q, k, v_image, row_ptr, col_idx, pairs, out, None)
        if ev:
            ev[3].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    nnz = int(info.cpu()[0])
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    t_est = [e[0].elapsed_time(e[1]) for e in events]
    t_vimg = [e[1].elapsed_time(e[2]) for e in events]
    t_attn = [e[2].elapsed_time(e[3]) for e in events]
    t_all = [e[0].elapsed_time(e[3]) for e in events]
    ms_est, ms_vimg, ms_attn = float(np.mean(t_est)), float(np.mean(t_vimg)), float(np.mean(t_attn))
    log(f"step {ms_step:.3f} ms  (estimate {ms_est:.3f}, v_image {ms_vimg:.3f}, sparse attention {ms_attn:.3f})")

    # the same step replayed from a HIP graph (launch overhead of the ~11 kernels taken out; matters
    # for the short workloads only)
    ms_graph = None
    if args.graph_reps > 0:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            step()
        stream.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.graph_reps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / args.graph_reps
        del graph
        log(f"step replayed from a HIP graph {ms_graph:.3f} ms")

    # dense baseline: the same attention kernel over the all-ones causal lists
    ms_dense = None
    if args.dense_reps > 0:
        rp_d = torch.empty_like(row_ptr)
        ci_d = torch.empty(pairs, dtype=torch.int32, device="cuda")
        pb.prism_causal_csr(params, rp_d, ci_d, pairs)
        out_d = torch.empty_like(q)
        pb.prism_sparse_attn_pre(params, q, k, v_image, rp_d, ci_d, pairs, out_d, None)   # warm-up
        torch.cuda.synchronize()
        evd = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(args.dense_reps)]
        for a, b in evd:
            a.record(stream)
            pb.prism_sparse_attn_pre(params, q, k, v_image, rp_d, ci_d, pairs, out_d, None)
            b.record(stream)
        torch.cuda.synchronize()
        ms_dense = float(np.mean([a.elapsed_time(b) for a, b in evd])) + ms_vimg
        del rp_d, ci_d, out_d
        log(f"dense causal (same kernel, all-ones lists) {ms_dense:.3f} ms")

    # memory side alone: the same kernel with its arithmetic left out (tile copies, waits, queue)
    ms_stream = None
    if args.stream_reps > 0:
        p_stream = pb.make_params(h, hkv, L, B, w.d_high, w.d_low, w.top_p, flags=pb.PRISM_FLAG_STREAM_ONLY)
        out_s = torch.empty_like(q)
        pb.prism_sparse_attn_pre(p_stream, q, k, v_image, row_ptr, col_idx, pairs, out_s, None)   # warm-up
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(args.stream_reps)]
        for a, b in evs:
            a.record(stream)
            pb.prism_sparse_attn_pre(p_stream, q, k, v_image, row_ptr, col_idx, pairs, out_s, None)
            b.record(stream)
        torch.cuda.synchronize()
        ms_stream = float(np.mean([a.elapsed_time(b) for a, b in evs]))
        del out_s
        log(f"sparse attention, tile streaming only (no arithmetic) {ms_stream:.3f} ms")

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                           # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # achievable peaks of this very box, measured after the timed region: an MFMA-only loop with
    # operands in registers and a 16-byte streaming read over an 8 GiB footprint
    peak_mfma = peak_stream = None
    if not args.no_peaks:
        rows = measure_peaks({"mfma_32x32x16_bf16_only": (2,), "stream_read_16B": (8192,)})
        peak_mfma = next(r for r in rows if r["probe"].startswith("mfma"))
        peak_stream = next(r for r in rows if r["probe"].startswith("stream"))

    def vs_measured(x, row):
        return None if row is None else round(x / row["rate"], 4)

    flop_block = 4.0 * B * B * d
    flop_dense = flop_block * pairs
    flop_exec = flop_block * nnz
    density = nnz / pairs
    eff_tflops = flop_dense / (ms_step * 1e-3) / 1e12
    exec_tflops = flop_exec / (ms_attn * 1e-3) / 1e12
    # the attention kernel against the memory roof: bytes that crossed the L2 <-> fabric boundary
    # per launch (rocprofv3 counters of the committed profile of this workload) over the launch time
    # measured here.  The no-reuse bytes (K and V^T tile per listed block, Q in, O out) are kept
    # beside it as the algorithmic figure; rows that share tiles are served by the L2s.
    w64 = (B == 128 and L % 128 == 0)
    pair = (B == 64 and N % 2 == 0 and h * N >= 4096)       # two q-blocks per workgroup (pair kernel)
    attn_kernel = ("sparse_attn_w64_kernel" if w64 else
                   f"sparse_attn_kernel<{B}, false, {d}, {'true' if pair else 'false'}>")
    attn_key = "sparse_attn_w64_kernel" if w64 else ("sparse_attn_kernel_pair" if pair else "sparse_attn_kernel")
    attn_traffic, attn_src = profiled_traffic(w.name, attn_key)
    attn_bytes = nnz * 2 * B * d * 2 + 2 * Qb.nbytes
    attn_gbs = None if attn_traffic is None else attn_traffic / (ms_attn * 1e-3) / 1e9
    est_bytes = (Qb.nbytes + Kb.nbytes)
    est_gbs = est_bytes / (ms_est * 1e-3) / 1e9
    est_traffic, est_src = profiled_traffic(w.name, "pool_energy_kernel")

    result = {
        "metric": "prefill attention effective TFLOP/s at 128K (estimate+sparse), ms alongside",
        "value": round(eff_tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "n_q_heads": h, "n_kv_heads": hkv, "seq_len": L, "block": B,
                   "head_dim": d, "d_high": w.d_high, "d_low": w.d_low, "top_p": w.top_p,
                   "rope_base": w.rope_base, "seed": w.seed},
        "library": os.path.relpath(pb.library_path(), ROOT),
        "detail": {
            "ms_estimate": round(ms_est, 4), "ms_v_image": round(ms_vimg, 4),
            "ms_sparse_attn": round(ms_attn, 4),
            "ms_step_events": stats(t_all), "ms_estimate_events": stats(t_est),
            "ms_sparse_attn_events": stats(t_attn),
            "ms_per_step_hip_graph": None if ms_graph is None else round(ms_graph, 4),
            "ms_sparse_attn_stream_only": None if ms_stream is None else round(ms_stream, 4),
            "ms_dense_same_kernel": None if ms_dense is None else round(ms_dense, 3),
            "speedup_vs_dense": None if ms_dense is None else round(ms_dense / ms_step, 3),
            "estimate_over_dense": None if ms_dense is None else round(ms_est / ms_dense, 5),
            "block_density": round(density, 5), "nnz_blocks": nnz,
            "executed_tflops": round(exec_tflops, 2),
            "executed_tflops_best_step": round(flop_exec / (min(t_attn) * 1e-3) / 1e12, 2),
            "dense_tflops": None if ms_dense is None else round(flop_dense / ((ms_dense - ms_vimg) * 1e-3) / 1e12, 2),
            "estimate_gbs": round(est_gbs, 1), "estimate_frac_hbm_peak": round(est_gbs / PEAK_HBM_GBS, 4),
            "paper_context": "paper reports up to 5.1x over FlashAttention-2 at 128K on one H100 (different hardware)",
        },
        "roofline": {"kernel": attn_kernel, "bound": "mfma", "achieved": round(exec_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(exec_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": attn_traffic, "traffic_source": attn_src,
                     "peak_measured": None if peak_mfma is None else peak_mfma["rate"],
                     "peak_measured_probe": None if peak_mfma is None else
                     f"mfma_32x32x16_bf16_only, 2 workgroups per CU, {peak_mfma['shader_mhz']:.0f} MHz under load",
                     "frac_of_measured": vs_measured(exec_tflops, peak_mfma),
                     "flops_per_launch": flop_exec, "avg_launch_ms": round(ms_attn, 4),
                     "launch_ms": stats(t_attn),
                     "note": "avg_launch_ms is the whole prism_sparse_attn_pre call (queue build + list check + "
                             "attention kernel), so `achieved` is a lower bound for the kernel alone"},
        "roofline_sparse_attn_memory": {"kernel": attn_kernel, "bound": "hbm",
                                        "achieved": None if attn_gbs is None else round(attn_gbs, 1),
                                        "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                        "frac": None if attn_gbs is None else round(attn_gbs / PEAK_HBM_GBS, 4),
                                        "traffic": attn_traffic, "traffic_source": attn_src,
                                        "peak_measured": None if peak_stream is None else peak_stream["rate"],
                                        "peak_measured_probe": None if peak_stream is None else
                                        "stream_read_16B over 8 GiB",
                                        "frac_of_measured": None if attn_gbs is None else vs_measured(attn_gbs, peak_stream),
                                        "bytes_per_launch_no_reuse": attn_bytes, "avg_launch_ms": round(ms_attn, 4),
                                        "stream_only_ms": None if ms_stream is None else round(ms_stream, 4),
                                        "note": "achieved = counter bytes of the committed profile / launch time of "
                                                "this run; bytes_per_launch_no_reuse = 64 KB per listed block pair + "
                                                "Q in + O out, what the kernel would move if no tile were shared"},
        "roofline_estimate": {"kernel": "prism_estimate (5 kernels; pool_energy_kernel carries the bytes)",
                              "bound": "hbm", "achieved": round(est_gbs, 1), "peak": PEAK_HBM_GBS,
                              "unit": "GB/s", "frac": round(est_gbs / PEAK_HBM_GBS, 4),
                              "traffic": est_traffic, "traffic_source": est_src,
                              "peak_measured": None if peak_stream is None else peak_stream["rate"],
                              "frac_of_measured": vs_measured(est_gbs, peak_stream),
                              "bytes_per_launch": est_bytes, "avg_launch_ms": round(ms_est, 4),
                              "launch_ms": stats(t_est)},
    }

    if not args.no_cpu_baseline:
        words = mask_bits.cpu().numpy().view(np.uint64)
        W = (N + 63) // 64
        bits = np.unpackbits(words.view(np.uint8).reshape(h, N, W * 8), axis=-1, bitorder="little")
        mask = bits[:, :, :N].astype(bool)
        t0 = time.perf_counter()
        result["cpu_baseline"] = cpu_baseline(w, Qb, Kb, Vb, mask, flop_dense)
        log(f"cpu baseline took {time.perf_counter() - t0:.1f}s")
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
