#!/usr/bin/env python3
"""Benchmark of the PureKV hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input, in the paper's order
(Sec. 3.1 / 3.2), for the 32-frame Qwen2.5-VL-7B-shaped workload:
    low layer : dense causal prefill (+ log-sum-exp)  -> recent-window column sums C (Eq. 2)
                -> V-norm top-h (Eq. 3) -> compaction
    high layer: ST-SpAttn prefill -> V-norm top-h with the low layer's C (Eq. 4) -> compaction
                -> append one decoded token -> decode attention on the compact cache
All inputs are resident in HBM before the timed region.  Prints one JSON line.

`value` is the metric's headline: TFLOP/s of the ST-SpAttn prefill counted on the key tiles it visits
(one launch; split text rows are combined inside it), from HIP events recorded on the launch stream inside the timed
steps.  The same line carries the per-stage times, GB/s of the HBM-bound stages, the roofline object and
the CPU oracle timed on a bounded sample.
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

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBPS = 8000.0
STAGES = ["dense_prefill", "importance", "topk_low", "compact_low", "st_prefill", "topk_high", "compact_high",
          "append_decode"]


def blas_threads() -> int:
    """Threads NumPy's BLAS actually uses for the oracle's matrix products."""
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return int(max(n))
    except Exception:
        pass
    return int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))


def profiled_traffic_bytes():
    """HBM bytes per ST-SpAttn prefill call from the committed rocprofv3 counter summary (the prefill kernel):
    FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB, the factors a 256 MiB device copy calibrates.  None if absent."""
    path = os.path.join(ROOT, "profiles", "prefill_kernel_st_qwen25vl_32f.md")
    try:
        total, in_table = 0.0, False
        for line in open(path):
            if line.startswith("## "):
                in_table = line.startswith("## Kernel durations")
            cells = [c.strip() for c in line.split("|")]
            if in_table and len(cells) >= 9 and cells[1].startswith("`prefill_kernel<128, true"):
                try:
                    total += float(cells[7]) * 2.0 * 1024 + float(cells[8]) * 1024
                except ValueError:
                    pass
        return int(total) if total > 0 else None
    except OSError:
        return None


PMC_PASSES = [
    "SQ_WAVES SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_SMEM SQ_INSTS_MFMA SQ_INSTS_BRANCH SQ_INSTS_VMEM",
    "SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS "
    "SQ_VALU_MFMA_BUSY_CYCLES SQ_LDS_BANK_CONFLICT",
    "SQ_ACTIVE_INST_ANY SQ_ACTIVE_INST_SCA SQ_WAIT_ANY SQ_LDS_IDX_ACTIVE SQ_LDS_ADDR_CONFLICT SQ_INSTS_VALU_MFMA_MOPS_BF16 "
    "SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_TRANS_F32",
]


def profile_commands(stage: str, steps: int):
    """The rocprofv3 commands whose output `--profile-summary` reads (run from /tmp with TMPDIR=/tmp; $R = repository
    root, $D = the directory given to --profile-summary)."""
    if stage == "whole_path":   # the benchmark command itself (as the driver runs it), kernel statistics only
        return [f"rocprofv3 --kernel-trace --stats --output-format csv -d $D/stats -o s -- python3 $R/bench.py --steps {steps} "
                "--warmup 5 --no-cpu-baseline"]
    run = f"python3 $R/bench.py --only-stage {stage}"
    cmds = [f"rocprofv3 --kernel-trace --stats --output-format csv -d $D/stats -o s -- {run} --steps {steps}",
            f"rocprofv3 --pmc FETCH_SIZE --output-format csv -d $D/fetch -o p -- {run} --steps 5",
            f"rocprofv3 --pmc WRITE_SIZE --output-format csv -d $D/write -o p -- {run} --steps 5"]
    cmds += [f"rocprofv3 --pmc {c} --output-format csv -d $D/p{i + 1} -o p -- {run} --steps 3" for i, c in enumerate(PMC_PASSES)]
    return cmds


def write_profile_summary(src_dir: str, stage: str, name: str, title: str, steps: int) -> str:
    """Turns the CSV files rocprofv3 wrote under `src_dir` (see profile_commands) into profiles/<name>.md: kernel
    durations per (kernel, grid), HBM-side byte counters, and the SQ counter passes per kernel.  Text in, text out."""
    import collections
    import csv
    import glob

    def short(k):
        k = k.replace("purekv::(anonymous namespace)::", "").replace("void ", "")
        return k.split("(")[0] if "rocclr" not in k else k

    def find(sub, pattern):
        hits = sorted(glob.glob(os.path.join(src_dir, sub, "**", pattern), recursive=True))
        return hits[0] if hits else None

    out = [f"# {title}\n", "Commands (run from /tmp with TMPDIR=/tmp on the MI355X box; `$R` = repository root, `$D` = output "
           "directory), then `python3 $R/bench.py --profile-summary $D --only-stage " + stage + " --profile-name " + name + "`:\n", "```"]
    out += profile_commands(stage, steps) + ["```\n"]
    if stage == "whole_path":
        out.append(f"The benchmark command as the driver runs it ({steps} timed steps after the clock ramp and 5 warm-up steps; the "
                   "graph replays, the back-to-back timings, the batched launches and the calibration loops of the same "
                   "command are in the table too).  The profiler serialises dispatches, so gaps between kernels differ from "
                   "an unprofiled run; kernel durations do not.\n")
    else:
        out.append(f"`--only-stage` runs one full warm-up step of the whole path (every kernel once, at its per-layer size) and "
                   f"then the named stage {steps} times (fewer in the counter runs).  Rows are per (kernel, grid size), so the "
                   "warm-up dispatches and the stage's own dispatches stay apart.\n")
    trace = find("stats", "*kernel_trace.csv")
    dur = collections.defaultdict(list)
    if trace:
        for r in csv.DictReader(open(trace)):
            g = int(r["Grid_Size_X"]) * int(r["Grid_Size_Y"]) * int(r["Grid_Size_Z"])
            dur[(short(r["Kernel_Name"]), g)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)

    def counters(sub):
        d = collections.defaultdict(lambda: collections.defaultdict(list))
        path = find(sub, "*counter_collection.csv")
        if path:
            for r in csv.DictReader(open(path)):
                d[(short(r["Kernel_Name"]), int(r["Grid_Size"]))][r["Counter_Name"]].append(float(r["Counter_Value"]))
        return d

    fetch, write = counters("fetch"), counters("write")
    out.append("## Kernel durations (kernel trace) and HBM-side byte counters (KiB per dispatch)\n")
    out.append("| kernel | grid (work-items) | dispatches | avg us | min us | max us | FETCH_SIZE KiB | WRITE_SIZE KiB |")
    out.append("|---|---|---|---|---|---|---|---|")
    for (k, g), v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        if "at::native" in k or ("rocclr" in k and stage != "copy_calib"):
            continue
        fv, wv = fetch.get((k, g), {}).get("FETCH_SIZE"), write.get((k, g), {}).get("WRITE_SIZE")
        fs = f"{sum(fv) / len(fv):.1f}" if fv else "-"
        ws = f"{sum(wv) / len(wv):.1f}" if wv else "-"
        out.append(f"| `{k[:64]}` | {g} | {len(v)} | {sum(v) / len(v):.2f} | {min(v):.2f} | {max(v):.2f} | {fs} | {ws} |")
    stats = find("stats", "*kernel_stats.csv")
    if stats:
        out.append("\n## rocprofv3 --stats summary (all dispatches of a kernel pooled)\n")
        out.append("| kernel | calls | avg us | min us | max us | % of GPU time |")
        out.append("|---|---|---|---|---|---|")
        for r in csv.DictReader(open(stats)):
            nm = short(r["Name"])
            if "at::native" in nm:
                continue
            out.append(f"| `{nm[:64]}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | "
                       f"{float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.2f} |")
    sq = collections.defaultdict(dict)
    for i in range(len(PMC_PASSES)):
        for key, cs in counters(f"p{i + 1}").items():
            for cname, vals in cs.items():
                sq[key][cname] = sum(vals) / len(vals)
    if sq:
        out.append("\n## SQ counters per dispatch (sums over the whole chip; three passes of 8 counters)\n")
        biggest = sorted(sq, key=lambda key: -sq[key].get("SQ_WAVE_CYCLES", sq[key].get("SQ_INSTS_VALU", 0)))[:3]
        names = sorted({c for key in biggest for c in sq[key]})
        out.append("| counter | " + " | ".join(f"`{k[:40]}` grid {g}" for k, g in biggest) + " |")
        out.append("|---|" + "---|" * len(biggest))
        for c in names:
            out.append(f"| {c} | " + " | ".join(f"{sq[key].get(c, float('nan')):.0f}" for key in biggest) + " |")
        out.append("\nDerived, per kernel (plain ratios of the rows above):\n")
        for key in biggest:
            c = sq[key]
            def ratio(a, b):
                return f"{c[a] / c[b]:.3f}" if a in c and c.get(b) else "n/a"
            out.append(f"* `{key[0][:48]}`: instructions per wavefront: vector {ratio('SQ_INSTS_VALU', 'SQ_WAVES')} "
                       f"(of them MFMA {ratio('SQ_INSTS_MFMA', 'SQ_WAVES')}, transcendental {ratio('SQ_INSTS_VALU_TRANS_F32', 'SQ_WAVES')}), "
                       f"scalar {ratio('SQ_INSTS_SALU', 'SQ_WAVES')}, LDS {ratio('SQ_INSTS_LDS', 'SQ_WAVES')}, vector memory "
                       f"{ratio('SQ_INSTS_VMEM', 'SQ_WAVES')}, branch {ratio('SQ_INSTS_BRANCH', 'SQ_WAVES')}; of a wavefront's "
                       f"cycles: an instruction active {ratio('SQ_ACTIVE_INST_ANY', 'SQ_WAVE_CYCLES')}, waiting for an issue slot "
                       f"{ratio('SQ_WAIT_INST_ANY', 'SQ_WAVE_CYCLES')}, waiting at a counter or barrier {ratio('SQ_WAIT_ANY', 'SQ_WAVE_CYCLES')}; "
                       f"MFMA-busy cycles / wavefront cycles {ratio('SQ_VALU_MFMA_BUSY_CYCLES', 'SQ_WAVE_CYCLES')}; "
                       f"LDS bank-conflict cycles / LDS active cycles {ratio('SQ_LDS_BANK_CONFLICT', 'SQ_LDS_IDX_ACTIVE')}")
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    path = os.path.join(ROOT, "profiles", name + ".md")
    open(path, "w").write("\n".join(out) + "\n")
    return path


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="qwen25vl_32f")
    ap.add_argument("--ratio", type=float, default=0.2)
    ap.add_argument("--batched-layers", type=int, default=26, help="layers per batched top-k/compaction launch")
    ap.add_argument("--ramp-ms", type=float, default=150.0,
                    help="untimed clock ramp before the warm-up steps: the board's calibration loop (tile-step skeleton) is "
                         "run for about this many milliseconds so that the shader clock has left its idle state, as it "
                         "has inside the prefill of a whole model; reported as `clock_ramp`; 0 disables it")
    ap.add_argument("--layout", default="packed", choices=["packed", "token_major"],
                    help="layout of Q, K, V, O in the per-layer step: packed [H, N, d], or token-major views of one "
                         "[N, (Hq + 2 Hkv) d] buffer as a decoder's QKV projection writes it (O as [N, Hq d]); the layer-"
                         "batched selection and compaction always read packed layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-heads", type=int, default=28, help="query heads in the oracle's timed sample")
    ap.add_argument("--stack", action="store_true",
                    help="time the whole layer stack of the workload (purekv_stack_layer per layer, then one batched "
                         "selection and compaction) instead of the one-layer-pair step; prints its own JSON line")
    ap.add_argument("--stack-layers", type=int, default=0, help="layers of the --stack run (default: the workload's)")
    ap.add_argument("--stack-dense", type=int, default=0, help="dense low layers of the --stack run (default: the "
                    "workload's, else 1); the last of them estimates the importance")
    ap.add_argument("--only-stage", default=None,
                    choices=STAGES + ["copy_calib", "topk_batched", "compact_batched", "spearman_batched", "dense_prefill_all_rows_lse", "mfma_calib", "whole_path"],
                    help="profiling aid: after one full warm-up step run only this stage --steps times and exit")
    ap.add_argument("--profile-summary", default=None, metavar="DIR",
                    help="no GPU work: turn the rocprofv3 CSV output under DIR (produced by the commands this prints with "
                         "--profile-commands for the stage given with --only-stage) into profiles/<--profile-name>.md")
    ap.add_argument("--profile-name", default=None)
    ap.add_argument("--profile-title", default=None)
    ap.add_argument("--profile-commands", action="store_true", help="print the rocprofv3 commands of a stage's profile and exit")
    args = ap.parse_args()
    if args.profile_commands or args.profile_summary:
        stage = args.only_stage or "st_prefill"
        steps = args.steps if args.steps != 200 else 30
        if stage == "whole_path" and args.steps == 200:
            steps = 20
        if args.profile_commands:
            print("\n".join(profile_commands(stage, steps)))
            return 0
        name = args.profile_name or f"{stage}_{args.workload}"
        title = args.profile_title or f"{stage}, workload {args.workload}"
        print("wrote", write_profile_summary(args.profile_summary, stage, name, title, steps))
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2510_25600_amd as pk
    from workloads import WORKLOADS, generate

    wl = WORKLOADS[args.workload]
    n, w, d, hq, hkv = wl.n_tokens, wl.window, wl.head_dim, wl.n_q_heads, wl.n_kv_heads
    h = pk.purekv_budget(n, w, args.ratio)
    n_keep, cap = h + w, h + w + 1
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    def to_dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(dev)

    low, high = generate(wl, seed=wl.seed, decode_steps=1), generate(wl, seed=wl.seed + 1, decode_steps=1)
    q0, k0, v0 = to_dev(low.q), to_dev(low.k), to_dev(low.v)
    q1, k1, v1 = to_dev(high.q), to_dev(high.k), to_dev(high.v)
    q_new, k_new, v_new = to_dev(high.q_new[0]), to_dev(high.k_new[0]), to_dev(high.v_new[0])
    calib_src = q0   # 4 MiB of finite bf16 values for the calibration loops
    st_packed = pk.Plan.for_workload(wl, pk.PATTERN_ST)   # the layer-batched calls read packed [L, Hkv, N, d] layers
    if args.layout == "token_major":
        row = (hq + 2 * hkv) * d

        def fuse(q_, k_, v_):
            buf = torch.empty((n, row), dtype=torch.bfloat16, device=dev)
            buf[:, :hq * d] = q_.permute(1, 0, 2).reshape(n, hq * d)
            buf[:, hq * d:(hq + hkv) * d] = k_.permute(1, 0, 2).reshape(n, hkv * d)
            buf[:, (hq + hkv) * d:] = v_.permute(1, 0, 2).reshape(n, hkv * d)
            return (buf[:, :hq * d].view(n, hq, d).permute(1, 0, 2), buf[:, hq * d:(hq + hkv) * d].view(n, hkv, d).permute(1, 0, 2),
                    buf[:, (hq + hkv) * d:].view(n, hkv, d).permute(1, 0, 2))

        v1_packed = v1
        k1_packed = k1
        q0, k0, v0 = fuse(q0, k0, v0)
        q1, k1, v1 = fuse(q1, k1, v1)
        strides = dict(q_strides=(d, row), kv_strides=(d, row), o_strides=(d, hq * d))
        dense = pk.Plan.for_workload(wl, pk.PATTERN_DENSE, lse_window=w, **strides)
        st = pk.Plan.for_workload(wl, pk.PATTERN_ST, **strides)
        out0, out1 = dense.empty_out(dev), st.empty_out(dev)
        layout = f"token-major: Q, K, V views of one [N, {row}] buffer (head stride {d}, token stride {row}), O [N, {hq * d}]"
    else:
        v1_packed, k1_packed = v1, k1
        # the designated low layer: a window plan (Eq. 2 reads the log-sum-exp of the last w rows only)
        dense = pk.Plan.for_workload(wl, pk.PATTERN_DENSE, lse_window=w)
        st = st_packed
        out0, out1 = torch.empty_like(q0), torch.empty_like(q1)
        layout = "packed [H, N, d] (head stride N*d, token stride d)"
    lse = torch.empty((hq, n), dtype=torch.float32, device=dev)
    c = torch.empty((hkv, n - w), dtype=torch.float32, device=dev)
    idx0 = torch.empty((1, hkv, n_keep), dtype=torch.int32, device=dev)
    idx1 = torch.empty((1, hkv, n_keep), dtype=torch.int32, device=dev)
    kc0 = torch.empty((hkv, cap, d), dtype=torch.bfloat16, device=dev)
    vc0, kc1, vc1 = torch.empty_like(kc0), torch.empty_like(kc0), torch.empty_like(kc0)
    o_dec = torch.empty((hq, d), dtype=torch.bfloat16, device=dev)

    def step(ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        pk.purekv_st_spattn_prefill(dense, q0, k0, v0, out=out0, lse=lse)
        mark(1)
        pk.purekv_lowlayer_importance(dense, q0, k0, lse, w, c_out=c)
        mark(2)
        pk.purekv_topk_select(dense, c, v0, w, h, idx_out=idx0)
        mark(3)
        pk.purekv_kv_compact(dense, k0, v0, idx0[0], cap=cap, kc=kc0, vc=vc0)
        mark(4)
        pk.purekv_st_spattn_prefill(st, q1, k1, v1, out=out1)
        mark(5)
        pk.purekv_topk_select(st, c, v1, w, h, idx_out=idx1)
        mark(6)
        pk.purekv_kv_compact(st, k1, v1, idx1[0], cap=cap, kc=kc1, vc=vc1)
        mark(7)
        pk.purekv_decode_step(st, q_new, k_new, v_new, kc1, vc1, n_keep, out=o_dec)
        mark(8)

    if args.stack:
        if args.layout != "packed":
            print("bench.py: --stack runs on packed layers", file=sys.stderr)
            return 2
        L = args.stack_layers or max(wl.n_layers, 2)
        st_layer = max(1, min(args.stack_dense or wl.n_dense_layers or 1, L))
        clie = st_layer - 1
        stack = pk.Stack(L, clie, st_layer, w, h)
        # per-layer data derived on the device from the two generated layers (rolled along the head axis)
        k_all = torch.empty((L, hkv, n, d), dtype=torch.bfloat16, device=dev)
        v_all, q_all = torch.empty_like(k_all), torch.empty((L, hq, n, d), dtype=torch.bfloat16, device=dev)
        for l in range(L):
            src_q, src_k, src_v = (q0, k0, v0) if l < st_layer else (q1, k1, v1)
            q_all[l], k_all[l], v_all[l] = src_q.roll(l, dims=0), src_k.roll(l, dims=0), src_v.roll(l, dims=0)
        out = torch.empty_like(q0)   # consumed by the rest of the model layer by layer: one buffer
        c_all = torch.empty((clie + 1, hkv, n - w), dtype=torch.float32, device=dev)
        idx_all = torch.empty((L, hkv, n_keep), dtype=torch.int32, device=dev)
        kc_all = torch.empty((L, hkv, n_keep, d), dtype=torch.bfloat16, device=dev)
        vc_all = torch.empty_like(kc_all)

        def run_stack():
            for l in range(L):
                pk.purekv_stack_layer(dense, st, stack, l, q_all[l], k_all[l], v_all[l], out, lse, c_all)
            pk.purekv_stack_select_compact(dense, st, stack, c_all, k_all, v_all, idx_all, kc_all, vc_all)

        reps = max(3, min(args.steps, 20))
        for _ in range(2):
            run_stack()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            run_stack()
        torch.cuda.synchronize()
        ms_eager = (time.perf_counter() - t0) * 1e3 / reps
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run_stack()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / reps
        flops = st_layer * dense.kept_tile_flops() + (L - st_layer) * st.kept_tile_flops()
        print(json.dumps({
            "metric": "layer_stack_prefill_select_compact_ms", "value": round(ms_graph, 3), "unit": "ms",
            "higher_is_better": False, "n_gpus": 1, "steps": reps, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"{wl.name}: {n} tokens, {hq}q/{hkv}kv heads, d={d}; {L} layers, dense below layer "
                                   f"{st_layer}, C from layer {clie}, keep ratio {args.ratio} (h={h}, w={w})"},
            "ms_eager": round(ms_eager, 3), "ms_one_graph_launch": round(ms_graph, 3),
            "prefill_tokens_per_s": round(n / (ms_graph * 1e-3), 1),
            "kept_tile_tflops_whole_stack": round(flops / (ms_graph * 1e-3) / 1e12, 1),
        }))
        return 0

    def make_batched(L):
        """Buffers of L high layers (Eq. 4: every high layer scores with the same C and its own V); distinct data
        per layer, derived on the device from the generated high layer."""
        v_all = torch.empty((L, hkv, n, d), dtype=torch.bfloat16, device=dev)
        k_all = torch.empty_like(v_all)
        for l in range(L):
            v_all[l] = v1_packed.roll(l, dims=1)
            k_all[l] = k1_packed.roll(l, dims=1)
        idx_all = torch.empty((L, hkv, n_keep), dtype=torch.int32, device=dev)
        kc_all = torch.empty((L, hkv, n_keep, d), dtype=torch.bfloat16, device=dev)
        vc_all = torch.empty_like(kc_all)
        return v_all, k_all, idx_all, kc_all, vc_all

    def mfma_calib(mix, random_operands, iters=40000):
        """One warm launch (≈ 20 ms: long enough for the clock to settle), then one event-timed launch of the
        board-calibration loop.  Returns (TFLOP/s, shader clock in GHz seen by wavefront 0)."""
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pk.purekv_calib_mfma(st, mix, random_operands, iters)
        torch.cuda.synchronize()
        a.record()
        flops, ticks = pk.purekv_calib_mfma(st, mix, random_operands, iters)
        b.record()
        torch.cuda.synchronize()
        cyc, ref = (int(x) for x in ticks.tolist())
        return flops / (a.elapsed_time(b) * 1e-3) / 1e12, cyc / max(ref, 1) / 10.0

    def step_calib(rows, iters=12000):
        """Tile-step skeleton (see purekv_calib_tile_step): one warm launch, one timed.  (TFLOP/s, us per step, GHz)"""
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pk.purekv_calib_tile_step(st, rows, iters, calib_src)
        torch.cuda.synchronize()
        a.record()
        flops, ticks = pk.purekv_calib_tile_step(st, rows, iters, calib_src)
        b.record()
        torch.cuda.synchronize()
        cyc, ref = (int(x) for x in ticks.tolist())
        ms = a.elapsed_time(b)
        return flops / (ms * 1e-3) / 1e12, ms * 1e3 / iters, cyc / max(ref, 1) / 10.0

    if args.only_stage == "mfma_calib":
        step()
        torch.cuda.synchronize()
        names = ["MFMA only", "MFMA + 1 KB LDS fragment read", "MFMA + LDS read + 2 fma + 2 exp + 1 convert"]
        for rnd in (False, True):
            for mix, name in enumerate(names):
                tf, ghz = mfma_calib(mix, rnd)
                print(f"{name:46s} {'random' if rnd else 'constant':8s} operands: {tf:7.1f} TFLOP/s at {ghz:.2f} GHz",
                      flush=True)
        for rows in (32, 64):
            tf, us, ghz = step_calib(rows)
            print(f"tile-step skeleton, {256 // rows} wavefronts x {rows} rows, random operands: {tf:7.1f} TFLOP/s, "
                  f"{us:.3f} us per step at {ghz:.2f} GHz", flush=True)
        return 0

    if args.only_stage is not None:
        step()
        torch.cuda.synchronize()
        if args.only_stage in ("topk_batched", "compact_batched"):
            v_all, k_all, idx_all, kc_all, vc_all = make_batched(args.batched_layers)
            pk.purekv_topk_select(st_packed, c, v_all, w, h, idx_out=idx_all)
        if args.only_stage == "copy_calib":
            calib_src = torch.empty(64 << 20, dtype=torch.float32, device=dev).normal_()
            calib_dst = torch.empty_like(calib_src)
        if args.only_stage == "spearman_batched":   # 26 layers x Hkv rows of N - w scores, correlated pairs
            sp_a = torch.randn((args.batched_layers * hkv, n - w), dtype=torch.float32, device=dev)
            sp_b = 0.5 * sp_a + torch.randn_like(sp_a)
        if args.only_stage == "dense_prefill_all_rows_lse":   # the low layer on a plain plan: every row's log-sum-exp
            dense_all = pk.Plan.for_workload(wl, pk.PATTERN_DENSE)
        stages = {
            "dense_prefill_all_rows_lse": lambda: pk.purekv_st_spattn_prefill(dense_all, q0, k0, v0, out=out0, lse=lse),
            "dense_prefill": lambda: pk.purekv_st_spattn_prefill(dense, q0, k0, v0, out=out0, lse=lse),
            "importance": lambda: pk.purekv_lowlayer_importance(dense, q0, k0, lse, w, c_out=c),
            "topk_low": lambda: pk.purekv_topk_select(dense, c, v0, w, h, idx_out=idx0),
            "compact_low": lambda: pk.purekv_kv_compact(dense, k0, v0, idx0[0], cap=cap, kc=kc0, vc=vc0),
            "st_prefill": lambda: pk.purekv_st_spattn_prefill(st, q1, k1, v1, out=out1),
            "topk_high": lambda: pk.purekv_topk_select(st, c, v1, w, h, idx_out=idx1),
            "compact_high": lambda: pk.purekv_kv_compact(st, k1, v1, idx1[0], cap=cap, kc=kc1, vc=vc1),
            "append_decode": lambda: pk.purekv_decode_step(st, q_new, k_new, v_new, kc1, vc1, n_keep, out=o_dec),
            # plain device copy of a known size (256 MiB read + 256 MiB written): scale for the HBM byte counters
            "copy_calib": lambda: calib_dst.copy_(calib_src),
            "topk_batched": lambda: pk.purekv_topk_select(st_packed, c, v_all, w, h, idx_out=idx_all),
            "compact_batched": lambda: pk.purekv_kv_compact(st_packed, k_all, v_all, idx_all, kc=kc_all, vc=vc_all),
            "spearman_batched": lambda: pk.purekv_spearman(sp_a, sp_b),
        }
        one = stages[args.only_stage]
        for _ in range(args.steps):
            one()
        torch.cuda.synchronize()
        print(f"ran {args.only_stage} x {args.steps}")
        return 0

    # ---- stated, untimed clock ramp: sustained matrix work, so that the timed steps run at the clock a model's
    # prefill (hundreds of milliseconds of such kernels back to back) runs at, not at the idle clock ----
    ramp = {"what": "purekv_calib_tile_step launches (tile-step skeleton on the prefill grid), untimed, before the warm-up steps",
            "requested_ms": args.ramp_ms, "launches": 0, "ms": 0.0}
    if args.ramp_ms > 0:
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        r0.record()
        per_launch_ms, launches = 23.0, 0
        while launches * per_launch_ms < args.ramp_ms:
            pk.purekv_calib_tile_step(st, 32, 12000, calib_src)
            launches += 1
        r1.record()
        torch.cuda.synchronize()
        ramp["launches"], ramp["ms"] = launches, round(r0.elapsed_time(r1), 1)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(9)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(events[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = {name: float(np.mean([events[s][i].elapsed_time(events[s][i + 1]) for s in range(args.steps)]))
                for i, name in enumerate(STAGES)}

    # ---- the same step recorded once in a HIP graph and replayed (no events inside): launch gaps removed ----
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(10):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- back-to-back launches of single stages (no other kernel in between): per-call durations ----
    def time_calls(fn, reps=30):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    st_ms = time_calls(lambda: pk.purekv_st_spattn_prefill(st, q1, k1, v1, out=out1))
    dense_ms = time_calls(lambda: pk.purekv_st_spattn_prefill(dense, q0, k0, v0, out=out0, lse=lse), reps=10)

    # batched over the high layers (Eq. 4: every high layer scores with the same C and its own V)
    L = args.batched_layers
    v_all, k_all, idx_all, kc_all, vc_all = make_batched(L)
    topk_b_ms = time_calls(lambda: pk.purekv_topk_select(st_packed, c, v_all, w, h, idx_out=idx_all))
    comp_b_ms = time_calls(lambda: pk.purekv_kv_compact(st_packed, k_all, v_all, idx_all, kc=kc_all, vc=vc_all))
    del v_all, k_all, kc_all, vc_all

    # what the board sustains for the bare matrix instruction, constant and random operands (power limit)
    calib_const, calib_rand = mfma_calib(0, False), mfma_calib(0, True)
    calib_step = step_calib(32)

    kept_flops, mask_flops = st.kept_tile_flops(), st.mask_flops()
    dense_kept = dense.kept_tile_flops()
    st_call_ms = stage_ms["st_prefill"]           # one launch, events inside the timed steps
    st_idx = STAGES.index("st_prefill")
    st_samples = [events[s_][st_idx].elapsed_time(events[s_][st_idx + 1]) for s_ in range(args.steps)]
    st_tflops = kept_flops / (st_call_ms * 1e-3) / 1e12
    topk_bytes = (n - w) * d * 2 * hkv + (n - w) * 4 * hkv * 3 + n_keep * 4 * hkv   # V read, C read, S write+read, idx
    comp_bytes = 2 * 2 * n_keep * d * 2 * hkv + n_keep * 4 * hkv                    # K,V rows read + written, idx
    dec_bytes = 2 * (n_keep + 1) * d * 2 * hkv

    result = {
        "metric": "st_spattn_prefill_kept_tile_tflops",
        "value": round(st_tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_graph_replay": round(ms_per_step_graph, 4),
        "clock_ramp": ramp,
        "layout": layout,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_frames}f x {wl.patch_h}x{wl.patch_w} + {wl.n_text} text = {n} tokens, "
                               f"{hq}q/{hkv}kv heads, d={d}, keep ratio {args.ratio} (h={h}, w={w})",
                   "tile": f"{pk.BLOCK}-row block x {pk.BLOCK}-key block ({pk.WAVES} wavefronts of {pk.BLOCK} rows per workgroup, {pk.BK}-key tiles)", "step": "low layer (dense prefill + log-sum-exp of the window rows, importance, top-h, compaction) + "
                   "high layer (ST-SpAttn prefill, top-h, compaction, append+decode)"},
        "prefill_ms_per_layer": round(st_call_ms, 4),
        "prefill_ms_per_layer_median": round(float(np.median(st_samples)), 4),
        "prefill_ms_per_layer_min": round(float(np.min(st_samples)), 4),
        "prefill_ms_per_layer_back_to_back": round(st_ms, 4),
        "mfma_peak_frac": round(st_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "mask_tflops": round(mask_flops / (st_call_ms * 1e-3) / 1e12, 2),
        "dense_prefill_ms_per_layer": round(dense_ms, 4),
        "dense_prefill_tflops": round(dense_kept / (dense_ms * 1e-3) / 1e12, 2),
        "dense_prefill_lse": f"last {w} rows (window plan: workgroups {dense.counts()['lse_queue0']}..255 keep the exact row sum)",
        "stage_ms_in_step": {k_: round(v_, 4) for k_, v_ in stage_ms.items()},
        "per_layer_gbps": {
            "topk": round(topk_bytes / (stage_ms["topk_high"] * 1e-3) / 1e9, 1),
            "compaction": round(comp_bytes / (stage_ms["compact_high"] * 1e-3) / 1e9, 1),
            "decode": round(dec_bytes / (stage_ms["append_decode"] * 1e-3) / 1e9, 1),
        },
        "batched": {
            "layers": L,
            "topk_ms": round(topk_b_ms, 4), "topk_gbps": round(L * topk_bytes / (topk_b_ms * 1e-3) / 1e9, 1),
            "compaction_ms": round(comp_b_ms, 4),
            "compaction_gbps": round(L * comp_bytes / (comp_b_ms * 1e-3) / 1e9, 1),
            "compaction_hbm_frac": round(L * comp_bytes / (comp_b_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "topk_hbm_frac": round(L * topk_bytes / (topk_b_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        },
        "roofline": {
            "kernel": "prefill_kernel<128, ST>, one ST-SpAttn layer (split text rows are combined inside the launch)",
            "bound": "mfma", "achieved": round(st_tflops, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(st_tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": profiled_traffic_bytes(),
            "algorithmic_flops_per_launch": kept_flops, "launch_ms": round(st_call_ms, 4),
            "mfma_loop_measured": {
                "what": "register-resident v_mfma_f32_32x32x16_bf16 loop, 256 workgroups x 8 wavefronts, ~20 ms",
                "constant_operands_tflops": round(calib_const[0], 1), "constant_operands_ghz": round(calib_const[1], 2),
                "random_operands_tflops": round(calib_rand[0], 1), "random_operands_ghz": round(calib_rand[1], 2),
            },
            "tile_step_skeleton_measured": {
                "what": "both products' MFMAs + LDS fragment reads + softmax vector work + 32 KB tile loads + one barrier "
                        "per 256 rows x 64 keys, 8 wavefronts x 32 rows, random operands, nothing else",
                "tflops": round(calib_step[0], 1), "us_per_tile_step": round(calib_step[1], 3),
                "ghz": round(calib_step[2], 2),
            },
        },
        "context": "paper: 5.0x KV compression, 3.16x prefill speed-up, whole model on 1x A100 40GB (not comparable)",
    }

    if not args.no_cpu_baseline:
        # The oracle as it stands, on the host cores, for the same step the GPU line reports: the metric's kernel
        # (ST-SpAttn attention, every head and row) gives `value`; the other stages' seconds stand beside it.
        from oracle import purekv_oracle as orc
        heads = list(range(0, hq, max(1, hq // args.cpu_heads)))[:args.cpu_heads]
        qf, kf, vf = (orc.bf16_bits_to_f64(x) for x in (high.q, high.k, high.v))
        secs = {}

        def timed(name, fn):
            t0 = time.perf_counter()
            r = fn()
            secs[name] = round(time.perf_counter() - t0, 3)
            return r

        timed("st_prefill", lambda: orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, 3, heads=heads))
        t_cpu = secs["st_prefill"]
        if len(heads) == hq:   # the rest of the step (skipped when only a sample of the heads was asked for)
            ql, kl, vl = (orc.bf16_bits_to_f64(x) for x in (low.q, low.k, low.v))
            timed("dense_prefill", lambda: orc.masked_attention(ql, kl, vl, wl.n_frames, wl.patches, wl.n_text, 0))
            c_ref = timed("importance", lambda: orc.window_column_sums(ql, kl, wl.n_frames, wl.patches, wl.n_text, 0, w))
            idx_l = timed("topk_low", lambda: orc.topk_select(orc.vnorm_scores(c_ref, vl), h, n, w))
            timed("compact_low", lambda: orc.compact(low.k, low.v, idx_l))
            idx_h = timed("topk_high", lambda: orc.topk_select(orc.vnorm_scores(c_ref, vf), h, n, w))
            kr, vr = timed("compact_high", lambda: orc.compact(high.k, high.v, idx_h))
            kcat = np.concatenate([orc.bf16_bits_to_f64(kr), orc.bf16_bits_to_f64(high.k_new[0])[:, None]], 1)
            vcat = np.concatenate([orc.bf16_bits_to_f64(vr), orc.bf16_bits_to_f64(high.v_new[0])[:, None]], 1)
            timed("append_decode", lambda: orc.decode_attention(orc.bf16_bits_to_f64(high.q_new[0]), kcat, vcat))
        sample_flops = mask_flops * len(heads) / hq
        result["cpu_baseline"] = {
            "value": round(sample_flops / t_cpu / 1e12, 5), "unit": "TFLOP/s", "cores": blas_threads(),
            "kind": "oracle",
            "sample": f"ST-SpAttn attention of {len(heads)} of {hq} query heads, all {n} rows, NumPy fp64 dense "
                      f"scores under the boolean mask; flops counted on allowed pairs only; {t_cpu:.1f} s",
            "oracle_seconds_per_stage": secs,
            "oracle_seconds_whole_step": round(sum(secs.values()), 2) if len(secs) > 1 else None,
        }
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
