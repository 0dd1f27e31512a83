"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The 8-frame and 32-frame shapes (the benchmark's) are compared in full: every query head, every row, dense and
ST-SpAttn.  At the 64- and 128-frame shapes the oracle computes sampled query rows exactly (rows are independent:
all text rows, rows around every frame boundary and tile edge, random video rows) for EVERY query head.  Importance
(window rows only), top-h, compaction and decode are checked in full everywhere.  Attention bounds are the stated
ones, unscaled (max-abs 2e-2, mean-abs 2e-3); only the 128-frame stack, whose frame chain inflates V to std 1.5 and
|O| to 5, uses the per-element bound of gpu_util.check_attention_wide_values.  Observed errors are printed.
"""
import numpy as np
import pytest
import torch

import paper_2510_25600_amd as pk
from oracle import purekv_oracle as orc
from workloads import WORKLOADS, generate

from gpu_util import (IMPORTANCE_REL, bits_of, check_attention, check_attention_wide_values, check_kept_sets, f64_of,
                      to_dev)

pytestmark = pytest.mark.gpu
F64 = orc.bf16_bits_to_f64


def sample_rows(wl, n_random, rng):
    P, nv, n = wl.patches, wl.n_video, wl.n_tokens
    rows = set(range(nv, n))                                   # every text row
    for f in range(1, wl.n_frames + 1):                        # around every frame boundary
        rows.update(r for r in (f * P - 2, f * P - 1, f * P, f * P + 1) if 0 <= r < n)
    rows.update(range(0, 3))
    rows.update(int(r) for r in rng.integers(0, nv, size=n_random))
    # rows at query-tile and key-tile edges
    rows.update(r for r in (127, 128, 129, 63, 64, 65, 31, 32, 33, n - 1) if r < n)
    return np.array(sorted(rows))


def compare_attention(wl, qf, kf, vf, pattern, out, lse, rows, what, wide=False, lse_row0=0):
    """All query heads, KV group by KV group (bounds the oracle's memory); rows = None: every row; the log-sum-exp
    is compared on the rows from lse_row0 on (a window plan writes no others)."""
    g = wl.group
    worst, total, count = 0.0, 0.0, 0
    v_absmax = float(np.abs(vf).max())
    sel = slice(None) if rows is None else torch.from_numpy(rows).cuda()
    for kv in range(wl.n_kv_heads):
        heads = list(range(kv * g, (kv + 1) * g))
        ref, ref_lse = orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, pattern, rows=rows,
                                            heads=heads)
        got = f64_of(out[heads][:, sel])
        if wide:
            mx, mean = check_attention_wide_values(got, ref, v_absmax, f"{what} heads {heads[0]}..{heads[-1]}")
        else:
            mx, mean = check_attention(got, ref, f"{what} heads {heads[0]}..{heads[-1]}")
        worst, total, count = max(worst, mx), total + mean * got.size, count + got.size
        if lse is not None:
            has = (np.arange(wl.n_tokens) if rows is None else rows) >= lse_row0
            assert has.sum() >= min(wl.window, 32)
            assert np.abs(f64_of(lse[heads][:, sel])[:, has] - ref_lse[:, has]).max() < 2e-3
    print(f"[observed] {what}: {count // wl.head_dim} (head, row) pairs, max abs err {worst:.5f}, "
          f"mean abs err {total / count:.6f}", flush=True)


def run_layer(wl, inp, ratios, n_random, decode_steps, seed, full=False, wide=False):
    """One layer-slice: dense pass -> C, ST prefill, select/compact per ratio, decode steps."""
    rng = np.random.default_rng(seed)
    n, w = wl.n_tokens, wl.window
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    qf, kf, vf = F64(inp.q), F64(inp.k), F64(inp.v)
    rows = None if full else sample_rows(wl, n_random, rng)
    # the low layer as the benchmark runs it: a window plan (the log-sum-exp of the recent window only)
    dense, st = pk.Plan.for_workload(wl, 0, lse_window=w), pk.Plan.for_workload(wl, 3)
    print(f"[case] {wl.name} low-layer plan: workgroups {dense.counts()['lse_queue0']}.. keep the exact row sum", flush=True)

    out_d, lse = pk.purekv_st_spattn_prefill(dense, q, k, v, want_lse=True)
    c = pk.purekv_lowlayer_importance(dense, q, k, lse, w)
    out_s = pk.purekv_st_spattn_prefill(st, q, k, v)
    torch.cuda.synchronize()

    for pattern, out in ((0, out_d), (3, out_s)):
        print(f"[case] {wl.name} prefill pattern {pattern}: {'all' if rows is None else rows.size} rows x "
              f"{wl.n_q_heads} heads", flush=True)
        compare_attention(wl, qf, kf, vf, pattern, out, lse if pattern == 0 else None, rows,
                          f"{wl.name} pattern {pattern}", wide, lse_row0=n - w)
    assert torch.isfinite(out_s.float()).all() and torch.isfinite(out_d.float()).all()

    c_ref = orc.window_column_sums(qf, kf, wl.n_frames, wl.patches, wl.n_text, 0, w)
    c_got = f64_of(c)
    rel = np.abs(c_got - c_ref) / np.maximum(np.abs(c_ref), 1e-12)
    assert rel.max() <= IMPORTANCE_REL, f"importance worst rel {rel.max():.3g}"
    print(f"[observed] {wl.name} importance: worst rel err {rel.max():.3g}", flush=True)
    # mass conservation at full size: window rows spread w*G probability over all keys
    assert np.all(c_got.sum(1) <= w * wl.group * (1 + 1e-4))

    s_ref = orc.vnorm_scores(c_ref, vf)
    for ratio in ratios:
        h = pk.purekv_budget(n, w, ratio)
        assert h == orc.budget(n, w, ratio)
        idx, s = pk.purekv_topk_select(st, c, v, w, h, want_scores=True)
        kc, vc = pk.purekv_kv_compact(st, k, v, idx, cap=h + w + decode_steps)
        torch.cuda.synchronize()
        idx_g = idx.cpu().numpy()
        assert np.abs(f64_of(s) - s_ref).max() <= 1e-3 * np.abs(s_ref).max()
        mism = check_kept_sets(idx_g, orc.topk_select(s_ref, h, n, w), s_ref, h)
        print(f"[case] {wl.name} ratio {ratio}: h={h}, {mism} keys inside the tie band differ", flush=True)
        kr, vr = orc.compact(inp.k, inp.v, idx_g)
        assert np.array_equal(bits_of(kc)[:, :h + w], kr) and np.array_equal(bits_of(vc)[:, :h + w], vr)
        # decode steps: the cache grows by the new token each step
        kcat, vcat = F64(kr), F64(vr)
        n_c = h + w
        for step in range(decode_steps):
            n_c = pk.purekv_kv_append(st, to_dev(inp.k_new[step]), to_dev(inp.v_new[step]), kc, vc, n_c)
            o = pk.purekv_decode_attn(st, to_dev(inp.q_new[step]), kc, vc, n_c)
            kcat = np.concatenate([kcat, F64(inp.k_new[step])[:, None]], 1)
            vcat = np.concatenate([vcat, F64(inp.v_new[step])[:, None]], 1)
            ref = orc.decode_attention(F64(inp.q_new[step]), kcat, vcat)
            if wide:
                check_attention_wide_values(f64_of(o), ref, float(np.abs(vf).max()), f"decode {step}")
            else:
                check_attention(f64_of(o), ref, f"decode {step}")


def test_videollama2_shape_full_size_every_head_every_row():
    wl = WORKLOADS["videollama2_8f"]
    run_layer(wl, generate(wl, decode_steps=1), wl.ratios, 0, 1, seed=1, full=True)


def test_qwen25vl_32f_full_size_bench_configuration_every_head_every_row():
    wl = WORKLOADS["qwen25vl_32f"]
    run_layer(wl, generate(wl), wl.ratios, 0, 1, seed=2, full=True)


def test_qwen25vl_64f_ratio_sweep_and_32_decode_steps():
    wl = WORKLOADS["qwen25vl_64f"]
    run_layer(wl, generate(wl), wl.ratios, 768, 32, seed=3)


@pytest.mark.parametrize("layer", [1, 2])
def test_qwen25vl_128f_stack_layer(layer):
    """Layers of the 128-frame stack: each layer's Q/K/V come from seed = layer index."""
    wl = WORKLOADS["qwen25vl_128f_stack"]
    run_layer(wl, generate(wl, seed=layer, decode_steps=1), wl.ratios, 512, 1, seed=10 + layer, wide=True)


def test_qwen25vl_128f_whole_stack_through_the_stack_entry_points(capsys):
    """The 128-frame configuration as what it is, a stack: 28 layers (layer l from seed l) through
    purekv_stack_layer, then ONE purekv_stack_select_compact.  Layers 0-1 dense, their column sums compared in
    full; attention of layers 0, 1, 2 and 27 on sampled rows for every head; kept sets and compact K/V of all 28
    layers (layer 0 with its own C, layers 1-27 with layer 1's C and their own V)."""
    wl = WORKLOADS["qwen25vl_128f_stack"]
    n, w, hq, hkv, d = wl.n_tokens, wl.window, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    L, st_layer = wl.n_layers, wl.n_dense_layers
    clie = st_layer - 1
    h = pk.purekv_budget(n, w, 0.2)
    check_layers = (0, 1, 2, L - 1)
    rows = sample_rows(wl, 256, np.random.default_rng(5))
    rows_dev = torch.from_numpy(rows).cuda()

    def say(msg):
        with capsys.disabled():
            print(f"[stack] {msg}", flush=True)

    dense, st = pk.Plan.for_workload(wl, 0, lse_window=w), pk.Plan.for_workload(wl, 3)
    stack = pk.Stack(L, clie, st_layer, w, h)
    k_all = torch.empty((L, hkv, n, d), dtype=torch.bfloat16, device="cuda")
    v_all = torch.empty_like(k_all)
    out = torch.empty((hq, n, d), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((hq, n), dtype=torch.float32, device="cuda")
    c_all = torch.full((clie + 1, hkv, n - w), float("nan"), dtype=torch.float32, device="cuda")
    k_bits, v_bits, q_bits, got_rows = [], [], {}, {}
    for l in range(L):
        inp = generate(wl, seed=l, decode_steps=0)
        k_bits.append(inp.k)
        v_bits.append(inp.v)
        k_all[l].copy_(to_dev(inp.k))
        v_all[l].copy_(to_dev(inp.v))
        pk.purekv_stack_layer(dense, st, stack, l, to_dev(inp.q), k_all[l], v_all[l], out, lse, c_all)
        if l in check_layers:
            q_bits[l] = inp.q
            got_rows[l] = f64_of(out[:, rows_dev])
        torch.cuda.synchronize()
        if l % 4 == 3:
            say(f"layers 0..{l} run")
    idx_all = torch.empty((L, hkv, h + w), dtype=torch.int32, device="cuda")
    kc_all = torch.zeros((L, hkv, h + w, d), dtype=torch.bfloat16, device="cuda")
    vc_all = torch.zeros_like(kc_all)
    pk.purekv_stack_select_compact(dense, st, stack, c_all, k_all, v_all, idx_all, kc_all, vc_all)
    torch.cuda.synchronize()
    say("selection and compaction of all layers done")

    # column sums of the dense layers, in full
    c_ref = []
    for l in range(clie + 1):
        c_ref.append(orc.window_column_sums(F64(q_bits[l]), F64(k_bits[l]), wl.n_frames, wl.patches, wl.n_text, 0, w))
        rel = np.abs(f64_of(c_all[l]) - c_ref[l]) / np.maximum(np.abs(c_ref[l]), 1e-12)
        assert rel.max() <= IMPORTANCE_REL, f"layer {l}: importance worst rel {rel.max():.3g}"
        say(f"layer {l} column sums: worst rel err {rel.max():.3g}")
    # attention of the sampled layers, every head, sampled rows
    for l in check_layers:
        qf, kf, vf = F64(q_bits[l]), F64(k_bits[l]), F64(v_bits[l])
        pattern = orc.stack_pattern(l, st_layer)
        v_absmax, worst, total = float(np.abs(vf).max()), 0.0, 0.0
        for kv in range(hkv):
            heads = list(range(kv * wl.group, (kv + 1) * wl.group))
            ref, _ = orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, pattern, rows=rows, heads=heads)
            mx, mean = check_attention_wide_values(got_rows[l][heads], ref, v_absmax, f"stack layer {l} kv {kv}")
            worst, total = max(worst, mx), total + mean / hkv
        say(f"layer {l} (pattern {pattern}) attention on {rows.size} rows x {hq} heads: max abs err {worst:.5f}, "
            f"mean abs err {total:.6f}")
        del qf, kf, vf
    # kept sets and compact cache of every layer
    idx_g = idx_all.cpu().numpy()
    differing = 0
    for l in range(L):
        s_ref = orc.vnorm_scores(c_ref[min(l, clie)], F64(v_bits[l]))
        differing += check_kept_sets(idx_g[l], orc.topk_select(s_ref, h, n, w), s_ref, h)
        kr, vr = orc.compact(k_bits[l], v_bits[l], idx_g[l])
        assert np.array_equal(bits_of(kc_all[l]), kr) and np.array_equal(bits_of(vc_all[l]), vr), f"layer {l}"
        if l % 7 == 6:
            say(f"kept sets and compact K/V of layers 0..{l} equal the oracle's ({differing} keys inside the tie band)")
