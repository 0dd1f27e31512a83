"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot form full attention at these sizes in test time, but rows are independent: it computes
sampled query rows exactly (all text rows, rows around every frame boundary, random video rows; two
query heads per KV group).  Importance (window rows only), top-h, compaction and decode are checked in full.
"""
import numpy as np
import pytest
import torch

import paper_2510_25600_amd as pk
from oracle import purekv_oracle as orc
from workloads import WORKLOADS, generate

from gpu_util import IMPORTANCE_REL, bits_of, check_attention, check_kept_sets, f64_of, to_dev, value_scale

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
    rows.update(r for r in (127, 128, 129, 63, 64, 65, n - 1) if r < n)
    return np.array(sorted(rows))


def sample_heads(wl):
    g = wl.group
    return sorted({kv * g for kv in range(wl.n_kv_heads)} | {kv * g + g - 1 for kv in range(wl.n_kv_heads)})


def run_layer(wl, inp, pattern_low_dense, ratios, n_random, decode_steps, seed):
    """One layer-slice: [dense pass -> C] if asked, ST prefill, select/compact per ratio, decode steps."""
    rng = np.random.default_rng(seed)
    n, w = wl.n_tokens, wl.window
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    qf, kf, vf = F64(inp.q), F64(inp.k), F64(inp.v)
    rows, heads = sample_rows(wl, n_random, rng), sample_heads(wl)
    vs = value_scale(vf)
    dense, st = pk.Plan.for_workload(wl, 0), pk.Plan.for_workload(wl, 3)

    out_d, lse = pk.purekv_st_spattn_prefill(dense, q, k, v, want_lse=True)
    c = pk.purekv_lowlayer_importance(dense, q, k, lse, w)
    out_s = pk.purekv_st_spattn_prefill(st, q, k, v)
    torch.cuda.synchronize()

    for pattern, out in ((0, out_d), (3, out_s)):
        print(f"[case] {wl.name} prefill pattern {pattern}: {rows.size} rows x {len(heads)} heads", flush=True)
        ref, ref_lse = orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, pattern,
                                            rows=rows, heads=heads)
        got = f64_of(out[heads][:, torch.from_numpy(rows).cuda()])
        check_attention(got, ref, f"{wl.name}/p{pattern}", vs)
        if pattern == 0:
            got_lse = f64_of(lse[heads][:, torch.from_numpy(rows).cuda()])
            assert np.abs(got_lse - ref_lse).max() < 2e-3
    assert torch.isfinite(out_s.float()).all() and torch.isfinite(out_d.float()).all()

    c_ref = orc.window_column_sums(qf, kf, wl.n_frames, wl.patches, wl.n_text, 0, w)
    c_got = f64_of(c)
    rel = np.abs(c_got - c_ref) / np.maximum(np.abs(c_ref), 1e-12)
    assert rel.max() <= IMPORTANCE_REL, f"importance worst rel {rel.max():.3g}"
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
            check_attention(f64_of(o), orc.decode_attention(F64(inp.q_new[step]), kcat, vcat), f"decode {step}", vs)


def test_videollama2_shape_full_size():
    wl = WORKLOADS["videollama2_8f"]
    run_layer(wl, generate(wl, decode_steps=1), True, wl.ratios, 768, 1, seed=1)


def test_qwen25vl_32f_full_size_bench_configuration():
    wl = WORKLOADS["qwen25vl_32f"]
    run_layer(wl, generate(wl), True, wl.ratios, 1024, 1, seed=2)


def test_qwen25vl_64f_ratio_sweep_and_32_decode_steps():
    wl = WORKLOADS["qwen25vl_64f"]
    run_layer(wl, generate(wl), True, wl.ratios, 768, 32, seed=3)


@pytest.mark.parametrize("layer", [1, 2])
def test_qwen25vl_128f_stack_layer(layer):
    """Layers of the 128-frame stack: each layer's Q/K/V come from seed = layer index."""
    wl = WORKLOADS["qwen25vl_128f_stack"]
    run_layer(wl, generate(wl, seed=layer, decode_steps=1), True, wl.ratios, 512, 1, seed=10 + layer)
