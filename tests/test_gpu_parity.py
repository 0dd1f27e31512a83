"""GPU parity: every C-ABI compute call against the CPU oracle on the same seeded bf16 bits.

Tolerances (written here, derived in the design notes): attention max-abs 2e-2 / mean-abs 2e-3;
column sums relative 1e-3; kept-index sets exact outside a 1e-5 band around the h-th score;
compacted K/V bit-exact given the indices.
"""
import math

import ctypes

import numpy as np
import pytest
import torch

import paper_2510_25600_amd as pk
from oracle import purekv_oracle as orc
from workloads import WORKLOADS, generate, small_variant

from gpu_util import (IMPORTANCE_REL, SCORE_BAND, bits_of, check_attention, check_kept_sets, f64_of, to_dev)

pytestmark = pytest.mark.gpu

F64 = orc.bf16_bits_to_f64

SMALL = {
    "tiny_4f": WORKLOADS["tiny_4f"],
    # ragged everywhere: P = 35 (no tile alignment), N = 124 < one query tile, d = 64
    "ragged_3f": small_variant("ragged_3f"),
    # query tiles straddle frame boundaries (P = 576 = 4.5 tiles), GQA 4:1, d = 128, one ragged tail tile
    "straddle_3f": small_variant("straddle_3f", n_frames=3, patch_h=24, patch_w=24, n_text=70, n_q_heads=4,
                                 n_kv_heads=1, head_dim=128),
    # no text at all, single KV head per query head
    "notext_5f": small_variant("notext_5f", n_frames=5, patch_h=8, patch_w=8, n_text=0, n_q_heads=2, n_kv_heads=2,
                               head_dim=128),
    # long text tail so that the text rows' key lists are split across work items and merged
    "longtext_2f": small_variant("longtext_2f", n_frames=2, patch_h=16, patch_w=16, n_text=2100, n_q_heads=2,
                                 n_kv_heads=1, head_dim=128),
    # workgroup shapes of the planner: 7 stacked heads x 1 row block (one wavefront idle), split text rows
    "heads7_3f": small_variant("heads7_3f", n_frames=3, patch_h=10, patch_w=10, n_text=900, n_q_heads=7,
                               n_kv_heads=1, head_dim=128),
    # 3 stacked heads x 2 row blocks (six wavefronts), two KV heads, P = 99 straddles row blocks and key halves
    "heads3_4f": small_variant("heads3_4f", n_frames=4, patch_h=9, patch_w=11, n_text=45, n_q_heads=6,
                               n_kv_heads=2, head_dim=64),
    # 12 query heads per KV head: two groups of 6 stacked heads
    "heads12_2f": small_variant("heads12_2f", n_frames=2, patch_h=12, patch_w=12, n_text=33, n_q_heads=12,
                                n_kv_heads=1, head_dim=128),
    # More units than workgroups, so that queues hold several units and every unit switch (output of the finished
    # unit, query prefetch, state reset) is compared exhaustively, not on sampled rows as in the full-size tests:
    # 7 stacked heads x 1 row block, P = 272 straddles key tiles (91 query tiles x 6 head groups: up to three units a queue)
    "manyunits_g7": small_variant("manyunits_g7", n_frames=10, patch_h=16, patch_w=17, n_text=190, n_q_heads=42,
                                  n_kv_heads=6, head_dim=128),
    # 2 stacked heads x 4 row blocks (18 query tiles x 16 head groups), d = 64
    "manyunits_g2": small_variant("manyunits_g2", n_frames=7, patch_h=15, patch_w=20, n_text=120, n_q_heads=32,
                                  n_kv_heads=16, head_dim=64),
    # one head x 8 row blocks (5 query tiles x 64 heads), d = 64
    "manyunits_g1": small_variant("manyunits_g1", n_frames=4, patch_h=16, patch_w=16, n_text=100, n_q_heads=64,
                                  n_kv_heads=64, head_dim=64),
    # degenerate shapes: a single frame (first frame = own frame, no previous one), one patch per frame (every
    # video key is its frame's only key), a single token, and a lone video token in front of a text
    "oneframe_1f": small_variant("oneframe_1f", n_frames=1, patch_h=6, patch_w=6, n_text=10, n_q_heads=4,
                                 n_kv_heads=2, head_dim=128),
    "onepatch_9f": small_variant("onepatch_9f", n_frames=9, patch_h=1, patch_w=1, n_text=3, n_q_heads=2,
                                 n_kv_heads=1, head_dim=64),
    "single_token": small_variant("single_token", n_frames=1, patch_h=1, patch_w=1, n_text=0, n_q_heads=3,
                                  n_kv_heads=3, head_dim=128),
    "mostly_text": small_variant("mostly_text", n_frames=1, patch_h=1, patch_w=1, n_text=200, n_q_heads=8,
                                 n_kv_heads=1, head_dim=64),
}


def _plan(wl, pattern):
    return pk.Plan.for_workload(wl, pattern)


@pytest.mark.parametrize("pattern", [0, 1, 2, 3])
@pytest.mark.parametrize("name", list(SMALL))
def test_prefill_matches_oracle(name, pattern):
    wl = SMALL[name]
    inp = generate(wl, seed=11)
    print(f"[case] prefill {name} pattern={pattern} N={wl.n_tokens}", flush=True)
    plan = _plan(wl, pattern)
    out, lse = pk.purekv_st_spattn_prefill(plan, to_dev(inp.q), to_dev(inp.k), to_dev(inp.v), want_lse=True)
    torch.cuda.synchronize()
    ref, ref_lse = orc.masked_attention(F64(inp.q), F64(inp.k), F64(inp.v), wl.n_frames, wl.patches, wl.n_text,
                                        pattern)
    check_attention(f64_of(out), ref, f"{name}/p{pattern}")
    assert np.abs(f64_of(lse) - ref_lse).max() < 2e-3
    if name == "longtext_2f":
        assert plan.counts()["n_split_qtiles"] > 0  # the merge path ran
    if name.startswith("manyunits"):
        c = plan.counts()
        assert max(len(plan.queue(g)) for g in range(c["n_workgroups"])) >= 2  # some queue switches units


@pytest.mark.parametrize("pattern", [0, 3])
@pytest.mark.parametrize("name,w", [("manyunits_g7", 190), ("manyunits_g7", 37), ("manyunits_g2", 120), ("manyunits_g2", 1),
                                    ("manyunits_g1", 100), ("manyunits_g1", 300), ("tiny_4f", 32), ("longtext_2f", 64)])
def test_window_plan_prefill_and_importance(name, w, pattern):
    """A window plan: outputs as for any plan; the log-sum-exp of the last w rows only, every other element of the
    buffer untouched; the importance read from it.  The larger shapes have more units than workgroups, so their
    plans are divided and the kernel with both copies of the tile loop runs."""
    wl = SMALL[name]
    inp = generate(wl, seed=21)
    n = wl.n_tokens
    print(f"[case] window plan {name} pattern={pattern} w={w} N={n}", flush=True)
    plan = pk.Plan.for_workload(wl, pattern, lse_window=w)
    c = plan.counts()
    # these are the cases meant to exercise the divided kernel, at both head dimensions (the planner leaves a plan whole
    # when the window's tiles are more than a quarter of the work, or when there are fewer units than workgroups)
    if (name, w, pattern) in {("manyunits_g7", 37, 0), ("manyunits_g7", 37, 3), ("manyunits_g2", 120, 0),
                              ("manyunits_g2", 1, 0), ("manyunits_g2", 1, 3)}:
        assert c["lse_queue0"] > 0, "this case is meant to exercise the divided kernel"
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    sentinel = -12345.0
    lse = torch.full((wl.n_q_heads, n), sentinel, dtype=torch.float32, device="cuda")
    out, _ = pk.purekv_st_spattn_prefill(plan, q, k, v, lse=lse)
    torch.cuda.synchronize()
    qf, kf, vf = F64(inp.q), F64(inp.k), F64(inp.v)
    ref, ref_lse = orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, pattern)
    check_attention(f64_of(out), ref, f"window {name}/p{pattern}/w{w}")
    got_lse = f64_of(lse)
    assert np.all(got_lse[:, :n - w] == sentinel), "rows before the window were written"
    assert np.abs(got_lse[:, n - w:] - ref_lse[:, n - w:]).max() < 2e-3
    # the same call without the log-sum-exp, and again with it: same output bits (the division changes who runs what,
    # never what is computed for a row)
    out2 = pk.purekv_st_spattn_prefill(plan, q, k, v)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out), bits_of(out2))
    cs = pk.purekv_lowlayer_importance(plan, q, k, lse, w)
    torch.cuda.synchronize()
    ref_c = orc.window_column_sums(qf, kf, wl.n_frames, wl.patches, wl.n_text, pattern, w)
    got_c = f64_of(cs)
    if ref_c.size:
        assert np.all(np.abs(got_c - ref_c) <= IMPORTANCE_REL * np.maximum(np.abs(ref_c), 1e-12))
    # a window wider than the plan's is refused: those rows of lse were never written
    if w < n:
        with pytest.raises(pk.PureKVError) as e:
            pk.purekv_lowlayer_importance(plan, q, k, lse, w + 1)
        assert e.value.status == pk.EINVAL
    # the V norms asked for together with the window's log-sum-exp come from their own pass: same values
    vn = torch.zeros((wl.n_kv_heads, n), dtype=torch.float32, device="cuda")
    lse3 = torch.full_like(lse, sentinel)
    out3, _ = pk.purekv_st_spattn_prefill(plan, q, k, v, lse=lse3, vnorm2=vn)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out), bits_of(out3)) and torch.equal(lse, lse3)
    ref_vn = (vf * vf).sum(-1)
    assert np.abs(f64_of(vn) - ref_vn).max() <= 2e-6 * max(1.0, ref_vn.max())


def test_prefill_is_deterministic_and_output_buffer_reuse():
    wl = SMALL["straddle_3f"]
    inp = generate(wl, seed=3)
    plan = _plan(wl, 3)
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    a = pk.purekv_st_spattn_prefill(plan, q, k, v)
    b = torch.full_like(a, float("nan"))
    pk.purekv_st_spattn_prefill(plan, q, k, v, out=b)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(a), bits_of(b))


def test_prefill_custom_scale():
    wl = SMALL["ragged_3f"]
    inp = generate(wl, seed=5)
    plan = pk.Plan(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, 3, 0.05)
    out = pk.purekv_st_spattn_prefill(plan, to_dev(inp.q), to_dev(inp.k), to_dev(inp.v))
    ref, _ = orc.masked_attention(F64(inp.q), F64(inp.k), F64(inp.v), wl.n_frames, wl.patches, wl.n_text, 3,
                                  scale=float(np.float32(0.05)))
    check_attention(f64_of(out), ref, "custom scale")


@pytest.mark.parametrize("name,pattern,w", [
    ("tiny_4f", 0, 32), ("tiny_4f", 3, 32), ("tiny_4f", 3, 100), ("tiny_4f", 2, 200), ("tiny_4f", 0, 288),
    ("ragged_3f", 3, 19), ("ragged_3f", 1, 50), ("straddle_3f", 3, 70), ("straddle_3f", 0, 700),
    ("notext_5f", 3, 33), ("longtext_2f", 0, 2100),
    ("oneframe_1f", 3, 10), ("oneframe_1f", 3, 30), ("oneframe_1f", 2, 46), ("onepatch_9f", 3, 5), ("onepatch_9f", 1, 12),
    ("single_token", 3, 1), ("mostly_text", 3, 64), ("mostly_text", 3, 201), ("heads7_3f", 3, 900), ("heads3_4f", 2, 150),
])
def test_importance_matches_oracle(name, pattern, w):
    wl = SMALL[name]
    inp = generate(wl, seed=12)
    print(f"[case] importance {name} pattern={pattern} w={w}", flush=True)
    plan = _plan(wl, pattern)
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    _, lse = pk.purekv_st_spattn_prefill(plan, q, k, v, want_lse=True)
    c = pk.purekv_lowlayer_importance(plan, q, k, lse, w)
    torch.cuda.synchronize()
    ref = orc.window_column_sums(F64(inp.q), F64(inp.k), wl.n_frames, wl.patches, wl.n_text, pattern, w)
    got = f64_of(c)
    assert got.shape == ref.shape
    if ref.size:
        assert np.all(np.abs(got - ref) <= IMPORTANCE_REL * np.maximum(np.abs(ref), 1e-12)), \
            f"worst rel {np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-12)):.3g}"
    # masked-out pairs contribute exactly nothing: a column no window row can see is exactly 0
    assert np.all(got[ref == 0] == 0)


@pytest.mark.parametrize("n_keys,h", [(256, 25), (256, 0), (256, 256), (1000, 1), (5000, 999), (40000, 8000)])
def test_topk_exact_on_given_scores(n_keys, h):
    """Stage-isolated: identical fp32 scores on both sides, so the kept sets must be identical (ties included)."""
    w = 16
    n = n_keys + w
    plan = pk.Plan(1, 1, n_keys, w, 3, 3, 64, 0)  # geometry only carries N and Hkv here
    rng = np.random.default_rng(n_keys + h)
    s = rng.random((3, n_keys)).astype(np.float32)
    s[1] = np.round(s[1] * 8) / 8                 # heavy ties
    s[2, ::3] = 0.0                               # zeros, some negative zero
    s[2, 3::6] = -0.0
    idx = pk.purekv_topk_select(plan, torch.from_numpy(s).cuda(), None, w, h)
    torch.cuda.synchronize()
    ref = orc.topk_select(s.astype(np.float64), h, n, w)
    assert np.array_equal(idx.cpu().numpy(), ref)


@pytest.mark.parametrize("n_keys", [8192, 8193, 16384, 20000, 32768, 32769, 50001])
def test_topk_row_lengths_across_kernel_variants(n_keys):
    """Row lengths on both sides of every switch between the register-resident variants (8, 16, 32 scores per
    thread) and the streaming variant of the selection kernel; heavy ties in one head."""
    w = 8
    plan = pk.Plan(1, 1, n_keys, w, 2, 2, 64, 0)
    rng = np.random.default_rng(n_keys)
    s = rng.random((2, n_keys)).astype(np.float32)
    s[1] = np.round(s[1] * 16) / 16
    for h in (1, n_keys // 5, n_keys):
        idx = pk.purekv_topk_select(plan, torch.from_numpy(s).cuda(), None, w, h)
        ref = orc.topk_select(s.astype(np.float64), h, n_keys + w, w)
        assert np.array_equal(idx.cpu().numpy(), ref), (n_keys, h)


def test_topk_negative_and_mixed_scores():
    w, n_keys = 8, 3000
    plan = pk.Plan(1, 1, n_keys, w, 2, 2, 64, 0)
    rng = np.random.default_rng(9)
    s = rng.standard_normal((2, n_keys)).astype(np.float32)
    s[1] = -np.abs(s[1])
    for h in (1, 500, 2999):
        idx = pk.purekv_topk_select(plan, torch.from_numpy(s).cuda(), None, w, h)
        ref = orc.topk_select(s.astype(np.float64), h, n_keys + w, w)
        assert np.array_equal(idx.cpu().numpy(), ref)


@pytest.mark.parametrize("name", ["tiny_4f", "ragged_3f", "straddle_3f"])
def test_vnorm_scores_and_selection_layers(name):
    """Eq. 3 / Eq. 4: several layers' V share one C; scores within fp32 rounding, kept sets exact outside the band."""
    wl = SMALL[name]
    n, w = wl.n_tokens, wl.window
    h = max(1, orc.budget(n, w, 0.3))
    layers = [generate(wl, seed=20 + l) for l in range(3)]
    rng = np.random.default_rng(1)
    c = rng.random((wl.n_kv_heads, n - w)).astype(np.float32)
    plan = _plan(wl, 3)
    v_all = torch.stack([to_dev(x.v) for x in layers])
    idx, s = pk.purekv_topk_select(plan, torch.from_numpy(c).cuda(), v_all, w, h, want_scores=True)
    idx2 = pk.purekv_topk_select(plan, torch.from_numpy(c).cuda(), v_all, w, h)  # workspace path
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), idx2.cpu().numpy())
    for l, x in enumerate(layers):
        s_ref = orc.vnorm_scores(c.astype(np.float64), F64(x.v))
        assert np.all(np.abs(f64_of(s[l]) - s_ref) <= 2e-6 * np.abs(s_ref) + 1e-30)
        check_kept_sets(idx[l].cpu().numpy(), orc.topk_select(s_ref, h, n, w), s_ref, h)


@pytest.mark.parametrize("name", ["tiny_4f", "ragged_3f", "straddle_3f"])
def test_compaction_bit_exact_and_append(name):
    wl = SMALL[name]
    n, w = wl.n_tokens, wl.window
    h = orc.budget(n, w, 0.4)
    layers = [generate(wl, seed=30 + l) for l in range(2)]
    rng = np.random.default_rng(2)
    idx = np.stack([orc.topk_select(rng.random((wl.n_kv_heads, n - w)), h, n, w) for _ in layers])
    plan = _plan(wl, 3)
    k_all = torch.stack([to_dev(x.k) for x in layers])
    v_all = torch.stack([to_dev(x.v) for x in layers])
    cap = h + w + 3
    kc = torch.zeros((2, wl.n_kv_heads, cap, wl.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    pk.purekv_kv_compact(plan, k_all, v_all, torch.from_numpy(idx).cuda(), cap=cap, kc=kc, vc=vc)
    torch.cuda.synchronize()
    for l, x in enumerate(layers):
        kr, vr = orc.compact(x.k, x.v, idx[l])
        assert np.array_equal(bits_of(kc[l])[:, :h + w], kr) and np.array_equal(bits_of(vc[l])[:, :h + w], vr)
        assert not bits_of(kc[l])[:, h + w:].any()  # rows beyond n_keep untouched
    # append one decoded token to layer 0's cache
    x = layers[0]
    n1 = pk.purekv_kv_append(plan, to_dev(x.k_new[0]) if x.k_new.shape[0] else to_dev(x.k[:, 0]),
                             to_dev(x.v_new[0]) if x.v_new.shape[0] else to_dev(x.v[:, 0]), kc[0], vc[0], h + w)
    torch.cuda.synchronize()
    assert n1 == h + w + 1
    src = x.k_new[0] if x.k_new.shape[0] else x.k[:, 0]
    assert np.array_equal(bits_of(kc[0])[:, h + w], src)


@pytest.mark.parametrize("hq,hkv,d,n_cached", [(2, 1, 64, 57), (28, 4, 128, 1690), (32, 8, 128, 948), (12, 1, 128, 5),
                                               (4, 4, 64, 1), (9, 3, 128, 333), (40, 2, 128, 300), (34, 2, 64, 129),
                                               (28, 4, 128, 128), (28, 4, 128, 6800), (4, 1, 64, 17000), (6, 2, 128, 33000)])
def test_decode_matches_oracle(hq, hkv, d, n_cached):
    rng = np.random.default_rng(n_cached)
    from workloads import f32_to_bf16_bits
    q = f32_to_bf16_bits(rng.standard_normal((hq, d)).astype(np.float32))
    cap = n_cached + 7
    kc = f32_to_bf16_bits(rng.standard_normal((hkv, cap, d)).astype(np.float32))
    vc = f32_to_bf16_bits(rng.standard_normal((hkv, cap, d)).astype(np.float32))
    plan = pk.Plan(1, 4, 4, 4, hq, hkv, d, 3)
    out = pk.purekv_decode_attn(plan, to_dev(q), to_dev(kc), to_dev(vc), n_cached)
    torch.cuda.synchronize()
    ref = orc.decode_attention(F64(q), F64(kc)[:, :n_cached], F64(vc)[:, :n_cached])
    check_attention(f64_of(out), ref, "decode")


@pytest.mark.parametrize("hq,hkv,d,n0,steps", [(28, 4, 128, 1689, 3), (40, 2, 64, 126, 5), (8, 8, 128, 0, 3),
                                               (12, 3, 128, 255, 3)])
def test_decode_step_appends_and_attends(hq, hkv, d, n0, steps):
    """The fused step = append + attention: the cache must equal the one the separate append call builds, bit for
    bit, the output must match the oracle on the grown cache, and consecutive calls (the arrival counters reset
    themselves) must keep doing so, also across a 256-key chunk boundary."""
    from workloads import f32_to_bf16_bits
    rng = np.random.default_rng(1000 * hq + n0)
    bits = lambda *shape: f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))  # noqa: E731
    cap = n0 + steps + 2
    kc_h, vc_h = bits(hkv, cap, d), bits(hkv, cap, d)
    kc, vc = to_dev(kc_h), to_dev(vc_h)           # fused path
    kc2, vc2 = to_dev(kc_h), to_dev(vc_h)         # separate append + attention
    plan = pk.Plan(1, 4, 4, 4, hq, hkv, d, 3)
    for t in range(steps):
        q, kn, vn = bits(hq, d), bits(hkv, d), bits(hkv, d)
        n = n0 + t
        out = pk.purekv_decode_step(plan, to_dev(q), to_dev(kn), to_dev(vn), kc, vc, n)
        pk.purekv_kv_append(plan, to_dev(kn), to_dev(vn), kc2, vc2, n)
        out2 = pk.purekv_decode_attn(plan, to_dev(q), kc2, vc2, n + 1)
        torch.cuda.synchronize()
        kc_h[:, n], vc_h[:, n] = kn, vn
        assert np.array_equal(bits_of(kc)[:, :n + 1], kc_h[:, :n + 1]) and np.array_equal(bits_of(kc), bits_of(kc2))
        assert np.array_equal(bits_of(vc)[:, :n + 1], vc_h[:, :n + 1]) and np.array_equal(bits_of(vc), bits_of(vc2))
        assert np.array_equal(bits_of(out), bits_of(out2))   # same kernel, same order of operations
        ref = orc.decode_attention(F64(q), F64(kc_h)[:, :n + 1], F64(vc_h)[:, :n + 1])
        check_attention(f64_of(out), ref, f"decode step {t}")


def test_tiny_config_end_to_end_chain():
    """Config 1: importance from the dense pass, ST-SpAttn prefill, V-norm top-h at ratio 0.2, compaction, one
    decode step -- every stage fed by the GPU's own previous stage and compared with the oracle's chain."""
    wl = WORKLOADS["tiny_4f"]
    inp = generate(wl)
    n, w = wl.n_tokens, wl.window
    h = pk.purekv_budget(n, w, 0.2)
    assert h == orc.budget(n, w, 0.2) == 25
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    dense, st = _plan(wl, 0), _plan(wl, 3)
    _, lse = pk.purekv_st_spattn_prefill(dense, q, k, v, want_lse=True)
    c = pk.purekv_lowlayer_importance(dense, q, k, lse, w)
    out = pk.purekv_st_spattn_prefill(st, q, k, v)
    idx = pk.purekv_topk_select(st, c, v, w, h)
    kc, vc = pk.purekv_kv_compact(st, k, v, idx, cap=h + w + 1)
    n1 = pk.purekv_kv_append(st, to_dev(inp.k_new[0]), to_dev(inp.v_new[0]), kc, vc, h + w)
    o_dec = pk.purekv_decode_attn(st, to_dev(inp.q_new[0]), kc, vc, n1)
    torch.cuda.synchronize()

    qf, kf, vf = F64(inp.q), F64(inp.k), F64(inp.v)
    c_ref = orc.window_column_sums(qf, kf, wl.n_frames, wl.patches, wl.n_text, 0, w)
    s_ref = orc.vnorm_scores(c_ref, vf)
    idx_ref = orc.topk_select(s_ref, h, n, w)
    out_ref, _ = orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, 3)
    check_attention(f64_of(out), out_ref, "chain prefill")
    assert np.all(np.abs(f64_of(c) - c_ref) <= IMPORTANCE_REL * np.maximum(c_ref, 1e-12))
    idx_g = idx.cpu().numpy()
    check_kept_sets(idx_g, idx_ref, s_ref, h)
    kr, vr = orc.compact(inp.k, inp.v, idx_g)  # bit-exact given the indices the GPU chose
    assert np.array_equal(bits_of(kc)[:, :h + w], kr) and np.array_equal(bits_of(vc)[:, :h + w], vr)
    kcat = np.concatenate([F64(kr), F64(inp.k_new[0])[:, None]], 1)
    vcat = np.concatenate([F64(vr), F64(inp.v_new[0])[:, None]], 1)
    check_attention(f64_of(o_dec), orc.decode_attention(F64(inp.q_new[0]), kcat, vcat), "chain decode")


def test_gpu_argument_errors():
    wl = WORKLOADS["tiny_4f"]
    plan = _plan(wl, 3)
    inp = generate(wl)
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    lib = pk.raw()
    c = torch.zeros((1, 256), dtype=torch.float32, device="cuda")
    idx = torch.zeros((1, 57), dtype=torch.int32, device="cuda")
    P = lambda t: t.data_ptr()  # noqa: E731
    assert lib.purekv_lowlayer_importance(plan.handle, P(q), P(k), P(c), 0, P(c), None, 0, None) == pk.EINVAL
    assert lib.purekv_lowlayer_importance(plan.handle, P(q), P(k), P(c), 289, P(c), None, 0, None) == pk.EINVAL
    assert lib.purekv_topk_select(plan.handle, P(c), None, 0, 1, 32, 257, P(idx), None, None, 0, None) == pk.EINVAL
    assert lib.purekv_topk_select(plan.handle, P(c), P(v), 0, 1, 32, 25, P(idx), None, None, 0, None) == pk.EWORKSPACE
    assert lib.purekv_topk_select(plan.handle, P(c), None, 0, 2, 32, 25, P(idx), None, None, 0, None) == pk.EINVAL
    assert lib.purekv_kv_compact(plan.handle, P(k), P(v), 0, 1, P(idx), 57, P(k), P(v), 56, None) == pk.EINVAL
    assert lib.purekv_kv_append(plan.handle, P(k), P(v), P(k), P(v), 57, 57, None) == pk.EINVAL
    assert lib.purekv_decode_attn(plan.handle, P(q), P(k), P(v), 0, 57, P(q), P(c), 1 << 20, None) == pk.EINVAL
    assert lib.purekv_decode_attn(plan.handle, P(q), P(k), P(v), 57, 57, P(q), None, 0, None) == pk.EWORKSPACE
    assert lib.purekv_decode_step(plan.handle, P(q), P(k), P(v), P(k), P(v), 57, 57, P(q), P(c), 1 << 20, None) == pk.EINVAL
    assert lib.purekv_decode_step(plan.handle, P(q), None, P(v), P(k), P(v), 5, 57, P(q), P(c), 1 << 20, None) == pk.EINVAL
    assert lib.purekv_decode_step(plan.handle, P(q), P(k), P(v), P(k), P(v), 5, 57, P(q), None, 0, None) == pk.EWORKSPACE
    dense_plan = _plan(wl, 0)
    for bad in (pk.Stack(0, 0, 1, 32, 25), pk.Stack(4, 2, 2, 32, 25), pk.Stack(4, 1, 5, 32, 25), pk.Stack(4, 1, 2, 0, 25),
                pk.Stack(4, 1, 2, 32, 257)):
        assert lib.purekv_stack_layer(dense_plan.handle, plan.handle, ctypes.byref(bad), 0, P(q), P(k), P(v), P(q), P(c),
                                      P(c), None, 0, None) == pk.EINVAL
    good = pk.Stack(4, 1, 2, 32, 25)
    args = (P(q), P(k), P(v), P(q), P(c), P(c), None, 0, None)
    assert lib.purekv_stack_layer(plan.handle, plan.handle, ctypes.byref(good), 0, *args) == pk.EINVAL   # not dense
    assert lib.purekv_stack_layer(dense_plan.handle, None, ctypes.byref(good), 3, *args) == pk.EINVAL    # needs ST plan
    assert lib.purekv_stack_layer(dense_plan.handle, plan.handle, ctypes.byref(good), 4, *args) == pk.EINVAL
    assert lib.purekv_stack_layer(dense_plan.handle, plan.handle, ctypes.byref(good), 0, P(q), P(k), P(v), P(q), None,
                                  P(c), None, 0, None) == pk.EINVAL   # a layer that emits C needs the LSE scratch
    assert lib.purekv_stack_select_compact(dense_plan.handle, plan.handle, ctypes.byref(good), P(c), P(k), P(v), 0, P(idx),
                                           P(k), P(v), 57, None, 0, None) == pk.EINVAL   # four layers need a layer stride
    assert lib.purekv_workspace_init(plan.handle, 9, None, 0, 0, 0, 0, None) == pk.EINVAL
    assert lib.purekv_workspace_init(plan.handle, pk.OP_DECODE, None, 0, 0, 0, 57, None) == pk.EWORKSPACE
    assert lib.purekv_workspace_init(plan.handle, pk.OP_COMPACT, None, 0, 0, 0, 0, None) == pk.OK   # needs none
    assert lib.purekv_calib_mfma(plan.handle, 3, 0, 10, P(c), P(c), None) == pk.EINVAL
    assert lib.purekv_calib_mfma(plan.handle, 0, 0, 0, P(c), P(c), None) == pk.EINVAL
    assert lib.purekv_calib_mfma(plan.handle, 0, 0, 10, None, P(c), None) == pk.EINVAL
    long = pk.Plan.for_workload(SMALL["longtext_2f"], 3)
    assert long.workspace_bytes(pk.OP_PREFILL) > 0
    assert lib.purekv_st_spattn_prefill(long.handle, P(q), P(k), P(v), P(q), None, None, 0, None) == pk.EWORKSPACE
    assert lib.purekv_workspace_init(long.handle, pk.OP_PREFILL, None, 0, 0, 0, 0, None) == pk.EWORKSPACE
    torch.cuda.synchronize()


@pytest.mark.gpu
@pytest.mark.parametrize("mix", [0, 1, 2])
def test_calibration_loop_runs_and_reports_its_clock(mix):
    """The board-calibration loop is not part of the method: it has to run on the plan's grid, write every sink
    element with a finite value and report a plausible shader clock."""
    plan = _plan(WORKLOADS["tiny_4f"], 3)
    n_wg = plan.counts()["n_workgroups"]
    sink = torch.full((512 * n_wg,), float("nan"), dtype=torch.float32, device="cuda")
    for rnd in (False, True):
        flops, ticks = pk.purekv_calib_mfma(plan, mix, rnd, 200, sink=sink)
        torch.cuda.synchronize()
        assert flops == 2.0 * 32 * 32 * 16 * 16 * 200 * 8 * n_wg
        assert bool(torch.isfinite(sink).all())
        cyc, ref = ticks.tolist()
        assert cyc >= 200 * 16 * 32 and ref > 0          # an MFMA of this shape holds the pipe 32 cycles
        assert 0.05 < cyc / ref / 10.0 < 3.0             # GHz


@pytest.mark.parametrize("clie,st_layer,layers", [(1, 3, 5), (0, 1, 3), (2, 3, 3)])
def test_layer_stack_matches_oracle(clie, st_layer, layers):
    """Layer stack: dense layers below st_layer, ST-SpAttn from there on; layers <= clie emit column sums, a
    layer below clie is selected with its own, the rest with layer clie's and their own V; one batched
    selection and one compaction for the whole stack.  Every layer has data of its own (seed = 40 + layer)."""
    wl = SMALL["straddle_3f"]
    n, w, hkv, d = wl.n_tokens, wl.window, wl.n_kv_heads, wl.head_dim
    h = orc.budget(n, w, 0.3)
    data = [generate(wl, seed=40 + l) for l in range(layers)]
    dense, st = _plan(wl, 0), _plan(wl, 3)
    stack = pk.Stack(layers, clie, st_layer, w, h)
    k_all = torch.stack([to_dev(x.k) for x in data])
    v_all = torch.stack([to_dev(x.v) for x in data])
    lse = torch.empty((wl.n_q_heads, n), dtype=torch.float32, device="cuda")
    c_all = torch.full((clie + 1, hkv, n - w), float("nan"), dtype=torch.float32, device="cuda")
    outs = []
    for l, x in enumerate(data):
        q = to_dev(x.q)
        outs.append(pk.purekv_stack_layer(dense, st if st_layer < layers else None, stack, l, q, k_all[l], v_all[l],
                                          torch.empty_like(q), lse, c_all))
    cap = h + w + 2
    idx_all = torch.empty((layers, hkv, h + w), dtype=torch.int32, device="cuda")
    kc_all = torch.zeros((layers, hkv, cap, d), dtype=torch.bfloat16, device="cuda")
    vc_all = torch.zeros_like(kc_all)
    pk.purekv_stack_select_compact(dense, st, stack, c_all, k_all, v_all, idx_all, kc_all, vc_all)
    torch.cuda.synchronize()

    c_ref = []
    for l, x in enumerate(data):
        qf, kf, vf = F64(x.q), F64(x.k), F64(x.v)
        pattern = orc.stack_pattern(l, st_layer)
        ref, _ = orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, pattern)
        check_attention(f64_of(outs[l]), ref, f"stack layer {l} pattern {pattern}")
        if l <= clie:
            c_ref.append(orc.window_column_sums(qf, kf, wl.n_frames, wl.patches, wl.n_text, 0, w))
            got = f64_of(c_all[l])
            assert np.all(np.abs(got - c_ref[l]) <= IMPORTANCE_REL * np.maximum(np.abs(c_ref[l]), 1e-12))
    idx_ref = orc.stack_selection(c_ref, [F64(x.v) for x in data], clie, h, n, w)
    for l, x in enumerate(data):
        s_ref = orc.vnorm_scores(c_ref[min(l, clie)], F64(x.v))
        got = idx_all[l].cpu().numpy()
        check_kept_sets(got, idx_ref[l], s_ref, h)
        kr, vr = orc.compact(x.k, x.v, got)   # compaction is a bit copy of what the GPU selected
        assert np.array_equal(bits_of(kc_all[l])[:, :h + w], kr) and np.array_equal(bits_of(vc_all[l])[:, :h + w], vr)
        assert not bits_of(kc_all[l])[:, h + w:].any()


@pytest.mark.parametrize("rows", [32, 64])
def test_tile_step_skeleton_runs(rows):
    """Second calibration loop: runs on the plan's grid, fills the sink with finite values, reports its clock,
    refuses bad arguments."""
    plan = _plan(WORKLOADS["tiny_4f"], 3)
    n_wg = plan.counts()["n_workgroups"]
    src = torch.randn(2 << 20, device="cuda").to(torch.bfloat16)   # 4 MiB
    sink = torch.full((512 * n_wg,), float("nan"), dtype=torch.float32, device="cuda")
    flops, ticks = pk.purekv_calib_tile_step(plan, rows, 50, src, sink=sink)
    torch.cuda.synchronize()
    assert flops == 4.0 * 256 * 64 * 128 * 50 * n_wg
    assert bool(torch.isfinite(sink[: (512 // (rows // 32)) * n_wg]).all())
    cyc, ref = ticks.tolist()
    assert cyc >= 50 * 32 * 32 and ref > 0 and 0.05 < cyc / ref / 10.0 < 3.0
    lib = pk.raw()
    P = lambda t: t.data_ptr()  # noqa: E731
    assert lib.purekv_calib_tile_step(plan.handle, 48, 50, P(src), P(sink), P(ticks), None) == pk.EINVAL
    assert lib.purekv_calib_tile_step(plan.handle, 32, 0, P(src), P(sink), P(ticks), None) == pk.EINVAL
    assert lib.purekv_calib_tile_step(plan.handle, 32, 50, None, P(sink), P(ticks), None) == pk.EINVAL
    with pytest.raises(ValueError):
        pk.purekv_calib_tile_step(plan, 32, 50, src[:1000])


@pytest.mark.parametrize("name,patterns", [
    ("longtext_2f", [3, 1]),                         # split text rows: the combination must leave the other head alone
    ("heads7_3f", [1, 2, 1, 2, 3, 3, 0]),            # all four patterns inside one KV group
    ("heads3_4f", [2, 2, 1, 1, 1, 2]),               # d = 64, two KV heads
    ("heads3_4f", [1, 1, 1, 3, 3, 3]),               # whole KV groups: the subset plans keep the stacked shape
    ("manyunits_g7", [3] * 7 + [1] * 14 + [2] * 7 + [0] * 14),   # 6 KV groups of 7 heads, split text rows
])
def test_per_head_patterns_through_head_subset_plans(name, patterns):
    """The other reading of the dual path: every query head has a pattern of its own.  One plan per pattern over
    the heads that use it, one prefill call per plan into the same output: every head must match the oracle under
    ITS pattern, and a call must not touch the rows of heads outside its plan."""
    wl = SMALL[name]
    assert len(patterns) == wl.n_q_heads
    inp = generate(wl, seed=17)
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((wl.n_q_heads, wl.n_tokens), float("nan"), dtype=torch.float32, device="cuda")
    done = np.zeros(wl.n_q_heads, bool)
    for pattern in sorted(set(patterns)):
        mask = [p == pattern for p in patterns]
        plan = pk.Plan(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads, wl.head_dim,
                       pattern, head_mask=mask)
        before = bits_of(out).copy()
        pk.purekv_st_spattn_prefill(plan, q, k, v, out=out, lse=lse)
        torch.cuda.synchronize()
        after = bits_of(out)
        untouched = ~np.array(mask)
        assert np.array_equal(after[untouched], before[untouched]), f"pattern {pattern} wrote outside its heads"
        done |= np.array(mask)
    assert done.all()
    qf, kf, vf = F64(inp.q), F64(inp.k), F64(inp.v)
    got, got_lse = f64_of(out), f64_of(lse)
    for pattern in sorted(set(patterns)):
        heads = [h for h, p in enumerate(patterns) if p == pattern]
        ref, ref_lse = orc.masked_attention(qf, kf, vf, wl.n_frames, wl.patches, wl.n_text, pattern, heads=heads)
        check_attention(got[heads], ref, f"{name} pattern {pattern} heads {heads}")   # the oracle returns the asked heads
        assert np.abs(got_lse[heads] - ref_lse).max() < 2e-3


def test_prefill_random_shapes_sweep():
    """Seeded sweep: odd frame sizes, texts from none to long, head groupings 1..7, both head sizes, every
    pattern, with and without the log-sum-exp output -- each through the kernel and against the oracle."""
    rng = np.random.default_rng(25600)
    for case in range(24):
        ph, pw = int(rng.integers(1, 14)), int(rng.integers(1, 14))
        F = int(rng.integers(1, max(2, min(10, 900 // (ph * pw)) + 1)))
        T = int(rng.choice([0, 1, 7, 33, 129, 700]))
        hkv = int(rng.choice([1, 2, 3]))
        g = int(rng.choice([1, 2, 4, 7]))
        d = int(rng.choice([64, 128]))
        pattern = int(rng.integers(0, 4))
        wl = small_variant(f"sweep{case}", n_frames=F, patch_h=ph, patch_w=pw, n_text=T, n_q_heads=hkv * g,
                           n_kv_heads=hkv, head_dim=d)
        print(f"[case] sweep {case}: F={F} P={ph}x{pw} T={T} heads {hkv * g}/{hkv} d={d} pattern={pattern}", flush=True)
        inp = generate(wl, seed=100 + case)
        plan = _plan(wl, pattern)
        q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
        out, lse = pk.purekv_st_spattn_prefill(plan, q, k, v, want_lse=True)
        out2 = pk.purekv_st_spattn_prefill(plan, q, k, v)
        torch.cuda.synchronize()
        ref, ref_lse = orc.masked_attention(F64(inp.q), F64(inp.k), F64(inp.v), F, ph * pw, T, pattern)
        check_attention(f64_of(out), ref, f"sweep {case} (lse variant)")
        check_attention(f64_of(out2), ref, f"sweep {case}")
        assert np.abs(f64_of(lse) - ref_lse).max() < 2e-3


def test_window_plan_random_shapes_sweep():
    """Seeded sweep of window plans with more units than workgroups (many heads on short sequences), so that most of
    them are divided: outputs and the window's log-sum-exp against the oracle, every other element of lse untouched,
    output bits equal to the undivided plan's where both run a row's list whole."""
    rng = np.random.default_rng(25601)
    divided = 0
    for case in range(10):
        ph, pw = int(rng.integers(4, 14)), int(rng.integers(4, 14))
        F = max(2, int(rng.integers(900, 1600)) // (ph * pw))
        T = int(rng.choice([0, 5, 40, 129]))
        hkv, g = [(8, 7), (16, 4), (12, 7)][int(rng.integers(0, 3))]
        d = int(rng.choice([64, 128]))
        pattern = int(rng.choice([0, 1, 3, 3]))
        wl = small_variant(f"wsweep{case}", n_frames=F, patch_h=ph, patch_w=pw, n_text=T, n_q_heads=hkv * g,
                           n_kv_heads=hkv, head_dim=d)
        n = wl.n_tokens
        w = int(rng.integers(1, 48))
        inp = generate(wl, seed=300 + case)
        plan, whole = pk.Plan.for_workload(wl, pattern, lse_window=w), pk.Plan.for_workload(wl, pattern)
        c = plan.counts()
        divided += c["lse_queue0"] > 0
        print(f"[case] window sweep {case}: F={F} P={ph}x{pw} T={T} heads {hkv * g}/{hkv} d={d} pattern={pattern} w={w} "
              f"N={n} lse_queue0={c['lse_queue0']}", flush=True)
        q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
        lse = torch.full((wl.n_q_heads, n), 7.5, dtype=torch.float32, device="cuda")
        out, _ = pk.purekv_st_spattn_prefill(plan, q, k, v, lse=lse)
        out_whole = pk.purekv_st_spattn_prefill(whole, q, k, v)
        torch.cuda.synchronize()
        ref, ref_lse = orc.masked_attention(F64(inp.q), F64(inp.k), F64(inp.v), F, ph * pw, T, pattern)
        check_attention(f64_of(out), ref, f"window sweep {case}")
        got = f64_of(lse)
        assert np.all(got[:, :n - w] == 7.5) and np.abs(got[:, n - w:] - ref_lse[:, n - w:]).max() < 2e-3
        if c["n_split_qtiles"] == 0 and whole.counts()["n_split_qtiles"] == 0:
            assert np.array_equal(bits_of(out), bits_of(out_whole))
    assert divided >= 5, divided   # (a plan stays whole when the window's tiles are over a quarter of the work)


def test_importance_random_shapes_sweep():
    """Seeded sweep of the column sums: window sizes from one row to the whole sequence (text rows only, video rows
    under a mask, windows that are not a multiple of the 32-row block), odd frame sizes, 1..7 heads per KV head."""
    rng = np.random.default_rng(314)
    for case in range(20):
        ph, pw = int(rng.integers(1, 12)), int(rng.integers(1, 12))
        F = int(rng.integers(1, max(2, min(8, 700 // (ph * pw)) + 1)))
        T = int(rng.choice([0, 5, 40, 130, 300]))
        hkv = int(rng.choice([1, 2]))
        g = int(rng.choice([1, 3, 7]))
        d = int(rng.choice([64, 128]))
        pattern = int(rng.integers(0, 4))
        n = F * ph * pw + T
        w = int(rng.choice([1, 31, 32, 33, max(1, T), max(1, n // 3), n]))
        w = min(max(w, 1), n)
        wl = small_variant(f"isweep{case}", n_frames=F, patch_h=ph, patch_w=pw, n_text=T, n_q_heads=hkv * g,
                           n_kv_heads=hkv, head_dim=d)
        print(f"[case] importance sweep {case}: N={n} w={w} heads {hkv * g}/{hkv} d={d} pattern={pattern}", flush=True)
        inp = generate(wl, seed=200 + case)
        plan = _plan(wl, pattern)
        q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
        _, lse = pk.purekv_st_spattn_prefill(plan, q, k, v, want_lse=True)
        c = pk.purekv_lowlayer_importance(plan, q, k, lse, w)
        torch.cuda.synchronize()
        ref = orc.window_column_sums(F64(inp.q), F64(inp.k), F, ph * pw, T, pattern, w)
        got = f64_of(c)
        assert got.shape == ref.shape
        if ref.size:
            rel = np.abs(got - ref) / np.maximum(np.abs(ref), 1e-12)
            assert rel.max() <= IMPORTANCE_REL, f"case {case}: worst rel {rel.max():.3g}"
            assert np.all(got[ref == 0] == 0)


def test_decode_random_shapes_sweep():
    """Seeded sweep of the decode step: cache lengths around the 32-key wavefront tiles and the 256-key chunks, 1 to
    20 query heads per KV head (more than one block of 16), both head sizes; fused append + attention against the
    oracle on the grown cache, and the cache rows themselves."""
    from workloads import f32_to_bf16_bits
    rng = np.random.default_rng(77)
    for case in range(24):
        hkv = int(rng.choice([1, 2, 5]))
        g = int(rng.choice([1, 2, 7, 16, 17, 20]))
        d = int(rng.choice([64, 128]))
        n0 = int(rng.choice([0, 1, 15, 16, 31, 32, 33, 255, 256, 257, 511, 513, 1000, 2049]))
        hq = hkv * g
        bits = lambda *shape: f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))  # noqa: E731
        cap = n0 + 3
        kc_h, vc_h = bits(hkv, cap, d), bits(hkv, cap, d)
        kc, vc = to_dev(kc_h), to_dev(vc_h)
        plan = pk.Plan(1, 4, 4, 4, hq, hkv, d, 3)
        print(f"[case] decode sweep {case}: heads {hq}/{hkv} d={d} n0={n0}", flush=True)
        for t in range(2):
            q, kn, vn = bits(hq, d), bits(hkv, d), bits(hkv, d)
            out = pk.purekv_decode_step(plan, to_dev(q), to_dev(kn), to_dev(vn), kc, vc, n0 + t)
            torch.cuda.synchronize()
            kc_h[:, n0 + t], vc_h[:, n0 + t] = kn, vn
            assert np.array_equal(bits_of(kc), kc_h) and np.array_equal(bits_of(vc), vc_h)
            ref = orc.decode_attention(F64(q), F64(kc_h)[:, :n0 + t + 1], F64(vc_h)[:, :n0 + t + 1])
            check_attention(f64_of(out), ref, f"decode sweep {case} step {t}")


def test_two_streams_share_one_plan():
    """A plan holds no mutable device state: decode calls and prefill calls (with split lists) on two streams, each
    with a workspace of its own, may overlap on the GPU.  Both streams' results against the oracle, several rounds."""
    wl = SMALL["heads7_3f"]          # text rows split into slices: the prefill hands partial results over in its workspace
    n, hq, hkv, d = wl.n_tokens, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    plan = _plan(wl, 3)
    assert plan.counts()["n_split_qtiles"] > 0
    data = [generate(wl, seed=80 + i, decode_steps=1) for i in range(2)]
    n_c = 1100                       # five chunks of cached keys: the decode kernel merges through its workspace
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    dev = [[to_dev(x) for x in (dt.q, dt.k, dt.v, dt.q_new[0])] for dt in data]
    torch.cuda.synchronize()
    outs, decs = [[], []], [[], []]
    for rnd in range(6):
        for i, s in enumerate(streams):
            with torch.cuda.stream(s):
                q, k, v, qn = dev[i]
                outs[i].append(pk.purekv_st_spattn_prefill(plan, q, k, v))
                decs[i].append(pk.purekv_decode_attn(plan, qn, k[:, :n_c].contiguous(), v[:, :n_c].contiguous(), n_c))
    torch.cuda.synchronize()
    for i, dt in enumerate(data):
        ref, _ = orc.masked_attention(F64(dt.q), F64(dt.k), F64(dt.v), wl.n_frames, wl.patches, wl.n_text, 3)
        dref = orc.decode_attention(F64(dt.q_new[0]), F64(dt.k)[:, :n_c], F64(dt.v)[:, :n_c])
        for rnd in range(6):
            check_attention(f64_of(outs[i][rnd]), ref, f"stream {i} round {rnd} prefill")
            check_attention(f64_of(decs[i][rnd]), dref, f"stream {i} round {rnd} decode")
            assert np.array_equal(bits_of(outs[i][rnd]), bits_of(outs[i][0]))   # and reproducible bit for bit
            assert np.array_equal(bits_of(decs[i][rnd]), bits_of(decs[i][0]))


@pytest.mark.parametrize("pattern", [0, 3])
@pytest.mark.parametrize("name", ["tiny_4f", "ragged_3f", "straddle_3f", "heads7_3f", "heads3_4f", "manyunits_g7",
                                  "manyunits_g1", "single_token", "longtext_2f"])
def test_prefill_emits_squared_v_norms(name, pattern):
    """The V-norm weighting without a second pass over V (Eq. 3 / Eq. 4): the prefill call that also emits
    ||v_j||^2 for every key writes every entry exactly once (NaN-filled buffer), equal to the oracle's norms, and
    leaves the attention output bit for bit what the plain call gives; the selection from C and these norms is the
    oracle's."""
    wl = SMALL[name]
    inp = generate(wl, seed=33)
    n, w = wl.n_tokens, min(wl.window if wl.window else 1, wl.n_tokens)
    w = max(w, 1)
    print(f"[case] prefill+vnorm {name} pattern={pattern}", flush=True)
    plan = _plan(wl, pattern)
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    out_plain, lse_plain = pk.purekv_st_spattn_prefill(plan, q, k, v, want_lse=True)
    vn2 = torch.full((wl.n_kv_heads, n), float("nan"), dtype=torch.float32, device="cuda")
    out, lse = pk.purekv_st_spattn_prefill(plan, q, k, v, want_lse=True, vnorm2=vn2)
    out_nolse = pk.purekv_st_spattn_prefill(plan, q, k, v, vnorm2=torch.empty_like(vn2))
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out), bits_of(out_plain)) and torch.equal(lse, lse_plain)
    assert np.array_equal(bits_of(out_nolse), bits_of(out_plain))
    vf = F64(inp.v)
    ref = (vf * vf).sum(2)
    got = f64_of(vn2)
    assert np.isfinite(got).all()
    assert np.all(np.abs(got - ref) <= 2e-6 * ref + 1e-30), f"worst rel {np.max(np.abs(got - ref) / np.maximum(ref, 1e-30)):.3g}"
    if n - w >= 1:
        h = max(1, orc.budget(n, w, 0.3)) if n - w >= 2 else 1
        h = min(h, n - w)
        c = np.random.default_rng(5).random((wl.n_kv_heads, n - w)).astype(np.float32)
        idx, s = pk.purekv_topk_select_vnorm(plan, torch.from_numpy(c).cuda(), vn2, w, h, want_scores=True)
        idx2 = pk.purekv_topk_select_vnorm(plan, torch.from_numpy(c).cuda(), vn2, w, h)   # workspace path
        torch.cuda.synchronize()
        assert torch.equal(idx, idx2)
        s_ref = orc.vnorm_scores(c.astype(np.float64), vf)
        assert np.all(np.abs(f64_of(s) - s_ref) <= 2e-6 * np.abs(s_ref) + 1e-30)
        check_kept_sets(idx.cpu().numpy(), orc.topk_select(s_ref, h, n, w), s_ref, h)


def test_prefill_vnorm_layers_and_head_subsets():
    """Layered norms [L, Hkv, N] through one batched selection, and a plan over a head subset: the KV heads none of
    whose query heads it covers keep what the buffer held."""
    wl = SMALL["heads3_4f"]       # 6 query heads on 2 KV heads
    n, w = wl.n_tokens, wl.window
    h = orc.budget(n, w, 0.4)
    layers = [generate(wl, seed=90 + l) for l in range(3)]
    plan = _plan(wl, 3)
    vn_all = torch.empty((3, wl.n_kv_heads, n), dtype=torch.float32, device="cuda")
    for l, x in enumerate(layers):
        pk.purekv_st_spattn_prefill(plan, to_dev(x.q), to_dev(x.k), to_dev(x.v), vnorm2=vn_all[l])
    c = np.random.default_rng(6).random((wl.n_kv_heads, n - w)).astype(np.float32)
    idx = pk.purekv_topk_select_vnorm(plan, torch.from_numpy(c).cuda(), vn_all, w, h)
    v_all = torch.stack([to_dev(x.v) for x in layers])
    idx_v = pk.purekv_topk_select(plan, torch.from_numpy(c).cuda(), v_all, w, h)
    torch.cuda.synchronize()
    for l, x in enumerate(layers):
        s_ref = orc.vnorm_scores(c.astype(np.float64), F64(x.v))
        check_kept_sets(idx[l].cpu().numpy(), orc.topk_select(s_ref, h, n, w), s_ref, h)
        check_kept_sets(idx_v[l].cpu().numpy(), orc.topk_select(s_ref, h, n, w), s_ref, h)
    sub = pk.Plan(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, 3,
                  head_mask=[0, 0, 0, 1, 0, 1])            # query heads 3 and 5: KV head 1 only
    x = layers[0]
    vn = torch.full((wl.n_kv_heads, n), -7.0, dtype=torch.float32, device="cuda")
    pk.purekv_st_spattn_prefill(sub, to_dev(x.q), to_dev(x.k), to_dev(x.v), vnorm2=vn)
    torch.cuda.synchronize()
    vf = F64(x.v)
    assert torch.all(vn[0] == -7.0)
    assert np.all(np.abs(f64_of(vn[1]) - (vf[1] ** 2).sum(1)) <= 2e-6 * (vf[1] ** 2).sum(1))


@pytest.mark.parametrize("n", [2, 3, 255, 256, 257, 1000, 8192, 20000])
def test_spearman_matches_oracle_exactly(n):
    """Sec. 3.3, Eq. 5-7: ranks are counts and the sum of squared rank differences an integer: bit-exact; rho is the
    correctly rounded quotient on both sides."""
    rng = np.random.default_rng(50 + n)
    rows = 5
    a = rng.standard_normal((rows, n)).astype(np.float32)
    b = (0.5 * a + rng.standard_normal((rows, n))).astype(np.float32)
    b[1] = a[1]                                                    # identical rankings
    b[2] = -a[2]                                                   # reversed
    a[3] = rng.integers(0, 4, size=n).astype(np.float32)           # heavy ties, signed zeros among them
    b[3] = rng.integers(0, 3, size=n).astype(np.float32)
    a[3, ::7] = -0.0
    b[4] = np.float32(1.5)                                         # one array constant: its ranks are the indices
    print(f"[case] spearman n={n}", flush=True)
    d2, rho = pk.purekv_spearman(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda())
    torch.cuda.synchronize()
    ref_d2, ref_rho = orc.spearman_rank_correlation(a.astype(np.float64), b.astype(np.float64))
    assert d2.cpu().numpy().tolist() == [int(x) for x in ref_d2]
    assert np.array_equal(rho.cpu().numpy(), ref_rho)
    assert rho[1].item() == 1.0
    if np.unique(a[2]).size == n:      # (two equal scores keep their index order in both arrays: not a full reversal)
        assert rho[2].item() == -1.0


def test_spearman_of_estimated_against_own_scores_through_the_library():
    """The check of Sec. 3.3 end to end on one synthetic layer pair: S-hat from the low layer's column sums and the
    high layer's V (Eq. 4), S from the high layer's own column sums (Eq. 6), both through the library, compared with
    the oracle's scores and ranks."""
    wl = SMALL["straddle_3f"]
    low, high = generate(wl, seed=31), generate(wl, seed=32)
    n, w = wl.n_tokens, wl.window
    h = pk.purekv_budget(n, w, 0.2)
    plan = pk.Plan.for_workload(wl, 0)
    scores = []
    for inp in (low, high):
        q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(high.v)
        _, lse = pk.purekv_st_spattn_prefill(plan, q, k, to_dev(inp.v), want_lse=True)
        c = pk.purekv_lowlayer_importance(plan, q, k, lse, w)
        _, s = pk.purekv_topk_select(plan, c, v, w, h, want_scores=True)
        scores.append(s.reshape(wl.n_kv_heads, n - w).contiguous())
    d2, rho = pk.purekv_spearman(scores[0], scores[1])
    torch.cuda.synchronize()
    # the oracle on the library's own fp32 scores: exact; and on its own fp64 scores: the same rho up to the few keys
    # whose order the fp32 rounding of nearly equal scores changes
    ref_d2, ref_rho = orc.spearman_rank_correlation(f64_of(scores[0]), f64_of(scores[1]))
    assert d2.cpu().numpy().tolist() == [int(x) for x in ref_d2] and np.array_equal(rho.cpu().numpy(), ref_rho)
    vf = F64(high.v)
    s_hat = orc.vnorm_scores(orc.window_column_sums(F64(low.q), F64(low.k), wl.n_frames, wl.patches, wl.n_text, 0, w), vf)
    s_own = orc.vnorm_scores(orc.window_column_sums(F64(high.q), F64(high.k), wl.n_frames, wl.patches, wl.n_text, 0, w), vf)
    _, rho64 = orc.spearman_rank_correlation(s_hat, s_own)
    assert np.abs(rho.cpu().numpy() - rho64).max() < 1e-3
    # the two layers' Q and K are independent draws here, but both score arrays carry the same V norms: the rankings
    # agree more than chance (n ~ 1700 keys: chance is |rho| < 0.08 at three sigma)
    assert (rho.cpu().numpy() > 0.08).all()


def test_spearman_argument_errors():
    a = torch.zeros((2, 8), dtype=torch.float32, device="cuda")
    out = torch.zeros(2, dtype=torch.int64, device="cuda")
    lib = pk.raw()
    assert lib.purekv_spearman(a.data_ptr(), a.data_ptr(), 2, 1, out.data_ptr(), None, None) == pk.EINVAL
    assert lib.purekv_spearman(a.data_ptr(), a.data_ptr(), 2, 131073, out.data_ptr(), None, None) == pk.EINVAL
    assert lib.purekv_spearman(a.data_ptr(), a.data_ptr(), 0, 8, out.data_ptr(), None, None) == pk.EINVAL
    assert lib.purekv_spearman(None, a.data_ptr(), 2, 8, out.data_ptr(), None, None) == pk.EINVAL
    assert lib.purekv_spearman(a.data_ptr(), a.data_ptr(), 2, 8, None, None, None) == pk.EINVAL
    assert lib.purekv_spearman(a.data_ptr(), a.data_ptr(), 2, 8, out.data_ptr(), None, None) == pk.OK   # rho is optional
    torch.cuda.synchronize()
    assert out.tolist() == [0, 0]
