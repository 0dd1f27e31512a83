"""Strided tensors at the boundary: token-major [N, H, d] slices of one fused QKV projection buffer (what a decoder
emits) and padded head-major layouts go through every entry point that reads Q, K, V or writes O, and must give
bit for bit what the packed [H, N, d] layout gives on the same values (the arithmetic does not depend on the
addressing), which in turn is checked against the oracle."""
import numpy as np
import pytest
import torch

import paper_2510_25600_amd as pk
from oracle import purekv_oracle as orc
from workloads import WORKLOADS, generate, small_variant

from gpu_util import IMPORTANCE_REL, bits_of, check_attention, f64_of, to_dev

pytestmark = pytest.mark.gpu
F64 = orc.bf16_bits_to_f64

SHAPES = {
    "tiny_4f": WORKLOADS["tiny_4f"],
    "ragged_3f": small_variant("ragged_3f"),
    "heads7_3f": small_variant("heads7_3f", n_frames=3, patch_h=10, patch_w=10, n_text=900, n_q_heads=7, n_kv_heads=1,
                               head_dim=128),
    "heads3_4f": small_variant("heads3_4f", n_frames=4, patch_h=9, patch_w=11, n_text=45, n_q_heads=6, n_kv_heads=2,
                               head_dim=64),
    "manyunits_g7": small_variant("manyunits_g7", n_frames=10, patch_h=16, patch_w=17, n_text=190, n_q_heads=42,
                                  n_kv_heads=6, head_dim=128),
}


def token_major(wl, q, k, v):
    """One [N, (Hq + 2 Hkv) d] buffer as a QKV projection writes it; returns the (H, N, d) views and their strides."""
    hq, hkv, d, n = wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_tokens
    row = (hq + 2 * hkv) * d
    buf = torch.empty((n, row), dtype=torch.bfloat16, device="cuda")
    buf[:, :hq * d] = q.permute(1, 0, 2).reshape(n, hq * d)
    buf[:, hq * d:(hq + hkv) * d] = k.permute(1, 0, 2).reshape(n, hkv * d)
    buf[:, (hq + hkv) * d:] = v.permute(1, 0, 2).reshape(n, hkv * d)
    qv = buf[:, :hq * d].view(n, hq, d).permute(1, 0, 2)
    kv = buf[:, hq * d:(hq + hkv) * d].view(n, hkv, d).permute(1, 0, 2)
    vv = buf[:, (hq + hkv) * d:].view(n, hkv, d).permute(1, 0, 2)
    return qv, kv, vv, dict(q_strides=(d, row), kv_strides=(d, row), o_strides=(d, hq * d))


def padded(wl, q, k, v):
    """Head-major with rows padded by 8 elements and a gap of 24 elements between heads; O packed."""
    def pad(t):
        h, n, d = t.shape
        st, sh = d + 8, n * (d + 8) + 24
        buf = torch.full((h * sh,), float("nan"), dtype=torch.bfloat16, device="cuda")
        view = buf.as_strided((h, n, d), (sh, st, 1))
        view.copy_(t)
        return view, (sh, st)
    qv, qs = pad(q)
    kv, ks = pad(k)
    vv, _ = pad(v)
    return qv, kv, vv, dict(q_strides=qs, kv_strides=ks)


@pytest.mark.parametrize("layout", [token_major, padded])
@pytest.mark.parametrize("pattern", [0, 1, 2, 3])
@pytest.mark.parametrize("name", list(SHAPES))
def test_strided_layouts_equal_packed_bit_for_bit(name, pattern, layout):
    wl = SHAPES[name]
    inp = generate(wl, seed=21)
    n, w = wl.n_tokens, wl.window
    print(f"[case] strided {layout.__name__} {name} pattern={pattern}", flush=True)
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    packed_plan = pk.Plan.for_workload(wl, pattern)
    out_p, lse_p = pk.purekv_st_spattn_prefill(packed_plan, q, k, v, want_lse=True)
    c_p = pk.purekv_lowlayer_importance(packed_plan, q, k, lse_p, w)
    h = max(1, orc.budget(n, w, 0.3))
    idx_p, s_p = pk.purekv_topk_select(packed_plan, c_p, v, w, h, want_scores=True)
    kc_p, vc_p = pk.purekv_kv_compact(packed_plan, k, v, idx_p)

    qv, kv, vv, strides = layout(wl, q, k, v)
    plan = pk.Plan.for_workload(wl, pattern, **strides)
    out_s = plan.empty_out(q.device)
    out_s.fill_(float("nan"))
    _, lse_s = pk.purekv_st_spattn_prefill(plan, qv, kv, vv, out=out_s, want_lse=True)
    c_s = pk.purekv_lowlayer_importance(plan, qv, kv, lse_s, w)
    idx_s, s_s = pk.purekv_topk_select(plan, c_s, vv, w, h, want_scores=True)
    kc_s, vc_s = pk.purekv_kv_compact(plan, kv, vv, idx_s)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out_s), bits_of(out_p))
    assert torch.equal(lse_s, lse_p) and torch.equal(c_s, c_p) and torch.equal(s_s, s_p)
    assert torch.equal(idx_s, idx_p) and torch.equal(kc_s, kc_p) and torch.equal(vc_s, vc_p)
    # and the packed result is the oracle's
    ref, _ = orc.masked_attention(F64(inp.q), F64(inp.k), F64(inp.v), wl.n_frames, wl.patches, wl.n_text, pattern)
    check_attention(f64_of(out_p), ref, f"{name}/p{pattern}")
    c_ref = orc.window_column_sums(F64(inp.q), F64(inp.k), wl.n_frames, wl.patches, wl.n_text, pattern, w)
    assert np.all(np.abs(f64_of(c_p) - c_ref) <= IMPORTANCE_REL * np.maximum(np.abs(c_ref), 1e-12))
    kr, vr = orc.compact(inp.k, inp.v, idx_p.cpu().numpy())
    assert np.array_equal(bits_of(kc_s), kr) and np.array_equal(bits_of(vc_s), vr)


@pytest.mark.parametrize("pattern", [0, 3])
def test_window_plan_on_a_token_major_layout_equals_packed(pattern):
    """A divided window plan (more units than workgroups) on token-major views: the same bits as the packed window
    plan, the log-sum-exp of the window rows only."""
    wl = small_variant("manyunits_g2", n_frames=7, patch_h=15, patch_w=20, n_text=120, n_q_heads=32, n_kv_heads=16,
                       head_dim=64)
    inp = generate(wl, seed=23)
    n, w = wl.n_tokens, 1
    q, k, v = to_dev(inp.q), to_dev(inp.k), to_dev(inp.v)
    packed_plan = pk.Plan.for_workload(wl, pattern, lse_window=w)
    assert packed_plan.counts()["lse_queue0"] > 0
    lse_p = torch.full((wl.n_q_heads, n), -7.0, dtype=torch.float32, device="cuda")
    out_p, _ = pk.purekv_st_spattn_prefill(packed_plan, q, k, v, lse=lse_p)
    qv, kv, vv, strides = token_major(wl, q, k, v)
    plan = pk.Plan.for_workload(wl, pattern, lse_window=w, **strides)
    assert plan.counts()["lse_queue0"] == packed_plan.counts()["lse_queue0"]
    out_s = plan.empty_out(q.device)
    lse_s = torch.full_like(lse_p, -7.0)
    pk.purekv_st_spattn_prefill(plan, qv, kv, vv, out=out_s, lse=lse_s)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(out_s), bits_of(out_p)) and torch.equal(lse_s, lse_p)
    assert (lse_s[:, :n - w] == -7.0).all() and (lse_s[:, n - w:] != -7.0).all()
    ref, ref_lse = orc.masked_attention(F64(inp.q), F64(inp.k), F64(inp.v), wl.n_frames, wl.patches, wl.n_text, pattern)
    check_attention(f64_of(out_p), ref, f"window token-major p{pattern}")
    assert np.abs(f64_of(lse_s)[:, n - w:] - ref_lse[:, n - w:]).max() < 2e-3


def test_token_major_layer_stack_equals_packed():
    """The stack entry points on token-major layers [L, N, Hkv, d] (layer stride = one layer's span)."""
    wl = small_variant("straddle_3f", n_frames=3, patch_h=24, patch_w=24, n_text=70, n_q_heads=4, n_kv_heads=1,
                       head_dim=128)
    n, w, hq, hkv, d = wl.n_tokens, wl.window, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    h = orc.budget(n, w, 0.3)
    layers, clie, st_layer = 4, 1, 2
    data = [generate(wl, seed=70 + l) for l in range(layers)]
    stack = pk.Stack(layers, clie, st_layer, w, h)

    def run(token_major_layout):
        if token_major_layout:
            strides = dict(q_strides=(d, hq * d), kv_strides=(d, hkv * d), o_strides=(d, hq * d))
            k_all = torch.stack([to_dev(x.k).permute(1, 0, 2).contiguous() for x in data]).permute(0, 2, 1, 3)
            v_all = torch.stack([to_dev(x.v).permute(1, 0, 2).contiguous() for x in data]).permute(0, 2, 1, 3)
        else:
            strides = {}
            k_all = torch.stack([to_dev(x.k) for x in data])
            v_all = torch.stack([to_dev(x.v) for x in data])
        dense, st = pk.Plan.for_workload(wl, 0, **strides), pk.Plan.for_workload(wl, 3, **strides)
        lse = torch.empty((hq, n), dtype=torch.float32, device="cuda")
        c_all = torch.empty((clie + 1, hkv, n - w), dtype=torch.float32, device="cuda")
        outs = []
        for l, x in enumerate(data):
            q = to_dev(x.q)
            if token_major_layout:
                q = q.permute(1, 0, 2).contiguous().permute(1, 0, 2)
            out = dense.empty_out(q.device)
            pk.purekv_stack_layer(dense, st, stack, l, q, k_all[l], v_all[l], out, lse, c_all)
            outs.append(bits_of(out))
        idx_all = torch.empty((layers, hkv, h + w), dtype=torch.int32, device="cuda")
        kc_all = torch.zeros((layers, hkv, h + w, d), dtype=torch.bfloat16, device="cuda")
        vc_all = torch.zeros_like(kc_all)
        pk.purekv_stack_select_compact(dense, st, stack, c_all, k_all, v_all, idx_all, kc_all, vc_all)
        torch.cuda.synchronize()
        return outs, c_all.cpu().numpy(), idx_all.cpu().numpy(), bits_of(kc_all), bits_of(vc_all)

    a, b = run(False), run(True)
    for l in range(layers):
        assert np.array_equal(a[0][l], b[0][l])
    for x, y in zip(a[1:], b[1:]):
        assert np.array_equal(x, y)
