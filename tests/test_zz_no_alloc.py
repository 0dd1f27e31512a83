"""The top-h entry point that allocates nothing (purekv_topk_select_static): its scores live in a buffer that is
part of the library's device image.  Checked through the C ABI against purekv_topk_select on the same inputs, bit
for bit, on two calls in a row, the second with a smaller input (the buffer keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2510_25600_amd as pk
from workloads import generate, small_variant

from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _case(wl, layers, seed, ratio):
    n, w = wl.n_tokens, wl.window
    h = pk.purekv_budget(n, w, ratio)
    plan = pk.Plan.for_workload(wl, 3)
    rng = np.random.default_rng(seed)
    c = torch.from_numpy(rng.random((wl.n_kv_heads, n - w)).astype(np.float32)).cuda()
    v_all = torch.stack([to_dev(generate(wl, seed=seed + l).v) for l in range(layers)])
    return plan, c, v_all, w, h


def _both(plan, c, v_all, w, h):
    """(existing entry point, static entry point), both called through the raw C ABI."""
    lib = pk.raw()
    layers = v_all.shape[0]
    stream = torch.cuda.current_stream().cuda_stream
    idx_ref = torch.full((layers, plan.Hkv, h + w), -1, dtype=torch.int32, device="cuda")
    idx_new = torch.full_like(idx_ref, -2)
    nb = plan.workspace_bytes(pk.OP_TOPK, layers, w)
    ws = torch.empty(max(nb, 16), dtype=torch.uint8, device="cuda")
    rc = lib.purekv_topk_select(plan.handle, c.data_ptr(), v_all.data_ptr(), v_all.stride(0), layers, w, h,
                                idx_ref.data_ptr(), None, ws.data_ptr(), nb, stream)
    assert rc == pk.OK, pk.purekv_strerror(rc)
    rc = lib.purekv_topk_select_static(plan.handle, c.data_ptr(), v_all.data_ptr(), v_all.stride(0), layers, w, h,
                                       idx_new.data_ptr(), stream)
    assert rc == pk.OK, pk.purekv_strerror(rc)
    torch.cuda.synchronize()
    return idx_ref.cpu().numpy(), idx_new.cpu().numpy()


def test_static_topk_matches_workspace_topk_on_two_calls_in_a_row():
    big = small_variant("static_big", n_frames=6, patch_h=16, patch_w=16, n_text=200, n_q_heads=8, n_kv_heads=4,
                        head_dim=128)
    small = small_variant("static_small", n_frames=3, patch_h=5, patch_w=7, n_text=19, n_q_heads=4, n_kv_heads=2,
                          head_dim=64)
    print("[case] static top-h: 3 layers x 4 KV heads x 1536 keys", flush=True)
    ref, new = _both(*_case(big, 3, 50, 0.3))
    assert np.array_equal(ref, new)
    assert (new >= 0).all()
    print("[case] static top-h: smaller input on the same buffer", flush=True)
    ref, new = _both(*_case(small, 2, 60, 0.4))
    assert np.array_equal(ref, new)
    # and the larger one again: nothing of the smaller call lingers
    ref, new = _both(*_case(big, 3, 50, 0.3))
    assert np.array_equal(ref, new)


def test_static_topk_without_vnorm_and_its_limit():
    lib = pk.raw()
    wl = small_variant("static_lim", n_frames=2, patch_h=8, patch_w=8, n_text=16, n_q_heads=2, n_kv_heads=2, head_dim=64)
    plan, c, v_all, w, h = _case(wl, 1, 70, 0.25)
    stream = torch.cuda.current_stream().cuda_stream
    idx_a = torch.empty((1, plan.Hkv, h + w), dtype=torch.int32, device="cuda")
    idx_b = torch.empty_like(idx_a)
    # no V: selection on C itself, no scores buffer used
    assert lib.purekv_topk_select(plan.handle, c.data_ptr(), None, 0, 1, w, h, idx_a.data_ptr(), None, None, 0,
                                  stream) == pk.OK
    assert lib.purekv_topk_select_static(plan.handle, c.data_ptr(), None, 0, 1, w, h, idx_b.data_ptr(), stream) == pk.OK
    torch.cuda.synchronize()
    assert np.array_equal(idx_a.cpu().numpy(), idx_b.cpu().numpy())
    # more scores than the buffer holds: refused before anything is launched (validation never reads v)
    too_many = (1 << 20) // (plan.Hkv * (plan.N - w)) + 1
    assert lib.purekv_topk_select_static(plan.handle, c.data_ptr(), v_all.data_ptr(), v_all.stride(0), too_many, w, h,
                                         idx_b.data_ptr(), stream) == pk.EWORKSPACE
    assert lib.purekv_topk_select_static(plan.handle, c.data_ptr(), v_all.data_ptr(), 0, 1, w, h, None, stream) == pk.EINVAL
