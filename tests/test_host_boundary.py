"""CPU-only tests of the C-ABI library: exports, argument validation (all done on the host before any
GPU call), the keep-budget rule, and the host planner's block lists against the oracle's boolean mask."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2510_25600_amd as pk
from oracle import purekv_oracle as orc
from workloads import WORKLOADS, small_variant

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "purekv.h")).read()
    declared = set(re.findall(r"PUREKV_API[^;(]*?\b(purekv_\w+)\s*\(", header))
    assert len(declared) >= 18
    lib = ctypes.CDLL(pk.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(pk.EXPORTS)


def test_status_strings():
    for st in (pk.OK, pk.EINVAL, pk.EUNSUPPORTED, pk.EWORKSPACE, pk.EHIP, pk.ENOMEM, -99):
        assert isinstance(pk.purekv_strerror(st), str) and pk.purekv_strerror(st)


def test_shape_validation_error_codes():
    lib = pk.raw()
    good = dict(n_frames=2, patch_h=4, patch_w=4, n_text=8, n_q_heads=4, n_kv_heads=2, head_dim=64, pattern=3,
                softmax_scale=0.0)

    def create(**kw):
        s = pk.Shape(**{**good, **kw})
        h = ctypes.c_void_p()
        rc = lib.purekv_plan_create_host(ctypes.byref(s), 256, ctypes.byref(h))
        if rc == 0:
            lib.purekv_plan_destroy(h)
        else:
            assert not h  # *out untouched on failure
        return rc

    assert create() == pk.OK
    assert create(n_text=0) == pk.OK
    assert create(n_frames=0) == pk.EINVAL
    assert create(patch_h=0) == pk.EINVAL
    assert create(n_text=-1) == pk.EINVAL
    assert create(n_q_heads=3) == pk.EINVAL          # not a multiple of the KV heads
    assert create(n_kv_heads=0) == pk.EINVAL
    assert create(softmax_scale=-1.0) == pk.EINVAL
    assert create(softmax_scale=float("nan")) == pk.EINVAL
    assert create(head_dim=96) == pk.EUNSUPPORTED
    assert create(pattern=4) == pk.EUNSUPPORTED
    h = ctypes.c_void_p()
    assert lib.purekv_plan_create_host(None, 256, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_create_host(ctypes.byref(pk.Shape(**good)), 256, None) == pk.EINVAL
    assert lib.purekv_plan_create_host(ctypes.byref(pk.Shape(**good)), 0, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_destroy(None) == pk.OK
    # strides (elements): a pair of zeros = packed; otherwise 16-byte rows, token stride >= d and < 2^23, span < 2^31
    n = 2 * 16 + 8
    assert create(q_stride_head=64, q_stride_tok=4 * 64, kv_stride_head=64, kv_stride_tok=2 * 64,
                  o_stride_head=64, o_stride_tok=4 * 64) == pk.OK                     # token-major [N, H, d]
    assert create(kv_stride_head=n * 72, kv_stride_tok=72) == pk.OK                   # padded rows
    assert create(q_stride_head=0, q_stride_tok=64) == pk.EINVAL                      # head stride missing
    assert create(q_stride_head=n * 64, q_stride_tok=0) == pk.EINVAL                  # token stride missing
    assert create(kv_stride_head=n * 64, kv_stride_tok=32) == pk.EINVAL               # token stride below head_dim
    assert create(o_stride_head=n * 64 + 4, o_stride_tok=64) == pk.EINVAL             # not a multiple of 8 elements
    assert create(q_stride_head=n * 68, q_stride_tok=68) == pk.EINVAL
    assert create(q_stride_head=-64, q_stride_tok=64) == pk.EINVAL
    assert create(kv_stride_head=64, kv_stride_tok=1 << 23) == pk.EINVAL              # 24-bit row stride in bytes
    assert create(q_stride_head=1 << 30, q_stride_tok=64) == pk.EINVAL                # span beyond 2^31 bytes
    assert create(n_frames=4096, patch_h=32, patch_w=32, n_kv_heads=4, head_dim=128) == pk.EINVAL   # packed span too


def test_compute_calls_validate_before_touching_the_gpu():
    """A host-only plan cannot be launched; null pointers and bad sizes are refused with EINVAL."""
    lib = pk.raw()
    plan = pk.Plan(2, 4, 4, 8, 4, 2, 64, host_only=True)
    h = plan.handle
    one = ctypes.c_void_p(16)  # never dereferenced: validation fails first
    assert lib.purekv_st_spattn_prefill(h, one, one, one, one, None, None, 0, None) == pk.EINVAL
    assert lib.purekv_st_spattn_prefill(None, one, one, one, one, None, None, 0, None) == pk.EINVAL
    assert lib.purekv_st_spattn_prefill_vnorm(h, one, one, one, one, None, one, None, 0, None) == pk.EINVAL
    assert lib.purekv_topk_select_vnorm(h, one, one, 0, 1, 8, 4, one, None, None, 0, None) == pk.EINVAL
    assert lib.purekv_lowlayer_importance(h, one, one, one, 8, one, None, 0, None) == pk.EINVAL
    assert lib.purekv_topk_select(h, one, None, 0, 1, 8, 4, one, None, None, 0, None) == pk.EINVAL
    assert lib.purekv_topk_select_static(h, one, one, 0, 1, 8, 4, one, None) == pk.EINVAL
    assert lib.purekv_topk_select_static(None, one, one, 0, 1, 8, 4, one, None) == pk.EINVAL
    assert lib.purekv_kv_compact(h, one, one, 0, 1, one, 4, one, one, 4, None) == pk.EINVAL
    assert lib.purekv_kv_append(h, one, one, one, one, 0, 4, None) == pk.EINVAL
    assert lib.purekv_decode_attn(h, one, one, one, 4, 4, one, one, 1 << 20, None) == pk.EINVAL
    assert lib.purekv_decode_step(h, one, one, one, one, one, 3, 4, one, one, 1 << 20, None) == pk.EINVAL
    assert lib.purekv_calib_mfma(h, 0, 0, 10, one, one, None) == pk.EINVAL
    assert lib.purekv_calib_tile_step(h, 32, 10, one, one, one, None) == pk.EINVAL
    assert lib.purekv_calib_tile_step_flops(h, 10) == 4.0 * 256 * 64 * 128 * 10 * plan.counts()["n_workgroups"]
    assert lib.purekv_calib_mfma_flops(None, 10) == 0.0
    assert lib.purekv_calib_mfma_flops(h, 10) == 2.0 * 32 * 32 * 16 * 16 * 10 * 8 * plan.counts()["n_workgroups"]
    stack = pk.Stack(4, 1, 2, 8, 4)
    assert lib.purekv_stack_layer(h, h, ctypes.byref(stack), 0, one, one, one, one, one, one, one, 1 << 20, None) == pk.EINVAL
    assert lib.purekv_workspace_init(h, pk.OP_PREFILL, one, 1 << 20, 0, 0, 0, None) == pk.EINVAL
    assert lib.purekv_stack_workspace_init(h, h, ctypes.byref(stack), one, 1 << 20, None) == pk.EINVAL
    assert lib.purekv_stack_select_compact(h, h, ctypes.byref(stack), one, one, one, 0, one, one, one, 16, one, 1 << 20,
                                           None) == pk.EINVAL
    assert lib.purekv_stack_workspace_bytes(h, h, ctypes.byref(stack)) == 0
    assert lib.purekv_stack_workspace_bytes(None, None, None) == 0
    assert lib.purekv_workspace_bytes(None, pk.OP_PREFILL, 0, 0, 0) == 0
    c = (ctypes.c_int64 * 16)()
    assert lib.purekv_plan_counts(None, c) == pk.EINVAL and lib.purekv_plan_counts(h, None) == pk.EINVAL
    assert lib.purekv_plan_qtile_list(h, 99, None, 0) == pk.EINVAL
    assert lib.purekv_plan_queue(h, 100000, None, 0) == pk.EINVAL
    assert lib.purekv_plan_item(h, -1, (ctypes.c_int32 * 6)()) == pk.EINVAL


def test_spearman_validates_before_touching_the_gpu():
    lib = pk.raw()
    buf = (ctypes.c_float * 8)()
    out = (ctypes.c_uint64 * 2)()
    for args in [(None, buf, 1, 8, out), (buf, None, 1, 8, out), (buf, buf, 1, 8, None), (buf, buf, 0, 8, out),
                 (buf, buf, 70000, 8, out), (buf, buf, 1, 1, out), (buf, buf, 1, 131073, out)]:
        a = [ctypes.cast(x, ctypes.c_void_p) if x is not None and not isinstance(x, int) else x for x in args]
        assert lib.purekv_spearman(a[0], a[1], a[2], a[3], a[4], None, None) == pk.EINVAL


def test_budget_matches_oracle_rule():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        n = int(rng.integers(1, 70000))
        w = int(rng.integers(1, n + 1))
        r = float(rng.choice([0.05, 0.1, 0.2, 0.33, 0.35, 0.5, rng.random()]))
        assert pk.purekv_budget(n, w, r) == orc.budget(n, w, r)
    assert pk.purekv_budget(8448, 256, 0.2) == 1433
    # decimal ratios mean what they say (0.29 * 100 is 28.999999999999996 in binary), independent of the oracle
    for n in (100, 288, 1000, 4736, 8448, 16640, 33280):
        for pct in range(0, 101):
            assert pk.purekv_budget(n, 0, pct / 100) == (pct * n) // 100, (n, pct)
    # no valid budget: negative sizes, ratios outside [0, 1] or not finite
    for bad in (float("nan"), float("inf"), -0.1, 1.5):
        assert pk.purekv_budget(100, 10, bad) == -1
    assert pk.purekv_budget(-1, 10, 0.2) == -1 and pk.purekv_budget(100, -1, 0.2) == -1
    assert pk.purekv_budget(100, 10, 1.0) == 90 and pk.purekv_budget(100, 10, 0.0) == 0


def _check_plan_against_oracle(F, ph, pw, T, hq, hkv, d, pattern, n_wg=256, window=0):
    """Tile lists, need bits and block kinds against the oracle's boolean mask; slices, units and queues are a
    partition of the work.  window > 0: a window plan (the last `window` rows want their log-sum-exp): the units of
    the query tiles that hold such rows, and no others, run on the workgroups from lse_queue0 on."""
    P, n = ph * pw, F * ph * pw + T
    plan = pk.Plan(F, ph, pw, T, hq, hkv, d, pattern, host_only=True, n_workgroups=n_wg, lse_window=window)
    c = plan.counts()
    assert c["lse_window"] == window and 0 <= c["lse_queue0"] < c["n_workgroups"]
    if window == 0:
        assert c["lse_queue0"] == 0
    R, gs, n_groups = c["row_blocks"], c["stacked_heads"], c["n_head_groups"]
    g = hq // hkv
    assert 1 <= gs * R <= pk.WAVES and g % gs == 0 and n_groups * gs == hq
    if pattern != 0 and g > 1 and any(g % x == 0 for x in range(2, pk.WAVES + 1)):
        assert gs > 1      # sparse patterns stack the heads of a KV group
    bq = R * pk.BLOCK
    assert c["N"] == n and c["n_qtiles"] == (n + bq - 1) // bq
    n_ktiles = (n + pk.BK - 1) // pk.BK
    total_pairs = refs = 0
    by_kind = [0, 0, 0, 0]
    for qt in range(c["n_qtiles"]):
        rows = np.arange(qt * bq, min((qt + 1) * bq, n))
        mask = orc.st_mask_rows(F, P, T, pattern, rows)
        total_pairs += int(mask.sum())
        padded = np.zeros((bq, n_ktiles * pk.BK), dtype=bool)
        padded[:rows.shape[0], :n] = mask
        blocks = padded.reshape(R, pk.BLOCK, n_ktiles, 2, pk.BLOCK)      # [rb, row, tile, kb, key]
        any_b = blocks.any(axis=(1, 4))                                      # [rb, tile, kb]
        lst = plan.qtile_list(qt)
        refs += len(lst)
        assert [t for t, _, _ in lst] == np.nonzero(any_b.any(axis=(0, 2)))[0].tolist(), (qt, pattern)
        row_idx = qt * bq + np.arange(bq).reshape(R, pk.BLOCK)               # absolute query rows
        real = row_idx < n
        for t, need, kinds in lst:
            want_need = sum(1 << (2 * rb + kb) for rb in range(R) for kb in range(2) if any_b[rb, t, kb])
            assert need == want_need, (qt, t, pattern)
            for rb in range(R):
                for kb in range(2):
                    if not any_b[rb, t, kb]:
                        continue
                    kind = (kinds >> (4 * rb + 2 * kb)) & 3
                    by_kind[kind] += 1
                    blk = blocks[rb, :, t, kb, :][real[rb]]                  # real rows only
                    i = row_idx[rb][real[rb]][:, None]
                    j = (t * pk.BK + kb * pk.BLOCK + np.arange(pk.BLOCK))[None, :]
                    # a cheaper kind is a promise about the mask of the block; the general kind promises nothing
                    if kind == pk.KIND_FULL:
                        assert blk.all(), (qt, t, rb, kb, pattern)
                    elif kind == pk.KIND_CAUSAL:
                        assert np.array_equal(blk, np.broadcast_to(j <= i, blk.shape)), (qt, t, rb, kb, pattern)
                    elif kind == pk.KIND_PREV:
                        assert np.array_equal(blk, np.broadcast_to(j == i - P, blk.shape)), (qt, t, rb, kb, pattern)
    assert refs == c["n_tile_refs"] and sum(by_kind) == c["n_blocks"]
    assert by_kind == [c["n_full_blocks"], c["n_causal_blocks"], c["n_prev_blocks"], c["n_general_blocks"]]
    if pattern == 0:
        assert by_kind[2] == 0 and by_kind[3] == 0     # the dense kernel variant only knows full and causal
    assert abs(plan.mask_flops() - 4.0 * d * total_pairs * hq) < 1e-3 * max(1.0, plan.mask_flops())
    assert plan.kept_tile_flops() == 4.0 * pk.BLOCK * pk.BLOCK * d * c["n_blocks"] * hq
    # work items: each query tile's list is covered exactly once, in order; slots are distinct
    begin = np.concatenate([[0], np.cumsum([len(plan.qtile_list(q)) for q in range(c["n_qtiles"])])])
    items = [plan.item(i) for i in range(c["n_items"])]
    assert all(items[i][2] >= items[i + 1][2] for i in range(len(items) - 1))  # longest first
    by_q = {}
    for qt, lb, nt, sp, ns, slot in items:
        by_q.setdefault(qt, []).append((sp, lb, nt, ns, slot))
    assert sorted(by_q) == list(range(c["n_qtiles"]))
    slots = []
    for qt, parts in by_q.items():
        parts.sort()
        assert [p[0] for p in parts] == list(range(len(parts))) and all(p[3] == len(parts) for p in parts)
        pos = begin[qt]
        for sp, lb, nt, ns, slot in parts:
            assert lb == pos and nt >= 1
            pos += nt
            assert (slot == -1) == (ns == 1)
            if ns > 1:
                slots.append(slot)
        assert pos == begin[qt + 1]
    assert sorted(slots) == list(range(len(slots)))
    assert c["n_split_qtiles"] == sum(1 for p in by_q.values() if len(p) > 1)
    # queues: every (work item, head group) unit runs exactly once
    assert 1 <= c["n_workgroups"] <= n_wg
    units = [u for q in range(c["n_workgroups"]) for u in plan.queue(q)]
    assert sorted(units) == [(i, h0) for i in range(c["n_items"]) for h0 in range(0, hq, gs)]
    # order inside a queue: slices of split lists first, whole lists next, the closing slice of a list last (the
    # workgroup that runs it is the one the cost model charges for combining the list's partial results)
    def order_class(i):
        _, _, _, sp, ns, _ = items[i]
        return 1 if ns == 1 else (2 if sp == ns - 1 else 0)
    for q in range(c["n_workgroups"]):
        classes = [order_class(i) for i, _ in plan.queue(q)]
        assert classes == sorted(classes), (q, classes)
    assert all(it[4] <= 32 for it in items)   # slices per list: what the combining wavefront's LDS table holds
    _check_steps_against_lists(plan, c, items, hq, hkv, d, n, R, gs)
    if c["lse_queue0"] > 0:
        for q in range(c["n_workgroups"]):
            for i, _ in plan.queue(q):
                holds_window_rows = (items[i][0] + 1) * bq > n - window
                assert holds_window_rows == (q >= c["lse_queue0"]), (q, i)
        # the set of the window's workgroups is about as large as its share of the steps (it also pays for the
        # exact row sum, its unit switches and combinations, and must not finish last)
        share = sum(items[i][2] for q in range(c["lse_queue0"], c["n_workgroups"]) for i, _ in plan.queue(q)) / \
            sum(items[i][2] for q in range(c["n_workgroups"]) for i, _ in plan.queue(q))
        assert share <= 0.25
        assert share * c["n_workgroups"] - 1 <= c["n_workgroups"] - c["lse_queue0"] <= 2.5 * share * c["n_workgroups"] + 9
    loads = [sum(items[i][2] for i, _ in plan.queue(q)) for q in range(c["n_workgroups"])]
    if len(units) >= 4 * c["n_workgroups"]:
        assert max(loads) <= 1.5 * (sum(loads) / len(loads)) + max(it[2] for it in items)
    plan.close()


def _check_steps_against_lists(plan, c, items, hq, hkv, d, n, R, gs, kv_strides=None):
    """The steps a workgroup executes against the lists they were made from: every unit runs, once and in order, the
    tiles of its slice of its query tile's list, with the addresses, first/last marks and row counts the kernel relies
    on, and every (KV head, key tile) has exactly one owner step."""
    g = hq // hkv
    kv_sh, kv_st = kv_strides if kv_strides else (n * d, d)
    owners = set()
    for q in range(c["n_workgroups"]):
        steps = plan.steps(q)
        pos = 0
        for it, head0 in plan.queue(q):
            qt, lb, nt, sp, ns, slot = items[it]
            kvh = head0 // g
            first_pos = lb - _list_begin(plan, c, qt)
            want = plan.qtile_list(qt)[first_pos:first_pos + nt]
            for i, (t, need, kinds) in enumerate(want):
                kv_off, flags, got_kinds, k0 = steps[pos + i]
                assert k0 == t * pk.BK and kv_off == ((kvh * kv_sh + k0 * kv_st) * 2) % 2**32
                assert flags & 0xFFFF == need and got_kinds == kinds
                assert (flags >> 17) & 1 == (i == 0) and (flags >> 16) & 1 == (i == nt - 1)
                assert ((flags >> 18) & 63) + 1 == min(pk.BK, n - k0)
                if (flags >> 24) & 1:
                    assert (kvh, t) not in owners
                    owners.add((kvh, t))
            pos += nt
        assert pos == len(steps), q
    n_ktiles = (n + pk.BK - 1) // pk.BK
    heads_run = sorted({h0 // g for q in range(c["n_workgroups"]) for _, h0 in plan.queue(q)})
    assert sorted(owners) == [(kvh, t) for kvh in heads_run for t in range(n_ktiles)]


def _list_begin(plan, c, qt):
    """First position of query tile qt's list in the flat tile list (work items address lists by flat position)."""
    if not hasattr(plan, "_list_begin"):
        plan._list_begin = np.concatenate([[0], np.cumsum([len(plan.qtile_list(q)) for q in range(c["n_qtiles"])])])
    return int(plan._list_begin[qt])


@pytest.mark.parametrize("pattern", [0, 1, 2, 3])
@pytest.mark.parametrize("heads", [(4, 2), (7, 1), (3, 3), (12, 2)])
@pytest.mark.parametrize("shape", [(4, 8, 8, 32), (3, 5, 7, 19), (1, 9, 9, 0), (5, 16, 16, 200), (2, 24, 24, 1),
                                   (9, 1, 1, 3), (1, 1, 1, 0), (1, 1, 1, 200), (1, 6, 6, 10)])
def test_plan_lists_match_oracle_mask_small(shape, pattern, heads):
    F, ph, pw, T = shape
    _check_plan_against_oracle(F, ph, pw, T, heads[0], heads[1], 64, pattern, n_wg=16)


@pytest.mark.parametrize("name", ["videollama2_8f", "qwen25vl_32f", "qwen25vl_64f", "qwen25vl_128f_stack"])
def test_plan_lists_match_oracle_mask_benchmark_shapes(name):
    wl = WORKLOADS[name]
    _check_plan_against_oracle(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads,
                               wl.head_dim, 3)


@pytest.mark.parametrize("pattern", [0, 3])
@pytest.mark.parametrize("name", ["videollama2_8f", "qwen25vl_32f", "qwen25vl_64f", "qwen25vl_128f_stack"])
def test_window_plans_benchmark_shapes(name, pattern):
    wl = WORKLOADS[name]
    if name == "qwen25vl_128f_stack" and pattern == 0:
        pytest.skip("a million steps: the 64-frame shape covers the same code in a tenth of the time")
    _check_plan_against_oracle(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads,
                               wl.head_dim, pattern, window=wl.window)


def test_window_plan_of_the_benchmark_low_layer_is_divided():
    wl = WORKLOADS["qwen25vl_32f"]
    plan = pk.Plan.for_workload(wl, 0, host_only=True, lse_window=wl.window)
    c = plan.counts()
    q0 = c["lse_queue0"]
    assert 232 <= q0 <= 240 and q0 % 4 == 0   # 6 % of the steps, 10 % dearer, slices: 16-24 of 256 workgroups, and every
    #                                            KV head (4) keeps the same number of workgroups in both sets
    loads = [sum(plan.item(i)[2] for i, _ in plan.queue(q)) for q in range(256)]
    assert max(loads[:q0]) <= 1.03 * sum(loads[:q0]) / q0          # the large set is balanced ...
    assert sum(loads[:q0]) / q0 <= 1.03 * sum(loads) / 256          # ... and barely longer than an undivided plan's queues
    assert 1.10 * max(loads[q0:]) + 20 <= max(loads[:q0])           # the small set, with its dearer steps, ends earlier
    g = wl.n_q_heads // wl.n_kv_heads
    for q in range(256):                                            # every unit on an XCD of its KV head
        assert all((q % 8) % wl.n_kv_heads == h0 // g for _, h0 in plan.queue(q))
    plan.close()


@pytest.mark.parametrize("window", [1, 19, 32, 200, 233])
@pytest.mark.parametrize("pattern", [0, 3])
@pytest.mark.parametrize("shape", [(4, 8, 8, 32), (3, 5, 7, 19), (5, 16, 16, 200), (40, 16, 16, 64)])
def test_window_plans_small(shape, pattern, window):
    F, ph, pw, T = shape
    if window > F * ph * pw + T:
        pytest.skip("window longer than the sequence")
    _check_plan_against_oracle(F, ph, pw, T, 4, 2, 64, pattern, n_wg=16, window=window)


def test_window_plan_argument_errors():
    lib = pk.raw()
    shape = pk.Shape(4, 8, 8, 32, 4, 2, 64, 3, 0.0, 0, 0, 0, 0, 0, 0)
    h = ctypes.c_void_p()
    for w in (0, -1, 4 * 64 + 32 + 1):
        assert lib.purekv_plan_create_window_host(ctypes.byref(shape), w, 16, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_create_window_host(ctypes.byref(shape), 32, 0, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_create_window_host(ctypes.byref(shape), 4 * 64 + 32, 16, ctypes.byref(h)) == pk.OK
    c = (ctypes.c_int64 * 16)()
    assert lib.purekv_plan_counts(h, c) == pk.OK and c[14] == 4 * 64 + 32 and c[15] == 0   # every tile holds window rows
    lib.purekv_plan_destroy(h)


def test_dense_plan_benchmark_shape():
    wl = WORKLOADS["qwen25vl_32f"]
    _check_plan_against_oracle(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads,
                               wl.head_dim, 0)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: the bench says so and exits before touching torch or the GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.parametrize("pattern", [1, 2, 3])
@pytest.mark.parametrize("mask", [[1, 0, 0, 1, 0, 1, 0, 0], [0, 0, 0, 0, 0, 0, 1, 0], [1, 1, 1, 0, 1, 1, 1, 1]])
def test_head_subset_plan_lists_only_the_selected_heads(mask, pattern):
    """A plan over a head subset: one head per workgroup, the same tile lists as the plan of all heads in that
    shape, every (work item, selected head) unit exactly once and no unit of any other head; flop counts scale
    with the number of selected heads; every queue holds at least one unit."""
    F, ph, pw, T, hq, hkv, d = 3, 6, 7, 300, 8, 2, 64
    sub = pk.Plan(F, ph, pw, T, hq, hkv, d, pattern, host_only=True, n_workgroups=16, head_mask=mask)
    c = sub.counts()
    assert c["stacked_heads"] == 1 and c["row_blocks"] == pk.WAVES and c["n_head_groups"] == hq
    # the reference: the same shape with one query head per KV head is planned head by head as well
    ref = pk.Plan(F, ph, pw, T, hkv, hkv, d, pattern, host_only=True, n_workgroups=16)
    cr = ref.counts()
    assert cr["stacked_heads"] == 1 and cr["n_qtiles"] == c["n_qtiles"] and cr["n_blocks"] == c["n_blocks"]
    assert all(sub.qtile_list(q) == ref.qtile_list(q) for q in range(c["n_qtiles"]))
    sel = [h for h in range(hq) if mask[h]]
    units = [u for q in range(c["n_workgroups"]) for u in sub.queue(q)]
    assert sorted(units) == [(i, h0) for i in range(c["n_items"]) for h0 in sel]
    assert all(len(sub.queue(q)) >= 1 for q in range(c["n_workgroups"]))
    assert sub.kept_tile_flops() == 4.0 * pk.BLOCK * pk.BLOCK * d * c["n_blocks"] * len(sel)
    full = pk.Plan(F, ph, pw, T, hq, hkv, d, pattern, host_only=True, n_workgroups=16)
    assert abs(sub.mask_flops() * hq - full.mask_flops() * len(sel)) <= 1e-9 * full.mask_flops() * hq
    for p in (sub, ref, full):
        p.close()


def test_head_subset_plan_argument_errors():
    lib = pk.raw()
    good = pk.Shape(2, 4, 4, 8, 4, 2, 64, 3, 0.0)
    h = ctypes.c_void_p()
    none = (ctypes.c_uint8 * 4)(0, 0, 0, 0)
    some = (ctypes.c_uint8 * 4)(0, 1, 0, 0)
    assert lib.purekv_plan_create_heads_host(ctypes.byref(good), none, 16, ctypes.byref(h)) == pk.EINVAL   # no head
    assert lib.purekv_plan_create_heads_host(ctypes.byref(good), None, 16, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_create_heads_host(ctypes.byref(good), some, 0, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_create_heads_host(None, some, 16, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_create_heads_host(ctypes.byref(good), some, 16, None) == pk.EINVAL
    assert lib.purekv_plan_create_heads(ctypes.byref(good), None, ctypes.byref(h), None) == pk.EINVAL
    assert lib.purekv_plan_create_heads_host(ctypes.byref(good), some, 16, ctypes.byref(h)) == pk.OK
    assert lib.purekv_plan_destroy(h) == pk.OK
    with pytest.raises(ValueError):
        pk.Plan(2, 4, 4, 8, 4, 2, 64, 3, host_only=True, head_mask=[1, 0])


@pytest.mark.parametrize("mask", [[0, 0, 0, 0, 1, 1, 1, 1], [1] * 8])
def test_head_subset_of_whole_kv_groups_keeps_the_stacked_shape(mask):
    F, ph, pw, T, hq, hkv, d = 3, 6, 7, 300, 8, 2, 64
    sub = pk.Plan(F, ph, pw, T, hq, hkv, d, 3, host_only=True, n_workgroups=16, head_mask=mask)
    full = pk.Plan(F, ph, pw, T, hq, hkv, d, 3, host_only=True, n_workgroups=16)
    c, cf = sub.counts(), full.counts()
    assert c["stacked_heads"] == cf["stacked_heads"] == 4 and c["row_blocks"] == cf["row_blocks"] == 2
    assert all(sub.qtile_list(q) == full.qtile_list(q) for q in range(c["n_qtiles"]))
    units = [u for q in range(c["n_workgroups"]) for u in sub.queue(q)]
    assert sorted(units) == [(i, h0) for i in range(c["n_items"]) for h0 in range(0, hq, 4) if mask[h0]]
    assert sub.kept_tile_flops() * hq == full.kept_tile_flops() * sum(mask)
    sub.close(), full.close()


def test_plan_lists_match_oracle_mask_random_shapes():
    """Seeded sweep over odd shapes (frame sizes that are not multiples of the key tile, frames shorter than a
    row block, long and empty texts, every pattern): the planner's shortcuts for known tiles must never change a
    list, a need bit or a kind."""
    rng = np.random.default_rng(2510)
    for _ in range(60):
        ph, pw = int(rng.integers(1, 14)), int(rng.integers(1, 14))
        F = int(rng.integers(1, max(2, min(12, 1200 // (ph * pw)) + 1)))
        T = int(rng.choice([0, 1, 7, 33, 64, 129, 400]))
        hkv = int(rng.choice([1, 2, 3]))
        g = int(rng.choice([1, 2, 4, 7]))
        pattern = int(rng.integers(0, 4))
        _check_plan_against_oracle(F, ph, pw, T, hkv * g, hkv, 64, pattern, n_wg=int(rng.choice([3, 16, 256])))


def test_host_code_under_address_and_undefined_behaviour_sanitizers():
    """The planner (346 lines of index arithmetic that size device tables) and the C ABI's host half, rebuilt with
    ASan + UBSan on the host side and driven over ~2000 shapes by tests/host_sanitizer_driver.cpp: any report or failed
    structural check makes the driver exit non-zero."""
    import importlib.util
    import subprocess
    spec = importlib.util.spec_from_file_location("_purekv_build", os.path.join(ROOT, "paper_2510_25600_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    exe = mod.build_host_sanitized(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "all checks passed" in run.stdout
