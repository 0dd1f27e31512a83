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
    assert len(declared) >= 17
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
        rc = lib.purekv_plan_create_host(ctypes.byref(s), ctypes.byref(h))
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
    assert lib.purekv_plan_create_host(None, ctypes.byref(h)) == pk.EINVAL
    assert lib.purekv_plan_create_host(ctypes.byref(pk.Shape(**good)), None) == pk.EINVAL
    assert lib.purekv_plan_destroy(None) == pk.OK


def test_compute_calls_validate_before_touching_the_gpu():
    """A host-only plan cannot be launched; null pointers and bad sizes are refused with EINVAL."""
    lib = pk.raw()
    plan = pk.Plan(2, 4, 4, 8, 4, 2, 64, host_only=True)
    h = plan.handle
    one = ctypes.c_void_p(16)  # never dereferenced: validation fails first
    assert lib.purekv_st_spattn_prefill(h, one, one, one, one, None, None, 0, None) == pk.EINVAL
    assert lib.purekv_st_spattn_prefill(None, one, one, one, one, None, None, 0, None) == pk.EINVAL
    assert lib.purekv_lowlayer_importance(h, one, one, one, 8, one, None, 0, None) == pk.EINVAL
    assert lib.purekv_topk_select(h, one, None, 0, 1, 8, 4, one, None, None, 0, None) == pk.EINVAL
    assert lib.purekv_kv_compact(h, one, one, 0, 1, one, 4, one, one, 4, None) == pk.EINVAL
    assert lib.purekv_kv_append(h, one, one, one, one, 0, 4, None) == pk.EINVAL
    assert lib.purekv_decode_attn(h, one, one, one, 4, 4, one, one, 1 << 20, None) == pk.EINVAL
    assert lib.purekv_workspace_bytes(None, pk.OP_PREFILL, 0, 0, 0) == 0
    c = (ctypes.c_int64 * 6)()
    assert lib.purekv_plan_counts(None, c) == pk.EINVAL and lib.purekv_plan_counts(h, None) == pk.EINVAL
    assert lib.purekv_plan_qtile_list(h, 99, None, 0) == pk.EINVAL
    assert lib.purekv_plan_item(h, -1, (ctypes.c_int32 * 6)()) == pk.EINVAL


def test_budget_matches_oracle_rule():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        n = int(rng.integers(1, 70000))
        w = int(rng.integers(1, n + 1))
        r = float(rng.choice([0.05, 0.1, 0.2, 0.33, 0.35, 0.5, rng.random()]))
        assert pk.purekv_budget(n, w, r) == orc.budget(n, w, r)
    assert pk.purekv_budget(8448, 256, 0.2) == 1433


def _block_part(wl_shape, pattern, rows):
    """The oracle's mask with the temporal path's side keys (previous-frame key, self key) removed."""
    F, P, T = wl_shape
    nv = F * P
    m = orc.st_mask_rows(F, P, T, pattern, rows).copy()
    if pattern != 0 and (pattern & 2):
        for r, i in enumerate(rows):
            if i < nv and i // P >= 2:
                assert m[r, i - P]
                m[r, i - P] = False
            if i < nv and not (pattern & 1) and i // P >= 1:
                assert m[r, i]
                m[r, i] = False
    return m


def _check_plan_against_oracle(F, ph, pw, T, hq, hkv, d, pattern):
    P, n = ph * pw, F * ph * pw + T
    plan = pk.Plan(F, ph, pw, T, hq, hkv, d, pattern, host_only=True)
    c = plan.counts()
    assert c["N"] == n and c["n_qtiles"] == (n + pk.BQ - 1) // pk.BQ
    n_ktiles = (n + pk.BK - 1) // pk.BK
    total_pairs = 0
    refs = 0
    for qt in range(c["n_qtiles"]):
        rows = np.arange(qt * pk.BQ, min((qt + 1) * pk.BQ, n))
        full_mask = orc.st_mask_rows(F, P, T, pattern, rows)
        total_pairs += int(full_mask.sum())
        b = _block_part((F, P, T), pattern, rows)
        padded = np.zeros((rows.shape[0], n_ktiles * pk.BK), dtype=bool)
        padded[:, :n] = b
        per_tile = padded.reshape(rows.shape[0], n_ktiles, pk.BK)
        any_t = per_tile.any(axis=(0, 2))
        all_t = per_tile.all(axis=(0, 2))
        lst = plan.qtile_list(qt)
        refs += len(lst)
        assert [t for t, _ in lst] == np.nonzero(any_t)[0].tolist(), (qt, pattern)
        assert [f for _, f in lst] == all_t[any_t].astype(int).tolist(), (qt, pattern)
    assert refs == c["n_tile_refs"]
    assert abs(plan.mask_flops() - 4.0 * d * total_pairs * hq) < 1e-3 * max(1.0, plan.mask_flops())
    assert plan.kept_tile_flops() == 4.0 * pk.BQ * pk.BK * d * refs * hq
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
    plan.close()


@pytest.mark.parametrize("pattern", [0, 1, 2, 3])
@pytest.mark.parametrize("shape", [(4, 8, 8, 32), (3, 5, 7, 19), (1, 9, 9, 0), (5, 16, 16, 200), (2, 24, 24, 1)])
def test_plan_lists_match_oracle_mask_small(shape, pattern):
    F, ph, pw, T = shape
    _check_plan_against_oracle(F, ph, pw, T, 4, 2, 64, pattern)


@pytest.mark.parametrize("name", ["videollama2_8f", "qwen25vl_32f", "qwen25vl_64f", "qwen25vl_128f_stack"])
def test_plan_lists_match_oracle_mask_benchmark_shapes(name):
    wl = WORKLOADS[name]
    _check_plan_against_oracle(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads,
                               wl.head_dim, 3)


def test_dense_plan_benchmark_shape():
    wl = WORKLOADS["qwen25vl_32f"]
    _check_plan_against_oracle(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, wl.n_q_heads, wl.n_kv_heads,
                               wl.head_dim, 0)
