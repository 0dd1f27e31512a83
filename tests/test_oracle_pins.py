"""Pins for the CPU oracle: closed forms, invariants, library special cases and brute force.

None of these re-types the oracle's own formula: each checks the oracle against
something fixed by the mathematics or by an independent construction, so that a
dropped term, a wrong sign or index, or a transposed operand fails at least one.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import purekv_oracle as orc
from workloads import WORKLOADS, generate, small_variant, f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _f64(bits):
    return orc.bf16_bits_to_f64(bits)


def _tiny():
    wl = WORKLOADS["tiny_4f"]
    inp = generate(wl)
    return wl, _f64(inp.q), _f64(inp.k), _f64(inp.v), inp


# ------------------------------------------------------------------ inputs / bf16

def test_bf16_roundtrip_matches_torch():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(4096).astype(np.float32) * 37.0
    bits = f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits, t.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(_f64(bits), t.to(torch.float64).numpy())


def test_generator_structure():
    wl = WORKLOADS["tiny_4f"]
    a, b = generate(wl), generate(wl)
    assert np.array_equal(a.k, b.k) and np.array_equal(a.q, b.q)
    assert a.q.shape == (2, 288, 64) and a.k.shape == (1, 288, 64)
    assert a.salient.shape == (12,) and len(set(a.salient.tolist())) == 12
    v = _f64(a.v)[0, :256].reshape(4, 64, 64)
    # frame-to-frame redundancy: successive V frames differ by noise of std ~0.1
    diff = (v[1:] - v[:-1]).std()
    assert 0.07 < diff < 0.13
    k = _f64(a.k)[0, :256]
    sal = np.zeros(256, bool)
    sal[a.salient] = True
    assert k[sal].std() > 2.5 * k[~sal].std()


# ------------------------------------------------------------------ mask

def _mask_triple_loop(F, ph, pw, T, pattern):
    """Independent construction: loops over (frame, patch) pairs, no index arithmetic on i, j."""
    P = ph * pw
    toks = [("v", f, p) for f in range(F) for p in range(P)] + [("t", t, 0) for t in range(T)]
    n = len(toks)
    m = np.zeros((n, n), dtype=bool)
    for i, (ki, fi, pi) in enumerate(toks):
        for j in range(i + 1):
            kj, fj, pj = toks[j]
            if pattern == 0 or ki == "t":
                m[i, j] = True
                continue
            if kj == "t":
                continue
            ok = False
            if pattern & 1:
                ok |= (fj == 0) or (fj == fi)
            if pattern & 2:
                ok |= (fj == 0) or (fj + 1 == fi and pj == pi) or (j == i)
            m[i, j] = ok
    return m


@pytest.mark.parametrize("pattern", [0, 1, 2, 3])
@pytest.mark.parametrize("shape", [(4, 2, 3, 5), (1, 3, 3, 4), (2, 2, 2, 0), (3, 1, 1, 2)])
def test_mask_against_triple_loop(shape, pattern):
    F, ph, pw, T = shape
    got = orc.st_mask(F, ph * pw, T, pattern)
    assert np.array_equal(got, _mask_triple_loop(F, ph, pw, T, pattern))


def test_mask_nnz_closed_form_and_rows():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "mask_nnz.txt")) if l.strip() and l[0] != "#"]
    for F, P, T, nnz in [(int(a), int(b), int(c), int(d)) for a, b, c, d in rows]:
        nv, n = F * P, F * P + T
        if n <= 9000:
            m = orc.st_mask(F, P, T, 3)
            assert int(m.sum()) == nnz
            cnt = m.sum(1)
        else:  # big shapes: row blocks
            cnt = np.concatenate([orc.st_mask_rows(F, P, T, 3, np.arange(r, min(r + 2048, n))).sum(1)
                                  for r in range(0, n, 2048)])
            assert int(cnt.sum()) == nnz
        i = np.arange(nv)
        f, p = i // P, i % P
        expect = np.where(f == 0, p + 1, np.where(f == 1, P + p + 1, P + p + 2))
        assert np.array_equal(cnt[:nv], expect)
        assert np.array_equal(cnt[nv:], nv + np.arange(T) + 1)
    # spatial-only drops exactly the previous-frame keys
    F, P, T = 4, 64, 32
    assert int(orc.st_mask(F, P, T, 1).sum()) == 29456 - P * (F - 2)
    # temporal-only: frame 0 causal; frame 1: P0 + self; frames >= 2: P0 + prev + self
    mt = orc.st_mask(F, P, T, 2).sum(1)
    assert np.array_equal(mt[:P], np.arange(P) + 1)
    assert np.all(mt[P:2 * P] == P + 1) and np.all(mt[2 * P:F * P] == P + 2)


def test_mask_is_lower_triangular_and_has_diagonal():
    for pattern in (0, 1, 2, 3):
        m = orc.st_mask(3, 6, 4, pattern)
        assert not np.triu(m, 1).any()
        assert np.diag(m).all()


# ------------------------------------------------------------------ attention

def test_dense_pattern_equals_library_sdpa():
    wl, q, k, v, _ = _tiny()
    out, lse = orc.masked_attention(q, k, v, wl.n_frames, wl.patches, wl.n_text, 0)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(wl.group, 0)[None], tv.repeat_interleave(wl.group, 0)[None],
        is_causal=True)[0].numpy()
    assert np.abs(out - ref).max() < 1e-12
    # log-sum-exp against the library routine
    s = torch.einsum("hid,hjd->hij", tq, tk.repeat_interleave(wl.group, 0)) / math.sqrt(wl.head_dim)
    s = s.masked_fill(~torch.tril(torch.ones(s.shape[1:], dtype=torch.bool)), -math.inf)
    assert np.abs(lse - torch.logsumexp(s, -1).numpy()).max() < 1e-12


def test_rows_sum_to_one_and_respect_mask():
    wl, q, k, v, _ = _tiny()
    rows = np.arange(wl.n_tokens)
    for pattern in (0, 1, 2, 3):
        mask = orc.st_mask_rows(wl.n_frames, wl.patches, wl.n_text, pattern, rows)
        a, _ = orc.attention_probs_rows(q[1], k[0], mask, 0.125)
        assert np.abs(a.sum(1) - 1).max() < 1e-12
        assert (a[~mask] == 0).all() and (a[mask] > 0).all()


def test_sparse_attention_equals_bruteforce_loops():
    """Tiny 1-head case against per-row Python loops written from the definition."""
    F, ph, pw, T, d = 3, 2, 2, 3, 8
    P, n = ph * pw, 3 * 4 + 3
    rng = np.random.default_rng(5)
    q, k, v = (_f64(f32_to_bf16_bits(rng.standard_normal((1, n, d)).astype(np.float32))) for _ in range(3))
    for pattern in (0, 1, 2, 3):
        m = _mask_triple_loop(F, ph, pw, T, pattern)
        out, lse = orc.masked_attention(q, k, v, F, P, T, pattern)
        for i in range(n):
            js = [j for j in range(n) if m[i, j]]
            logits = [sum(q[0, i, c] * k[0, j, c] for c in range(d)) / math.sqrt(d) for j in js]
            mx = max(logits)
            ws = [math.exp(x - mx) for x in logits]
            z = sum(ws)
            o = [sum(ws[t] * v[0, j, c] for t, j in enumerate(js)) / z for c in range(d)]
            assert np.abs(out[0, i] - np.array(o)).max() < 1e-12
            assert abs(lse[0, i] - (mx + math.log(z))) < 1e-12


def test_identical_keys_give_mean_of_allowed_values():
    wl, q, k, v, _ = _tiny()
    k_same = np.broadcast_to(k[:, :1], k.shape).copy()
    out, _ = orc.masked_attention(q, k_same, v, wl.n_frames, wl.patches, wl.n_text, 3)
    m = orc.st_mask(wl.n_frames, wl.patches, wl.n_text, 3)
    expect = (m.astype(np.float64) @ v[0]) / m.sum(1, keepdims=True)
    assert np.abs(out[0] - expect).max() < 1e-12 and np.abs(out[1] - expect).max() < 1e-12


def test_identical_values_pass_through_and_dominant_key_wins():
    wl, q, k, v, _ = _tiny()
    v_same = np.broadcast_to(v[:, 7:8], v.shape).copy()
    out, _ = orc.masked_attention(q, k, v_same, wl.n_frames, wl.patches, wl.n_text, 3)
    assert np.abs(out - v[0, 7]).max() < 1e-12
    # key 5 (first frame: visible to every row >= 5) made to dominate row 200 of head 0
    k2 = k.copy()
    k2[0, 5] = 40.0 * q[0, 200]
    out2, _ = orc.masked_attention(q, k2, v, wl.n_frames, wl.patches, wl.n_text, 3, rows=np.array([200]), heads=[0])
    assert np.abs(out2[0, 0] - v[0, 5]).max() < 1e-9


def test_gqa_head_mapping():
    """Query head hq must read KV head hq // G: make KV heads distinguishable."""
    wl = small_variant("gqa", n_q_heads=4, n_kv_heads=2)
    inp = generate(wl)
    q, k, v = _f64(inp.q), _f64(inp.k), _f64(inp.v)
    v[0] = 1.0
    v[1] = -2.0
    out, _ = orc.masked_attention(q, k, v, wl.n_frames, wl.patches, wl.n_text, 3)
    assert np.allclose(out[:2], 1.0) and np.allclose(out[2:], -2.0)


# ------------------------------------------------------------------ importance

def test_column_sums_identical_keys_harmonic_closed_form():
    wl, q, k, v, _ = _tiny()
    n, w, g = wl.n_tokens, wl.window, wl.group
    k_same = np.broadcast_to(k[:, :1], k.shape).copy()
    c = orc.window_column_sums(q, k_same, wl.n_frames, wl.patches, wl.n_text, 0, w)
    # row i spreads 1/(i+1) on each key: sum_{i=N-w}^{N-1} 1/(i+1) = H_N - H_{N-w}
    expect = g * sum(1.0 / (i + 1) for i in range(n - w, n))
    assert c.shape == (1, n - w)
    assert np.abs(c - expect).max() < 1e-12


def test_column_sums_mass_conservation_and_bruteforce():
    wl, q, k, v, _ = _tiny()
    n, w, g = wl.n_tokens, wl.window, wl.group
    scale = 1 / math.sqrt(wl.head_dim)
    for pattern, win in ((0, w), (3, w), (3, 100), (0, n)):
        c = orc.window_column_sums(q, k, wl.n_frames, wl.patches, wl.n_text, pattern, win)
        mask = orc.st_mask(wl.n_frames, wl.patches, wl.n_text, pattern)
        full = np.zeros(n)
        for hq in range(wl.n_q_heads):  # explicit full matrix A, summed over the window rows
            a, _ = orc.attention_probs_rows(q[hq], k[0], mask, scale)
            full += a[n - win:].sum(0)
        assert (c >= 0).all()
        assert c.shape == (1, n - win)
        assert np.abs(c[0] - full[:n - win]).max(initial=0.0) < 1e-12
        assert abs(c.sum() + full[n - win:].sum() - win * g) < 1e-10
    # independent check of one column through the library softmax
    s = torch.from_numpy(q[0] @ k[0].T * scale).masked_fill(
        ~torch.tril(torch.ones(n, n, dtype=torch.bool)), -math.inf)
    s1 = torch.from_numpy(q[1] @ k[0].T * scale).masked_fill(
        ~torch.tril(torch.ones(n, n, dtype=torch.bool)), -math.inf)
    col = (torch.softmax(s, -1)[n - w:, 17].sum() + torch.softmax(s1, -1)[n - w:, 17].sum()).item()
    c = orc.window_column_sums(q, k, wl.n_frames, wl.patches, wl.n_text, 0, w)
    assert abs(c[0, 17] - col) < 1e-12


def test_vnorm_against_library_norm():
    wl, q, k, v, _ = _tiny()
    c = np.random.default_rng(2).random((1, 256))
    s = orc.vnorm_scores(c, v)
    assert np.abs(s - c * np.linalg.norm(v[:, :256], axis=2)).max() < 1e-12
    v_unit = v / np.linalg.norm(v, axis=2, keepdims=True)
    assert np.abs(orc.vnorm_scores(c, v_unit) - c).max() < 1e-12


# ------------------------------------------------------------------ selection / compaction / decode

def test_topk_against_bruteforce_sort_with_ties():
    rng = np.random.default_rng(3)
    n, w = 200, 16
    s = rng.integers(0, 12, size=(3, n - w)).astype(np.float64)  # many ties
    for h in (0, 1, 17, n - w):
        idx = orc.topk_select(s, h, n, w)
        for kv in range(3):
            ranked = sorted(range(n - w), key=lambda j: (-s[kv, j], j))[:h]
            assert idx[kv, :h].tolist() == sorted(ranked)
            assert idx[kv, h:].tolist() == list(range(n - w, n))
    same = np.ones((1, n - w))
    assert orc.topk_select(same, 9, n, w)[0, :9].tolist() == list(range(9))


def test_budget_matches_paper_ratio():
    frac, factor, reduction = [float(x) for x in
                               [l for l in open(os.path.join(GOLDEN, "budget_ratios.txt")) if l[0] != "#"][0].split()]
    for wl in WORKLOADS.values():
        n, w = wl.n_tokens, wl.window
        h = orc.budget(n, w, frac)
        kept = h + w
        assert kept <= frac * n < kept + 1
        assert n / kept >= factor > n / (kept + 1)
        assert abs(100 * (1 - kept / n) - reduction) < 0.5
    assert orc.budget(100, 50, 0.2) == 0
    assert [orc.budget(16640, 256, r) for r in (0.1, 0.2, 0.33)] == [1408, 3072, 5235]
    assert orc.budget(8448, 256, 0.2) == 1433 and orc.budget(4736, 128, 0.2) == 819
    # the ratio is the decimal number as written: integer arithmetic on percent and per-mille values
    for n in (100, 288, 1000, 4736, 8448, 16640, 33280):
        for pct in range(0, 101):
            assert orc.budget(n, 0, pct / 100) == (pct * n) // 100, (n, pct)
        for pm in range(0, 1001, 7):
            assert orc.budget(n, 3, pm / 1000) == max(0, (pm * n) // 1000 - 3), (n, pm)


def test_salient_keys_are_selected():
    wl, q, k, v, inp = _tiny()
    n, w = wl.n_tokens, wl.window
    c = orc.window_column_sums(q, k, wl.n_frames, wl.patches, wl.n_text, 0, w)
    s = orc.vnorm_scores(c, v)
    idx = orc.topk_select(s, orc.budget(n, w, 0.2), n, w)
    kept = set(idx[0].tolist())
    hit = sum(1 for j in inp.salient if j in kept)
    assert hit >= 0.75 * len(inp.salient)  # sanity (not parity): x3 keys draw the window's attention


def test_compaction_roundtrip_and_decode_equals_masked_full_attention():
    wl, q, k, v, inp = _tiny()
    n, w = wl.n_tokens, wl.window
    rng = np.random.default_rng(4)
    idx = orc.topk_select(rng.random((1, n - w)), 25, n, w)
    kc, vc = orc.compact(inp.k, inp.v, idx)
    assert kc.dtype == np.uint16 and kc.shape == (1, 57, 64)
    back = np.zeros_like(inp.k)
    back[0, idx[0]] = kc[0]
    assert np.array_equal(back[0, idx[0]], inp.k[0, idx[0]]) and np.array_equal(vc[0, 3], inp.v[0, idx[0, 3]])
    # decode on the compacted cache (plus the new token's own k, v) equals dense attention of the new
    # query over the full K/V restricted to "key is kept" -- computed here with the library softmax
    qn, kn, vn = _f64(inp.q_new[0]), _f64(inp.k_new[0]), _f64(inp.v_new[0])
    kcat = np.concatenate([_f64(kc), kn[:, None]], 1)
    vcat = np.concatenate([_f64(vc), vn[:, None]], 1)
    o = orc.decode_attention(qn, kcat, vcat)
    kept = np.zeros(n + 1, bool)
    kept[idx[0]] = True
    kept[n] = True
    kfull = np.concatenate([k[0], kn], 0)
    vfull = np.concatenate([v[0], vn], 0)
    for hq in range(wl.n_q_heads):
        s = torch.from_numpy(kfull @ qn[hq] / math.sqrt(wl.head_dim))
        s[torch.from_numpy(~kept)] = -math.inf
        ref = (torch.softmax(s, 0).numpy() @ vfull)
        assert np.abs(o[hq] - ref).max() < 1e-12


def test_stack_selection_shares_the_estimating_layers_column_sums():
    """Layer stack: a layer below the estimating layer is selected with its own column sums, the estimating
    layer and every later one with the estimating layer's.  Pinned by construction: every layer gets a C that
    puts all its mass on a set of keys of its own, and the same all-ones V, so the kept set names the C that
    was used; a V that zeroes one key in one layer only must drop that key there and nowhere else."""
    n, w, h, hkv, d, layers, clie = 40, 4, 5, 2, 8, 5, 2
    rng = np.random.default_rng(9)
    hot = [np.sort(rng.choice(n - w, size=h, replace=False)) for _ in range(layers)]
    c_layers = []
    for l in range(layers):
        c = np.full((hkv, n - w), 1e-3)
        c[:, hot[l]] = 1.0 + np.arange(h)
        c_layers.append(c)
    v_layers = [np.ones((hkv, n, d)) for _ in range(layers)]
    idx = orc.stack_selection(c_layers, v_layers, clie, h, n, w)
    for l in range(layers):
        want = hot[min(l, clie)]
        for kv in range(hkv):
            assert np.array_equal(idx[l][kv, :h], want) and np.array_equal(idx[l][kv, h:], np.arange(n - w, n))
    # Eq. 4 weighs the shared C with the layer's OWN V
    v_layers[4][:, hot[clie][0], :] = 0.0
    idx2 = orc.stack_selection(c_layers, v_layers, clie, h, n, w)
    assert hot[clie][0] not in idx2[4][0, :h] and np.array_equal(idx2[3], idx[3])
    assert [orc.stack_pattern(l, 3) for l in range(5)] == [0, 0, 0, 3, 3] and orc.stack_pattern(4, 5) == 0


# ------------------------------------------------------------------ several KV heads (GQA indexing)
# Every pin above that touches column sums, V-norms, compaction or decode runs on one KV head, where
# "query head hq reads KV head hq // G" cannot be told from hq % Hkv, nor idx[kv] from idx[0].  The pins
# below use Hq = 6, Hkv = 3 (G = 2: hq // G = 0 0 1 1 2 2, hq % Hkv = 0 1 2 0 1 2) with KV heads that can be
# told apart, and never call the oracle to build their expected values.

def _gqa_inputs(seed=11):
    wl = small_variant("gqa_3kv", n_frames=3, patch_h=3, patch_w=4, n_text=9, n_q_heads=6, n_kv_heads=3, head_dim=16)
    inp = generate(wl, seed=seed, decode_steps=1)
    return wl, _f64(inp.q), _f64(inp.k), _f64(inp.v), inp


def _library_probs(q_h, k_h, mask, scale):
    s = torch.from_numpy(q_h @ k_h.T * scale).masked_fill(~torch.from_numpy(mask), -math.inf)
    return torch.softmax(s, -1).numpy()


@pytest.mark.parametrize("pattern", [0, 3])
def test_column_sums_per_kv_head_against_library_softmax(pattern):
    """Eq. 2 under GQA: the column sums of KV head kv collect the query heads kv*G .. kv*G+G-1, each scored
    against THAT head's keys.  Expected values from the library softmax on explicit per-head matrices."""
    wl, q, k, v, _ = _gqa_inputs()
    n, w, g = wl.n_tokens, 7, wl.group
    scale = 1 / math.sqrt(wl.head_dim)
    mask = _mask_triple_loop(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, pattern)
    c = orc.window_column_sums(q, k, wl.n_frames, wl.patches, wl.n_text, pattern, w)
    assert c.shape == (3, n - w)
    for kv in range(3):
        expect = np.zeros(n)
        for hq in (kv * g, kv * g + 1):
            expect += _library_probs(q[hq], k[kv], mask, scale)[n - w:].sum(0)
        assert np.abs(c[kv] - expect[:n - w]).max() < 1e-12
        # the other heads' expected values are far away: a wrong head mapping cannot pass by accident
        other = np.zeros(n)
        for hq in (kv, kv + 3):   # the query heads hq % Hkv == kv
            other += _library_probs(q[hq], k[hq // g], mask, scale)[n - w:].sum(0)
        assert np.abs(c[kv] - other[:n - w]).max() > 1e-3


def test_column_sums_harmonic_value_only_on_the_head_with_identical_keys():
    """One KV head whose keys are all identical gives G * (H_N - H_{N-w}) on every column of ITS row of C
    (closed form, dense pattern); the other KV heads, with distinct keys, do not."""
    wl, q, k, v, _ = _gqa_inputs()
    n, w, g = wl.n_tokens, wl.window, wl.group
    harmonic = g * sum(1.0 / (i + 1) for i in range(n - w, n))
    for same in range(3):
        k2 = k.copy()
        k2[same] = k[same, :1]
        c = orc.window_column_sums(q, k2, wl.n_frames, wl.patches, wl.n_text, 0, w)
        for kv in range(3):
            dev = np.abs(c[kv] - harmonic).max()
            assert (dev < 1e-12) if kv == same else (dev > 1e-2)


def test_vnorm_per_kv_head_constant_norms():
    """Eq. 3: a V whose rows all have norm 2, 3, 5 in KV heads 0, 1, 2 scales each head's C by that number."""
    rng = np.random.default_rng(12)
    hkv, n, d, m = 3, 30, 16, 23
    v = rng.standard_normal((hkv, n, d))
    norms = np.array([2.0, 3.0, 5.0])
    v *= (norms[:, None] / np.sqrt((v * v).sum(2)))[:, :, None]
    c = rng.random((hkv, m)) + 0.1
    s = orc.vnorm_scores(c, v)
    assert s.shape == (hkv, m)
    for kv in range(hkv):
        assert np.abs(s[kv] / c[kv] - norms[kv]).max() < 1e-12
    # one key of one head zeroed: only that entry of that head drops to zero
    v[1, 4] = 0.0
    s2 = orc.vnorm_scores(c, v)
    assert s2[1, 4] == 0.0 and np.array_equal(np.delete(s2.ravel(), 1 * m + 4), np.delete(s.ravel(), 1 * m + 4))


def test_compaction_uses_each_heads_own_index_list():
    """Rows carry (head, row) in their bits, every KV head has a different index list: row r of head kv of the
    compact cache must be row idx[kv, r] of head kv, checked element by element in Python."""
    hkv, n, d, keep = 3, 20, 4, 6
    k_bits = np.zeros((hkv, n, d), np.uint16)
    v_bits = np.zeros((hkv, n, d), np.uint16)
    for kv in range(hkv):
        for j in range(n):
            k_bits[kv, j] = 1000 * kv + 10 * j + np.arange(d)
            v_bits[kv, j] = 40000 + 1000 * kv + 10 * j + np.arange(d)
    idx = np.array([[0, 2, 4, 6, 8, 19], [1, 3, 5, 7, 9, 11], [12, 13, 14, 15, 16, 17]], np.int32)
    kc, vc = orc.compact(k_bits, v_bits, idx)
    assert kc.shape == (hkv, keep, d) and vc.shape == (hkv, keep, d)
    for kv in range(hkv):
        for r in range(keep):
            for e in range(d):
                assert kc[kv, r, e] == 1000 * kv + 10 * int(idx[kv, r]) + e
                assert vc[kv, r, e] == 40000 + 1000 * kv + 10 * int(idx[kv, r]) + e


def test_decode_reads_the_kv_head_of_the_query_heads_group():
    """Decode under GQA: with V constant per KV head (1, 2, 3) the output of query head hq is hq // G + 1
    whatever the scores; with real V, every query head equals the library softmax over ITS group's cache."""
    wl, q, k, v, inp = _gqa_inputs()
    g, d = wl.group, wl.head_dim
    qn = _f64(inp.q_new[0])
    kc, vc = k[:, 5:25], v[:, 5:25]
    v_const = np.empty_like(vc)
    for kv in range(3):
        v_const[kv] = kv + 1.0
    o = orc.decode_attention(qn, kc, v_const)
    assert o.shape == (6, d)
    for hq in range(6):
        assert np.abs(o[hq] - (hq // g + 1.0)).max() < 1e-12
    o = orc.decode_attention(qn, kc, vc)
    for hq in range(6):
        p = torch.softmax(torch.from_numpy(kc[hq // g] @ qn[hq] / math.sqrt(d)), 0).numpy()
        assert np.abs(o[hq] - p @ vc[hq // g]).max() < 1e-12
        p_wrong = torch.softmax(torch.from_numpy(kc[hq % 3] @ qn[hq] / math.sqrt(d)), 0).numpy()
        if hq % 3 != hq // g:
            assert np.abs(o[hq] - p_wrong @ vc[hq % 3]).max() > 1e-3


def test_attention_and_lse_per_kv_head_against_library_softmax():
    """Prefill under GQA with real K/V: every query head against the library softmax over its group's K/V."""
    wl, q, k, v, _ = _gqa_inputs()
    scale = 1 / math.sqrt(wl.head_dim)
    mask = _mask_triple_loop(wl.n_frames, wl.patch_h, wl.patch_w, wl.n_text, 3)
    out, lse = orc.masked_attention(q, k, v, wl.n_frames, wl.patches, wl.n_text, 3)
    for hq in range(6):
        kv = hq // wl.group
        a = _library_probs(q[hq], k[kv], mask, scale)
        assert np.abs(out[hq] - a @ v[kv]).max() < 1e-12
        s = torch.from_numpy(q[hq] @ k[kv].T * scale).masked_fill(~torch.from_numpy(mask), -math.inf)
        assert np.abs(lse[hq] - torch.logsumexp(s, -1).numpy()).max() < 1e-12


# ---- Spearman's rank correlation (Sec. 3.3, Eq. 5-7) --------------------------------------------------------------

def _ranks_by_definition(s):
    """rank of s_j = number of scores that come before it in descending order, ties to the lower index: two loops."""
    n = len(s)
    return [sum(1 for k in range(n) if s[k] > s[j] or (s[k] == s[j] and k < j)) for j in range(n)]


def test_score_ranks_equal_the_definition_including_ties():
    rng = np.random.default_rng(40)
    for n in (2, 3, 17, 64):
        for _ in range(5):
            s = rng.integers(0, 5, size=n).astype(np.float64)      # many ties
            s[rng.integers(0, n)] = -0.0
            assert orc.score_ranks(s).tolist() == _ranks_by_definition(s.tolist())
    s = rng.standard_normal((3, 4, 50))
    r = orc.score_ranks(s)
    assert r.shape == s.shape
    for a in range(3):
        for b in range(4):
            assert r[a, b].tolist() == _ranks_by_definition(s[a, b].tolist())
            assert sorted(r[a, b].tolist()) == list(range(50))     # a permutation


def test_spearman_closed_forms():
    n = 1000
    x = np.arange(n, dtype=np.float64)
    d2, rho = orc.spearman_rank_correlation(x[None], x[None])
    assert d2[0] == 0 and rho[0] == 1.0                                            # identical rankings
    d2, rho = orc.spearman_rank_correlation(x[None], -x[None])
    assert d2[0] == n * (n * n - 1) // 3 and rho[0] == -1.0                         # reversed: sum d^2 = n(n^2-1)/3
    y = x.copy()
    y[[10, 11]] = y[[11, 10]]                                                       # one adjacent transposition
    d2, rho = orc.spearman_rank_correlation(x[None], y[None])
    assert d2[0] == 2 and abs(rho[0] - (1 - 12 / (n * (n * n - 1)))) < 1e-18
    # five scores, ranks differ by (1, -1, 0, 0, 0): rho = 1 - 6 * 2 / (5 * 24) = 0.9
    d2, rho = orc.spearman_rank_correlation(np.array([[5., 4., 3., 2., 1.]]), np.array([[4., 5., 3., 2., 1.]]))
    assert d2[0] == 2 and rho[0] == 0.9
    with pytest.raises(ValueError):
        orc.spearman_rank_correlation(np.zeros((1, 1)), np.zeros((1, 1)))


def test_spearman_against_the_library_routine_and_invariances():
    scipy_stats = pytest.importorskip("scipy.stats")
    rng = np.random.default_rng(41)
    for n in (2, 3, 10, 257, 4096):
        a, b = rng.standard_normal(n), rng.standard_normal(n)
        b = 0.6 * a + 0.8 * b                                                       # correlated, tie-free
        _, rho = orc.spearman_rank_correlation(a[None], b[None])
        assert abs(rho[0] - scipy_stats.spearmanr(a, b).statistic) < 1e-12
        # symmetric; unchanged by strictly increasing maps of either argument; sign flips under a decreasing one
        _, rho_ba = orc.spearman_rank_correlation(b[None], a[None])
        _, rho_mono = orc.spearman_rank_correlation(np.exp(a)[None], (3 * b + 7)[None])
        _, rho_neg = orc.spearman_rank_correlation(a[None], -b[None])
        assert rho_ba[0] == rho[0] and rho_mono[0] == rho[0] and abs(rho_neg[0] + rho[0]) < 1e-15
    # rows are independent
    s_hat, s = rng.standard_normal((2, 3, 100)), rng.standard_normal((2, 3, 100))
    d2, rho = orc.spearman_rank_correlation(s_hat, s)
    assert d2.shape == (2, 3)
    for i in range(2):
        for j in range(3):
            d2_1, rho_1 = orc.spearman_rank_correlation(s_hat[i, j][None], s[i, j][None])
            assert d2[i, j] == d2_1[0] and rho[i, j] == rho_1[0]


def test_spearman_of_a_planted_mistake_is_caught_by_the_pins():
    """The pins above tell a wrong rank convention apart: ascending ranks give the same rho (so they are no mistake),
    but ranks that break ties to the HIGHER index, or a denominator n (n^2 + 1), do not survive them."""
    s = np.array([1.0, 1.0, 0.0])
    assert orc.score_ranks(s).tolist() == [0, 1, 2]                    # ties: lower index first
    wrong = np.argsort(np.argsort(-s[::-1], kind="stable"), kind="stable")[::-1]   # ties to the higher index
    assert wrong.tolist() != [0, 1, 2]
    n = 5
    assert 1 - 6 * 2 / (n * (n * n + 1)) != 0.9
