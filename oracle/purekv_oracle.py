"""CPU oracle for the PureKV hot path (NumPy, fp64).

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow definition that the
GPU library is checked against.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import it; the product path never does.  It shares no code
with the HIP implementation and imports nothing from it.

Every function is the definition written out; nothing is tiled, fused or
reordered beyond blocking query rows to bound memory (rows are independent).

Notation (paper, Sec. 3.1 and 3.2):  l = N tokens = F frames x P patches of
video followed by T text tokens; w = recent window; h = number of non-recent
keys kept; A = attention probabilities; C = recent-window column sums (Eq. 2);
S = C * ||V|| (Eq. 3 / Eq. 4); rank(S) and Spearman's rho between two score vectors (Sec. 3.3, Eq. 5-7).

Readings of the paper where it is silent (all listed in the design notes):
  * spatial and temporal paths are combined as a union in one mask;
  * attention is always causal (j <= i);
  * text queries attend causally to every earlier token;
  * under GQA the score of a KV head is the sum over its query heads;
  * kept entries are stored in ascending original index, window last;
  * ties in the top-h go to the lower index, and ranks are assigned the same way (no averaged ranks).
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import Optional, Sequence, Tuple

import numpy as np

DENSE = 0
SPATIAL = 1
TEMPORAL = 2


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns (uint16) to float64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# ST-SpAttn mask (Sec. 3.2, the spatial and the temporal paragraph)
# --------------------------------------------------------------------------

def st_mask_rows(n_frames: int, patches: int, n_text: int, pattern: int,
                 rows: np.ndarray) -> np.ndarray:
    """Boolean mask M[r, j] for query rows `rows` against all N keys.

    pattern 0: dense causal (Eq. 1 with the lower-triangular structure).
    bit 0 (spatial):  key in the first frame, or in the query's own frame.
    bit 1 (temporal): key in the first frame, or the same patch of the previous
                      frame, or the query itself.
    Text queries (index >= F*P) see every earlier token.
    """
    nv = n_frames * patches
    n = nv + n_text
    i = np.asarray(rows, dtype=np.int64)[:, None]
    j = np.arange(n, dtype=np.int64)[None, :]
    causal = j <= i
    if pattern == DENSE:
        return causal
    video_i = i < nv
    video_j = j < nv
    fi, fj = i // patches, j // patches
    pi, pj = i % patches, j % patches
    allowed = np.zeros((i.shape[0], n), dtype=bool)
    if pattern & SPATIAL:
        allowed |= video_j & ((fj == 0) | (fj == fi))
    if pattern & TEMPORAL:
        allowed |= video_j & ((fj == 0) | ((fj == fi - 1) & (pj == pi)) | (j == i))
    return causal & (~video_i | allowed)


def st_mask(n_frames: int, patches: int, n_text: int, pattern: int) -> np.ndarray:
    n = n_frames * patches + n_text
    return st_mask_rows(n_frames, patches, n_text, pattern, np.arange(n))


# --------------------------------------------------------------------------
# Masked softmax attention (Eq. 1 under the mask)
# --------------------------------------------------------------------------

def attention_probs_rows(q_rows: np.ndarray, k: np.ndarray, mask_rows: np.ndarray,
                         scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """A[r, j] = softmax_j(q_r . k_j * scale) over allowed j; also row log-sum-exp."""
    s = (q_rows @ k.T) * scale
    s = np.where(mask_rows, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=1, keepdims=True)
    return e / z, (m + np.log(z))[:, 0]


def masked_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray,
                     n_frames: int, patches: int, n_text: int, pattern: int,
                     scale: Optional[float] = None,
                     rows: Optional[np.ndarray] = None,
                     heads: Optional[Sequence[int]] = None,
                     row_block: int = 1024) -> Tuple[np.ndarray, np.ndarray]:
    """O = A V for the selected query heads and rows.

    q [Hq, N, d], k/v [Hkv, N, d] float64.  Returns (O [len(heads), len(rows), d],
    LSE [len(heads), len(rows)]).  Query head hq uses KV head hq // (Hq / Hkv).
    """
    hq_total, n, d = q.shape
    group = hq_total // k.shape[0]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    rows = np.arange(n) if rows is None else np.asarray(rows, dtype=np.int64)
    heads = list(range(hq_total)) if heads is None else list(heads)
    out = np.empty((len(heads), rows.shape[0], d), dtype=np.float64)
    lse = np.empty((len(heads), rows.shape[0]), dtype=np.float64)
    for r0 in range(0, rows.shape[0], row_block):
        rr = rows[r0:r0 + row_block]
        mask = st_mask_rows(n_frames, patches, n_text, pattern, rr)
        for hi, hq in enumerate(heads):
            kv = hq // group
            a, l = attention_probs_rows(q[hq, rr], k[kv], mask, scale)
            out[hi, r0:r0 + rr.shape[0]] = a @ v[kv]
            lse[hi, r0:r0 + rr.shape[0]] = l
    return out, lse


# --------------------------------------------------------------------------
# Importance (Eq. 2), V-norm weighting (Eq. 3 / Eq. 4)
# --------------------------------------------------------------------------

def window_column_sums(q: np.ndarray, k: np.ndarray, n_frames: int, patches: int,
                       n_text: int, pattern: int, w: int,
                       scale: Optional[float] = None) -> np.ndarray:
    """C[kv, j] = sum over query heads of the group and rows i = N-w .. N-1 of A[i, j], j < N-w."""
    hq_total, n, d = q.shape
    hkv = k.shape[0]
    group = hq_total // hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    rows = np.arange(n - w, n)
    mask = st_mask_rows(n_frames, patches, n_text, pattern, rows)
    c = np.zeros((hkv, n - w), dtype=np.float64)
    for hq in range(hq_total):
        a, _ = attention_probs_rows(q[hq, rows], k[hq // group], mask, scale)
        c[hq // group] += a[:, :n - w].sum(axis=0)
    return c


def vnorm_scores(c: np.ndarray, v: np.ndarray) -> np.ndarray:
    """S[kv, j] = C[kv, j] * ||V[kv, j, :]||_2 for the non-recent keys j < C.shape[1]."""
    m = c.shape[1]
    return c * np.sqrt((v[:, :m, :] ** 2).sum(axis=2))


# --------------------------------------------------------------------------
# Selection, compaction, decode
# --------------------------------------------------------------------------

def budget(n: int, w: int, ratio: float) -> int:
    """h such that window + top-h holds floor(ratio * N) entries (never negative).

    The ratio is the decimal number as written (the paper's budgets are 5 %, 20 %, 35 %, 50 % of the
    sequence, Sec. 4.2), so the product is formed in exact rational arithmetic: floor(0.29 * 100) is 29,
    not the 28 that the binary double nearest to 0.29 would give."""
    kept = math.floor(Fraction(repr(float(ratio))) * n)
    return max(0, int(kept) - w)


def topk_select(s: np.ndarray, h: int, n: int, w: int) -> np.ndarray:
    """Per KV head: the h highest-scoring non-recent keys (ties to the lower index),
    in ascending index order, followed by the recent window N-w .. N-1."""
    hkv = s.shape[0]
    idx = np.empty((hkv, h + w), dtype=np.int32)
    for kv in range(hkv):
        order = np.argsort(-s[kv], kind="stable")
        idx[kv, :h] = np.sort(order[:h])
        idx[kv, h:] = np.arange(n - w, n)
    return idx


def score_ranks(s: np.ndarray) -> np.ndarray:
    """rank(S) of Sec. 3.3: r[..., j] = position of s[..., j] when the scores of a row are put in descending order,
    0 = the highest score; equal scores keep their index order (the tie rule of the top-h selection: the lower
    index ranks first), so the ranks of a row are always a permutation of 0 .. n-1."""
    s = np.asarray(s, dtype=np.float64)
    order = np.argsort(-s, axis=-1, kind="stable")
    ranks = np.empty(s.shape, dtype=np.int64)
    np.put_along_axis(ranks, order, np.broadcast_to(np.arange(s.shape[-1], dtype=np.int64), s.shape), axis=-1)
    return ranks


def spearman_rank_correlation(s_hat: np.ndarray, s: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Spearman's rank correlation of Sec. 3.3 (Eq. 5-7) between the estimated scores s_hat (Eq. 4: low-layer column
    sums, the layer's own V norms) and the scores s of the layer's own attention (Eq. 6), row by row over the last
    axis (n = l - w non-recent keys):  rho = 1 - 6 sum_j (r_hat_j - r_j)^2 / (n (n^2 - 1)).
    Returns (sum of squared rank differences as exact integers, rho in fp64 from exact rational arithmetic)."""
    n = s.shape[-1]
    if n < 2 or s_hat.shape != s.shape:
        raise ValueError("two score arrays of the same shape with at least two scores a row")
    d = score_ranks(s_hat) - score_ranks(s)
    sum_d2 = np.array([sum(int(x) * int(x) for x in row) for row in d.reshape(-1, n)], dtype=object).reshape(d.shape[:-1])
    denom = n * (n * n - 1)
    rho = np.array([float(1 - Fraction(6 * int(x), denom)) for x in sum_d2.reshape(-1)], dtype=np.float64).reshape(d.shape[:-1])
    return sum_d2, rho


def stack_pattern(layer: int, st_layer: int, sparse_pattern: int = 3) -> int:
    """Attention pattern of a layer of the stack: dense below the first ST-SpAttn layer (Sec. 3.1: the lower layers
    compute attention scores), the sparse pattern from there on (Sec. 3.2; layer-index study of Sec. 4.5)."""
    return 0 if layer < st_layer else sparse_pattern


def stack_selection(c_layers, v_layers, clie_layer: int, h: int, n: int, w: int):
    """Kept indices of every layer of a stack.  A layer below the estimating layer has column sums of its own and is
    scored with them (Eq. 3); the estimating layer and every later one are scored with the estimating layer's column
    sums and their own V (Eq. 4).  c_layers[l] is only read for l <= clie_layer."""
    return [topk_select(vnorm_scores(c_layers[min(l, clie_layer)], v), h, n, w) for l, v in enumerate(v_layers)]


def compact(k_bits: np.ndarray, v_bits: np.ndarray, idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Kc[kv, r, :] = K[kv, idx[kv, r], :] on raw bit patterns; V likewise."""
    hkv = k_bits.shape[0]
    kc = np.stack([k_bits[kv, idx[kv]] for kv in range(hkv)])
    vc = np.stack([v_bits[kv, idx[kv]] for kv in range(hkv)])
    return kc, vc


def decode_attention(q_new: np.ndarray, kc: np.ndarray, vc: np.ndarray,
                     scale: Optional[float] = None) -> np.ndarray:
    """o[hq] = softmax(q_new[hq] . Kc[kv]^T * scale) Vc[kv]; q_new [Hq, d], kc/vc [Hkv, n, d]."""
    hq_total, d = q_new.shape
    group = hq_total // kc.shape[0]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    out = np.empty((hq_total, d), dtype=np.float64)
    for hq in range(hq_total):
        kv = hq // group
        s = (kc[kv] @ q_new[hq]) * scale
        e = np.exp(s - s.max())
        out[hq] = (e / e.sum()) @ vc[kv]
    return out
