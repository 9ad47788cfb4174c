"""Float64 CPU oracle for one PyramidInfer prefill layer step.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, dense
implementation of what the GPU library computes, written from the paper
(PyramidInfer, arXiv 2405.12532) and used only by the tests, by the smoke
check and by the benchmark's CPU-baseline leg.  It shares no code with the
HIP path and never calls it.

The step, following Algorithm 1 ("One forward pass in PyramidInfer") and
Section 4.1 (prefill phase), for every sequence of a packed batch:

  1. attention weights A of the layer: the ordinary causal softmax
     (Algorithm 1, "compute attention weights of KV");
  2. ensemble weights A_e: the average, over the last L query rows (the
     recent sequence S_r) and over heads, of the weight each row gives to a
     key (Algorithm 1, weighted_avg(A[-L:, :-L]); Section 3.2.1 describes
     the averaging of the weights of subsequent tokens);
  3. TopP: keep the context keys with the largest A_e, a fixed count of them
     (Section 3.1.1 calls p a retention ratio), the recent window always
     survives because A_e only ranks the columns :-L;
  4. Gather: K, V and the hidden rows of the kept tokens, in position order,
     form the shorter sequence the next layer sees (Algorithm 1, Gather;
     Figure 2(c): only the crucial keys and values are computed further on);
  5. the retention count shrinks from layer to layer and never drops below
     the minimum PvC length N_l (Algorithm 1, the len(KV) > N_l guard and the
     decay of p).

Readings taken where the paper leaves a choice (each listed in the design
notes of this repository): averaging weights are an input, uniform unless
given, normalised by their sum; mean over all query
heads gives one index set per sequence; with grouped-query attention query
head h reads key/value head h // (Hq // Hkv); the softmax of a recent row
runs over all its causal columns, recent ones included; ties in the top-k
go to the lower position; keep counts are rounded half-up in integers.

Pins (see tests/test_oracle_*.py): brute-force loops on tiny inputs, the
float64 library attention routine of PyTorch, closed forms for K = 0 and for
constant V, the row-sum and score-sum invariants, one-hot and split averaging
weights, exhaustive top-k on tiny score vectors, exact rational arithmetic for
the schedule, positions carried through two layers against the composed index,
the generation-phase update against the prefill step on the same rows and against
scalar loops.  No function here
is "parity unpinned" against the mathematics; nothing can be pinned against
numbers printed in the paper because it prints none for this step.
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "attention_rows",
    "causal_attention",
    "consistency_score",
    "select_pvc",
    "gather_rows",
    "gather_positions",
    "schedule_next",
    "schedule_plan",
    "prefill_layer",
    "decode_update",
]


def _softmax_scale(d: int, scale) -> float:
    return float(scale) if (scale is not None and scale > 0) else 1.0 / np.sqrt(float(d))


def attention_rows(q, k, v, rows, scale=None):
    """Causal softmax attention of ONE sequence, evaluated on chosen rows.

    Algorithm 1, "compute attention weights of KV" (the standard causal
    attention of a decoder layer).

    q: [S, Hq, d], k, v: [S, Hkv, d] float64; rows: 1-D int array of query
    positions.  Query head h uses key/value head h // (Hq // Hkv).
    Returns (out [len(rows), Hq, d], P [Hq, len(rows), S]) with
    P[h, r, j] = softmax_j(scale * q[rows[r], h] . k[j, h//g]) over j <= rows[r]
    and exact zeros for j > rows[r].
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    S, Hq, d = q.shape
    Hkv = k.shape[1]
    assert Hq % Hkv == 0 and k.shape == v.shape and k.shape[0] == S
    g = Hq // Hkv
    sc = _softmax_scale(d, scale)
    n = rows.shape[0]
    out = np.zeros((n, Hq, d), dtype=np.float64)
    P = np.zeros((Hq, n, S), dtype=np.float64)
    cols = np.arange(S, dtype=np.int64)
    visible = cols[None, :] <= rows[:, None]           # [n, S] causal mask
    for h in range(Hq):
        kh = k[:, h // g, :]
        vh = v[:, h // g, :]
        s = sc * (q[rows, h, :] @ kh.T)                # [n, S]
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        e = np.exp(s)                                  # exp(-inf) = 0 on masked columns
        p = e / e.sum(axis=1, keepdims=True)
        P[h] = p
        out[:, h, :] = p @ vh
    return out, P


def causal_attention(q, k, v, scale=None):
    """All rows of attention_rows; returns out [S, Hq, d] only."""
    S = np.asarray(q).shape[0]
    out, _ = attention_rows(q, k, v, np.arange(S), scale)
    return out


def consistency_score(q, k, w, scale=None, row_weights=None):
    """Ensemble attention weight of every key of ONE sequence.

    Algorithm 1, A_e = weighted_avg(A[-L:, :-L], dim=-2), and the mean over heads:
        score[t] = 1/Hq * sum_h sum_{i=S-L'}^{S-1} omega_i A_h[i, t] / sum_i omega_i,  L' = min(L, S).
    row_weights=None gives the uniform average (omega_i = 1).  Otherwise row_weights is a
    vector of L non-negative numbers, one per row of a full recent window in position order
    (Section 4.1, prefill phase: more recent rows may be given larger weights; the paper
    prints no values, so they are an input).  A sequence shorter than the window uses the
    LAST L' of them: the most recent row always takes row_weights[L-1].
    The vector is returned for ALL S columns (the recent columns too, where
    causality zeroes part of the rows) so that it sums to one; only the
    first S - L' entries are candidates for eviction.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    S, Hq, d = q.shape
    L = min(int(w), S)
    rows = np.arange(S - L, S)
    if row_weights is None:
        omega = np.ones(L, dtype=np.float64)
    else:
        rw = np.asarray(row_weights, dtype=np.float64)
        if rw.shape != (int(w),) or np.any(rw < 0) or not np.all(np.isfinite(rw)):
            raise ValueError("row_weights must hold w finite non-negative numbers")
        omega = rw[int(w) - L:]
        if not omega.sum() > 0:
            raise ValueError("the weights of the rows in use must not all be zero")
    # v does not enter the weights; pass k in its place to reuse the routine.
    _, P = attention_rows(q, k, k, rows, scale)         # [Hq, L', S]
    return np.einsum("hrs,r->s", P, omega) / (float(Hq) * omega.sum())


def select_pvc(score, w, keep_len):
    """Positions of ONE sequence that survive, ascending.

    Algorithm 1, TopP(A_e, p) followed by keeping the recent window: the
    keep_len - L' context positions with the largest score (ties: lower
    position first) together with the last L' positions.
    """
    score = np.asarray(score)
    S = score.shape[0]
    L = min(int(w), S)
    keep_len = int(keep_len)
    if not (L <= keep_len <= S):
        raise ValueError("keep_len must lie in [min(w, S), S]")
    n_ctx = S - L
    need = keep_len - L
    ctx = score[:n_ctx]
    order = np.argsort(-ctx, kind="stable")            # descending, equal scores keep position order
    chosen = np.sort(order[:need])
    recent = np.arange(n_ctx, S, dtype=np.int64)
    return np.concatenate([chosen.astype(np.int64), recent])


def gather_rows(x, idx):
    """Algorithm 1, Gather(KV, index): rows of x at idx, in that order."""
    return np.asarray(x)[np.asarray(idx, dtype=np.int64)]


def gather_positions(pos, idx):
    """Position ids of the kept tokens: pos[idx].

    Appendix A.2 (Table 5): after tokens are evicted the survivors keep the position
    encodings they had, gathered with the same index as the keys and values, instead of
    being renumbered 0..k-1.  Carried through every layer, pos always names the token's
    place in the original prompt.
    """
    return np.asarray(pos)[np.asarray(idx, dtype=np.int64)]


def schedule_next(S, w, num, den, floor_len):
    """Keep count for the next layer.

    Algorithm 1: the ratio p shrinks layer by layer and no compression
    happens once the length is at or below the minimum PvC length.  With the
    ratio num/den applied to the whole surviving length and rounded half-up:
        k = max(floor((num*S + den//2) / den), floor_len, min(w, S)), capped at S.
    """
    S, w, num, den, floor_len = int(S), int(w), int(num), int(den), int(floor_len)
    if S < 0 or w < 1 or den <= 0 or num < 0 or num > den or floor_len < 0:
        raise ValueError("bad schedule arguments")
    k = (num * S + den // 2) // den
    k = max(k, floor_len, min(w, S))
    return min(k, S)


def schedule_plan(S, w, nums, den, floors, context_relative=False):
    """Lengths of one sequence through a stack of layers: [S_0, S_1, ..., S_n].

    Algorithm 1 with a ratio and a minimum PvC length of its own per layer (input N = {N_0, ..., N_l, ...};
    "reduce p by multiplying a decay ratio", so p_l is whatever sequence the caller chose: geometric, or the
    patterns of the decay ablation of Section 5).  Layer l keeps
        whole-length reading:   k = round_half_up(p_l * S_l)
        context reading:        k = L' + round_half_up(p_l * (S_l - L')),  L' = min(w, S_l)
    (Algorithm 1 ranks only the columns :-L, so read literally p is a fraction of the context), then
    k = max(k, N_l, L') capped at S_l, and S_{l+1} = k.
    """
    S, w, den = int(S), int(w), int(den)
    if len(nums) != len(floors):
        raise ValueError("one ratio and one minimum length per layer")
    out = [S]
    for num, floor_len in zip(nums, floors):
        num, floor_len = int(num), int(floor_len)
        if context_relative:
            if S < 0 or w < 1 or den <= 0 or num < 0 or num > den or floor_len < 0:
                raise ValueError("bad schedule arguments")
            L = min(w, S)
            k = L + (num * (S - L) + den // 2) // den
            S = min(max(k, floor_len, L), S)
        else:
            S = schedule_next(S, w, num, den, floor_len)
        out.append(S)
    return out


def prefill_layer(q, k, v, seq_offsets, w, keep_len, scale=None, hidden=None, out_rows=None, row_weights=None,
                  pos=None):
    """One layer step over a packed batch.

    q: [T, Hq, d]; k, v: [T, Hkv, d]; seq_offsets: int [B+1]; keep_len: int [B];
    hidden: optional [T, D]; row_weights: optional [w] (see consistency_score); pos: optional
    int [T], position ids of the rows.  out_rows: None (all rows) or a list with, per
    sequence, the local query positions at which `out` is evaluated (the
    scores, the selection and the gathers are always complete).

    Returns a dict: out (list per sequence of [n_rows, Hq, d]), out_rows,
    scores [T], kept_idx (global packed rows, int64 [T']), out_offsets [B+1],
    k_out, v_out, hidden_out, pos_out.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    seq_offsets = np.asarray(seq_offsets, dtype=np.int64)
    keep_len = np.asarray(keep_len, dtype=np.int64)
    B = seq_offsets.shape[0] - 1
    T = q.shape[0]
    assert seq_offsets[0] == 0 and seq_offsets[-1] == T
    scores = np.zeros(T, dtype=np.float64)
    outs, rows_used, kept = [], [], []
    out_offsets = np.zeros(B + 1, dtype=np.int64)
    for b in range(B):
        r0, r1 = int(seq_offsets[b]), int(seq_offsets[b + 1])
        S = r1 - r0
        if S == 0:
            outs.append(np.zeros((0,) + q.shape[1:]))
            rows_used.append(np.zeros(0, dtype=np.int64))
            out_offsets[b + 1] = out_offsets[b]
            continue
        qb, kb, vb = q[r0:r1], k[r0:r1], v[r0:r1]
        rows = np.arange(S) if out_rows is None else np.asarray(out_rows[b], dtype=np.int64)
        o, _ = attention_rows(qb, kb, vb, rows, scale)
        outs.append(o)
        rows_used.append(rows)
        sb = consistency_score(qb, kb, w, scale, row_weights)
        scores[r0:r1] = sb
        sel = select_pvc(sb, w, keep_len[b])
        kept.append(sel + r0)
        out_offsets[b + 1] = out_offsets[b] + sel.shape[0]
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, dtype=np.int64)
    res = {
        "out": outs,
        "out_rows": rows_used,
        "scores": scores,
        "kept_idx": kept_idx,
        "out_offsets": out_offsets,
        "k_out": gather_rows(k, kept_idx),
        "v_out": gather_rows(v, kept_idx),
    }
    if hidden is not None:
        res["hidden_out"] = gather_rows(hidden, kept_idx)
    if pos is not None:
        res["pos_out"] = gather_positions(pos, kept_idx)
    return res


def decode_update(q_win, k, v, seq_offsets, w, keep_len, scale=None, row_weights=None, pos=None):
    """Generation-phase update of one layer's compressed cache (Algorithm 1 run with a
    non-empty cache: KV = cat(PvC_past, KV); Section 4.1, generation phase: the recent
    window slides over the newly generated tokens and the PvC is selected again, "the
    operation is the same as the prefill phase").

    k, v: [T, Hkv, d], the packed caches AFTER the new tokens' rows were appended: per
    sequence the kept context rows followed by the recent rows, S_b rows in all.
    q_win: [B, w, Hq, d], the queries of the recent rows, right-aligned: q_win[b, w-1] is
    the newest token's query; a sequence with S_b < w uses the last S_b slots.
    Row i of the window (cache row S_b - L' + i) sees every cache row up to itself.
    The ensemble weights, the selection and the gathers are those of the prefill step.
    Returns scores [T], kept_idx, out_offsets, k_out, v_out (and pos_out).
    """
    q_win = np.asarray(q_win, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    seq_offsets = np.asarray(seq_offsets, dtype=np.int64)
    keep_len = np.asarray(keep_len, dtype=np.int64)
    B = seq_offsets.shape[0] - 1
    T = k.shape[0]
    w = int(w)
    assert q_win.shape[0] == B and q_win.shape[1] == w
    scores = np.zeros(T, dtype=np.float64)
    kept = []
    out_offsets = np.zeros(B + 1, dtype=np.int64)
    for b in range(B):
        r0, r1 = int(seq_offsets[b]), int(seq_offsets[b + 1])
        S = r1 - r0
        if S == 0:
            out_offsets[b + 1] = out_offsets[b]
            continue
        L = min(w, S)
        # the score only reads the last L' query rows: place them there, the rest is never touched
        qb = np.full((S,) + q_win.shape[2:], np.nan)
        qb[S - L:] = q_win[b, w - L:]
        sb = consistency_score(qb, k[r0:r1], w, scale, row_weights)
        scores[r0:r1] = sb
        sel = select_pvc(sb, w, keep_len[b])
        kept.append(sel + r0)
        out_offsets[b + 1] = out_offsets[b] + sel.shape[0]
    kept_idx = np.concatenate(kept) if kept else np.zeros(0, dtype=np.int64)
    res = {"scores": scores, "kept_idx": kept_idx, "out_offsets": out_offsets,
           "k_out": gather_rows(k, kept_idx), "v_out": gather_rows(v, kept_idx)}
    if pos is not None:
        res["pos_out"] = gather_positions(pos, kept_idx)
    return res
