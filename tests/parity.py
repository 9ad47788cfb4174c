"""Shared comparison helpers of the GPU parity tests (no GPU code, no oracle arithmetic)."""
import numpy as np

from oracle import pyr_oracle as orc

OUT_MAX_ABS = 2e-2        # attention output, bf16 in / fp32 accumulate
OUT_MEAN_ABS = 2e-3
SCORE_RTOL = 1e-3         # token scores
SCORE_ATOL = 1e-10        # only guards scores that are exactly or almost zero
BAND = 1e-3               # relative half-width of the tie band at the k-th score


def keep_lens(wl, lib=None):
    """Keep count of every sequence of a workload.  The input generator only names the rule
    (ratio, floor); the oracle side evaluates it with the oracle's schedule and, when `lib` (the
    C-ABI binding) is given, the library side with pyr_schedule_next: both must agree before
    anything is launched with them."""
    num, den, floor = wl.schedule_args()
    ref = np.asarray([orc.schedule_next(S, wl.w, num, den, floor) for S in wl.seq_lens], dtype=np.int32)
    if lib is not None:
        got = np.asarray([lib.schedule_next(S, wl.w, num, den, floor) for S in wl.seq_lens], dtype=np.int32)
        assert got.tolist() == ref.tolist(), "library and oracle schedules disagree"
    return ref


def inputs(wl, lib=None, **kw):
    """synth.make_inputs plus the keep counts (see keep_lens)."""
    from paper_2405_12532_amd import synth
    x = synth.make_inputs(wl, **kw)
    x["keep_len"] = keep_lens(wl, lib)
    return x


def check_index_sets(kept_gpu, ref, seq_offsets, keep_len, w):
    """kept_gpu must equal the oracle's set except inside the band around the oracle's k-th
    largest context score; it must always be sorted, unique, of the right length and contain
    the recent window.  Returns (n_sequences_identical, n_positions_in_band_swapped)."""
    oo = ref["out_offsets"]
    identical, swapped = 0, 0
    for b in range(len(keep_len)):
        r0, S = int(seq_offsets[b]), int(seq_offsets[b + 1] - seq_offsets[b])
        L = min(w, S)
        g = np.asarray(kept_gpu[oo[b]:oo[b + 1]], dtype=np.int64) - r0
        r = np.asarray(ref["kept_idx"][oo[b]:oo[b + 1]], dtype=np.int64) - r0
        assert len(g) == keep_len[b]
        if len(g) == 0:
            identical += 1
            continue
        assert np.all(np.diff(g) > 0), "kept positions must be strictly ascending"
        assert g.min() >= 0 and g.max() < S
        assert g[len(g) - L:].tolist() == list(range(S - L, S)), "the recent window is always kept"
        if np.array_equal(g, r):
            identical += 1
            continue
        sc = ref["scores"][r0:r0 + S]
        tau = sc[r[: len(r) - L]].min()                      # oracle's k-th largest context score
        diff = np.setxor1d(g, r)
        assert np.all(np.abs(sc[diff] - tau) <= BAND * tau), "index sets differ outside the tie band"
        swapped += len(diff) // 2
    return identical, swapped


def check_out(out_bits_gpu, ref, seq_offsets, to_f64):
    """Attention output against the oracle on the rows the oracle evaluated."""
    tot_abs, n, mx = 0.0, 0, 0.0
    for b, rows in enumerate(ref["out_rows"]):
        if len(rows) == 0:
            continue
        g = to_f64(out_bits_gpu[int(seq_offsets[b]) + np.asarray(rows)])
        e = np.abs(g - ref["out"][b])
        mx = max(mx, float(e.max()))
        tot_abs += float(e.sum())
        n += e.size
    mean = tot_abs / max(n, 1)
    assert mx <= OUT_MAX_ABS, f"attention output max-abs error {mx}"
    assert mean <= OUT_MEAN_ABS, f"attention output mean-abs error {mean}"
    return mx, mean


def check_scores(scores_gpu, ref):
    np.testing.assert_allclose(scores_gpu, ref["scores"], rtol=SCORE_RTOL, atol=SCORE_ATOL)
    denom = np.maximum(ref["scores"], 1e-30)
    return float(np.max(np.abs(scores_gpu - ref["scores"]) / denom))
