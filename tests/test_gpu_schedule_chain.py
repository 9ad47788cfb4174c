"""Layer chains on the GPU whose lengths come from pyr_schedule_plan (Algorithm 1: a minimum PvC length N_l per
layer and a retention ratio p that decays from layer to layer; Section 5, "PvC Length Decay").

The three decay patterns of the ablation are read as follows (the paper gives one figure per pattern): the
cache length falls by 15 % / 10 % / 7 % of the prompt over the first half of the layers, geometrically, and the
ratio of the second half is the one geometric ratio that brings the mean length over all layers to 60 % of the
prompt, so the three plans cost the same memory.  Plans are integer ratios num[l]/1000.

Every layer of every chain: lengths from the library's plan, equal to the oracle's plan; the whole layer step
against the oracle (attention output, scores, index sets, bit-exact gathers); hidden rows and position ids
carried from layer to layer and compared at the end with the composed index."""
import numpy as np
import pytest

from oracle import pyr_oracle as orc
from paper_2405_12532_amd import synth
from tests.test_gpu_layer import run_and_check

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

DEN = 1000


def decay_plan(n_layers, first_half_drop, mean_target=0.6):
    """num[l] (over DEN) of one of the ablation's patterns, as read above."""
    half = n_layers // 2
    pa = (1.0 - first_half_drop) ** (1.0 / half)

    def mean_len(pb):
        cur, tot = 1.0, 0.0
        for l in range(n_layers):
            tot += cur                                  # layer l attends over the length it receives
            cur *= pa if l < half else pb
        return tot / n_layers

    lo, hi = 0.0, 1.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if mean_len(mid) > mean_target:
            hi = mid
        else:
            lo = mid
    return [int(round(DEN * (pa if l < half else hi))) for l in range(n_layers)]


def run_chain(lib, lens0, nums, floors, context_relative, Hq=8, Hkv=4, d=128, w=32, D=128, seed_layer0=0):
    base = synth.shrunk(synth.workload("cfg2"), lens0, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, w=w, hidden_dim=D)
    n_layers = len(nums)
    plans = [lib.schedule_plan(S, w, nums, DEN, floors, context_relative) for S in lens0]
    for S, p in zip(lens0, plans):
        assert p == [int(v) for v in orc.schedule_plan(S, w, nums, DEN, floors, context_relative)]
    hid0 = synth.make_hidden(base)
    hidden = hid0
    origin = np.arange(sum(lens0), dtype=np.int64)
    pos = np.concatenate([np.arange(S, dtype=np.int32) for S in lens0])
    identity_layers = 0
    for l in range(n_layers):
        lens = [p[l] for p in plans]
        wl = synth.shrunk(base, lens)
        x = synth.make_inputs(wl, layer=seed_layer0 + l, want_hidden=False)
        x["hidden"] = hidden
        x["keep_len"] = np.asarray([p[l + 1] for p in plans], dtype=np.int32)
        identity_layers += int(all(p[l + 1] == p[l] for p in plans))
        res, ref, _ = run_and_check(lib, wl, x=x, pos=pos)
        kept = res["kept_idx"]
        assert np.array_equal(res["hidden_out"], hidden[kept])
        hidden, pos, origin = res["hidden_out"], res["pos_out"], origin[kept]
    assert [len(hidden)] == [sum(p[-1] for p in plans)]
    assert np.array_equal(hidden, hid0[origin]), "surviving hidden rows are the original rows at the composed index"
    off0 = np.concatenate([[0], np.cumsum(lens0)])
    seq_of = np.searchsorted(off0, origin, side="right") - 1
    assert np.array_equal(pos, (origin - off0[seq_of]).astype(np.int32)), "position ids name the original places"
    return plans, identity_layers


LENS = (700, 512, 300, 257, 90, 40)


@pytest.mark.parametrize("name,drop", [("reduce_more", 0.15), ("uniform", 0.10), ("power_law", 0.07)])
def test_decay_patterns_at_equal_memory(lib, name, drop):
    n_layers = 16
    nums = decay_plan(n_layers, drop)
    plans, _ = run_chain(lib, LENS, nums, [0] * n_layers, False)
    p = plans[0]
    mean = sum(p[:n_layers]) / (n_layers * p[0])
    print(f"[{name}] ratios/1000 {nums}; lengths of the {p[0]}-token sequence {p}; mean length {mean:.3f} of the prompt")
    assert abs(p[n_layers // 2] / p[0] - (1.0 - drop)) < 0.01        # the first half drops what the pattern says
    assert abs(mean - 0.6) < 0.02                                     # ... at the same memory for all three


def test_context_relative_ratio(lib):
    """p as a fraction of the context columns (Algorithm 1 ranks A[-L:, :-L] only): k = L' + half_up(p (S - L'))."""
    n_layers = 6
    plans, _ = run_chain(lib, LENS, [800] * n_layers, [0] * n_layers, True, seed_layer0=20)
    for S, p in zip(LENS, plans):
        L = min(32, S)
        assert p[1] == L + (800 * (S - L) + DEN // 2) // DEN


def test_minimum_pvc_lengths_stop_compression_mid_stack(lib):
    """N_l per layer: layers whose input is at or below N_l pass it on unchanged (identity layers), here from
    layer 3 on for every sequence, and already from the start for the short ones."""
    nums = [700, 700, 700, 700, 700, 700]
    floors = [100, 100, 100, 4096, 4096, 150]
    plans, identity_layers = run_chain(lib, LENS, nums, floors, False, seed_layer0=40)
    assert identity_layers == 2
    for S, p in zip(LENS, plans):
        assert p[3] == p[4] == p[5]
        assert p[6] == max((700 * p[5] + DEN // 2) // DEN, min(150, p[5]), min(32, p[5]))
    assert plans[4] == [90] * 6 + [90] and plans[5] == [40] * 7      # at or below every floor: never compressed
