"""GPU parity of the generation-phase cache update (pyr_decode_update) against the float64 oracle."""
import numpy as np
import pytest

from oracle import pyr_oracle as orc
from paper_2405_12532_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
F64 = synth.bf16_bits_to_f64


def window_queries(q_bits, seq_offsets, w):
    """[B, w, Hq, d] bit patterns: the last min(w, S_b) query rows of every sequence, right-aligned; the unused
    slots hold a bf16 NaN pattern, which would poison the result if it were ever read."""
    B = len(seq_offsets) - 1
    out = np.full((B, w) + q_bits.shape[1:], 0x7FC1, dtype=np.uint16)
    for b in range(B):
        S = int(seq_offsets[b + 1] - seq_offsets[b])
        L = min(w, S)
        if L:
            out[b, w - L:] = q_bits[seq_offsets[b + 1] - L:seq_offsets[b + 1]]
    return out


def run_and_check(lib, wl, row_weights=None, with_pos=False, scale=0.0):
    x = parity.inputs(wl, lib, want_hidden=False)
    off, keep = x["seq_offsets"], x["keep_len"]
    q_win = window_queries(x["q"], off, wl.w)
    pos = np.random.default_rng(3).integers(0, 1 << 20, x["k"].shape[0]).astype(np.int32) if with_pos else None
    res = lib.decode_update_from_numpy(q_win, x["k"], x["v"], off, keep, wl.w, softmax_scale=scale,
                                       row_weights=row_weights, pos=pos)
    qw = F64(q_win.reshape(-1)).reshape(q_win.shape)
    ref = orc.decode_update(qw, F64(x["k"]), F64(x["v"]), off, wl.w, keep, scale=scale if scale > 0 else None,
                            row_weights=row_weights, pos=pos)
    rel = parity.check_scores(res["scores"], ref)
    same, swapped = parity.check_index_sets(res["kept_idx"], ref, off, keep, wl.w)
    assert res["out_offsets"].tolist() == ref["out_offsets"].tolist()
    kidx = res["kept_idx"]
    assert np.array_equal(res["k_out"], x["k"][kidx]) and np.array_equal(res["v_out"], x["v"][kidx])
    if with_pos:
        assert np.array_equal(res["pos_out"], pos[kidx])
    for b in range(wl.n_seqs):
        if off[b + 1] > off[b]:
            assert abs(float(res["scores"][off[b]:off[b + 1]].astype(np.float64).sum()) - 1.0) < 1e-4
    print(f"[{wl.name} decode] score rel {rel:.2e}; identical index sets {same}/{wl.n_seqs}, swapped in band {swapped}")
    return res, ref, x


@pytest.mark.parametrize("lens,Hq,Hkv,d,w", [
    ((300, 97, 513, 20), 4, 2, 128, 32),      # ragged, GQA 2, one sequence shorter than the window
    ((1, 2, 31, 33, 64, 65), 2, 2, 64, 16),   # tiny sequences, d 64
    ((700,), 8, 1, 128, 64),                  # GQA 8
    ((256, 512, 768), 8, 8, 64, 48),          # exact multiples of the key block
    ((1000, 40), 16, 8, 128, 100),            # window not a multiple of 32, a sequence of S < w
])
def test_decode_update_small_shapes(lib, lens, Hq, Hkv, d, w):
    wl = synth.shrunk(synth.workload("cfg2"), lens, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, w=w, hidden_dim=0)
    run_and_check(lib, wl)


def test_decode_update_weights_positions_scale(lib):
    wl = synth.shrunk(synth.workload("cfg2"), (333, 100, 7), n_q_heads=4, n_kv_heads=4, head_dim=64, w=20, hidden_dim=0)
    rw = (np.arange(1, 21, dtype=np.float32) / 20) ** 2
    rw[3] = 0.0
    run_and_check(lib, wl, row_weights=rw, with_pos=True, scale=0.2)


def test_decode_update_agrees_with_the_prefill_step(lib):
    """On an uncompressed prompt the update is the prefill step's score pass with denominators found anew."""
    wl = synth.shrunk(synth.workload("cfg2"), (600, 129), n_q_heads=8, n_kv_heads=4, head_dim=128, w=64, hidden_dim=0)
    res, ref, x = run_and_check(lib, wl)
    pre = lib.prefill_layer_from_numpy(x, wl.w)
    np.testing.assert_allclose(res["scores"], pre["scores"], rtol=2e-5, atol=1e-12)


def test_decode_update_at_bench_shape_sampled(lib):
    """Heads and head dim of the 64x2k workload, caches of up to 2048 rows."""
    wl = synth.shrunk(synth.workload("64x2k"), (2048, 1984, 1500, 2048))
    run_and_check(lib, wl)


def test_decode_fixed_budget_generation(lib):
    """Token by token with a fixed PvC budget (Section 4.1: unbounded input): every step's update is checked
    against the oracle on the same cache, then the GPU's result becomes the next cache."""
    rng = np.random.default_rng(9)
    B, Hq, Hkv, d, w, budget = 3, 4, 2, 64, 8, 40
    start = [30, 5, 39]
    def rnd(shape):
        t = torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(np.uint16)
    k = [rnd((n, Hkv, d)) for n in start]
    v = [rnd((n, Hkv, d)) for n in start]
    qs = [rnd((n, Hq, d)) for n in start]                     # queries of the tokens still in the window (and before)
    pos = [np.arange(n, dtype=np.int32) for n in start]
    nxt = list(start)
    for step in range(24):
        for b in range(B):                                    # append the new token of every sequence
            k[b] = np.concatenate([k[b], rnd((1, Hkv, d))]); v[b] = np.concatenate([v[b], rnd((1, Hkv, d))])
            qs[b] = np.concatenate([qs[b], rnd((1, Hq, d))])[-w:]
            pos[b] = np.concatenate([pos[b], [nxt[b]]]).astype(np.int32); nxt[b] += 1
        lens = [a.shape[0] for a in k]
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        keep = np.array([min(n, budget) for n in lens])
        q_win = np.full((B, w, Hq, d), 0x7FC1, dtype=np.uint16)
        for b in range(B):
            L = min(w, lens[b])
            q_win[b, w - L:] = qs[b][-L:]
        kk, vv, pp = np.concatenate(k), np.concatenate(v), np.concatenate(pos)
        res = lib.decode_update_from_numpy(q_win, kk, vv, off, keep, w, pos=pp)
        ref = orc.decode_update(F64(q_win.reshape(-1)).reshape(q_win.shape), F64(kk), F64(vv), off, w, keep, pos=pp)
        parity.check_scores(res["scores"], ref)
        parity.check_index_sets(res["kept_idx"], ref, off, keep, w)
        oo = res["out_offsets"]
        assert oo.tolist() == np.concatenate([[0], np.cumsum(keep)]).tolist()
        for b in range(B):
            k[b], v[b], pos[b] = res["k_out"][oo[b]:oo[b + 1]], res["v_out"][oo[b]:oo[b + 1]], res["pos_out"][oo[b]:oo[b + 1]]
            assert k[b].shape[0] <= budget and np.all(np.diff(pos[b]) > 0)
            Lb = min(w, lens[b])
            assert pos[b][-Lb:].tolist() == list(range(nxt[b] - Lb, nxt[b]))   # the window is the newest tokens
    print(f"[decode generation] 24 steps, budget {budget}: cache sizes {[a.shape[0] for a in k]}")


def test_decode_update_with_empty_sequences(lib):
    wl = synth.shrunk(synth.workload("cfg2"), (0, 130, 0, 9, 0), n_q_heads=4, n_kv_heads=2, head_dim=128, w=32,
                      hidden_dim=0)
    run_and_check(lib, wl, with_pos=True)
