"""The merged layer step (pyr_prefill_layer_fused: attention, score pass with the KV heads split over workgroups
at small batch, selection, one gather for K, V, hidden rows and position ids) against the
oracle and against the same step through the separate entry points."""
import numpy as np
import pytest

from paper_2405_12532_amd import synth
from tests import parity
from tests.test_gpu_layer import run_and_check, sample_rows

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def separate_calls(lib, x, wl, pos):
    """attention, score, select, K+V gather, hidden gather, position gather: six launches through the C ABI."""
    q, k, v = (lib.to_device_bf16(x[n]) for n in ("q", "k", "v"))
    hid = lib.to_device_bf16(x["hidden"])
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    off_h = torch.from_numpy(np.ascontiguousarray(x["seq_offsets"], dtype=np.int32))
    keep_h = torch.from_numpy(np.ascontiguousarray(x["keep_len"], dtype=np.int32))
    off_d, keep_d = off_h.cuda(), keep_h.cuda()
    n_kept = int(keep_h.sum())
    shape = lib.make_shape(wl.n_seqs, T, max(wl.seq_lens), Hq, Hkv, d)
    lse = torch.empty((T, Hq), dtype=torch.float32, device="cuda")
    tile_map = torch.empty(wl.n_seqs + 1, dtype=torch.int32, device="cuda")
    out = torch.empty_like(q)
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    kept = torch.empty(n_kept, dtype=torch.int32, device="cuda")
    out_off = torch.empty(wl.n_seqs + 1, dtype=torch.int32, device="cuda")
    k_out = torch.empty((n_kept, Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)
    hid_out = torch.empty((n_kept, hid.shape[1]), dtype=torch.bfloat16, device="cuda")
    pos_d = torch.from_numpy(pos).cuda()
    pos_out = torch.empty(n_kept, dtype=torch.int32, device="cuda")
    lib.attention(q, k, v, off_d, off_h, shape, 0.0, out, lse, tile_map)
    lib.score(q, k, lse, off_d, off_h, shape, wl.w, 0.0, scores)
    lib.select(scores, off_d, off_h, keep_d, keep_h, wl.n_seqs, wl.w, kept, out_off)
    lib.compact2(k, k_out, v, v_out, Hkv * d * 2, kept, n_kept)
    lib.compact(hid, hid.shape[1] * 2, kept, n_kept, hid_out)
    lib.gather_positions(pos_d, kept, n_kept, pos_out)
    torch.cuda.synchronize()
    return dict(out=lib.to_host_bits(out), scores=scores.cpu().numpy(), kept_idx=kept.cpu().numpy().astype(np.int64),
                out_offsets=out_off.cpu().numpy(), k_out=lib.to_host_bits(k_out), v_out=lib.to_host_bits(v_out),
                hidden_out=lib.to_host_bits(hid_out), pos_out=pos_out.cpu().numpy())


@pytest.mark.parametrize("lens,Hq,Hkv,d,w", [
    ((2048,), 32, 32, 128, 64),               # one prompt at the 7B head shape: 16 head groups
    ((1000,), 32, 32, 128, 64),               # ... a shorter one, its last key block ragged
    ((700, 33, 1000), 16, 8, 128, 64),        # ragged, GQA 2: 4 head groups
    ((256,), 8, 8, 64, 16),                   # the smallest workload's shape: 4 head groups
    ((5000, 300), 8, 4, 64, 32),              # a long and a short sequence, 2 head groups
    ((300, 0, 120), 4, 4, 64, 16),            # an empty sequence
    ((900,) * 40, 8, 8, 128, 64),             # enough key blocks for the chip: one head group
    ((2048,) * 20, 8, 8, 128, 64),            # ... with longer sequences
    ((300,) * 8, 8, 8, 64, 32),               # equal lengths, eight sequences: a sequence per XCD, 2 head groups
    ((130,) * 16, 4, 2, 128, 64),             # ... GQA 2, three key blocks each, the last one ragged
    ((1100,) * 24, 16, 16, 64, 64),           # ... one head group
])
def test_fused_step_equals_the_separate_calls(lib, lens, Hq, Hkv, d, w):
    wl = synth.shrunk(synth.workload("cfg2"), lens, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, w=w, hidden_dim=256)
    x = parity.inputs(wl, lib)
    pos = np.random.default_rng(2).integers(0, 1 << 28, sum(lens)).astype(np.int32)
    a = lib.prefill_layer_from_numpy(x, wl.w, hidden=x["hidden"], pos=pos)
    b = separate_calls(lib, x, wl, pos)
    assert np.array_equal(a["out"], b["out"])
    np.testing.assert_allclose(a["scores"], b["scores"], rtol=2e-6, atol=1e-12)      # (partial sums round once more)
    assert a["out_offsets"].tolist() == b["out_offsets"].tolist()
    if np.array_equal(a["scores"], b["scores"]):
        assert np.array_equal(a["kept_idx"], b["kept_idx"])
    ka = a["kept_idx"]
    assert np.array_equal(a["k_out"], x["k"][ka]) and np.array_equal(a["v_out"], x["v"][ka])
    assert np.array_equal(a["hidden_out"], x["hidden"][ka]) and np.array_equal(a["pos_out"], pos[ka])
    # the selection is exact on the scores the fused pass itself produced
    off = x["seq_offsets"]
    oo = a["out_offsets"]
    for s_i, S in enumerate(lens):
        L = min(w, S)
        g = ka[oo[s_i]:oo[s_i + 1]] - off[s_i]
        ctx = g[: len(g) - L]
        sc = a["scores"][off[s_i]:off[s_i + 1]]
        if 0 < len(ctx) < S - L:
            dropped = np.setdiff1d(np.arange(S - L), ctx, assume_unique=True)
            assert sc[ctx].min() >= sc[dropped].max()


def test_single_prompt_against_the_oracle(lib):
    """1 x 2048 tokens, 32 heads, d 128 (the small-batch regime of Appendix A.1) through the fused call."""
    wl = synth.workload("1x2k")
    run_and_check(lib, wl, out_rows=sample_rows(wl, 48, 5))


def test_single_long_prompt_against_the_oracle(lib):
    wl = synth.shrunk(synth.workload("1x8k"), (6000,), n_q_heads=8, n_kv_heads=8)
    run_and_check(lib, wl, out_rows=sample_rows(wl, 24, 6))


def test_fused_step_twice_on_one_workspace(lib):
    """The arrival counters are left at zero: a second step on the same workspace, without clearing it, is right."""
    wl = synth.shrunk(synth.workload("cfg2"), (1000, 700), n_q_heads=8, n_kv_heads=8, head_dim=64, w=32, hidden_dim=64)
    x = parity.inputs(wl, lib)
    q, k, v = (lib.to_device_bf16(x[n]) for n in ("q", "k", "v"))
    hid = lib.to_device_bf16(x["hidden"])
    T, Hq, d = q.shape
    off_h = torch.from_numpy(np.ascontiguousarray(x["seq_offsets"], dtype=np.int32))
    keep_h = torch.from_numpy(np.ascontiguousarray(x["keep_len"], dtype=np.int32))
    off_d, keep_d = off_h.cuda(), keep_h.cuda()
    n_kept = int(keep_h.sum())
    shape = lib.make_shape(2, T, 1000, Hq, Hq, d)
    ws_bytes = lib.workspace_bytes(shape, wl.w)
    ws = torch.full((ws_bytes,), 0x5C, dtype=torch.uint8, device="cuda")
    res = []
    for _ in range(3):
        out = torch.empty_like(q)
        scores = torch.full((T,), -1.0, dtype=torch.float32, device="cuda")
        kept = torch.full((n_kept,), -1, dtype=torch.int32, device="cuda")
        out_off = torch.empty(3, dtype=torch.int32, device="cuda")
        k_out = torch.empty((n_kept, Hq, d), dtype=torch.bfloat16, device="cuda")
        v_out = torch.empty_like(k_out)
        hid_out = torch.empty((n_kept, 64), dtype=torch.bfloat16, device="cuda")
        lib.prefill_layer_fused(q, k, v, off_d, off_h, shape, wl.w, 0.0, keep_d, keep_h, None, hid, 128, None, out, scores,
                                kept, out_off, k_out, v_out, hid_out, None, ws, ws_bytes)
        torch.cuda.synchronize()
        res.append((scores.cpu().numpy(), kept.cpu().numpy(), lib.to_host_bits(hid_out)))
    for r in res[1:]:
        assert np.array_equal(r[0], res[0][0]) and np.array_equal(r[1], res[0][1]) and np.array_equal(r[2], res[0][2])
    assert (res[0][1] >= 0).all()


def test_static_step_replays_from_a_hip_graph(lib):
    """The step that allocates nothing (pyr_prefill_layer_static) captured into a HIP graph: three replays, with eager
    work of the same library and synchronisations in between, each equal to the eager result."""
    wl = synth.shrunk(synth.workload("cfg2"), (700, 300), n_q_heads=8, n_kv_heads=8, head_dim=64, w=32, hidden_dim=0)
    x = parity.inputs(wl, lib, want_hidden=False)
    q, k, v = (lib.to_device_bf16(x[n]) for n in ("q", "k", "v"))
    T, Hq, d = q.shape
    off_h = torch.from_numpy(np.ascontiguousarray(x["seq_offsets"], dtype=np.int32))
    keep_h = torch.from_numpy(np.ascontiguousarray(x["keep_len"], dtype=np.int32))
    off_d, keep_d = off_h.cuda(), keep_h.cuda()
    n_kept = int(keep_h.sum())
    shape = lib.make_shape(2, T, 700, Hq, Hq, d)
    out = torch.empty_like(q)
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    kept = torch.empty(n_kept, dtype=torch.int32, device="cuda")
    out_off = torch.empty(3, dtype=torch.int32, device="cuda")
    k_out = torch.empty((n_kept, Hq, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)

    def step():
        lib.prefill_layer_static(q, k, v, off_d, off_h, shape, wl.w, 0.0, keep_d, keep_h, out, scores, kept, out_off, k_out,
                                 v_out)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (out, scores, kept, out_off, k_out, v_out)]

    step()                                        # eager: also does the once-per-device set-up outside the capture
    ref = snapshot()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        for t in (out, scores, k_out, v_out):
            t.zero_()
        kept.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(got, ref):
            assert torch.equal(a.view(torch.uint8) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.uint8) if b.dtype == torch.bfloat16 else b), f"replay {rep}"
        step()                                    # eager work of the library between the replays
        torch.cuda.synchronize()
