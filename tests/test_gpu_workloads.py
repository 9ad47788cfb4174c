"""GPU parity at the FULL sizes of the five workloads, in the launch configuration bench.py times.

The GPU always runs the complete batch.  The float64 oracle is evaluated on a stated sample:
scores, selection and gathers for the sampled sequences (complete within a sequence), the
attention output on sampled rows of them.  Every sequence additionally passes the checks
that hold at any size (index invariants, bit-exact gathers, score mass one).  The oracle
treats the sequences of a packed batch independently (pinned on the CPU), so a sub-batch of
sequences is a legitimate oracle call.
"""
import time

import numpy as np
import pytest

from oracle import pyr_oracle as orc
from paper_2405_12532_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
F64 = synth.bf16_bits_to_f64


class DeviceLayer:
    """One layer call through the per-step entry points of the C ABI, exactly as bench.py issues them."""

    def __init__(self, lib, x, wl, hidden_dev=None):
        self.lib, self.wl = lib, wl
        self.q, self.k, self.v = (lib.to_device_bf16(x[n]) for n in ("q", "k", "v"))
        T, Hq, d = self.q.shape
        Hkv = self.k.shape[1]
        self.off_h = torch.from_numpy(np.ascontiguousarray(x["seq_offsets"], dtype=np.int32))
        self.keep_h = torch.from_numpy(np.ascontiguousarray(x["keep_len"], dtype=np.int32))
        self.off_d, self.keep_d = self.off_h.cuda(), self.keep_h.cuda()
        self.n_kept = int(self.keep_h.sum())
        self.shape = lib.make_shape(wl.n_seqs, T, max(wl.seq_lens), Hq, Hkv, d)
        self.lse = torch.empty((T, Hq), dtype=torch.float32, device="cuda")
        self.tile_map = torch.empty(wl.n_seqs + 1, dtype=torch.int32, device="cuda")
        self.out = torch.empty_like(self.q)
        self.scores = torch.empty(T, dtype=torch.float32, device="cuda")
        self.kept = torch.empty(self.n_kept, dtype=torch.int32, device="cuda")
        self.out_off = torch.empty(wl.n_seqs + 1, dtype=torch.int32, device="cuda")
        self.k_out = torch.empty((self.n_kept, Hkv, d), dtype=torch.bfloat16, device="cuda")
        self.v_out = torch.empty_like(self.k_out)
        self.hidden = hidden_dev
        self.hidden_out = None
        if hidden_dev is not None:
            self.hidden_out = torch.empty((self.n_kept, hidden_dev.shape[1]), dtype=torch.bfloat16, device="cuda")

    def run(self):
        lib, wl = self.lib, self.wl
        lib.attention(self.q, self.k, self.v, self.off_d, self.off_h, self.shape, 0.0, self.out, self.lse,
                      self.tile_map)
        lib.score(self.q, self.k, self.lse, self.off_d, self.off_h, self.shape, wl.w, 0.0, self.scores)
        lib.select(self.scores, self.off_d, self.off_h, self.keep_d, self.keep_h, wl.n_seqs, wl.w, self.kept,
                   self.out_off)
        lib.compact2(self.k, self.k_out, self.v, self.v_out, self.k.shape[1] * self.k.shape[2] * 2, self.kept,
                     self.n_kept)
        if self.hidden is not None:
            lib.compact(self.hidden, self.hidden.shape[1] * 2, self.kept, self.n_kept, self.hidden_out)
        torch.cuda.synchronize()


def check_all_sequences(dl, x, wl):
    """Checks that need no oracle arithmetic and hold for every sequence at any size."""
    kept = dl.kept.cpu().numpy().astype(np.int64)
    scores = dl.scores.cpu().numpy()
    off, keep = x["seq_offsets"].astype(np.int64), x["keep_len"].astype(np.int64)
    oo = np.concatenate([[0], np.cumsum(keep)])
    assert dl.out_off.cpu().numpy().tolist() == oo.tolist()
    for b, S in enumerate(wl.seq_lens):
        g = kept[oo[b]:oo[b + 1]] - off[b]
        L = min(wl.w, S)
        assert len(g) == keep[b] and np.all(np.diff(g) > 0) and g[0] >= 0 and g[-1] < S
        assert g[len(g) - L:].tolist() == list(range(S - L, S))
        sc = scores[off[b]:off[b + 1]]
        assert np.all(sc >= 0) and abs(float(sc.astype(np.float64).sum()) - 1.0) < 1e-4
        # exactness of the selection on the GPU's own fp32 scores: nothing dropped outranks anything kept
        ctx_kept = g[: len(g) - L]
        if 0 < len(ctx_kept) < S - L:
            dropped = np.setdiff1d(np.arange(S - L), ctx_kept, assume_unique=True)
            assert sc[ctx_kept].min() >= sc[dropped].max()
        heavy_ctx = x["heavy"][b][x["heavy"][b] < S - L]
        if wl.heavy_frac > 0 and keep[b] - L >= len(heavy_ctx):
            assert np.isin(heavy_ctx, ctx_kept).all(), "planted heavy keys must be retained"
    # gathers are bit-exact given the indices
    kb = dl.lib.to_host_bits(dl.k_out)
    assert np.array_equal(kb, x["k"][kept]), "gathered K"
    del kb
    vb = dl.lib.to_host_bits(dl.v_out)
    assert np.array_equal(vb, x["v"][kept]), "gathered V"
    del vb
    return kept, scores


def check_sampled(dl, x, wl, seqs, out_rows, kept, scores):
    """Oracle comparison on the sequences `seqs` (out on out_rows[i] of seqs[i])."""
    off = x["seq_offsets"].astype(np.int64)
    keep = x["keep_len"].astype(np.int64)
    oo = np.concatenate([[0], np.cumsum(keep)])
    rows_glob = np.concatenate([np.arange(off[b], off[b + 1]) for b in seqs])
    sub_off = np.concatenate([[0], np.cumsum([off[b + 1] - off[b] for b in seqs])])
    ref = orc.prefill_layer(F64(x["q"][rows_glob]), F64(x["k"][rows_glob]), F64(x["v"][rows_glob]), sub_off, wl.w,
                            keep[seqs], out_rows=out_rows)
    # device results of the sampled sequences, re-packed like the sub-batch
    out_rows_glob = np.concatenate([off[b] + np.asarray(r) for b, r in zip(seqs, out_rows)])
    out_gpu = np.zeros((len(rows_glob),) + tuple(dl.out.shape[1:]), dtype=np.uint16)
    sel = torch.from_numpy(out_rows_glob).cuda()
    got = dl.lib.to_host_bits(dl.out[sel])
    pos_in_sub = np.concatenate([sub_off[i] + np.asarray(r) for i, r in enumerate(out_rows)])
    out_gpu[pos_in_sub] = got
    mx, mean = parity.check_out(out_gpu, ref, sub_off, F64)
    sc_gpu = scores[rows_glob]
    rel = parity.check_scores(sc_gpu, ref)
    kept_sub = np.concatenate([kept[oo[b]:oo[b + 1]] - off[b] + sub_off[i] for i, b in enumerate(seqs)])
    same, swapped = parity.check_index_sets(kept_sub, ref, sub_off, keep[seqs], wl.w)
    return mx, mean, rel, same, swapped


def sample_rows(S, w, n_random, rng, full=False):
    if full:
        return np.arange(S)
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256, S // 2, S - w - 1, S - w, S - 2, S - 1]
    fixed = [r for r in fixed if 0 <= r < S]
    return np.unique(np.asarray(fixed + rng.integers(0, S, size=n_random).tolist(), dtype=np.int64))


def run_workload(lib, wl, seqs, n_random_rows, full_seq=None, layer=0, seed=0):
    t0 = time.time()
    x = parity.inputs(wl, lib, layer=layer)
    hid = lib.to_device_bf16(x["hidden"]) if "hidden" in x else None
    dl = DeviceLayer(lib, x, wl, hid)
    t1 = time.time()
    dl.run()
    kept, scores = check_all_sequences(dl, x, wl)
    if hid is not None:
        assert np.array_equal(lib.to_host_bits(dl.hidden_out), x["hidden"][kept]), "gathered hidden rows"
    rng = np.random.default_rng(seed)
    rows = [sample_rows(wl.seq_lens[b], wl.w, n_random_rows, rng, full=(b == full_seq)) for b in seqs]
    t2 = time.time()
    mx, mean, rel, same, swapped = check_sampled(dl, x, wl, list(seqs), rows, kept, scores)
    print(f"[{wl.name} full size] T={wl.total_tokens}: oracle on sequences {list(seqs)} "
          f"({sum(len(r) for r in rows)} output rows): out max {mx:.2e} mean {mean:.2e}; score rel {rel:.2e}; "
          f"identical index sets {same}/{len(seqs)}, swapped in band {swapped}; "
          f"inputs {t1 - t0:.0f} s, oracle {time.time() - t2:.0f} s", flush=True)


def test_64x2k_bench_configuration(lib):
    """The shape bench.py times (first layer of the pyramid: 64 x 2048, 32 heads, d 128, hidden 4096,
    1905 kept): oracle on 12 sequences, all output rows of sequence 0, 40 sampled rows of the others."""
    wl = synth.workload("64x2k")
    run_workload(lib, wl, seqs=(0, 1, 7, 8, 15, 16, 31, 32, 40, 55, 62, 63), n_random_rows=24, full_seq=0)


def test_cfg4_ragged_full_size(lib):
    """Config 4: 32 packed sequences, lengths 512..8192, 40 heads, keep 0.6: oracle on the shortest, the
    longest and four other sequences, sampled output rows."""
    wl = synth.workload("cfg4")
    lens = np.asarray(wl.seq_lens)
    seqs = sorted({int(lens.argmin()), int(lens.argmax()), 0, 5, 17, 31})
    run_workload(lib, wl, seqs=seqs, n_random_rows=16, seed=4)


def test_cfg5_long_gqa_full_size(lib):
    """Config 5: 4 x 32768 tokens, 64 query / 8 KV heads, w 128, keep 0.5: oracle on sequences 0 and 3."""
    wl = synth.workload("cfg5")
    run_workload(lib, wl, seqs=(0, 3), n_random_rows=16, seed=5)


class PyramidChain:
    """State of the 32-layer pyramid of config 3 at batch 64: fresh planted Q/K/V per layer at the surviving
    length, the hidden rows generated once and compacted layer after layer."""

    def __init__(self, lib):
        self.lib = lib
        self.base = synth.workload("cfg3")
        B, S = self.base.n_seqs, self.base.seq_lens[0]
        self.hid0 = synth.make_hidden(synth.shrunk(self.base, (S,) * B))
        self.hid_dev = lib.to_device_bf16(self.hid0)
        self.origin = np.arange(B * S, dtype=np.int64)      # original packed row of every surviving row
        # position ids carried on the device (Appendix A.2): position inside the own prompt
        self.pos_dev = torch.arange(S, dtype=torch.int32, device="cuda").repeat(B)
        self.lengths = [S]
        self.next_layer = 0
        self.worst = [0.0, 0.0, 0.0]
        self.swapped = 0

    def step(self, with_oracle):
        lib, base, layer = self.lib, self.base, self.next_layer
        B, S = base.n_seqs, self.lengths[-1]
        t0 = time.time()
        wl = synth.shrunk(base, (S,) * B)
        x = parity.inputs(wl, lib, layer=layer, want_hidden=False)
        assert int(x["keep_len"][0]) == lib.schedule_next(S, wl.w, 93, 100, 192)
        dl = DeviceLayer(lib, x, wl, self.hid_dev)
        dl.run()
        kept, scores = check_all_sequences(dl, x, wl)
        msg = ""
        if with_oracle:
            seqs = sorted({(7 * layer + j * 16) % B for j in range(4)})
            rng = np.random.default_rng(1000 + layer)
            rows = [sample_rows(S, wl.w, 6, rng) for _ in seqs]
            mx, mean, rel, same, swapped = check_sampled(dl, x, wl, seqs, rows, kept, scores)
            self.worst = [max(self.worst[0], mx), max(self.worst[1], mean), max(self.worst[2], rel)]
            self.swapped += swapped
            msg = f", oracle on {seqs}: out max {mx:.2e}, score rel {rel:.2e}, {same}/{len(seqs)} identical sets"
        self.origin = self.origin[kept]
        self.hid_dev = dl.hidden_out
        pos_out = torch.empty(dl.n_kept, dtype=torch.int32, device="cuda")
        lib.gather_positions(self.pos_dev, dl.kept, dl.n_kept, pos_out)
        self.pos_dev = pos_out
        self.lengths.append(int(x["keep_len"][0]))
        self.next_layer += 1
        print(f"  layer {layer:2d}: S {S} -> {self.lengths[-1]}{msg}, {time.time() - t0:.0f} s", flush=True)

    def run_through(self, last_layer):
        """Layers up to last_layer (inclusive).  Layers a previous test of this module has not run yet are
        run first (on the GPU, with the any-size checks only), so every test also works alone."""
        while self.next_layer <= last_layer:
            self.step(with_oracle=True)


@pytest.fixture(scope="module")
def chain(lib):
    return PyramidChain(lib)


# Config 3, the 32-layer pyramid at batch 64, in four stretches of about equal cost.  Every layer: invariants
# and bit-exact gathers for all 64 sequences; oracle scores / selection / sampled output rows for 4 sequences
# (rotating with the layer).
@pytest.mark.parametrize("last_layer", [3, 9, 19, 31])
def test_cfg3_pyramid_chain(chain, last_layer):
    chain.run_through(last_layer)
    if last_layer == 31:
        golden = open(__file__.rsplit("/", 1)[0] + "/golden/pyramid_lengths_2048_093_192.txt").readline().split()
        assert chain.lengths == [int(t) for t in golden]
        # the surviving hidden rows are the original rows at the composed positions
        assert np.array_equal(chain.lib.to_host_bits(chain.hid_dev), chain.hid0[chain.origin])
        # ... and the position ids carried through 32 gathers name those original places
        assert np.array_equal(chain.pos_dev.cpu().numpy(), chain.origin % chain.base.seq_lens[0])
        print(f"[cfg3 chain] worst out max {chain.worst[0]:.2e} mean {chain.worst[1]:.2e}, "
              f"score rel {chain.worst[2]:.2e}, swapped in band {chain.swapped}", flush=True)


@pytest.mark.gpu
def test_diagnostic_launches_complete():
    """The two ceilings bench.py reports (MFMA only, read only) run to completion and leave their sinks alone."""
    import torch
    from paper_2405_12532_amd import binding as pyr
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    flops = pyr.diag_mfma_only(10, sink)
    assert flops > 0
    data = torch.ones(4 << 20, dtype=torch.uint8, device="cuda")
    isink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for k_layout in (0, 1):
        pyr.diag_read_stream(data, data.numel(), k_layout, isink)
    torch.cuda.synchronize()
    assert float(sink.item()) == 0.0 and int(isink.item()) == 0
