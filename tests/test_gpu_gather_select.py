"""GPU parity of the gather and selection kernels in isolation (bit-exact), through the C ABI."""
import numpy as np
import pytest

from oracle import pyr_oracle as orc

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _gather_case(lib, n_src, n_kept, row_bytes, seed, two=False):
    rng = np.random.default_rng(seed)
    src = rng.integers(0, 256, size=(n_src, row_bytes), dtype=np.uint8)
    idx = np.sort(rng.choice(n_src, size=n_kept, replace=False)).astype(np.int32) if n_kept <= n_src else None
    d_src = torch.from_numpy(src).cuda()
    d_idx = torch.from_numpy(idx).cuda()
    d_dst = torch.full((max(n_kept, 1) + 1, row_bytes), 0xAB, dtype=torch.uint8, device="cuda")
    if two:
        src1 = rng.integers(0, 256, size=(n_src, row_bytes), dtype=np.uint8)
        d_src1 = torch.from_numpy(src1).cuda()
        d_dst1 = torch.full_like(d_dst, 0xCD)
        lib.compact2(d_src, d_dst, d_src1, d_dst1, row_bytes, d_idx, n_kept)
        torch.cuda.synchronize()
        assert np.array_equal(d_dst1.cpu().numpy()[:n_kept], orc.gather_rows(src1, idx))
        assert np.all(d_dst1.cpu().numpy()[n_kept:] == 0xCD)
    else:
        lib.compact(d_src, row_bytes, d_idx, n_kept, d_dst)
        torch.cuda.synchronize()
    got = d_dst.cpu().numpy()
    assert np.array_equal(got[:n_kept], orc.gather_rows(src, idx))
    assert np.all(got[n_kept:] == 0xAB), "nothing may be written past the kept rows"


@pytest.mark.parametrize("n_src,n_kept,row_bytes", [
    (1, 1, 16), (7, 3, 16), (100, 100, 48), (1000, 613, 1024), (513, 200, 2048), (300, 299, 8192),
    (257, 129, 10240), (64, 17, 16 * 1027),            # rows longer than one unrolled sweep, ragged tail
])
def test_gather_bit_exact(lib, n_src, n_kept, row_bytes):
    _gather_case(lib, n_src, n_kept, row_bytes, seed=n_src + row_bytes)


def test_gather_two_sources_one_launch(lib):
    _gather_case(lib, 700, 431, 8192, seed=5, two=True)
    _gather_case(lib, 9, 4, 32, seed=6, two=True)


def test_gather_many_rows_uses_the_stride_loop(lib):
    _gather_case(lib, 200000, 150001, 64, seed=7)


def test_gather_unsorted_and_repeated_indices(lib):
    rng = np.random.default_rng(11)
    src = rng.integers(0, 256, size=(50, 256), dtype=np.uint8)
    idx = rng.integers(0, 50, size=120).astype(np.int32)
    d_dst = torch.empty((120, 256), dtype=torch.uint8, device="cuda")
    lib.compact(torch.from_numpy(src).cuda(), 256, torch.from_numpy(idx).cuda(), 120, d_dst)
    torch.cuda.synchronize()
    assert np.array_equal(d_dst.cpu().numpy(), src[idx])


# --------------------------------------------------------------------------- select
def _select_case(lib, lens, w, keep, scores):
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keep = np.asarray(keep, dtype=np.int32)
    off_h, keep_h = torch.from_numpy(off), torch.from_numpy(keep)
    n_kept = int(keep.sum())
    kept = torch.full((n_kept + 8,), -7, dtype=torch.int32, device="cuda")
    out_off = torch.full((len(lens) + 1,), -1, dtype=torch.int32, device="cuda")
    lib.select(torch.from_numpy(scores).cuda(), off_h.cuda(), off_h, keep_h.cuda(), keep_h, len(lens), w, kept, out_off)
    torch.cuda.synchronize()
    got = kept.cpu().numpy()
    assert np.all(got[n_kept:] == -7), "nothing may be written past sum(keep_len)"
    ref = [orc.select_pvc(scores[off[b]:off[b + 1]], w, keep[b]) + off[b] for b in range(len(lens))]
    ref = np.concatenate(ref) if ref else np.zeros(0, dtype=np.int64)
    assert np.array_equal(got[:n_kept].astype(np.int64), ref), "selection must be exact on the given fp32 scores"
    assert out_off.cpu().numpy().tolist() == np.concatenate([[0], np.cumsum(keep)]).tolist()


@pytest.mark.parametrize("seed", range(6))
def test_select_exact_random(lib, seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 9))
    lens = rng.integers(1, 3000, size=B)
    w = int(rng.integers(1, 100))
    keep = [int(rng.integers(min(w, S), S + 1)) for S in lens]
    scores = rng.random(int(lens.sum()), dtype=np.float32) ** 4
    _select_case(lib, lens, w, keep, scores)


def test_select_heavy_ties_lower_position_wins(lib):
    rng = np.random.default_rng(3)
    lens = [2048, 777, 64, 5000]
    scores = (rng.integers(0, 5, size=sum(lens)) / 8.0).astype(np.float32)        # 5 distinct values
    _select_case(lib, lens, 64, [1434, 500, 64, 2500], scores)
    const = np.full(sum(lens), 0.25, dtype=np.float32)                          # one value only
    _select_case(lib, lens, 64, [1434, 500, 64, 2500], const)
    zeros = np.zeros(sum(lens), dtype=np.float32)
    zeros[::7] = -0.0
    _select_case(lib, lens, 64, [1000, 65, 64, 4999], zeros)


def test_select_edges(lib):
    rng = np.random.default_rng(4)
    lens = [1, 16, 17, 300, 300, 300]
    scores = rng.random(sum(lens), dtype=np.float32)
    _select_case(lib, lens, 16, [1, 16, 17, 16, 300, 17], scores)   # S<w, S==w, keep all, local only, identity, one ctx
    _select_case(lib, [300], 16, [299], scores[:300])               # evict exactly one


def test_select_long_sequences_staged_and_unstaged(lib):
    rng = np.random.default_rng(5)
    lens = [32768, 36864 + 128, 50000]                  # in LDS / just over the LDS capacity / far over
    scores = (rng.random(sum(lens), dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
    scores[::5] = scores[3]                             # a big tie class as well
    _select_case(lib, lens, 128, [16384, 20000, 128 + 1], scores)


def test_select_tiny_and_denormal_scores(lib):
    rng = np.random.default_rng(6)
    scores = rng.random(4096, dtype=np.float32) * np.float32(1e-38)
    scores[100:200] = 0.0
    _select_case(lib, [4096], 64, [2000], scores.astype(np.float32))


@pytest.mark.parametrize("n_src,n_kept", [(1, 1), (1000, 777), (3_000_000, 2_500_001)])
def test_gather_positions_bit_exact(lib, n_src, n_kept):
    rng = np.random.default_rng(n_kept)
    pos = rng.integers(-(1 << 31), 1 << 31, n_src, dtype=np.int64).astype(np.int32)
    idx = np.sort(rng.choice(n_src, n_kept, replace=False)).astype(np.int32)
    pos_d, idx_d = torch.from_numpy(pos).cuda(), torch.from_numpy(idx).cuda()
    out = torch.full((n_kept + 8,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    lib.gather_positions(pos_d, idx_d, n_kept, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[:n_kept], pos[idx])
    assert np.all(got[n_kept:] == 0x5A5A5A5A), "nothing is written past n_kept"
