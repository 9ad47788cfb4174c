"""CPU-only checks of the C-ABI library: it loads, exports what include/pyr.h declares,
and its host-side logic (schedule, workspace size, argument validation) behaves.
No kernel is launched here: every call below must fail (or finish) on the host."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import pyr_oracle as orc
from paper_2405_12532_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pyr.h")).read()
    return sorted(set(re.findall(r"PYR_API\s+[\w\s\*]+?\b(pyr_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_functions()
    assert len(names) >= 10
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert getattr(lib, n) is not None


def test_strerror_and_version():
    assert binding.version() >= 100
    assert binding.strerror(0) == "ok"
    for st in range(-7, 0):
        assert binding.strerror(st) not in ("ok", "unknown pyr status")
    assert binding.strerror(-99) == "unknown pyr status"


def test_schedule_matches_oracle_and_golden():
    for S in list(range(0, 400)) + [2048, 8191, 32768]:
        for (num, den, fl, w) in [(93, 100, 192, 64), (7, 10, 0, 64), (1, 2, 0, 128), (6, 10, 0, 64)]:
            assert binding.schedule_next(S, w, num, den, fl) == orc.schedule_next(S, w, num, den, fl)
    golden = [int(x) for x in open(os.path.join(ROOT, "tests", "golden", "pyramid_lengths_2048_093_192.txt"))
              .read().split("#")[0].split()]
    S = 2048
    for l in range(32):
        S = binding.schedule_next(S, 64, 93, 100, 192)
        assert S == golden[l + 1]
    for bad in [(-1, 64, 1, 2, 0), (10, 0, 1, 2, 0), (10, 4, 3, 2, 0), (10, 4, 1, 0, 0), (10, 4, -1, 2, 0)]:
        with pytest.raises(binding.PyrError) as e:
            binding.schedule_next(*bad)
        assert e.value.status == -2


def test_workload_keep_counts_agree_between_library_and_oracle():
    """The input generator holds no schedule arithmetic: each side derives its own counts, and they agree."""
    from paper_2405_12532_amd import synth
    from tests import parity
    for name in ["cfg1", "cfg2", "64x2k", "cfg4", "cfg5"]:
        wl = synth.workload(name)
        keep = parity.keep_lens(wl, binding)
        assert len(keep) == wl.n_seqs and all(min(wl.w, S) <= k <= S for k, S in zip(keep, wl.seq_lens))
    assert not hasattr(synth.Workload, "keep_len")


def test_workspace_bytes():
    s = binding.make_shape(3, 1000, 512, 8, 2, 128)
    n = binding.workspace_bytes(s, 16)
    assert n >= 1000 * 8 * 4 + 4 * 4 and n % 256 == 0
    with pytest.raises(binding.PyrError) as e:
        binding.workspace_bytes(binding.make_shape(3, 1000, 512, 8, 2, 96), 16)
    assert e.value.status == -3
    with pytest.raises(binding.PyrError) as e:
        binding.workspace_bytes(binding.make_shape(3, 1000, 512, 8, 3, 128), 16)
    assert e.value.status == -3
    with pytest.raises(binding.PyrError) as e:
        binding.workspace_bytes(binding.make_shape(3, 1000, 2000, 8, 2, 128), 16)
    assert e.value.status == -2


class FakeDev:
    """Stands in for a device tensor: the checks under test never dereference it."""
    def __init__(self, addr=0x10000):
        self.addr = addr

    def data_ptr(self):
        return self.addr


class Host:
    def __init__(self, values):
        self.a = np.ascontiguousarray(values, dtype=np.int32)

    def data_ptr(self):
        return self.a.ctypes.data


def _call_layer(off, keep, shape, w=4, ws_bytes=1 << 20, ws_addr=0x40000, q_addr=0x10000, k_out=True, v_out=True):
    lib = binding.load()
    d = FakeDev
    return lib.pyr_prefill_layer(
        q_addr, 0x20000, 0x30000, 0x50000, Host(off).data_ptr(), ctypes.byref(shape), w, 0.0, 0x60000,
        Host(keep).data_ptr(), 0x70000, 0x80000, 0x90000, 0xA0000, 0xB0000 if k_out else None,
        0xC0000 if v_out else None, ws_addr, ws_bytes, None)


def test_prefill_layer_rejects_bad_arguments_before_launching():
    shape = binding.make_shape(2, 30, 20, 4, 2, 64)
    ok_off, ok_keep = [0, 10, 30], [6, 12]
    assert _call_layer([1, 10, 30], ok_keep, shape) == -5          # not 0-based
    assert _call_layer([0, 12, 11], ok_keep, shape) == -5          # not monotone
    assert _call_layer([0, 10, 29], ok_keep, shape) == -5          # does not end at T
    assert _call_layer(ok_off, [3, 12], shape) == -4               # below the window
    assert _call_layer(ok_off, [6, 21], shape) == -4               # above the length
    assert _call_layer(ok_off, ok_keep, shape, w=0) == -2
    assert _call_layer(ok_off, ok_keep, shape, ws_bytes=16) == -6
    assert _call_layer(ok_off, ok_keep, shape, ws_addr=0x40010) == -6
    assert _call_layer(ok_off, ok_keep, shape, q_addr=0x10008) == -3    # misaligned q
    assert _call_layer(ok_off, ok_keep, shape, v_out=False) == -1       # only one of k_out / v_out
    assert _call_layer(ok_off, ok_keep, binding.make_shape(2, 30, 5, 4, 2, 64)) == -2   # max_seqlen too small
    assert _call_layer(ok_off, ok_keep, binding.make_shape(2, 30, 20, 4, 2, 32)) == -3
    # a sequence shorter than the window must be kept whole
    assert _call_layer([0, 2, 30], [1, 12], binding.make_shape(2, 30, 28, 4, 2, 64)) == -4


def test_compact_and_select_reject_bad_arguments():
    lib = binding.load()
    assert lib.pyr_compact(0x1000, 24, 0x2000, 5, 0x3000, None) == -3       # row not a multiple of 16
    assert lib.pyr_compact(0x1008, 32, 0x2000, 5, 0x3000, None) == -3       # misaligned
    assert lib.pyr_compact(0x1000, 32, None, 5, 0x3000, None) == -1
    assert lib.pyr_compact(0x1000, 32, 0x2000, -1, 0x3000, None) == -2
    assert lib.pyr_compact(0x1000, 32, 0x2000, 0, 0x3000, None) == 0        # nothing to do, nothing launched
    assert lib.pyr_compact2(0x1000, 0x2000, None, 0x4000, 32, 0x5000, 3, None) == -1
    off, keep = Host([0, 5, 9]), Host([2, 9])
    assert lib.pyr_select(0x1000, 0x2000, off.data_ptr(), 0x3000, keep.data_ptr(), 2, 2, 0x4000, 0x5000, None) == -4
    assert lib.pyr_select(0x1000, 0x2000, off.data_ptr(), 0x3000, keep.data_ptr(), 2, 0, 0x4000, 0x5000, None) == -2
    assert lib.pyr_select(None, 0x2000, off.data_ptr(), 0x3000, keep.data_ptr(), 2, 2, 0x4000, 0x5000, None) == -1


def test_diagnostics_reject_bad_arguments_before_launching():
    lib = binding.load()
    fl = ctypes.c_double(0.0)
    assert lib.pyr_diag_mfma_only(10, None, None, ctypes.byref(fl)) == -1
    assert lib.pyr_diag_mfma_only(0, 0x1000, None, ctypes.byref(fl)) == -2
    assert lib.pyr_diag_read_stream(None, 1 << 19, 0, 0x2000, None) == -1
    assert lib.pyr_diag_read_stream(0x1000, 1 << 19, 0, None, None) == -1
    assert lib.pyr_diag_read_stream(0x1000, 0, 0, 0x2000, None) == -2
    assert lib.pyr_diag_read_stream(0x1000, (1 << 19) + 16, 1, 0x2000, None) == -2      # not whole workgroups


def test_position_and_weight_entry_points_reject_bad_arguments():
    lib = binding.load()
    assert lib.pyr_gather_positions(0x1000, 0x2000, -1, 0x3000, None) == -2
    assert lib.pyr_gather_positions(0x1000, 0x2000, 0, 0x3000, None) == 0          # nothing to do, nothing launched
    assert lib.pyr_gather_positions(None, 0x2000, 3, 0x3000, None) == -1
    assert lib.pyr_gather_positions(0x1000, 0x2000, 3, None, None) == -1
    shape = binding.make_shape(2, 30, 20, 4, 2, 64)
    off, keep = Host([0, 10, 30]), Host([6, 12])

    def layer_ex(pos, pos_out, offsets=off):
        return lib.pyr_prefill_layer_ex(
            0x10000, 0x20000, 0x30000, 0x50000, offsets.data_ptr(), ctypes.byref(shape), 4, 0.0, 0x60000,
            keep.data_ptr(), 0xD0000, pos, 0x70000, 0x80000, 0x90000, 0xA0000, 0xB0000, 0xC0000, pos_out,
            0x40000, 1 << 20, None)
    assert layer_ex(0xE0000, None) == -1                                            # ids in but nowhere to put them
    assert layer_ex(None, 0xF0000) == -1
    assert layer_ex(0xE0000, 0xF0000, Host([0, 12, 11])) == -5                      # same checks as pyr_prefill_layer
    assert lib.pyr_score_weighted(0x1000, 0x2000, None, 0x3000, off.data_ptr(), ctypes.byref(shape), 4, 0.0, 0x4000,
                                  0x5000, None) == -1
    assert lib.pyr_score_weighted(0x1000, 0x2000, 0x6000, 0x3000, off.data_ptr(), ctypes.byref(shape), 0, 0.0, 0x4000,
                                  0x5000, None) == -2


def test_decode_update_rejects_bad_arguments_before_launching():
    lib = binding.load()
    shape = binding.make_shape(2, 30, 20, 4, 2, 64)
    n = binding.decode_workspace_bytes(shape, 4)
    assert n % 256 == 0 and n >= 2 * 4 * 4 * 4 + 1 * 2 * 4 * 4 * 8        # denominators + one key block of statistics
    off, keep = Host([0, 10, 30]), Host([6, 12])

    def call(q_win=0x10000, offsets=off, keeps=keep, w=4, ws=0x40000, ws_bytes=1 << 20, pos=None, pos_out=None, v_out=0xC0000):
        return lib.pyr_decode_update(q_win, 0x20000, 0x30000, 0x50000, offsets.data_ptr(), ctypes.byref(shape), w, 0.0,
                                     0x60000, keeps.data_ptr(), None, pos, 0x80000, 0x90000, 0xA0000, 0xB0000, v_out,
                                     pos_out, ws, ws_bytes, None)
    assert call(q_win=None) == -1
    assert call(q_win=0x10008) == -3
    assert call(offsets=Host([0, 12, 11])) == -5
    assert call(keeps=Host([3, 12])) == -4                                   # below the window
    assert call(w=0) == -2
    assert call(ws_bytes=64) == -6
    assert call(ws=0x40010) == -6
    assert call(pos=0xE0000) == -1                                           # ids in but nowhere to put them
    assert call(v_out=None) == -1


def test_schedule_plan_matches_oracle():
    rng = np.random.default_rng(80)
    for _ in range(300):
        S0, w, den = int(rng.integers(0, 40000)), int(rng.integers(1, 300)), int(rng.integers(1, 1000))
        n = int(rng.integers(0, 40))
        nums, floors = rng.integers(0, den + 1, n).tolist(), rng.integers(0, 400, n).tolist()
        for ctx in (False, True):
            assert binding.schedule_plan(S0, w, nums, den, floors, ctx) == orc.schedule_plan(S0, w, nums, den, floors, ctx)
    golden = [int(x) for x in open(os.path.join(ROOT, "tests", "golden", "pyramid_lengths_2048_093_192.txt"))
              .read().split("#")[0].split()]
    assert binding.schedule_plan(2048, 64, [93] * 32, 100, [192] * 32) == golden
    for bad in [(-1, 4, [1], 2, [0]), (10, 0, [1], 2, [0]), (10, 4, [3], 2, [0]), (10, 4, [1], 0, [0]), (10, 4, [1], 2, [-1])]:
        with pytest.raises(binding.PyrError) as e:
            binding.schedule_plan(*bad)
        assert e.value.status == -2


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
