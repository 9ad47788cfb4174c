"""Seeded synthetic inputs for the prefill layer step.

This module only draws random numbers, rounds them to bfloat16 bit patterns
and lays them out in the packed [tokens, heads, head_dim] format.  It holds
none of the method's arithmetic (no attention, no scoring, no selection) and
imports neither the HIP library nor the CPU oracle; both are fed from here.

The shapes follow the workloads of the paper (64 prompts of 2k tokens on a
7B-shaped model in Figure 1, a 13B-shaped model in Table 1, long inputs in
the LEval runs of Section 5) and the value structure plants what Recent
Attention Consistency (Section 3.2) describes: a minority of "heavy" context
keys that the recent queries of every head attend to.
"""

from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
import os

import numpy as np

BASE_SEED = 20240512


# --------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(u: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(u).astype(np.float64)


# --------------------------------------------------------------------------- workload table
@dataclass(frozen=True)
class Workload:
    name: str
    seq_lens: tuple            # surviving length of every sequence
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    w: int                     # recent window L
    keep_num: int              # keep ratio = keep_num / keep_den of the whole length, half-up ...
    keep_den: int
    keep_floor: int = 0        # ... never below this (minimum PvC length) nor below w
    keep_fixed: int = 0        # if > 0: this many tokens are kept instead of a ratio
    heavy_frac: float = 0.0    # fraction of positions with a planted heavy key (0: plain N(0,1))
    k_amp: float = 3.0
    q_amp: float = 1.5
    hidden_dim: int = 0
    seed: int = BASE_SEED
    n_layers: int = 1

    @property
    def n_seqs(self) -> int:
        return len(self.seq_lens)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seq_lens))

    def schedule_args(self):
        """(num, den, floor) of this workload's retention rule, in the form the schedule functions of the
        library and of the oracle take; a fixed count is the ratio 0 with that count as the floor.  The
        rule itself is not evaluated here: each side computes its keep counts with its own schedule."""
        if self.keep_fixed > 0:
            return 0, 1, int(self.keep_fixed)
        return int(self.keep_num), int(self.keep_den), int(self.keep_floor)

    def seq_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seq_lens)]).astype(np.int32)


def _ragged_lengths(n, lo, hi, seed):
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0xA11])))
    return tuple(int(x) for x in rng.integers(lo, hi + 1, size=n))


def workload(name: str) -> Workload:
    """The five synthetic configurations of this build, by name ("cfg1" .. "cfg5"),
    plus "64x2k": the first layer of cfg3, the shape throughput is quoted on, and
    "1x2k" / "1x8k": a single prompt on the same layer shape (small-batch timing)."""
    if name == "cfg1":
        return Workload("cfg1", (256,), 8, 8, 64, 16, 1, 2, keep_fixed=128, seed=BASE_SEED + 1)
    if name == "cfg2":
        return Workload("cfg2", (2048,) * 8, 32, 32, 128, 64, 7, 10, heavy_frac=0.10, seed=BASE_SEED + 2)
    if name in ("cfg3", "64x2k"):
        return Workload(name, (2048,) * 64, 32, 32, 128, 64, 93, 100, keep_floor=192, heavy_frac=0.10,
                        hidden_dim=4096, seed=BASE_SEED + 3, n_layers=32 if name == "cfg3" else 1)
    if name in ("1x2k", "1x8k"):            # one prompt on the 7B-shaped layer: the small-batch regime of Appendix A.1
        return Workload(name, (2048 if name == "1x2k" else 8192,), 32, 32, 128, 64, 93, 100, keep_floor=192,
                        heavy_frac=0.10, hidden_dim=4096, seed=BASE_SEED + 6)
    if name == "cfg4":
        lens = _ragged_lengths(32, 512, 8192, BASE_SEED + 4)
        return Workload("cfg4", lens, 40, 40, 128, 64, 6, 10, heavy_frac=0.10, seed=BASE_SEED + 4)
    if name == "cfg5":
        return Workload("cfg5", (32768,) * 4, 64, 8, 128, 128, 1, 2, heavy_frac=0.05, seed=BASE_SEED + 5)
    raise KeyError(name)


def shrunk(wl: Workload, seq_lens, **kw) -> Workload:
    """Same recipe at other lengths (the pyramid's deeper layers, reduced test sizes)."""
    return replace(wl, seq_lens=tuple(int(s) for s in seq_lens), **kw)


# --------------------------------------------------------------------------- generation
def _seq_rng(seed, layer, b, stream):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, layer, b, stream])))


def _gen_sequence(wl: Workload, layer: int, b: int, u_kv: np.ndarray, want_hidden: bool):
    S, Hq, Hkv, d = wl.seq_lens[b], wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    g = Hq // Hkv
    q = _seq_rng(wl.seed, layer, b, 1).standard_normal((S, Hq, d), dtype=np.float32)
    k = _seq_rng(wl.seed, layer, b, 2).standard_normal((S, Hkv, d), dtype=np.float32)
    v = _seq_rng(wl.seed, layer, b, 3).standard_normal((S, Hkv, d), dtype=np.float32)
    heavy = np.zeros(0, dtype=np.int64)
    if wl.heavy_frac > 0.0 and S > 0:
        n_heavy = int(round(wl.heavy_frac * S))
        heavy = np.sort(_seq_rng(wl.seed, layer, b, 4).choice(S, size=n_heavy, replace=False)).astype(np.int64)
        k[heavy] += np.float32(wl.k_amp) * u_kv[None, :, :]
        q += np.float32(wl.q_amp) * np.repeat(u_kv, g, axis=0)[None, :, :]
    res = {"q": f32_to_bf16_bits(q), "k": f32_to_bf16_bits(k), "v": f32_to_bf16_bits(v), "heavy": heavy}
    if want_hidden and wl.hidden_dim > 0:
        res["hidden"] = _gen_hidden(wl, layer, b)
    return res


def _gen_hidden(wl: Workload, layer: int, b: int):
    h = _seq_rng(wl.seed, layer, b, 5).standard_normal((wl.seq_lens[b], wl.hidden_dim), dtype=np.float32)
    return f32_to_bf16_bits(h)


def make_hidden(wl: Workload, layer: int = 0, threads: int | None = None):
    """The hidden rows of make_inputs alone (same values), [T, D] uint16 bf16 bit patterns."""
    if threads is None:
        threads = max(1, min(16, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return np.concatenate(list(ex.map(lambda b: _gen_hidden(wl, layer, b), range(wl.n_seqs))), axis=0)


def make_inputs(wl: Workload, layer: int = 0, want_hidden: bool = True, threads: int | None = None):
    """Packed inputs of one layer call.

    Returns a dict of numpy arrays: q [T,Hq,d], k, v [T,Hkv,d] (uint16 bf16 bit
    patterns), hidden [T,D] (if the workload has one), seq_offsets int32 [B+1],
    heavy (list per sequence of planted local positions).  The keep counts are not
    part of the inputs: they come from the schedule of whoever consumes them.
    Every sequence has its own counter-seeded generator, so any subset of
    sequences can be regenerated alone and the result does not depend on the
    number of worker threads.
    """
    Hkv, d = wl.n_kv_heads, wl.head_dim
    u = _seq_rng(wl.seed, layer, 1 << 20, 0).standard_normal((Hkv, d)).astype(np.float32)
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    if threads is None:
        threads = max(1, min(16, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(lambda b: _gen_sequence(wl, layer, b, u, want_hidden), range(wl.n_seqs)))
    out = {
        "q": np.concatenate([p["q"] for p in parts], axis=0),
        "k": np.concatenate([p["k"] for p in parts], axis=0),
        "v": np.concatenate([p["v"] for p in parts], axis=0),
        "seq_offsets": wl.seq_offsets(),
        "heavy": [p["heavy"] for p in parts],
    }
    if want_hidden and wl.hidden_dim > 0:
        out["hidden"] = np.concatenate([p["hidden"] for p in parts], axis=0)
    return out
