"""ctypes binding of libpyr: argument marshalling only, same names as include/pyr.h.

Every function takes torch tensors that already live on the GPU (or host int32 tensors
for the *_host arguments), passes their addresses and the current HIP stream to the C
ABI and raises on a non-zero status.  There is no fallback: if the library has not been
built (python __graft_entry__.py) importing a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os

# PYR_LIB may point at another build of the same ABI (tuning experiments); default: the in-tree library
_LIB_PATH = os.environ.get("PYR_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpyr.so")
_lib = None


class PyrShape(ctypes.Structure):
    _fields_ = [("n_seqs", ctypes.c_int32), ("total_tokens", ctypes.c_int32), ("max_seqlen", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32)]


class PyrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: pyr status {status}: {strerror(status)}")


_VP, _I32, _I64, _SZ, _F32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float
_SIGNATURES = {
    "pyr_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "pyr_version": (ctypes.c_int, []),
    "pyr_workspace_bytes": (ctypes.c_int, [ctypes.POINTER(PyrShape), _I32, ctypes.POINTER(_SZ)]),
    "pyr_schedule_next": (ctypes.c_int, [_I32, _I32, _I32, _I32, _I32, ctypes.POINTER(_I32)]),
    "pyr_schedule_plan": (ctypes.c_int, [_I32, _I32, _I32, ctypes.POINTER(_I32), _I32, ctypes.POINTER(_I32), _I32,
                                         ctypes.POINTER(_I32)]),
    "pyr_attention": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _F32, _VP, _VP, _VP, _VP]),
    "pyr_score": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _I32, _F32, _VP, _VP]),
    "pyr_score_weighted": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _I32, _F32, _VP, _VP, _VP]),
    "pyr_select": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, _I32, _I32, _VP, _VP, _VP]),
    "pyr_compact": (ctypes.c_int, [_VP, _SZ, _VP, _I64, _VP, _VP]),
    "pyr_compact2": (ctypes.c_int, [_VP, _VP, _VP, _VP, _SZ, _VP, _I64, _VP]),
    "pyr_gather_positions": (ctypes.c_int, [_VP, _VP, _I64, _VP, _VP]),
    "pyr_prefill_layer_ex": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _I32, _F32, _VP, _VP,
                                            _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _SZ, _VP]),
    "pyr_prefill_layer_fused": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _I32, _F32, _VP, _VP,
                                               _VP, _VP, _SZ, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _SZ, _VP]),
    "pyr_prefill_layer_static": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _I32, _F32, _VP, _VP,
                                                _VP, _VP, _VP, _VP, _VP, _VP, _VP]),
    "pyr_decode_workspace_bytes": (ctypes.c_int, [ctypes.POINTER(PyrShape), _I32, ctypes.POINTER(_SZ)]),
    "pyr_decode_update": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _I32, _F32, _VP, _VP,
                                         _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _SZ, _VP]),
    "pyr_prefill_layer": (ctypes.c_int, [_VP, _VP, _VP, _VP, _VP, ctypes.POINTER(PyrShape), _I32, _F32, _VP, _VP,
                                         _VP, _VP, _VP, _VP, _VP, _VP, _VP, _SZ, _VP]),
    "pyr_diag_mfma_only": (ctypes.c_int, [_I32, _VP, _VP, ctypes.POINTER(ctypes.c_double)]),
    "pyr_diag_read_stream": (ctypes.c_int, [_VP, _SZ, _I32, _VP, _VP]),
}
EXPORTS = tuple(_SIGNATURES)


def load():
    """Load libpyr.so (once) and declare the signatures; raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python __graft_entry__.py`")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def lib_path() -> str:
    return _LIB_PATH


def strerror(status: int) -> str:
    return load().pyr_strerror(status).decode()


def version() -> int:
    return load().pyr_version()


def _check(status: int, where: str):
    if status != 0:
        raise PyrError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def make_shape(n_seqs, total_tokens, max_seqlen, n_q_heads, n_kv_heads, head_dim) -> PyrShape:
    return PyrShape(int(n_seqs), int(total_tokens), int(max_seqlen), int(n_q_heads), int(n_kv_heads), int(head_dim))


def workspace_bytes(shape: PyrShape, w: int) -> int:
    out = _SZ(0)
    _check(load().pyr_workspace_bytes(ctypes.byref(shape), int(w), ctypes.byref(out)), "pyr_workspace_bytes")
    return int(out.value)


def schedule_next(S: int, w: int, num: int, den: int, floor_len: int) -> int:
    out = _I32(0)
    _check(load().pyr_schedule_next(int(S), int(w), int(num), int(den), int(floor_len), ctypes.byref(out)),
           "pyr_schedule_next")
    return int(out.value)


def schedule_plan(S: int, w: int, nums, den: int, floors, context_relative: bool = False):
    n = len(nums)
    if len(floors) != n:
        raise ValueError("one ratio and one minimum length per layer")
    num_a, floor_a, out = (_I32 * max(n, 1))(*nums), (_I32 * max(n, 1))(*floors), (_I32 * (n + 1))()
    _check(load().pyr_schedule_plan(int(S), int(w), n, num_a, int(den), floor_a, int(bool(context_relative)), out),
           "pyr_schedule_plan")
    return list(out)


def attention(q, k, v, seq_offsets_dev, seq_offsets_host, shape, softmax_scale, out, lse, tile_map, stream=None):
    _check(load().pyr_attention(_ptr(q), _ptr(k), _ptr(v), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                                ctypes.byref(shape), float(softmax_scale), _ptr(out), _ptr(lse), _ptr(tile_map),
                                _stream(stream)), "pyr_attention")


def score(q, k, lse, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, scores, stream=None):
    _check(load().pyr_score(_ptr(q), _ptr(k), _ptr(lse), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                            ctypes.byref(shape), int(w), float(softmax_scale), _ptr(scores), _stream(stream)),
           "pyr_score")


def score_weighted(q, k, lse, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, row_weights_dev, scores,
                   stream=None):
    _check(load().pyr_score_weighted(_ptr(q), _ptr(k), _ptr(lse), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                                     ctypes.byref(shape), int(w), float(softmax_scale), _ptr(row_weights_dev),
                                     _ptr(scores), _stream(stream)), "pyr_score_weighted")


def select(scores, seq_offsets_dev, seq_offsets_host, keep_len_dev, keep_len_host, n_seqs, w, kept_idx,
           out_offsets_dev, stream=None):
    _check(load().pyr_select(_ptr(scores), _ptr(seq_offsets_dev), _ptr(seq_offsets_host), _ptr(keep_len_dev),
                             _ptr(keep_len_host), int(n_seqs), int(w), _ptr(kept_idx), _ptr(out_offsets_dev),
                             _stream(stream)), "pyr_select")


def compact(src, row_bytes, kept_idx, n_kept, dst, stream=None):
    _check(load().pyr_compact(_ptr(src), int(row_bytes), _ptr(kept_idx), int(n_kept), _ptr(dst), _stream(stream)),
           "pyr_compact")


def compact2(src0, dst0, src1, dst1, row_bytes, kept_idx, n_kept, stream=None):
    _check(load().pyr_compact2(_ptr(src0), _ptr(dst0), _ptr(src1), _ptr(dst1), int(row_bytes), _ptr(kept_idx),
                               int(n_kept), _stream(stream)), "pyr_compact2")


def gather_positions(pos, kept_idx, n_kept, pos_out, stream=None):
    _check(load().pyr_gather_positions(_ptr(pos), _ptr(kept_idx), int(n_kept), _ptr(pos_out), _stream(stream)),
           "pyr_gather_positions")


def prefill_layer_ex(q, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev, keep_len_host,
                     row_weights_dev, pos, out, scores, kept_idx, out_offsets_dev, k_out, v_out, pos_out, workspace,
                     workspace_bytes_, stream=None):
    _check(load().pyr_prefill_layer_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                                       ctypes.byref(shape), int(w), float(softmax_scale), _ptr(keep_len_dev),
                                       _ptr(keep_len_host), _ptr(row_weights_dev), _ptr(pos), _ptr(out), _ptr(scores),
                                       _ptr(kept_idx), _ptr(out_offsets_dev), _ptr(k_out), _ptr(v_out), _ptr(pos_out),
                                       _ptr(workspace), int(workspace_bytes_), _stream(stream)), "pyr_prefill_layer_ex")


def prefill_layer(q, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev, keep_len_host,
                  out, scores, kept_idx, out_offsets_dev, k_out, v_out, workspace, workspace_bytes_, stream=None):
    _check(load().pyr_prefill_layer(_ptr(q), _ptr(k), _ptr(v), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                                    ctypes.byref(shape), int(w), float(softmax_scale), _ptr(keep_len_dev),
                                    _ptr(keep_len_host), _ptr(out), _ptr(scores), _ptr(kept_idx),
                                    _ptr(out_offsets_dev), _ptr(k_out), _ptr(v_out), _ptr(workspace),
                                    int(workspace_bytes_), _stream(stream)), "pyr_prefill_layer")


def prefill_layer_fused(q, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev, keep_len_host,
                        row_weights_dev, hidden, hidden_row_bytes, pos, out, scores, kept_idx, out_offsets_dev, k_out, v_out,
                        hidden_out, pos_out, workspace, workspace_bytes_, stream=None):
    _check(load().pyr_prefill_layer_fused(_ptr(q), _ptr(k), _ptr(v), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                                          ctypes.byref(shape), int(w), float(softmax_scale), _ptr(keep_len_dev),
                                          _ptr(keep_len_host), _ptr(row_weights_dev), _ptr(hidden), int(hidden_row_bytes),
                                          _ptr(pos), _ptr(out), _ptr(scores), _ptr(kept_idx), _ptr(out_offsets_dev),
                                          _ptr(k_out), _ptr(v_out), _ptr(hidden_out), _ptr(pos_out), _ptr(workspace),
                                          int(workspace_bytes_), _stream(stream)), "pyr_prefill_layer_fused")


def prefill_layer_static(q, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev,
                         keep_len_host, out, scores, kept_idx, out_offsets_dev, k_out, v_out, stream=None):
    _check(load().pyr_prefill_layer_static(_ptr(q), _ptr(k), _ptr(v), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                                           ctypes.byref(shape), int(w), float(softmax_scale), _ptr(keep_len_dev),
                                           _ptr(keep_len_host), _ptr(out), _ptr(scores), _ptr(kept_idx),
                                           _ptr(out_offsets_dev), _ptr(k_out), _ptr(v_out), _stream(stream)),
           "pyr_prefill_layer_static")


def diag_mfma_only(iters, sink, stream=None) -> float:
    """Launch the MFMA-only diagnostic; returns the floating-point operations of the launch."""
    fl = ctypes.c_double(0.0)
    _check(load().pyr_diag_mfma_only(int(iters), _ptr(sink), _stream(stream), ctypes.byref(fl)), "pyr_diag_mfma_only")
    return float(fl.value)


def diag_read_stream(data, nbytes, k_layout, sink, stream=None) -> None:
    """Launch the read-only diagnostic over the first nbytes of data (LDS-direct loads, discarded)."""
    _check(load().pyr_diag_read_stream(_ptr(data), int(nbytes), int(bool(k_layout)), _ptr(sink), _stream(stream)),
           "pyr_diag_read_stream")


def decode_workspace_bytes(shape: PyrShape, w: int) -> int:
    out = _SZ(0)
    _check(load().pyr_decode_workspace_bytes(ctypes.byref(shape), int(w), ctypes.byref(out)), "pyr_decode_workspace_bytes")
    return int(out.value)


def decode_update(q_win, k, v, seq_offsets_dev, seq_offsets_host, shape, w, softmax_scale, keep_len_dev, keep_len_host,
                  row_weights_dev, pos, scores, kept_idx, out_offsets_dev, k_out, v_out, pos_out, workspace,
                  workspace_bytes_, stream=None):
    _check(load().pyr_decode_update(_ptr(q_win), _ptr(k), _ptr(v), _ptr(seq_offsets_dev), _ptr(seq_offsets_host),
                                    ctypes.byref(shape), int(w), float(softmax_scale), _ptr(keep_len_dev),
                                    _ptr(keep_len_host), _ptr(row_weights_dev), _ptr(pos), _ptr(scores), _ptr(kept_idx),
                                    _ptr(out_offsets_dev), _ptr(k_out), _ptr(v_out), _ptr(pos_out), _ptr(workspace),
                                    int(workspace_bytes_), _stream(stream)), "pyr_decode_update")


# ----------------------------------------------------------------------------- convenience for tests / smoke
def to_device_bf16(bits_u16):
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on the GPU (same bits)."""
    import numpy as np
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).cuda().view(torch.bfloat16)


def to_host_bits(t):
    """torch.bfloat16 tensor -> numpy uint16 bit patterns."""
    import numpy as np
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def prefill_layer_from_numpy(x, w, hidden=None, softmax_scale=0.0, row_weights=None, pos=None):
    """Upload the arrays of synth.make_inputs, run the layer step through ONE entry point, download
    everything.  Buffers are allocated with torch; every step of the path runs in the library.
    With hidden rows the call is pyr_prefill_layer_fused, with row_weights (float [w]) and/or
    pos (int [T]) but no hidden rows pyr_prefill_layer_ex, else pyr_prefill_layer."""
    import numpy as np
    import torch
    q, k, v = (to_device_bf16(x[n]) for n in ("q", "k", "v"))
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    off_h = torch.from_numpy(np.ascontiguousarray(x["seq_offsets"], dtype=np.int32))
    keep_h = torch.from_numpy(np.ascontiguousarray(x["keep_len"], dtype=np.int32))
    off_d, keep_d = off_h.cuda(), keep_h.cuda()
    B = keep_h.numel()
    lens = np.diff(x["seq_offsets"])
    shape = make_shape(B, T, int(lens.max()) if B else 0, Hq, Hkv, d)
    n_kept = int(keep_h.sum())
    ws_bytes = workspace_bytes(shape, w)
    ws = torch.full((ws_bytes,), 0xAB, dtype=torch.uint8, device="cuda")     # the library must not rely on its contents
    out = torch.empty_like(q)
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    kept = torch.empty(max(n_kept, 1), dtype=torch.int32, device="cuda")
    out_off = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    k_out = torch.empty((max(n_kept, 1), Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)
    res = {}
    rw_d = None if row_weights is None else torch.from_numpy(np.ascontiguousarray(row_weights, dtype=np.float32)).cuda()
    pos_d = None if pos is None else torch.from_numpy(np.ascontiguousarray(pos, dtype=np.int32)).cuda()
    pos_out = None if pos is None else torch.empty(max(n_kept, 1), dtype=torch.int32, device="cuda")
    if hidden is not None:                      # everything in one call: pyr_prefill_layer_fused
        hid = to_device_bf16(hidden)
        hid_out = torch.empty((max(n_kept, 1), hid.shape[1]), dtype=torch.bfloat16, device="cuda")
        prefill_layer_fused(q, k, v, off_d, off_h, shape, w, softmax_scale, keep_d, keep_h, rw_d, hid, hid.shape[1] * 2,
                            pos_d, out, scores, kept, out_off, k_out, v_out, hid_out, pos_out, ws, ws_bytes)
        res["hidden_out"] = to_host_bits(hid_out)[:n_kept]
    elif row_weights is None and pos is None:
        prefill_layer(q, k, v, off_d, off_h, shape, w, softmax_scale, keep_d, keep_h, out, scores, kept, out_off,
                      k_out, v_out, ws, ws_bytes)
    else:
        prefill_layer_ex(q, k, v, off_d, off_h, shape, w, softmax_scale, keep_d, keep_h, rw_d, pos_d, out, scores, kept,
                         out_off, k_out, v_out, pos_out, ws, ws_bytes)
    if pos is not None:
        res["pos_out"] = pos_out.cpu().numpy()[:n_kept]
    torch.cuda.synchronize()
    res.update(out=to_host_bits(out), scores=scores.cpu().numpy(), kept_idx=kept.cpu().numpy()[:n_kept].astype(np.int64),
               out_offsets=out_off.cpu().numpy(), k_out=to_host_bits(k_out)[:n_kept], v_out=to_host_bits(v_out)[:n_kept],
               lse=ws[: T * Hq * 4].view(torch.float32).reshape(T, Hq).cpu().numpy())
    return res


def decode_update_from_numpy(q_win_bits, k_bits, v_bits, seq_offsets, keep_len, w, softmax_scale=0.0, row_weights=None,
                             pos=None):
    """Upload a compressed cache (bf16 bit patterns) and the window's queries, run pyr_decode_update, download."""
    import numpy as np
    import torch
    q_win, k, v = (to_device_bf16(a) for a in (q_win_bits, k_bits, v_bits))
    B, _, Hq, d = q_win.shape
    T, Hkv = k.shape[0], k.shape[1]
    off_h = torch.from_numpy(np.ascontiguousarray(seq_offsets, dtype=np.int32))
    keep_h = torch.from_numpy(np.ascontiguousarray(keep_len, dtype=np.int32))
    off_d, keep_d = off_h.cuda(), keep_h.cuda()
    lens = np.diff(seq_offsets)
    shape = make_shape(B, T, int(lens.max()) if B else 0, Hq, Hkv, d)
    n_kept = int(keep_h.sum())
    ws_bytes = decode_workspace_bytes(shape, w)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    scores = torch.empty(T, dtype=torch.float32, device="cuda")
    kept = torch.empty(max(n_kept, 1), dtype=torch.int32, device="cuda")
    out_off = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    k_out = torch.empty((max(n_kept, 1), Hkv, d), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)
    rw_d = None if row_weights is None else torch.from_numpy(np.ascontiguousarray(row_weights, dtype=np.float32)).cuda()
    pos_d = None if pos is None else torch.from_numpy(np.ascontiguousarray(pos, dtype=np.int32)).cuda()
    pos_out = None if pos is None else torch.empty(max(n_kept, 1), dtype=torch.int32, device="cuda")
    decode_update(q_win, k, v, off_d, off_h, shape, w, softmax_scale, keep_d, keep_h, rw_d, pos_d, scores, kept, out_off,
                  k_out, v_out, pos_out, ws, ws_bytes)
    torch.cuda.synchronize()
    res = dict(scores=scores.cpu().numpy(), kept_idx=kept.cpu().numpy()[:n_kept].astype(np.int64),
               out_offsets=out_off.cpu().numpy(), k_out=to_host_bits(k_out)[:n_kept], v_out=to_host_bits(v_out)[:n_kept])
    if pos is not None:
        res["pos_out"] = pos_out.cpu().numpy()[:n_kept]
    return res
