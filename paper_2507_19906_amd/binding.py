"""ctypes binding of libcalidrop.so: the same entry points as include/calidrop.h, taking torch
tensors for the device pointers.  Argument marshalling only - every step of the method runs in
the HIP kernels.  There is no CPU fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libcalidrop.so")

OK, EINVAL, ESHAPE, EALIGN, EWORKSPACE, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4, -5, -6
BF16, FP32 = 0, 1
FLAG_NONE, FLAG_CALIBRATED, FLAG_RECOMPUTE, FLAG_RECOMPUTED = 0, 1, 2, 3
REGION_ROW_LSE, REGION_SCORE, REGION_VOTE_PLANES = 0, 1, 2
OPT_WRITE_SCORES, OPT_WIDE_SELECTION = 1, 2


class CalidropError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"calidrop status {status}: {message}")
        self.status = status


class Params(ctypes.Structure):
    """Mirror of calidrop_params."""
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("batch", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("window", ctypes.c_int32),
        ("budget", ctypes.c_int32),
        ("pool_kernel", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("theta1", ctypes.c_float),
        ("theta2", ctypes.c_float),
        ("calib_size", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
    ]


def make_params(*, dtype, batch, n_q_heads, n_kv_heads, head_dim, window, budget, pool_kernel,
                scale=0.0, theta1=0.7, theta2=0.85, calib_size=0, flags=0) -> Params:
    if isinstance(dtype, torch.dtype):
        dtype = BF16 if dtype == torch.bfloat16 else FP32
    elif isinstance(dtype, str):
        dtype = BF16 if dtype == "bf16" else FP32
    return Params(ctypes.sizeof(Params), dtype, batch, n_q_heads, n_kv_heads, head_dim, window,
                  budget, pool_kernel, scale, theta1, theta2, calib_size, flags)


_lib = None


def lib() -> ctypes.CDLL:
    """Load libcalidrop.so (built in-tree by paper_2507_19906_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2507_19906_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        pp = ctypes.POINTER(Params)
        L.calidrop_last_error.restype = ctypes.c_char_p
        L.calidrop_last_error.argtypes = []
        L.calidrop_version.restype = ctypes.c_int
        L.calidrop_version.argtypes = []
        L.calidrop_compress_workspace_bytes.restype = sz
        L.calidrop_compress_workspace_bytes.argtypes = [pp, i64, i32]
        L.calidrop_decode_workspace_bytes.restype = sz
        L.calidrop_decode_workspace_bytes.argtypes = [pp, i32]
        L.calidrop_compress_workspace_region.restype = ctypes.c_int
        L.calidrop_compress_workspace_region.argtypes = [pp, i64, i32, i32, ctypes.POINTER(sz),
                                                         ctypes.POINTER(sz)]
        L.calidrop_compress.restype = ctypes.c_int
        L.calidrop_compress.argtypes = [pp, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp,
                                        vp, vp, vp, sz, vp]
        L.calidrop_compress_with_lse.restype = ctypes.c_int
        L.calidrop_compress_with_lse.argtypes = [pp, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                 vp, vp, vp, sz, vp]
        L.calidrop_decode.restype = ctypes.c_int
        L.calidrop_decode.argtypes = [pp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz,
                                      vp]
        L.calidrop_decode_static.restype = ctypes.c_int
        L.calidrop_decode_static.argtypes = [pp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.calidrop_recalibrate_workspace_bytes.restype = sz
        L.calidrop_recalibrate_workspace_bytes.argtypes = [pp, i32]
        L.calidrop_recalibrate.restype = ctypes.c_int
        L.calidrop_recalibrate.argtypes = [pp, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.calidrop_compress_given_workspace_bytes.restype = sz
        L.calidrop_compress_given_workspace_bytes.argtypes = [pp, i32]
        L.calidrop_streaming_indices.restype = ctypes.c_int
        L.calidrop_streaming_indices.argtypes = [pp, i32, vp, i64, i32, vp, vp]
        L.calidrop_compress_given.restype = ctypes.c_int
        L.calidrop_compress_given.argtypes = [pp, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp,
                                              vp, sz, vp]
        L.calidrop_packed_rows.restype = i32
        L.calidrop_packed_rows.argtypes = [pp, i32]
        L.calidrop_pack_evicted_workspace_bytes.restype = sz
        L.calidrop_pack_evicted_workspace_bytes.argtypes = [pp, i32]
        L.calidrop_pack_evicted.restype = ctypes.c_int
        L.calidrop_pack_evicted.argtypes = [pp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.calidrop_recalibrate_packed_workspace_bytes.restype = sz
        L.calidrop_recalibrate_packed_workspace_bytes.argtypes = [pp, i32]
        L.calidrop_recalibrate_packed.restype = ctypes.c_int
        L.calidrop_recalibrate_packed.argtypes = [pp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.calidrop_compress_h2o_workspace_bytes.restype = sz
        L.calidrop_compress_h2o_workspace_bytes.argtypes = [pp, i32, i64, i32]
        L.calidrop_compress_h2o_workspace_region.restype = ctypes.c_int
        L.calidrop_compress_h2o_workspace_region.argtypes = [pp, i32, i64, i32, i32, ctypes.POINTER(sz),
                                                             ctypes.POINTER(sz)]
        L.calidrop_compress_h2o.restype = ctypes.c_int
        L.calidrop_compress_h2o.argtypes = [pp, i32, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                            vp, sz, vp]
        L.calidrop_append.restype = ctypes.c_int
        L.calidrop_append.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def calidrop_last_error() -> str:
    return lib().calidrop_last_error().decode()


def _check(status: int) -> None:
    if status != OK:
        raise CalidropError(status, calidrop_last_error())


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def calidrop_compress_workspace_bytes(p: Params, total_tokens: int, max_seq_len: int) -> int:
    n = lib().calidrop_compress_workspace_bytes(ctypes.byref(p), total_tokens, max_seq_len)
    if n == 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_decode_workspace_bytes(p: Params, max_cache_len: int) -> int:
    n = lib().calidrop_decode_workspace_bytes(ctypes.byref(p), max_cache_len)
    if n == 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_compress_workspace_region(p: Params, total_tokens: int, max_seq_len: int, region: int):
    off, nbytes = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().calidrop_compress_workspace_region(ctypes.byref(p), total_tokens, max_seq_len,
                                                    region, ctypes.byref(off), ctypes.byref(nbytes)))
    return off.value, nbytes.value


def calidrop_compress(p: Params, q_win, k, v, seq_offsets, total_tokens: int, max_seq_len: int,
                      q_cal, k_c, v_c, cache_offsets, cache_lens, indices, cal_indices, c_q, c_out, c_lse,
                      workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_compress(
        ctypes.byref(p), _ptr(q_win), _ptr(k), _ptr(v), _ptr(seq_offsets), total_tokens, max_seq_len,
        _ptr(q_cal), _ptr(k_c), _ptr(v_c), _ptr(cache_offsets), _ptr(cache_lens), _ptr(indices),
        _ptr(cal_indices), _ptr(c_q), _ptr(c_out), _ptr(c_lse), _ptr(workspace), ws_bytes, _stream(stream)))


def calidrop_compress_with_lse(p: Params, q_win, k, v, seq_offsets, total_tokens: int, max_seq_len: int,
                               win_lse, q_cal, k_c, v_c, cache_offsets, cache_lens, indices, cal_indices, c_q,
                               c_out, c_lse, workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_compress_with_lse(
        ctypes.byref(p), _ptr(q_win), _ptr(k), _ptr(v), _ptr(seq_offsets), total_tokens, max_seq_len,
        _ptr(win_lse), _ptr(q_cal), _ptr(k_c), _ptr(v_c), _ptr(cache_offsets), _ptr(cache_lens), _ptr(indices),
        _ptr(cal_indices), _ptr(c_q), _ptr(c_out), _ptr(c_lse), _ptr(workspace), ws_bytes, _stream(stream)))


def calidrop_decode(p: Params, q_t, k_c, v_c, cache_offsets, cache_lens, max_cache_len: int, c_q,
                    c_out, c_lse, out, a_lse, flags, workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_decode(
        ctypes.byref(p), _ptr(q_t), _ptr(k_c), _ptr(v_c), _ptr(cache_offsets), _ptr(cache_lens),
        max_cache_len, _ptr(c_q), _ptr(c_out), _ptr(c_lse), _ptr(out), _ptr(a_lse), _ptr(flags),
        _ptr(workspace), ws_bytes, _stream(stream)))


STATIC_SCRATCH_BYTES = 8 << 20      # CALIDROP_STATIC_SCRATCH_BYTES


def calidrop_decode_static(p: Params, q_t, k_c, v_c, cache_offsets, cache_lens, max_cache_len: int, c_q,
                           c_out, c_lse, out, a_lse, flags, stream=None) -> None:
    _check(lib().calidrop_decode_static(
        ctypes.byref(p), _ptr(q_t), _ptr(k_c), _ptr(v_c), _ptr(cache_offsets), _ptr(cache_lens),
        max_cache_len, _ptr(c_q), _ptr(c_out), _ptr(c_lse), _ptr(out), _ptr(a_lse), _ptr(flags),
        _stream(stream)))


def calidrop_append(p: Params, k_new, v_new, k_c, v_c, cache_offsets, cache_lens, stream=None) -> None:
    _check(lib().calidrop_append(ctypes.byref(p), _ptr(k_new), _ptr(v_new), _ptr(k_c), _ptr(v_c),
                                 _ptr(cache_offsets), _ptr(cache_lens), _stream(stream)))


def calidrop_recalibrate_workspace_bytes(p: Params, max_seq_len: int) -> int:
    n = lib().calidrop_recalibrate_workspace_bytes(ctypes.byref(p), max_seq_len)
    if n == 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_recalibrate(p: Params, q_t, k, v, seq_offsets, total_tokens: int, max_seq_len: int, indices,
                         cal_indices, flags, a_lse, out, c_q, c_out, c_lse, workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_recalibrate(
        ctypes.byref(p), _ptr(q_t), _ptr(k), _ptr(v), _ptr(seq_offsets), total_tokens, max_seq_len,
        _ptr(indices), _ptr(cal_indices), _ptr(flags), _ptr(a_lse), _ptr(out), _ptr(c_q), _ptr(c_out),
        _ptr(c_lse), _ptr(workspace), ws_bytes, _stream(stream)))


def calidrop_compress_given_workspace_bytes(p: Params, max_seq_len: int) -> int:
    n = lib().calidrop_compress_given_workspace_bytes(ctypes.byref(p), max_seq_len)
    if n == 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_streaming_indices(p: Params, n_sink: int, seq_offsets, total_tokens: int, max_seq_len: int,
                               indices, stream=None) -> None:
    _check(lib().calidrop_streaming_indices(ctypes.byref(p), n_sink, _ptr(seq_offsets), total_tokens,
                                            max_seq_len, _ptr(indices), _stream(stream)))


def calidrop_compress_given(p: Params, q_cal, k, v, seq_offsets, total_tokens: int, max_seq_len: int,
                            indices, k_c, v_c, cache_offsets, cache_lens, c_q, c_out, c_lse, workspace,
                            stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_compress_given(
        ctypes.byref(p), _ptr(q_cal), _ptr(k), _ptr(v), _ptr(seq_offsets), total_tokens, max_seq_len,
        _ptr(indices), _ptr(k_c), _ptr(v_c), _ptr(cache_offsets), _ptr(cache_lens), _ptr(c_q), _ptr(c_out),
        _ptr(c_lse), _ptr(workspace), ws_bytes, _stream(stream)))


def calidrop_compress_h2o_workspace_bytes(p: Params, n_local: int, total_tokens: int, max_seq_len: int) -> int:
    n = lib().calidrop_compress_h2o_workspace_bytes(ctypes.byref(p), n_local, total_tokens, max_seq_len)
    if n == 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_compress_h2o_workspace_region(p: Params, n_local: int, total_tokens: int, max_seq_len: int,
                                           region: int):
    off, nbytes = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().calidrop_compress_h2o_workspace_region(ctypes.byref(p), n_local, total_tokens, max_seq_len,
                                                        region, ctypes.byref(off), ctypes.byref(nbytes)))
    return off.value, nbytes.value


def calidrop_compress_h2o(p: Params, n_local: int, q_full, k, v, seq_offsets, total_tokens: int, max_seq_len: int,
                          k_c, v_c, cache_offsets, cache_lens, indices, cal_indices, c_q, c_out, c_lse, workspace,
                          stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_compress_h2o(
        ctypes.byref(p), n_local, _ptr(q_full), _ptr(k), _ptr(v), _ptr(seq_offsets), total_tokens, max_seq_len,
        _ptr(k_c), _ptr(v_c), _ptr(cache_offsets), _ptr(cache_lens), _ptr(indices), _ptr(cal_indices), _ptr(c_q),
        _ptr(c_out), _ptr(c_lse), _ptr(workspace), ws_bytes, _stream(stream)))


def calidrop_packed_rows(p: Params, seq_len: int) -> int:
    n = lib().calidrop_packed_rows(ctypes.byref(p), seq_len)
    if n < 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_pack_evicted_workspace_bytes(p: Params, max_seq_len: int) -> int:
    n = lib().calidrop_pack_evicted_workspace_bytes(ctypes.byref(p), max_seq_len)
    if n == 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_pack_evicted(p: Params, k, v, seq_offsets, total_tokens: int, max_seq_len: int, indices,
                          cal_indices, k_e, v_e, evict_offsets, evict_lens, evict_indices, workspace,
                          stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_pack_evicted(
        ctypes.byref(p), _ptr(k), _ptr(v), _ptr(seq_offsets), total_tokens, max_seq_len, _ptr(indices),
        _ptr(cal_indices), _ptr(k_e), _ptr(v_e), _ptr(evict_offsets), _ptr(evict_lens), _ptr(evict_indices),
        _ptr(workspace), ws_bytes, _stream(stream)))


def calidrop_recalibrate_packed_workspace_bytes(p: Params, max_evict_len: int) -> int:
    n = lib().calidrop_recalibrate_packed_workspace_bytes(ctypes.byref(p), max_evict_len)
    if n == 0:
        raise CalidropError(EINVAL, calidrop_last_error())
    return n


def calidrop_recalibrate_packed(p: Params, q_t, k_e, v_e, evict_offsets, evict_lens, max_evict_len: int,
                                flags, a_lse, out, c_q, c_out, c_lse, workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().calidrop_recalibrate_packed(
        ctypes.byref(p), _ptr(q_t), _ptr(k_e), _ptr(v_e), _ptr(evict_offsets), _ptr(evict_lens),
        max_evict_len, _ptr(flags), _ptr(a_lse), _ptr(out), _ptr(c_q), _ptr(c_out), _ptr(c_lse),
        _ptr(workspace), ws_bytes, _stream(stream)))


class EvictedStore:
    """The packed KV_evict of a CompressBuffers: allocation and the two calls, nothing else.
    `host=True` moves the packed rows to page-locked host memory after packing (the offloaded
    form); recalibrate() then reads them from there."""

    def __init__(self, bufs: "CompressBuffers", seq_lens, host: bool = False, extra_rows=None,
                 staged: bool = False):
        """`staged=True` (with `host=True`): recalibrate() brings the rows back with plain copies into two
        device staging buffers, one sequence ahead of the recomputation, instead of letting the kernel
        read page-locked memory over the host link (Alg. 2 step 4's load overlapped with steps 5-8)."""
        assert host or not staged
        self.staged = staged
        self._stage = None
        p = bufs.p
        dev = bufs.out.device
        dt = torch.bfloat16 if p.dtype == BF16 else torch.float32
        rows = [calidrop_packed_rows(p, int(n)) for n in seq_lens]
        caps = [max(r, 1) for r in rows]                      # every sequence owns at least one row slot
        if extra_rows is not None:                            # slack behind each sequence's rows
            caps = [c + int(e) for c, e in zip(caps, extra_rows)]
        offs = [0]
        for c in caps:
            offs.append(offs[-1] + c)
        self.p, self.bufs, self.rows, self.host = p, bufs, rows, host
        self.max_evict_len = max(max(rows), 1)
        self.evict_offsets = torch.tensor(offs, dtype=torch.int32, device=dev)
        self.evict_lens = torch.zeros(p.batch, dtype=torch.int32, device=dev)
        tot = offs[-1] * p.n_kv_heads
        self.evict_indices = torch.zeros(tot, dtype=torch.int32, device=dev)
        self.k_e = torch.zeros(tot * p.head_dim, dtype=dt, device=dev)
        self.v_e = torch.zeros(tot * p.head_dim, dtype=dt, device=dev)
        self.offs = offs
        self.ws_pack = torch.empty(calidrop_pack_evicted_workspace_bytes(p, bufs.max_seq_len),
                                   dtype=torch.uint8, device=dev)
        self.ws_recal = torch.empty(calidrop_recalibrate_packed_workspace_bytes(p, self.max_evict_len),
                                    dtype=torch.uint8, device=dev)

    def pack(self, k, v, seq_offsets, stream=None):
        b = self.bufs
        calidrop_pack_evicted(self.p, k, v, seq_offsets, b.total_tokens, b.max_seq_len, b.indices,
                              b.cal_indices, self.k_e, self.v_e, self.evict_offsets, self.evict_lens,
                              self.evict_indices, self.ws_pack, stream)
        if self.host:                                         # offload: plain copies into pinned memory
            k_h = torch.empty(self.k_e.shape, dtype=self.k_e.dtype, pin_memory=True)
            v_h = torch.empty(self.v_e.shape, dtype=self.v_e.dtype, pin_memory=True)
            k_h.copy_(self.k_e)
            v_h.copy_(self.v_e)
            torch.cuda.synchronize()
            self.k_dev, self.v_dev = self.k_e, self.v_e
            self.k_e, self.v_e = k_h, v_h

    def _recalibrate_staged(self, q_t, stream=None):
        """Per sequence: a copy stream fills one staging buffer with the sequence's packed rows while
        the recomputation of the previous sequence reads the other one.  Copies, events and
        per-sequence calls of calidrop_recalibrate_packed (batch 1); no arithmetic here."""
        p, b = self.p, self.bufs
        Hkv, D = p.n_kv_heads, p.head_dim
        dev = b.out.device
        if stream is None:
            stream = torch.cuda.current_stream()
        elif isinstance(stream, int):
            stream = torch.cuda.ExternalStream(stream)
        if self._stage is None:
            cap = max(self.offs[i + 1] - self.offs[i] for i in range(p.batch))
            p1 = Params.from_buffer_copy(p)
            p1.batch = 1
            self._stage = {
                "p1": p1, "copy": torch.cuda.Stream(device=dev),
                "k": [torch.empty(cap * Hkv * D, dtype=self.k_e.dtype, device=dev) for _ in range(2)],
                "v": [torch.empty(cap * Hkv * D, dtype=self.k_e.dtype, device=dev) for _ in range(2)],
                # per-sequence (offsets, length) arguments, each row 16-byte aligned as the library asks
                "offs": torch.tensor([[0, self.offs[i + 1] - self.offs[i], 0, 0] for i in range(p.batch)],
                                     dtype=torch.int32, device=dev),
                "lens": torch.zeros((p.batch, 4), dtype=torch.int32, device=dev),
                "ready": [torch.cuda.Event() for _ in range(2)],
                "free": [torch.cuda.Event() for _ in range(2)],
            }
        st = self._stage
        copy = st["copy"]
        assert p.n_q_heads % 4 == 0                # per-sequence slices of the fp32 state stay 16-byte aligned
        with torch.cuda.stream(stream):
            st["lens"][:, 0].copy_(self.evict_lens)
        for s in range(2):
            st["free"][s].record(stream)          # what ran before on `stream` may still read the buffers
        for i in range(p.batch):
            s = i & 1
            lo, hi = self.offs[i] * Hkv * D, self.offs[i + 1] * Hkv * D
            copy.wait_event(st["free"][s])
            with torch.cuda.stream(copy):
                st["k"][s][:hi - lo].copy_(self.k_e[lo:hi], non_blocking=True)
                st["v"][s][:hi - lo].copy_(self.v_e[lo:hi], non_blocking=True)
                st["ready"][s].record(copy)
            stream.wait_event(st["ready"][s])
            calidrop_recalibrate_packed(st["p1"], q_t[i:i + 1], st["k"][s], st["v"][s], st["offs"][i],
                                        st["lens"][i], max(self.rows[i], 1), b.flags[i:i + 1],
                                        b.a_lse[i:i + 1], b.out[i:i + 1], b.c_q[i:i + 1], b.c_out[i:i + 1],
                                        b.c_lse[i:i + 1], self.ws_recal, stream)
            st["free"][s].record(stream)

    def recalibrate(self, q_t, stream=None):
        if self.staged:
            return self._recalibrate_staged(q_t, stream)
        b = self.bufs
        calidrop_recalibrate_packed(self.p, q_t, self.k_e, self.v_e, self.evict_offsets, self.evict_lens,
                                    self.max_evict_len, b.flags, b.a_lse, b.out, b.c_q, b.c_out, b.c_lse,
                                    self.ws_recal, stream)

    def view(self, which: str, b: int) -> torch.Tensor:
        """[Hkv][cap_b][D] view of sequence b inside k_e / v_e ('idx': [Hkv][cap_b] positions)."""
        Hkv, D = self.p.n_kv_heads, self.p.head_dim
        cap = self.offs[b + 1] - self.offs[b]
        lo = self.offs[b] * Hkv
        if which == "idx":
            return self.evict_indices[lo:lo + cap * Hkv].view(Hkv, cap)
        t = self.k_e if which == "k" else self.v_e
        return t[lo * D:(lo + cap * Hkv) * D].view(Hkv, cap, D)


# ---- device-memory plumbing (allocation only) ----------------------------------------------
class CompressBuffers:
    """Output and workspace tensors for calidrop_compress / calidrop_decode, allocated with
    torch on `device`.  Cache capacity per sequence = budget + extra_capacity, or, with
    `capacities` (one row count per sequence, each >= min(budget, n_b)), exactly those: the
    compressed caches are then packed back to back behind cache_offsets with no slack."""

    def __init__(self, p: Params, seq_lens, device, extra_capacity: int = 0, capacities=None):
        dt = torch.bfloat16 if p.dtype == BF16 else torch.float32
        self.p = p
        B, Hq, Hkv, D, nb = p.budget, p.n_q_heads, p.n_kv_heads, p.head_dim, p.batch
        assert len(seq_lens) == nb
        self.total_tokens = int(sum(seq_lens))
        self.max_seq_len = int(max(seq_lens))
        caps = [B + extra_capacity] * nb if capacities is None else [int(c) for c in capacities]
        assert len(caps) == nb
        offs = [0]
        for c in caps:
            offs.append(offs[-1] + c)
        self.caps, self.offs = caps, offs
        cap = max(caps)
        self.cap = cap                                  # the largest capacity (= every capacity when uniform)
        self.uniform = all(c == cap for c in caps)
        self.cache_offsets = torch.tensor(offs, dtype=torch.int32, device=device)
        self.k_c = torch.zeros(offs[-1] * Hkv * D, dtype=dt, device=device)
        self.v_c = torch.zeros(offs[-1] * Hkv * D, dtype=dt, device=device)
        self.cache_lens = torch.zeros(nb, dtype=torch.int32, device=device)
        self.indices = torch.zeros((nb, Hkv, B), dtype=torch.int32, device=device)
        self.cal_indices = (torch.zeros((nb, Hkv, p.calib_size), dtype=torch.int32, device=device)
                            if p.calib_size > 0 else None)
        self.c_q = torch.zeros((nb, Hq, D), dtype=torch.float32, device=device)
        self.c_out = torch.zeros((nb, Hq, D), dtype=torch.float32, device=device)
        self.c_lse = torch.zeros((nb, Hq), dtype=torch.float32, device=device)
        self.ws_compress = torch.empty(
            calidrop_compress_workspace_bytes(p, self.total_tokens, self.max_seq_len),
            dtype=torch.uint8, device=device)
        self.max_cache_len = cap
        self.ws_decode = torch.empty(calidrop_decode_workspace_bytes(p, cap), dtype=torch.uint8,
                                     device=device)
        self.out = torch.zeros((nb, Hq, D), dtype=dt, device=device)
        self.a_lse = torch.zeros((nb, Hq), dtype=torch.float32, device=device)
        self.flags = torch.zeros((nb, Hq), dtype=torch.uint8, device=device)

    def compress(self, q_win, k, v, seq_offsets, q_cal=None, stream=None, win_lse=None):
        """win_lse: [batch][Hq][w] fp32 log-sum-exp of the window rows from the caller's prefill
        attention (natural log); None = the library computes it."""
        if win_lse is None:
            calidrop_compress(self.p, q_win, k, v, seq_offsets, self.total_tokens, self.max_seq_len,
                              q_cal, self.k_c, self.v_c, self.cache_offsets, self.cache_lens,
                              self.indices, self.cal_indices, self.c_q, self.c_out, self.c_lse,
                              self.ws_compress, stream)
        else:
            calidrop_compress_with_lse(self.p, q_win, k, v, seq_offsets, self.total_tokens, self.max_seq_len,
                                       win_lse, q_cal, self.k_c, self.v_c, self.cache_offsets, self.cache_lens,
                                       self.indices, self.cal_indices, self.c_q, self.c_out, self.c_lse,
                                       self.ws_compress, stream)

    def compress_given(self, q_cal, k, v, seq_offsets, stream=None):
        """Alg. 1 steps 4-8 for the retained lists already in self.indices."""
        if getattr(self, "ws_given", None) is None:
            self.ws_given = torch.empty(calidrop_compress_given_workspace_bytes(self.p, self.max_seq_len),
                                        dtype=torch.uint8, device=self.out.device)
        calidrop_compress_given(self.p, q_cal, k, v, seq_offsets, self.total_tokens, self.max_seq_len,
                                self.indices, self.k_c, self.v_c, self.cache_offsets, self.cache_lens,
                                self.c_q, self.c_out, self.c_lse, self.ws_given, stream)

    def compress_h2o(self, q_full, k, v, seq_offsets, n_local=0, stream=None):
        """Alg. 1 with H2O as the eviction strategy; the workspace (self.ws_h2o) keeps the votes."""
        if getattr(self, "ws_h2o", None) is None:
            self.ws_h2o = torch.empty(
                calidrop_compress_h2o_workspace_bytes(self.p, n_local, self.total_tokens, self.max_seq_len),
                dtype=torch.uint8, device=self.out.device)
        calidrop_compress_h2o(self.p, n_local, q_full, k, v, seq_offsets, self.total_tokens, self.max_seq_len,
                              self.k_c, self.v_c, self.cache_offsets, self.cache_lens, self.indices,
                              self.cal_indices, self.c_q, self.c_out, self.c_lse, self.ws_h2o, stream)

    def h2o_region(self, region: int, n_local=0) -> torch.Tensor:
        off, nbytes = calidrop_compress_h2o_workspace_region(self.p, n_local, self.total_tokens,
                                                             self.max_seq_len, region)
        return self.ws_h2o[off:off + nbytes].view(torch.float32)

    def streaming_indices(self, n_sink, seq_offsets, stream=None):
        calidrop_streaming_indices(self.p, n_sink, seq_offsets, self.total_tokens, self.max_seq_len,
                                   self.indices, stream)

    def decode(self, q_t, stream=None, max_cache_len=None, pass_offsets=None):
        # when every sequence has the same capacity and the call's max_cache_len is that capacity the
        # offsets need not be passed (pass_offsets=True still passes them)
        mcl = max_cache_len or self.max_cache_len
        if pass_offsets is None:
            pass_offsets = mcl != self.cap or not self.uniform
        if not pass_offsets and (mcl != self.cap or not self.uniform):
            raise ValueError("the offsets can only be left out when every capacity equals max_cache_len")
        offs = self.cache_offsets if pass_offsets else None
        calidrop_decode(self.p, q_t, self.k_c, self.v_c, offs, self.cache_lens, mcl, self.c_q, self.c_out,
                        self.c_lse, self.out, self.a_lse, self.flags, self.ws_decode, stream)

    def append(self, k_new, v_new, stream=None):
        """Append the K/V rows of the token just generated ([batch][Hkv][D]) to every sequence."""
        calidrop_append(self.p, k_new, v_new, self.k_c, self.v_c, self.cache_offsets, self.cache_lens, stream)

    def recalibrate(self, q_t, k, v, seq_offsets, stream=None):
        """Recomputation branch for the heads the last decode() flagged (updates out/flags/state)."""
        if getattr(self, "ws_recal", None) is None:
            self.ws_recal = torch.empty(calidrop_recalibrate_workspace_bytes(self.p, self.max_seq_len),
                                        dtype=torch.uint8, device=self.out.device)
        calidrop_recalibrate(self.p, q_t, k, v, seq_offsets, self.total_tokens, self.max_seq_len,
                             self.indices, self.cal_indices, self.flags, self.a_lse, self.out, self.c_q,
                             self.c_out, self.c_lse, self.ws_recal, stream)

    def region(self, region: int) -> torch.Tensor:
        off, nbytes = calidrop_compress_workspace_region(self.p, self.total_tokens,
                                                         self.max_seq_len, region)
        return self.ws_compress[off:off + nbytes].view(torch.float32)

    def cache_view(self, which: str, b: int) -> torch.Tensor:
        """[Hkv][cap_b][D] view of sequence b inside k_c / v_c."""
        t = self.k_c if which == "k" else self.v_c
        Hkv, D = self.p.n_kv_heads, self.p.head_dim
        lo, cap = self.offs[b] * Hkv * D, self.caps[b]
        return t[lo:lo + Hkv * cap * D].view(Hkv, cap, D)


def default_scale(head_dim: int) -> float:
    return 1.0 / math.sqrt(head_dim)
