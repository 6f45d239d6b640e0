"""ctypes binding of libiwdft.so -- same names as include/iwdft.h, argument marshalling only.

torch is used for device buffers and streams; every arithmetic step runs in the
library's HIP kernels.  There is no fallback: if the shared library is missing
or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

IWDFT_OK = 0
IWDFT_ERR_ARG, IWDFT_ERR_BINS, IWDFT_ERR_SIZE = -1, -2, -3
IWDFT_ERR_STATE, IWDFT_ERR_HIP, IWDFT_ERR_UNSUPPORTED = -4, -5, -6
IWDFT_F32, IWDFT_BF16 = 0, 1
IWDFT_FLAG_DIRECT_SYNTHESIS = 1
IWDFT_FLAG_DENSE_PREFILL = 2
IWDFT_FLAG_FFT_PREFILL = 4
IWDFT_FLAG_SHORTCUT = 8
IWDFT_FLAG_SERIAL_PHASES = 16
IWDFT_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTED = [
    "iwdft_query_bytes", "iwdft_create", "iwdft_destroy", "iwdft_prefill", "iwdft_append",
    "iwdft_reconstruct", "iwdft_reconstruct_grid", "compressed_decode_attn", "iwdft_append_attn", "iwdft_export_coeffs", "iwdft_export_bins",
    "iwdft_num_tokens", "iwdft_set_num_tokens", "iwdft_last_error", "iwdft_phase_timing", "iwdft_phase_times", "iwdft_prefill_kind", "iwdft_attn_kind", "iwdft_attn_pipelined",
    "iwdft_select_bins", "iwdft_ablate_chunk", "iwdft_flush", "compressed_decode_attn_static",
]

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libiwdft.so")


class IwdftError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libiwdft error {code}: {msg}")
        self.code = code


class iwdft_desc(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("batch", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
        ("M", ctypes.c_int64),
        ("bin_offsets", ctypes.POINTER(ctypes.c_int64)),
        ("bins", ctypes.POINTER(ctypes.c_int32)),
        ("bin_weights", ctypes.POINTER(ctypes.c_float)),
        ("flags", ctypes.c_uint32), ("n_sink", ctypes.c_int32), ("n_recent", ctypes.c_int32),
        ("write_every", ctypes.c_uint32),
    ]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libiwdft.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2507_20030_amd.build` "
                          "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    dp = ctypes.POINTER(iwdft_desc)
    szp = ctypes.POINTER(ctypes.c_size_t)
    lib.iwdft_query_bytes.argtypes = [dp, szp, szp]
    lib.iwdft_create.argtypes = [dp, vp, ctypes.c_size_t, vp, ctypes.c_size_t, ctypes.POINTER(vp)]
    lib.iwdft_destroy.argtypes = [vp]
    lib.iwdft_prefill.argtypes = [vp, vp, vp, vp]
    lib.iwdft_append.argtypes = [vp, vp, vp, vp]
    lib.iwdft_reconstruct.argtypes = [vp, i32, i64, i64, vp, vp, vp]
    lib.iwdft_reconstruct_grid.argtypes = [vp, i32, i64, i64, i64, vp, vp, vp]
    lib.compressed_decode_attn.argtypes = [vp, vp, vp, f32, vp]
    lib.compressed_decode_attn_static.argtypes = [vp, vp, vp, f32, vp]
    lib.iwdft_append_attn.argtypes = [vp, vp, vp, vp, vp, f32, vp]
    lib.iwdft_prefill_kind.argtypes = [vp]
    lib.iwdft_attn_kind.argtypes = [vp]
    lib.iwdft_attn_pipelined.argtypes = [vp]
    lib.iwdft_flush.argtypes = [vp, vp]
    lib.iwdft_select_bins.argtypes = [ctypes.POINTER(ctypes.c_float), i32, i32, i64, ctypes.c_double,
                                      ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32), i64]
    lib.iwdft_ablate_chunk.argtypes = [vp, vp, i64, i64, i32, i32, i32, i32, vp]
    lib.iwdft_phase_timing.argtypes = [vp, i32]
    lib.iwdft_phase_times.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.iwdft_export_coeffs.argtypes = [vp, i32, vp, vp, vp]
    lib.iwdft_export_bins.argtypes = [vp, i32, vp, vp]
    lib.iwdft_num_tokens.argtypes = [vp]
    lib.iwdft_num_tokens.restype = i64
    lib.iwdft_set_num_tokens.argtypes = [vp, i64]
    lib.iwdft_last_error.argtypes = []
    lib.iwdft_last_error.restype = ctypes.c_char_p
    for name in EXPORTED:
        if name not in ("iwdft_num_tokens", "iwdft_last_error"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def iwdft_last_error() -> str:
    return load_library().iwdft_last_error().decode()


def _check(rc: int) -> None:
    if rc != IWDFT_OK:
        raise IwdftError(rc, iwdft_last_error())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


class Descriptor:
    """Host-side description of a cache; keeps the numpy arrays the C struct points into."""

    def __init__(self, n_layers: int, batch: int, n_kv_heads: int, n_q_heads: int, head_dim: int,
                 kv_dtype: int, M: int, bins: Sequence[np.ndarray],
                 bin_weights: Optional[Sequence[np.ndarray]] = None, flags: int = 0,
                 n_sink: int = 0, n_recent: int = 0, write_every: int = 0):
        self.bins = [np.ascontiguousarray(b, dtype=np.int32) for b in bins]
        self._offsets = np.zeros(len(self.bins) + 1, dtype=np.int64)
        self._offsets[1:] = np.cumsum([len(b) for b in self.bins])
        self._flat = np.ascontiguousarray(np.concatenate(self.bins) if self.bins else np.zeros(0, np.int32))
        self._w = None
        if bin_weights is not None:
            self._w = np.ascontiguousarray(np.concatenate([np.asarray(w, np.float32) for w in bin_weights]))
        self.c = iwdft_desc(
            n_layers, batch, n_kv_heads, n_q_heads, head_dim, kv_dtype, M,
            self._offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
            self._flat.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
            self._w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) if self._w is not None else None,
            flags, n_sink, n_recent, write_every)


def iwdft_query_bytes(desc: Descriptor):
    s, w = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().iwdft_query_bytes(ctypes.byref(desc.c), ctypes.byref(s), ctypes.byref(w)))
    return s.value, w.value


def iwdft_create(desc: Descriptor, state: torch.Tensor, workspace: torch.Tensor) -> ctypes.c_void_p:
    ctx = ctypes.c_void_p()
    _check(load_library().iwdft_create(ctypes.byref(desc.c), _ptr(state), state.numel() * state.element_size(),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       ctypes.byref(ctx)))
    return ctx


def iwdft_destroy(ctx) -> None:
    _check(load_library().iwdft_destroy(ctx))


def iwdft_prefill(ctx, K: torch.Tensor, V: torch.Tensor, stream=None) -> None:
    _check(load_library().iwdft_prefill(ctx, _ptr(K), _ptr(V), _stream(stream)))


def iwdft_append(ctx, tok_k: torch.Tensor, tok_v: torch.Tensor, stream=None) -> None:
    _check(load_library().iwdft_append(ctx, _ptr(tok_k), _ptr(tok_v), _stream(stream)))


def iwdft_reconstruct(ctx, layer: int, a0: int, n_slots: int, Kt, Vt, stream=None) -> None:
    _check(load_library().iwdft_reconstruct(ctx, layer, a0, n_slots, _ptr(Kt), _ptr(Vt), _stream(stream)))


def iwdft_reconstruct_grid(ctx, layer: int, a0: int, stride: int, n_slots: int, Kt, Vt, stream=None) -> None:
    _check(load_library().iwdft_reconstruct_grid(ctx, layer, a0, stride, n_slots, _ptr(Kt), _ptr(Vt), _stream(stream)))


def compressed_decode_attn(ctx, q: torch.Tensor, out: torch.Tensor, scale: float = 0.0, stream=None) -> None:
    _check(load_library().compressed_decode_attn(ctx, _ptr(q), _ptr(out), scale, _stream(stream)))


def compressed_decode_attn_static(ctx, q: torch.Tensor, out: torch.Tensor, scale: float = 0.0, stream=None) -> None:
    _check(load_library().compressed_decode_attn_static(ctx, _ptr(q), _ptr(out), scale, _stream(stream)))


def iwdft_append_attn(ctx, tok_k, tok_v, q, out, scale: float = 0.0, stream=None) -> None:
    _check(load_library().iwdft_append_attn(ctx, _ptr(tok_k), _ptr(tok_v), _ptr(q), _ptr(out), scale,
                                            _stream(stream)))


def iwdft_select_bins(delta: np.ndarray, M: int, r: float):
    """Per-layer kept-bin lists (int32 arrays) from a [layers, chunks] importance matrix."""
    delta = np.ascontiguousarray(delta, dtype=np.float32)
    n_layers, n_chunks = delta.shape
    lib = load_library()
    off = (ctypes.c_int64 * (n_layers + 1))()
    dp = delta.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
    rc = lib.iwdft_select_bins(dp, n_layers, n_chunks, M, float(r), off, None, 0)   # sizing call
    if rc != IWDFT_ERR_SIZE:
        _check(rc)
    bins = np.empty(max(int(off[n_layers]), 1), dtype=np.int32)
    _check(lib.iwdft_select_bins(dp, n_layers, n_chunks, M, float(r), off,
                                 bins.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), bins.size))
    return [bins[off[l]:off[l + 1]].copy() for l in range(n_layers)]


def iwdft_ablate_chunk(x: torch.Tensor, out: torch.Tensor, n_chunks: int, chunk: int, stream=None) -> None:
    """x, out: [..., M, head_dim] contiguous device tensors of the same shape and dtype."""
    M, D = x.shape[-2], x.shape[-1]
    n_slices = x.numel() // (M * D)
    _check(load_library().iwdft_ablate_chunk(_ptr(x), _ptr(out), n_slices, M, D,
                                             IWDFT_F32 if x.dtype == torch.float32 else IWDFT_BF16,
                                             n_chunks, chunk, _stream(stream)))


def iwdft_flush(ctx, stream=None) -> None:
    _check(load_library().iwdft_flush(ctx, _stream(stream)))


def iwdft_prefill_kind(ctx) -> str:
    return {0: "dense", 1: "fft"}[load_library().iwdft_prefill_kind(ctx)]


def iwdft_attn_kind(ctx) -> str:
    return {0: "direct", 1: "fft", 2: "chirp"}[load_library().iwdft_attn_kind(ctx)]


def iwdft_attn_pipelined(ctx) -> bool:
    return load_library().iwdft_attn_pipelined(ctx) == 1


def iwdft_phase_timing(ctx, enable: bool) -> None:
    _check(load_library().iwdft_phase_timing(ctx, 1 if enable else 0))


def iwdft_phase_times(ctx):
    """(ms of phases A, B, C summed over the marked calls since the last read-out, number of calls)."""
    ms = (ctypes.c_double * 3)()
    n = ctypes.c_int64(0)
    _check(load_library().iwdft_phase_times(ctx, ms, ctypes.byref(n)))
    return [ms[0], ms[1], ms[2]], n.value


def iwdft_export_coeffs(ctx, layer: int, SK, SV, stream=None) -> None:
    _check(load_library().iwdft_export_coeffs(ctx, layer, _ptr(SK), _ptr(SV), _stream(stream)))


def iwdft_export_bins(ctx, layer: int, out: torch.Tensor, stream=None) -> None:
    _check(load_library().iwdft_export_bins(ctx, layer, _ptr(out), _stream(stream)))


def iwdft_num_tokens(ctx) -> int:
    return int(load_library().iwdft_num_tokens(ctx))


def iwdft_set_num_tokens(ctx, T: int) -> None:
    _check(load_library().iwdft_set_num_tokens(ctx, T))


class Cache:
    """Owns the torch buffers behind one iwdft_ctx; methods forward to the C calls."""

    def __init__(self, n_layers, batch, n_kv_heads, n_q_heads, head_dim, dtype: torch.dtype, M,
                 bins, bin_weights=None, flags=0, device="cuda:0", n_sink=0, n_recent=0, write_every=0):
        if dtype not in (torch.float32, torch.bfloat16):
            raise ValueError("dtype must be float32 or bfloat16")
        self.dtype, self.device = dtype, torch.device(device)
        self.desc = Descriptor(n_layers, batch, n_kv_heads, n_q_heads, head_dim,
                               IWDFT_F32 if dtype == torch.float32 else IWDFT_BF16, M, bins, bin_weights, flags,
                               n_sink, n_recent, write_every)
        self.state_bytes, self.ws_bytes = iwdft_query_bytes(self.desc)
        with torch.cuda.device(self.device):
            self.state = torch.empty(self.state_bytes, dtype=torch.uint8, device=self.device)
            self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
            self.ctx = iwdft_create(self.desc, self.state, self.workspace)
        self.shape = (n_layers, batch, n_kv_heads, n_q_heads, head_dim)

    def close(self):
        if self.ctx is not None:
            iwdft_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def T(self) -> int:
        return iwdft_num_tokens(self.ctx)

    def prefill(self, K, V, stream=None):
        iwdft_prefill(self.ctx, K, V, stream)

    def append(self, tok_k, tok_v, stream=None):
        iwdft_append(self.ctx, tok_k, tok_v, stream)

    def attend(self, q, out=None, scale=0.0, stream=None):
        if out is None:
            out = torch.empty_like(q)
        compressed_decode_attn(self.ctx, q, out, scale, stream)
        return out

    def step(self, tok_k, tok_v, q, out=None, scale=0.0, stream=None):
        """Fused decode step: append (tok_k, tok_v), then attend with q."""
        if out is None:
            out = torch.empty_like(q)
        iwdft_append_attn(self.ctx, tok_k, tok_v, q, out, scale, stream)
        return out

    def flush(self, stream=None):
        iwdft_flush(self.ctx, stream)

    def reconstruct(self, layer, a0, n_slots, want_k=True, want_v=True, stream=None, stride=1):
        L, B, H, _, D = self.shape
        mk = lambda: torch.empty((B, H, n_slots, D), dtype=self.dtype, device=self.device)
        Kt, Vt = (mk() if want_k else None), (mk() if want_v else None)
        if stride == 1:
            iwdft_reconstruct(self.ctx, layer, a0, n_slots, Kt, Vt, stream)
        else:
            iwdft_reconstruct_grid(self.ctx, layer, a0, stride, n_slots, Kt, Vt, stream)
        return Kt, Vt

    def export_coeffs(self, layer, stream=None):
        L, B, H, _, D = self.shape
        nb = len(self.desc.bins[layer])
        SK = torch.empty((B, H, nb, D, 2), dtype=torch.float32, device=self.device)
        SV = torch.empty_like(SK)
        iwdft_export_coeffs(self.ctx, layer, SK, SV, stream)
        return torch.view_as_complex(SK), torch.view_as_complex(SV)

    def export_bins(self, layer, stream=None):
        out = torch.empty(len(self.desc.bins[layer]), dtype=torch.int32, device=self.device)
        iwdft_export_bins(self.ctx, layer, out, stream)
        return out
