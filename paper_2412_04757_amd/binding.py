"""ctypes binding of libltri.so.

The functions carry the names of the C ABI (include/ltri.h).  torch is used only to
allocate device memory and to name the stream; nothing here computes.  If the shared
library is missing the import of any entry point fails loudly: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None

LTRI_F32, LTRI_BF16 = 0, 1
MAP_SOFTMAX, MAP_LOGIT = 0, 1
REP_MEAN, REP_DYNAMIC = 0, 1
RATIO_ROW, RATIO_COL, RATIO_ROWCOL = 0, 1, 2

EXPORTED_SYMBOLS = [
    "ltri_workspace_bytes", "ltri_create", "ltri_create_dry", "ltri_destroy", "ltri_reset",
    "ltri_set_stream", "ltri_set_attend_stages", "ltri_set_step_timing",
    "ltri_read_step_timing",
    "ltri_append_chunk", "ltri_append_chunk_with_spans", "ltri_retrieve", "ltri_retrieve_persistent",
    "ltri_retrieve_collaborative",
    "ltri_sel_capacity",
    "ltri_force_selection", "ltri_attend", "ltri_attend_static", "ltri_step", "ltri_gather_pack", "ltri_list_capacity",
    "ltri_sync_status", "ltri_token_count", "ltri_span_count", "ltri_get_spans",
    "ltri_get_rep_keys", "ltri_get_selection", "ltri_get_token_list", "ltri_get_index_tokens", "ltri_get_theta",
    "ltri_strerror",
    "ltri_last_error", "ltri_version",
    # include/ltri_bench.h: measurement helpers, not part of the product boundary
    "ltri_measure_mfma_peak", "ltri_measure_copy_peak", "ltri_measure_read_peak",
]


class LtriError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libltri status {status}: {text}")
        self.status = status


class LtriConfig(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("dtype", C.c_int32), ("n_layers", C.c_int32), ("n_seqs", C.c_int32),
        ("max_tokens", C.c_int64), ("chunk_max", C.c_int32), ("n_sink", C.c_int32),
        ("window", C.c_int32), ("k_max", C.c_int32), ("budget_tokens", C.c_int64),
        ("seg_map", C.c_int32), ("theta", C.c_float), ("phi", C.c_float),
        ("max_spans_per_chunk", C.c_int32), ("rep_mode", C.c_int32), ("max_spans", C.c_int32),
        ("lam", C.c_float), ("index_min", C.c_int32), ("index_max", C.c_int32), ("ratio_mode", C.c_int32),
        ("theta_quantile", C.c_float), ("unit_tokens", C.c_int32), ("kv_offload", C.c_int32),
        ("index_block_max", C.c_int32),
    ]


def library_path() -> str:
    return os.path.join(_HERE, "libltri.so")


def load_library() -> C.CDLL:
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python __graft_entry__.py` "
                          "(there is no fallback implementation)")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    pi32 = C.POINTER(C.c_int32)
    sig = {
        "ltri_workspace_bytes": [C.POINTER(LtriConfig), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)],
        "ltri_create": [C.POINTER(LtriConfig), vp, vp, vp, vp, vp, C.POINTER(vp)],
        "ltri_create_dry": [C.POINTER(LtriConfig), C.POINTER(vp)],
        "ltri_destroy": [vp],
        "ltri_reset": [vp, i32],
        "ltri_set_stream": [vp, vp],
        "ltri_set_attend_stages": [vp, i32],
        "ltri_append_chunk": [vp, i32, i32, i32, vp, vp, vp, i32],
        "ltri_append_chunk_with_spans": [vp, i32, i32, vp, vp, i32, pi32, pi32],
        "ltri_retrieve": [vp, i32, i32, i32, vp, i32, vp, vp],
        "ltri_sel_capacity": [vp],
        "ltri_retrieve_persistent": [vp, i32, i32, i32],
        "ltri_retrieve_collaborative": [vp, i32, i32, i32, vp, i32, C.POINTER(C.c_float), vp, vp],
        "ltri_force_selection": [vp, i32, i32, i32, pi32, i32],
        "ltri_attend": [vp, i32, i32, i32, vp, i32, vp, vp],
        "ltri_attend_static": [vp, i32, i32, i32, vp, i32, vp, vp],
        "ltri_set_step_timing": [vp, i32],
        "ltri_read_step_timing": [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), i32, pi32],
        "ltri_step": [vp, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp],
        "ltri_gather_pack": [vp, i32, i32, vp, vp, vp],
        "ltri_list_capacity": [vp],
        "ltri_sync_status": [vp],
        "ltri_token_count": [vp, i32, i32, C.POINTER(i64)],
        "ltri_span_count": [vp, i32, i32, i32, pi32],
        "ltri_get_spans": [vp, i32, i32, i32, pi32, pi32, i32],
        "ltri_get_rep_keys": [vp, i32, i32, i32, vp, i32],
        "ltri_get_selection": [vp, i32, i32, i32, pi32, i32, pi32, C.POINTER(C.c_double)],
        "ltri_get_token_list": [vp, i32, i32, i32, pi32, i32, pi32],
        "ltri_get_index_tokens": [vp, i32, i32, i32, C.POINTER(C.c_uint32), i32],
        "ltri_get_theta": [vp, i32, i32, i32, C.POINTER(C.c_double)],
        "ltri_measure_mfma_peak": [vp, C.c_size_t, i32, vp, C.POINTER(C.c_double)],
        "ltri_measure_copy_peak": [vp, vp, C.c_size_t, vp, C.POINTER(C.c_double)],
        "ltri_measure_read_peak": [vp, C.c_size_t, vp, C.c_size_t, vp, C.POINTER(C.c_double)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int32
    lib.ltri_strerror.argtypes = [i32]
    lib.ltri_strerror.restype = C.c_char_p
    lib.ltri_last_error.argtypes = [vp]
    lib.ltri_last_error.restype = C.c_char_p
    lib.ltri_version.argtypes = []
    lib.ltri_version.restype = C.c_char_p
    _LIB = lib
    return lib


def config_from_workload(w, max_tokens: Optional[int] = None, theta: float = 0.0, phi: float = 0.0,
                         seg_map: int = MAP_LOGIT, n_layers: Optional[int] = None,
                         n_seqs: Optional[int] = None, max_spans: int = 0,
                         max_spans_per_chunk: int = 0, window: Optional[int] = None,
                         n_sink: Optional[int] = None, k_max: Optional[int] = None,
                         budget_tokens: Optional[int] = None, chunk_max: Optional[int] = None,
                         rep_mode: int = REP_MEAN, lam: float = 3.0, index_min: int = 1, index_max: int = 0,
                         ratio_mode: int = RATIO_ROW, theta_quantile: float = 0.0,
                         unit_tokens: int = 0, kv_offload: int = 0, index_block_max: int = 0) -> LtriConfig:
    return LtriConfig(
        n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
        dtype=LTRI_F32 if w.dtype == "f32" else LTRI_BF16,
        n_layers=w.n_layers if n_layers is None else n_layers,
        n_seqs=w.n_seqs if n_seqs is None else n_seqs,
        max_tokens=w.context if max_tokens is None else max_tokens,
        chunk_max=w.chunk if chunk_max is None else chunk_max,
        n_sink=w.n_sink if n_sink is None else n_sink,
        window=w.window if window is None else window,
        k_max=w.k_max if k_max is None else k_max,
        budget_tokens=w.budget_tokens if budget_tokens is None else budget_tokens,
        seg_map=seg_map, theta=theta, phi=phi, max_spans_per_chunk=max_spans_per_chunk,
        rep_mode=rep_mode, max_spans=max_spans, lam=lam, index_min=index_min, index_max=index_max,
        ratio_mode=ratio_mode, theta_quantile=theta_quantile, unit_tokens=unit_tokens, kv_offload=kv_offload,
        index_block_max=index_block_max)


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None) -> Optional[int]:
    """Device address of a dense tensor (the C ABI takes plain pointers to row-major buffers)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):      # a stand-in with an address (dry contexts in the host tests)
        return t.data_ptr()
    if not t.is_contiguous():
        raise ValueError(f"libltri takes dense row-major buffers; got strides {tuple(t.stride())} for shape {tuple(t.shape)}")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected a {dtype} tensor, got {t.dtype}")
    return t.data_ptr()


class LtriContext:
    """Owns the device buffers (torch tensors) and the ltri_ctx handle."""

    def __init__(self, cfg: LtriConfig, device: Optional[torch.device], dry: bool = False,
                 stream: Optional[torch.cuda.Stream] = None):
        self.lib = load_library()
        self.cfg = cfg
        self.dry = dry
        self.handle = C.c_void_p()
        self.tdtype = torch.float32 if cfg.dtype == LTRI_F32 else torch.bfloat16
        sb, cb = C.c_size_t(), C.c_size_t()
        self._check(self.lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)), None)
        self.state_bytes, self.scratch_bytes = sb.value, cb.value
        if dry:
            self._check(self.lib.ltri_create_dry(C.byref(cfg), C.byref(self.handle)), None)
            return
        self.device = device
        n_arena = cfg.n_layers * cfg.n_seqs * cfg.n_kv_heads * cfg.max_tokens * cfg.head_dim
        if cfg.kv_offload:      # host arenas in pinned memory (device-visible); the device pools live in `state`
            self.k_arena = torch.empty(n_arena, dtype=self.tdtype, pin_memory=True)
            self.v_arena = torch.empty(n_arena, dtype=self.tdtype, pin_memory=True)
        else:
            self.k_arena = torch.empty(n_arena, dtype=self.tdtype, device=device)
            self.v_arena = torch.empty(n_arena, dtype=self.tdtype, device=device)
        self.state = torch.empty(self.state_bytes, dtype=torch.uint8, device=device)
        self.scratch = torch.empty(self.scratch_bytes, dtype=torch.uint8, device=device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(device)
        self._check(self.lib.ltri_create(C.byref(cfg), self.k_arena.data_ptr(), self.v_arena.data_ptr(),
                                         self.state.data_ptr(), self.scratch.data_ptr(),
                                         self.stream.cuda_stream, C.byref(self.handle)), None)
        self.sel_cap = self.lib.ltri_sel_capacity(self.handle)
        self.list_cap = self.lib.ltri_list_capacity(self.handle)

    def _check(self, status: int, _unused) -> None:
        if status != 0:
            detail = ""
            if self.handle:
                detail = self.lib.ltri_last_error(self.handle).decode()
            raise LtriError(status, f"{self.lib.ltri_strerror(status).decode()}: {detail}")

    def close(self) -> None:
        if self.handle:
            self.lib.ltri_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # arenas viewed as [n_layers][n_seqs][n_kv_heads][max_tokens][head_dim]
    def arena_views(self) -> Tuple[torch.Tensor, torch.Tensor]:
        c = self.cfg
        shape = (c.n_layers, c.n_seqs, c.n_kv_heads, c.max_tokens, c.head_dim)
        return self.k_arena.view(shape), self.v_arena.view(shape)

    # ---- the C ABI, same names ----
    def set_stream(self, stream: "torch.cuda.Stream") -> None:
        self._check(self.lib.ltri_set_stream(self.handle, stream.cuda_stream), None)
        self.stream = stream

    def set_step_timing(self, on: bool) -> None:
        self._check(self.lib.ltri_set_step_timing(self.handle, int(on)), None)

    def read_step_timing(self, cap: int = 4096) -> Tuple[np.ndarray, np.ndarray]:
        """Durations (ms) of the two attention launches of every ltri_step since the last read."""
        a = np.zeros(cap, np.float32)
        b = np.zeros(cap, np.float32)
        n = C.c_int32()
        self._check(self.lib.ltri_read_step_timing(self.handle, a.ctypes.data_as(C.POINTER(C.c_float)),
                                                   b.ctypes.data_as(C.POINTER(C.c_float)), cap, C.byref(n)), None)
        return a[:n.value], b[:n.value]

    def set_attend_stages(self, stages: int) -> None:
        self._check(self.lib.ltri_set_attend_stages(self.handle, stages), None)

    def reset(self, seq: int) -> None:
        self._check(self.lib.ltri_reset(self.handle, seq), None)

    def append_chunk(self, layer: int, seq_begin: int, seq_count: int, n_new: int,
                     k_chunk: Optional[torch.Tensor] = None, v_chunk: Optional[torch.Tensor] = None,
                     q_seg: Optional[torch.Tensor] = None) -> None:
        t = self.tdtype
        self._check(self.lib.ltri_append_chunk(self.handle, layer, seq_begin, seq_count, _ptr(k_chunk, t),
                                               _ptr(v_chunk, t), _ptr(q_seg, t), n_new), None)

    def append_chunk_with_spans(self, layer: int, seq: int, n_new: int, bounds: List[np.ndarray],
                                k_chunk: Optional[torch.Tensor] = None,
                                v_chunk: Optional[torch.Tensor] = None) -> None:
        flat = np.concatenate([np.asarray(b, np.int32) for b in bounds]).astype(np.int32)
        nb = np.asarray([len(b) for b in bounds], np.int32)
        self._check(self.lib.ltri_append_chunk_with_spans(
            self.handle, layer, seq, _ptr(k_chunk, self.tdtype), _ptr(v_chunk, self.tdtype), n_new,
            flat.ctypes.data_as(C.POINTER(C.c_int32)), nb.ctypes.data_as(C.POINTER(C.c_int32))), None)

    def retrieve(self, layer: int, seq_begin: int, seq_count: int, q: torch.Tensor,
                 sel_ids: Optional[torch.Tensor] = None, sel_cnt: Optional[torch.Tensor] = None) -> None:
        n_q = q.shape[-3]
        self._check(self.lib.ltri_retrieve(self.handle, layer, seq_begin, seq_count, _ptr(q, self.tdtype), n_q,
                                           _ptr(sel_ids, torch.int32), _ptr(sel_cnt, torch.int32)), None)

    def retrieve_collaborative(self, layer: int, seq_begin: int, seq_count: int, q: torch.Tensor, layer_weights,
                               sel_ids: Optional[torch.Tensor] = None, sel_cnt: Optional[torch.Tensor] = None) -> None:
        w = np.asarray(list(layer_weights), np.float32)
        n_q = q.shape[-3]
        self._check(self.lib.ltri_retrieve_collaborative(self.handle, layer, seq_begin, seq_count, _ptr(q, self.tdtype), n_q,
                                                         w.ctypes.data_as(C.POINTER(C.c_float)), _ptr(sel_ids, torch.int32),
                                                         _ptr(sel_cnt, torch.int32)), None)

    def retrieve_persistent(self, layer: int, seq_begin: int, seq_count: int) -> None:
        self._check(self.lib.ltri_retrieve_persistent(self.handle, layer, seq_begin, seq_count), None)

    def force_selection(self, layer: int, seq: int, kv_head: int, ids) -> None:
        arr = np.asarray(list(ids), np.int32)
        self._check(self.lib.ltri_force_selection(self.handle, layer, seq, kv_head,
                                                  arr.ctypes.data_as(C.POINTER(C.c_int32)), len(arr)), None)

    def attend(self, layer: int, seq_begin: int, seq_count: int, q: torch.Tensor,
               out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None) -> torch.Tensor:
        n_q = q.shape[-3]
        if out is None and not self.dry:
            out = torch.empty((seq_count, n_q, self.cfg.n_q_heads, self.cfg.head_dim), dtype=self.tdtype,
                              device=q.device)
        self._check(self.lib.ltri_attend(self.handle, layer, seq_begin, seq_count, _ptr(q, self.tdtype), n_q,
                                         _ptr(out, self.tdtype) if out is not None else 1, _ptr(lse, torch.float32)), None)
        return out

    def attend_static(self, layer: int, seq_begin: int, seq_count: int, q: torch.Tensor, out: torch.Tensor,
                      lse: Optional[torch.Tensor] = None) -> torch.Tensor:
        """ltri_attend_static: the caller passes `out`; nothing is allocated by the call."""
        n_q = q.shape[-3]
        self._check(self.lib.ltri_attend_static(self.handle, layer, seq_begin, seq_count, _ptr(q, self.tdtype), n_q,
                                                _ptr(out, self.tdtype) if out is not None else 1,
                                                _ptr(lse, torch.float32)), None)
        return out

    def step(self, layer: int, seq_begin: int, seq_count: int, k_chunk: Optional[torch.Tensor],
             v_chunk: Optional[torch.Tensor], q: torch.Tensor, q_seg: Optional[torch.Tensor] = None,
             out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None) -> torch.Tensor:
        n_new = q.shape[-3]
        if out is None and not self.dry:
            out = torch.empty((seq_count, n_new, self.cfg.n_q_heads, self.cfg.head_dim), dtype=self.tdtype,
                              device=q.device)
        t = self.tdtype
        self._check(self.lib.ltri_step(self.handle, layer, seq_begin, seq_count, _ptr(k_chunk, t), _ptr(v_chunk, t),
                                       _ptr(q_seg, t), _ptr(q, t), n_new, _ptr(out, t) if out is not None else 1,
                                       _ptr(lse, torch.float32)), None)
        return out

    def gather_pack(self, layer: int, seq: int, k_packed: torch.Tensor, v_packed: torch.Tensor,
                    n_tokens: Optional[torch.Tensor] = None) -> None:
        self._check(self.lib.ltri_gather_pack(self.handle, layer, seq, _ptr(k_packed, self.tdtype),
                                              _ptr(v_packed, self.tdtype), _ptr(n_tokens, torch.int32)), None)

    def sync_status(self) -> int:
        return int(self.lib.ltri_sync_status(self.handle))

    def token_count(self, layer: int, seq: int) -> int:
        n = C.c_int64()
        self._check(self.lib.ltri_token_count(self.handle, layer, seq, C.byref(n)), None)
        return n.value

    def span_count(self, layer: int, seq: int, kv_head: int) -> int:
        n = C.c_int32()
        self._check(self.lib.ltri_span_count(self.handle, layer, seq, kv_head, C.byref(n)), None)
        return n.value

    def get_spans(self, layer: int, seq: int, kv_head: int) -> Tuple[np.ndarray, np.ndarray]:
        n = self.span_count(layer, seq, kv_head)
        s = np.zeros(max(n, 1), np.int32)
        l = np.zeros(max(n, 1), np.int32)
        self._check(self.lib.ltri_get_spans(self.handle, layer, seq, kv_head,
                                            s.ctypes.data_as(C.POINTER(C.c_int32)),
                                            l.ctypes.data_as(C.POINTER(C.c_int32)), n), None)
        return s[:n], l[:n]

    def get_rep_keys(self, layer: int, seq: int, kv_head: int) -> torch.Tensor:
        n = self.span_count(layer, seq, kv_head)
        buf = torch.zeros((max(n, 1), self.cfg.head_dim), dtype=self.tdtype)
        self._check(self.lib.ltri_get_rep_keys(self.handle, layer, seq, kv_head, buf.data_ptr(), n), None)
        return buf[:n]

    def get_selection(self, layer: int, seq: int, kv_head: int) -> Tuple[np.ndarray, np.ndarray]:
        n_sp = self.span_count(layer, seq, kv_head)
        ids = np.zeros(max(self.sel_cap, 1), np.int32)
        scores = np.zeros(max(n_sp, 1), np.float64)
        n = C.c_int32()
        self._check(self.lib.ltri_get_selection(self.handle, layer, seq, kv_head,
                                                ids.ctypes.data_as(C.POINTER(C.c_int32)), self.sel_cap,
                                                C.byref(n), scores.ctypes.data_as(C.POINTER(C.c_double))), None)
        return ids[:n.value], scores[:n_sp]

    def get_token_list(self, layer: int, seq: int, kv_head: int) -> np.ndarray:
        toks = np.zeros(max(self.list_cap, 1), np.int32)
        n = C.c_int32()
        self._check(self.lib.ltri_get_token_list(self.handle, layer, seq, kv_head,
                                                 toks.ctypes.data_as(C.POINTER(C.c_int32)), self.list_cap,
                                                 C.byref(n)), None)
        return toks[:n.value]

    def get_index_tokens(self, layer: int, seq: int, kv_head: int, chunk_len: int) -> np.ndarray:
        """Chunk-local positions of the index tokens of the chunk appended last (dynamic index vectors)."""
        words = np.zeros((chunk_len + 31) // 32, np.uint32)
        self._check(self.lib.ltri_get_index_tokens(self.handle, layer, seq, kv_head,
                                                   words.ctypes.data_as(C.POINTER(C.c_uint32)), len(words)), None)
        bits = np.unpackbits(words.view(np.uint8), bitorder="little")[:chunk_len]
        return np.flatnonzero(bits).astype(np.int64)

    def get_theta(self, layer: int, seq: int, kv_head: int) -> float:
        """The percentile threshold the last append used for (layer, seq, kv_head) (ltri_get_theta)."""
        out = C.c_double()
        self._check(self.lib.ltri_get_theta(self.handle, layer, seq, kv_head, C.byref(out)), None)
        return out.value


def measure_mfma_peak(device, random_operands: bool = False) -> float:
    """TFLOP/s of back-to-back bf16 matrix-core products on `device` (ltri_measure_mfma_peak)."""
    lib = load_library()
    sink = torch.empty(1 << 17, dtype=torch.float32, device=device)
    out = C.c_double()
    st = lib.ltri_measure_mfma_peak(sink.data_ptr(), sink.numel() * 4, int(random_operands),
                                    torch.cuda.current_stream(device).cuda_stream,
                                    C.byref(out))
    if st != 0:
        raise LtriError(st, lib.ltri_strerror(st).decode())
    return out.value


def measure_copy_peak(device, n_bytes: int = 1 << 30) -> float:
    """GB/s (read + write) of a plain device copy of n_bytes on `device` (ltri_measure_copy_peak)."""
    lib = load_library()
    src = torch.empty(n_bytes, dtype=torch.uint8, device=device)
    dst = torch.empty_like(src)
    src.zero_()
    out = C.c_double()
    st = lib.ltri_measure_copy_peak(dst.data_ptr(), src.data_ptr(), n_bytes, torch.cuda.current_stream(device).cuda_stream,
                                    C.byref(out))
    if st != 0:
        raise LtriError(st, lib.ltri_strerror(st).decode())
    return out.value


def measure_read_peak(device, n_bytes: int = 1 << 30) -> float:
    """GB/s of a streaming read of n_bytes on `device` (ltri_measure_read_peak)."""
    lib = load_library()
    src = torch.empty(n_bytes, dtype=torch.uint8, device=device)
    src.zero_()
    sink = torch.empty(1 << 17, dtype=torch.int32, device=device)
    out = C.c_double()
    st = lib.ltri_measure_read_peak(src.data_ptr(), n_bytes, sink.data_ptr(), sink.numel() * 4,
                                    torch.cuda.current_stream(device).cuda_stream, C.byref(out))
    if st != 0:
        raise LtriError(st, lib.ltri_strerror(st).decode())
    return out.value
