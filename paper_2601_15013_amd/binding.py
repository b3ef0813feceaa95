"""ctypes binding of libradixmlp.so: same names as the C ABI, argument marshalling only.

Every step of the path runs inside the library's HIP kernels.  PyTorch is used here for
device memory (tensors are passed as raw device pointers) and for the current HIP stream.
There is no fallback: if the shared library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Any, Mapping, Optional, Sequence, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libradixmlp.so")

RADIX_F32, RADIX_BF16, RADIX_F16 = 0, 1, 2
_DTYPES = {"f32": RADIX_F32, "bf16": RADIX_BF16, "f16": RADIX_F16}

EXPORTS = (
    "radix_model_create", "radix_model_destroy", "radix_model_hilo_layers", "radix_index_workspace_bytes", "radix_workspace_bytes",
    "radix_build_index", "radix_build_index_static", "radix_prefill_forward", "radix_prefill_forward_nodedup",
    "radix_dedup_decision",
    "radix_lm_head_workspace_bytes", "radix_lm_head",
    "radix_index_select_rows", "radix_device_status", "radix_status_string",
    "radix_timing_enable", "radix_timing_collect", "radix_debug_gemm_tile", "radix_debug_gemm_band",
)

TIMING_CATEGORIES = ("gemm_qkv", "gemm_o", "gemm_gateup", "gemm_down", "attention", "scatter", "gather", "rowops",
                     "gemm_hilo_layers")


class RadixError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib().radix_status_string(code).decode() if _LIB is not None else "?"
        super().__init__(f"{where}: {msg} (status {code})")


class radix_model_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d", "n_q_heads", "n_kv_heads", "head_dim", "d_int", "vocab",
                                          "max_pos", "qk_norm", "dtype", "compute_dtype", "hilo_layers", "fold_norms", "lm_head")] + [("eps", C.c_float), ("rope_base", C.c_float)]


class radix_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "wq", "wk", "wv", "gq", "gk", "wo", "g2", "wg", "wu", "wd")]


class radix_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("gf", C.c_void_p), ("layers_host", C.POINTER(radix_layer_weights)),
                ("lm_head", C.c_void_p)]


class radix_fwd_opts(C.Structure):
    _fields_ = [("threshold", C.c_float), ("force_dedup", C.c_int32), ("attention_mode", C.c_int32),
                ("pad_compact_to", C.c_int32)]


_LIB: Optional[C.CDLL] = None


def _lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2601_15013_amd.build). "
                "There is no CPU or PyTorch fallback for this path.")
        lib = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        lib.radix_model_create.argtypes = [C.POINTER(radix_model_config), C.POINTER(radix_weights), C.POINTER(vp)]
        lib.radix_model_destroy.argtypes = [vp]
        lib.radix_model_hilo_layers.argtypes = [vp]
        lib.radix_index_workspace_bytes.argtypes = [i32, C.POINTER(sz)]
        lib.radix_workspace_bytes.argtypes = [vp, i32, i32, C.POINTER(sz)]
        lib.radix_build_index.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, C.POINTER(i32), vp, sz, vp]
        lib.radix_build_index_static.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, C.POINTER(i32), vp]
        lib.radix_prefill_forward.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, i32, C.POINTER(radix_fwd_opts),
                                              vp, vp, sz, vp]
        lib.radix_prefill_forward_nodedup.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, sz, vp]
        lib.radix_dedup_decision.argtypes = [C.POINTER(radix_model_config), i32, i32, i32, C.POINTER(radix_fwd_opts),
                                             C.POINTER(i32)]
        lib.radix_index_select_rows.argtypes = [vp, i32, vp, i32, sz, vp, vp, vp]
        lib.radix_lm_head_workspace_bytes.argtypes = [vp, i32, C.POINTER(sz)]
        lib.radix_lm_head.argtypes = [vp, vp, i32, vp, i32, vp, vp, sz, vp]
        lib.radix_device_status.argtypes = [vp, sz, vp]
        lib.radix_timing_enable.argtypes = [C.c_uint32, C.c_uint32]
        lib.radix_timing_collect.argtypes = [C.POINTER(C.c_float), C.POINTER(i32)]
        lib.radix_debug_gemm_tile.argtypes = [i32, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
        lib.radix_debug_gemm_band.argtypes = [i32, i32, i32]
        lib.radix_status_string.argtypes = [C.c_int]
        lib.radix_status_string.restype = C.c_char_p
        for n in EXPORTS:
            if n != "radix_status_string":
                getattr(lib, n).restype = C.c_int
        _LIB = lib
    return _LIB


def load_library() -> C.CDLL:
    """Load libradixmlp.so (raises if it has not been built)."""
    return _lib()


def _check(code: int, where: str) -> None:
    if code != 0:
        raise RadixError(code, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _i32(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous int32 CUDA tensor")
    return t


class Model:
    """Owns a radix_model handle."""

    def __init__(self, handle: int, cfg: radix_model_config):
        self.handle = handle
        self.cfg = cfg

    @property
    def hilo_layers(self) -> int:
        """Leading layers with (hi, lo) GEMM inputs, as resolved by radix_model_create."""
        n = _lib().radix_model_hilo_layers(self.handle)
        _check(min(n, 0), "radix_model_hilo_layers")
        return n

    @property
    def compute_dtype(self) -> str:
        return {v: k for k, v in _DTYPES.items()}[self.cfg.compute_dtype]

    def close(self) -> None:
        if self.handle:
            _lib().radix_model_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def default_compute_dtype(weight_dtype: str) -> str:
    """Operand type the library is used with unless a caller says otherwise: fp32 weights multiply in fp32,
    bf16 weights as fp16 operands (see radixmlp.h, compute_dtype)."""
    return "f32" if weight_dtype == "f32" else "f16"


def make_config(cfg: Any, compute_dtype: Optional[str] = None, hilo_layers: int = 0,
                lm_head: int = 0, fold_norms: int = 0) -> radix_model_config:
    """cfg: any object with the shape attributes (n_layers, d, n_q_heads, ..., dtype).  The library-side
    settings are arguments of their own: compute_dtype ("f32" / "f16" / "bf16"; None = the default for the
    weight type), hilo_layers and lm_head as in radixmlp.h."""
    compute = compute_dtype or default_compute_dtype(cfg.dtype)
    return radix_model_config(cfg.n_layers, cfg.d, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_int, cfg.vocab,
                              cfg.max_pos, int(cfg.qk_norm), _DTYPES[cfg.dtype], _DTYPES[compute],
                              int(hilo_layers), int(fold_norms), int(lm_head), cfg.eps, cfg.rope_base)


def radix_model_create(cfg: Any, embed: torch.Tensor, gf: torch.Tensor,
                       layers: Sequence[Mapping[str, torch.Tensor]], lm_head: Optional[torch.Tensor] = None,
                       compute_dtype: Optional[str] = None, hilo_layers: int = 0, lm_head_mode: int = 0,
                       fold_norms: int = 0) -> Model:
    """embed/gf/layers/lm_head: CUDA tensors ([out, in] matrices in the config dtype, fp32 gains)."""
    c = make_config(cfg, compute_dtype, hilo_layers, lm_head_mode, fold_norms)
    arr = (radix_layer_weights * len(layers))()
    for l, lw in enumerate(layers):
        for name, _ in radix_layer_weights._fields_:
            t = lw.get(name)
            setattr(arr[l], name, None if t is None else t.data_ptr())
    w = radix_weights(embed.data_ptr(), gf.data_ptr(), arr, _ptr(lm_head))
    out = C.c_void_p()
    _check(_lib().radix_model_create(C.byref(c), C.byref(w), C.byref(out)), "radix_model_create")
    return Model(out.value, c)


def radix_index_workspace_bytes(max_B: int) -> int:
    n = C.c_size_t()
    _check(_lib().radix_index_workspace_bytes(max_B, C.byref(n)), "radix_index_workspace_bytes")
    return n.value


def radix_workspace_bytes(model: Model, max_N: int, max_B: int) -> int:
    n = C.c_size_t()
    _check(_lib().radix_workspace_bytes(model.handle, max_N, max_B, C.byref(n)), "radix_workspace_bytes")
    return n.value


def alloc_workspace(nbytes: int, device: str = "cuda") -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def radix_build_index(tok: torch.Tensor, pos: Optional[torch.Tensor], cu_seqlens: torch.Tensor, ws: torch.Tensor,
                      I_scatter: Optional[torch.Tensor] = None, I_gather: Optional[torch.Tensor] = None,
                      n_compact_dev: Optional[torch.Tensor] = None, sync: bool = True,
                      stream: Optional[torch.cuda.Stream] = None
                      ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, Optional[int]]:
    """Returns (I_scatter[N], I_gather[N] (first N' valid), n_compact_dev[1], N' or None if not sync)."""
    N, B = tok.numel(), cu_seqlens.numel() - 1
    dev = cu_seqlens.device
    if I_scatter is None:
        I_scatter = torch.empty(N, dtype=torch.int32, device=dev)
    if I_gather is None:
        I_gather = torch.empty(N, dtype=torch.int32, device=dev)
    if n_compact_dev is None:
        n_compact_dev = torch.empty(1, dtype=torch.int32, device=dev)
    host = C.c_int32(-1)
    rc = _lib().radix_build_index(_ptr(_i32(tok, "tok")) if N else None, _ptr(pos), _ptr(_i32(cu_seqlens, "cu_seqlens")),
                                  B, N, _ptr(I_scatter), _ptr(I_gather), _ptr(n_compact_dev),
                                  C.byref(host) if sync else None, _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "radix_build_index")
    return I_scatter, I_gather, n_compact_dev, (host.value if sync else None)


def radix_build_index_static(tok: torch.Tensor, pos: Optional[torch.Tensor], cu_seqlens: torch.Tensor,
                             I_scatter: torch.Tensor, I_gather: torch.Tensor, n_compact_dev: torch.Tensor,
                             sync: bool = True, stream: Optional[torch.cuda.Stream] = None) -> Optional[int]:
    """radix_build_index without a workspace (the library's static scratch array); every buffer is the
    caller's, nothing is allocated here or in the library.  Returns N' (None if not sync)."""
    N, B = tok.numel(), cu_seqlens.numel() - 1
    host = C.c_int32(-1)
    rc = _lib().radix_build_index_static(_ptr(_i32(tok, "tok")) if N else None, _ptr(pos),
                                         _ptr(_i32(cu_seqlens, "cu_seqlens")), B, N, _ptr(I_scatter), _ptr(I_gather),
                                         _ptr(n_compact_dev), C.byref(host) if sync else None, _stream(stream))
    _check(rc, "radix_build_index_static")
    return host.value if sync else None


def radix_prefill_forward(model: Model, tok: torch.Tensor, pos: Optional[torch.Tensor], cu_seqlens: torch.Tensor,
                          max_seqlen: int, I_scatter: torch.Tensor, I_gather: torch.Tensor, n_compact: int,
                          ws: torch.Tensor, out: Optional[torch.Tensor] = None, threshold: Optional[float] = None,
                          force_dedup: bool = False, stream: Optional[torch.cuda.Stream] = None,
                          fused_attention: Optional[bool] = None, pad_compact_to: int = 0) -> torch.Tensor:
    """fused_attention: None = RADIX_ATTN_AUTO, False = RADIX_ATTN_THREE_KERNELS, True = RADIX_ATTN_FUSED;
    threshold: None = RADIX_THRESHOLD_AUTO."""
    N, B = tok.numel(), cu_seqlens.numel() - 1
    if out is None:
        out = torch.empty((N, model.cfg.d), dtype=torch.float32, device=cu_seqlens.device)
    mode = 0 if fused_attention is None else (2 if fused_attention else 1)
    opts = radix_fwd_opts(-1.0 if threshold is None else threshold, int(force_dedup), mode, int(pad_compact_to))
    rc = _lib().radix_prefill_forward(model.handle, _ptr(tok), _ptr(pos), _ptr(cu_seqlens), B, N, max_seqlen,
                                      _ptr(I_scatter), _ptr(I_gather), n_compact, C.byref(opts), _ptr(out),
                                      _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "radix_prefill_forward")
    return out


def radix_dedup_decision(config: radix_model_config, B: int, N: int, n_compact: int, threshold: Optional[float] = None,
                         force_dedup: bool = False, fused_attention: Optional[bool] = None) -> bool:
    """Would radix_prefill_forward deduplicate this batch?  Host arithmetic in the library, no GPU involved."""
    mode = 0 if fused_attention is None else (2 if fused_attention else 1)
    opts = radix_fwd_opts(-1.0 if threshold is None else threshold, int(force_dedup), mode, 0)
    out = C.c_int32(-1)
    _check(_lib().radix_dedup_decision(C.byref(config), B, N, n_compact, C.byref(opts), C.byref(out)),
           "radix_dedup_decision")
    return bool(out.value)


def radix_prefill_forward_nodedup(model: Model, tok: torch.Tensor, pos: Optional[torch.Tensor],
                                  cu_seqlens: torch.Tensor, max_seqlen: int, ws: torch.Tensor,
                                  out: Optional[torch.Tensor] = None,
                                  stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    N, B = tok.numel(), cu_seqlens.numel() - 1
    if out is None:
        out = torch.empty((N, model.cfg.d), dtype=torch.float32, device=cu_seqlens.device)
    rc = _lib().radix_prefill_forward_nodedup(model.handle, _ptr(tok), _ptr(pos), _ptr(cu_seqlens), B, N, max_seqlen,
                                              _ptr(out), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "radix_prefill_forward_nodedup")
    return out


def radix_lm_head_workspace_bytes(model: Model, max_rows: int) -> int:
    n = C.c_size_t()
    _check(_lib().radix_lm_head_workspace_bytes(model.handle, max_rows, C.byref(n)), "radix_lm_head_workspace_bytes")
    return n.value


def radix_lm_head(model: Model, hidden: torch.Tensor, rows: Optional[torch.Tensor], ws: torch.Tensor,
                  out: Optional[torch.Tensor] = None, n_rows: Optional[int] = None,
                  stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """logits[n_rows, vocab] (fp32) of hidden[rows] (or of the first n_rows rows when rows is None)."""
    if hidden.dtype != torch.float32 or not hidden.is_contiguous():
        raise TypeError("hidden must be a contiguous fp32 tensor")
    n_src = hidden.shape[0]
    n = rows.numel() if rows is not None else (n_src if n_rows is None else n_rows)
    if out is None:
        out = torch.empty((n, model.cfg.vocab), dtype=torch.float32, device=hidden.device)
    rc = _lib().radix_lm_head(model.handle, _ptr(hidden), n_src, None if rows is None else _ptr(_i32(rows, "rows")), n,
                              _ptr(out), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "radix_lm_head")
    return out


def radix_index_select_rows(src: torch.Tensor, idx: torch.Tensor, out: Optional[torch.Tensor] = None,
                            status: Optional[torch.Tensor] = None,
                            stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """out[r] = src[idx[r]] over the leading axis (contiguous rows)."""
    assert src.is_contiguous()
    n_rows = idx.numel()
    row_bytes = (src.numel() // max(src.shape[0], 1)) * src.element_size()
    if out is None:
        out = torch.empty((n_rows,) + tuple(src.shape[1:]), dtype=src.dtype, device=src.device)
    rc = _lib().radix_index_select_rows(_ptr(src), src.shape[0], _ptr(_i32(idx, "idx")), n_rows, row_bytes, _ptr(out),
                                        _ptr(status), _stream(stream))
    _check(rc, "radix_index_select_rows")
    return out


def radix_device_status(ws: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> int:
    return _lib().radix_device_status(_ptr(ws), ws.numel(), _stream(stream))


def radix_timing_enable(categories: Sequence[str], every_nth: int = 1) -> None:
    mask = 0
    for c in categories:
        mask |= 1 << TIMING_CATEGORIES.index(c)
    _check(_lib().radix_timing_enable(mask, every_nth), "radix_timing_enable")


def radix_timing_collect() -> dict:
    """{category: (total_ms, launches)} since the last collect."""
    n = len(TIMING_CATEGORIES)
    ms = (C.c_float * n)()
    cnt = (C.c_int32 * n)()
    _check(_lib().radix_timing_collect(ms, cnt), "radix_timing_collect")
    return {TIMING_CATEGORIES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}


def radix_status_string(code: int) -> str:
    return _lib().radix_status_string(code).decode()
