"""ctypes binding of libd2ft.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
include/d2ft.h) and does nothing but turn torch tensors into device pointers,
fill the C structs and check the status code.  There is no fallback: if the
shared library is missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libd2ft.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python paper_2504_12471_amd/build.py` "
        "(there is no CPU or PyTorch fallback for the HIP path)")
_lib = C.CDLL(LIB_PATH)

OK, EINVAL, ESHAPE, EDEVICE = 0, 1, 2, 3
OP_FULL, OP_FWD, OP_SKIP = 1, 2, 3
F32, BF16 = 0, 1
FLAG_ACCUM_GRADS, FLAG_NO_MFMA, FLAG_GATE_FFN, FLAG_ONE_STREAM, FLAG_DEFER_JOIN = 1, 2, 4, 8, 16
MAX_HEADS = 64

WEIGHT_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
                 "w1", "b1", "w2", "b2", "lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v")


class BlockDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("tokens", C.c_int32), ("width", C.c_int32), ("heads", C.c_int32),
                ("head_dim", C.c_int32), ("mlp_hidden", C.c_int32), ("lora_rank", C.c_int32),
                ("ln_eps", C.c_float), ("lora_scale", C.c_float), ("dtype", C.c_int32), ("flags", C.c_uint32)]


class _Ptrs(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in WEIGHT_FIELDS]


class D2ftError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {d2ft_status_string(status)} (status {status})")


_lib.d2ft_status_string.restype = C.c_char_p
_lib.d2ft_status_string.argtypes = [C.c_int]
_lib.d2ft_block_saved_bytes.restype = C.c_size_t
_lib.d2ft_block_saved_bytes.argtypes = [C.POINTER(BlockDesc)]
_lib.d2ft_block_scratch_bytes.restype = C.c_size_t
_lib.d2ft_block_scratch_bytes.argtypes = [C.POINTER(BlockDesc)]
_lib.d2ft_compact_heads.restype = C.c_int
_lib.d2ft_compact_heads.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
_lib.d2ft_block_fwd.restype = C.c_int
_lib.d2ft_block_fwd.argtypes = [C.POINTER(BlockDesc), C.POINTER(_Ptrs), C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.c_void_p, C.c_void_p]
_lib.d2ft_block_bwd.restype = C.c_int
_lib.d2ft_block_bwd.argtypes = [C.POINTER(BlockDesc), C.POINTER(_Ptrs), C.c_void_p, C.c_void_p, C.c_void_p,
                                C.c_void_p, C.POINTER(_Ptrs), C.c_void_p, C.c_void_p, C.c_void_p]
_lib.d2ft_block_saved_bytes_mb.restype = C.c_size_t
_lib.d2ft_block_saved_bytes_mb.argtypes = [C.POINTER(BlockDesc), C.c_int32, C.c_void_p]
_lib.d2ft_block_fwd_mb.restype = C.c_int
_lib.d2ft_block_fwd_mb.argtypes = [C.POINTER(BlockDesc), C.POINTER(_Ptrs), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.d2ft_block_bwd_mb.restype = C.c_int
_lib.d2ft_block_bwd_mb.argtypes = [C.POINTER(BlockDesc), C.POINTER(_Ptrs), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.POINTER(_Ptrs), C.c_void_p, C.c_void_p, C.c_void_p]
_lib.d2ft_knapsack_workspace_bytes.restype = C.c_size_t
_lib.d2ft_knapsack_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
_lib.d2ft_select_knapsack.restype = C.c_int
_lib.d2ft_select_knapsack.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.d2ft_knapsack_static_bytes.restype = C.c_size_t
_lib.d2ft_knapsack_static_bytes.argtypes = []
_lib.d2ft_select_knapsack_static.restype = C.c_int
_lib.d2ft_select_knapsack_static.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]


_lib.d2ft_scores_workspace_bytes.restype = C.c_size_t
_lib.d2ft_scores_workspace_bytes.argtypes = [C.POINTER(BlockDesc)]
_lib.d2ft_subnet_scores.restype = C.c_int
_lib.d2ft_subnet_scores.argtypes = [C.POINTER(BlockDesc), C.POINTER(_Ptrs), C.c_int32, C.c_void_p, C.c_void_p,
                                    C.c_size_t, C.c_void_p]
SCORE_FISHER, SCORE_MAGNITUDE = 0, 1


class SgdParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float)]


_lib.d2ft_sgd_step.restype = C.c_int
_lib.d2ft_sgd_step.argtypes = [C.POINTER(BlockDesc), C.POINTER(_Ptrs), C.POINTER(_Ptrs), C.POINTER(_Ptrs),
                               C.POINTER(_Ptrs), C.c_void_p, C.POINTER(SgdParams), C.c_void_p]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 96), ("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


_lib.d2ft_timing_enable.restype = C.c_int
_lib.d2ft_timing_enable.argtypes = [C.c_int32]
_lib.d2ft_timing_read.restype = C.c_int32
_lib.d2ft_timing_read.argtypes = [C.POINTER(KernelTime), C.c_int32]


_lib.d2ft_join.restype = C.c_int
_lib.d2ft_join.argtypes = [C.c_void_p]


def d2ft_join(stream: Optional["torch.cuda.Stream"] = None) -> None:
    _check(_lib.d2ft_join(_stream_ptr(stream)), "d2ft_join")


def d2ft_timing_enable(on: bool) -> None:
    _check(_lib.d2ft_timing_enable(1 if on else 0), "d2ft_timing_enable")


def d2ft_timing_read(max_entries: int = 64):
    """List of dicts (name, launches, ms, flops, bytes), one per kernel class."""
    buf = (KernelTime * max_entries)()
    n = _lib.d2ft_timing_read(buf, max_entries)
    if n < 0:
        raise D2ftError(EDEVICE, "d2ft_timing_read")
    return [dict(name=buf[i].name.decode(), launches=int(buf[i].launches), ms=float(buf[i].ms),
                 flops=float(buf[i].flops), bytes=float(buf[i].bytes)) for i in range(n)]


def d2ft_status_string(status: int) -> str:
    return _lib.d2ft_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise D2ftError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to libd2ft must be contiguous")
    return t.data_ptr()


def _ptr_struct(tensors: Dict[str, Optional[torch.Tensor]]) -> _Ptrs:
    s = _Ptrs()
    for name in WEIGHT_FIELDS:
        setattr(s, name, _ptr(tensors.get(name)))
    return s


def _ops_array(ops: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(ops, dtype=np.uint8))


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def d2ft_block_saved_bytes(desc: BlockDesc) -> int:
    return int(_lib.d2ft_block_saved_bytes(C.byref(desc)))


def d2ft_block_scratch_bytes(desc: BlockDesc) -> int:
    return int(_lib.d2ft_block_scratch_bytes(C.byref(desc)))


def d2ft_compact_heads(ops: Sequence[int]):
    """Returns (live list, n_full, n_live)."""
    a = _ops_array(ops)
    live = np.zeros(max(1, a.size), dtype=np.int32)
    nf, nl = C.c_int32(0), C.c_int32(0)
    st = _lib.d2ft_compact_heads(a.ctypes.data, int(a.size), live.ctypes.data, C.byref(nf), C.byref(nl))
    _check(st, "d2ft_compact_heads")
    return live[:nl.value].tolist(), nf.value, nl.value


def d2ft_block_fwd(desc: BlockDesc, weights: Dict[str, Optional[torch.Tensor]], ops: Sequence[int],
                   x: torch.Tensor, y: torch.Tensor, saved: torch.Tensor, scratch: torch.Tensor,
                   stream: Optional[torch.cuda.Stream] = None) -> None:
    a = _ops_array(ops)
    w = _ptr_struct(weights)
    st = _lib.d2ft_block_fwd(C.byref(desc), C.byref(w), a.ctypes.data, _ptr(x), _ptr(y), _ptr(saved), _ptr(scratch),
                             _stream_ptr(stream))
    _check(st, "d2ft_block_fwd")


def d2ft_block_bwd(desc: BlockDesc, weights: Dict[str, Optional[torch.Tensor]], ops: Sequence[int],
                   x: torch.Tensor, dy: torch.Tensor, dx: torch.Tensor, grads: Dict[str, Optional[torch.Tensor]],
                   saved: torch.Tensor, scratch: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    a = _ops_array(ops)
    w = _ptr_struct(weights)
    g = _ptr_struct(grads)
    st = _lib.d2ft_block_bwd(C.byref(desc), C.byref(w), a.ctypes.data, _ptr(x), _ptr(dy), _ptr(dx), C.byref(g),
                             _ptr(saved), _ptr(scratch), _stream_ptr(stream))
    _check(st, "d2ft_block_bwd")


def _mb_arrays(desc: BlockDesc, mb_images: Sequence[int], ops) -> tuple:
    mb = np.ascontiguousarray(np.asarray(mb_images, dtype=np.int32))
    a = np.ascontiguousarray(np.asarray(ops, dtype=np.uint8))
    if a.shape != (mb.shape[0], desc.heads):
        raise ValueError("ops must be [n_micro, heads]")
    return mb, a


def d2ft_block_saved_bytes_mb(desc: BlockDesc, mb_images: Sequence[int]) -> int:
    mb = np.ascontiguousarray(np.asarray(mb_images, dtype=np.int32))
    return int(_lib.d2ft_block_saved_bytes_mb(C.byref(desc), mb.shape[0], mb.ctypes.data))


def d2ft_block_fwd_mb(desc: BlockDesc, weights: Dict[str, Optional[torch.Tensor]], mb_images: Sequence[int], ops,
                      x: torch.Tensor, y: torch.Tensor, saved: torch.Tensor, scratch: torch.Tensor,
                      stream: Optional[torch.cuda.Stream] = None) -> None:
    mb, a = _mb_arrays(desc, mb_images, ops)
    w = _ptr_struct(weights)
    st = _lib.d2ft_block_fwd_mb(C.byref(desc), C.byref(w), mb.shape[0], mb.ctypes.data, a.ctypes.data, _ptr(x), _ptr(y),
                                _ptr(saved), _ptr(scratch), _stream_ptr(stream))
    _check(st, "d2ft_block_fwd_mb")


def d2ft_block_bwd_mb(desc: BlockDesc, weights: Dict[str, Optional[torch.Tensor]], mb_images: Sequence[int], ops,
                      x: torch.Tensor, dy: torch.Tensor, dx: torch.Tensor, grads: Dict[str, Optional[torch.Tensor]],
                      saved: torch.Tensor, scratch: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    mb, a = _mb_arrays(desc, mb_images, ops)
    w = _ptr_struct(weights)
    g = _ptr_struct(grads)
    st = _lib.d2ft_block_bwd_mb(C.byref(desc), C.byref(w), mb.shape[0], mb.ctypes.data, a.ctypes.data, _ptr(x), _ptr(dy),
                                _ptr(dx), C.byref(g), _ptr(saved), _ptr(scratch), _stream_ptr(stream))
    _check(st, "d2ft_block_bwd_mb")


def d2ft_knapsack_workspace_bytes(n_knapsacks: int, n_items: int, cap_full, cap_fwd) -> int:
    cf = np.ascontiguousarray(cap_full, dtype=np.int32)
    co = np.ascontiguousarray(cap_fwd, dtype=np.int32)
    return int(_lib.d2ft_knapsack_workspace_bytes(n_knapsacks, n_items, cf.ctypes.data, co.ctypes.data))


def d2ft_select_knapsack(score_full, score_fwd, cost_fwd, cost_bwd, cap_full, cap_fwd,
                         workspace: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> np.ndarray:
    """Returns the uint8 [n_knapsacks, n_items] table of op codes (host array)."""
    sf = np.ascontiguousarray(score_full, dtype=np.float64)
    so = np.ascontiguousarray(score_fwd, dtype=np.float64)
    if sf.ndim != 2 or sf.shape != so.shape:
        raise ValueError("scores must be two [n_knapsacks, n_items] arrays")
    K, n = sf.shape
    arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in (cost_fwd, cost_bwd, cap_full, cap_fwd)]
    if any(a.shape != (K,) for a in arrs):
        raise ValueError("costs and capacities must have one entry per knapsack")
    cf, cb, capf, capo = arrs
    need = int(_lib.d2ft_knapsack_workspace_bytes(K, n, capf.ctypes.data, capo.ctypes.data))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    out = np.zeros((K, n), dtype=np.uint8)
    st = _lib.d2ft_select_knapsack(K, n, sf.ctypes.data, so.ctypes.data, cf.ctypes.data, cb.ctypes.data,
                                   capf.ctypes.data, capo.ctypes.data, out.ctypes.data, _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    _check(st, "d2ft_select_knapsack")
    return out


def d2ft_knapsack_static_bytes() -> int:
    return int(_lib.d2ft_knapsack_static_bytes())


def d2ft_select_knapsack_static(score_full, score_fwd, cost_fwd, cost_bwd, cap_full, cap_fwd,
                                stream: Optional[torch.cuda.Stream] = None) -> np.ndarray:
    """d2ft_select_knapsack on the library's own fixed device array; nothing is allocated on the device."""
    sf = np.ascontiguousarray(score_full, dtype=np.float64)
    so = np.ascontiguousarray(score_fwd, dtype=np.float64)
    if sf.ndim != 2 or sf.shape != so.shape:
        raise ValueError("scores must be two [n_knapsacks, n_items] arrays")
    K, n = sf.shape
    arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in (cost_fwd, cost_bwd, cap_full, cap_fwd)]
    if any(a.shape != (K,) for a in arrs):
        raise ValueError("costs and capacities must have one entry per knapsack")
    cf, cb, capf, capo = arrs
    out = np.zeros((K, n), dtype=np.uint8)
    st = _lib.d2ft_select_knapsack_static(K, n, sf.ctypes.data, so.ctypes.data, cf.ctypes.data, cb.ctypes.data,
                                          capf.ctypes.data, capo.ctypes.data, out.ctypes.data, _stream_ptr(stream))
    _check(st, "d2ft_select_knapsack_static")
    return out


def d2ft_subnet_scores(desc: BlockDesc, tensors: Dict[str, Optional[torch.Tensor]], kind: int,
                       workspace: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> np.ndarray:
    """Per-head contribution scores (host float64 [heads]) of tensors laid out like the block's weights."""
    need = int(_lib.d2ft_scores_workspace_bytes(C.byref(desc)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    out = np.zeros(desc.heads, dtype=np.float64)
    ptrs = _ptr_struct(tensors)
    st = _lib.d2ft_subnet_scores(C.byref(desc), C.byref(ptrs), int(kind), out.ctypes.data, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    _check(st, "d2ft_subnet_scores")
    return out


def d2ft_sgd_step(desc: BlockDesc, weights: Dict[str, Optional[torch.Tensor]], grads: Dict[str, Optional[torch.Tensor]],
                  momentum: Dict[str, Optional[torch.Tensor]], master: Optional[Dict[str, Optional[torch.Tensor]]],
                  ops: Sequence[int], lr: float, mu: float, weight_decay: float = 0.0,
                  stream: Optional[torch.cuda.Stream] = None) -> None:
    """SGD with momentum on the slices of the p_f heads (and on the shared tensors), in place."""
    a = _ops_array(ops)
    w, g, v = _ptr_struct(weights), _ptr_struct(grads), _ptr_struct(momentum)
    m = None if master is None else _ptr_struct(master)
    prm = SgdParams(lr, mu, weight_decay)
    st = _lib.d2ft_sgd_step(C.byref(desc), C.byref(w), C.byref(g), C.byref(v), None if m is None else C.byref(m),
                            a.ctypes.data, C.byref(prm), _stream_ptr(stream))
    _check(st, "d2ft_sgd_step")


class EmbedDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("channels", C.c_int32), ("height", C.c_int32), ("width_px", C.c_int32),
                ("patch", C.c_int32), ("width", C.c_int32), ("dtype", C.c_int32), ("flags", C.c_uint32)]


class HeadDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("tokens", C.c_int32), ("width", C.c_int32), ("classes", C.c_int32),
                ("ln_eps", C.c_float), ("dtype", C.c_int32), ("flags", C.c_uint32)]


_lib.d2ft_embed_saved_bytes.restype = C.c_size_t
_lib.d2ft_embed_saved_bytes.argtypes = [C.POINTER(EmbedDesc)]
_lib.d2ft_embed_scratch_bytes.restype = C.c_size_t
_lib.d2ft_embed_scratch_bytes.argtypes = [C.POINTER(EmbedDesc)]
_lib.d2ft_patch_embed_fwd.restype = C.c_int
_lib.d2ft_patch_embed_fwd.argtypes = [C.POINTER(EmbedDesc)] + [C.c_void_p] * 9
_lib.d2ft_patch_embed_bwd.restype = C.c_int
_lib.d2ft_patch_embed_bwd.argtypes = [C.POINTER(EmbedDesc)] + [C.c_void_p] * 8
_lib.d2ft_head_scratch_bytes.restype = C.c_size_t
_lib.d2ft_head_scratch_bytes.argtypes = [C.POINTER(HeadDesc)]
_lib.d2ft_classifier_fwd_bwd.restype = C.c_int
_lib.d2ft_classifier_fwd_bwd.argtypes = [C.POINTER(HeadDesc)] + [C.c_void_p] * 14


def d2ft_embed_saved_bytes(desc: EmbedDesc) -> int:
    return int(_lib.d2ft_embed_saved_bytes(C.byref(desc)))


def d2ft_embed_scratch_bytes(desc: EmbedDesc) -> int:
    return int(_lib.d2ft_embed_scratch_bytes(C.byref(desc)))


def d2ft_patch_embed_fwd(desc: EmbedDesc, images, w_pe, b_pe, cls, pos, tokens, saved, scratch, stream=None) -> None:
    st = _lib.d2ft_patch_embed_fwd(C.byref(desc), _ptr(images), _ptr(w_pe), _ptr(b_pe), _ptr(cls), _ptr(pos), _ptr(tokens),
                                   _ptr(saved), _ptr(scratch), _stream_ptr(stream))
    _check(st, "d2ft_patch_embed_fwd")


def d2ft_patch_embed_bwd(desc: EmbedDesc, dtokens, g_w_pe, g_b_pe, g_cls, g_pos, saved, scratch, stream=None) -> None:
    st = _lib.d2ft_patch_embed_bwd(C.byref(desc), _ptr(dtokens), _ptr(g_w_pe), _ptr(g_b_pe), _ptr(g_cls), _ptr(g_pos),
                                   _ptr(saved), _ptr(scratch), _stream_ptr(stream))
    _check(st, "d2ft_patch_embed_bwd")


def d2ft_head_scratch_bytes(desc: HeadDesc) -> int:
    return int(_lib.d2ft_head_scratch_bytes(C.byref(desc)))


def d2ft_classifier_fwd_bwd(desc: HeadDesc, tokens, ln_g, ln_b, w_c, b_c, labels, dtokens, g_ln_g, g_ln_b, g_w_c, g_b_c,
                            scratch, stream=None) -> float:
    """Returns the mean cross-entropy loss; dtokens and the non-None gradient tensors are written."""
    lab = np.ascontiguousarray(np.asarray(labels, dtype=np.int32))
    if lab.shape != (desc.batch,):
        raise ValueError("one label per image")
    loss = C.c_float(0.0)
    st = _lib.d2ft_classifier_fwd_bwd(C.byref(desc), _ptr(tokens), _ptr(ln_g), _ptr(ln_b), _ptr(w_c), _ptr(b_c),
                                      lab.ctypes.data, C.addressof(loss), _ptr(dtokens), _ptr(g_ln_g), _ptr(g_ln_b),
                                      _ptr(g_w_c), _ptr(g_b_c), _ptr(scratch), _stream_ptr(stream))
    _check(st, "d2ft_classifier_fwd_bwd")
    return float(loss.value)


def exported_symbols():
    """Names this binding resolves in the shared library (used by the load test)."""
    return ["d2ft_status_string", "d2ft_block_saved_bytes", "d2ft_block_scratch_bytes", "d2ft_compact_heads",
            "d2ft_block_fwd", "d2ft_block_bwd", "d2ft_block_saved_bytes_mb", "d2ft_block_fwd_mb", "d2ft_block_bwd_mb",
            "d2ft_knapsack_workspace_bytes", "d2ft_select_knapsack", "d2ft_knapsack_static_bytes",
            "d2ft_select_knapsack_static",
            "d2ft_scores_workspace_bytes", "d2ft_subnet_scores", "d2ft_sgd_step", "d2ft_embed_saved_bytes",
            "d2ft_embed_scratch_bytes", "d2ft_patch_embed_fwd", "d2ft_patch_embed_bwd", "d2ft_head_scratch_bytes",
            "d2ft_classifier_fwd_bwd", "d2ft_timing_enable", "d2ft_timing_read", "d2ft_join"]
