"""Python binding of libems: the ragged verification step of batched speculative
decoding (EMS-SD, arXiv 2405.07542) on one MI355X.

Argument marshalling only: every step runs in the HIP kernels behind the C ABI
declared in ``include/ems.h``.  PyTorch supplies device memory (``data_ptr()``)
and the current stream; there is no CPU fallback -- if ``libems.so`` has not
been built (``python -m paper_2405_07542_amd.build``) importing the entry
points raises.
"""
from __future__ import annotations

import ctypes
import os
import threading
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libems.so")

EMS_OK, EMS_ERR_INVALID_ARG, EMS_ERR_UNSUPPORTED, EMS_ERR_WORKSPACE, EMS_ERR_HIP = range(5)
EMS_F16, EMS_BF16, EMS_F32 = 0, 1, 2
EMS_MAX_QUERY_ROWS = 64
EMS_ROWS_PER_GROUP = 16
_DT = {torch.float16: EMS_F16, torch.bfloat16: EMS_BF16, torch.float32: EMS_F32}


class EmsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("ems status %d: %s" % (status, message))
        self.status = status


class KvCacheStruct(ctypes.Structure):
    """Mirror of ``ems_kv_cache``."""
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("row_stride", ctypes.c_int64), ("head_stride", ctypes.c_int64),
                ("rows", ctypes.c_int64)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it was not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libems.so is missing: build it with "
                              "`python -m paper_2405_07542_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        L.ems_last_error_string.restype = ctypes.c_char_p
        L.ems_version.restype = ctypes.c_char_p
        L.ems_device_memory_figures.restype = i32
        L.ems_device_memory_figures.argtypes = [ctypes.POINTER(ctypes.c_int)] * 2
        L.ems_attention_workspace_bytes.restype = sz
        L.ems_attention_workspace_bytes.argtypes = [i32] * 5
        L.ems_workspace_bytes.restype = sz
        L.ems_workspace_bytes.argtypes = [i32] * 5
        L.ems_accept_workspace_bytes.restype = sz
        L.ems_accept_workspace_bytes.argtypes = [i32, i32]
        L.ems_verify_attention.restype = i32
        L.ems_verify_attention.argtypes = [vp, vp, vp, ctypes.POINTER(KvCacheStruct), vp, vp, vp,
                                           vp, i32, i32, i32, i32, i32, i32, i32,
                                           ctypes.c_float, i32, vp, sz, vp]
        L.ems_verify_attention_write_through.restype = i32
        L.ems_verify_attention_write_through.argtypes = L.ems_verify_attention.argtypes
        L.ems_verify_attention_noalloc.restype = i32
        L.ems_verify_attention_noalloc.argtypes = [vp, vp, vp, ctypes.POINTER(KvCacheStruct), vp, vp, vp,
                                                   vp, i32, i32, i32, i32, i32, i32, i32,
                                                   ctypes.c_float, i32, vp]
        L.ems_kv_advance.restype = i32
        L.ems_kv_advance.argtypes = [vp, vp, vp, i32, vp]
        L.ems_tree_verify_attention.restype = i32
        L.ems_tree_verify_attention.argtypes = [vp, vp, vp, ctypes.POINTER(KvCacheStruct), vp, vp, vp, vp,
                                                vp, i32, i32, i32, i32, i32, i32, i32,
                                                ctypes.c_float, i32, vp, sz, vp]
        L.ems_pack_tokens.restype = i32
        L.ems_pack_tokens.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.ems_validate_tree.restype = i32
        L.ems_validate_tree.argtypes = [vp, vp, i32, i32, vp]
        L.ems_tree_accept.restype = i32
        L.ems_tree_accept.argtypes = [vp, i32, i32, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.ems_kv_append_rows.restype = i32
        L.ems_kv_append_rows.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp),
                                         ctypes.POINTER(KvCacheStruct), i32, vp, vp, vp, vp, vp,
                                         i32, i32, i32, i32, i32, vp]
        L.ems_greedy_accept.restype = i32
        L.ems_greedy_accept.argtypes = [vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
        L.ems_kv_append.restype = i32
        L.ems_kv_append.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp),
                                    ctypes.POINTER(KvCacheStruct), i32, vp, vp, vp, vp, vp,
                                    i32, i32, i32, i32, i32, vp]
        L.ems_greedy_accept_append.restype = i32
        L.ems_greedy_accept_append.argtypes = [vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz,
                                               ctypes.POINTER(vp), ctypes.POINTER(vp),
                                               ctypes.POINTER(KvCacheStruct), i32, vp, vp, vp,
                                               i32, i32, i32, vp]
        L.ems_validate_inputs.restype = i32
        L.ems_validate_inputs.argtypes = [vp, vp, vp, i32, i32, i32, i32, i64, vp]
        L.ems_padded_verify_attention.restype = i32
        L.ems_padded_verify_attention.argtypes = [vp, vp, vp, ctypes.POINTER(KvCacheStruct), i64, vp,
                                                  vp, vp, i32, i32, i32, i32, i32, i32,
                                                  ctypes.c_float, i32, vp, sz, vp]
        L.ems_padded_kv_append.restype = i32
        L.ems_padded_kv_append.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp),
                                           ctypes.POINTER(KvCacheStruct), i32, i64, vp, vp,
                                           i32, i32, i32, i32, i32, i32, i32, vp]
        L.ems_profile_enable.restype = i32
        L.ems_profile_enable.argtypes = [i32]
        L.ems_stream_read_probe.restype = i32
        L.ems_stream_read_probe.argtypes = [vp, ctypes.c_size_t, vp, vp]
        L.ems_set_attention_variant.restype = i32
        L.ems_set_attention_variant.argtypes = [i32]
        L.ems_get_attention_variant.restype = i32
        L.ems_get_attention_variant.argtypes = []
        L.ems_profile_read.restype = i32
        L.ems_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        L.ems_profile_read_calls.restype = i32
        L.ems_profile_read_calls.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(i32)]
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


# The C layer sees raw addresses: it cannot tell an int64 index array from an int32 one, a strided
# view from a dense tensor, or host memory from device memory, and a kernel that reads such an
# argument reads out of bounds.  So the binding checks what only it can see, before anything is
# launched: element type, density, residence and element count of every tensor it passes on.
def _need(name: str, t: Optional[torch.Tensor], dtype, numel: Optional[int] = None, shape=None,
          optional: bool = False, at_least: Optional[int] = None) -> None:
    if t is None:
        if optional:
            return
        _refuse(TypeError, "%s must be a tensor, not None" % name)
    if not isinstance(t, torch.Tensor):
        _refuse(TypeError, "%s must be a torch.Tensor, got %s" % (name, type(t).__name__))
    dtypes = dtype if isinstance(dtype, (tuple, list)) else (dtype,)
    if t.dtype not in dtypes:
        _refuse(TypeError, "%s must have dtype %s, got %s" % (name, " or ".join(str(d) for d in dtypes), t.dtype))
    if not t.is_contiguous():
        _refuse(ValueError, "%s must be contiguous (dense, row-major); got strides %s for shape %s"
                         % (name, tuple(t.stride()), tuple(t.shape)))
    if shape is not None and tuple(t.shape) != tuple(shape):
        _refuse(ValueError, "%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if numel is not None and t.numel() != numel:
        _refuse(ValueError, "%s must hold %d elements, got %d" % (name, numel, t.numel()))
    if at_least is not None and t.numel() < at_least:
        _refuse(ValueError, "%s must hold at least %d elements, got %d" % (name, at_least, t.numel()))
    _seen.pending.append((name, t))


def _refuse(kind, message: str):
    _seen.pending = []          # a refused call leaves nothing behind for the next one
    raise kind(message)


class _Seen(threading.local):
    def __init__(self):
        self.pending = []


_seen = _Seen()


def _check(status: int) -> None:
    """Turns a non-OK status of a C call into an exception carrying the library's message."""
    if status != EMS_OK:
        raise EmsError(status, lib().ems_last_error_string().decode())


def _resident() -> None:
    """Every tensor checked by _need since the last call must live in GPU memory (checked after all
    type and shape checks, so that those are reported first and can be tested without a GPU)."""
    pending, _seen.pending = _seen.pending, []
    for name, t in pending:
        if not t.is_cuda:
            raise ValueError("%s must live in GPU memory, got a tensor on %s" % (name, t.device))


_I32 = torch.int32
_F16S = (torch.float16, torch.bfloat16)


def _need_packed(q, k_new, v_new, out, names=("q", "k_new", "v_new", "out")) -> None:
    """q, k_new, v_new: dense [T,H,D] of one 16-bit type; out: the same shape in that type or fp32."""
    if not isinstance(q, torch.Tensor) or q.dim() != 3:
        _refuse(ValueError, "%s must be a [T, H, D] tensor" % names[0])
    _need(names[0], q, _F16S)
    _need(names[1], k_new, q.dtype, shape=q.shape)
    _need(names[2], v_new, q.dtype, shape=q.shape)
    _need(names[3], out, (q.dtype, torch.float32), shape=q.shape)


def _need_layers(k_new_layers, v_new_layers, n: int) -> None:
    if len(k_new_layers) != n or len(v_new_layers) != n or n < 1:
        _refuse(ValueError, "need one k_new and one v_new tensor per cache (%d caches)" % n)
    first = k_new_layers[0]
    if not isinstance(first, torch.Tensor) or first.dim() != 3:
        _refuse(ValueError, "k_new_layers[0] must be a [T, H, D] tensor")
    _need("k_new_layers[0]", first, _F16S)
    for l in range(n):
        _need("k_new_layers[%d]" % l, k_new_layers[l], first.dtype, shape=first.shape)
        _need("v_new_layers[%d]" % l, v_new_layers[l], first.dtype, shape=first.shape)


def _need_accept(logits, target_ids, input_ids, cu_seqlens, accepted, accepted_cu, out_tokens, workspace,
                 parent=None, accepted_rows=None, tree: bool = False) -> None:
    B, T = accepted.numel() if isinstance(accepted, torch.Tensor) else 0, \
        input_ids.numel() if isinstance(input_ids, torch.Tensor) else 0
    _need("input_ids", input_ids, _I32)
    _need("accepted", accepted, _I32)
    _need("cu_seqlens", cu_seqlens, _I32, numel=B + 1)
    _need("accepted_cu", accepted_cu, _I32, numel=B + 1)
    _need("target_ids", target_ids, _I32, at_least=T)
    _need("out_tokens", out_tokens, _I32, at_least=T, optional=True)
    if logits is not None:
        if not isinstance(logits, torch.Tensor) or logits.dim() != 2 or logits.shape[0] != T:
            _refuse(ValueError, "logits must be a [T, V] tensor with T = %d rows" % T)
        _need("logits", logits, _F16S + (torch.float32,))
        _need("workspace", workspace, torch.uint8, optional=T == 0)
    if tree:
        _need("parent", parent, _I32, numel=T)
        _need("accepted_rows", accepted_rows, _I32, at_least=T, optional=True)


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def kv_cache(k: torch.Tensor, v: torch.Tensor, row_stride: int, head_stride: int,
             rows: int) -> KvCacheStruct:
    """The strided view of one layer's K and V arenas (dense 16-bit GPU tensors of one type)."""
    _need("k arena", k, _F16S)
    _need("v arena", v, k.dtype, numel=k.numel())
    _resident()
    return KvCacheStruct(k.data_ptr(), v.data_ptr(), int(row_stride), int(head_stride), int(rows))


def ems_attention_workspace_bytes(B: int, T: int, H: int, D: int, max_kv_len: int) -> int:
    return int(lib().ems_attention_workspace_bytes(B, T, H, D, max_kv_len))


def ems_workspace_bytes(B: int, T: int, H: int, D: int, max_kv_len: int) -> int:
    return int(lib().ems_workspace_bytes(B, T, H, D, max_kv_len))


def ems_accept_workspace_bytes(T: int, V: int) -> int:
    return int(lib().ems_accept_workspace_bytes(T, V))


def ems_verify_attention(q, k_new, v_new, cache: KvCacheStruct, cu_seqlens, kv_start, kv_len,
                         out, *, max_k: int, max_kv_len: int, scale: float,
                         workspace: torch.Tensor, stream=None, write_through: bool = False) -> None:
    """out[T,H,D] <- packed multi-token attention over the per-sample caches.
    write_through=True calls ems_verify_attention_write_through (new rows' K/V also stored)."""
    _need_packed(q, k_new, v_new, out)
    T, H, D = q.shape
    _need("kv_start", kv_start, _I32)
    B = kv_start.numel()
    _need("kv_len", kv_len, _I32, numel=B)
    _need("cu_seqlens", cu_seqlens, _I32, numel=B + 1)
    _need("workspace", workspace, torch.uint8)
    fn = lib().ems_verify_attention_write_through if write_through else lib().ems_verify_attention
    _resident()
    _check(fn(
        _ptr(q), _ptr(k_new), _ptr(v_new), ctypes.byref(cache), _ptr(cu_seqlens), _ptr(kv_start),
        _ptr(kv_len), _ptr(out), _DT[out.dtype], B, T, H, D, int(max_k), int(max_kv_len),
        float(scale), _DT[q.dtype], _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)))


def ems_verify_attention_noalloc(q, k_new, v_new, cache: KvCacheStruct, cu_seqlens, kv_start, kv_len,
                                 out, *, max_k: int, max_kv_len: int, scale: float, stream=None) -> None:
    """ems_verify_attention without a workspace: the partials go to the library's own device buffer."""
    _need_packed(q, k_new, v_new, out)
    T, H, D = q.shape
    _need("kv_start", kv_start, _I32)
    B = kv_start.numel()
    _need("kv_len", kv_len, _I32, numel=B)
    _need("cu_seqlens", cu_seqlens, _I32, numel=B + 1)
    _resident()
    _check(lib().ems_verify_attention_noalloc(
        _ptr(q), _ptr(k_new), _ptr(v_new), ctypes.byref(cache), _ptr(cu_seqlens), _ptr(kv_start),
        _ptr(kv_len), _ptr(out), _DT[out.dtype], B, T, H, D, int(max_k), int(max_kv_len),
        float(scale), _DT[q.dtype], _stream(stream)))


def ems_greedy_accept(logits: Optional[torch.Tensor], target_ids, input_ids, cu_seqlens,
                      accepted, accepted_cu, out_tokens: Optional[torch.Tensor], *,
                      workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    _need_accept(logits, target_ids, input_ids, cu_seqlens, accepted, accepted_cu, out_tokens, workspace)
    B = accepted.numel()
    T = input_ids.numel()
    V = logits.shape[1] if logits is not None else 0
    dt = _DT[logits.dtype] if logits is not None else EMS_F16
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _resident()
    _check(lib().ems_greedy_accept(
        _ptr(logits), dt, V, _ptr(target_ids), _ptr(input_ids), _ptr(cu_seqlens), B, T,
        _ptr(accepted), _ptr(accepted_cu), _ptr(out_tokens), _ptr(workspace), ws_bytes,
        _stream(stream)))


def ems_kv_append(k_new_layers: Sequence[torch.Tensor], v_new_layers: Sequence[torch.Tensor],
                  caches: Sequence[KvCacheStruct], cu_seqlens, accepted, kv_start, kv_len,
                  kv_len_out: Optional[torch.Tensor], stream=None) -> None:
    n = len(caches)
    _need_layers(k_new_layers, v_new_layers, n)
    T, H, D = k_new_layers[0].shape
    _need("kv_start", kv_start, _I32)
    B = kv_start.numel()
    _need("kv_len", kv_len, _I32, numel=B)
    _need("kv_len_out", kv_len_out, _I32, numel=B, optional=True)
    _need("cu_seqlens", cu_seqlens, _I32, numel=B + 1)
    _need("accepted", accepted, _I32, numel=B)
    karr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in k_new_layers])
    varr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in v_new_layers])
    carr = (KvCacheStruct * n)(*caches)
    _resident()
    _check(lib().ems_kv_append(karr, varr, carr, n, _ptr(cu_seqlens), _ptr(accepted),
                               _ptr(kv_start), _ptr(kv_len), _ptr(kv_len_out), B, T, H, D,
                               _DT[k_new_layers[0].dtype], _stream(stream)))


def ems_greedy_accept_append(logits: Optional[torch.Tensor], target_ids, input_ids, cu_seqlens,
                             accepted, accepted_cu, out_tokens: Optional[torch.Tensor],
                             k_new_layers: Sequence[torch.Tensor], v_new_layers: Sequence[torch.Tensor],
                             caches: Sequence[KvCacheStruct], kv_start, kv_len,
                             kv_len_out: Optional[torch.Tensor], *,
                             workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """ems_greedy_accept and ems_kv_append of the counts it found, as one call."""
    _need_accept(logits, target_ids, input_ids, cu_seqlens, accepted, accepted_cu, out_tokens, workspace)
    B = accepted.numel()
    T = input_ids.numel()
    V = logits.shape[1] if logits is not None else 0
    dt = _DT[logits.dtype] if logits is not None else EMS_F16
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    n = len(caches)
    _need_layers(k_new_layers, v_new_layers, n)
    Tk, H, D = k_new_layers[0].shape
    if Tk != T:
        _refuse(ValueError, "k_new_layers hold %d rows, input_ids %d" % (Tk, T))
    _need("kv_start", kv_start, _I32, numel=B)
    _need("kv_len", kv_len, _I32, numel=B)
    _need("kv_len_out", kv_len_out, _I32, numel=B, optional=True)
    karr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in k_new_layers])
    varr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in v_new_layers])
    carr = (KvCacheStruct * n)(*caches)
    _resident()
    _check(lib().ems_greedy_accept_append(
        _ptr(logits), dt, V, _ptr(target_ids), _ptr(input_ids), _ptr(cu_seqlens), B, T,
        _ptr(accepted), _ptr(accepted_cu), _ptr(out_tokens), _ptr(workspace), ws_bytes,
        karr, varr, carr, n, _ptr(kv_start), _ptr(kv_len), _ptr(kv_len_out), H, D,
        _DT[k_new_layers[0].dtype], _stream(stream)))


def ems_tree_verify_attention(q, k_new, v_new, cache: KvCacheStruct, cu_seqlens, parent, kv_start,
                              kv_len, out, *, max_k: int, max_kv_len: int, scale: float,
                              workspace: torch.Tensor, stream=None) -> None:
    """As ems_verify_attention, with a per-sample token tree: parent[T] int32."""
    _need_packed(q, k_new, v_new, out)
    T, H, D = q.shape
    _need("kv_start", kv_start, _I32)
    B = kv_start.numel()
    _need("kv_len", kv_len, _I32, numel=B)
    _need("cu_seqlens", cu_seqlens, _I32, numel=B + 1)
    _need("parent", parent, _I32, numel=T)
    _need("workspace", workspace, torch.uint8)
    _resident()
    _check(lib().ems_tree_verify_attention(
        _ptr(q), _ptr(k_new), _ptr(v_new), ctypes.byref(cache), _ptr(cu_seqlens), _ptr(parent),
        _ptr(kv_start), _ptr(kv_len), _ptr(out), _DT[out.dtype], B, T, H, D, int(max_k),
        int(max_kv_len), float(scale), _DT[q.dtype], _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def ems_pack_tokens(padded_ids, token_nums, cu_seqlens, packed_ids, stream=None) -> None:
    """Alg. 1 on the device: padded [B, k_max] ids + counts -> cu_seqlens [B+1], packed ids."""
    if not isinstance(padded_ids, torch.Tensor) or padded_ids.dim() != 2:
        _refuse(ValueError, "padded_ids must be a [B, k_max] tensor")
    B, k_max = padded_ids.shape
    _need("padded_ids", padded_ids, _I32)
    _need("token_nums", token_nums, _I32, numel=B)
    _need("cu_seqlens", cu_seqlens, _I32, numel=B + 1)
    _need("packed_ids", packed_ids, _I32, at_least=B * k_max)
    _resident()
    _check(lib().ems_pack_tokens(_ptr(padded_ids), _ptr(token_nums), B, k_max, _ptr(cu_seqlens),
                                 _ptr(packed_ids), _stream(stream)))


def ems_validate_tree(cu_seqlens, parent, stream=None) -> None:
    _need("cu_seqlens", cu_seqlens, _I32, at_least=2)
    _need("parent", parent, _I32)
    _resident()
    _check(lib().ems_validate_tree(_ptr(cu_seqlens), _ptr(parent), cu_seqlens.numel() - 1, parent.numel(),
                                   _stream(stream)))


def ems_tree_accept(logits: Optional[torch.Tensor], target_ids, input_ids, parent, cu_seqlens,
                    accepted, accepted_cu, out_tokens: Optional[torch.Tensor],
                    accepted_rows: Optional[torch.Tensor], *,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    _need_accept(logits, target_ids, input_ids, cu_seqlens, accepted, accepted_cu, out_tokens, workspace,
                 parent=parent, accepted_rows=accepted_rows, tree=True)
    B = accepted.numel()
    T = input_ids.numel()
    V = logits.shape[1] if logits is not None else 0
    dt = _DT[logits.dtype] if logits is not None else EMS_F16
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _resident()
    _check(lib().ems_tree_accept(
        _ptr(logits), dt, V, _ptr(target_ids), _ptr(input_ids), _ptr(parent), _ptr(cu_seqlens), B, T,
        _ptr(accepted), _ptr(accepted_cu), _ptr(out_tokens), _ptr(accepted_rows), _ptr(workspace),
        ws_bytes, _stream(stream)))


def ems_kv_append_rows(k_new_layers: Sequence[torch.Tensor], v_new_layers: Sequence[torch.Tensor],
                       caches: Sequence[KvCacheStruct], accepted_rows, accepted_cu, kv_start, kv_len,
                       kv_len_out: Optional[torch.Tensor], stream=None) -> None:
    n = len(caches)
    _need_layers(k_new_layers, v_new_layers, n)
    T, H, D = k_new_layers[0].shape
    _need("kv_start", kv_start, _I32)
    B = kv_start.numel()
    _need("kv_len", kv_len, _I32, numel=B)
    _need("kv_len_out", kv_len_out, _I32, numel=B, optional=True)
    _need("accepted_cu", accepted_cu, _I32, numel=B + 1)
    _need("accepted_rows", accepted_rows, _I32)
    karr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in k_new_layers])
    varr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in v_new_layers])
    carr = (KvCacheStruct * n)(*caches)
    _resident()
    _check(lib().ems_kv_append_rows(karr, varr, carr, n, _ptr(accepted_rows), _ptr(accepted_cu),
                                    _ptr(kv_start), _ptr(kv_len), _ptr(kv_len_out), B, T, H, D,
                                    _DT[k_new_layers[0].dtype], _stream(stream)))


def ems_verify_attention_write_through(q, k_new, v_new, cache, cu_seqlens, kv_start, kv_len, out, **kw) -> None:
    ems_verify_attention(q, k_new, v_new, cache, cu_seqlens, kv_start, kv_len, out, write_through=True, **kw)


def ems_kv_advance(kv_len, accepted, kv_len_out, stream=None) -> None:
    _need("kv_len", kv_len, _I32)
    _need("accepted", accepted, _I32, numel=kv_len.numel())
    _need("kv_len_out", kv_len_out, _I32, numel=kv_len.numel())
    _resident()
    _check(lib().ems_kv_advance(_ptr(kv_len), _ptr(accepted), _ptr(kv_len_out), kv_len.numel(),
                                _stream(stream)))


def ems_validate_inputs(cu_seqlens, kv_start, kv_len, *, T: int, max_k: int, max_kv_len: int,
                        rows: int, stream=None) -> None:
    _need("kv_start", kv_start, _I32)
    _need("kv_len", kv_len, _I32, numel=kv_start.numel())
    _need("cu_seqlens", cu_seqlens, _I32, numel=kv_start.numel() + 1)
    _resident()
    _check(lib().ems_validate_inputs(_ptr(cu_seqlens), _ptr(kv_start), _ptr(kv_len),
                                     kv_start.numel(), T, max_k, max_kv_len, rows,
                                     _stream(stream)))


def ems_padded_verify_attention(q_pad, k_new_pad, v_new_pad, cache: KvCacheStruct, cap: int,
                                key_mask, k_valid, out_pad, *, k_max: int, l_pad: int, scale: float,
                                workspace: torch.Tensor, stream=None) -> None:
    """Ablation: the padded (vanilla) method; tensors are [B*k_max, H, D]."""
    _need_packed(q_pad, k_new_pad, v_new_pad, out_pad, names=("q_pad", "k_new_pad", "v_new_pad", "out_pad"))
    _, H, D = q_pad.shape
    _need("k_valid", k_valid, _I32)
    B = k_valid.numel()
    if q_pad.shape[0] != B * int(k_max):
        _refuse(ValueError, "q_pad must have B * k_max = %d rows, got %d" % (B * int(k_max), q_pad.shape[0]))
    _need("key_mask", key_mask, torch.uint8, numel=B * int(cap))
    _need("workspace", workspace, torch.uint8)
    _resident()
    _check(lib().ems_padded_verify_attention(
        _ptr(q_pad), _ptr(k_new_pad), _ptr(v_new_pad), ctypes.byref(cache), int(cap), _ptr(key_mask),
        _ptr(k_valid), _ptr(out_pad), _DT[out_pad.dtype], B, int(k_max), int(l_pad), H, D,
        float(scale), _DT[q_pad.dtype], _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)))


def ems_padded_kv_append(k_new_pad_layers, v_new_pad_layers, caches, cap: int, key_mask, accepted, *,
                         k_max: int, l_pad: int, tau_max: int, stream=None) -> None:
    n = len(caches)
    _need_layers(k_new_pad_layers, v_new_pad_layers, n)
    _, H, D = k_new_pad_layers[0].shape
    _need("accepted", accepted, _I32)
    B = accepted.numel()
    if k_new_pad_layers[0].shape[0] != B * int(k_max):
        _refuse(ValueError, "k_new_pad must have B * k_max = %d rows" % (B * int(k_max)))
    _need("key_mask", key_mask, torch.uint8, numel=B * int(cap))
    karr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in k_new_pad_layers])
    varr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in v_new_pad_layers])
    carr = (KvCacheStruct * n)(*caches)
    _resident()
    _check(lib().ems_padded_kv_append(karr, varr, carr, n, int(cap), _ptr(key_mask), _ptr(accepted),
                                      B, int(k_max), int(l_pad), int(tau_max), H, D,
                                      _DT[k_new_pad_layers[0].dtype], _stream(stream)))


def ems_stream_read_probe(buf, sink, stream=None) -> None:
    """One launch of the read-only streaming kernel over the whole tensor `buf`."""
    if not (isinstance(buf, torch.Tensor) and buf.is_cuda and buf.is_contiguous()):
        _refuse(ValueError, "buf must be a contiguous GPU tensor")
    _need("sink", sink, _I32, at_least=1)
    _resident()
    _check(lib().ems_stream_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink),
                                       _stream(stream)))


EMS_ATTN_MFMA, EMS_ATTN_VALU = 0, 1


def ems_set_attention_variant(variant: int) -> None:
    _check(lib().ems_set_attention_variant(int(variant)))


def ems_get_attention_variant() -> int:
    return int(lib().ems_get_attention_variant())


def ems_device_memory_figures():
    """(memory clock in kHz, memory bus width in bits) as the HIP runtime reports them."""
    clock, width = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().ems_device_memory_figures(ctypes.byref(clock), ctypes.byref(width)))
    return clock.value, width.value


def ems_profile_enable(max_records: int) -> None:
    _check(lib().ems_profile_enable(int(max_records)))


def ems_profile_read():
    """(summed milliseconds of the timed attention kernels, number of launches timed)."""
    ms = ctypes.c_double(0.0)
    n = ctypes.c_int(0)
    _check(lib().ems_profile_read(ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def ems_profile_read_calls():
    """(ms of the timed main attention kernels, ms of the whole attention calls incl. the merge, launches)."""
    ms = ctypes.c_double(0.0)
    ms_call = ctypes.c_double(0.0)
    n = ctypes.c_int(0)
    _check(lib().ems_profile_read_calls(ctypes.byref(ms), ctypes.byref(ms_call), ctypes.byref(n)))
    return ms.value, ms_call.value, n.value


EMS_NOALLOC_SCRATCH_BYTES = 18 << 20

__all__ = ["ems_verify_attention_noalloc", "EMS_NOALLOC_SCRATCH_BYTES", "ems_workspace_bytes", "ems_profile_read_calls", "ems_pack_tokens", "ems_validate_tree", "ems_tree_verify_attention", "ems_tree_accept", "ems_kv_append_rows", "ems_stream_read_probe", "ems_set_attention_variant", "ems_get_attention_variant", "EMS_ATTN_MFMA", "EMS_ATTN_VALU", "ems_verify_attention_write_through", "ems_kv_advance", "ems_padded_verify_attention", "ems_padded_kv_append", "ems_profile_enable", "ems_profile_read", "EmsError", "KvCacheStruct", "kv_cache", "lib", "ems_attention_workspace_bytes",
           "ems_accept_workspace_bytes", "ems_verify_attention", "ems_greedy_accept",
           "ems_kv_append", "ems_validate_inputs", "EMS_F16", "EMS_BF16", "EMS_F32"]
