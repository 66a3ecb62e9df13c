"""fp64 CPU oracle of the ragged verification step -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares nothing with the HIP library: the arithmetic lives in
``ems_oracle.c`` (plain C, fp64), compiled with gcc into ``libems_oracle.so``
and called here through ctypes with numpy arrays.

16-bit floating inputs are passed as their raw bit patterns (``uint16``) plus a
dtype tag, so fp16 and bf16 are widened to fp64 exactly inside the C code.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ems_oracle.c")
_LIB = os.path.join(_HERE, "libems_oracle.so")

F16, BF16 = 0, 1
_DTYPES = {"f16": F16, "fp16": F16, "float16": F16, "bf16": BF16, "bfloat16": BF16}


def build(force: bool = False) -> str:
    """Compile ems_oracle.c with gcc (-O2, OpenMP).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # (tests/test_oracle_mutants.py points this at a deliberately broken build of a COPY of
        # the source, to show that the pins notice; nothing else sets it)
        lib = ctypes.CDLL(os.environ.get("EMS_ORACLE_LIBRARY") or build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_restore_index.argtypes = [i32p, ctypes.c_int, ctypes.c_int, i32p, i32p]
        lib.oracle_verify_attention.argtypes = [
            u16p, u16p, u16p, u16p, u16p, ctypes.c_int64, ctypes.c_int64,
            i32p, i32p, i32p, f64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_float, ctypes.c_int]
        lib.oracle_argmax.argtypes = [u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p]
        lib.oracle_argmax_f32.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int, ctypes.c_int, i32p]
        lib.oracle_tree_verify_attention.argtypes = [
            u16p, u16p, u16p, u16p, u16p, ctypes.c_int64, ctypes.c_int64,
            i32p, i32p, i32p, i32p, f64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_float, ctypes.c_int]
        lib.oracle_concatenate_tokens.argtypes = [i32p, i32p, ctypes.c_int, ctypes.c_int, i32p, i32p]
        lib.oracle_concatenate_tokens.restype = ctypes.c_int
        lib.oracle_tree_accept.argtypes = [i32p, i32p, i32p, i32p, ctypes.c_int, i32p, i32p, i32p, i32p]
        lib.oracle_kv_append_rows.argtypes = [
            u16p, u16p, ctypes.c_int64, ctypes.c_int64, u16p, u16p,
            i32p, i32p, i32p, i32p, i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_greedy_accept.argtypes = [i32p, i32p, i32p, ctypes.c_int, i32p, i32p, i32p]
        lib.oracle_kv_append.argtypes = [
            u16p, u16p, ctypes.c_int64, ctypes.c_int64, u16p, u16p,
            i32p, i32p, i32p, i32p, i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        u8p = ctypes.POINTER(ctypes.c_uint8)
        lib.oracle_padded_verify_attention.argtypes = [
            u16p, u16p, u16p, u16p, u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, u8p, i32p,
            f64p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_float, ctypes.c_int]
        lib.oracle_padded_kv_append.argtypes = [
            u16p, u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, u8p, u16p, u16p, i32p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_kv_write_through.argtypes = [
            u16p, u16p, ctypes.c_int64, ctypes.c_int64, u16p, u16p, i32p, i32p, i32p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int]
        _lib = lib
    return _lib


def _dt(dtype) -> int:
    if isinstance(dtype, int):
        return dtype
    return _DTYPES[str(dtype).replace("torch.", "")]


def _u16(a, writable=False) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("16-bit float data must come as float16 or raw uint16 bits, got %s" % a.dtype)
    if not a.flags.c_contiguous:
        raise ValueError("oracle arrays must be C-contiguous")
    if writable and not a.flags.writeable:
        raise ValueError("array must be writable")
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def restore_index(token_nums_per_sample, r: int):
    """Alg. 2: (sample, position) of packed row r."""
    t = _i32(token_nums_per_sample)
    s = ctypes.c_int32(-1)
    p = ctypes.c_int32(-1)
    rc = _load().oracle_restore_index(_p(t, ctypes.c_int32), len(t), int(r),
                                      ctypes.byref(s), ctypes.byref(p))
    if rc:
        raise IndexError("row %d is beyond the packed tokens" % r)
    return int(s.value), int(p.value)


def verify_attention(q, k_new, v_new, k_cache, v_cache, row_stride, head_stride,
                     cu_seqlens, kv_start, kv_len, H, D, scale, dtype) -> np.ndarray:
    """fp64 [T, H, D] attention output; strides in elements."""
    q, k_new, v_new = _u16(q), _u16(k_new), _u16(v_new)
    k_cache, v_cache = _u16(k_cache), _u16(v_cache)
    cu, ks, kl = _i32(cu_seqlens), _i32(kv_start), _i32(kv_len)
    B = len(ks)
    T = int(cu[B])
    assert len(cu) == B + 1 and len(kl) == B and cu[0] == 0
    assert q.size == T * H * D and k_new.size == T * H * D and v_new.size == T * H * D
    for i in range(B):          # every cache element the oracle will touch exists
        if kl[i] > 0 and cu[i + 1] > cu[i]:
            last = (int(ks[i]) + int(kl[i]) - 1) * row_stride + (H - 1) * head_stride + D - 1
            assert 0 <= last < k_cache.size and last < v_cache.size, "cache region out of bounds"
    out = np.zeros((T, H, D), dtype=np.float64)
    rc = _load().oracle_verify_attention(
        _p(q, ctypes.c_uint16), _p(k_new, ctypes.c_uint16), _p(v_new, ctypes.c_uint16),
        _p(k_cache, ctypes.c_uint16), _p(v_cache, ctypes.c_uint16),
        int(row_stride), int(head_stride),
        _p(cu, ctypes.c_int32), _p(ks, ctypes.c_int32), _p(kl, ctypes.c_int32),
        _p(out, ctypes.c_double), B, int(H), int(D), float(scale), _dt(dtype))
    if rc:
        raise MemoryError("oracle_verify_attention ran out of memory")
    return out


def argmax(logits, dtype) -> np.ndarray:
    """Lowest-index arg-max of each row of a 16-bit float [T, V] matrix."""
    lg = _u16(logits)
    T, V = lg.shape
    x = np.zeros(T, dtype=np.int32)
    if T:
        _load().oracle_argmax(_p(lg, ctypes.c_uint16), _dt(dtype), T, V, _p(x, ctypes.c_int32))
    return x


def greedy_accept(target_ids, input_ids, cu_seqlens):
    """Returns (accepted[B], accepted_cu[B+1], out_tokens[sum accepted])."""
    x, ids, cu = _i32(target_ids), _i32(input_ids), _i32(cu_seqlens)
    B = len(cu) - 1
    T = int(cu[B])
    assert len(x) == T and len(ids) == T
    acc = np.zeros(B, dtype=np.int32)
    acc_cu = np.zeros(B + 1, dtype=np.int32)
    out = np.full(max(T, 1), -1, dtype=np.int32)
    _load().oracle_greedy_accept(_p(x, ctypes.c_int32), _p(ids, ctypes.c_int32),
                                 _p(cu, ctypes.c_int32), B, _p(acc, ctypes.c_int32),
                                 _p(acc_cu, ctypes.c_int32), _p(out, ctypes.c_int32))
    return acc, acc_cu, out[:int(acc_cu[B])].copy()


def kv_append(k_cache, v_cache, row_stride, head_stride, k_new, v_new,
              cu_seqlens, accepted, kv_start, kv_len, H, D) -> np.ndarray:
    """Appends in place into k_cache / v_cache (uint16 bits); returns kv_len_out."""
    k_cache, v_cache = _u16(k_cache, True), _u16(v_cache, True)
    k_new, v_new = _u16(k_new), _u16(v_new)
    cu, acc, ks, kl = _i32(cu_seqlens), _i32(accepted), _i32(kv_start), _i32(kv_len)
    B = len(ks)
    for i in range(B):
        assert 0 <= acc[i] <= cu[i + 1] - cu[i]
        if acc[i] > 0:
            last = (int(ks[i]) + int(kl[i]) + int(acc[i]) - 1) * row_stride \
                + (H - 1) * head_stride + D - 1
            assert last < k_cache.size and last < v_cache.size, "append beyond the arena"
    out = np.zeros(B, dtype=np.int32)
    _load().oracle_kv_append(
        _p(k_cache, ctypes.c_uint16), _p(v_cache, ctypes.c_uint16), int(row_stride),
        int(head_stride), _p(k_new, ctypes.c_uint16), _p(v_new, ctypes.c_uint16),
        _p(cu, ctypes.c_int32), _p(acc, ctypes.c_int32), _p(ks, ctypes.c_int32),
        _p(kl, ctypes.c_int32), _p(out, ctypes.c_int32), B, int(H), int(D))
    return out


def padded_verify_attention(q_pad, k_new_pad, v_new_pad, k_cache, v_cache, row_stride, head_stride,
                            cap, key_mask, k_valid, k_max, l_pad, H, D, scale, dtype) -> np.ndarray:
    """The padded (vanilla) method: fp64 [B*k_max, H, D], padding rows included."""
    q_pad, k_new_pad, v_new_pad = _u16(q_pad), _u16(k_new_pad), _u16(v_new_pad)
    k_cache, v_cache = _u16(k_cache), _u16(v_cache)
    km = np.ascontiguousarray(key_mask, dtype=np.uint8)
    kv = _i32(k_valid)
    B = len(kv)
    assert km.shape == (B, cap) and l_pad <= cap and q_pad.size == B * k_max * H * D
    last = (B * cap - 1) * row_stride + (H - 1) * head_stride + D - 1 if row_stride >= head_stride \
        else (H - 1) * head_stride + (B * cap - 1) * row_stride + D - 1
    assert last < k_cache.size and last < v_cache.size
    out = np.zeros((B * k_max, H, D), dtype=np.float64)
    rc = _load().oracle_padded_verify_attention(
        _p(q_pad, ctypes.c_uint16), _p(k_new_pad, ctypes.c_uint16), _p(v_new_pad, ctypes.c_uint16),
        _p(k_cache, ctypes.c_uint16), _p(v_cache, ctypes.c_uint16), int(row_stride),
        int(head_stride), int(cap), _p(km, ctypes.c_uint8), _p(kv, ctypes.c_int32),
        _p(out, ctypes.c_double), B, int(k_max), int(l_pad), int(H), int(D), float(scale), _dt(dtype))
    if rc:
        raise MemoryError("oracle_padded_verify_attention ran out of memory")
    return out


def padded_kv_append(k_cache, v_cache, row_stride, head_stride, cap, key_mask, k_new_pad, v_new_pad,
                     accepted, k_max, l_pad, tau_max, H, D) -> None:
    """Vanilla append in place: tau_max rows per sample at aligned row l_pad, mask updated."""
    k_cache, v_cache = _u16(k_cache, True), _u16(v_cache, True)
    k_new_pad, v_new_pad = _u16(k_new_pad), _u16(v_new_pad)
    acc = _i32(accepted)
    B = len(acc)
    assert key_mask.dtype == np.uint8 and key_mask.flags.c_contiguous and key_mask.shape == (B, cap)
    assert 0 <= tau_max <= k_max and l_pad + tau_max <= cap
    _load().oracle_padded_kv_append(
        _p(k_cache, ctypes.c_uint16), _p(v_cache, ctypes.c_uint16), int(row_stride),
        int(head_stride), int(cap), _p(key_mask, ctypes.c_uint8), _p(k_new_pad, ctypes.c_uint16),
        _p(v_new_pad, ctypes.c_uint16), _p(acc, ctypes.c_int32), B, int(k_max), int(l_pad),
        int(tau_max), int(H), int(D))


def kv_write_through(k_cache, v_cache, row_stride, head_stride, k_new, v_new, cu_seqlens, kv_start,
                     kv_len, H, D) -> None:
    """Paper order: all k_i new rows of every sample go to cache rows kv_len + j, in place."""
    k_cache, v_cache = _u16(k_cache, True), _u16(v_cache, True)
    k_new, v_new = _u16(k_new), _u16(v_new)
    cu, ks, kl = _i32(cu_seqlens), _i32(kv_start), _i32(kv_len)
    B = len(ks)
    for i in range(B):
        k = int(cu[i + 1] - cu[i])
        if k > 0:
            last = (int(ks[i]) + int(kl[i]) + k - 1) * row_stride + (H - 1) * head_stride + D - 1
            assert last < k_cache.size and last < v_cache.size, "write-through beyond the arena"
    _load().oracle_kv_write_through(
        _p(k_cache, ctypes.c_uint16), _p(v_cache, ctypes.c_uint16), int(row_stride), int(head_stride),
        _p(k_new, ctypes.c_uint16), _p(v_new, ctypes.c_uint16), _p(cu, ctypes.c_int32),
        _p(ks, ctypes.c_int32), _p(kl, ctypes.c_int32), B, int(H), int(D))


def tree_verify_attention(q, k_new, v_new, k_cache, v_cache, row_stride, head_stride,
                          cu_seqlens, parent, kv_start, kv_len, H, D, scale, dtype) -> np.ndarray:
    """fp64 [T, H, D] attention output under a per-sample token tree (parent[T]: index of the
    parent row inside the sample, -1 for a sample's row 0)."""
    q, k_new, v_new = _u16(q), _u16(k_new), _u16(v_new)
    k_cache, v_cache = _u16(k_cache), _u16(v_cache)
    cu, par, ks, kl = _i32(cu_seqlens), _i32(parent), _i32(kv_start), _i32(kv_len)
    B = len(ks)
    T = int(cu[B])
    assert len(cu) == B + 1 and len(kl) == B and cu[0] == 0 and len(par) == T
    assert q.size == T * H * D and k_new.size == T * H * D and v_new.size == T * H * D
    for i in range(B):
        if kl[i] > 0 and cu[i + 1] > cu[i]:
            last = (int(ks[i]) + int(kl[i]) - 1) * row_stride + (H - 1) * head_stride + D - 1
            assert 0 <= last < k_cache.size and last < v_cache.size, "cache region out of bounds"
    out = np.zeros((T, H, D), dtype=np.float64)
    rc = _load().oracle_tree_verify_attention(
        _p(q, ctypes.c_uint16), _p(k_new, ctypes.c_uint16), _p(v_new, ctypes.c_uint16),
        _p(k_cache, ctypes.c_uint16), _p(v_cache, ctypes.c_uint16),
        int(row_stride), int(head_stride),
        _p(cu, ctypes.c_int32), _p(par, ctypes.c_int32), _p(ks, ctypes.c_int32), _p(kl, ctypes.c_int32),
        _p(out, ctypes.c_double), B, int(H), int(D), float(scale), _dt(dtype))
    if rc == 2:
        raise ValueError("parent[] is not a tree in topological order")
    if rc:
        raise MemoryError("oracle_tree_verify_attention ran out of memory")
    return out


def tree_accept(target_ids, input_ids, parent, cu_seqlens):
    """Returns (accepted[B], accepted_cu[B+1], out_tokens[sum], accepted_rows[sum])."""
    x, ids, par, cu = _i32(target_ids), _i32(input_ids), _i32(parent), _i32(cu_seqlens)
    B = len(cu) - 1
    T = int(cu[B])
    assert len(x) == T and len(ids) == T and len(par) == T
    acc = np.zeros(B, dtype=np.int32)
    acc_cu = np.zeros(B + 1, dtype=np.int32)
    out = np.full(max(T, 1), -1, dtype=np.int32)
    rows = np.full(max(T, 1), -1, dtype=np.int32)
    _load().oracle_tree_accept(_p(x, ctypes.c_int32), _p(ids, ctypes.c_int32), _p(par, ctypes.c_int32),
                               _p(cu, ctypes.c_int32), B, _p(acc, ctypes.c_int32),
                               _p(acc_cu, ctypes.c_int32), _p(out, ctypes.c_int32),
                               _p(rows, ctypes.c_int32))
    n = int(acc_cu[B])
    return acc, acc_cu, out[:n].copy(), rows[:n].copy()


def kv_append_rows(k_cache, v_cache, row_stride, head_stride, k_new, v_new,
                   accepted_rows, accepted_cu, kv_start, kv_len, H, D) -> np.ndarray:
    """Gathers the packed rows accepted_rows into the caches in place; returns kv_len_out."""
    k_cache, v_cache = _u16(k_cache, True), _u16(v_cache, True)
    k_new, v_new = _u16(k_new), _u16(v_new)
    rows, acu, ks, kl = _i32(accepted_rows), _i32(accepted_cu), _i32(kv_start), _i32(kv_len)
    B = len(ks)
    assert len(acu) == B + 1 and len(rows) >= int(acu[B])
    T = k_new.size // (H * D)
    for i in range(B):
        a = int(acu[i + 1] - acu[i])
        assert a >= 0
        if a > 0:
            assert all(0 <= int(r) < T for r in rows[acu[i]:acu[i + 1]])
            last = (int(ks[i]) + int(kl[i]) + a - 1) * row_stride + (H - 1) * head_stride + D - 1
            assert last < k_cache.size and last < v_cache.size, "append beyond the arena"
    out = np.zeros(B, dtype=np.int32)
    _load().oracle_kv_append_rows(
        _p(k_cache, ctypes.c_uint16), _p(v_cache, ctypes.c_uint16), int(row_stride),
        int(head_stride), _p(k_new, ctypes.c_uint16), _p(v_new, ctypes.c_uint16),
        _p(rows, ctypes.c_int32), _p(acu, ctypes.c_int32), _p(ks, ctypes.c_int32),
        _p(kl, ctypes.c_int32), _p(out, ctypes.c_int32), B, int(H), int(D))
    return out


def concatenate_tokens(padded_ids, lens):
    """Alg. 1.  Returns (concatenated[total], token_nums_per_sample[B], total)."""
    ids, ln = _i32(padded_ids), _i32(lens)
    B = len(ln)
    k_max = ids.size // B if B else 0
    assert ids.size == B * k_max and all(0 <= int(x) <= k_max for x in ln)
    out = np.full(max(1, B * k_max), -1, dtype=np.int32)
    nums = np.zeros(B, dtype=np.int32)
    total = _load().oracle_concatenate_tokens(_p(ids, ctypes.c_int32), _p(ln, ctypes.c_int32), B, k_max,
                                              _p(out, ctypes.c_int32), _p(nums, ctypes.c_int32))
    return out[:total].copy(), nums, int(total)


def argmax_f32(logits) -> np.ndarray:
    """Greedy target token per row of an fp32 [T, V] array (lowest index on ties)."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    T, V = lg.shape
    x = np.zeros(T, dtype=np.int32)
    if T:
        _load().oracle_argmax_f32(_p(lg, ctypes.c_float), T, V, _p(x, ctypes.c_int32))
    return x
