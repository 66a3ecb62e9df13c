"""Shared plumbing of the GPU parity tests: run one batch through the C ABI (via the
Python binding) and through the oracle.  No arithmetic of the method lives here."""
import numpy as np
import torch

import oracle
from workloads import bits


def to_device(b, device="cuda"):
    """A copy of the batch with every tensor on `device`."""
    import dataclasses
    kw = {}
    for f in dataclasses.fields(b):
        v = getattr(b, f.name)
        kw[f.name] = v.to(device) if isinstance(v, torch.Tensor) else v
    return type(b)(**kw)


GUARD_BYTES = 256
GUARD_PATTERN = 0xA5


def guarded(nbytes, device):
    """A uint8 device buffer of nbytes followed by GUARD_BYTES of a fixed pattern that nobody may write."""
    buf = torch.empty(nbytes + GUARD_BYTES, dtype=torch.uint8, device=device)
    buf[nbytes:] = GUARD_PATTERN
    return buf


def assert_guard_intact(buf, nbytes, what):
    tail = buf[nbytes:].cpu()
    assert bool((tail == GUARD_PATTERN).all()), "%s: bytes beyond its end were written (first at +%d)" % (
        what, int((tail != GUARD_PATTERN).nonzero()[0]))


def hip_attention(b, out_dtype=None, k_cache=None, v_cache=None, kv_len=None, max_kv_len=None):
    """One ems_verify_attention call.  `out` (NaN-filled) and the workspace are each followed by
    guard bytes that must come back untouched."""
    import paper_2405_07542_amd as ems
    odt = out_dtype or b.dtype
    out_bytes = b.T * b.H * b.D * torch.empty((), dtype=odt).element_size()
    out_buf = guarded(out_bytes, b.q.device)
    out = out_buf[:out_bytes].view(odt).view(b.T, b.H, b.D)
    out.fill_(float("nan"))
    max_kv = b.max_kv_len if max_kv_len is None else max_kv_len
    ws_bytes = ems.ems_workspace_bytes(b.B, b.T, b.H, b.D, max_kv)
    ws_buf = guarded(ws_bytes, b.q.device)
    ws = ws_buf[:ws_bytes]
    cache = ems.kv_cache(b.k_cache if k_cache is None else k_cache,
                         b.v_cache if v_cache is None else v_cache,
                         b.row_stride, b.head_stride, b.rows)
    ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start,
                             b.kv_len if kv_len is None else kv_len, out,
                             max_k=b.max_k, max_kv_len=max_kv, scale=b.scale, workspace=ws)
    torch.cuda.synchronize()
    assert_guard_intact(out_buf, out_bytes, "out")
    assert_guard_intact(ws_buf, ws_bytes, "attention workspace")
    return out


def oracle_attention(b, k_cache=None, v_cache=None, kv_len=None):
    return oracle.verify_attention(
        bits(b.q), bits(b.k_new), bits(b.v_new),
        bits(b.k_cache if k_cache is None else k_cache),
        bits(b.v_cache if v_cache is None else v_cache),
        b.row_stride, b.head_stride, b.cu_seqlens.cpu().numpy(), b.kv_start.cpu().numpy(),
        (b.kv_len if kv_len is None else kv_len).cpu().numpy(), b.H, b.D, b.scale, b.dtype)


def hip_accept(b, use_logits=True, want_tokens=True):
    import paper_2405_07542_amd as ems
    dev = b.q.device
    accepted = torch.full((b.B,), -7, dtype=torch.int32, device=dev)
    accepted_cu = torch.full((b.B + 1,), -7, dtype=torch.int32, device=dev)
    out_tokens = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device=dev) if want_tokens else None
    logits = b.logits if use_logits else None
    if logits is not None:
        target = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device=dev)
        ws = torch.empty(max(8, ems.ems_accept_workspace_bytes(b.T, b.V)), dtype=torch.uint8, device=dev)
    else:
        target = b.target_ids.clone()
        ws = None
    ems.ems_greedy_accept(logits, target, b.input_ids, b.cu_seqlens, accepted, accepted_cu,
                          out_tokens, workspace=ws)
    torch.cuda.synchronize()
    return target[:b.T], accepted, accepted_cu, out_tokens


def oracle_accept(b, use_logits=True):
    x = oracle.argmax(bits(b.logits), b.dtype) if (use_logits and b.logits is not None) \
        else b.target_ids.cpu().numpy()
    acc, acc_cu, out = oracle.greedy_accept(x, b.input_ids.cpu().numpy(), b.cu_seqlens.cpu().numpy())
    return x, acc, acc_cu, out


def attention_tolerance(b, want: np.ndarray, out_dtype) -> np.ndarray:
    """Element-wise bound on |HIP - oracle|: 2e-3 (the stated bar for 16-bit inputs with
    fp32 accumulation), plus, for bf16 OUTPUT only, the rounding of the result itself to
    bf16 (half an ulp <= 2^-8 |x|), which the bar cannot absorb once |x| > 0.5."""
    tol = np.full(want.shape, 2e-3)
    if out_dtype == torch.bfloat16:
        tol = tol + np.abs(want) * 2.0 ** -8
    return tol
