"""ems_verify_attention_noalloc (the attention call for callers that cannot allocate device
memory: its partial results go to a buffer inside the library's own device image) against
ems_verify_attention on the same inputs, through the C ABI: two calls in a row, the second on
a smaller input, so that what the first call left in the shared buffer must not matter.
Both entry points run the same kernels, so the outputs must agree bit for bit (which is
within the max-abs 2e-3 bar a fortiori); the second call is also compared with the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2405_07542_amd as ems
from workloads import HEAD_MAJOR, make_batch, make_config
from helpers import hip_attention, oracle_attention, to_device

pytestmark = pytest.mark.gpu


def noalloc_attention(b, out_dtype=None):
    out = torch.full((b.T, b.H, b.D), float("nan"), dtype=out_dtype or b.dtype, device=b.q.device)
    cache = ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows)
    ems.ems_verify_attention_noalloc(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                     max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale)
    torch.cuda.synchronize()
    return out


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


def test_two_calls_in_a_row_the_second_smaller():
    # first: config 4's own shape (B=64, bf16, every wave of the launch holds partials) ...
    big_cpu = make_config(4, with_logits=False)
    big = to_device(big_cpu)
    print("noalloc case: config 4, T", big.T, flush=True)
    want_big = hip_attention(big)
    got_big = noalloc_attention(big)
    assert same_bits(got_big, want_big)
    # ... then a small ragged batch in the other layout and dtype, pairs cut over many waves
    small_cpu = make_batch([3000, 10, 2500, 0, 77], [16, 1, 4, 7, 0], H=2, D=64, dtype=torch.float16, seed=4242,
                           layout=HEAD_MAJOR)
    small = to_device(small_cpu)
    print("noalloc case: small ragged batch, T", small.T, flush=True)
    got_small = noalloc_attention(small, out_dtype=torch.float32)
    want_small = hip_attention(small, out_dtype=torch.float32)
    assert same_bits(got_small, want_small)
    err = float(np.abs(got_small.double().cpu().numpy() - oracle_attention(small_cpu)).max())
    assert err <= 2e-3, err
    # and the first input once more: nothing of the small call lingers
    assert same_bits(noalloc_attention(big), want_big)


def test_limits_are_refused_with_the_sizes_in_the_message():
    b = to_device(make_batch([40, 9], [20, 3], H=2, D=64, seed=4243, capacity=64))
    out = torch.empty_like(b.q)
    cache = ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows)
    with pytest.raises(ems.EmsError) as e:
        ems.ems_verify_attention_noalloc(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                         max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale)
    assert e.value.status == ems.EMS_ERR_UNSUPPORTED and "max_k <= 16" in str(e.value)
    # the same host checks as the call with a workspace
    L = ems.lib()
    c = ems.KvCacheStruct(0x1000, 0x1000, 4096, 128, 1024)
    assert L.ems_verify_attention_noalloc(0x1000, 0x1000, 0x1000, ctypes.byref(c), 0x1000, 0x1000, 0x1000, 0x1000,
                                          ems.EMS_F16, 4, 8, 32, 96, 4, 100, 0.1, ems.EMS_F16, None) == ems.EMS_ERR_UNSUPPORTED
    assert L.ems_verify_attention_noalloc(0x1000, 0x1000, 0x1000, ctypes.byref(c), 0x1000, 0x1000, 0x1000, 0x1000,
                                          ems.EMS_F16, 0, 8, 32, 128, 4, 100, 0.1, ems.EMS_F16, None) == ems.EMS_ERR_INVALID_ARG
