"""The Python binding passes raw addresses to the C ABI, so it is the only place where a wrong
element type, a strided view or a host tensor can be caught; it must refuse them before anything
is launched.  These cases run without a GPU: every check fires on the host, and a correct CPU
tensor is refused for where it lives."""
import pytest
import torch

import paper_2405_07542_amd as ems


def packed(T=6, H=2, D=64, dtype=torch.float16):
    return torch.zeros((T, H, D), dtype=dtype)


def i32(n):
    return torch.zeros(n, dtype=torch.int32)


def attention_args(**over):
    B, T = 2, 6
    a = dict(q=packed(), k_new=packed(), v_new=packed(), cache=ems.KvCacheStruct(16, 16, 128, 64, 32),
             cu_seqlens=i32(B + 1), kv_start=i32(B), kv_len=i32(B), out=packed())
    a.update(over)
    return a


def call_attention(a, fn=None):
    (fn or ems.ems_verify_attention)(a["q"], a["k_new"], a["v_new"], a["cache"], a["cu_seqlens"], a["kv_start"],
                                     a["kv_len"], a["out"], max_k=4, max_kv_len=16, scale=0.125,
                                     workspace=torch.zeros(1 << 16, dtype=torch.uint8))


@pytest.mark.parametrize("over,exc,text", [
    (dict(cu_seqlens=torch.zeros(3, dtype=torch.int64)), TypeError, "cu_seqlens must have dtype torch.int32"),
    (dict(kv_start=torch.arange(2)), TypeError, "kv_start must have dtype torch.int32"),
    (dict(kv_len=torch.zeros(2, dtype=torch.int64)), TypeError, "kv_len must have dtype torch.int32"),
    (dict(kv_len=i32(3)), ValueError, "kv_len must hold 2 elements"),
    (dict(cu_seqlens=i32(2)), ValueError, "cu_seqlens must hold 3 elements"),
    (dict(cu_seqlens=i32(6)[::2]), ValueError, "cu_seqlens must be contiguous"),
    (dict(q=packed(12)[::2]), ValueError, "q must be contiguous"),
    (dict(q=packed(D=128)[:, :, :64]), ValueError, "q must be contiguous"),
    (dict(k_new=packed(dtype=torch.bfloat16)), TypeError, "k_new must have dtype torch.float16"),
    (dict(v_new=packed(T=5)), ValueError, "v_new must have shape"),
    (dict(out=packed(dtype=torch.float64)), TypeError, "out must have dtype"),
    (dict(q=torch.zeros((6, 2, 64), dtype=torch.float32), k_new=torch.zeros((6, 2, 64), dtype=torch.float32)),
     TypeError, "q must have dtype"),
    (dict(), ValueError, "must live in GPU memory"),          # all correct, but host tensors
])
def test_attention_binding_refuses_what_the_c_layer_cannot_see(over, exc, text):
    with pytest.raises(exc, match=text):
        call_attention(attention_args(**over))
    with pytest.raises(exc, match=text):
        call_attention(attention_args(**over), fn=ems.ems_verify_attention_write_through)


def test_tree_attention_binding_checks_the_parent_array():
    a = attention_args()
    with pytest.raises(TypeError, match="kv_len must have dtype"):
        ems.ems_tree_verify_attention(a["q"], a["k_new"], a["v_new"], a["cache"], a["cu_seqlens"],
                                      torch.zeros(6, dtype=torch.int64), a["kv_start"],
                                      torch.zeros(2, dtype=torch.int64), a["out"], max_k=4, max_kv_len=16,
                                      scale=0.125, workspace=torch.zeros(1 << 16, dtype=torch.uint8))


def test_accept_binding_refuses_wrong_index_types_and_sizes():
    B, T = 2, 6
    ok = dict(logits=None, target_ids=i32(T), input_ids=i32(T), cu_seqlens=i32(B + 1), accepted=i32(B),
              accepted_cu=i32(B + 1), out_tokens=i32(T))

    def call(**over):
        a = dict(ok)
        a.update(over)
        ems.ems_greedy_accept(a["logits"], a["target_ids"], a["input_ids"], a["cu_seqlens"], a["accepted"],
                              a["accepted_cu"], a["out_tokens"], workspace=a.get("workspace"))
    with pytest.raises(TypeError, match="input_ids must have dtype torch.int32"):
        call(input_ids=torch.zeros(T, dtype=torch.int64))
    with pytest.raises(TypeError, match="cu_seqlens must have dtype torch.int32"):
        call(cu_seqlens=torch.cumsum(torch.ones(B + 1, dtype=torch.int32), 0))      # torch's cumsum gives int64
    with pytest.raises(ValueError, match="accepted_cu must hold 3 elements"):
        call(accepted_cu=i32(B))
    with pytest.raises(ValueError, match="target_ids must hold at least 6"):
        call(target_ids=i32(T - 1))
    with pytest.raises(ValueError, match="logits must be a \\[T, V\\] tensor"):
        call(logits=torch.zeros((T + 1, 50), dtype=torch.float16))
    with pytest.raises(ValueError, match="logits must be contiguous"):
        call(logits=torch.zeros((T, 100), dtype=torch.float16)[:, ::2], workspace=torch.zeros(64, dtype=torch.uint8))
    with pytest.raises(TypeError, match="workspace must be a tensor"):
        call(logits=torch.zeros((T, 50), dtype=torch.float16))
    with pytest.raises(ValueError, match="must live in GPU memory"):
        call()


def test_append_binding_refuses_wrong_layers_and_index_types():
    B, T = 2, 6
    cache = ems.KvCacheStruct(16, 16, 128, 64, 32)

    def call(k=None, v=None, **over):
        a = dict(cu_seqlens=i32(B + 1), accepted=i32(B), kv_start=i32(B), kv_len=i32(B), kv_len_out=i32(B))
        a.update(over)
        ems.ems_kv_append([packed()] if k is None else k, [packed()] if v is None else v, [cache],
                          a["cu_seqlens"], a["accepted"], a["kv_start"], a["kv_len"], a["kv_len_out"])
    with pytest.raises(TypeError, match="accepted must have dtype torch.int32"):
        call(accepted=torch.zeros(B, dtype=torch.int64))
    with pytest.raises(ValueError, match="v_new_layers\\[0\\] must be contiguous"):
        call(v=[packed(12)[::2]])
    with pytest.raises(ValueError, match="one k_new and one v_new tensor per cache"):
        call(k=[packed(), packed()])
    with pytest.raises(ValueError, match="kv_len_out must hold 2 elements"):
        call(kv_len_out=i32(3))
    with pytest.raises(ValueError, match="must live in GPU memory"):
        call()


def test_accept_append_binding_checks_both_halves():
    B, T = 2, 6
    cache = ems.KvCacheStruct(16, 16, 128, 64, 32)

    def call(rows=6, **over):
        a = dict(target_ids=i32(T), input_ids=i32(T), cu_seqlens=i32(B + 1), accepted=i32(B), accepted_cu=i32(B + 1),
                 kv_start=i32(B), kv_len=i32(B), kv_len_out=i32(B))
        a.update(over)
        ems.ems_greedy_accept_append(None, a["target_ids"], a["input_ids"], a["cu_seqlens"], a["accepted"],
                                     a["accepted_cu"], None, [packed(rows)], [packed(rows)], [cache],
                                     a["kv_start"], a["kv_len"], a["kv_len_out"])
    with pytest.raises(TypeError, match="input_ids must have dtype torch.int32"):
        call(input_ids=torch.zeros(T, dtype=torch.int64))
    with pytest.raises(TypeError, match="kv_len must have dtype torch.int32"):
        call(kv_len=torch.zeros(B, dtype=torch.int64))
    with pytest.raises(ValueError, match="kv_start must hold 2 elements"):
        call(kv_start=i32(3))
    with pytest.raises(ValueError, match="k_new_layers hold 8 rows, input_ids 6"):
        call(rows=8)
    with pytest.raises(ValueError, match="must live in GPU memory"):
        call()


def test_kv_cache_refuses_mismatched_arenas():
    with pytest.raises(TypeError, match="k arena must have dtype"):
        ems.kv_cache(torch.zeros(64, dtype=torch.float32), torch.zeros(64, dtype=torch.float32), 64, 64, 1)
    with pytest.raises(TypeError, match="v arena must have dtype"):
        ems.kv_cache(torch.zeros(64, dtype=torch.float16), torch.zeros(64, dtype=torch.bfloat16), 64, 64, 1)
    with pytest.raises(ValueError, match="must live in GPU memory"):
        ems.kv_cache(torch.zeros(64, dtype=torch.float16), torch.zeros(64, dtype=torch.float16), 64, 64, 1)
