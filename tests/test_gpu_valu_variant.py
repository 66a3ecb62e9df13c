"""GPU parity of the vector-ALU formulation of the attention kernel (a measurement aid
selected with ems_set_attention_variant): same inputs, same oracle, same tolerance as the
default matrix-core formulation, including pairs that are merged from partials."""
import numpy as np
import pytest
import torch

import paper_2405_07542_amd as ems
from workloads import HEAD_MAJOR, TOKEN_MAJOR, make_batch, make_config
from helpers import hip_attention, to_device
from test_gpu_parity import RAGGED_K, RAGGED_KV, check_attention

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def valu_variant():
    ems.ems_set_attention_variant(ems.EMS_ATTN_VALU)
    assert ems.ems_get_attention_variant() == ems.EMS_ATTN_VALU
    yield
    ems.ems_set_attention_variant(ems.EMS_ATTN_MFMA)


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_tiny_config(layout):
    check_attention(make_config(1, layout=layout), label="valu tiny")
    check_attention(make_config(1, layout=layout), out_dtype=torch.float32, label="valu tiny f32")


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
@pytest.mark.parametrize("D", [128, 64])
def test_ragged_lengths(dtype, layout, D):
    b = make_batch(RAGGED_KV, RAGGED_K, H=4, D=D, dtype=dtype, seed=40, capacity=300, layout=layout)
    check_attention(b, out_dtype=torch.float32, label="valu ragged f32 out")
    check_attention(b, label="valu ragged 16-bit out")


def test_pairs_merged_from_partials_and_degenerate_batches():
    check_attention(make_batch([6000], [9], H=1, D=128, dtype=torch.float16, seed=41),
                    out_dtype=torch.float32, label="valu one pair")
    check_attention(make_batch([3000, 10, 2500], [16, 1, 4], H=2, D=64, dtype=torch.bfloat16, seed=42,
                               layout=HEAD_MAJOR), out_dtype=torch.float32, label="valu three pairs")
    check_attention(make_batch([0, 0, 0], [4, 1, 16], H=2, D=128, seed=43, capacity=32), label="valu empty caches")
    check_attention(make_batch([40, 9, 70, 3], [2, 0, 0, 16], H=3, D=64, seed=44, capacity=100),
                    label="valu finished samples")


def test_config_2_full_size_and_agreement_with_the_default():
    b_cpu = make_config(2)
    check_attention(b_cpu, label="valu config 2")
    b = to_device(b_cpu)
    valu = hip_attention(b, out_dtype=torch.float32)
    ems.ems_set_attention_variant(ems.EMS_ATTN_MFMA)
    mfma = hip_attention(b, out_dtype=torch.float32)
    assert float((valu - mfma).abs().max()) <= 2e-3


def test_setter_rejects_unknown_values():
    with pytest.raises(ems.EmsError):
        ems.ems_set_attention_variant(7)
    assert ems.ems_get_attention_variant() == ems.EMS_ATTN_VALU


def test_large_batches_and_the_lds_limit():
    """The per-row state lives in LDS (4 x 36 KiB at D = 128) next to the tile prefix sums: B = 3900
    fits the 160 KiB of a workgroup, B = 8192 does not and is refused on the host; D = 64 (4 x 18
    KiB) takes the maximum batch."""
    rng = np.random.default_rng(73)
    B = 3900
    b = make_batch(rng.integers(0, 41, B).tolist(), rng.integers(0, 4, B).tolist(), H=1, D=128,
                   dtype=torch.bfloat16, seed=74, capacity=48)
    check_attention(b, out_dtype=torch.float32, label="valu B=3900 D=128")
    B = 8192
    kv, k = rng.integers(0, 41, B).tolist(), rng.integers(0, 4, B).tolist()
    check_attention(make_batch(kv, k, H=1, D=64, dtype=torch.float16, seed=75, capacity=48),
                    out_dtype=torch.float32, label="valu B=8192 D=64")
    big = to_device(make_batch(kv, k, H=1, D=128, dtype=torch.float16, seed=76, capacity=48))
    with pytest.raises(ems.EmsError) as e:
        hip_attention(big)
    assert e.value.status == ems.EMS_ERR_UNSUPPORTED and "LDS" in str(e.value)
