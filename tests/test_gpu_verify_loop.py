"""GPU parity of the multi-layer, multi-step verify loop (BASELINE config 5) against the oracle
carried through the same steps: accepted counts, offsets, lengths and cache bytes bit-exact,
attention within 2e-3.  At full size (32 layers, B=128, 20 steps, ~75 GB of caches) the oracle
follows three sampled layers through all 20 steps; the other layers' caches are cross-checked
against a plain index-copy of the accepted rows."""
import numpy as np
import pytest
import torch

import oracle
from workloads import arena_view, bits, make_verify_loop
from helpers import attention_tolerance

pytestmark = pytest.mark.gpu


def run_and_check(loop, oracle_layers, attn_steps, plain_bar=True):
    """plain_bar: the stated max-abs 2e-3 as it is; False only for bf16 outputs over short caches,
    whose own rounding (2^-8 |x|) exceeds the bar once |x| > 0.5 (helpers.attention_tolerance)."""
    from paper_2405_07542_amd.verify_loop import VerifyLoopRunner
    B, H, D = loop.B, loop.H, loop.D
    kv_len = loop.kv_len0.clone()
    runner = VerifyLoopRunner(k_caches=loop.k_caches, v_caches=loop.v_caches, row_stride=loop.row_stride,
                              head_stride=loop.head_stride, rows=loop.rows, kv_start=loop.kv_start,
                              kv_len=kv_len, H=H, D=D, V=loop.V, dtype=loop.dtype, scale=loop.scale,
                              max_k=loop.max_k, max_kv_len=loop.max_kv_len,
                              max_rows=max(st.T for st in loop.steps))
    # the oracle's own copies of the sampled layers, taken before anything runs
    o_k = {l: bits(loop.k_caches[l]).copy() for l in oracle_layers}
    o_v = {l: bits(loop.v_caches[l]).copy() for l in oracle_layers}
    starts = loop.kv_start.cpu().numpy()
    o_len = loop.kv_len0.cpu().numpy().copy()
    # a layer the oracle does not follow: remember what must have been appended where
    other = next((l for l in range(loop.n_layers) if l not in oracle_layers), None)
    expect_rows = []
    worst = 0.0
    for s, st in enumerate(loop.steps):
        print("verify loop step", s, "T", st.T, flush=True)
        cu = st.cu_seqlens.cpu().numpy()
        runner.step(st.q, st.k_new, st.v_new, st.cu_seqlens, st.logits, st.input_ids,
                    None if st.logits is not None else st.target_ids)
        torch.cuda.synchronize()
        x = oracle.argmax(bits(st.logits), loop.dtype) if st.logits is not None else st.target_ids.cpu().numpy()
        acc, acc_cu, toks = oracle.greedy_accept(x, st.input_ids.cpu().numpy(), cu)
        assert np.array_equal(runner.accepted.cpu().numpy(), acc), "step %d" % s
        assert np.array_equal(runner.accepted_cu.cpu().numpy(), acc_cu)
        assert np.array_equal(runner.out_tokens.cpu().numpy()[:acc_cu[-1]], toks)
        k = np.diff(cu)
        assert ((acc >= 1) & (acc <= k)).all()
        for l in oracle_layers:
            if s in attn_steps:
                want = oracle.verify_attention(bits(st.q[l]), bits(st.k_new[l]), bits(st.v_new[l]), o_k[l],
                                               o_v[l], loop.row_stride, loop.head_stride, cu, starts, o_len,
                                               H, D, loop.scale, loop.dtype)
                got = runner.out[l][:st.T].double().cpu().numpy()
                assert np.isfinite(got).all()
                err = np.abs(got - want)                     # outputs are in the input dtype
                worst = max(worst, float(err.max()))
                tol = 2e-3 if plain_bar else attention_tolerance(None, want, loop.dtype)
                assert (err <= tol).all(), "layer %d step %d: max abs err %.3e" % (l, s, err.max())
            new_len = oracle.kv_append(o_k[l], o_v[l], loop.row_stride, loop.head_stride, bits(st.k_new[l]),
                                       bits(st.v_new[l]), cu, acc, starts, o_len, H, D)
        if other is not None:
            for i in range(B):
                for j in range(acc[i]):
                    expect_rows.append((int(starts[i] + o_len[i] + j), s, int(cu[i] + j)))
        o_len = new_len if oracle_layers else o_len + acc
        assert np.array_equal(kv_len.cpu().numpy(), o_len)
    for l in oracle_layers:
        assert np.array_equal(bits(loop.k_caches[l]), o_k[l]), "K cache of layer %d" % l
        assert np.array_equal(bits(loop.v_caches[l]), o_v[l]), "V cache of layer %d" % l
    if other is not None and expect_rows:
        view = arena_view(loop.k_caches[other], loop.layout, loop.rows, H, D)
        dst = torch.tensor([r[0] for r in expect_rows], device=view.device)
        got = view[dst]
        want = torch.stack([loop.steps[s].k_new[other][r] for _, s, r in expect_rows])
        assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert (o_len - loop.kv_len0.cpu().numpy()).min() >= len(loop.steps)
    print("verify loop: attention max abs err %.3e over layers %s, steps %s (bar 2e-3)"
          % (worst, list(oracle_layers), list(attn_steps)), flush=True)


def test_small_loop_every_layer_every_step():
    loop = make_verify_loop(n_layers=3, n_steps=5, B=9, H=4, D=128, V=4096, device="cuda", mean_len=150,
                            max_len=400, dtype=torch.bfloat16, seed=123)
    run_and_check(loop, oracle_layers=[0, 1, 2], attn_steps=range(5), plain_bar=False)


def test_config5_full_size_sampled_layers():
    loop = make_verify_loop(device="cuda")              # 32 layers, B=128, 20 steps, fp16
    run_and_check(loop, oracle_layers=[0, 15, 31], attn_steps=range(20))
