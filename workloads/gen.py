"""Seeded synthetic inputs for the ragged verification step.

This module serves both the CPU oracle's tests and the HIP library's tests and
bench.  It holds none of the method's arithmetic: it only draws lengths, values
and token ids, and lays them out.  Everything is derived from an explicit seed.

Shapes follow the OPT-6.7b attention geometry used in the paper's experiments
(H=32, D=128, vocabulary 50272) and its regime of ragged draft counts (a
retrieval-based predictor proposes 0..7 drafts per sample, Sec. 4.1); the
paper's datasets and weights are replaced by N(0,1) values rounded to
fp16/bf16.

Layout of a batch (all torch tensors on ``device``):
  q, k_new, v_new   [T, H, D]   packed rows, T = sum k_i (Alg. 1's concatenation)
  cu_seqlens        [B+1] i32   running sum of token_nums_per_sample
  kv_start, kv_len  [B]   i32   per-sample region of the shared cache arena
  k_cache, v_cache  flat arenas of R rows; element (r, h, d) sits at
                    r*row_stride + h*head_stride + d
                    token-major: row_stride=H*D, head_stride=D
                    head-major : row_stride=D,   head_stride=R*D
  logits            [T, V] or None
  target_ids        [T] i32     the row maxima's positions, known by construction
  input_ids         [T] i32     row 0 of a sample = last emitted token, rows 1.. = drafts
Rows of the arena outside every [kv_start, kv_start+kv_len) hold a NaN bit
pattern, so a read of a row that is not part of a cache poisons the result.
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Sequence

import numpy as np
import torch

BASE_SEED = 240507542
SENTINEL_BITS = {torch.float16: 0x7E00, torch.bfloat16: 0x7FC0}   # quiet NaNs
PLANTED_MAX = 8.0      # exactly representable in fp16 and bf16; N(0,1) never reaches it
TOKEN_MAJOR, HEAD_MAJOR = "token_major", "head_major"


@dataclasses.dataclass
class VerifyBatch:
    B: int
    H: int
    D: int
    T: int
    V: int
    dtype: torch.dtype
    scale: float
    layout: str
    rows: int
    row_stride: int
    head_stride: int
    cu_seqlens: torch.Tensor
    kv_start: torch.Tensor
    kv_len: torch.Tensor
    q: torch.Tensor
    k_new: torch.Tensor
    v_new: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    logits: Optional[torch.Tensor]
    target_ids: torch.Tensor
    input_ids: torch.Tensor
    max_k: int
    max_kv_len: int
    name: str = ""
    parent: Optional[torch.Tensor] = None     # [T] i32, token trees only: parent row inside the sample, -1 for row 0

    def clone_caches(self):
        return self.k_cache.clone(), self.v_cache.clone()


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of an fp16/bf16 tensor as a C-contiguous uint16 numpy array."""
    assert t.dtype in (torch.float16, torch.bfloat16)
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def from_bits(a: np.ndarray, dtype: torch.dtype, device="cpu") -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16).copy()).view(dtype).to(device)


def strides_for(layout: str, rows: int, H: int, D: int):
    if layout == TOKEN_MAJOR:
        return H * D, D
    if layout == HEAD_MAJOR:
        return D, rows * D
    raise ValueError(layout)


def arena_view(arena: torch.Tensor, layout: str, rows: int, H: int, D: int) -> torch.Tensor:
    """A [rows, H, D] strided view of a flat arena (no copy)."""
    rs, hs = strides_for(layout, rows, H, D)
    return arena.as_strided((rows, H, D), (rs, hs, 1))


def _randn(shape, dtype, gen, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(dtype)


def make_batch(kv_len: Sequence[int], k: Sequence[int], *, H: int, D: int,
               dtype: torch.dtype = torch.float16, seed: int = BASE_SEED,
               kv_start: Optional[Sequence[int]] = None, capacity: Optional[int] = None,
               rows: Optional[int] = None, layout: str = TOKEN_MAJOR, V: int = 0,
               vocab_for_ids: Optional[int] = None, match_p: float = 0.7,
               scale: Optional[float] = None, device="cpu", name: str = "",
               tie_rows: float = 0.25) -> VerifyBatch:
    """Build one batch.  Draw order: K cache, V cache, Q, K new, V new, logits, ids."""
    kv_len = [int(x) for x in kv_len]
    k = [int(x) for x in k]
    B = len(kv_len)
    assert len(k) == B and B >= 1
    if kv_start is None:
        cap = capacity if capacity is not None else max(L + kk for L, kk in zip(kv_len, k))
        kv_start = [i * cap for i in range(B)]
    kv_start = [int(x) for x in kv_start]
    if rows is None:
        cap = capacity if capacity is not None else 0
        rows = max(max(s + L + kk for s, L, kk in zip(kv_start, kv_len, k)),
                   max(s + cap for s in kv_start))
    T = sum(k)
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(k)
    rs, hs = strides_for(layout, rows, H, D)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)

    sent = SENTINEL_BITS[dtype]
    sent_i16 = sent - 65536 if sent >= 32768 else sent
    k_cache = torch.full((rows * H * D,), sent_i16, dtype=torch.int16, device=dev).view(dtype)
    v_cache = torch.full((rows * H * D,), sent_i16, dtype=torch.int16, device=dev).view(dtype)
    for arena in (k_cache, v_cache):
        view = arena_view(arena, layout, rows, H, D)
        for i in range(B):
            if kv_len[i] > 0:
                view[kv_start[i]:kv_start[i] + kv_len[i]] = _randn((kv_len[i], H, D), dtype, gen, dev)
    q = _randn((T, H, D), dtype, gen, dev)
    k_new = _randn((T, H, D), dtype, gen, dev)
    v_new = _randn((T, H, D), dtype, gen, dev)

    vocab = V if V > 0 else (vocab_for_ids or 50)
    cpu_gen = torch.Generator(device="cpu")
    cpu_gen.manual_seed(seed + 1)
    target_ids = torch.randint(0, vocab, (T,), generator=cpu_gen, dtype=torch.int64)
    logits = None
    if V > 0:
        logits = _randn((T, V), dtype, gen, dev)
        # The row maximum is planted, so target_ids is known without computing
        # anything: PLANTED_MAX at target_ids[r]; a share of the rows gets the same
        # value again at a higher index (a tie that the lowest index must win).
        rows_idx = torch.arange(T, device=dev)
        tgt_dev = target_ids.to(dev)
        if T:
            logits[rows_idx, tgt_dev] = PLANTED_MAX
            dup = torch.rand(T, generator=cpu_gen) < tie_rows
            hi = torch.minimum(target_ids + 1 + torch.randint(0, vocab, (T,), generator=cpu_gen),
                               torch.full((T,), vocab - 1, dtype=torch.int64))
            sel = dup.nonzero().flatten()
            logits[rows_idx[sel.to(dev)], hi[sel].to(dev)] = PLANTED_MAX
    # Drafts: input row j+1 repeats the target token of row j with probability
    # match_p, otherwise it is some other id.  Row 0 of a sample is free.
    input_ids = torch.randint(0, vocab, (T,), generator=cpu_gen, dtype=torch.int64)
    agree = torch.rand(T, generator=cpu_gen) < match_p
    other = torch.randint(1, vocab, (T,), generator=cpu_gen, dtype=torch.int64) if vocab > 1 \
        else torch.zeros(T, dtype=torch.int64)
    for i in range(B):
        for j in range(k[i] - 1):
            r = int(cu[i]) + j
            input_ids[r + 1] = target_ids[r] if agree[r] else (target_ids[r] + other[r]) % vocab

    def i32(a):
        return torch.tensor(np.asarray(a, dtype=np.int32), dtype=torch.int32, device=dev)

    return VerifyBatch(
        B=B, H=H, D=D, T=T, V=V, dtype=dtype,
        # the C ABI takes the scale as a float: keep the value that float holds
        scale=float(np.float32(scale if scale is not None else 1.0 / np.sqrt(D))),
        layout=layout, rows=rows, row_stride=rs, head_stride=hs,
        cu_seqlens=i32(cu), kv_start=i32(kv_start), kv_len=i32(kv_len),
        q=q, k_new=k_new, v_new=v_new, k_cache=k_cache, v_cache=v_cache, logits=logits,
        target_ids=target_ids.to(torch.int32).to(dev), input_ids=input_ids.to(torch.int32).to(dev),
        max_k=max(k) if k else 0, max_kv_len=max(kv_len) if kv_len else 0, name=name)


def grow_trees(b: VerifyBatch, seed: int, match_p: float = 0.7, shape: str = "random",
               duplicate_p: float = 0.15) -> VerifyBatch:
    """The same batch with its new rows arranged as one token tree per sample (inputs of
    tree-structured verification).  Row 0 of a sample is the root; parent[j] < j.
      shape "random": parent drawn uniformly among the earlier rows (bushy, Medusa-like mixes);
            "chain" : parent[j] = j - 1 (ordinary drafts);
            "star"  : every row hangs off the root (many candidates for one position);
            "wide"  : parent drawn among the last three rows (several long branches).
    input_ids are redrawn to fit the tree: with probability match_p one child of a row (picked
    at random) carries that row's target token, the other children carry other tokens that
    differ from it; with probability duplicate_p a later sibling repeats an earlier sibling's
    token (so that "the lowest-indexed matching child" is exercised).  target_ids, logits and
    everything else are shared with `b`."""
    import dataclasses
    rng = np.random.default_rng(seed)
    cu = b.cu_seqlens.cpu().numpy()
    x = b.target_ids.cpu().numpy()
    ids = b.input_ids.cpu().numpy().copy()
    vocab = int(max(2, b.V if b.V else max(int(x.max(initial=0)), int(ids.max(initial=0))) + 1))
    parent = np.full(len(x), -1, dtype=np.int32)
    for i in range(b.B):
        c0, k = int(cu[i]), int(cu[i + 1] - cu[i])
        for j in range(1, k):
            if shape == "chain":
                parent[c0 + j] = j - 1
            elif shape == "star":
                parent[c0 + j] = 0
            elif shape == "wide":
                parent[c0 + j] = int(rng.integers(max(0, j - 3), j))
            else:
                parent[c0 + j] = int(rng.integers(0, j))
        for u in range(k):
            kids = [c for c in range(u + 1, k) if parent[c0 + c] == u]
            if not kids:
                continue
            lucky = kids[int(rng.integers(0, len(kids)))] if rng.random() < match_p else -1
            for n_c, c in enumerate(kids):
                if c == lucky:
                    ids[c0 + c] = x[c0 + u]
                elif n_c > 0 and rng.random() < duplicate_p:
                    ids[c0 + c] = ids[c0 + kids[int(rng.integers(0, n_c))]]
                else:
                    ids[c0 + c] = (int(x[c0 + u]) + 1 + int(rng.integers(0, vocab - 1))) % vocab
    dev = b.input_ids.device
    return dataclasses.replace(b, input_ids=torch.from_numpy(ids).to(torch.int32).to(dev),
                               parent=torch.from_numpy(parent).to(dev), name=b.name + "+tree:" + shape)


def draw_lengths(n: int, seed: int):
    """kv_len and k of BASELINE config n (drawn first, from their own numpy stream)."""
    rng = np.random.default_rng(seed)
    if n == 1:
        return [17, 40], [3, 5]
    if n == 2:
        B = 8
        return rng.integers(256, 1025, B).tolist(), rng.integers(1, 7, B).tolist()
    if n == 3:
        B = 32
        return rng.integers(512, 2049, B).tolist(), rng.integers(1, 7, B).tolist()
    if n == 4:
        B = 64
        return rng.integers(1024, 2049, B).tolist(), (rng.integers(0, 11, B) + 1).tolist()
    if n == 5:
        B = 128
        L = np.clip(rng.geometric(1.0 / 1024.0, B), 16, 4096)
        return L.tolist(), rng.integers(1, 7, B).tolist()
    raise ValueError("config %r" % n)


CONFIG_NAMES = {
    1: "tiny B=2 H=2 D=64 fp16",
    2: "OPT-6.7b layer B=8 fp16 kv U[256,1024] k U[1,6]",
    3: "OPT-6.7b layer B=32 fp16 kv U[512,2048] k U[1,6]",
    4: "OPT-6.7b layer B=64 bf16 kv U[1024,2048] k U[0,10]+1",
    5: "OPT-6.7b layer B=128 fp16 kv geometric(1024) k U[1,6]",
}


def make_config(n: int, *, seed: int = BASE_SEED, device="cpu", layout: str = TOKEN_MAJOR,
                with_logits: bool = True, variant: int = 0, k_range=None) -> VerifyBatch:
    """The single-layer, single-step batch of BASELINE config n (1..5).

    ``variant`` selects an independent draw of the same distribution (used to
    rotate buffer sets so that a timed call does not find its data in cache).
    ``k_range = (lo, hi)`` replaces the config's rows per sample by U{lo..hi} (token
    trees are larger than the config's draft chains); everything else stays.
    """
    s = seed + n + 1000 * variant
    kv_len, k = draw_lengths(n, s)
    if k_range is not None:
        lo, hi = k_range
        k = np.random.default_rng(s + 77).integers(lo, hi + 1, len(k)).tolist()
    if n == 1:
        return make_batch(kv_len, k, H=2, D=64, dtype=torch.float16, seed=s, kv_start=[0, 64],
                          rows=128, layout=layout, V=0, vocab_for_ids=50, match_p=0.6,
                          scale=0.125, device=device, name=CONFIG_NAMES[1])
    V = 50272 if with_logits else 0
    if n == 2:
        return make_batch(kv_len, k, H=32, D=128, dtype=torch.float16, seed=s, capacity=2048,
                          layout=layout, V=V, vocab_for_ids=50272, device=device,
                          name=CONFIG_NAMES[2])
    if n == 3:
        return make_batch(kv_len, k, H=32, D=128, dtype=torch.float16, seed=s, capacity=4096,
                          layout=layout, V=V, vocab_for_ids=50272, device=device,
                          name=CONFIG_NAMES[3])
    if n == 4:
        return make_batch(kv_len, k, H=32, D=128, dtype=torch.bfloat16, seed=s, capacity=4096,
                          layout=layout, V=V, vocab_for_ids=50272, device=device,
                          name=CONFIG_NAMES[4])
    if n == 5:
        # per-sample capacity = len + room for 20 steps of up to 6 tokens, rounded to 64 rows
        caps = [((L + 120 + 63) // 64) * 64 for L in kv_len]
        starts = np.concatenate([[0], np.cumsum(caps)[:-1]]).tolist()
        return make_batch(kv_len, k, H=32, D=128, dtype=torch.float16, seed=s, kv_start=starts,
                          rows=int(sum(caps)), layout=layout, V=V, vocab_for_ids=50272,
                          device=device, name=CONFIG_NAMES[5])
    raise ValueError("config %r" % n)


@dataclasses.dataclass
class PaddedBatch:
    """The same batch laid out for the padded ("vanilla") method of Sec. 3.1."""
    B: int
    H: int
    D: int
    k_max: int
    l_pad: int
    cap: int
    dtype: torch.dtype
    scale: float
    layout: str
    rows: int
    row_stride: int
    head_stride: int
    q_pad: torch.Tensor       # [B*k_max, H, D]
    k_new_pad: torch.Tensor
    v_new_pad: torch.Tensor
    k_cache: torch.Tensor     # aligned arena of B*cap rows
    v_cache: torch.Tensor
    key_mask: torch.Tensor    # [B, cap] uint8, 1 = real key
    k_valid: torch.Tensor     # [B] int32
    real_rows: torch.Tensor   # [T] int64: padded row index of every packed row of the source batch


def pad_batch(b: VerifyBatch, *, seed: int = 7, interleave: bool = True, extra_pad: int = 0) -> PaddedBatch:
    """Re-lay an unpadded batch as the vanilla method would hold it: inputs padded to k_max
    rows per sample, caches aligned to l_pad rows with padding keys scattered between the real
    ones (as they accumulate over decoding steps, Table 1) and marked in a byte mask.
    Padding rows and keys hold finite N(0,1) junk, as real padding tokens would."""
    dev = b.q.device
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    cpu_gen = torch.Generator(device="cpu")
    cpu_gen.manual_seed(seed)
    cu = b.cu_seqlens.cpu().tolist()
    kv_len = b.kv_len.cpu().tolist()
    kv_start = b.kv_start.cpu().tolist()
    k = [cu[i + 1] - cu[i] for i in range(b.B)]
    k_max = max(max(k), 1)
    l_pad = max(kv_len) + extra_pad
    cap = ((l_pad + k_max + 31) // 32) * 32
    rows = b.B * cap
    rs, hs = strides_for(b.layout, rows, b.H, b.D)
    src_k = arena_view(b.k_cache, b.layout, b.rows, b.H, b.D)
    src_v = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D)
    k_cache = _randn((rows * b.H * b.D,), b.dtype, gen, dev)
    v_cache = _randn((rows * b.H * b.D,), b.dtype, gen, dev)
    dst_k = arena_view(k_cache, b.layout, rows, b.H, b.D)
    dst_v = arena_view(v_cache, b.layout, rows, b.H, b.D)
    key_mask = torch.zeros((b.B, cap), dtype=torch.uint8, device=dev)
    q_pad = _randn((b.B * k_max, b.H, b.D), b.dtype, gen, dev)
    k_new_pad = _randn((b.B * k_max, b.H, b.D), b.dtype, gen, dev)
    v_new_pad = _randn((b.B * k_max, b.H, b.D), b.dtype, gen, dev)
    real_rows = []
    for i in range(b.B):
        L = kv_len[i]
        if interleave:
            pos = torch.randperm(l_pad, generator=cpu_gen)[:L].sort().values
        else:
            pos = torch.arange(l_pad - L, l_pad)
        pos_dev = pos.to(dev)
        if L > 0:
            dst_k[i * cap + pos_dev] = src_k[kv_start[i]:kv_start[i] + L]
            dst_v[i * cap + pos_dev] = src_v[kv_start[i]:kv_start[i] + L]
            key_mask[i, pos_dev] = 1
        sl = slice(cu[i], cu[i + 1])
        q_pad[i * k_max:i * k_max + k[i]] = b.q[sl]
        k_new_pad[i * k_max:i * k_max + k[i]] = b.k_new[sl]
        v_new_pad[i * k_max:i * k_max + k[i]] = b.v_new[sl]
        real_rows += [i * k_max + j for j in range(k[i])]
    return PaddedBatch(
        B=b.B, H=b.H, D=b.D, k_max=k_max, l_pad=l_pad, cap=cap, dtype=b.dtype, scale=b.scale,
        layout=b.layout, rows=rows, row_stride=rs, head_stride=hs, q_pad=q_pad,
        k_new_pad=k_new_pad, v_new_pad=v_new_pad, k_cache=k_cache, v_cache=v_cache,
        key_mask=key_mask, k_valid=torch.tensor(k, dtype=torch.int32, device=dev),
        real_rows=torch.tensor(real_rows, dtype=torch.int64, device=dev))


@dataclasses.dataclass
class LoopStep:
    """Inputs of one verification step of a multi-layer loop (caches live elsewhere)."""
    k: list                     # rows per sample
    T: int
    cu_seqlens: torch.Tensor    # [B+1] i32
    q: list                     # per layer [T,H,D]
    k_new: list
    v_new: list
    logits: Optional[torch.Tensor]
    target_ids: torch.Tensor    # planted row maxima (or the given ids when logits is None)
    input_ids: torch.Tensor


@dataclasses.dataclass
class VerifyLoop:
    """BASELINE config 5: an n_layers-deep, several-steps-long verify loop over ragged caches."""
    B: int
    H: int
    D: int
    V: int
    dtype: torch.dtype
    scale: float
    n_layers: int
    rows: int
    row_stride: int
    head_stride: int
    layout: str
    kv_start: torch.Tensor      # [B] i32
    kv_len0: torch.Tensor       # [B] i32 initial lengths
    k_caches: list              # per layer flat arena
    v_caches: list
    steps: list                 # of LoopStep
    max_k: int
    max_kv_len: int             # upper bound over the whole loop


def make_verify_loop(*, n_layers: int = 32, n_steps: int = 20, B: int = 128, H: int = 32, D: int = 128,
                     V: int = 50272, seed: int = BASE_SEED + 5, device="cpu", layout: str = TOKEN_MAJOR,
                     dtype: torch.dtype = torch.float16, mean_len: int = 1024, max_len: int = 4096,
                     k_hi: int = 6, match_p: float = 0.7) -> VerifyLoop:
    """Cached lengths geometric(mean_len) clipped to [16, max_len]; rows per sample U[1, k_hi]
    redrawn every step; every sample's region has room for n_steps * k_hi more rows (rounded to
    64) and the regions are packed back to back, which is what keeps 128 ragged caches x 32
    layers within one GPU's memory."""
    rng = np.random.default_rng(seed)
    kv_len = np.clip(rng.geometric(1.0 / mean_len, B), 16, max_len).astype(np.int64)
    caps = ((kv_len + n_steps * k_hi + 63) // 64) * 64
    starts = np.concatenate([[0], np.cumsum(caps)[:-1]])
    rows = int(caps.sum())
    rs, hs = strides_for(layout, rows, H, D)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    sent = SENTINEL_BITS[dtype]
    k_caches, v_caches = [], []
    for _ in range(n_layers):
        pair = []
        for _kv in range(2):
            arena = torch.full((rows * H * D,), sent, dtype=torch.int16, device=dev).view(dtype)
            view = arena_view(arena, layout, rows, H, D)
            for i in range(B):
                view[int(starts[i]):int(starts[i] + kv_len[i])] = _randn((int(kv_len[i]), H, D), dtype, gen, dev)
            pair.append(arena)
        k_caches.append(pair[0])
        v_caches.append(pair[1])
    steps = []
    for s in range(n_steps):
        k = rng.integers(1, k_hi + 1, B).tolist()
        first = make_batch([1] * B, k, H=1, D=8, dtype=dtype, seed=seed + 100 + s, V=V,
                           vocab_for_ids=50272, match_p=match_p, device=device)
        T = first.T
        steps.append(LoopStep(
            k=k, T=T, cu_seqlens=first.cu_seqlens,
            q=[_randn((T, H, D), dtype, gen, dev) for _ in range(n_layers)],
            k_new=[_randn((T, H, D), dtype, gen, dev) for _ in range(n_layers)],
            v_new=[_randn((T, H, D), dtype, gen, dev) for _ in range(n_layers)],
            logits=first.logits, target_ids=first.target_ids, input_ids=first.input_ids))

    def i32(a):
        return torch.tensor(np.asarray(a, dtype=np.int32), dtype=torch.int32, device=dev)

    return VerifyLoop(B=B, H=H, D=D, V=V, dtype=dtype, scale=float(np.float32(1.0 / np.sqrt(D))),
                      n_layers=n_layers, rows=rows, row_stride=rs, head_stride=hs, layout=layout,
                      kv_start=i32(starts), kv_len0=i32(kv_len), k_caches=k_caches, v_caches=v_caches,
                      steps=steps, max_k=k_hi, max_kv_len=int(kv_len.max()) + n_steps * k_hi)
