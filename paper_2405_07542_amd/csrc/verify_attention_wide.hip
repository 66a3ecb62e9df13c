// Packed multi-token attention for samples that bring MORE than 16 rows per step (up to 64:
// token trees commonly have 32-64 nodes), in the forms where ONE wave per SIMD holds a pair's rows
// in registers -- what head dim 64 runs, and what very large batches fall back to; head dims 80
// and 128 run the staged kernel of verify_attention_staged.hip, which this file launches and
// whose partials it merges.  Same tile line, same loads, same two tile buffers, same partial
// format as verify_attention.hip; what changes:
//   * a wave keeps TWO blocks of 16 query rows of its pair in flight: two B operands (in
//     wave-private LDS, in exactly the per-lane layout the MFMA wants, re-read for every tile)
//     and two sets of accumulators.  Per tile, the scores and the online softmax run block
//     after block (phase 1), leaving the P operands of both blocks in registers; then every
//     V^T operand is built once and multiplied into the accumulators of both blocks (phase 2).
//     So up to 32 rows share one stream of the cache.  (Four blocks in registers -- were
//     tried: the allocator runs out of the 256 non-accumulator registers and spills, and
//     both ways out, one tile buffer instead of two or spilling, were slower than two
//     streams of two blocks.)
//   * a sample with more than 32 rows: (NB = 4, head dim 64) the wave keeps the
//     state of all four blocks, two of them in registers and two parked in wave-private LDS,
//     and per tile runs the two resident blocks, swaps the two pairs (16 LDS reads and writes
//     per lane) and runs the other two on the same tile registers, so the cache is still
//     streamed once; the pair that ran last stays resident for the next tile.  (NB = 2, used
//     when LDS can hold neither the parked states nor the staged kernel's tile rings -- very
//     large batches -- : two pairs per head, (sample, head, half), rows 0..31 and 32..63, each
//     streaming the cache once.)
//   * a sample's new tokens take ceil(k/32) tiles after the cache tiles; the visible set of
//     a row among the new rows is a 64-bit set (a causal prefix, or the row's ancestors in
//     a token tree), of which every new-token tile uses its 32 bits (the first half never
//     sees a key of the second tile: that tile costs it one empty pass);
//   * the Q rows of the next pair are loaded at the switch (no prefetch);
//   * partials that the waves of a workgroup share are merged in LDS as in the 16-row
//     kernel (32 rows of them: at 32 rows per sample the workspace would otherwise take
//     34 MB of writes in the middle of the read stream); not with NB = 4, where LDS is taken.

#include "attention_tiles.h"

namespace ems {

constexpr int kWideBlocks = 2;                             // blocks of 16 rows resident in registers
constexpr int kWideRows = kWideBlocks * kMaxRows;          // 32 rows: a pair with NB = 2, half the rows a pair may have with NB = 4

// NB = blocks of 16 rows a pair may have: 2 (a sample of more than 32 rows is two pairs per
// head) or 4 (one pair per head; two blocks resident, two parked in LDS).
template <int NB> __device__ __forceinline__ int halves_of(int ktot) { return NB == 4 ? 1 : wide_halves(ktot); }

// One (sample, head, half) pair's share of a wave's tile range (wave-uniform).
template <int NB>
struct WideSegment {
    int i, h, half;      // sample, head, which 32 rows of the sample
    int cu_i, ktot, k;   // first packed row of the sample; its rows (<= 64); rows of this pair (<= 16 NB)
    int L;               // cached keys; ceil(L/32) cache tiles, then ceil(ktot/32) tiles of new tokens
    int t0, t1;          // this wave consumes tiles [t0, t1) of the pair
    int64_t cache_off;   // byte offset of (first cache row of the sample, head h) in the arenas
    int64_t new_off;     // byte offset of (first packed row of the sample, head h) in q / k_new / v_new
    __device__ __forceinline__ int ntc() const { return (L + kTileKeys - 1) / kTileKeys; }
    __device__ __forceinline__ int nt() const { return ntc() + new_tiles(ktot); }
    __device__ __forceinline__ int blocks() const { return (k + kMaxRows - 1) / kMaxRows; }
    __device__ __forceinline__ int row0() const { return kWideRows * half; }   // first row of the pair in the sample
    __device__ __forceinline__ void set_half(int hf) {
        half = hf;
        k = min(NB * kMaxRows, ktot - kWideRows * hf);
    }
};

template <int D, int NB>
__device__ __forceinline__ WideSegment<NB> make_wide_segment(const AttnParams& p, const int32_t* prefix, int i,
                                                             int gpos, int gend) {
    WideSegment<NB> s;
    while (uniform(prefix[i + 1]) <= gpos) ++i;
    s.i = i;
    s.cu_i = uniform(p.cu[i]);
    s.ktot = min(kMaxRowsWide, uniform(p.cu[i + 1]) - s.cu_i);   // (never more than the kernel holds)
    s.L = uniform(p.kv_len[i]);
    const int64_t start = (int64_t)uniform(p.kv_start[i]);
    const int nt = s.nt();
    const int rem = gpos - uniform(prefix[i]);
    const int pair = uniform(rem / nt);            // pair of this sample: head-major, then half
    const int halves = halves_of<NB>(s.ktot);
    s.h = uniform(pair / halves);
    s.set_half(pair - s.h * halves);
    s.t0 = rem - pair * nt;
    s.t1 = min(nt, s.t0 + (gend - gpos));
    s.cache_off = start * p.row_stride_b + (int64_t)s.h * p.head_stride_b;
    s.new_off = ((int64_t)s.cu_i * p.H + s.h) * (D * 2);
    return s;
}

template <int D, int NB>
__device__ __forceinline__ WideSegment<NB> next_wide_segment(const AttnParams& p, const int32_t* prefix,
                                                             const WideSegment<NB>& c, int gpos, int gend) {
    if (c.half + 1 < halves_of<NB>(c.ktot)) {      // second half of the same (sample, head)
        WideSegment<NB> s = c;
        s.set_half(c.half + 1);
        s.t0 = 0;
        s.t1 = min(c.nt(), gend - gpos);
        return s;
    }
    if (c.h + 1 >= p.H) return make_wide_segment<D, NB>(p, prefix, c.i + 1, gpos, gend);
    WideSegment<NB> s = c;
    s.h = c.h + 1;
    s.set_half(0);
    s.t0 = 0;
    s.t1 = min(c.nt(), gend - gpos);
    s.cache_off = c.cache_off + p.head_stride_b;
    s.new_off = c.new_off + D * 2;
    return s;
}


// One tile against the (up to two) blocks of query rows of a pair.  Cache tile: `lim` visible keys (the same
// for every row; MASKED when < 32).  Tile of new tokens (NEW): vis[b] = this lane's row of
// block b sees key n of the tile iff bit n is set; a block may see nothing of the tile.
// q_lds: this lane's slot of the wave's Q^T store; operand (block b, k-step s) is at q_lds[(b*KS + s)*64].
template <typename ET, int D, bool MASKED, bool NEW>
__device__ __forceinline__ void compute_tile_wide(const TileRegs<D>& t, const u32x4* q_lds,
                                                  SoftmaxState<ET, D>* st, int nblocks, float scale_log2,
                                                  int lim, const uint32_t* vis, int g) {
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    constexpr bool kSplitP = PSplit<ET>::value;
    // P operands of the blocks; a block the pair does not have keeps zeros (phase 2 then adds
    // nothing to its accumulators, and needs no branch)
    u32x4 pb[kWideBlocks], pl[kWideBlocks];
#pragma unroll
    for (int b = 0; b < kWideBlocks; ++b) {
        pb[b] = u32x4{0u, 0u, 0u, 0u};
        pl[b] = u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int b = 0; b < kWideBlocks; ++b) {
        if (b < nblocks) {                           // wave-uniform
            f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const u32x4 qv = q_lds[(b * KS + s) * kWave];
                sa = mfma16x16x32(ET{}, t.ka[s], qv, sa);
                sb = mfma16x16x32(ET{}, t.kb[s], qv, sb);
            }
            float x[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[i] = sa[i] * scale_log2;
                x[4 + i] = sb[i] * scale_log2;
                if (NEW) {
                    if (((vis[b] >> (4 * g + i)) & 1u) == 0) x[i] = -INFINITY;
                    if (((vis[b] >> (16 + 4 * g + i)) & 1u) == 0) x[4 + i] = -INFINITY;
                } else if (MASKED) {
                    if (4 * g + i >= lim) x[i] = -INFINITY;
                    if (16 + 4 * g + i >= lim) x[4 + i] = -INFINITY;
                }
            }
            const float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                                   fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            // The running reference m only has to keep exp2(x - m) in range, it need not be the
            // true maximum: it moves when a tile exceeds it by more than 2^kMaxSlack, which after
            // a row's first tiles is rare, and while it stays the accumulators (which live in
            // accumulation registers, where a rescale costs three instructions per value) are
            // left alone.  acc / l is the same quotient either way.
            const float m_tile = quad_max(mx);
            const float m_new = m_tile > st[b].m + kMaxSlack ? m_tile : st[b].m;
            const float m_sub = (NEW && m_new == -INFINITY) ? 0.f : m_new;   // nothing visible yet
            const float alpha = fast_exp2(st[b].m - m_sub);
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                x[i] = fast_exp2(x[i] - m_sub);
                psum += x[i];
            }
            st[b].l = st[b].l * alpha + psum;
            st[b].m = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int c = 0; c < VW; ++c) st[b].acc[c] *= alpha;
            }
            pb[b][0] = pack2(ET{}, x[0], x[1]);
            pb[b][1] = pack2(ET{}, x[2], x[3]);
            pb[b][2] = pack2(ET{}, x[4], x[5]);
            pb[b][3] = pack2(ET{}, x[6], x[7]);
            if (kSplitP) {                           // bf16: P as hi + lo, as in the 16-row kernel
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] -= round16(ET{}, x[i]);
                pl[b][0] = pack2(ET{}, x[0], x[1]);
                pl[b][1] = pack2(ET{}, x[2], x[3]);
                pl[b][2] = pack2(ET{}, x[4], x[5]);
                pl[b][3] = pack2(ET{}, x[6], x[7]);
            }
        }
        // one block at a time: the scheduler would otherwise interleave the four independent
        // blocks and keep all their temporaries live at once
        __builtin_amdgcn_sched_barrier(0);
    }
    // every V^T operand is built once and serves all blocks
#pragma unroll
    for (int c = 0; c < VW; ++c) {
        u32x4 va;
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            const uint32_t w0 = t.v[2 * pr][c >> 1];
            const uint32_t w1 = t.v[2 * pr + 1][c >> 1];
            va[pr] = (c & 1) ? pair_hi(w0, w1) : pair_lo(w0, w1);
        }
#pragma unroll
        for (int b = 0; b < kWideBlocks; ++b) {
            st[b].acc[c] = mfma16x16x32(ET{}, va, pb[b], st[b].acc[c]);
            if (kSplitP) st[b].acc[c] = mfma16x16x32(ET{}, va, pl[b], st[b].acc[c]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// LDS of the wide kernel after the tile prefix sums: the waves' Q^T stores (NB blocks each), then
// NB = 2: the parked partials of waves 1..3 for the in-workgroup merge and a word of flags per
// wave; NB = 4: every wave's two parked blocks.
template <int D, int NB> constexpr size_t wide_q_lds_bytes() {
    return (size_t)kWavesPerBlock * NB * TileRegs<D>::KS * kWave * sizeof(u32x4);
}
template <int D> constexpr size_t wide_fold_lds_bytes() {
    return (size_t)(kWavesPerBlock - 1) * kWideBlocks * FoldSlot<D>::floats * sizeof(float) + kWavesPerBlock * sizeof(int32_t);
}
template <int D> constexpr size_t wide_swap_lds_bytes() {
    return (size_t)kWavesPerBlock * kWideBlocks * FoldSlot<D>::floats * sizeof(float);
}

template <typename ET, int D, int NB>
__global__ __launch_bounds__(kAttnThreads, 1) void verify_attention_wide_kernel(AttnParams p) {
    extern __shared__ int32_t prefix[];
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    constexpr int kSlotRows = NB * kMaxRows;      // rows of one partial slot
    typedef TileRegs<D> TR;
    typedef WideSegment<NB> Seg;
    build_tile_prefix<NB == 4 ? kWide64Line : kWideLine>(p, prefix);
    if (blockIdx.x == 0)       // the merge kernel reads the tile prefix from the workspace header
        for (int i = threadIdx.x; i <= p.B; i += blockDim.x) p.ws_header[i] = prefix[i];
    const int total = prefix[p.B];
    const int per = (total + p.num_waves - 1) / p.num_waves;
    const int wave = uniform((int)(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)));
    const int gbeg = wave * per;
    const int gend = min(total, gbeg + per);
    const int lane = threadIdx.x & 63;
    const int n = lane & 15;       // query row inside a block (MFMA column) of this lane
    const int g = lane >> 4;       // which quarter of the k-slots / key rows
    // In-workgroup merge, as in the 16-row kernel: after the prefix sums and the Q^T stores, LDS
    // holds one parked partial (both blocks) per wave 1..3 and a word of flags per wave: bit 0 =
    // this wave parked the partial of the pair it continues, bit 1 = that pair ends in its range.
    const int lw = uniform((int)(threadIdx.x >> 6));
    char* const lds_after_prefix = reinterpret_cast<char*>(prefix) + (((p.B + 1) * 4 + 15) & ~15);
    float* const fold_lds = reinterpret_cast<float*>(lds_after_prefix + wide_q_lds_bytes<D, NB>());
    int32_t* const fold_flags = reinterpret_cast<int32_t*>(fold_lds + (kWavesPerBlock - 1) * kWideBlocks * FoldSlot<D>::floats);
    const bool wg_fold = NB == 2 && p.wg_fold != 0;    // (the host leaves it off for very short walks)
    // NB = 4: this wave's two parked blocks, in the same place (this lane's words)
    float* const swap_lds = fold_lds + lw * kWideBlocks * FoldSlot<D>::floats;
    if (wg_fold && lane == 0) fold_flags[lw] = 0;
    if (gbeg >= gend) {            // (only past the end of a short line) nothing to walk, nothing to merge
        if (wg_fold) __syncthreads();
        return;
    }
    const uint32_t new_row_bytes = (uint32_t)p.H * (D * 2);
    const uint32_t cache_row_bytes = (uint32_t)p.row_stride_b;

    int lo = 0, hi = p.B;          // invariant: prefix[lo] <= gbeg < prefix[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (prefix[mid] <= gbeg) lo = mid; else hi = mid;
    }

    Seg cur = make_wide_segment<D, NB>(p, prefix, uniform(lo), gbeg, gend);
    int cur_end = gbeg + (cur.t1 - cur.t0);
    Seg nxt = cur;
    if (cur_end < gend) nxt = next_wide_segment<D, NB>(p, prefix, cur, cur_end, gend);

    // Q^T of the pair's blocks as B operands of S^T = K Q^T: wave-private LDS, one 16-byte slot
    // per (block, k-step, lane)
    u32x4* const q_lds = reinterpret_cast<u32x4*>(lds_after_prefix) + lw * (NB * KS * kWave) + lane;
    SoftmaxState<ET, D> st[kWideBlocks];   // the two resident blocks: blocks 2*res and 2*res + 1 of the pair
    uint64_t vis[NB];                      // this lane's row of block b: visible new rows of the sample
    int res = 0;                           // NB = 4: which two blocks are resident (wave-uniform)

    // NB = 4: exchange the resident blocks with the parked ones
    auto swap_blocks = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < kWideBlocks; ++b) {
            float* f = swap_lds + b * FoldSlot<D>::floats;
#pragma unroll
            for (int c = 0; c < VW; ++c) {
                f32x4* at = reinterpret_cast<f32x4*>(f + (c * kWave + lane) * 4);
                const f32x4 other = *at;
                *at = st[b].acc[c];
                st[b].acc[c] = other;
            }
            const float m = f[FoldSlot<D>::m_at + lane], l = f[FoldSlot<D>::l_at + lane];
            f[FoldSlot<D>::m_at + lane] = st[b].m;
            f[FoldSlot<D>::l_at + lane] = st[b].l;
            st[b].m = m;
            st[b].l = l;
        }
        res ^= 1;
    };

    // Q rows, per-row state and visible sets of a pair, when it becomes current
    auto begin_segment = [&](const Seg& s) __attribute__((always_inline)) {
        const uint64_t qaddr = uniform_addr(p.q + s.new_off);
        int par = -1;
        if (p.parent != nullptr)
            par = gload<int32_t>(uniform_addr(p.parent + s.cu_i), (uint32_t)min(lane, s.ktot - 1) * 4u);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < s.blocks()) {
                const int row = min(s.row0() + kMaxRows * b + n, s.ktot - 1);   // rows beyond the last repeat it, zeroed below
                const uint32_t qoff = (uint32_t)row * new_row_bytes;
                const bool real = kMaxRows * b + n < s.k;
                u32x4 qv[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) qv[ks] = gload<u32x4>(qaddr, qoff + TR::piece(ks, g));
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const u32x4 z = {0u, 0u, 0u, 0u};
                    q_lds[(b * KS + ks) * kWave] = (real && TR::piece_valid(ks, g)) ? qv[ks] : z;
                }
            }
        }
#pragma unroll
        for (int b = 0; b < kWideBlocks; ++b) {
#pragma unroll
            for (int c = 0; c < VW; ++c) st[b].acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
            st[b].m = -INFINITY;
            st[b].l = 0.f;
        }
        res = 0;                           // blocks 0 and 1 are resident, blocks 2 and 3 (if any) start parked
        if (NB == 4 && s.blocks() > kWideBlocks) {
#pragma unroll
            for (int b = 0; b < kWideBlocks; ++b) {
                float* f = swap_lds + b * FoldSlot<D>::floats;
#pragma unroll
                for (int c = 0; c < VW; ++c)
                    *reinterpret_cast<f32x4*>(f + (c * kWave + lane) * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
                f[FoldSlot<D>::m_at + lane] = -INFINITY;
                f[FoldSlot<D>::l_at + lane] = 0.f;
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < s.blocks()) {
                // among the new rows a row sees itself and the rows before it; in a token tree,
                // itself and its ancestors
                const int row = min(s.row0() + kMaxRows * b + n, s.ktot - 1);
                vis[b] = row >= 63 ? ~0ull : (1ull << (row + 1)) - 1;
                if (p.parent != nullptr) vis[b] = tree_visibility64(par, lane, s.ktot, row);
            }
        }
    };

    auto issue = [&](TileRegs<D>& t, int tile, int L, int k, int64_t cache_off, int64_t new_off)
                     __attribute__((always_inline)) {
        TileSrc src;
        const int ntc = (L + kTileKeys - 1) / kTileKeys;
        const bool is_new = tile >= ntc;                               // wave-uniform
        src.kbase = uniform_addr(is_new ? p.k_new + new_off : p.k_cache + cache_off);
        src.vbase = uniform_addr(is_new ? p.v_new + new_off : p.v_cache + cache_off);
        src.row_bytes = is_new ? new_row_bytes : cache_row_bytes;
        src.n0 = is_new ? (tile - ntc) * kTileKeys : tile * kTileKeys;
        src.last = is_new ? k - 1 : L - 1;
        src.mask_base = 0;
        load_tile<D, false>(t, src, n, g);
    };

    // one tile against the two resident blocks (blocks 2*res and 2*res + 1 of the pair)
    auto run_resident = [&](const TileRegs<D>& t, const Seg& s, int tile) __attribute__((always_inline)) {
        const int nb = min(kWideBlocks, s.blocks() - kWideBlocks * res);
        const u32x4* q = q_lds + res * (kWideBlocks * KS * kWave);
        if (tile < s.ntc()) {
            const int lim = s.L - tile * kTileKeys;
            if (lim >= kTileKeys)
                compute_tile_wide<ET, D, false, false>(t, q, st, nb, p.scale_log2, lim, nullptr, g);
            else
                compute_tile_wide<ET, D, true, false>(t, q, st, nb, p.scale_log2, lim, nullptr, g);
            return;
        }
        const int key0 = kTileKeys * (tile - s.ntc());                 // first new row of this tile
        uint32_t v32[kWideBlocks];
#pragma unroll
        for (int b = 0; b < kWideBlocks; ++b) {
            uint64_t v = vis[b];
            if constexpr (NB == 4) v = res ? vis[kWideBlocks + b] : v;
            v32[b] = (uint32_t)(v >> key0);
        }
        compute_tile_wide<ET, D, true, true>(t, q, st, nb, p.scale_log2, 0, v32, g);
    };

    auto consume = [&](const TileRegs<D>& t, const Seg& s, int tile) __attribute__((always_inline)) {
        // NB = 4 and more than two blocks: the resident two, a swap, the other two on the same
        // tile; those stay resident for the next tile
        const int passes = (NB == 4 && s.blocks() > kWideBlocks) ? 2 : 1;
#pragma unroll 1
        for (int pass = 0; pass < passes; ++pass) {
            if (pass) swap_blocks();
            run_resident(t, s, tile);
        }
        if (tile < s.ntc()) return;
        const int key0 = kTileKeys * (tile - s.ntc());
        if (p.write_through && s.half == 0) {      // (both halves read the new rows, one stores them)
            // Paper order (Sec. 3.2): the new rows' K/V go to the sample's own location, cache
            // rows kv_len + j, straight from the registers of this tile (new rows key0 .. key0+31).
            const uint32_t row_b = cache_row_bytes;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int key = key0 + 16 * half + n;
                if (key < s.ktot) {
                    char* kdst = const_cast<char*>(p.k_cache) + s.cache_off + (uint64_t)(uint32_t)(s.L + key) * row_b;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        if (TR::piece_valid(ks, g))
                            *reinterpret_cast<u32x4*>(kdst + TR::piece(ks, g)) = half ? t.kb[ks] : t.ka[ks];
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = key0 + (e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4));
                if (key < s.ktot && n < TR::kVLanes) {
                    char* vdst = const_cast<char*>(p.v_cache) + s.cache_off + (uint64_t)(uint32_t)(s.L + key) * row_b + n * (VW * 2);
                    *reinterpret_cast<typename TileRegs<D>::vrow_t*>(vdst) = t.v[e];
                }
            }
        }
    };

    // the resident blocks' states normalised into out[cu_i + row0 + 16 (2 res + b) + n, h, :]
    auto write_out = [&](const Seg& s) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < kWideBlocks; ++b) {
            if (kWideBlocks * res + b < s.blocks()) {
                const float l = quad_sum(st[b].l);     // the four lanes of a row hold disjoint shares
                const int r_in_pair = kMaxRows * (kWideBlocks * res + b) + n;
                if (r_in_pair < s.k) {
                    const float inv = 1.0f / l;
                    const int64_t row = ((int64_t)(s.cu_i + s.row0() + r_in_pair) * p.H + s.h) * D;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (4 * g + r >= TR::kVLanes) continue;
                        const int d0 = (4 * g + r) * VW;
                        float o[VW];
#pragma unroll
                        for (int c = 0; c < VW; ++c) o[c] = st[b].acc[c][r] * inv;
                        if (p.out_f32) {
                            float* dst = reinterpret_cast<float*>(p.out) + row + d0;
#pragma unroll
                            for (int c = 0; c < VW; c += 4)
                                *reinterpret_cast<f32x4*>(dst + c) = f32x4{o[c], o[c + 1], o[c + 2], o[c + 3]};
                        } else {
                            uint16_t* dst = reinterpret_cast<uint16_t*>(p.out) + row + d0;
                            typename TileRegs<D>::vrow_t pk;
#pragma unroll
                            for (int c = 0; c < VW; c += 2) pk[c >> 1] = pack2(ET{}, o[c], o[c + 1]);
                            *reinterpret_cast<typename TileRegs<D>::vrow_t*>(dst) = pk;
                        }
                    }
                }
            }
        }
    };
    // the resident blocks' states as a partial in the workspace: slot 2w holds one that continues
    // a pair begun by an earlier wave, slot 2w+1 one that starts a pair and leaves its end to
    // later waves; 16 NB rows per slot
    auto write_partial = [&](const Seg& s) __attribute__((always_inline)) {
        const int slot = 2 * wave + (s.t0 == 0 ? 1 : 0);
#pragma unroll
        for (int b = 0; b < kWideBlocks; ++b) {
            if (kWideBlocks * res + b < s.blocks()) {
                const float l = quad_sum(st[b].l);
                const int r_in_pair = kMaxRows * (kWideBlocks * res + b) + n;
                if (r_in_pair < s.k) {
                    float* dst = p.ws + ((int64_t)slot * kSlotRows + r_in_pair) * (D + kPartialPad);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (4 * g + r >= TR::kVLanes) continue;
                        const int d0 = (4 * g + r) * VW;
#pragma unroll
                        for (int c = 0; c < VW; c += 4)
                            *reinterpret_cast<f32x4*>(dst + d0 + c) =
                                f32x4{st[b].acc[c][r], st[b].acc[c + 1][r], st[b].acc[c + 2][r], st[b].acc[c + 3][r]};
                    }
                    if (g == 0) {
                        dst[D] = st[b].m;
                        dst[D + 1] = l;
                    }
                }
            }
        }
    };

    auto finish_segment = [&](const Seg& s) __attribute__((always_inline)) {
        const bool continues = s.t0 != 0;          // an earlier wave holds the pair's first tiles
        const bool open = s.t1 != s.nt();          // later waves hold its last tiles (then this is the wave's last segment)
        if (NB == 4) {                             // the resident blocks, then the parked ones
            const int passes = s.blocks() > kWideBlocks ? 2 : 1;
#pragma unroll 1
            for (int pass = 0; pass < passes; ++pass) {
                if (pass) swap_blocks();
                if (!continues && !open) write_out(s); else write_partial(s);
            }
        } else if (!continues && !open) {
            write_out(s);
        } else if (!wg_fold) {
            write_partial(s);                      // every wave's partials go to the workspace
        } else if (open && (lw == 0 || !continues)) {
            // stays in registers: after the barrier this wave folds in what the waves after it parked
        } else if (lw == 0) {
            write_partial(s);                      // the pair began in an earlier workgroup
        } else {
#pragma unroll
            for (int b = 0; b < kWideBlocks; ++b) {
                if (b < s.blocks()) {
                    float* f = fold_lds + ((lw - 1) * kWideBlocks + b) * FoldSlot<D>::floats;
#pragma unroll
                    for (int c = 0; c < VW; ++c) *reinterpret_cast<f32x4*>(f + (c * kWave + lane) * 4) = st[b].acc[c];
                    f[FoldSlot<D>::m_at + lane] = st[b].m;
                    f[FoldSlot<D>::l_at + lane] = st[b].l;
                }
            }
            if (lane == 0) fold_flags[lw] = 1 | (open ? 0 : 2);
        }
    };

    int con_t = cur.t0;              // tile of `cur` that is consumed next

    // One step of the walk: issue flat tile c+1 into `fill`, consume flat tile c from `use`.
    auto step = [&](int c, const TileRegs<D>& use, TileRegs<D>& fill) __attribute__((always_inline)) {
        if (c + 1 < gend) {
            const bool same = con_t + 1 < cur.t1;        // else: first tile of the next pair
            issue(fill, same ? con_t + 1 : nxt.t0, same ? cur.L : nxt.L, same ? cur.ktot : nxt.ktot,
                  same ? cur.cache_off : nxt.cache_off, same ? cur.new_off : nxt.new_off);
        }
        consume(use, cur, con_t);
        ++con_t;
        if (con_t == cur.t1) {
            finish_segment(cur);
            if (c + 1 < gend) {
                cur = nxt;
                con_t = cur.t0;
                cur_end = c + 1 + (cur.t1 - cur.t0);
                begin_segment(cur);
                if (cur_end < gend) nxt = next_wide_segment<D, NB>(p, prefix, cur, cur_end, gend);
            }
        }
    };

    TileRegs<D> ta, tb;
    issue(ta, cur.t0, cur.L, cur.ktot, cur.cache_off, cur.new_off);
    begin_segment(cur);
    for (int c = gbeg; c < gend; c += 2) {
        step(c, ta, tb);
        if (c + 1 < gend) step(c + 1, tb, ta);
    }

    if (wg_fold) {
        // `cur` is the wave's last segment and `st` still holds its state
        __syncthreads();
        const bool continues = cur.t0 != 0;
        if (cur.t1 != cur.nt() && (lw == 0 || !continues)) {
            bool complete = false;
            for (int j = lw + 1; j < kWavesPerBlock && !complete; ++j) {
                const int flags = uniform(fold_flags[j]);
                if ((flags & 1) == 0) break;     // (never while the pair is open: wave j holds its next tiles)
#pragma unroll
                for (int b = 0; b < kWideBlocks; ++b) {
                    if (b < cur.blocks()) {
                        const float* f = fold_lds + ((j - 1) * kWideBlocks + b) * FoldSlot<D>::floats;
                        const float mb = f[FoldSlot<D>::m_at + lane];
                        const float lb = f[FoldSlot<D>::l_at + lane];
                        const float mn = fmaxf(st[b].m, mb);
                        // (a range that holds only new-token tiles no key of which the row sees: max -inf, sum 0)
                        const float ms = mn == -INFINITY ? 0.f : mn;
                        const float ea = fast_exp2(st[b].m - ms), eb = fast_exp2(mb - ms);
#pragma unroll
                        for (int c = 0; c < VW; ++c)
                            st[b].acc[c] = st[b].acc[c] * ea + *reinterpret_cast<const f32x4*>(f + (c * kWave + lane) * 4) * eb;
                        st[b].l = st[b].l * ea + lb * eb;
                        st[b].m = mn;
                    }
                }
                complete = (flags & 2) != 0;
            }
            if (complete && !continues)
                write_out(cur);
            else
                write_partial(cur);
        }
    }
}

// Merge of the partials of pairs shared by several waves, as in the 16-row kernels, with 16 NB
// rows per slot and, with NB = 2, up to two pairs per (sample, head).
template <int D> struct WideCombine {
    static constexpr int lanes_per_row = D / 4;
    static constexpr int rows_per_pass = 8;
    static constexpr int threads = rows_per_pass * lanes_per_row;
};

template <typename ET, int D, int NB>
__global__ __launch_bounds__(WideCombine<D>::threads) void combine_wide_partials_kernel(AttnParams p) {
    constexpr int kSlotRows = NB * kMaxRows;
    const int i = blockIdx.y, h = blockIdx.x;
    const int cu_i = p.cu[i];
    const int ktot = min(kMaxRowsWide, p.cu[i + 1] - cu_i);
    const int total = p.ws_header[p.B];
    const int first = p.ws_header[i];
    const int next = p.ws_header[i + 1];
    if (ktot <= 0) return;
    const int per = (total + p.num_waves - 1) / p.num_waves;
    const int halves = halves_of<NB>(ktot);
    const int nt = (next - first) / (p.H * halves);
    constexpr int pitch = D + kPartialPad;
    constexpr int lanes_per_row = WideCombine<D>::lanes_per_row;
    const int c4 = (threadIdx.x % lanes_per_row) * 4;
    for (int half = 0; half < halves; ++half) {        // the pairs of this (sample, head)
    const int g0 = first + (h * halves + half) * nt;
    const int w0 = g0 / per, w1 = (g0 + nt - 1) / per;
    if (w0 == w1) continue;                // one wave saw the whole pair and wrote `out` itself
    // With the in-workgroup merge only the first wave of the pair and the first wave of every
    // later workgroup it reaches have written a slot; a pair inside one workgroup is done.
    const int wstep = p.wg_fold ? kWavesPerBlock : 1;
    if (p.wg_fold && w0 / kWavesPerBlock == w1 / kWavesPerBlock) continue;
    const int wsecond = p.wg_fold ? (w0 / kWavesPerBlock + 1) * kWavesPerBlock : w0 + 1;
    const int k = min(kSlotRows, ktot - kWideRows * half);
    for (int j = threadIdx.x / lanes_per_row; j < k; j += WideCombine<D>::rows_per_pass) {
        auto slot_row = [&](int w) -> const float* {
            const int slot = 2 * w + (w == w0 ? 1 : 0);
            return p.ws + ((int64_t)slot * kSlotRows + j) * pitch;
        };
        float M = -INFINITY, den = 0.f;
        f32x4 num = {0.f, 0.f, 0.f, 0.f};
        auto fold = [&](float m, float l, f32x4 v) {
            const float Mn = fmaxf(M, m);
            // (a range that holds only new-token tiles no key of which the row sees: max -inf, sum 0)
            const float Ms = Mn == -INFINITY ? 0.f : Mn;
            const float a = fast_exp2(M - Ms), b = fast_exp2(m - Ms);
            num = num * a + v * b;
            den = den * a + l * b;
            M = Mn;
        };
        {
            const float* s0 = slot_row(w0);
            fold(s0[D], s0[D + 1], *reinterpret_cast<const f32x4*>(s0 + c4));
        }
        int w = wsecond;
        for (; w + wstep <= w1; w += 2 * wstep) {
            const float* s0 = slot_row(w);
            const float* s1 = slot_row(w + wstep);
            const float m0 = s0[D], l0 = s0[D + 1], m1 = s1[D], l1 = s1[D + 1];
            const f32x4 v0 = *reinterpret_cast<const f32x4*>(s0 + c4);
            const f32x4 v1 = *reinterpret_cast<const f32x4*>(s1 + c4);
            fold(m0, l0, v0);
            fold(m1, l1, v1);
        }
        if (w <= w1) {
            const float* s0 = slot_row(w);
            fold(s0[D], s0[D + 1], *reinterpret_cast<const f32x4*>(s0 + c4));
        }
        const float inv = 1.0f / den;
        const int64_t idx = ((int64_t)(cu_i + kWideRows * half + j) * p.H + h) * D + c4;
        if (p.out_f32) {
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(p.out) + idx) = num * inv;
        } else {
            u32x2 pk;
            pk[0] = pack2(ET{}, num[0] * inv, num[1] * inv);
            pk[1] = pack2(ET{}, num[2] * inv, num[3] * inv);
            *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(p.out) + idx) = pk;
        }
    }
    }
}

// LDS a launch needs; NB = 4 only fits while the tile prefix sums leave room (B up to a few thousand).
template <int D, int NB> static size_t wide_lds_bytes(int B, bool wg_fold) {
    size_t lds = ((((size_t)(B + 1) * sizeof(int32_t)) + 15) & ~(size_t)15) + wide_q_lds_bytes<D, NB>();
    if (NB == 4) return lds + wide_swap_lds_bytes<D>();
    return wg_fold ? lds + wide_fold_lds_bytes<D>() : lds;
}

template <typename ET, int D, int NB>
static hipError_t launch_wide_typed(const AttnParams& params, int blocks, hipStream_t stream,
                                    hipEvent_t ev_start, hipEvent_t ev_stop) {
    AttnParams p = params;
    if (NB == 4) p.wg_fold = 0;        // LDS holds the parked blocks instead
    // tile prefix sums (at most 32 KiB) + the waves' Q^T stores (4 x 8 KiB at D = 128 with NB = 2)
    // + three parked partials of two blocks (51 KiB at D = 128) or, with NB = 4, twice the Q^T
    // stores and every wave's two parked blocks (68 KiB): above the 64 KiB a kernel gets by
    // default on some HIP platforms, so ask for the device's 160 KiB
    const size_t lds = wide_lds_bytes<D, NB>(p.B, p.wg_fold != 0);
    if (lds > (size_t)kMaxLdsBytes) return hipErrorInvalidValue;     // (the API layer picks NB = 2 first)
    hipError_t e;
    if (lds > 64 * 1024) {
        static std::atomic<uint64_t> raised{0};
        e = allow_max_lds(reinterpret_cast<const void*>(&verify_attention_wide_kernel<ET, D, NB>), raised);
        if (e != hipSuccess) return e;
    }
    if (ev_start && (e = hipEventRecord(ev_start, stream)) != hipSuccess) return e;
    hipLaunchKernelGGL((verify_attention_wide_kernel<ET, D, NB>), dim3(blocks), dim3(kAttnThreads), lds,
                       stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev_stop && (e = hipEventRecord(ev_stop, stream)) != hipSuccess) return e;
    hipLaunchKernelGGL((combine_wide_partials_kernel<ET, D, NB>), dim3(p.H, p.B),
                       dim3(WideCombine<D>::threads), 0, stream, p);
    return hipGetLastError();
}

template <int NB>
static hipError_t launch_wide_blocks(const AttnParams& p, int blocks, int D, bool bf16, hipStream_t stream,
                                     hipEvent_t ev_start, hipEvent_t ev_stop) {
    if (D == 128) return bf16 ? launch_wide_typed<BF16, 128, NB>(p, blocks, stream, ev_start, ev_stop)
                              : launch_wide_typed<F16, 128, NB>(p, blocks, stream, ev_start, ev_stop);
    if (D == 80) return bf16 ? launch_wide_typed<BF16, 80, NB>(p, blocks, stream, ev_start, ev_stop)
                             : launch_wide_typed<F16, 80, NB>(p, blocks, stream, ev_start, ev_stop);
    return bf16 ? launch_wide_typed<BF16, 64, NB>(p, blocks, stream, ev_start, ev_stop)
                : launch_wide_typed<F16, 64, NB>(p, blocks, stream, ev_start, ev_stop);
}

// The staged kernel (verify_attention_staged.hip) and the merge of its partials: 32-row slots and
// one pair per head when the call said at most 32 rows, 64-row slots otherwise.
template <typename ET, int D>
static hipError_t launch_staged_and_merge(const AttnParams& params, int blocks, bool bf16, hipStream_t stream,
                                          hipEvent_t ev_start, hipEvent_t ev_stop) {
    AttnParams p = params;
    p.wg_fold = 0;                               // partials go through the workspace
    p.num_waves = blocks * kStagedStreams;       // the tile line is cut per stream
    hipError_t e;
    if (ev_start && (e = hipEventRecord(ev_start, stream)) != hipSuccess) return e;
    if ((e = launch_verify_attention_staged(p, blocks, D, bf16, stream)) != hipSuccess) return e;
    if (ev_stop && (e = hipEventRecord(ev_stop, stream)) != hipSuccess) return e;
    if (p.multi == 2)
        hipLaunchKernelGGL((combine_wide_partials_kernel<ET, D, 4>), dim3(p.H, p.B), dim3(WideCombine<D>::threads), 0, stream, p);
    else
        hipLaunchKernelGGL((combine_wide_partials_kernel<ET, D, 2>), dim3(p.H, p.B), dim3(WideCombine<D>::threads), 0, stream, p);
    return hipGetLastError();
}

// Whether all 64 rows of a sample can share one stream of the cache at this batch size (else a
// sample of more than 32 rows is two pairs per head): head dims 80 and 128 ask the staged kernel's
// LDS, head dim 64 the one-wave form's with two parked blocks.
bool wide_rows64_fits(int B, int D) {
    if (D != 64) return staged_attention_lds_bytes(B, D) <= (size_t)kMaxLdsBytes;
    return wide_lds_bytes<64, 4>(B, false) <= (size_t)kMaxLdsBytes;
}

hipError_t launch_verify_attention_wide(const AttnParams& p, int blocks, int D, bool bf16,
                                        hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    // Head dims 80 and 128: the staged kernel, 17..64 rows, while its LDS fits (then p.multi = 1
    // means that the call said at most 32 rows, since above 32 rows the API layer sets p.multi = 2
    // exactly when wide_rows64_fits).
    if (D != 64 && staged_attention_lds_bytes(p.B, D) <= (size_t)kMaxLdsBytes) {
        if (D == 128) return bf16 ? launch_staged_and_merge<BF16, 128>(p, blocks, bf16, stream, ev_start, ev_stop)
                                  : launch_staged_and_merge<F16, 128>(p, blocks, bf16, stream, ev_start, ev_stop);
        return bf16 ? launch_staged_and_merge<BF16, 80>(p, blocks, bf16, stream, ev_start, ev_stop)
                    : launch_staged_and_merge<F16, 80>(p, blocks, bf16, stream, ev_start, ev_stop);
    }
    // Head dim 64, or a batch too large for the staged kernel's LDS: one wave per SIMD holds 32
    // rows (a sample of more is two pairs per head) or, head dim 64 only, 64 rows with two of its
    // four blocks parked in LDS.
    if (p.multi == 2) return bf16 ? launch_wide_typed<BF16, 64, 4>(p, blocks, stream, ev_start, ev_stop)
                                  : launch_wide_typed<F16, 64, 4>(p, blocks, stream, ev_start, ev_stop);
    return launch_wide_blocks<2>(p, blocks, D, bf16, stream, ev_start, ev_stop);
}

}  // namespace ems
