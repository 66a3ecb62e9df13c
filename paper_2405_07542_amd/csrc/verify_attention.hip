// Packed multi-token attention over per-sample KV caches (EMS-SD Sec. 3.2:
// "Unpad KV cache" -- every sample has its own cache start location -- and
// "Unpad input tokens" -- the inputs of all samples are concatenated, and the
// kernel recovers which sample and position a packed row belongs to, Alg. 2).
//
// Design for gfx950 (differs from the paper's one-thread-block-per-token grid,
// Appendix D Eq. 12, which re-streams a sample's cache once per query row):
//   * work is measured in tiles of 32 keys; a (sample, head) pair owns
//     ceil(kv_len/32) cache tiles plus one tile holding its new tokens;
//   * the tiles of all pairs are laid on one line and cut into equal ranges,
//     one per wave, so ragged lengths are balanced without any host knowledge
//     of kv_len[] (the per-sample tile counts are prefix-summed in LDS);
//   * a wave keeps all k_i <= 16 query rows of its pair in registers as an
//     MFMA operand, so each K/V byte is fetched from HBM exactly once and is
//     shared by all query rows;
//   * S^T = K Q^T and O^T = V^T P^T run on v_mfma_f32_16x16x32_{f16,bf16}:
//     K rows are loaded straight into the A-operand layout (64-byte pieces),
//     V rows are loaded fully coalesced (one row = 16 lanes x 16 B) and
//     transposed in registers with v_perm_b32; the S^T accumulator layout is
//     already the B-operand layout of the second product, so P never moves
//     between lanes;
//   * online softmax in the log2 domain; the row maximum is shared by the four
//     lanes that hold one query row via two cross-lane shuffles per tile;
//   * a range that covers only part of a pair leaves an fp32 partial
//     (accumulator, running max, running sum).  Writes to HBM in the middle of
//     the read stream are costly far beyond their size (17 MB of partials at 16
//     rows per sample cost 25 us of 290), so the four waves of a workgroup, whose
//     ranges are neighbours on the line, merge what they share in LDS: a wave
//     that continues a pair of the wave before it in the same workgroup parks
//     that partial in LDS; a wave whose range ends inside a pair keeps that
//     state in registers and, after a barrier at the end of the walk, folds in
//     the parked partials of the waves after it, in wave order.  Only what
//     crosses a workgroup's edge is written to the workspace, and a second
//     small kernel merges those by log-sum-exp.
#include <atomic>

#include "attention_tiles.h"

namespace ems {

// ---------------------------------------------------------------------------------------
// The same tile on the vector ALU instead of the matrix cores (selected at run time; kept
// to measure what the MFMA formulation buys, not as the default).  Loads and the tile
// registers are identical.  Scores: lane (n, g) holds keys n and 16+n, head-dim slice
// [32s + 8g, 32s + 8g + 8) of every k-step s, so a score is 16 two-way dot products per
// key against the query row read from LDS (a broadcast read), then a sum over the four g
// lanes.  The probabilities of a query row cross lanes through LDS (the lanes that hold a
// V row's slice need the weights of keys 4g..4g+3 and 16+4g..16+4g+3) as 16-bit numbers,
// exactly as the matrix-core path feeds them (bf16: hi + lo), and meet V as pairs of
// neighbouring keys in a second run of two-way dot products.  The query rows are walked by
// a run-time loop; the unnormalised outputs of all rows live in wave-private LDS (registers
// cannot be indexed by a run-time row), the running max and sum of row q in lane q of one
// register each.  Cost grows with the number of rows k: roughly 100 (fp16) to 140 (bf16)
// vector instructions plus an LDS round trip per row per tile, where the MFMA path pays
// the same for any k <= 16.
struct ValuState {
    float m, l;          // lane q: running max (log2 domain) and running sum of query row q
};

__device__ __forceinline__ float dot2(F16, uint32_t a, uint32_t b, float c) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, a), __builtin_bit_cast(h2, b), c, false);
}
__device__ __forceinline__ float dot2(BF16, uint32_t a, uint32_t b, float c) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2, a), __builtin_bit_cast(b2, b), c, false);
}

// Rotation by R lanes inside each row of 16 lanes (DPP row_ror).
template <int R>
__device__ __forceinline__ float row_ror(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0x120 + R,
                                                              0xf, 0xf, false));
}
__device__ __forceinline__ float row16_max(float x) {
    x = fmaxf(x, row_ror<8>(x));
    x = fmaxf(x, row_ror<4>(x));
    x = fmaxf(x, row_ror<2>(x));
    return fmaxf(x, row_ror<1>(x));
}
__device__ __forceinline__ float row16_sum(float x) {
    x += row_ror<8>(x);
    x += row_ror<4>(x);
    x += row_ror<2>(x);
    return x + row_ror<1>(x);
}
__device__ __forceinline__ float lane_get(float reg, int lane) {      // lane: wave-uniform
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, reg), lane));
}
__device__ __forceinline__ float lane_set(float reg, int lane, float value, int my_lane) {
    return my_lane == lane ? value : reg;
}

// Wave-private LDS of the vector-ALU formulation: query rows (16-bit, row-major), P of one
// row (hi and lo halves, 32 keys each), and the per-lane shares of the outputs of 16 rows.
template <int D> struct ValuLds {
    static constexpr int q_bytes = kMaxRows * D * 2;
    static constexpr int p_bytes = 2 * kTileKeys * 2;
    static constexpr int acc_bytes = kMaxRows * kWave * (D / 16) * 4;
    static constexpr int bytes = q_bytes + p_bytes + acc_bytes;
};

// `lim` = visible keys of a cache tile (same for every row); the new-token tile (NEW) shows
// row q its own key and the ones before it.
template <typename ET, int D, bool MASKED, bool NEW>
__device__ __forceinline__ void valu_tile(const TileRegs<D>& t, char* lds, ValuState& st,
                                          float scale_log2, int k, int lim, int lane, int n, int g) {
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    constexpr bool kSplitP = PSplit<ET>::value;
    const char* const q_lds = lds;
    uint16_t* const p_hi = reinterpret_cast<uint16_t*>(lds + ValuLds<D>::q_bytes);
    uint16_t* const p_lo = p_hi + kTileKeys;
    float* const acc_lds = reinterpret_cast<float*>(lds + ValuLds<D>::q_bytes + ValuLds<D>::p_bytes);
    // V as pairs of neighbouring keys per head-dim element (the transposition the
    // matrix-core path does too), once per tile
    uint32_t vt[VW][4];
#pragma unroll
    for (int c = 0; c < VW; ++c)
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            const uint32_t w0 = t.v[2 * pr][c >> 1];
            const uint32_t w1 = t.v[2 * pr + 1][c >> 1];
            vt[c][pr] = (c & 1) ? pair_hi(w0, w1) : pair_lo(w0, w1);
        }
#pragma unroll 1
    for (int q = 0; q < k; ++q) {                        // wave-uniform trip count
        float acc[VW];
        float* const my_acc = acc_lds + (q * kWave + lane) * VW;
#pragma unroll
        for (int c = 0; c < VW; c += 4) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(my_acc + c);
            acc[c] = a[0]; acc[c + 1] = a[1]; acc[c + 2] = a[2]; acc[c + 3] = a[3];
        }
        float pa = 0.f, pb = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const u32x4 qv = *reinterpret_cast<const u32x4*>(q_lds + q * (D * 2) + s * 64 + g * 16);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                pa = dot2(ET{}, t.ka[s][w], qv[w], pa);
                pb = dot2(ET{}, t.kb[s][w], qv[w], pb);
            }
        }
        pa = quad_sum(pa) * scale_log2;
        pb = quad_sum(pb) * scale_log2;
        if (MASKED) {
            const int vis = NEW ? min(k, q + 1) : lim;
            if (n >= vis) pa = -INFINITY;
            if (16 + n >= vis) pb = -INFINITY;
        }
        // the 16 lanes of a row hold different keys, the four rows hold copies: after the
        // row reductions every lane holds the same max and sum
        const float m_old = lane_get(st.m, q);
        const float m_new = fmaxf(m_old, row16_max(fmaxf(pa, pb)));
        const float alpha = fast_exp2(m_old - m_new);
        pa = fast_exp2(pa - m_new);
        pb = fast_exp2(pb - m_new);
        const float l_new = lane_get(st.l, q) * alpha + row16_sum(pa + pb);
        st.m = lane_set(st.m, q, m_new, lane);
        st.l = lane_set(st.l, q, l_new, lane);
        if (g == 0) {
            p_hi[n] = (uint16_t)pack2(ET{}, pa, 0.f);
            p_hi[16 + n] = (uint16_t)pack2(ET{}, pb, 0.f);
            if (kSplitP) {
                p_lo[n] = (uint16_t)pack2(ET{}, pa - round16(ET{}, pa), 0.f);
                p_lo[16 + n] = (uint16_t)pack2(ET{}, pb - round16(ET{}, pb), 0.f);
            }
        }
        const u32x2 h0 = *reinterpret_cast<const u32x2*>(p_hi + 4 * g);
        const u32x2 h1 = *reinterpret_cast<const u32x2*>(p_hi + 16 + 4 * g);
        u32x2 l0 = {0u, 0u}, l1 = {0u, 0u};
        if (kSplitP) {
            l0 = *reinterpret_cast<const u32x2*>(p_lo + 4 * g);
            l1 = *reinterpret_cast<const u32x2*>(p_lo + 16 + 4 * g);
        }
#pragma unroll
        for (int c = 0; c < VW; ++c) {
            float a = acc[c] * alpha;
            a = dot2(ET{}, vt[c][0], h0[0], a);
            a = dot2(ET{}, vt[c][1], h0[1], a);
            a = dot2(ET{}, vt[c][2], h1[0], a);
            a = dot2(ET{}, vt[c][3], h1[1], a);
            if (kSplitP) {
                a = dot2(ET{}, vt[c][0], l0[0], a);
                a = dot2(ET{}, vt[c][1], l0[1], a);
                a = dot2(ET{}, vt[c][2], l1[0], a);
                a = dot2(ET{}, vt[c][3], l1[1], a);
            }
            acc[c] = a;
        }
#pragma unroll
        for (int c = 0; c < VW; c += 4)
            *reinterpret_cast<f32x4*>(my_acc + c) = f32x4{acc[c], acc[c + 1], acc[c + 2], acc[c + 3]};
    }
}

// One (sample, head) pair's share of a wave's tile range; everything is wave-uniform and
// kept small, so that two of them live in scalar registers.
struct Segment {
    int i, h;            // sample, head
    int cu_i, k, k_real; // first packed row, rows, real rows (k_real < k only in the padded ablation)
    int L;               // cached keys; ceil(L/32) cache tiles, then the new-token tile
    int t0, t1;          // this wave consumes tiles [t0, t1) of the pair
    int64_t cache_off;   // byte offset of (first cache row of the sample, head h) in the arenas
    int64_t new_off;     // byte offset of (first packed row of the sample, head h) in q / k_new / v_new
    int64_t mask_off;    // padded ablation: offset of the sample's key-mask row
    __device__ __forceinline__ int ntc() const { return (L + kTileKeys - 1) / kTileKeys; }
    __device__ __forceinline__ int nt() const { return ntc() + 1; }
};

// The segment that starts at flat tile index gpos (< gend); `i` is a sample at or before it.
// `stash`: the workgroup's LDS copy of cu_seqlens [B+1], kv_len [B] and kv_start [B], or nullptr
// (large batches, padded ablation: the arrays are read from global memory then).
template <int D, bool PADDED>
__device__ __forceinline__ Segment make_segment(const AttnParams& p, const int32_t* prefix,
                                                const int32_t* stash, int i, int gpos, int gend) {
    Segment s;
    while (uniform(prefix[i + 1]) <= gpos) ++i;
    s.i = i;
    int cu0 = 0, cu1 = 0, len = 0, start32 = 0;
    if (!PADDED) {
        if (stash != nullptr) {
            cu0 = uniform(stash[i]);
            cu1 = uniform(stash[i + 1]);
            len = uniform(stash[p.B + 1 + i]);
            start32 = uniform(stash[2 * p.B + 1 + i]);
        } else {
            cu0 = uniform(p.cu[i]);
            cu1 = uniform(p.cu[i + 1]);
            len = uniform(p.kv_len[i]);
            start32 = uniform(p.kv_start[i]);
        }
    }
    // padded ablation: k_max rows and l_pad aligned cache rows for every sample
    s.cu_i = PADDED ? i * p.k_max : cu0;
    // (never more than the 16 rows one MFMA tile holds, whatever cu_seqlens claims)
    s.k = min(kMaxRows, PADDED ? p.k_max : cu1 - cu0);
    s.L = PADDED ? p.l_pad : len;
    const int64_t start = PADDED ? (int64_t)i * p.cap : (int64_t)start32;
    s.k_real = PADDED ? uniform(p.k_valid[i]) : s.k;
    const int nt = s.nt();
    const int rem = gpos - uniform(prefix[i]);
    s.h = uniform(rem / nt);
    s.t0 = rem - s.h * nt;
    s.t1 = min(nt, s.t0 + (gend - gpos));
    s.cache_off = start * p.row_stride_b + (int64_t)s.h * p.head_stride_b;
    s.new_off = ((int64_t)s.cu_i * p.H + s.h) * (D * 2);
    s.mask_off = PADDED ? (int64_t)i * p.cap : 0;
    return s;
}

// The segment after `c` in the wave's range; it starts at flat tile gpos (< gend), the first
// tile of the next pair.  The next head of the same sample needs no memory access at all;
// only a change of sample reads the index arrays again.
template <int D, bool PADDED>
__device__ __forceinline__ Segment next_segment(const AttnParams& p, const int32_t* prefix,
                                                const int32_t* stash, const Segment& c, int gpos, int gend) {
    if (c.h + 1 >= p.H) return make_segment<D, PADDED>(p, prefix, stash, c.i + 1, gpos, gend);
    Segment s = c;
    s.h = c.h + 1;
    s.t0 = 0;
    s.t1 = min(c.nt(), gend - gpos);
    s.cache_off = c.cache_off + p.head_stride_b;
    s.new_off = c.new_off + D * 2;
    return s;
}

// LDS after the tile prefix sums: the parked partials of waves 1..3 and one word of flags per wave.
template <int D> constexpr size_t fold_lds_bytes() {
    return (size_t)(kWavesPerBlock - 1) * FoldSlot<D>::floats * sizeof(float) + kWavesPerBlock * sizeof(int32_t);
}

template <typename ET, int D, bool PADDED, bool VALU = false>
__global__ __launch_bounds__(kAttnThreads, 1) void verify_attention_kernel(AttnParams p) {
    extern __shared__ int32_t prefix[];
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    static_assert(!(VALU && PADDED), "the vector-ALU formulation exists for the unpadded layout only");
    static_assert(!(VALU && D == 80), "the vector-ALU formulation exists for head dims 64 and 128 only");
    typedef TileRegs<D> TR;
    // Tile counts per sample and, for batches that fit, the index arrays themselves into LDS: one
    // round trip to memory for everything a wave will ever need to know about the batch's shape.
    int32_t* const stash_w = attn_stash_lds_bytes(p.B, PADDED || VALU) != 0
                                 ? reinterpret_cast<int32_t*>(reinterpret_cast<char*>(prefix) + attn_prefix_lds_bytes(p.B))
                                 : nullptr;
    const int32_t* const stash = stash_w;
    if (PADDED || stash_w == nullptr) {
        build_tile_prefix<PADDED ? kPaddedLine : kPlainLine>(p, prefix);
    } else {
        for (int i = threadIdx.x; i < p.B; i += blockDim.x) {
            const int c0 = p.cu[i], c1 = p.cu[i + 1], len = p.kv_len[i], start = p.kv_start[i];
            prefix[i + 1] = p.H * tiles_of_sample(c1 - c0, len);
            stash_w[i] = c0;
            if (i == p.B - 1) stash_w[p.B] = c1;
            stash_w[p.B + 1 + i] = len;
            stash_w[2 * p.B + 1 + i] = start;
        }
        if (threadIdx.x == 0) prefix[0] = 0;
        scan_tile_counts(prefix, p.B);
    }
    if (blockIdx.x == 0)       // the merge kernel reads the tile prefix from the workspace header
        for (int i = threadIdx.x; i <= p.B; i += blockDim.x) p.ws_header[i] = prefix[i];
    const int total = prefix[p.B];
    const int wave = uniform((int)(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)));
    // (a line of fewer tiles than waves is cut for as many waves as it has tiles, so that the
    // waves that hold tiles are always the first ones, with no empty range in between)
    const int num_waves = min(p.num_waves, total);
    const LineCut cut(total, max(num_waves, 1));
    const int gbeg = wave < num_waves ? uniform(cut.begin(wave)) : 0;
    const int gend = wave < num_waves ? uniform(cut.begin(wave + 1)) : 0;
    const int lane = threadIdx.x & 63;
    const int n = lane & 15;       // query row (MFMA column) of this lane
    const int g = lane >> 4;       // which quarter of the k-slots / key rows
    // In-workgroup merge (matrix-core builds): after the prefix sums, LDS holds one parked
    // partial per wave 1..3 (the state registers as they are, lane by lane) and a word of
    // flags per wave: bit 0 = this wave parked the partial of the pair it continues, bit 1 =
    // that pair ends inside this wave's range.
    const int lw = uniform((int)(threadIdx.x >> 6));
    float* const fold_lds = reinterpret_cast<float*>(reinterpret_cast<char*>(prefix) + attn_index_lds_bytes(p.B, PADDED || VALU));
    int32_t* const fold_flags = reinterpret_cast<int32_t*>(fold_lds + (kWavesPerBlock - 1) * FoldSlot<D>::floats);
    const bool wg_fold = !VALU && p.wg_fold != 0;      // (the host leaves it off for very short walks)
    if (wg_fold && lane == 0) fold_flags[lw] = 0;
    if (gbeg >= gend) {            // (only when the line has fewer tiles than there are waves) nothing to walk, nothing to merge
        if (wg_fold) __syncthreads();
        return;
    }
    const uint32_t new_row_bytes = (uint32_t)p.H * (D * 2);
    const uint32_t cache_row_bytes = (uint32_t)p.row_stride_b;

    // sample of the first tile: prefix[i] <= gbeg < prefix[i+1]
    int lo = 0, hi = p.B;          // invariant: prefix[lo] <= gbeg < prefix[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (prefix[mid] <= gbeg) lo = mid; else hi = mid;
    }

    // The wave walks its flat tile range [gbeg, gend).  `cur` is the pair being consumed,
    // `nxt` the one after it (its index arrays are fetched a whole segment ahead); the loads
    // of flat tile c+1 -- possibly the first tile of `nxt` -- are issued before tile c is
    // consumed, so the stream of loads does not drain at a pair boundary.
    Segment cur = make_segment<D, PADDED>(p, prefix, stash, uniform(lo), gbeg, gend);
    int cur_end = gbeg + (cur.t1 - cur.t0);            // flat index one past cur's last tile
    Segment nxt = cur;
    if (cur_end < gend) nxt = next_segment<D, PADDED>(p, prefix, stash, cur, cur_end, gend);

    u32x4 qb[KS];                // Q^T of `cur` as the B operand of S^T = K Q^T
    u32x4 qn[KS];                // the same for `nxt`, fetched a whole segment ahead
    SoftmaxState<ET, D> st;
    int vis_new = 0;             // this lane's row: visible keys of the new-token tile, one bit per key
    int par_n = -1;              // token trees: parent of row n of `nxt`, fetched with its Q
    // vector-ALU formulation: per-row state in registers, Q rows and P in wave-private LDS
    ValuState vs;
    char* const vlds = reinterpret_cast<char*>(prefix) + attn_index_lds_bytes(p.B, PADDED || VALU) +
                       (threadIdx.x >> 6) * ValuLds<D>::bytes;
    float* const acc_lds = reinterpret_cast<float*>(vlds + ValuLds<D>::q_bytes + ValuLds<D>::p_bytes);

    // Q rows of a pair (k rows at qaddr), raw: rows beyond k repeat row k-1 and are zeroed
    // by use_q when the pair becomes current -- touching the values here would make the wave
    // wait for the load (and for every tile load issued before it) at once.
    auto load_q = [&](u32x4* dst, int64_t new_off, int k) __attribute__((always_inline)) {
        const uint64_t qaddr = uniform_addr(p.q + new_off);
        const uint32_t qoff = (uint32_t)min(n, k - 1) * new_row_bytes;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) dst[ks] = gload<u32x4>(qaddr, qoff + TR::piece(ks, g));
    };
    auto load_parent = [&](int cu_i, int k) __attribute__((always_inline)) {
        if (!PADDED && p.parent != nullptr)
            par_n = gload<int32_t>(uniform_addr(p.parent + cu_i), (uint32_t)min(n, k - 1) * 4u);
    };
    auto use_q = [&](const u32x4* src, int k) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            if (VALU)    // lane (n, g) holds Q[n][32ks + 8g .. +8): the LDS image is row-major Q
                *reinterpret_cast<u32x4*>(vlds + n * (D * 2) + ks * 64 + g * 16) = src[ks];
            else
                qb[ks] = (n < k && TR::piece_valid(ks, g)) ? src[ks] : z;
        }
    };

    auto begin_segment = [&](const Segment& s) __attribute__((always_inline)) {
        if (VALU) {
            vs.m = -INFINITY;
            vs.l = 0.f;
            for (int q = 0; q < s.k; ++q)
#pragma unroll
                for (int c = 0; c < VW; c += 4)
                    *reinterpret_cast<f32x4*>(acc_lds + (q * kWave + lane) * VW + c) = f32x4{0.f, 0.f, 0.f, 0.f};
            return;
        }
#pragma unroll
        for (int c = 0; c < VW; ++c) st.acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.m = -INFINITY;
        st.l = 0.f;
        // visible keys of the new-token tile for this lane's row: itself and the rows before
        // it (padded: rows and keys at or beyond k_real are padding; padding rows see the real keys);
        // in a token tree: itself and its ancestors
        vis_new = (1 << min(s.k_real, n + 1)) - 1;
        if (!PADDED && p.parent != nullptr) vis_new = tree_visibility(par_n, n, s.k);
    };

    // Loads of tile `tile` of a pair described by plain values (never by a pointer to a
    // Segment, so that both segments stay in scalar registers).
    auto issue = [&](TileRegs<D>& t, int tile, int L, int k, int64_t cache_off, int64_t new_off,
                     int64_t mask_off) __attribute__((always_inline)) {
        TileSrc src;
        const bool is_new = tile >= (L + kTileKeys - 1) / kTileKeys;   // wave-uniform
        src.kbase = uniform_addr(is_new ? p.k_new + new_off : p.k_cache + cache_off);
        src.vbase = uniform_addr(is_new ? p.v_new + new_off : p.v_cache + cache_off);
        src.row_bytes = is_new ? new_row_bytes : cache_row_bytes;
        src.n0 = is_new ? 0 : tile * kTileKeys;
        src.last = is_new ? k - 1 : L - 1;
        src.mask_base = (PADDED && !is_new) ? uniform_addr(p.key_mask + mask_off) : 0;
        load_tile<D, PADDED>(t, src, n, g);
    };

    auto consume = [&](const TileRegs<D>& t, const Segment& s, int tile) __attribute__((always_inline)) {
        if (tile < s.ntc()) {
            const int lim = s.L - tile * kTileKeys;
            if (VALU) {
                if (lim >= kTileKeys)
                    valu_tile<ET, D, false, false>(t, vlds, vs, p.scale_log2, s.k, lim, lane, n, g);
                else
                    valu_tile<ET, D, true, false>(t, vlds, vs, p.scale_log2, s.k, lim, lane, n, g);
            } else if (lim >= kTileKeys && !PADDED)
                compute_tile<ET, D, false>(t, qb, st, p.scale_log2, lim, g);
            else
                compute_tile<ET, D, true, PADDED>(t, qb, st, p.scale_log2, lim, g);
        } else {
            if (VALU)
                valu_tile<ET, D, true, true>(t, vlds, vs, p.scale_log2, s.k, 0, lane, n, g);
            else
                compute_tile<ET, D, true, PADDED, true>(t, qb, st, p.scale_log2, vis_new, g);
            if (!PADDED && p.write_through) {
                // Paper order (Sec. 3.2): the new rows' K/V go to the sample's own location,
                // cache rows kv_len + j, j < k_i, straight from the registers of this tile.
                // Exactly one wave holds the new-token tile of a (sample, head) pair.
                const uint32_t row_b = cache_row_bytes;
                if (n < s.k) {
                    char* kdst = const_cast<char*>(p.k_cache) + s.cache_off + (uint64_t)(uint32_t)(s.L + n) * row_b;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        if (TR::piece_valid(ks, g))
                            *reinterpret_cast<u32x4*>(kdst + TR::piece(ks, g)) = t.ka[ks];
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = 4 * g + e;
                    if (key < s.k && n < TR::kVLanes) {
                        char* vdst = const_cast<char*>(p.v_cache) + s.cache_off + (uint64_t)(uint32_t)(s.L + key) * row_b + n * (VW * 2);
                        *reinterpret_cast<typename TileRegs<D>::vrow_t*>(vdst) = t.v[e];
                    }
                }
            }
        }
    };

    // vector-ALU formulation: reduce the shares over lanes, then the same outputs / partials
    auto finish_segment_valu = [&](const Segment& s) __attribute__((always_inline)) {
        const bool whole = s.t0 == 0 && s.t1 == s.nt();
        const int slot = 2 * wave + (s.t0 == 0 ? 1 : 0);
#pragma unroll 1
        for (int q = 0; q < s.k; ++q) {
            {
                const float l = lane_get(vs.l, q);
                float o[VW];
#pragma unroll
                for (int c = 0; c < VW; c += 4) {
                    const f32x4 a = *reinterpret_cast<const f32x4*>(acc_lds + (q * kWave + lane) * VW + c);
                    o[c] = quad_sum(a[0]); o[c + 1] = quad_sum(a[1]);
                    o[c + 2] = quad_sum(a[2]); o[c + 3] = quad_sum(a[3]);
                }
                if (g == 0) {
                    if (whole) {
                        const float inv = 1.0f / l;
                        const int64_t idx = ((int64_t)(s.cu_i + q) * p.H + s.h) * D + n * VW;
                        if (p.out_f32) {
                            float* dst = reinterpret_cast<float*>(p.out) + idx;
#pragma unroll
                            for (int c = 0; c < VW; c += 4)
                                *reinterpret_cast<f32x4*>(dst + c) =
                                    f32x4{o[c] * inv, o[c + 1] * inv, o[c + 2] * inv, o[c + 3] * inv};
                        } else {
                            typename TileRegs<D>::vrow_t pk;
#pragma unroll
                            for (int c = 0; c < VW; c += 2) pk[c >> 1] = pack2(ET{}, o[c] * inv, o[c + 1] * inv);
                            *reinterpret_cast<typename TileRegs<D>::vrow_t*>(
                                reinterpret_cast<uint16_t*>(p.out) + idx) = pk;
                        }
                    } else {
                        float* dst = p.ws + ((int64_t)slot * 16 + q) * (D + kPartialPad);
#pragma unroll
                        for (int c = 0; c < VW; c += 4)
                            *reinterpret_cast<f32x4*>(dst + n * VW + c) = f32x4{o[c], o[c + 1], o[c + 2], o[c + 3]};
                        if (n == 0) {
                            dst[D] = lane_get(vs.m, q);
                            dst[D + 1] = l;
                        }
                    }
                }
            }
        }
    };

    // `st` normalised into out[cu_i + n, h, :]
    auto write_out = [&](const Segment& s) __attribute__((always_inline)) {
        // the four lanes of a query row hold disjoint shares of the sum
        const float l = quad_sum(st.l);
        if (n < s.k) {
            const float inv = 1.0f / l;
            const int64_t row = ((int64_t)(s.cu_i + n) * p.H + s.h) * D;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (4 * g + r >= TR::kVLanes) continue;      // head dim 80: output rows 10..15 hold nothing
                const int d0 = (4 * g + r) * VW;
                float o[VW];
#pragma unroll
                for (int c = 0; c < VW; ++c) o[c] = st.acc[c][r] * inv;
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
    };
    // `st` as a partial in the workspace: slot 2w holds one that continues a pair begun by an
    // earlier wave, slot 2w+1 one that starts a pair and leaves its end to later waves
    auto write_partial = [&](const Segment& s) __attribute__((always_inline)) {
        const float l = quad_sum(st.l);
        const int slot = 2 * wave + (s.t0 == 0 ? 1 : 0);
        if (n < s.k) {
            float* dst = p.ws + ((int64_t)slot * 16 + n) * (D + kPartialPad);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (4 * g + r >= TR::kVLanes) continue;
                const int d0 = (4 * g + r) * VW;
#pragma unroll
                for (int c = 0; c < VW; c += 4)
                    *reinterpret_cast<f32x4*>(dst + d0 + c) =
                        f32x4{st.acc[c][r], st.acc[c + 1][r], st.acc[c + 2][r], st.acc[c + 3][r]};
            }
            if (g == 0) {
                dst[D] = st.m;
                dst[D + 1] = l;
            }
        }
    };

    auto finish_segment = [&](const Segment& s) __attribute__((always_inline)) {
        if (VALU) {
            finish_segment_valu(s);
            return;
        }
        const bool continues = s.t0 != 0;          // an earlier wave holds the pair's first tiles
        const bool open = s.t1 != s.nt();          // later waves hold its last tiles (then this is the wave's last segment)
        if (!continues && !open) {
            write_out(s);
        } else if (!wg_fold) {
            write_partial(s);                      // every wave's partials go to the workspace
        } else if (open && (lw == 0 || !continues)) {
            // stays in registers: after the barrier this wave folds in what the waves after it parked
        } else if (lw == 0) {
            write_partial(s);                      // the pair began in an earlier workgroup
        } else {
            float* f = fold_lds + (lw - 1) * FoldSlot<D>::floats;
#pragma unroll
            for (int c = 0; c < VW; ++c) *reinterpret_cast<f32x4*>(f + (c * kWave + lane) * 4) = st.acc[c];
            f[FoldSlot<D>::m_at + lane] = st.m;
            f[FoldSlot<D>::l_at + lane] = st.l;
            if (lane == 0) fold_flags[lw] = 1 | (open ? 0 : 2);
        }
    };

    int con_t = cur.t0;              // tile of `cur` that is consumed next

    // One step of the walk: issue flat tile c+1 into `fill`, consume flat tile c from `use`.
    auto step = [&](int c, const TileRegs<D>& use, TileRegs<D>& fill) __attribute__((always_inline)) {
        if (c + 1 < gend) {
            const bool same = con_t + 1 < cur.t1;        // else: first tile of the next pair
            issue(fill, same ? con_t + 1 : nxt.t0, same ? cur.L : nxt.L, same ? cur.k : nxt.k,
                  same ? cur.cache_off : nxt.cache_off, same ? cur.new_off : nxt.new_off,
                  same ? cur.mask_off : nxt.mask_off);
        }
        consume(use, cur, con_t);
        ++con_t;
        if (con_t == cur.t1) {
            finish_segment(cur);
            if (c + 1 < gend) {
                cur = nxt;
                con_t = cur.t0;
                cur_end = c + 1 + (cur.t1 - cur.t0);
                use_q(qn, cur.k);
                begin_segment(cur);
                if (cur_end < gend) {
                    nxt = next_segment<D, PADDED>(p, prefix, stash, cur, cur_end, gend);
                    load_q(qn, nxt.new_off, nxt.k);
                    load_parent(nxt.cu_i, nxt.k);
                }
            }
        }
    };

    TileRegs<D> ta, tb;
    load_q(qn, cur.new_off, cur.k);
    load_parent(cur.cu_i, cur.k);
    use_q(qn, cur.k);
    begin_segment(cur);
    if (cur_end < gend) {
        load_q(qn, nxt.new_off, nxt.k);
        load_parent(nxt.cu_i, nxt.k);
    }
    issue(ta, cur.t0, cur.L, cur.k, cur.cache_off, cur.new_off, cur.mask_off);
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
                const float* f = fold_lds + (j - 1) * FoldSlot<D>::floats;
                const float mb = f[FoldSlot<D>::m_at + lane];
                const float lb = f[FoldSlot<D>::l_at + lane];
                const float mn = fmaxf(st.m, mb);
                // (padded ablation: a range of nothing but padding keys has max -inf and sum 0)
                const float ms = mn == -INFINITY ? 0.f : mn;
                const float ea = fast_exp2(st.m - ms), eb = fast_exp2(mb - ms);
#pragma unroll
                for (int c = 0; c < VW; ++c)
                    st.acc[c] = st.acc[c] * ea + *reinterpret_cast<const f32x4*>(f + (c * kWave + lane) * 4) * eb;
                st.l = st.l * ea + lb * eb;
                st.m = mn;
                complete = (flags & 2) != 0;
            }
            if (complete && !continues)
                write_out(cur);
            else
                write_partial(cur);
        }
    }
}

// Merge the partials of every (sample, head) pair whose tiles were shared by several
// waves.  Grid (H, B); 8 x D/4 threads: D/4 lanes per output row, 4 columns per lane, 8 rows
// per pass (most blocks find nothing to merge and leave at once; one-wave blocks were tried and
// ran slower, 6.3 vs 4.4 us: the few blocks that do merge then take more passes).
// The slots of a pair are folded in wave order into a running
// (max, sum, accumulator), so the result does not depend on timing; a slot's loads do not
// depend on the running state, so two slots are fetched before either is folded.
template <int D> struct Combine {
    static constexpr int lanes_per_row = D / 4;
    static constexpr int rows_per_pass = 8;
    static constexpr int threads = rows_per_pass * lanes_per_row;
};

template <typename ET, int D, bool PADDED>
__global__ __launch_bounds__(Combine<D>::threads) void combine_partials_kernel(AttnParams p) {
    const int i = blockIdx.y, h = blockIdx.x;
    const int cu_i = PADDED ? i * p.k_max : p.cu[i];
    const int k = min(kMaxRows, PADDED ? p.k_max : p.cu[i + 1] - cu_i);
    const int total = p.ws_header[p.B];
    const int first = p.ws_header[i];
    const int next = p.ws_header[i + 1];
    if (k <= 0) return;
    const int num_waves = min(p.num_waves, total);     // (as the attention kernel cuts the line)
    const int nt = (next - first) / p.H;
    const int g0 = first + h * nt;
    const LineCut cut(total, max(num_waves, 1));
    const int w0 = cut.wave_of(g0), w1 = cut.wave_of(g0 + nt - 1);
    if (w0 == w1) return;                  // one wave saw the whole pair and wrote `out` itself
    // With the in-workgroup merge only the first wave of the pair and the first wave of every
    // later workgroup it reaches have written a slot; a pair inside one workgroup is done.
    const int wstep = p.wg_fold ? kWavesPerBlock : 1;
    if (p.wg_fold && w0 / kWavesPerBlock == w1 / kWavesPerBlock) return;
    const int wsecond = p.wg_fold ? (w0 / kWavesPerBlock + 1) * kWavesPerBlock : w0 + 1;
    constexpr int pitch = D + kPartialPad;
    constexpr int lanes_per_row = Combine<D>::lanes_per_row;
    const int c4 = (threadIdx.x % lanes_per_row) * 4;
    for (int j = threadIdx.x / lanes_per_row; j < k; j += Combine<D>::rows_per_pass) {
        // slot of wave w for this pair: 2w+1 if the pair starts in w's range, 2w if it continues
        auto slot_row = [&](int w) -> const float* {
            const int slot = 2 * w + (w == w0 ? 1 : 0);
            return p.ws + ((int64_t)slot * 16 + j) * pitch;
        };
        float M = -INFINITY, den = 0.f;
        f32x4 num = {0.f, 0.f, 0.f, 0.f};
        auto fold = [&](float m, float l, f32x4 v) {
            const float Mn = fmaxf(M, m);
            // (padded ablation: a range of nothing but padding keys has max -inf and sum 0)
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
        const int64_t idx = ((int64_t)(cu_i + j) * p.H + h) * D + c4;
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

template <typename ET, int D, bool PADDED>
static hipError_t launch_typed(const AttnParams& params, int blocks, bool valu, hipStream_t stream,
                               hipEvent_t ev_start, hipEvent_t ev_stop) {
    valu = valu && !PADDED && D != 80;      // the vector-ALU formulation exists for these only
    AttnParams p = params;
    if (valu) p.wg_fold = 0;
    size_t lds = attn_index_lds_bytes(p.B, PADDED || valu);     // (the vector-ALU build needs its LDS for per-row state)
    hipError_t e;
    if (ev_start && (e = hipEventRecord(ev_start, stream)) != hipSuccess) return e;
    bool launched = false;
    if (p.wg_fold) lds += fold_lds_bytes<D>();     // at most 32 KiB of tile prefix (24 KiB of index arrays) + 26 KiB
    if constexpr (!PADDED && D != 80) {
        if (valu) {
            lds += (size_t)kWavesPerBlock * ValuLds<D>::bytes;
            // prefix sums + 4 x 36 KiB (D = 128) of wave-private state: well above the 64 KiB a
            // kernel may use by default on some HIP platforms, so ask for the device's 160 KiB
            if (lds > kMaxLdsBytes) return hipErrorInvalidValue;   // (the API layer rejects such B first)
            static std::atomic<uint64_t> raised{0};
            e = allow_max_lds(reinterpret_cast<const void*>(&verify_attention_kernel<ET, D, false, true>), raised);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((verify_attention_kernel<ET, D, false, true>), dim3(blocks),
                               dim3(kAttnThreads), lds, stream, p);
            launched = true;
        }
    }
    if (!launched)
        hipLaunchKernelGGL((verify_attention_kernel<ET, D, PADDED, false>), dim3(blocks),
                           dim3(kAttnThreads), lds, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev_stop && (e = hipEventRecord(ev_stop, stream)) != hipSuccess) return e;
    hipLaunchKernelGGL((combine_partials_kernel<ET, D, PADDED>), dim3(p.H, p.B),
                       dim3(Combine<D>::threads), 0, stream, p);
    return hipGetLastError();
}

template <bool PADDED>
static hipError_t launch_layout(const AttnParams& p, int blocks, int D, bool bf16, bool valu,
                                hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    if (D == 128) return bf16 ? launch_typed<BF16, 128, PADDED>(p, blocks, valu, stream, ev_start, ev_stop)
                              : launch_typed<F16, 128, PADDED>(p, blocks, valu, stream, ev_start, ev_stop);
    if constexpr (!PADDED) {
        if (D == 80) return bf16 ? launch_typed<BF16, 80, false>(p, blocks, false, stream, ev_start, ev_stop)
                                 : launch_typed<F16, 80, false>(p, blocks, false, stream, ev_start, ev_stop);
    }
    return bf16 ? launch_typed<BF16, 64, PADDED>(p, blocks, valu, stream, ev_start, ev_stop)
                : launch_typed<F16, 64, PADDED>(p, blocks, valu, stream, ev_start, ev_stop);
}

size_t valu_attention_lds_bytes(int B, int D) {
    return attn_index_lds_bytes(B, true) + (size_t)kWavesPerBlock * (D == 128 ? ValuLds<128>::bytes : ValuLds<64>::bytes);
}

hipError_t launch_verify_attention(const AttnParams& p, int blocks, int D, bool bf16, bool padded,
                                   bool valu, hipStream_t stream, hipEvent_t ev_start,
                                   hipEvent_t ev_stop) {
    if (!padded && p.multi) return launch_verify_attention_wide(p, blocks, D, bf16, stream, ev_start, ev_stop);
    return padded ? launch_layout<true>(p, blocks, D, bf16, false, stream, ev_start, ev_stop)
                  : launch_layout<false>(p, blocks, D, bf16, valu, stream, ev_start, ev_stop);
}

}  // namespace ems