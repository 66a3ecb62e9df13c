// Packed multi-token attention for samples that bring 17..64 rows per step (token trees commonly
// have 32-64 nodes), head dims 80 and 128: the tiles of the cache are STAGED through LDS by waves
// that do nothing else, and consumed there by waves that never touch memory.
//
// Why: a wave that holds a pair's rows in registers (verify_attention.hip: 16 rows; the one-wave
// forms of verify_attention_wide.hip: 32, or 64 with half of them parked) issues its own loads,
// and on this machine a load instruction blocks the wave that issues it for as long as the memory
// pipeline is full -- which, in a kernel that is meant to keep it full, is most of the time
// (measured: a wave that asks for a quarter of a 16 KiB tile sits 0.7 us in those four
// instructions).  With 16 rows there is little arithmetic to delay; with 32 or 64 rows the wave's
// arithmetic is as long as the tile's transfer and the two add up instead of overlapping.
// Here a workgroup walks TWO streams of tiles (the tile line is cut for two streams per
// workgroup).  Per stream:
//   * one requesting wave asks for tile after tile with direct loads (global_load ... lds: memory
//     to LDS without passing through registers; each lane's 16 bytes land in its own slot) into a
//     ring of four tiles, as fast as the memory pipeline takes them; it waits only for a free
//     ring slot, and tells through a counter in LDS which tiles have landed (its loads
//     complete in order, so "at most one tile's loads outstanding" means the tile before landed);
//   * four computing waves, one per SIMD, each keep ONE block of 16 rows of the pair: Q^T in
//     registers, the tile's K and V pieces read from LDS in MFMA operand layout, online softmax
//     and accumulators as in the 16-row kernel; each tells through its own counter which tiles it
//     is done with.  A pair of 17..32 rows keeps two of them busy, 33..48 three, 49..64 four.
// No barrier in the walk.  Every wave's waits end: a counter is polled a bounded number of times.
// Measured (B = 64, 2048 cached tokens per sample, H = 32, D = 128, bf16; one box, the two
// libraries one after the other; the one-wave-per-SIMD and two-waves-per-SIMD forms this one
// replaced in parentheses): 352 us at 17 rows (388), 372 at 32 (404), 399 at 33 (464), 410 at 48
// (473), 448 at 64 (487); its loads alone (no arithmetic) take 378 us.  At 64 rows the four
// computing waves of a stream are the limit (1.7 us per tile against 1.45 us for its transfer);
// up to 48 rows the kernel runs at the rate of its loads.
// What was tried on the way (none kept): the same four-waves-per-stream split with every wave
// requesting a quarter of the tile and one barrier per tile (531 us at 64 rows: the blocked
// requests are on every wave's critical path); requesting waves in lock-step with the
// computing ones through that barrier (499); the scores of tile t + 1 computed among the
// exponentials of tile t (no gain, and slower once that tile must have landed first).
#include "attention_tiles.h"

namespace ems {

// A (sample, head) pair's share of a stream's tile range (wave-uniform).  A pair has all the rows
// of its sample (at most row_cap), ceil(L/32) cache tiles and then ceil(rows/32) tiles of new rows.
struct StagedSegment {
    int i, h;            // sample, head
    int cu_i, ktot, k;   // first packed row of the sample; its rows (k == ktot: one pair per head)
    int L;               // cached keys
    int t0, t1;          // the stream consumes tiles [t0, t1) of the pair
    int64_t cache_off;   // byte offset of (first cache row of the sample, head h) in the arenas
    int64_t new_off;     // byte offset of (first packed row of the sample, head h) in q / k_new / v_new
    __device__ __forceinline__ int ntc() const { return (L + kTileKeys - 1) / kTileKeys; }
    __device__ __forceinline__ int nt() const { return ntc() + new_tiles(ktot); }
};

__device__ __forceinline__ int staged_tiles_of_sample(int k, int L) {
    return k > 0 ? (L + kTileKeys - 1) / kTileKeys + new_tiles(k) : 0;
}

template <int D>
__device__ __forceinline__ StagedSegment make_staged_segment(const AttnParams& p, const int32_t* prefix, int i,
                                                             int gpos, int gend, int row_cap) {
    StagedSegment s;
    while (uniform(prefix[i + 1]) <= gpos) ++i;
    s.i = i;
    s.cu_i = uniform(p.cu[i]);
    s.ktot = s.k = min(row_cap, uniform(p.cu[i + 1]) - s.cu_i);   // (never more than the kernel holds)
    s.L = uniform(p.kv_len[i]);
    const int64_t start = (int64_t)uniform(p.kv_start[i]);
    const int nt = s.nt();
    const int rem = gpos - uniform(prefix[i]);
    s.h = uniform(rem / nt);
    s.t0 = rem - s.h * nt;
    s.t1 = min(nt, s.t0 + (gend - gpos));
    s.cache_off = start * p.row_stride_b + (int64_t)s.h * p.head_stride_b;
    s.new_off = ((int64_t)s.cu_i * p.H + s.h) * (D * 2);
    return s;
}

// the segment after c, which ends at line position gpos: the sample's next head, or the next sample
template <int D>
__device__ __forceinline__ StagedSegment next_staged_segment(const AttnParams& p, const int32_t* prefix,
                                                             const StagedSegment& c, int gpos, int gend, int row_cap) {
    if (c.h + 1 >= p.H) return make_staged_segment<D>(p, prefix, c.i + 1, gpos, gend, row_cap);
    StagedSegment s = c;
    s.h = c.h + 1;
    s.t0 = 0;
    s.t1 = min(c.nt(), gend - gpos);
    s.cache_off = c.cache_off + p.head_stride_b;
    s.new_off = c.new_off + D * 2;
    return s;
}

// One 32-key tile in LDS, one 16-byte slot per lane (so every access is 64 consecutive slots):
// 2 KS slot rows of K pieces (keys n and 16 + n of lane (n, g)), then 8 slot rows of V pieces --
// the per-lane layout in which the 16-row kernel loads a tile into registers.
template <int D> struct StagedTile {
    static_assert(TileRegs<D>::VW == 8, "V pieces of 16 bytes");
    static constexpr int k_slots = 2 * TileRegs<D>::KS;
    static constexpr int v_slots = 8;
    static constexpr int slots = (k_slots + v_slots) * kWave;         // in 16-byte units
    static constexpr int bytes = slots * (int)sizeof(u32x4);
};

// 16 bytes per lane from memory (base + this lane's offset) into 64 consecutive LDS slots starting
// at `dst` (wave-uniform), lane l into slot l; non-temporal like the register loads of the
// cache.  Completion is counted like any load of the wave (vmcnt).
__device__ __forceinline__ void load_to_lds(uint64_t base, uint32_t off, u32x4* dst) {
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const __attribute__((address_space(1))) void*>(base + off),
                                     (__attribute__((address_space(3))) void*)dst, 16, 0, 2 /* nt */);
}

// One staged tile against one block of 16 rows; kt / vt: this lane's slot in the tile's first K / V
// slot row; vis: bit j set = this lane's row sees key j of the tile.  The V pieces are requested
// from LDS before the scores are computed, so that they have arrived when the softmax is done;
// tiles every key of which every row sees (all but a pair's last cache tile and its tiles of new
// rows) skip the masking; the two products of a bf16 P (hi, lo) into one accumulator are kept two
// matrix instructions apart.
template <typename ET, int D>
__device__ __forceinline__ void compute_tile_one(const u32x4* kt, const u32x4* vt, const u32x4* q,
                                                 SoftmaxState<ET, D>& st, float scale_log2, uint32_t vis, int g) {
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    constexpr bool kSplitP = PSplit<ET>::value;
    u32x4 k[2 * KS], v[8];
#pragma unroll
    for (int s = 0; s < 2 * KS; ++s) k[s] = kt[s * kWave];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = vt[e * kWave];
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        sa = mfma16x16x32(ET{}, k[s], q[s], sa);
        sb = mfma16x16x32(ET{}, k[KS + s], q[s], sb);
    }
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[i] = sa[i] * scale_log2;
        x[4 + i] = sb[i] * scale_log2;
    }
    if (__builtin_amdgcn_ballot_w64(vis != ~0u) != 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (((vis >> (4 * g + i)) & 1u) == 0) x[i] = -INFINITY;
            if (((vis >> (16 + 4 * g + i)) & 1u) == 0) x[4 + i] = -INFINITY;
        }
    }
    const float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                           fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    // lazy running reference: it moves only when a tile exceeds it by more than 2^kMaxSlack, so the
    // accumulators are almost never rescaled after a row's first tiles
    const float m_tile = quad_max(mx);
    const float m_new = m_tile > st.m + kMaxSlack ? m_tile : st.m;
    const float m_sub = m_new == -INFINITY ? 0.f : m_new;   // nothing visible yet
    const float alpha = fast_exp2(st.m - m_sub);
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        x[i] = fast_exp2(x[i] - m_sub);
        psum += x[i];
    }
    st.l = st.l * alpha + psum;
    st.m = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int c = 0; c < VW; ++c) st.acc[c] *= alpha;
    }
    u32x4 pb, pl;
    pb[0] = pack2(ET{}, x[0], x[1]);
    pb[1] = pack2(ET{}, x[2], x[3]);
    pb[2] = pack2(ET{}, x[4], x[5]);
    pb[3] = pack2(ET{}, x[6], x[7]);
    if (kSplitP) {                           // bf16: P as hi + lo, as in the 16-row kernel
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] -= round16(ET{}, x[i]);
        pl[0] = pack2(ET{}, x[0], x[1]);
        pl[1] = pack2(ET{}, x[2], x[3]);
        pl[2] = pack2(ET{}, x[4], x[5]);
        pl[3] = pack2(ET{}, x[6], x[7]);
    }
#pragma unroll
    for (int c = 0; c < VW; c += 2) {
        u32x4 va[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                const uint32_t w0 = v[2 * pr][(c + j) >> 1];
                const uint32_t w1 = v[2 * pr + 1][(c + j) >> 1];
                va[j][pr] = ((c + j) & 1) ? pair_hi(w0, w1) : pair_lo(w0, w1);
            }
        st.acc[c] = mfma16x16x32(ET{}, va[0], pb, st.acc[c]);
        st.acc[c + 1] = mfma16x16x32(ET{}, va[1], pb, st.acc[c + 1]);
        if (kSplitP) {
            st.acc[c] = mfma16x16x32(ET{}, va[0], pl, st.acc[c]);
            st.acc[c + 1] = mfma16x16x32(ET{}, va[1], pl, st.acc[c + 1]);
        }
    }
}

constexpr int kStagedComputeWaves = 4 * kStagedStreams;     // four blocks of 16 rows per stream
constexpr int kStagedThreads = (kStagedComputeWaves + kStagedStreams) * kWave;   // + one requesting wave per stream
constexpr int kStagedRing = 4;           // tiles per stream in LDS
template <int D> constexpr size_t staged_lds_bytes(int B) {
    return ((((size_t)(B + 1) * sizeof(int32_t)) + 15) & ~(size_t)15) + (size_t)kStagedStreams * kStagedRing * StagedTile<D>::bytes +
           kStagedStreams * 8 * sizeof(int32_t);      // tile prefix sums, the rings, the streams' counters
}
// Polls of a counter before a wave stops waiting for it and goes on (about half a second; never
// reached unless another wave of the workgroup died): no wave of this kernel can wait for ever.
constexpr int kStagedSpinLimit = 1 << 22;

// wait until at most N of this wave's memory operations are outstanding (nothing else is waited for)
template <int N> __device__ __forceinline__ void wait_loads_outstanding() {
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

template <typename ET, int D>
__global__ __launch_bounds__(kStagedThreads, 1) void verify_attention_staged_kernel(AttnParams p) {
    extern __shared__ int32_t prefix[];
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    constexpr int kOps = 2 * KS + 8;              // direct loads per tile: 2 KS slot rows of K, 8 of V
    typedef TileRegs<D> TR;
    typedef StagedSegment Seg;
    typedef StagedTile<D> DT;
    typedef typename TileRegs<D>::vrow_t vrow_t;
    // per stream: tiles landed (written by the requesting wave), tiles consumed by each computing wave
    typedef volatile __attribute__((address_space(3))) int32_t lds_counter_t;
    lds_counter_t* const counters = (lds_counter_t*)(
        reinterpret_cast<char*>(prefix) + (((p.B + 1) * 4 + 15) & ~15) + (size_t)kStagedStreams * kStagedRing * StagedTile<D>::bytes);
    if (threadIdx.x < kStagedStreams * 8) counters[threadIdx.x] = 0;
    // rows a pair may have, and rows of one partial slot: 32 (the call said at most 32) or 64
    const int row_cap = kMaxRows << p.multi;
    for (int i = threadIdx.x; i < p.B; i += blockDim.x)
        prefix[i + 1] = p.H * staged_tiles_of_sample(min(p.cu[i + 1] - p.cu[i], row_cap), p.kv_len[i]);
    if (threadIdx.x == 0) prefix[0] = 0;
    scan_tile_counts(prefix, p.B);
    if (blockIdx.x == 0)       // the merge kernel reads the tile prefix from the workspace header
        for (int i = threadIdx.x; i <= p.B; i += blockDim.x) p.ws_header[i] = prefix[i];
    const int total = uniform(prefix[p.B]);
    const int per = (total + p.num_waves - 1) / p.num_waves;     // (num_waves counts streams here)
    const int lw = uniform((int)(threadIdx.x >> 6));             // 0..9
    const bool loader = lw >= kStagedComputeWaves;                 // waves 8, 9: the tiles of stream 0, 1
    const int ul = loader ? lw - kStagedComputeWaves : lw >> 2;     // stream of this wave inside the workgroup
    const int blk = lw & 3;                                       // a computing wave's block of 16 rows
    const int unit = uniform((int)(blockIdx.x * kStagedStreams + ul));
    const int gbeg = min(total, unit * per);
    const int gend = min(total, gbeg + per);
    const int lane = threadIdx.x & 63;
    const int n = lane & 15;
    const int g = lane >> 4;
    u32x4* const tiles = reinterpret_cast<u32x4*>(reinterpret_cast<char*>(prefix) + (((p.B + 1) * 4 + 15) & ~15)) +
                         ul * kStagedRing * DT::slots;
    const uint32_t new_row_bytes = (uint32_t)p.H * (D * 2);
    const uint32_t cache_row_bytes = (uint32_t)p.row_stride_b;
    const bool live = gbeg < gend;

    Seg cur, iss;                          // the pair being consumed / the pair whose tiles are being requested
    int con_t = 0, iss_t = 0, issued = gbeg;     // next tile of cur / of iss; line position of the next request
    u32x4 q[KS];                           // Q^T of this wave's block, B operand of S^T = K Q^T
    SoftmaxState<ET, D> st;
    uint64_t vis = 0;                      // this lane's row: visible new rows of the sample
    const int row_base = kMaxRows * blk;

    auto begin_segment = [&](const Seg& s) __attribute__((always_inline)) {
        const uint64_t qaddr = uniform_addr(p.q + s.new_off);
        int par = -1;
        if (p.parent != nullptr)
            par = gload<int32_t>(uniform_addr(p.parent + s.cu_i), (uint32_t)min(lane, s.ktot - 1) * 4u);
        const int row = min(row_base + n, s.ktot - 1);     // rows beyond the last repeat it, zeroed below
        const bool real = row_base + n < s.ktot;
        const uint32_t qoff = (uint32_t)row * new_row_bytes;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            const u32x4 qv = gload<u32x4>(qaddr, qoff + TR::piece(ks, g));
            q[ks] = (real && TR::piece_valid(ks, g)) ? qv : z;
        }
#pragma unroll
        for (int c = 0; c < VW; ++c) st.acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.m = -INFINITY;
        st.l = 0.f;
        vis = row >= 63 ? ~0ull : (1ull << (row + 1)) - 1;
        if (p.parent != nullptr) vis = tree_visibility64(par, lane, s.ktot, row);
    };

    // (requesting wave) tile `tile` of pair s, all its pieces, from memory straight into ring slot `buf`
    auto issue = [&](int buf, const Seg& s, int tile) __attribute__((always_inline)) {
        const int ntc = s.ntc();
        const bool is_new = tile >= ntc;                               // wave-uniform
        const uint32_t row_bytes = is_new ? new_row_bytes : cache_row_bytes;
        const int n0 = is_new ? (tile - ntc) * kTileKeys : tile * kTileKeys;
        const int last = is_new ? s.ktot - 1 : s.L - 1;
        u32x4* const kt = tiles + buf * DT::slots;
        u32x4* const vt = kt + DT::k_slots * kWave;
        const uint64_t kbase = uniform_addr(is_new ? p.k_new + s.new_off : p.k_cache + s.cache_off);
        const uint64_t vbase = uniform_addr(is_new ? p.v_new + s.new_off : p.v_cache + s.cache_off);
        const uint32_t ra = (uint32_t)min(n0 + n, last) * row_bytes;
        const uint32_t rb = (uint32_t)min(n0 + 16 + n, last) * row_bytes;
        const uint32_t vcol = (uint32_t)min(n, TR::kVLanes - 1) * (VW * 2);
#pragma unroll
        for (int o = 0; o < kOps; ++o) {
            if (o < 2 * KS) {
                const int sk = o < KS ? o : o - KS;
                load_to_lds(kbase, (o < KS ? ra : rb) + TR::piece(sk, g), kt + o * kWave);
            } else {
                const int e = o - 2 * KS;
                const int key = n0 + (e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4));
                load_to_lds(vbase, (uint32_t)min(key, last) * row_bytes + vcol, vt + e * kWave);
            }
        }
    };
    // the next tile of the range is requested, if there is one
    auto issue_next = [&]() __attribute__((always_inline)) {
        if (issued >= gend) return;
        issue((issued - gbeg) & (kStagedRing - 1), iss, iss_t);
        ++issued;
        ++iss_t;
        if (iss_t == iss.t1 && issued < gend) {
            iss = next_staged_segment<D>(p, prefix, iss, issued, gend, row_cap);
            iss_t = iss.t0;
        }
    };

    auto consume = [&](int buf, const Seg& s, int tile) __attribute__((always_inline)) {
        const u32x4* const kt = tiles + buf * DT::slots + lane;
        const u32x4* const vt = kt + DT::k_slots * kWave;
        const bool is_new = tile >= s.ntc();
        const int key0 = is_new ? kTileKeys * (tile - s.ntc()) : 0;   // first new row of a tile of new rows
        if (row_base < s.k) {                   // (else: the pair has no rows for this wave)
            const int lim = s.L - tile * kTileKeys;                     // visible keys of a cache tile
            const uint32_t cached = lim >= kTileKeys ? ~0u : (1u << max(lim, 0)) - 1u;
            const uint32_t v32 = is_new ? (uint32_t)(vis >> key0) : cached;
            compute_tile_one<ET, D>(kt, vt, q, st, p.scale_log2, v32, g);
        }
        if (!is_new) return;
        if (!p.write_through) return;
        // the paper's order (Sec. 3.2): the new rows go into the cache (rows beyond the cached length,
        // which nobody reads in this call), each computing wave a quarter of the tile's slot rows
#pragma unroll
        for (int o = 0; o < kOps; ++o) {
            if ((o & 3) != blk) continue;
            if (o < 2 * KS) {
                const int hf = o < KS ? 0 : 1, ks = o < KS ? o : o - KS;
                const int key = key0 + 16 * hf + n;
                if (key < s.ktot && TR::piece_valid(ks, g)) {
                    char* kdst = const_cast<char*>(p.k_cache) + s.cache_off + (uint64_t)(uint32_t)(s.L + key) * cache_row_bytes;
                    *reinterpret_cast<u32x4*>(kdst + TR::piece(ks, g)) = kt[o * kWave];
                }
            } else {
                const int e = o - 2 * KS;
                const int kl = e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4);
                if (key0 + kl < s.ktot && n < TR::kVLanes) {
                    char* vdst = const_cast<char*>(p.v_cache) + s.cache_off + (uint64_t)(uint32_t)(s.L + key0 + kl) * cache_row_bytes + n * (VW * 2);
                    *reinterpret_cast<u32x4*>(vdst) = vt[e * kWave];
                }
            }
        }
    };

    // this wave's block normalised into `out`, or as its rows of the stream's partial slot
    auto finish_segment = [&](const Seg& s) __attribute__((always_inline)) {
        const bool whole = s.t0 == 0 && s.t1 == s.nt();
        const int slot = 2 * unit + (s.t0 == 0 ? 1 : 0);
        const float l = quad_sum(st.l);         // the four lanes of a row hold disjoint shares
        const int r_in_pair = row_base + n;
        if (r_in_pair >= s.k) return;
        if (whole) {
            const float inv = 1.0f / l;
            const int64_t row = ((int64_t)(s.cu_i + r_in_pair) * p.H + s.h) * D;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (4 * g + r >= TR::kVLanes) continue;
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
                    vrow_t pk;
#pragma unroll
                    for (int c = 0; c < VW; c += 2) pk[c >> 1] = pack2(ET{}, o[c], o[c + 1]);
                    *reinterpret_cast<vrow_t*>(dst) = pk;
                }
            }
        } else {
            float* dst = p.ws + ((int64_t)slot * row_cap + r_in_pair) * (D + kPartialPad);
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

    if (live) {
        int lo = 0, hi = p.B;          // invariant: prefix[lo] <= gbeg < prefix[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (prefix[mid] <= gbeg) lo = mid; else hi = mid;
        }
        cur = make_staged_segment<D>(p, prefix, uniform(lo), gbeg, gend, row_cap);
        iss = cur;
        con_t = iss_t = cur.t0;
    }
    // No barrier in the walk: the requesting wave of a stream runs up to three tiles ahead of the
    // four computing waves and the two sides meet through counters in LDS.  A request blocks the
    // wave that makes it while the memory pipeline is full, which is most of the time: that is why
    // the waves that compute make none, and why the requesting wave waits for nothing else than a
    // free ring slot.
    lds_counter_t* const landed = counters + ul * 8;          // tiles of this stream that are in LDS
    lds_counter_t* const consumed = counters + ul * 8 + 1;    // [4]: tiles each computing wave is done with
    const int ntiles = gend - gbeg;
    if (loader) {
#pragma unroll 1
        for (int j = 0; j < ntiles; ++j) {
            if (j >= kStagedRing) {                          // the slot still holds tile j - 4
                int spins = 0;
                while (__builtin_amdgcn_ballot_w64(lane < 4 && consumed[lane & 3] < j - (kStagedRing - 1)) != 0 &&
                       ++spins < kStagedSpinLimit)
                    __builtin_amdgcn_s_sleep(1);
            }
            issue_next();
            if (j >= 1) {                                  // tiles up to j - 1
                wait_loads_outstanding<kOps>();
                if (lane == 0) *landed = j;
            }
        }
        wait_loads_outstanding<0>();
        if (lane == 0 && ntiles > 0) *landed = ntiles;
        return;
    }
    if (live) begin_segment(cur);
#pragma unroll 1
    for (int t = 0; t < ntiles; ++t) {
        {
            int spins = 0;
            while (*landed <= t && ++spins < kStagedSpinLimit) __builtin_amdgcn_s_sleep(1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");   // the tile is read after the counter
        consume(t & (kStagedRing - 1), cur, con_t);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // every read of the tile has returned
        if (lane == 0) consumed[blk] = t + 1;
        ++con_t;
        if (con_t == cur.t1) {
            finish_segment(cur);
            if (t + 1 < ntiles) {
                cur = next_staged_segment<D>(p, prefix, cur, gbeg + t + 1, gend, row_cap);
                con_t = cur.t0;
                begin_segment(cur);
            }
        }
    }
}

size_t staged_attention_lds_bytes(int B, int D) {
    return D == 128 ? staged_lds_bytes<128>(B) : D == 80 ? staged_lds_bytes<80>(B) : ~(size_t)0;
}

template <typename ET, int D>
static hipError_t launch_staged_typed(const AttnParams& p, int blocks, hipStream_t stream) {
    const size_t lds = staged_lds_bytes<D>(p.B);       // ~128 KiB of rings + the tile prefix sums
    if (lds > (size_t)kMaxLdsBytes) return hipErrorInvalidValue;     // (the caller asks staged_attention_lds_bytes first)
    static std::atomic<uint64_t> raised{0};
    hipError_t e = allow_max_lds(reinterpret_cast<const void*>(&verify_attention_staged_kernel<ET, D>), raised);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((verify_attention_staged_kernel<ET, D>), dim3(blocks), dim3(kStagedThreads), lds, stream, p);
    return hipGetLastError();
}

// p.num_waves counts streams (blocks * kStagedStreams); p.multi: 1 = at most 32 rows per sample
// and 32-row partial slots, 2 = at most 64 and 64-row slots.  Launches the main kernel only: the
// partials are merged by the caller's merge kernel.
hipError_t launch_verify_attention_staged(const AttnParams& p, int blocks, int D, bool bf16, hipStream_t stream) {
    if (D == 128) return bf16 ? launch_staged_typed<BF16, 128>(p, blocks, stream) : launch_staged_typed<F16, 128>(p, blocks, stream);
    if (D == 80) return bf16 ? launch_staged_typed<BF16, 80>(p, blocks, stream) : launch_staged_typed<F16, 80>(p, blocks, stream);
    return hipErrorInvalidValue;
}

}  // namespace ems
