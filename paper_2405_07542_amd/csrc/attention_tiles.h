// Device-side pieces shared by the attention kernels of libems (gfx950, wave64): the 32-key
// tile as registers, how it is loaded and consumed on the matrix cores, the per-sample tile
// counts laid on one line, and the visible-set construction for token trees.
#pragma once
#include <atomic>

#include "ems_device.h"
#include "ems_kernels.h"

namespace ems {

// Host: let `kernel` use all of a workgroup's LDS.  Kernels get 64 KiB of dynamic LDS by
// default; the limit is a property of (kernel, device), so it is raised once per device
// (`done` = the kernel's own set of devices already served, one bit each).
inline hipError_t allow_max_lds(const void* kernel, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load() & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    if (e == hipSuccess) done.fetch_or(bit);
    return e;
}

constexpr int kTileKeys = 32;
constexpr int kMaxRows = 16;             // query rows per MFMA column block
constexpr float kMaxSlack = 6.f;         // lazy softmax reference: P entries stay below 2^6, exact in fp32, far inside fp16 / bf16 range
constexpr int kMaxRowsWide = 64;         // query rows per sample in the wide kernel (two pairs of two blocks)
constexpr int kAttnThreads = 256;
constexpr int kWavesPerBlock = kAttnThreads / kWave;

__device__ __forceinline__ int tiles_of_sample(int k, int L) {
    return k > 0 ? ((L + kTileKeys - 1) / kTileKeys + 1) : 0;
}
// The wide kernel (up to 64 rows per sample): a (sample, head) is one pair of up to 32 rows, or
// two when the sample brings more; every pair has the cache tiles and then ceil(k/32) tiles of
// new tokens.
__device__ __forceinline__ int new_tiles(int k) { return (k + kTileKeys - 1) / kTileKeys; }
__device__ __forceinline__ int wide_halves(int k) { return k > 32 ? 2 : 1; }
__device__ __forceinline__ int tiles_of_sample_wide(int k, int L) {
    k = min(k, kMaxRowsWide);
    return k > 0 ? wide_halves(k) * ((L + kTileKeys - 1) / kTileKeys + new_tiles(k)) : 0;
}
// ... or, when the wave keeps all four blocks of 16 rows (two of them parked in LDS), one pair.
__device__ __forceinline__ int tiles_of_sample_wide64(int k, int L) {
    k = min(k, kMaxRowsWide);
    return k > 0 ? ((L + kTileKeys - 1) / kTileKeys + new_tiles(k)) : 0;
}
enum { kPlainLine = 0, kPaddedLine = 1, kWideLine = 2, kWide64Line = 3 };

// prefix[1..B] holds each sample's tile count, prefix[0] = 0: turned into running sums by the
// block's first wave (64 entries a pass); barriers before and after.
__device__ __forceinline__ void scan_tile_counts(int32_t* prefix, int B) {
    const int tid = threadIdx.x;
    __syncthreads();
    if (tid < kWave) {
        int carry = 0;
        for (int base = 1; base <= B; base += kWave) {
            const int idx = base + tid;
            int v = idx <= B ? prefix[idx] : 0;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                int u = __shfl_up(v, off);
                if (tid >= off) v += u;
            }
            if (idx <= B) prefix[idx] = v + carry;
            carry += __shfl(v, kWave - 1);
        }
    }
    __syncthreads();
}

// prefix[i] = H * sum_{j<i} tiles(j), i = 0..B, built by the whole block in LDS.
template <int LINE>
__device__ __forceinline__ void build_tile_prefix(const AttnParams& p, int32_t* prefix) {
    const int tid = threadIdx.x;
    for (int i = tid; i < p.B; i += blockDim.x)
        prefix[i + 1] = LINE == kPaddedLine ? p.H * tiles_of_sample(p.k_max, p.l_pad)
                        : LINE == kWideLine ? p.H * tiles_of_sample_wide(p.cu[i + 1] - p.cu[i], p.kv_len[i])
                        : LINE == kWide64Line ? p.H * tiles_of_sample_wide64(p.cu[i + 1] - p.cu[i], p.kv_len[i])
                                            : p.H * tiles_of_sample(p.cu[i + 1] - p.cu[i], p.kv_len[i]);
    if (tid == 0) prefix[0] = 0;
    scan_tile_counts(prefix, p.B);
}

// The tile line is cut into ranges that differ by at most one tile: of `waves` waves
// (waves <= total, so no range is empty) the first total % waves own total / waves + 1 tiles
// each, the others total / waves.  Only 32-bit divisions: a 64-bit one costs a wave most of
// a microsecond before it has asked memory for anything.
struct LineCut {
    int q, r;          // tiles per wave (rounded down), waves that own one more
    __device__ __forceinline__ LineCut(int total, int waves) : q(total / waves), r(total - (total / waves) * waves) {}
    __device__ __forceinline__ int begin(int wave) const { return wave * q + min(wave, r); }
    __device__ __forceinline__ int wave_of(int g) const {          // the wave whose range holds tile g
        const int big = r * (q + 1);
        return g < big ? g / (q + 1) : r + (g - big) / q;
    }
};

// Head dims: 64 and 128 fill every lane; 80 (a row of 160 bytes) is run as a 96-wide
// score product whose last k-step is half empty (the lane quarters g >= 2 re-read the
// pieces of g - 2 and meet zeros in Q) and a V / output layout of 8 elements per lane in
// which only 10 of the 16 lanes of a row hold data (the others re-read lane 9's piece and
// their results are never stored).
template <int D>
struct TileRegs {
    static_assert(D == 64 || D == 80 || D == 128, "head dims 64, 80 and 128");
    static constexpr int KS = (D + 31) / 32;          // MFMA k-steps over the head dim
    static constexpr int VW = D == 64 ? 4 : 8;        // head-dim elements per lane per V row
    static constexpr int kVLanes = D / VW;            // lanes of a 16-lane row that hold V / output data
    static constexpr int kTailQ = (D % 32) / 8;       // valid lane quarters of the last k-step; 0 = all four
    // byte offset of lane quarter g's 16-byte piece of k-step s inside a K or Q row
    static __device__ __forceinline__ uint32_t piece(int s, int g) {
        return (uint32_t)(64 * s + 16 * ((kTailQ != 0 && s == KS - 1) ? g % (kTailQ != 0 ? kTailQ : 1) : g));
    }
    static __device__ __forceinline__ bool piece_valid(int s, int g) {
        return !(kTailQ != 0 && s == KS - 1 && g >= kTailQ);
    }
    typedef uint32_t vrow_t __attribute__((ext_vector_type(VW / 2)));
    u32x4 ka[KS], kb[KS];                    // keys 0..15 / 16..31 of the tile, A-operand layout
    vrow_t v[8];                             // this lane's 8 keys x VW head-dim elements
    uint32_t mka, mkb;                       // padded ablation only: key-mask bytes of this lane's keys
};

// Where the 32 keys of one tile live: a run of rows of `row_bytes` starting at kbase/vbase
// (already offset to the head), first key n0, last valid row `last` (rows are clamped to
// it so that masked keys still read valid, finite data).
struct TileSrc {
    uint64_t kbase, vbase;   // wave-uniform
    uint32_t row_bytes;
    int n0, last;
    uint64_t mask_base;      // padded ablation only: key-mask row of the sample, 0 = no mask bytes
};

template <int D, bool PADDED>
__device__ __forceinline__ void load_tile(TileRegs<D>& t, const TileSrc& src, int n, int g) {
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    const uint32_t ra = (uint32_t)min(src.n0 + n, src.last) * src.row_bytes;
    const uint32_t rb = (uint32_t)min(src.n0 + 16 + n, src.last) * src.row_bytes;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        t.ka[s] = gload_stream<u32x4>(src.kbase, ra + TileRegs<D>::piece(s, g));
        t.kb[s] = gload_stream<u32x4>(src.kbase, rb + TileRegs<D>::piece(s, g));
    }
    const uint32_t vcol = (uint32_t)min(n, TileRegs<D>::kVLanes - 1) * (VW * 2);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int key = src.n0 + (e < 4 ? 4 * g + e : 16 + 4 * g + (e - 4));
        const uint32_t off = (uint32_t)min(key, src.last) * src.row_bytes + vcol;
        t.v[e] = gload_stream<typename TileRegs<D>::vrow_t>(src.vbase, off);
    }
    if (PADDED) {
        t.mka = t.mkb = 0x01010101u;
        if (src.mask_base != 0) {            // wave-uniform
            t.mka = gload<uint32_t>(src.mask_base, (uint32_t)(src.n0 + 4 * g));
            t.mkb = gload<uint32_t>(src.mask_base, (uint32_t)(src.n0 + 16 + 4 * g));
        }
    }
}

template <typename ET> struct PSplit { static constexpr bool value = false; };
template <> struct PSplit<BF16> { static constexpr bool value = true; };

template <typename ET, int D>
struct SoftmaxState {
    static constexpr int VW = TileRegs<D>::VW;
    f32x4 acc[VW];     // acc[c][i] = O[query n][d = (4g+i)*VW + c], unnormalised (rows 4g+i < kVLanes)
    float m;           // running max (log2 domain), same in the 4 lanes of a query
    float l;           // this lane's share of the running sum
};

// A partial parked in LDS for the in-workgroup merge: the VW accumulator registers, the
// running max and this lane's share of the running sum, for each of the 64 lanes.
template <int D> struct FoldSlot {
    static constexpr int m_at = TileRegs<D>::VW * kWave * 4;
    static constexpr int l_at = m_at + kWave;
    static constexpr int floats = l_at + kWave;
};
// One tile: scores, masked online softmax, PV.  `lim` = number of visible keys
// of this tile for this lane's query row (>= 32 means no masking); with BITS it is
// instead a bit set over the tile's 32 keys (bit n = key n visible), the form a tile of
// new tokens uses: a causal prefix, or a row's ancestors in a token tree.
template <typename ET, int D, bool MASKED, bool PADDED = false, bool BITS = false>
__device__ __forceinline__ void compute_tile(const TileRegs<D>& t, const u32x4* qb,
                                             SoftmaxState<ET, D>& st, float scale_log2, int lim,
                                             int g) {
    constexpr int KS = TileRegs<D>::KS;
    constexpr int VW = TileRegs<D>::VW;
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        sa = mfma16x16x32(ET{}, t.ka[s], qb[s], sa);
        sb = mfma16x16x32(ET{}, t.kb[s], qb[s], sb);
    }
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[i] = sa[i] * scale_log2;
        x[4 + i] = sb[i] * scale_log2;
        if (MASKED && BITS) {
            if (((lim >> (4 * g + i)) & 1) == 0) x[i] = -INFINITY;
            if (((lim >> (16 + 4 * g + i)) & 1) == 0) x[4 + i] = -INFINITY;
        } else if (MASKED) {
            if (4 * g + i >= lim) x[i] = -INFINITY;
            if (16 + 4 * g + i >= lim) x[4 + i] = -INFINITY;
        }
        if (PADDED) {                        // padding keys of the aligned cache
            if (((t.mka >> (8 * i)) & 0xffu) == 0) x[i] = -INFINITY;
            if (((t.mkb >> (8 * i)) & 0xffu) == 0) x[4 + i] = -INFINITY;
        }
    }
    float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                     fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    const float m_new = fmaxf(st.m, quad_max(mx));
    // Unpadded: every tile holds at least one visible key for every row, so m_new is
    // finite.  Padded: a tile may be all padding; subtract 0 instead of -inf then.
    const float m_sub = (PADDED && m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(st.m - m_sub);     // exp2(-inf) = 0 on the first tile
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
    // P^T as the B operand: slot e of this lane = key (e<4 ? 4g+e : 16+4g+e-4).
    // bf16 keeps 8 significant bits, too few for P when a row has only a handful of
    // keys; there P is fed as hi + lo (two products), which restores ~16 bits.
    constexpr bool kSplitP = PSplit<ET>::value;
    u32x4 pb, pl;
    pb[0] = pack2(ET{}, x[0], x[1]);
    pb[1] = pack2(ET{}, x[2], x[3]);
    pb[2] = pack2(ET{}, x[4], x[5]);
    pb[3] = pack2(ET{}, x[6], x[7]);
    if (kSplitP) {
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] -= round16(ET{}, x[i]);
        pl[0] = pack2(ET{}, x[0], x[1]);
        pl[1] = pack2(ET{}, x[2], x[3]);
        pl[2] = pack2(ET{}, x[4], x[5]);
        pl[3] = pack2(ET{}, x[6], x[7]);
    }
    // V^T as the A operand: for head-dim element c of this lane, the 8 keys' values.
#pragma unroll
    for (int c = 0; c < VW; ++c) {
        u32x4 va;
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            const uint32_t w0 = t.v[2 * pr][c >> 1];
            const uint32_t w1 = t.v[2 * pr + 1][c >> 1];
            va[pr] = (c & 1) ? pair_hi(w0, w1) : pair_lo(w0, w1);
        }
        st.acc[c] = mfma16x16x32(ET{}, va, pb, st.acc[c]);
        if (kSplitP) st.acc[c] = mfma16x16x32(ET{}, va, pl, st.acc[c]);
    }
}

// Token trees: the new rows a row sees are itself and its ancestors.  Lane n of every
// 16-lane row holds parent[n] of the pair's sample; four rounds of pointer doubling
// (each row adopts the set of the row it currently points to, then points where that
// row pointed) cover any depth up to 16.  Anything that is not a valid parent (not in
// [0, n), or n >= k) counts as "no parent", so the exchanges stay inside the sample.
__device__ __forceinline__ int tree_visibility(int parent_n, int n, int k) {
    int jump = (n < k && parent_n >= 0 && parent_n < n) ? parent_n : -1;
    int seen = 1 << n;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int src = jump >= 0 ? jump : n;
        const int seen_src = __shfl(seen, src, 16);
        const int jump_src = __shfl(jump, src, 16);
        if (jump >= 0) {
            seen |= seen_src;
            jump = jump_src;
        }
    }
    return seen;
}

// The same for up to 64 rows: lane j holds parent[j] of row j, six rounds cover any depth,
// and the sets take two words.  Returns the set of row `want` (a lane-dependent row index).
__device__ __forceinline__ uint64_t tree_visibility64(int parent_j, int lane, int k, int want) {
    int jump = (lane < k && parent_j >= 0 && parent_j < lane) ? parent_j : -1;
    uint32_t lo = lane < 32 ? 1u << lane : 0u, hi = lane >= 32 ? 1u << (lane - 32) : 0u;
#pragma unroll
    for (int t = 0; t < 6; ++t) {
        const int src = jump >= 0 ? jump : lane;
        const uint32_t lo_src = __shfl(lo, src), hi_src = __shfl(hi, src);
        const int jump_src = __shfl(jump, src);
        if (jump >= 0) {
            lo |= lo_src;
            hi |= hi_src;
            jump = jump_src;
        }
    }
    const uint32_t wl = __shfl(lo, want), wh = __shfl(hi, want);
    return ((uint64_t)wh << 32) | wl;
}

}  // namespace ems
