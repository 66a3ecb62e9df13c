// C ABI of libems: argument validation (host only, before any HIP call),
// launch sizing, error strings.  See include/ems.h for the contract.
#include "../../include/ems.h"
#include "../../include/ems_measure.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <vector>

#include "ems_kernels.h"

namespace {

thread_local char g_err[512] = "";

ems_status fail(ems_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

ems_status hip_fail(const char* what, hipError_t e) {
    return fail(EMS_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr int kTileKeys = 32;
constexpr int kWavesPerBlock = 4;
constexpr int kMinTilesPerWave = 4;
constexpr int kMaxAttnBlocks = 1024;
constexpr int kMaxB = 8192;

// The three launch shapes of the attention call: up to 16 rows per (sample, head) pair; up to 32
// (the wide kernel; a sample of more rows is two pairs per head); up to 64 (the wide kernel
// with two of a pair's four blocks parked in LDS, while LDS has room for that).
enum AttnShape { kRows16 = 0, kRows32 = 1, kRows64 = 2 };
int rows_per_slot(AttnShape shape) { return 16 << shape; }

// Upper bound of the number of 32-key tiles of the whole batch (host-known bounds only); with
// more than 32 rows a sample has two tiles of new tokens and, as two pairs per head, all tiles twice.
int64_t tile_upper_bound(int B, int H, int max_kv_len, AttnShape shape, int max_k) {
    const int64_t cache_tiles = (max_kv_len + kTileKeys - 1) / kTileKeys;
    const int64_t per_pair = cache_tiles + (max_k > 32 ? 2 : 1);
    return (int64_t)B * H * (shape == kRows32 && max_k > 32 ? 2 * per_pair : per_pair);
}

int attn_blocks_for(int64_t tiles, int max_blocks) {
    int64_t want = (tiles + kWavesPerBlock * kMinTilesPerWave - 1) / (kWavesPerBlock * kMinTilesPerWave);
    return (int)std::max<int64_t>(1, std::min<int64_t>(want, max_blocks));
}

// Workspace = header (the B+1 tile prefix sums, padded to 256 B) + partial slots.
size_t attn_ws_header_bytes(int B) { return ((size_t)(B + 1) * sizeof(int32_t) + 255) / 256 * 256; }

// Two partial slots per wave, of 16, 32 or 64 rows each.
size_t attn_ws_bytes_for(int blocks, int B, int D, AttnShape shape) {
    return attn_ws_header_bytes(B) +
           (size_t)2 * blocks * kWavesPerBlock * rows_per_slot(shape) * (D + ems::kPartialPad) * sizeof(float);
}

// Workgroups launched for the attention kernel: one per CU, i.e. one wave per SIMD.  Two
// per CU measured slower (275 vs 256 us at config 4): the SIMD arbitrates oldest-first, the
// older workgroup's waves finish long before the younger one's and the tail runs half empty.
int resident_attn_blocks() {
    // per-device fact, cached on first use; threads that race here store the same value
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int blocks = cached[dev].load(std::memory_order_relaxed);
    if (blocks == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        blocks = std::min(kMaxAttnBlocks, cus);
        cached[dev].store(blocks, std::memory_order_relaxed);
    }
    return blocks;
}

void accept_slicing(int T, int V, int* slices, int* slice_len) {
    // enough blocks to fill the chip (about 2048), slices a multiple of 8 columns, at least 2048
    // columns each.  No more slices than that: measured with 128256 columns, 16 slices of 8192
    // (one round of loads per block) ran 150 us at 3008 rows where 1 to 4 slices ran 125 us,
    // and with 50272 columns 1 to 7 slices are equal.
    int s = T > 0 ? (2048 + T - 1) / T : 1;
    // ... except that a few more are taken when they make a slice fit one round of four 16-byte
    // loads per thread (8192 columns): 7 instead of 6 at 384 rows of 50272 columns, 9.7 vs 10.8 us
    const int one_round = (V + 8191) / 8192;
    if (one_round > s && one_round <= s + s / 2 + 1) s = one_round;
    s = std::max(1, std::min(s, 16));
    int len = (V + s - 1) / s;
    len = std::max(2048, (len + 7) / 8 * 8);
    *slice_len = len;
    *slices = std::max(1, (V + len - 1) / len);
}

bool dtype16(ems_dtype d) { return d == EMS_F16 || d == EMS_BF16; }

// Measurement aids, both per calling thread, so that one thread's measurement never changes
// what another thread's attention call runs or records: optional timing of the attention
// call with HIP events (before the main kernel, after it, after the merge kernel), and
// which formulation of the main kernel this thread's calls use.
struct Profile {
    std::vector<hipEvent_t> start, stop, end;
    int used = 0;
};
thread_local Profile g_prof;
thread_local int g_attn_variant = EMS_ATTN_MFMA;

}  // namespace

extern "C" {

const char* ems_last_error_string(void) { return g_err; }

const char* ems_version(void) { return "0.1"; }

ems_status ems_device_memory_figures(int* memory_clock_khz, int* memory_bus_width_bits) {
    if (!memory_clock_khz || !memory_bus_width_bits) return fail(EMS_ERR_INVALID_ARG, "NULL output pointer");
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(memory_clock_khz, hipDeviceAttributeMemoryClockRate, dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(memory_bus_width_bits, hipDeviceAttributeMemoryBusWidth, dev);
    if (e != hipSuccess) return fail(EMS_ERR_HIP, "device attributes: %s", hipGetErrorString(e));
    return EMS_OK;
}

size_t ems_workspace_bytes(int B, int T, int H, int D, int max_kv_len) {
    return ems_attention_workspace_bytes(B, T, H, D, max_kv_len);
}

size_t ems_attention_workspace_bytes(int B, int T, int H, int D, int max_kv_len) {
    (void)T;
    if (B < 1 || H < 1 || D < 1 || max_kv_len < 0) return 256;
    // (sized for the largest of the launch shapes, as max_k is not known here: the most tiles
    // and the widest slots; one workgroup per CU of the current device, as the launch itself is
    // sized, or 256 when there is no device)
    const int blocks = attn_blocks_for(tile_upper_bound(B, H, max_kv_len, kRows32, 64), resident_attn_blocks());
    return std::max<size_t>(256, attn_ws_bytes_for(blocks, B, D, kRows64));
}

}  // extern "C"

namespace {

struct PaddedArgs {
    const uint8_t* key_mask;
    const int32_t* k_valid;
    int k_max, l_pad;
    int64_t cap;
};

// Shared by the unpadded entry point and the padded ablation (pad != nullptr).
ems_status run_attention(const void* q, const void* k_new, const void* v_new,
                         const ems_kv_cache* cache, const int32_t* cu_seqlens,
                         const int32_t* kv_start, const int32_t* kv_len, void* out,
                         ems_dtype out_dtype, int B, int T, int H, int D, int max_k,
                         int max_kv_len, float scale, ems_dtype dtype, void* workspace,
                         size_t workspace_bytes, void* hip_stream, const PaddedArgs* pad,
                         bool write_through = false, const int32_t* parent = nullptr) {
    if (B < 1) return fail(EMS_ERR_INVALID_ARG, "B = %d, need B >= 1", B);
    if (T < 0) return fail(EMS_ERR_INVALID_ARG, "T = %d, need T >= 0", T);
    if (H < 1) return fail(EMS_ERR_INVALID_ARG, "H = %d, need H >= 1", H);
    if (max_k < 0 || max_kv_len < 0)
        return fail(EMS_ERR_INVALID_ARG, "max_k = %d, max_kv_len = %d must not be negative", max_k, max_kv_len);
    if (!std::isfinite(scale)) return fail(EMS_ERR_INVALID_ARG, "scale is not finite");
    if (!dtype16(dtype)) return fail(EMS_ERR_INVALID_ARG, "dtype must be EMS_F16 or EMS_BF16");
    if (out_dtype != dtype && out_dtype != EMS_F32)
        return fail(EMS_ERR_INVALID_ARG, "out_dtype must equal dtype or be EMS_F32");
    if (!pad && (!cu_seqlens || !kv_start || !kv_len))
        return fail(EMS_ERR_INVALID_ARG, "cu_seqlens, kv_start and kv_len must not be NULL");
    if (D != 64 && D != 80 && D != 128)
        return fail(EMS_ERR_UNSUPPORTED, "D = %d, supported head dims are 64, 80 and 128", D);
    if (D == 80 && pad) return fail(EMS_ERR_UNSUPPORTED, "the padded ablation has head dims 64 and 128 only");
    if (D == 80 && g_attn_variant == EMS_ATTN_VALU)
        return fail(EMS_ERR_UNSUPPORTED, "EMS_ATTN_VALU has head dims 64 and 128 only");
    if (!pad && g_attn_variant == EMS_ATTN_VALU && ems::valu_attention_lds_bytes(B, D) > (size_t)ems::kMaxLdsBytes)
        return fail(EMS_ERR_UNSUPPORTED, "EMS_ATTN_VALU keeps its per-row state in LDS: B = %d at D = %d needs %zu of %d bytes",
                    B, D, ems::valu_attention_lds_bytes(B, D), ems::kMaxLdsBytes);
    if (max_k > EMS_MAX_QUERY_ROWS)
        return fail(EMS_ERR_UNSUPPORTED, "max_k = %d, at most %d rows per sample", max_k, EMS_MAX_QUERY_ROWS);
    const bool wide = max_k > EMS_ROWS_PER_GROUP;      // the wide kernel
    if (wide && pad) return fail(EMS_ERR_UNSUPPORTED, "the padded ablation takes at most %d rows per sample", EMS_ROWS_PER_GROUP);
    if (wide && g_attn_variant == EMS_ATTN_VALU)
        return fail(EMS_ERR_UNSUPPORTED, "EMS_ATTN_VALU takes at most %d rows per sample", EMS_ROWS_PER_GROUP);
    if (B > kMaxB) return fail(EMS_ERR_UNSUPPORTED, "B = %d, at most %d samples", B, kMaxB);
    if (T == 0) return EMS_OK;
    if (!q || !k_new || !v_new || !out) return fail(EMS_ERR_INVALID_ARG, "q, k_new, v_new and out must not be NULL");
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out))
        return fail(EMS_ERR_INVALID_ARG, "q, k_new, v_new and out must be 16-byte aligned");
    if (!cache) return fail(EMS_ERR_INVALID_ARG, "cache must not be NULL");
    if (cache->row_stride < D || cache->head_stride < D || (cache->row_stride & 7) || (cache->head_stride & 7))
        return fail(EMS_ERR_INVALID_ARG, "cache strides must be multiples of 8 elements and at least D");
    if (max_kv_len > 0 && (!cache->k || !cache->v || !aligned16(cache->k) || !aligned16(cache->v)))
        return fail(EMS_ERR_INVALID_ARG, "cache arenas must be non-NULL and 16-byte aligned");
    if (cache->rows < 0) return fail(EMS_ERR_INVALID_ARG, "cache rows must not be negative");
    // a sample's cache is addressed with 32-bit byte offsets from its first row
    if (((int64_t)max_kv_len + kTileKeys) * cache->row_stride * 2 >= ((int64_t)1 << 32))
        return fail(EMS_ERR_UNSUPPORTED, "max_kv_len * row_stride exceeds 4 GiB per sample");
    const AttnShape shape = !wide ? kRows16 : (max_k > 32 && ems::wide_rows64_fits(B, D)) ? kRows64 : kRows32;
    const int64_t tiles = tile_upper_bound(B, H, max_kv_len, shape, max_k);
    if (tiles >= ((int64_t)1 << 31)) return fail(EMS_ERR_UNSUPPORTED, "too many key tiles");

    const int blocks = attn_blocks_for(tiles, resident_attn_blocks());
    const size_t need = attn_ws_bytes_for(blocks, B, D, shape);
    if (!workspace || workspace_bytes < need)
        return fail(EMS_ERR_WORKSPACE, "attention workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : (size_t)0);
    if (!aligned16(workspace)) return fail(EMS_ERR_INVALID_ARG, "workspace must be 16-byte aligned");

    ems::AttnParams p;
    std::memset(&p, 0, sizeof p);
    p.q = static_cast<const char*>(q);
    p.k_new = static_cast<const char*>(k_new);
    p.v_new = static_cast<const char*>(v_new);
    p.k_cache = static_cast<const char*>(cache->k);
    p.v_cache = static_cast<const char*>(cache->v);
    p.row_stride_b = cache->row_stride * 2;
    p.head_stride_b = cache->head_stride * 2;
    p.cu = cu_seqlens;
    p.kv_start = kv_start;
    p.kv_len = kv_len;
    p.parent = parent;
    p.out = out;
    p.ws_header = static_cast<int32_t*>(workspace);
    p.ws = reinterpret_cast<float*>(static_cast<char*>(workspace) + attn_ws_header_bytes(B));
    p.out_f32 = out_dtype == EMS_F32;
    p.B = B;
    p.H = H;
    p.num_waves = blocks * kWavesPerBlock;
    p.scale_log2 = scale * 1.4426950408889634f;
    p.write_through = write_through ? 1 : 0;
    p.multi = (int)shape;
    // The in-workgroup merge of partials saves HBM writes in the middle of the read stream and
    // costs a barrier and a fold at the end of the walk (~1 us): measured break-even at ~13 tiles
    // per wave (B = 16, 1024 cached tokens), a loss of 1.5 us at 6, gains from 25 on.
    p.wg_fold = tiles >= (int64_t)12 * p.num_waves ? 1 : 0;
    if (pad) {
        p.key_mask = pad->key_mask;
        p.k_valid = pad->k_valid;
        p.k_max = pad->k_max;
        p.l_pad = pad->l_pad;
        p.cap = pad->cap;
    }
    hipEvent_t ev0 = nullptr, ev1 = nullptr, ev2 = nullptr;
    if (g_prof.used < (int)g_prof.start.size()) {
        ev0 = g_prof.start[g_prof.used];
        ev1 = g_prof.stop[g_prof.used];
        ev2 = g_prof.end[g_prof.used];
        ++g_prof.used;
    }
    hipError_t e = ems::launch_verify_attention(p, blocks, D, dtype == EMS_BF16, pad != nullptr,
                                                g_attn_variant == EMS_ATTN_VALU,
                                                static_cast<hipStream_t>(hip_stream), ev0, ev1);
    if (e != hipSuccess) return hip_fail("attention launch", e);
    if (ev2 && (e = hipEventRecord(ev2, static_cast<hipStream_t>(hip_stream))) != hipSuccess)
        return hip_fail("attention timing", e);
    return EMS_OK;
}

}  // namespace

extern "C" {

ems_status ems_verify_attention(const void* q, const void* k_new, const void* v_new,
                                const ems_kv_cache* cache, const int32_t* cu_seqlens,
                                const int32_t* kv_start, const int32_t* kv_len, void* out,
                                ems_dtype out_dtype, int B, int T, int H, int D, int max_k,
                                int max_kv_len, float scale, ems_dtype dtype, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
    return run_attention(q, k_new, v_new, cache, cu_seqlens, kv_start, kv_len, out, out_dtype, B, T,
                         H, D, max_k, max_kv_len, scale, dtype, workspace, workspace_bytes,
                         hip_stream, nullptr);
}

ems_status ems_verify_attention_write_through(const void* q, const void* k_new, const void* v_new,
                                              const ems_kv_cache* cache, const int32_t* cu_seqlens,
                                              const int32_t* kv_start, const int32_t* kv_len,
                                              void* out, ems_dtype out_dtype, int B, int T, int H,
                                              int D, int max_k, int max_kv_len, float scale,
                                              ems_dtype dtype, void* workspace,
                                              size_t workspace_bytes, void* hip_stream) {
    if (cache && T > 0 && (!cache->k || !cache->v))
        return fail(EMS_ERR_INVALID_ARG, "cache arenas must not be NULL");
    return run_attention(q, k_new, v_new, cache, cu_seqlens, kv_start, kv_len, out, out_dtype, B, T,
                         H, D, max_k, max_kv_len, scale, dtype, workspace, workspace_bytes,
                         hip_stream, nullptr, true);
}

}  // extern "C"

// The buffer of ems_verify_attention_noalloc: part of this library's device image, one copy per
// GPU.  In host code its name is only a handle for hipGetSymbolAddress; the device address is
// looked up once per device (with that device current) and kept.  (No `used` attribute: the
// compiler gives a static device variable a global symbol in the device image exactly when host
// code refers to it, as noalloc_scratch() does; marked `used` it stays a local symbol there,
// the runtime cannot find it by name, and the first lookup aborts the process.)
static __device__ __align__(256) unsigned char scratch[EMS_NOALLOC_SCRATCH_BYTES];

namespace {

ems_status noalloc_scratch(void** ptr) {
    static std::atomic<void*> per_device[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail("hipGetDevice", e);
    if (dev < 0 || dev >= 64) return fail(EMS_ERR_UNSUPPORTED, "device ordinal %d beyond the 64 this call keeps track of", dev);
    void* p = per_device[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) return hip_fail("hipGetSymbolAddress(scratch)", e);
        per_device[dev].store(p, std::memory_order_release);     // (threads that race here store the same address)
    }
    *ptr = p;
    return EMS_OK;
}

}  // namespace

extern "C" {

ems_status ems_verify_attention_noalloc(const void* q, const void* k_new, const void* v_new,
                                        const ems_kv_cache* cache, const int32_t* cu_seqlens,
                                        const int32_t* kv_start, const int32_t* kv_len, void* out,
                                        ems_dtype out_dtype, int B, int T, int H, int D, int max_k,
                                        int max_kv_len, float scale, ems_dtype dtype, void* hip_stream) {
    if (max_k > EMS_ROWS_PER_GROUP)
        return fail(EMS_ERR_UNSUPPORTED, "ems_verify_attention_noalloc takes max_k <= %d, got %d", EMS_ROWS_PER_GROUP, max_k);
    // what the launch would need, from the same arithmetic as the call with a workspace
    if (B >= 1 && B <= kMaxB && H >= 1 && max_kv_len >= 0 && (D == 64 || D == 80 || D == 128)) {
        const int blocks = attn_blocks_for(tile_upper_bound(B, H, max_kv_len, kRows16, max_k), resident_attn_blocks());
        const size_t need = attn_ws_bytes_for(blocks, B, D, kRows16);
        if (need > (size_t)EMS_NOALLOC_SCRATCH_BYTES)
            return fail(EMS_ERR_UNSUPPORTED, "this launch needs %zu bytes for its partial results, the library's own "
                        "buffer holds %zu (EMS_NOALLOC_SCRATCH_BYTES)", need, (size_t)EMS_NOALLOC_SCRATCH_BYTES);
    }
    void* ptr = nullptr;
    if (T > 0) {
        const ems_status st = noalloc_scratch(&ptr);
        if (st != EMS_OK) return st;
    }
    return run_attention(q, k_new, v_new, cache, cu_seqlens, kv_start, kv_len, out, out_dtype, B, T,
                         H, D, max_k, max_kv_len, scale, dtype, ptr, T > 0 ? (size_t)EMS_NOALLOC_SCRATCH_BYTES : 0,
                         hip_stream, nullptr);
}

ems_status ems_tree_verify_attention(const void* q, const void* k_new, const void* v_new,
                                     const ems_kv_cache* cache, const int32_t* cu_seqlens,
                                     const int32_t* parent, const int32_t* kv_start,
                                     const int32_t* kv_len, void* out, ems_dtype out_dtype, int B,
                                     int T, int H, int D, int max_k, int max_kv_len, float scale,
                                     ems_dtype dtype, void* workspace, size_t workspace_bytes,
                                     void* hip_stream) {
    if (!parent && T > 0) return fail(EMS_ERR_INVALID_ARG, "parent must not be NULL");
    if (g_attn_variant == EMS_ATTN_VALU)
        return fail(EMS_ERR_UNSUPPORTED, "EMS_ATTN_VALU has no token-tree mask");
    return run_attention(q, k_new, v_new, cache, cu_seqlens, kv_start, kv_len, out, out_dtype, B, T,
                         H, D, max_k, max_kv_len, scale, dtype, workspace, workspace_bytes,
                         hip_stream, nullptr, false, parent);
}

ems_status ems_kv_advance(const int32_t* kv_len, const int32_t* accepted, int32_t* kv_len_out, int B,
                          void* hip_stream) {
    if (B < 1) return fail(EMS_ERR_INVALID_ARG, "B = %d, need B >= 1", B);
    if (!kv_len || !accepted || !kv_len_out)
        return fail(EMS_ERR_INVALID_ARG, "kv_len, accepted and kv_len_out must not be NULL");
    hipError_t e = ems::launch_advance_kv_len(kv_len, accepted, nullptr, kv_len_out, B,
                                              static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail("ems_kv_advance launch", e);
    return EMS_OK;
}

ems_status ems_padded_verify_attention(const void* q_pad, const void* k_new_pad,
                                       const void* v_new_pad, const ems_kv_cache* cache,
                                       int64_t cap, const uint8_t* key_mask,
                                       const int32_t* k_valid, void* out_pad, ems_dtype out_dtype,
                                       int B, int k_max, int l_pad, int H, int D, float scale,
                                       ems_dtype dtype, void* workspace, size_t workspace_bytes,
                                       void* hip_stream) {
    if (k_max < 1) return fail(EMS_ERR_INVALID_ARG, "k_max = %d, need k_max >= 1", k_max);
    if (l_pad < 0) return fail(EMS_ERR_INVALID_ARG, "l_pad = %d, need l_pad >= 0", l_pad);
    if (cap < l_pad || cap < kTileKeys || (cap % kTileKeys) != 0)
        return fail(EMS_ERR_INVALID_ARG, "cap = %lld must be a multiple of %d and at least l_pad",
                    (long long)cap, kTileKeys);
    if (!key_mask || !k_valid) return fail(EMS_ERR_INVALID_ARG, "key_mask and k_valid must not be NULL");
    if (reinterpret_cast<uintptr_t>(key_mask) & 3u)
        return fail(EMS_ERR_INVALID_ARG, "key_mask must be 4-byte aligned");
    if (B >= 1 && cache && cache->rows < (int64_t)B * cap)
        return fail(EMS_ERR_INVALID_ARG, "cache holds %lld rows, B * cap = %lld needed",
                    (long long)cache->rows, (long long)B * cap);
    if (B >= 1 && (int64_t)B * k_max > 0x7fffffff) return fail(EMS_ERR_UNSUPPORTED, "B * k_max too large");
    PaddedArgs pad{key_mask, k_valid, k_max, l_pad, cap};
    return run_attention(q_pad, k_new_pad, v_new_pad, cache, nullptr, nullptr, nullptr, out_pad,
                         out_dtype, B, B >= 1 ? B * k_max : 0, H, D, k_max, l_pad, scale, dtype,
                         workspace, workspace_bytes, hip_stream, &pad);
}

size_t ems_accept_workspace_bytes(int T, int V) {
    if (T <= 0 || V <= 0) return 0;
    // at most 16 slices per row whatever T is, so the figure also covers every smaller T
    return (size_t)T * 16 * sizeof(ems::ArgmaxPartial);
}

}  // extern "C"

namespace {

// Shared by ems_greedy_accept (parent == nullptr) and ems_tree_accept.
// Checks the arguments of an acceptance call and fills its kernel parameters.
ems_status prepare_accept(const void* logits, ems_dtype dtype, int V, int32_t* target_ids,
                          const int32_t* input_ids, const int32_t* parent, const int32_t* cu_seqlens,
                          int B, int T, int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens,
                          int32_t* accepted_rows, void* workspace, size_t workspace_bytes,
                          ems::AcceptParams* out) {
    if (B < 1) return fail(EMS_ERR_INVALID_ARG, "B = %d, need B >= 1", B);
    if (T < 0) return fail(EMS_ERR_INVALID_ARG, "T = %d, need T >= 0", T);
    if (V < 0) return fail(EMS_ERR_INVALID_ARG, "V = %d, need V >= 0", V);
    if (B > kMaxB) return fail(EMS_ERR_UNSUPPORTED, "B = %d, at most %d samples", B, kMaxB);
    if (T > 65535) return fail(EMS_ERR_UNSUPPORTED, "T = %d, at most 65535 packed rows", T);
    if (!cu_seqlens || !accepted || !accepted_cu)
        return fail(EMS_ERR_INVALID_ARG, "cu_seqlens, accepted and accepted_cu must not be NULL");
    if (T > 0 && (!target_ids || !input_ids))
        return fail(EMS_ERR_INVALID_ARG, "target_ids and input_ids must not be NULL");
    ems::AcceptParams& p = *out;
    std::memset(&p, 0, sizeof p);
    if (logits != nullptr) {
        if (!dtype16(dtype) && dtype != EMS_F32)
            return fail(EMS_ERR_INVALID_ARG, "logits dtype must be EMS_F16, EMS_BF16 or EMS_F32");
        if (V < 1) return fail(EMS_ERR_INVALID_ARG, "logits given but V = %d", V);
        if (!aligned16(logits)) return fail(EMS_ERR_INVALID_ARG, "logits must be 16-byte aligned");
        accept_slicing(T, V, &p.slices, &p.slice_len);
        const size_t need = (size_t)T * p.slices * sizeof(ems::ArgmaxPartial);
        if (T > 0 && (!workspace || workspace_bytes < need))
            return fail(EMS_ERR_WORKSPACE, "accept workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
        if (T > 0 && (reinterpret_cast<uintptr_t>(workspace) & 7u))
            return fail(EMS_ERR_INVALID_ARG, "workspace must be 8-byte aligned");
    }
    p.logits = logits;
    p.logits_dtype = dtype == EMS_BF16 ? 1 : dtype == EMS_F32 ? 2 : 0;
    p.V = V;
    p.partial = static_cast<ems::ArgmaxPartial*>(workspace);
    p.target_ids = target_ids;
    p.input_ids = input_ids;
    p.cu = cu_seqlens;
    p.B = B;
    p.T = T;
    p.accepted = accepted;
    p.accepted_cu = accepted_cu;
    p.out_tokens = out_tokens;
    p.parent = parent;
    p.accepted_rows = accepted_rows;
    return EMS_OK;
}

ems_status run_accept(const void* logits, ems_dtype dtype, int V, int32_t* target_ids,
                      const int32_t* input_ids, const int32_t* parent, const int32_t* cu_seqlens,
                      int B, int T, int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens,
                      int32_t* accepted_rows, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
    ems::AcceptParams p;
    const ems_status st = prepare_accept(logits, dtype, V, target_ids, input_ids, parent, cu_seqlens, B, T, accepted,
                                         accepted_cu, out_tokens, accepted_rows, workspace, workspace_bytes, &p);
    if (st != EMS_OK) return st;
    hipError_t e = ems::launch_greedy_accept(p, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail("accept launch", e);
    return EMS_OK;
}

ems_status check_append(const void* const* k_new_layers, const void* const* v_new_layers,
                        const ems_kv_cache* caches, int n_layers, const int32_t* kv_start,
                        const int32_t* kv_len, int B, int T, int H, int D, ems_dtype dtype);
void fill_append(ems::AppendParams& p, const void* const* k_new_layers, const void* const* v_new_layers,
                 const ems_kv_cache* caches, int l0, int n, const int32_t* cu_seqlens, const int32_t* accepted,
                 const int32_t* rows, const int32_t* rows_cu, const int32_t* kv_start, const int32_t* kv_len,
                 int32_t* kv_len_out, int B, int T, int H, int D);
// Shared by ems_kv_append (rows == nullptr) and ems_kv_append_rows (cu_seqlens, accepted unused).
ems_status run_append(const void* const* k_new_layers, const void* const* v_new_layers,
                      const ems_kv_cache* caches, int n_layers, const int32_t* cu_seqlens,
                      const int32_t* accepted, const int32_t* rows, const int32_t* rows_cu,
                      const int32_t* kv_start, const int32_t* kv_len, int32_t* kv_len_out, int B,
                      int T, int H, int D, ems_dtype dtype, void* hip_stream);

}  // namespace

extern "C" {

ems_status ems_greedy_accept(const void* logits, ems_dtype dtype, int V, int32_t* target_ids,
                             const int32_t* input_ids, const int32_t* cu_seqlens, int B, int T,
                             int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run_accept(logits, dtype, V, target_ids, input_ids, nullptr, cu_seqlens, B, T, accepted,
                      accepted_cu, out_tokens, nullptr, workspace, workspace_bytes, hip_stream);
}

ems_status ems_tree_accept(const void* logits, ems_dtype dtype, int V, int32_t* target_ids,
                           const int32_t* input_ids, const int32_t* parent,
                           const int32_t* cu_seqlens, int B, int T, int32_t* accepted,
                           int32_t* accepted_cu, int32_t* out_tokens, int32_t* accepted_rows,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (T > 0 && !parent) return fail(EMS_ERR_INVALID_ARG, "parent must not be NULL");
    return run_accept(logits, dtype, V, target_ids, input_ids, parent, cu_seqlens, B, T, accepted,
                      accepted_cu, out_tokens, accepted_rows, workspace, workspace_bytes, hip_stream);
}

ems_status ems_kv_append(const void* const* k_new_layers, const void* const* v_new_layers,
                         const ems_kv_cache* caches, int n_layers, const int32_t* cu_seqlens,
                         const int32_t* accepted, const int32_t* kv_start, const int32_t* kv_len,
                         int32_t* kv_len_out, int B, int T, int H, int D, ems_dtype dtype,
                         void* hip_stream) {
    if (!cu_seqlens || !accepted)
        return fail(EMS_ERR_INVALID_ARG, "cu_seqlens, accepted, kv_start and kv_len must not be NULL");
    return run_append(k_new_layers, v_new_layers, caches, n_layers, cu_seqlens, accepted, nullptr,
                      nullptr, kv_start, kv_len, kv_len_out, B, T, H, D, dtype, hip_stream);
}

ems_status ems_greedy_accept_append(const void* logits, ems_dtype logits_dtype, int V, int32_t* target_ids,
                                    const int32_t* input_ids, const int32_t* cu_seqlens, int B, int T,
                                    int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens,
                                    void* workspace, size_t workspace_bytes,
                                    const void* const* k_new_layers, const void* const* v_new_layers,
                                    const ems_kv_cache* caches, int n_layers, const int32_t* kv_start,
                                    const int32_t* kv_len, int32_t* kv_len_out, int H, int D,
                                    ems_dtype dtype, void* hip_stream) {
    // every argument is checked before anything is launched
    ems::AcceptParams pa;
    ems_status st = prepare_accept(logits, logits_dtype, V, target_ids, input_ids, nullptr, cu_seqlens, B, T,
                                   accepted, accepted_cu, out_tokens, nullptr, workspace, workspace_bytes, &pa);
    if (st != EMS_OK) return st;
    st = check_append(k_new_layers, v_new_layers, caches, n_layers, kv_start, kv_len, B, T, H, D, dtype);
    if (st != EMS_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // One launch finds the counts and copies the rows, unless the lengths are updated in place
    // (the copying blocks still read them), the layers need several launches, or there is nothing
    // to copy: then the two calls run one after the other.
    if (T == 0 || n_layers > ems::kMaxLayersPerLaunch || kv_len_out == kv_len) {
        hipError_t e = ems::launch_greedy_accept(pa, stream);
        if (e != hipSuccess) return hip_fail("accept launch", e);
        return run_append(k_new_layers, v_new_layers, caches, n_layers, cu_seqlens, accepted, nullptr, nullptr,
                          kv_start, kv_len, kv_len_out, B, T, H, D, dtype, hip_stream);
    }
    ems::AppendParams pp;
    fill_append(pp, k_new_layers, v_new_layers, caches, 0, n_layers, cu_seqlens, nullptr, nullptr, nullptr,
                kv_start, kv_len, kv_len_out, B, T, H, D);
    hipError_t e = ems::launch_accept_append(pa, pp, stream);
    if (e != hipSuccess) return hip_fail("accept and append launch", e);
    return EMS_OK;
}

ems_status ems_kv_append_rows(const void* const* k_new_layers, const void* const* v_new_layers,
                              const ems_kv_cache* caches, int n_layers, const int32_t* accepted_rows,
                              const int32_t* accepted_cu, const int32_t* kv_start,
                              const int32_t* kv_len, int32_t* kv_len_out, int B, int T, int H, int D,
                              ems_dtype dtype, void* hip_stream) {
    if (!accepted_rows || !accepted_cu)
        return fail(EMS_ERR_INVALID_ARG, "accepted_rows and accepted_cu must not be NULL");
    return run_append(k_new_layers, v_new_layers, caches, n_layers, nullptr, nullptr, accepted_rows,
                      accepted_cu, kv_start, kv_len, kv_len_out, B, T, H, D, dtype, hip_stream);
}

}  // extern "C"

namespace {

ems_status check_append(const void* const* k_new_layers, const void* const* v_new_layers,
                        const ems_kv_cache* caches, int n_layers, const int32_t* kv_start,
                        const int32_t* kv_len, int B, int T, int H, int D, ems_dtype dtype) {
    if (n_layers < 1) return fail(EMS_ERR_INVALID_ARG, "n_layers = %d, need n_layers >= 1", n_layers);
    if (B < 1) return fail(EMS_ERR_INVALID_ARG, "B = %d, need B >= 1", B);
    if (B > 65535 * 32) return fail(EMS_ERR_UNSUPPORTED, "B = %d is too large", B);
    if (T < 0) return fail(EMS_ERR_INVALID_ARG, "T = %d, need T >= 0", T);
    if (H < 1) return fail(EMS_ERR_INVALID_ARG, "H = %d, need H >= 1", H);
    if (D < 8 || (D & 7)) return fail(EMS_ERR_INVALID_ARG, "D = %d, need a positive multiple of 8", D);
    if (!dtype16(dtype)) return fail(EMS_ERR_INVALID_ARG, "dtype must be EMS_F16 or EMS_BF16");
    if (!k_new_layers || !v_new_layers || !caches)
        return fail(EMS_ERR_INVALID_ARG, "layer arrays must not be NULL");
    if (!kv_start || !kv_len)
        return fail(EMS_ERR_INVALID_ARG, "cu_seqlens, accepted, kv_start and kv_len must not be NULL");
    for (int l = 0; l < n_layers; ++l) {
        const ems_kv_cache& c = caches[l];
        if (T > 0 && (!k_new_layers[l] || !v_new_layers[l] || !c.k || !c.v))
            return fail(EMS_ERR_INVALID_ARG, "layer %d: NULL tensor", l);
        if (!aligned16(k_new_layers[l]) || !aligned16(v_new_layers[l]) || !aligned16(c.k) || !aligned16(c.v))
            return fail(EMS_ERR_INVALID_ARG, "layer %d: tensors must be 16-byte aligned", l);
        if (c.row_stride < D || c.head_stride < D || (c.row_stride & 7) || (c.head_stride & 7))
            return fail(EMS_ERR_INVALID_ARG, "layer %d: cache strides must be multiples of 8 elements and at least D", l);
    }
    return EMS_OK;
}

// The parameters of one append launch: layers l0 .. l0 + n - 1.
void fill_append(ems::AppendParams& p, const void* const* k_new_layers, const void* const* v_new_layers,
                 const ems_kv_cache* caches, int l0, int n, const int32_t* cu_seqlens, const int32_t* accepted,
                 const int32_t* rows, const int32_t* rows_cu, const int32_t* kv_start, const int32_t* kv_len,
                 int32_t* kv_len_out, int B, int T, int H, int D) {
    std::memset(&p, 0, sizeof p);
    p.n_layers = n;
    for (int l = 0; l < n; ++l) {
        ems::AppendLayer& ly = p.layer[l];
        ly.k_new = static_cast<const char*>(k_new_layers[l0 + l]);
        ly.v_new = static_cast<const char*>(v_new_layers[l0 + l]);
        ly.k_cache = static_cast<char*>(caches[l0 + l].k);
        ly.v_cache = static_cast<char*>(caches[l0 + l].v);
        ly.row_stride_b = caches[l0 + l].row_stride * 2;
        ly.head_stride_b = caches[l0 + l].head_stride * 2;
    }
    p.cu = cu_seqlens;
    p.accepted = accepted;
    p.rows = rows;
    p.rows_cu = rows_cu;
    p.T = T;
    p.kv_start = kv_start;
    p.kv_len = kv_len;
    p.kv_len_out = kv_len_out;
    p.B = B;
    p.H = H;
    p.vec_per_head = D / 8;
}

ems_status run_append(const void* const* k_new_layers, const void* const* v_new_layers,
                      const ems_kv_cache* caches, int n_layers, const int32_t* cu_seqlens,
                      const int32_t* accepted, const int32_t* rows, const int32_t* rows_cu,
                      const int32_t* kv_start, const int32_t* kv_len, int32_t* kv_len_out, int B,
                      int T, int H, int D, ems_dtype dtype, void* hip_stream) {
    const ems_status st = check_append(k_new_layers, v_new_layers, caches, n_layers, kv_start, kv_len, B, T, H, D, dtype);
    if (st != EMS_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // kv_len_out is written by the first copy launch unless it aliases kv_len
    bool lengths_pending = kv_len_out != nullptr;
    const bool in_place = kv_len_out == kv_len;
    if (T > 0) {
        for (int l0 = 0; l0 < n_layers; l0 += ems::kMaxLayersPerLaunch) {
            ems::AppendParams p;
            fill_append(p, k_new_layers, v_new_layers, caches, l0, std::min(ems::kMaxLayersPerLaunch, n_layers - l0),
                        cu_seqlens, accepted, rows, rows_cu, kv_start, kv_len,
                        (lengths_pending && !in_place) ? kv_len_out : nullptr, B, T, H, D);
            hipError_t e = ems::launch_kv_append(p, stream);
            if (e != hipSuccess) return hip_fail("ems_kv_append launch", e);
            if (!in_place) lengths_pending = false;
        }
    }
    if (lengths_pending) {
        hipError_t e = ems::launch_advance_kv_len(kv_len, accepted, rows_cu, kv_len_out, B, stream);
        if (e != hipSuccess) return hip_fail("ems_kv_append length update launch", e);
    }
    return EMS_OK;
}

}  // namespace

extern "C" {

ems_status ems_padded_kv_append(const void* const* k_new_pad_layers,
                                const void* const* v_new_pad_layers, const ems_kv_cache* caches,
                                int n_layers, int64_t cap, uint8_t* key_mask,
                                const int32_t* accepted, int B, int k_max, int l_pad, int tau_max,
                                int H, int D, ems_dtype dtype, void* hip_stream) {
    if (n_layers < 1) return fail(EMS_ERR_INVALID_ARG, "n_layers = %d, need n_layers >= 1", n_layers);
    if (B < 1 || B > 65535 * 32) return fail(EMS_ERR_INVALID_ARG, "B = %d out of range", B);
    if (H < 1) return fail(EMS_ERR_INVALID_ARG, "H = %d, need H >= 1", H);
    if (D < 8 || (D & 7)) return fail(EMS_ERR_INVALID_ARG, "D = %d, need a positive multiple of 8", D);
    if (!dtype16(dtype)) return fail(EMS_ERR_INVALID_ARG, "dtype must be EMS_F16 or EMS_BF16");
    if (k_max < 1 || tau_max < 0 || tau_max > k_max)
        return fail(EMS_ERR_INVALID_ARG, "need 0 <= tau_max (%d) <= k_max (%d)", tau_max, k_max);
    if (l_pad < 0 || cap < (int64_t)l_pad + tau_max)
        return fail(EMS_ERR_INVALID_ARG, "l_pad + tau_max = %lld exceeds cap = %lld",
                    (long long)l_pad + tau_max, (long long)cap);
    if (!k_new_pad_layers || !v_new_pad_layers || !caches || !key_mask || !accepted)
        return fail(EMS_ERR_INVALID_ARG, "NULL argument");
    for (int l = 0; l < n_layers; ++l) {
        const ems_kv_cache& c = caches[l];
        if (!k_new_pad_layers[l] || !v_new_pad_layers[l] || !c.k || !c.v)
            return fail(EMS_ERR_INVALID_ARG, "layer %d: NULL tensor", l);
        if (!aligned16(k_new_pad_layers[l]) || !aligned16(v_new_pad_layers[l]) || !aligned16(c.k) || !aligned16(c.v))
            return fail(EMS_ERR_INVALID_ARG, "layer %d: tensors must be 16-byte aligned", l);
        if (c.row_stride < D || c.head_stride < D || (c.row_stride & 7) || (c.head_stride & 7))
            return fail(EMS_ERR_INVALID_ARG, "layer %d: cache strides must be multiples of 8 elements and at least D", l);
        if (c.rows < (int64_t)B * cap)
            return fail(EMS_ERR_INVALID_ARG, "layer %d: cache holds fewer than B * cap rows", l);
    }
    if (tau_max == 0) return EMS_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (int l0 = 0; l0 < n_layers; l0 += ems::kMaxLayersPerLaunch) {
        ems::PaddedAppendParams p;
        std::memset(&p, 0, sizeof p);
        p.n_layers = std::min(ems::kMaxLayersPerLaunch, n_layers - l0);
        for (int l = 0; l < p.n_layers; ++l) {
            ems::AppendLayer& ly = p.layer[l];
            ly.k_new = static_cast<const char*>(k_new_pad_layers[l0 + l]);
            ly.v_new = static_cast<const char*>(v_new_pad_layers[l0 + l]);
            ly.k_cache = static_cast<char*>(caches[l0 + l].k);
            ly.v_cache = static_cast<char*>(caches[l0 + l].v);
            ly.row_stride_b = caches[l0 + l].row_stride * 2;
            ly.head_stride_b = caches[l0 + l].head_stride * 2;
        }
        p.key_mask = key_mask;
        p.accepted = accepted;
        p.B = B;
        p.H = H;
        p.vec_per_head = D / 8;
        p.k_max = k_max;
        p.l_pad = l_pad;
        p.tau_max = tau_max;
        p.cap = cap;
        hipError_t e = ems::launch_padded_kv_append(p, stream);
        if (e != hipSuccess) return hip_fail("ems_padded_kv_append launch", e);
    }
    return EMS_OK;
}

ems_status ems_pack_tokens(const int32_t* padded_ids, const int32_t* token_nums, int B, int k_max,
                           int32_t* cu_seqlens, int32_t* packed_ids, void* hip_stream) {
    if (B < 1) return fail(EMS_ERR_INVALID_ARG, "B = %d, need B >= 1", B);
    if (B > kMaxB) return fail(EMS_ERR_UNSUPPORTED, "B = %d, at most %d samples", B, kMaxB);
    if (k_max < 0) return fail(EMS_ERR_INVALID_ARG, "k_max = %d, need k_max >= 0", k_max);
    if (!token_nums || !cu_seqlens) return fail(EMS_ERR_INVALID_ARG, "token_nums and cu_seqlens must not be NULL");
    if (k_max > 0 && (!padded_ids || !packed_ids))
        return fail(EMS_ERR_INVALID_ARG, "padded_ids and packed_ids must not be NULL");
    ems::PackParams p;
    p.padded_ids = padded_ids;
    p.token_nums = token_nums;
    p.cu = cu_seqlens;
    p.packed_ids = packed_ids;
    p.B = B;
    p.k_max = k_max;
    hipError_t e = ems::launch_pack_tokens(p, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail("ems_pack_tokens launch", e);
    return EMS_OK;
}

ems_status ems_stream_read_probe(const void* buf, size_t bytes, void* sink, void* hip_stream) {
    if (!buf || !sink) return fail(EMS_ERR_INVALID_ARG, "buf and sink must not be NULL");
    if (!aligned16(buf) || (reinterpret_cast<uintptr_t>(sink) & 3) != 0)
        return fail(EMS_ERR_INVALID_ARG, "buf must be 16-byte aligned, sink 4-byte aligned");
    if (bytes < 1024) return fail(EMS_ERR_INVALID_ARG, "bytes = %zu is less than one 1 KiB line", bytes);
    // one workgroup of four waves per CU, the attention kernel's own launch shape: measured 7.1 TB/s
    // where 2, 4 and 8 workgroups per CU gave 7.0, 6.9 and 6.7
    hipError_t e = ems::launch_stream_read(buf, bytes, static_cast<uint32_t*>(sink), resident_attn_blocks(),
                                           static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail("stream probe launch", e);
    return EMS_OK;
}

ems_status ems_set_attention_variant(int variant) {
    if (variant != EMS_ATTN_MFMA && variant != EMS_ATTN_VALU)
        return fail(EMS_ERR_INVALID_ARG, "attention variant %d is neither EMS_ATTN_MFMA nor EMS_ATTN_VALU", variant);
    g_attn_variant = variant;
    return EMS_OK;
}

int ems_get_attention_variant(void) { return g_attn_variant; }

ems_status ems_profile_enable(int max_records) {
    for (auto* evs : {&g_prof.start, &g_prof.stop, &g_prof.end}) {
        for (hipEvent_t ev : *evs) (void)hipEventDestroy(ev);
        evs->clear();
    }
    g_prof.used = 0;
    if (max_records < 0 || max_records > 65536)
        return fail(EMS_ERR_INVALID_ARG, "max_records = %d outside [0, 65536]", max_records);
    for (int i = 0; i < max_records; ++i) {
        for (auto* evs : {&g_prof.start, &g_prof.stop, &g_prof.end}) {
            hipEvent_t ev = nullptr;
            hipError_t e = hipEventCreate(&ev);
            if (e != hipSuccess) return hip_fail("hipEventCreate", e);
            evs->push_back(ev);
        }
    }
    return EMS_OK;
}

ems_status ems_profile_read_calls(double* total_ms, double* total_call_ms, int* launches) {
    if (!total_ms || !launches) return fail(EMS_ERR_INVALID_ARG, "total_ms and launches must not be NULL");
    double sum = 0.0, sum_call = 0.0;
    for (int i = 0; i < g_prof.used; ++i) {
        hipError_t e = hipEventSynchronize(g_prof.end[i]);
        float ms = 0.f, ms_call = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms_call, g_prof.start[i], g_prof.end[i]);
        if (e != hipSuccess) return hip_fail("ems_profile_read", e);
        sum += ms;
        sum_call += ms_call;
    }
    *total_ms = sum;
    if (total_call_ms) *total_call_ms = sum_call;
    *launches = g_prof.used;
    g_prof.used = 0;
    return EMS_OK;
}

ems_status ems_profile_read(double* total_ms, int* launches) {
    return ems_profile_read_calls(total_ms, nullptr, launches);
}

ems_status ems_validate_inputs(const int32_t* cu_seqlens, const int32_t* kv_start,
                               const int32_t* kv_len, int B, int T, int max_k, int max_kv_len,
                               int64_t rows, void* hip_stream) {
    if (B < 1 || T < 0 || max_k < 0 || max_kv_len < 0 || rows < 0)
        return fail(EMS_ERR_INVALID_ARG, "negative size (B=%d T=%d max_k=%d max_kv_len=%d)", B, T, max_k, max_kv_len);
    if (!cu_seqlens || !kv_start || !kv_len)
        return fail(EMS_ERR_INVALID_ARG, "cu_seqlens, kv_start and kv_len must not be NULL");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    std::vector<int32_t> cu(B + 1), ks(B), kl(B);
    hipError_t e = hipMemcpyAsync(cu.data(), cu_seqlens, sizeof(int32_t) * (B + 1), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(ks.data(), kv_start, sizeof(int32_t) * B, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(kl.data(), kv_len, sizeof(int32_t) * B, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_fail("ems_validate_inputs copy", e);
    if (cu[0] != 0) return fail(EMS_ERR_INVALID_ARG, "cu_seqlens[0] = %d, must be 0", cu[0]);
    if (cu[B] != T) return fail(EMS_ERR_INVALID_ARG, "cu_seqlens[B] = %d, must equal T = %d", cu[B], T);
    std::vector<std::pair<int64_t, int64_t>> regions;
    for (int i = 0; i < B; ++i) {
        const int k = cu[i + 1] - cu[i];
        if (k < 0) return fail(EMS_ERR_INVALID_ARG, "cu_seqlens decreases at sample %d", i);
        if (k > max_k) return fail(EMS_ERR_INVALID_ARG, "sample %d has %d rows, max_k = %d", i, k, max_k);
        if (kl[i] < 0 || kl[i] > max_kv_len)
            return fail(EMS_ERR_INVALID_ARG, "kv_len[%d] = %d outside [0, %d]", i, kl[i], max_kv_len);
        if (ks[i] < 0) return fail(EMS_ERR_INVALID_ARG, "kv_start[%d] = %d is negative", i, ks[i]);
        if ((int64_t)ks[i] + kl[i] + k > rows)
            return fail(EMS_ERR_INVALID_ARG, "sample %d: kv_start+kv_len+k = %lld exceeds the arena's %lld rows",
                        i, (long long)ks[i] + kl[i] + k, (long long)rows);
        if (kl[i] + k > 0) regions.emplace_back((int64_t)ks[i], (int64_t)ks[i] + kl[i] + k);
    }
    std::sort(regions.begin(), regions.end());
    for (size_t r = 1; r < regions.size(); ++r)
        if (regions[r].first < regions[r - 1].second)
            return fail(EMS_ERR_INVALID_ARG, "cache regions overlap near row %lld", (long long)regions[r].first);
    return EMS_OK;
}

ems_status ems_validate_tree(const int32_t* cu_seqlens, const int32_t* parent, int B, int T,
                             void* hip_stream) {
    if (B < 1 || T < 0) return fail(EMS_ERR_INVALID_ARG, "B = %d, T = %d out of range", B, T);
    if (!cu_seqlens || (T > 0 && !parent)) return fail(EMS_ERR_INVALID_ARG, "cu_seqlens and parent must not be NULL");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    std::vector<int32_t> cu(B + 1), par(T);
    hipError_t e = hipMemcpyAsync(cu.data(), cu_seqlens, sizeof(int32_t) * (B + 1), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess && T > 0)
        e = hipMemcpyAsync(par.data(), parent, sizeof(int32_t) * T, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_fail("ems_validate_tree copy", e);
    if (cu[0] != 0 || cu[B] != T)
        return fail(EMS_ERR_INVALID_ARG, "cu_seqlens must run from 0 to T = %d (got %d .. %d)", T, cu[0], cu[B]);
    for (int i = 0; i < B; ++i) {
        const int k = cu[i + 1] - cu[i];
        if (k < 0 || cu[i + 1] > T) return fail(EMS_ERR_INVALID_ARG, "cu_seqlens decreases or overruns at sample %d", i);
        for (int j = 0; j < k; ++j) {
            const int pj = par[cu[i] + j];
            if (j == 0 ? pj != -1 : (pj < 0 || pj >= j))
                return fail(EMS_ERR_INVALID_ARG, "sample %d, row %d: parent = %d (row 0 needs -1, row j a value in [0, j))",
                            i, j, pj);
        }
    }
    return EMS_OK;
}

}  // extern "C"
