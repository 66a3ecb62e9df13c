// Stand-ins for the kernel launchers of libems, so that the host layer of the C ABI (argument
// validation, launch sizing, parameter marshalling: the host side of csrc/ems_api.hip)
// can run to the end of every entry point on a machine without a GPU, under the address
// and undefined-behaviour sanitizers.  Nothing is launched; each stand-in checks the few
// facts a real launch relies on and counts the call.  Test infrastructure only.
#include <cstdlib>
#include <cstdio>

#include "../../paper_2405_07542_amd/csrc/ems_kernels.h"

extern "C" int ems_stub_launches = 0;

#define STUB_CHECK(c) do { if (!(c)) { std::fprintf(stderr, "launch stub: %s violated\n", #c); std::abort(); } } while (0)

namespace ems {

size_t valu_attention_lds_bytes(int B, int D) { return (size_t)(B + 1) * 4 + 4 * (size_t)(D == 128 ? 36 : 19) * 1024; }
bool wide_rows64_fits(int B, int D) { return (size_t)B * 4 + (D >= 128 ? 136 : 72) * 1024u <= (size_t)kMaxLdsBytes; }

hipError_t launch_verify_attention(const AttnParams& p, int blocks, int D, bool, bool padded, bool, hipStream_t,
                                   hipEvent_t, hipEvent_t) {
    STUB_CHECK(blocks >= 1 && blocks <= 1024 && p.num_waves == 4 * blocks);
    STUB_CHECK(D == 64 || D == 80 || D == 128);
    STUB_CHECK(p.B >= 1 && p.H >= 1 && p.q && p.out && p.ws && p.ws_header);
    STUB_CHECK(padded ? (p.key_mask && p.k_valid) : (p.cu && p.kv_start && p.kv_len));
    STUB_CHECK((const char*)p.ws > (const char*)p.ws_header);
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_verify_attention_wide(const AttnParams&, int, int, bool, hipStream_t, hipEvent_t, hipEvent_t) {
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_greedy_accept(const AcceptParams& p, hipStream_t) {
    STUB_CHECK(p.B >= 1 && p.T >= 0);
    if (p.logits) STUB_CHECK(p.slices >= 1 && p.slice_len >= 8 && (p.slice_len % 8) == 0 &&
                             (long long)p.slices * p.slice_len >= p.V && (p.partial || p.T == 0));
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_kv_append(const AppendParams& p, hipStream_t) {
    STUB_CHECK(p.n_layers >= 1 && p.n_layers <= kMaxLayersPerLaunch);
    for (int l = 0; l < p.n_layers; ++l) STUB_CHECK(p.layer[l].k_new && p.layer[l].k_cache && p.layer[l].row_stride_b > 0);
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_accept_append(const AcceptParams& pa, const AppendParams& pp, hipStream_t) {
    STUB_CHECK(pa.B >= 1 && pa.T >= 1 && pa.B == pp.B && pa.parent == nullptr && pa.cu == pp.cu);
    STUB_CHECK(pp.n_layers >= 1 && pp.n_layers <= kMaxLayersPerLaunch && pp.rows == nullptr && pp.kv_len_out != pp.kv_len);
    for (int l = 0; l < pp.n_layers; ++l) STUB_CHECK(pp.layer[l].k_new && pp.layer[l].k_cache && pp.layer[l].row_stride_b > 0);
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_padded_kv_append(const PaddedAppendParams& p, hipStream_t) {
    STUB_CHECK(p.n_layers >= 1 && p.n_layers <= kMaxLayersPerLaunch && p.tau_max >= 1);
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_advance_kv_len(const int32_t* kv_len, const int32_t*, const int32_t*, int32_t* out, int B, hipStream_t) {
    STUB_CHECK(kv_len && out && B >= 1);
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_pack_tokens(const PackParams& p, hipStream_t) {
    STUB_CHECK(p.B >= 1 && p.cu && p.token_nums);
    ++ems_stub_launches;
    return hipSuccess;
}
hipError_t launch_stream_read(const void* buf, uint64_t bytes, uint32_t* sink, int blocks, hipStream_t) {
    STUB_CHECK(buf && sink && bytes >= 1024 && blocks >= 1);
    ++ems_stub_launches;
    return hipSuccess;
}

}  // namespace ems
