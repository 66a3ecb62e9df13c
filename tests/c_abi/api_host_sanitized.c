/* Host layer of the C ABI under -fsanitize=address,undefined, without a GPU: this program is
 * linked with csrc/ems_api.hip (its host side instrumented) and with launch_stubs.cpp in place of
 * the kernels.  It walks every entry point down both its refusals (bad scalars, NULL or
 * misaligned pointers, small workspaces) and its accepted paths (to the launch, which the
 * stubs count), with host arrays sized exactly.  Device pointers are never dereferenced by
 * the host layer, so plain aligned fake addresses serve.  Exit code 0 and "ok" = clean. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ems.h"
#include "ems_measure.h"

extern int ems_stub_launches;

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d): %s\n", #c, __LINE__, ems_last_error_string()); exit(1); } } while (0)
#define FAKE ((void*)0x10000)
#define FAKE32 ((int32_t*)0x10000)

static ems_status attention(int B, int T, int H, int D, int max_k, int max_kv_len, size_t ws_bytes, void* ws,
                            const ems_kv_cache* cache, int variant) {
    if (variant == 1)
        return ems_verify_attention_write_through(FAKE, FAKE, FAKE, cache, FAKE32, FAKE32, FAKE32, FAKE, EMS_F32, B, T,
                                                  H, D, max_k, max_kv_len, 0.1f, EMS_BF16, ws, ws_bytes, NULL);
    if (variant == 2)
        return ems_tree_verify_attention(FAKE, FAKE, FAKE, cache, FAKE32, FAKE32, FAKE32, FAKE32, FAKE, EMS_F16, B, T,
                                         H, D, max_k, max_kv_len, 0.1f, EMS_F16, ws, ws_bytes, NULL);
    return ems_verify_attention(FAKE, FAKE, FAKE, cache, FAKE32, FAKE32, FAKE32, FAKE, EMS_F16, B, T, H, D, max_k,
                                max_kv_len, 0.1f, EMS_F16, ws, ws_bytes, NULL);
}

int main(void) {
    ems_kv_cache cache = {FAKE, FAKE, 32 * 128, 128, 1 << 20};
    /* workspace sizes: host arithmetic, monotone in the bounds, both names agree */
    CHECK(ems_workspace_bytes(64, 384, 32, 128, 2048) == ems_attention_workspace_bytes(64, 384, 32, 128, 2048));
    CHECK(ems_workspace_bytes(0, 0, 0, 0, 0) >= 256 && ems_workspace_bytes(1, 1, 1, 64, 0) >= 256);
    CHECK(ems_workspace_bytes(8192, 65535, 64, 128, 1 << 17) >= ems_workspace_bytes(64, 384, 32, 128, 2048));
    CHECK(ems_accept_workspace_bytes(0, 50272) == 0 && ems_accept_workspace_bytes(384, 50272) >= 384 * 8);

    /* attention: every shape class reaches its launch with the advertised workspace */
    const int shapes[][6] = {{64, 384, 32, 128, 11, 2048}, {8, 28, 32, 128, 6, 1024}, {1, 1, 1, 64, 1, 0},
                             {128, 448, 40, 80, 6, 4096}, {64, 2048, 32, 128, 32, 2048}, {64, 4096, 32, 128, 64, 2048},
                             {8192, 8192, 2, 64, 64, 40}, {3, 48, 4, 64, 16, 300000}};
    for (size_t s = 0; s < sizeof shapes / sizeof shapes[0]; ++s)
        for (int variant = 0; variant < 3; ++variant) {
            const int* a = shapes[s];
            const size_t need = ems_workspace_bytes(a[0], a[1], a[2], a[3], a[5]);
            const int before = ems_stub_launches;
            CHECK(attention(a[0], a[1], a[2], a[3], a[4], a[5], need, FAKE, &cache, variant) == EMS_OK);
            CHECK(ems_stub_launches == before + 1);
            CHECK(attention(a[0], a[1], a[2], a[3], a[4], a[5], 64, FAKE, &cache, variant) == EMS_ERR_WORKSPACE);
            CHECK(attention(a[0], a[1], a[2], a[3], a[4], a[5], need, NULL, &cache, variant) == EMS_ERR_WORKSPACE);
        }
    CHECK(attention(0, 8, 32, 128, 4, 100, 1 << 30, FAKE, &cache, 0) == EMS_ERR_INVALID_ARG);
    CHECK(attention(4, -1, 32, 128, 4, 100, 1 << 30, FAKE, &cache, 0) == EMS_ERR_INVALID_ARG);
    CHECK(attention(4, 8, 32, 96, 4, 100, 1 << 30, FAKE, &cache, 1) == EMS_ERR_UNSUPPORTED);
    CHECK(attention(4, 8, 32, 128, 65, 100, 1 << 30, FAKE, &cache, 2) == EMS_ERR_UNSUPPORTED);
    CHECK(attention(9000, 8, 32, 128, 4, 100, 1 << 30, FAKE, &cache, 0) == EMS_ERR_UNSUPPORTED);
    CHECK(attention(4, 8, 32, 128, 4, 1 << 20, 1 << 30, FAKE, &cache, 0) == EMS_ERR_UNSUPPORTED);
    CHECK(attention(4, 8, 32, 128, 4, 100, 1 << 30, FAKE, NULL, 0) == EMS_ERR_INVALID_ARG);
    CHECK(attention(4, 0, 32, 128, 4, 100, 0, NULL, &cache, 0) == EMS_OK);          /* no rows: a no-op */
    CHECK(strlen(ems_last_error_string()) > 0);

    /* the vector-ALU formulation is this thread's own switch */
    CHECK(ems_set_attention_variant(EMS_ATTN_VALU) == EMS_OK && ems_get_attention_variant() == EMS_ATTN_VALU);
    CHECK(attention(64, 384, 32, 128, 11, 2048, 1 << 30, FAKE, &cache, 0) == EMS_OK);
    CHECK(attention(64, 384, 32, 128, 32, 2048, 1 << 30, FAKE, &cache, 0) == EMS_ERR_UNSUPPORTED);
    CHECK(attention(64, 384, 32, 128, 11, 2048, 1 << 30, FAKE, &cache, 2) == EMS_ERR_UNSUPPORTED);
    CHECK(ems_set_attention_variant(7) == EMS_ERR_INVALID_ARG && ems_set_attention_variant(EMS_ATTN_MFMA) == EMS_OK);

    /* padded ablation */
    CHECK(ems_padded_verify_attention(FAKE, FAKE, FAKE, &cache, 2048, (const uint8_t*)FAKE, FAKE32, FAKE, EMS_F16, 64,
                                      11, 2040, 32, 128, 0.1f, EMS_F16, FAKE,
                                      ems_workspace_bytes(64, 64 * 11, 32, 128, 2040), NULL) == EMS_OK);
    CHECK(ems_padded_verify_attention(FAKE, FAKE, FAKE, &cache, 2047, (const uint8_t*)FAKE, FAKE32, FAKE, EMS_F16, 64,
                                      11, 2040, 32, 128, 0.1f, EMS_F16, FAKE, 1 << 30, NULL) == EMS_ERR_INVALID_ARG);

    /* accept */
    int before = ems_stub_launches;
    CHECK(ems_greedy_accept(FAKE, EMS_BF16, 50272, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, FAKE32, FAKE,
                            ems_accept_workspace_bytes(384, 50272), NULL) == EMS_OK);
    CHECK(ems_greedy_accept(NULL, EMS_F16, 0, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, NULL, NULL, 0, NULL) == EMS_OK);
    CHECK(ems_tree_accept(FAKE, EMS_F32, 128256, FAKE32, FAKE32, FAKE32, FAKE32, 8, 65535, FAKE32, FAKE32, FAKE32,
                          FAKE32, FAKE, ems_accept_workspace_bytes(65535, 128256), NULL) == EMS_OK);
    CHECK(ems_stub_launches == before + 3);
    CHECK(ems_greedy_accept(FAKE, EMS_BF16, 50272, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, FAKE32, FAKE, 8,
                            NULL) == EMS_ERR_WORKSPACE);
    CHECK(ems_greedy_accept(FAKE, EMS_BF16, 50272, FAKE32, FAKE32, FAKE32, 64, 70000, FAKE32, FAKE32, FAKE32, FAKE,
                            1 << 30, NULL) == EMS_ERR_UNSUPPORTED);

    /* append: 70 layers go out in three launches; the host arrays hold exactly 70 entries */
    enum { LAYERS = 70 };
    const void** knew = malloc(LAYERS * sizeof *knew);
    const void** vnew = malloc(LAYERS * sizeof *vnew);
    ems_kv_cache* caches = malloc(LAYERS * sizeof *caches);
    CHECK(knew && vnew && caches);
    for (int l = 0; l < LAYERS; ++l) { knew[l] = vnew[l] = FAKE; caches[l] = cache; }
    before = ems_stub_launches;
    CHECK(ems_kv_append(knew, vnew, caches, LAYERS, FAKE32, FAKE32, FAKE32, FAKE32, FAKE32 + 64, 64, 384, 32, 128,
                        EMS_F16, NULL) == EMS_OK);
    CHECK(ems_stub_launches == before + 3);
    before = ems_stub_launches;      /* lengths updated in place: one more, tiny launch */
    CHECK(ems_kv_append(knew, vnew, caches, LAYERS, FAKE32, FAKE32, FAKE32, FAKE32, FAKE32, 64, 384, 32, 128, EMS_F16,
                        NULL) == EMS_OK);
    CHECK(ems_stub_launches == before + 4);
    CHECK(ems_kv_append_rows(knew, vnew, caches, LAYERS, FAKE32, FAKE32, FAKE32, FAKE32, NULL, 64, 384, 32, 128,
                             EMS_BF16, NULL) == EMS_OK);
    /* acceptance and append as one call: one launch for up to 32 layers with lengths written elsewhere;
       the two calls one after the other (1 + 3 launches, + 1 for lengths in place) beyond that */
    before = ems_stub_launches;
    CHECK(ems_greedy_accept_append(NULL, EMS_F16, 0, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, NULL, NULL, 0,
                                   knew, vnew, caches, 32, FAKE32, FAKE32, FAKE32 + 64, 32, 128, EMS_F16, NULL) == EMS_OK);
    CHECK(ems_stub_launches == before + 1);
    before = ems_stub_launches;
    CHECK(ems_greedy_accept_append(FAKE, EMS_BF16, 50272, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, FAKE32, FAKE,
                                   ems_accept_workspace_bytes(384, 50272), knew, vnew, caches, LAYERS, FAKE32, FAKE32,
                                   FAKE32 + 64, 32, 128, EMS_F16, NULL) == EMS_OK);
    CHECK(ems_stub_launches == before + 4);
    before = ems_stub_launches;
    CHECK(ems_greedy_accept_append(NULL, EMS_F16, 0, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, NULL, NULL, 0,
                                   knew, vnew, caches, 1, FAKE32, FAKE32, FAKE32, 32, 128, EMS_F16, NULL) == EMS_OK);
    CHECK(ems_stub_launches == before + 3);
    before = ems_stub_launches;      /* a refused call launches nothing, whichever half refuses */
    CHECK(ems_greedy_accept_append(FAKE, EMS_BF16, 50272, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, FAKE32, FAKE, 8,
                                   knew, vnew, caches, 1, FAKE32, FAKE32, NULL, 32, 128, EMS_F16, NULL) == EMS_ERR_WORKSPACE);
    CHECK(ems_greedy_accept_append(NULL, EMS_F16, 0, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, NULL, NULL, 0,
                                   knew, vnew, caches, 1, FAKE32, NULL, NULL, 32, 128, EMS_F16, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_greedy_accept_append(NULL, EMS_F16, 0, FAKE32, FAKE32, FAKE32, 64, 384, FAKE32, FAKE32, NULL, NULL, 0,
                                   knew, vnew, caches, 1, FAKE32, FAKE32, NULL, 32, 100, EMS_F16, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_greedy_accept_append(NULL, EMS_F16, 0, FAKE32, FAKE32, NULL, 64, 384, FAKE32, FAKE32, NULL, NULL, 0,
                                   knew, vnew, caches, 1, FAKE32, FAKE32, NULL, 32, 128, EMS_F16, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_stub_launches == before);
    knew[LAYERS - 1] = NULL;
    CHECK(ems_kv_append(knew, vnew, caches, LAYERS, FAKE32, FAKE32, FAKE32, FAKE32, NULL, 64, 384, 32, 128, EMS_F16,
                        NULL) == EMS_ERR_INVALID_ARG);
    knew[LAYERS - 1] = FAKE;
    caches[LAYERS - 1].row_stride = 100;
    CHECK(ems_kv_append(knew, vnew, caches, LAYERS, FAKE32, FAKE32, FAKE32, FAKE32, NULL, 64, 384, 32, 128, EMS_F16,
                        NULL) == EMS_ERR_INVALID_ARG);
    caches[LAYERS - 1] = cache;
    CHECK(ems_padded_kv_append(knew, vnew, caches, LAYERS, 2048, (uint8_t*)FAKE, FAKE32, 64, 11, 2032, 7, 32, 128,
                               EMS_F16, NULL) == EMS_OK);
    CHECK(ems_padded_kv_append(knew, vnew, caches, LAYERS, 2048, (uint8_t*)FAKE, FAKE32, 64, 11, 2045, 7, 32, 128,
                               EMS_F16, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_kv_advance(FAKE32, FAKE32, FAKE32, 64, NULL) == EMS_OK);
    CHECK(ems_kv_advance(FAKE32, NULL, FAKE32, 64, NULL) == EMS_ERR_INVALID_ARG);
    free(knew); free(vnew); free(caches);

    CHECK(ems_pack_tokens(FAKE32, FAKE32, 64, 11, FAKE32, FAKE32, NULL) == EMS_OK);
    CHECK(ems_pack_tokens(FAKE32, NULL, 64, 11, FAKE32, FAKE32, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_stream_read_probe(FAKE, 1 << 20, FAKE, NULL) == EMS_OK);
    CHECK(ems_stream_read_probe(FAKE, 100, FAKE, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_profile_enable(-1) == EMS_ERR_INVALID_ARG && ems_profile_enable(0) == EMS_OK);
    double ms = -1.0, ms_call = -1.0;
    int launches = -1;
    CHECK(ems_profile_read_calls(&ms, &ms_call, &launches) == EMS_OK && launches == 0 && ms == 0.0 && ms_call == 0.0);
    CHECK(ems_profile_read(NULL, &launches) == EMS_ERR_INVALID_ARG);
    CHECK(ems_device_memory_figures(NULL, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_validate_inputs(FAKE32, FAKE32, FAKE32, 0, 0, 1, 1, 10, NULL) == EMS_ERR_INVALID_ARG);
    CHECK(ems_validate_tree(NULL, FAKE32, 4, 8, NULL) == EMS_ERR_INVALID_ARG);
    printf("ok %d launches reached\n", ems_stub_launches);
    return 0;
}
