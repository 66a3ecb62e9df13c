/* Memory-safety run of the CPU oracle: built together with oracle/ems_oracle.c under
 * -fsanitize=address,undefined, this program drives every oracle function over small ragged
 * inputs whose buffers are sized EXACTLY (no slack), so that a read or write one element
 * beyond any array, an overflowing index or another undefined operation ends the run with
 * a sanitizer report.  It also checks a few facts that hold for any input (weights sum to
 * one, counts in range, untouched sentinels).  Exit code 0 and "ok" = clean.
 * Test infrastructure only; no GPU, no Python. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_restore_index(const int32_t*, int, int, int32_t*, int32_t*);
int oracle_verify_attention(const uint16_t*, const uint16_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                            int64_t, int64_t, const int32_t*, const int32_t*, const int32_t*, double*, int, int,
                            int, float, int);
int oracle_argmax(const uint16_t*, int, int, int, int32_t*);
int oracle_argmax_f32(const float*, int, int, int32_t*);
int oracle_greedy_accept(const int32_t*, const int32_t*, const int32_t*, int, int32_t*, int32_t*, int32_t*);
int oracle_kv_append(uint16_t*, uint16_t*, int64_t, int64_t, const uint16_t*, const uint16_t*, const int32_t*,
                     const int32_t*, const int32_t*, const int32_t*, int32_t*, int, int, int);
int oracle_padded_verify_attention(const uint16_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                                   const uint16_t*, int64_t, int64_t, int64_t, const uint8_t*, const int32_t*,
                                   double*, int, int, int, int, int, float, int);
int oracle_padded_kv_append(uint16_t*, uint16_t*, int64_t, int64_t, int64_t, uint8_t*, const uint16_t*,
                            const uint16_t*, const int32_t*, int, int, int, int, int, int);
int oracle_kv_write_through(uint16_t*, uint16_t*, int64_t, int64_t, const uint16_t*, const uint16_t*,
                            const int32_t*, const int32_t*, const int32_t*, int, int, int);
int oracle_tree_verify_attention(const uint16_t*, const uint16_t*, const uint16_t*, const uint16_t*,
                                 const uint16_t*, int64_t, int64_t, const int32_t*, const int32_t*, const int32_t*,
                                 const int32_t*, double*, int, int, int, float, int);
int oracle_tree_accept(const int32_t*, const int32_t*, const int32_t*, const int32_t*, int, int32_t*, int32_t*,
                       int32_t*, int32_t*);
int oracle_kv_append_rows(uint16_t*, uint16_t*, int64_t, int64_t, const uint16_t*, const uint16_t*, const int32_t*,
                          const int32_t*, const int32_t*, const int32_t*, int32_t*, int, int, int);
int oracle_concatenate_tokens(const int32_t*, const int32_t*, int, int, int32_t*, int32_t*);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) {
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
/* a finite 16-bit float pattern of moderate size: sign, exponent around the bias, any mantissa */
static uint16_t rnd16(int bf16) {
    uint32_t sign = rnd() & 1u, mant = rnd();
    if (bf16) return (uint16_t)((sign << 15) | ((124u + rnd() % 5u) << 7) | (mant & 0x7fu));
    return (uint16_t)((sign << 15) | ((12u + rnd() % 5u) << 10) | (mant & 0x3ffu));
}
#define SENT 0x7e7eu
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(1); } } while (0)

static void* exact(size_t n) { void* p = malloc(n ? n : 1); CHECK(p != NULL); return p; }

static void one_batch(int bf16, int head_major) {
    enum { B = 6, H = 3, D = 64 };
    const int k[B] = {3, 0, 16, 1, 7, 2}, L[B] = {0, 33, 100, 1, 64, 5};
    int32_t cu[B + 1], start[B], len[B], T = 0, rows = 0;
    cu[0] = 0;
    for (int i = 0; i < B; ++i) {
        start[i] = rows;
        len[i] = L[i];
        rows += L[i] + k[i];                 /* room for every new row, and not one row more */
        cu[i + 1] = cu[i] + k[i];
    }
    T = cu[B];
    const int64_t rs = head_major ? D : (int64_t)H * D, hs = head_major ? (int64_t)rows * D : D;
    const size_t arena = (size_t)rows * H * D, packed = (size_t)T * H * D;
    uint16_t *kc = exact(arena * 2), *vc = exact(arena * 2), *q = exact(packed * 2), *kn = exact(packed * 2),
             *vn = exact(packed * 2);
    for (size_t e = 0; e < arena; ++e) kc[e] = vc[e] = SENT;
    for (int i = 0; i < B; ++i)
        for (int n = 0; n < L[i]; ++n)
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d) {
                    kc[(start[i] + n) * rs + h * hs + d] = rnd16(bf16);
                    vc[(start[i] + n) * rs + h * hs + d] = rnd16(bf16);
                }
    for (size_t e = 0; e < packed; ++e) { q[e] = rnd16(bf16); kn[e] = rnd16(bf16); vn[e] = rnd16(bf16); }
    double* out = exact(packed * sizeof(double));
    CHECK(oracle_verify_attention(q, kn, vn, kc, vc, rs, hs, cu, start, len, out, B, H, D, 0.125f, bf16) == 0);
    for (size_t e = 0; e < packed; ++e) CHECK(isfinite(out[e]) && fabs(out[e]) <= 32.0);   /* inside the values' hull */

    /* a token tree per sample (parent of row j: some earlier row) */
    int32_t* parent = exact((size_t)T * 4);
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < k[i]; ++j) parent[cu[i] + j] = j == 0 ? -1 : (int32_t)(rnd() % (uint32_t)j);
    CHECK(oracle_tree_verify_attention(q, kn, vn, kc, vc, rs, hs, cu, parent, start, len, out, B, H, D, 0.125f,
                                       bf16) == 0);
    for (size_t e = 0; e < packed; ++e) CHECK(isfinite(out[e]));

    /* arg-max, acceptance, running sums: V columns exactly */
    const int V = 37;
    uint16_t* logits = exact((size_t)T * V * 2);
    float* logits32 = exact((size_t)T * V * 4);
    for (size_t e = 0; e < (size_t)T * V; ++e) { logits[e] = rnd16(bf16); logits32[e] = (float)(rnd() % 1000u) - 500.f; }
    int32_t *x = exact((size_t)T * 4), *x32 = exact((size_t)T * 4), *ids = exact((size_t)T * 4);
    CHECK(oracle_argmax(logits, bf16, T, V, x) == 0 && oracle_argmax_f32(logits32, T, V, x32) == 0);
    for (int r = 0; r < T; ++r) CHECK(x[r] >= 0 && x[r] < V && x32[r] >= 0 && x32[r] < V);
    for (int r = 0; r < T; ++r) ids[r] = (r > 0 && rnd() % 10u < 7u) ? x[r - 1] : (int32_t)(rnd() % (uint32_t)V);
    int32_t acc[B], acc_cu[B + 1], *toks = exact((size_t)T * 4), *path = exact((size_t)T * 4);
    CHECK(oracle_greedy_accept(x, ids, cu, B, acc, acc_cu, toks) == 0);
    for (int i = 0; i < B; ++i) CHECK(k[i] == 0 ? acc[i] == 0 : (acc[i] >= 1 && acc[i] <= k[i]));
    CHECK(acc_cu[B] <= T);

    /* append of the accepted rows into exactly-sized arenas; write-through of all rows */
    int32_t new_len[B];
    CHECK(oracle_kv_append(kc, vc, rs, hs, kn, vn, cu, acc, start, len, new_len, B, H, D) == 0);
    for (int i = 0; i < B; ++i) {
        CHECK(new_len[i] == L[i] + acc[i]);
        for (int j = acc[i]; j < k[i]; ++j) CHECK(kc[(start[i] + L[i] + j) * rs] == SENT);   /* beyond the new length */
    }
    CHECK(oracle_kv_write_through(kc, vc, rs, hs, kn, vn, cu, start, len, B, H, D) == 0);

    /* the same through the tree calls */
    int32_t tacc[B], tacc_cu[B + 1];
    CHECK(oracle_tree_accept(x, ids, parent, cu, B, tacc, tacc_cu, toks, path) == 0);
    for (int e = 0; e < tacc_cu[B]; ++e) CHECK(path[e] >= 0 && path[e] < T);
    CHECK(oracle_kv_append_rows(kc, vc, rs, hs, kn, vn, path, tacc_cu, start, len, new_len, B, H, D) == 0);

    /* Alg. 1 / Alg. 2: packed ids and the way back, every packed row and the first row beyond */
    const int k_max = 16;
    int32_t *padded = exact((size_t)B * k_max * 4), *packed_ids = exact((size_t)T * 4), nums[B], lens[B];
    for (int e = 0; e < B * k_max; ++e) padded[e] = (int32_t)rnd();
    for (int i = 0; i < B; ++i) lens[i] = k[i];
    CHECK(oracle_concatenate_tokens(padded, lens, B, k_max, packed_ids, nums) == T);
    for (int r = 0; r < T; ++r) {
        int32_t s = -1, p = -1;
        CHECK(oracle_restore_index(nums, B, r, &s, &p) == 0 && packed_ids[r] == padded[s * k_max + p]);
    }
    int32_t s_, p_;
    CHECK(oracle_restore_index(nums, B, T, &s_, &p_) != 0);

    /* the padded (vanilla) method: aligned caches of exactly B * cap rows */
    const int l_pad = 100, cap = 128, tau_max = 7;
    const int64_t prs = head_major ? D : (int64_t)H * D, phs = head_major ? (int64_t)B * cap * D : D;
    const size_t parena = (size_t)B * cap * H * D, ppacked = (size_t)B * k_max * H * D;
    uint16_t *pkc = exact(parena * 2), *pvc = exact(parena * 2), *pq = exact(ppacked * 2), *pkn = exact(ppacked * 2),
             *pvn = exact(ppacked * 2);
    uint8_t* mask = exact((size_t)B * cap);
    int32_t kvalid[B], pacc[B];
    for (size_t e = 0; e < parena; ++e) { pkc[e] = rnd16(bf16); pvc[e] = rnd16(bf16); }
    for (size_t e = 0; e < ppacked; ++e) { pq[e] = rnd16(bf16); pkn[e] = rnd16(bf16); pvn[e] = rnd16(bf16); }
    for (int i = 0; i < B; ++i) {
        kvalid[i] = k[i] > 0 ? k[i] : 1;
        pacc[i] = 1 + (int32_t)(rnd() % (uint32_t)(kvalid[i] < tau_max ? kvalid[i] : tau_max));
        for (int n = 0; n < cap; ++n) mask[i * cap + n] = (uint8_t)(n < L[i]);
    }
    double* pout = exact(ppacked * sizeof(double));
    CHECK(oracle_padded_verify_attention(pq, pkn, pvn, pkc, pvc, prs, phs, cap, mask, kvalid, pout, B, k_max, l_pad,
                                         H, D, 0.125f, bf16) == 0);
    CHECK(oracle_padded_kv_append(pkc, pvc, prs, phs, cap, mask, pkn, pvn, pacc, B, k_max, l_pad, tau_max, H, D) == 0);

    free(kc); free(vc); free(q); free(kn); free(vn); free(out); free(parent); free(logits); free(logits32);
    free(x); free(x32); free(ids); free(toks); free(path); free(padded); free(packed_ids); free(pkc); free(pvc);
    free(pq); free(pkn); free(pvn); free(mask); free(pout);
}

int main(void) {
    for (int bf16 = 0; bf16 < 2; ++bf16)
        for (int head_major = 0; head_major < 2; ++head_major) one_batch(bf16, head_major);
    printf("ok\n");
    return 0;
}
