/*
 * ems_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what the ragged verification step of
 * batched speculative decoding computes (EMS-SD, arXiv 2405.07542).  It shares
 * no code with the HIP library and is only ever called by the tests, the smoke
 * check and the bench's cpu_baseline leg.
 *
 * Notation (Sec. 3.2 "Unpad KV cache" / "Unpad input tokens", Appendix D):
 *   B samples; sample i brings k_i packed query rows (row 0 = last emitted
 *   token, rows 1.. = draft tokens), cu[i] = k_0 + ... + k_{i-1}  (the running
 *   sum of Alg. 1's token_nums_per_sample), T = cu[B].
 *   Sample i owns cache rows [kv_start[i], kv_start[i] + kv_len[i]) of a shared
 *   arena; element (row r, head h, dim d) sits at r*row_stride + h*head_stride + d.
 *   Packed tensors (q, k_new, v_new, out) are [T, H, D], d fastest.
 *
 * Every function states the passage it follows.  There is no tiling, fusion or
 * reordering: each output is computed from its definition.  The only
 * parallelism is an OpenMP `parallel for` over independent (sample, head)
 * pairs / independent rows; every output element is produced by one thread
 * with a fixed summation order, so results do not depend on the thread count.
 *
 * Parity pins (tests/test_oracle_*.py): dense padded per-sample brute force,
 * torch's CPU attention in the k_i = 1 and kv_len = 0 special cases,
 * autoregressive equivalence, closed forms, the paper's Table 1, Alg. 2 run
 * literally (and as the inverse of Alg. 1), sentinel-filled arenas; for the tree functions: reduction to the
 * causal ones on a chain, causal attention along every root-to-row path, a dense
 * brute force with a matrix-closure mask, a per-node validity rule for acceptance,
 * a numpy gather for the append; tests/test_oracle_mutants.py plants single mistakes in a
 * copy of this file and checks that those pins notice each.  No function here is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Exact widening of one IEEE binary16 / bfloat16 bit pattern to double. */
static double widen(uint16_t bits, int dtype) {
    if (dtype == ORACLE_BF16) {
        uint32_t u = (uint32_t)bits << 16;
        float f;
        memcpy(&f, &u, sizeof f);
        return (double)f;
    }
    int sign = bits >> 15;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double mag;
    if (expo == 0)
        mag = ldexp((double)frac, -24);            /* zero and subnormals */
    else if (expo == 31)
        mag = frac ? NAN : INFINITY;
    else
        mag = ldexp((double)(frac | 0x400), expo - 25);
    return sign ? -mag : mag;
}

/* Which sample a packed row belongs to, and which of that sample's rows it is (what
 * Appendix D's Alg. 2 recovers inside the kernel).  By definition: with first_i = rows_0 +
 * ... + rows_{i-1}, packed row r belongs to the one sample i with first_i <= r < first_i +
 * rows_i, and is its row r - first_i.  Returns 0 on success, 1 if r is not a packed row. */
int oracle_restore_index(const int32_t* rows_per_sample, int B, int r,
                         int32_t* sample, int32_t* position) {
    int64_t first = 0;
    for (int i = 0; i < B; ++i) {
        if (r >= first && r < first + rows_per_sample[i]) {
            *sample = i;
            *position = (int32_t)(r - first);
            return 0;
        }
        first += rows_per_sample[i];
    }
    return 1;
}

/*
 * Packed multi-token attention over per-sample caches (Sec. 3.2: every token
 * attends to its own sample's cached rows, found through the per-sample start
 * location, and causally to its own sample's new tokens; Fig. 3).
 *
 * For sample i, head h, query row j (0 <= j < k_i), with L = kv_len[i]:
 *   key n   = cache row kv_start[i]+n           for n <  L
 *           = new row   cu[i] + (n - L)          for n >= L      (N = L + k_i keys)
 *   mask[n] = (n <= L + j)       -- the new token sees itself (inclusive causal)
 *   S[n]    = scale * <q_j, key_n>     where mask, else -inf
 *   p       = softmax_n(S)  (max-subtracted),  out_j = sum_n p[n] * val_n
 * Inputs are widened exactly to fp64; out is fp64 [T, H, D].
 */
int oracle_verify_attention(const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new,
                            const uint16_t* k_cache, const uint16_t* v_cache,
                            int64_t row_stride, int64_t head_stride,
                            const int32_t* cu, const int32_t* kv_start, const int32_t* kv_len,
                            double* out, int B, int H, int D, float scale, int dtype) {
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int i = 0; i < B; ++i) {
        for (int h = 0; h < H; ++h) {
            const int k = cu[i + 1] - cu[i];
            const int L = kv_len[i];
            const int64_t s = kv_start[i];
            const int N = L + k;
            if (k <= 0) continue;
            double* key = (double*)malloc(sizeof(double) * (size_t)N * D);
            double* val = (double*)malloc(sizeof(double) * (size_t)N * D);
            double* S = (double*)malloc(sizeof(double) * (size_t)N);
            double* p = (double*)malloc(sizeof(double) * (size_t)N);
            unsigned char* mask = (unsigned char*)malloc((size_t)N);
            if (!key || !val || !S || !p || !mask) {
#pragma omp atomic write
                failed = 1;
                free(key); free(val); free(S); free(p); free(mask);
                continue;
            }
            for (int n = 0; n < N; ++n) {
                for (int d = 0; d < D; ++d) {
                    if (n < L) {
                        int64_t off = (s + n) * row_stride + (int64_t)h * head_stride + d;
                        key[(size_t)n * D + d] = widen(k_cache[off], dtype);
                        val[(size_t)n * D + d] = widen(v_cache[off], dtype);
                    } else {
                        int64_t off = ((int64_t)(cu[i] + n - L) * H + h) * D + d;
                        key[(size_t)n * D + d] = widen(k_new[off], dtype);
                        val[(size_t)n * D + d] = widen(v_new[off], dtype);
                    }
                }
            }
            for (int j = 0; j < k; ++j) {
                const int64_t qoff = ((int64_t)(cu[i] + j) * H + h) * D;
                for (int n = 0; n < N; ++n) mask[n] = (unsigned char)(n <= L + j);
                double m = -INFINITY;
                for (int n = 0; n < N; ++n) {
                    if (mask[n]) {
                        double dot = 0.0;
                        for (int d = 0; d < D; ++d)
                            dot += widen(q[qoff + d], dtype) * key[(size_t)n * D + d];
                        S[n] = (double)scale * dot;
                    } else {
                        S[n] = -INFINITY;
                    }
                    if (S[n] > m) m = S[n];
                }
                double Z = 0.0;
                for (int n = 0; n < N; ++n) {
                    p[n] = mask[n] ? exp(S[n] - m) : 0.0;
                    Z += p[n];
                }
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n) acc += p[n] * val[(size_t)n * D + d];
                    out[qoff + d] = acc / Z;
                }
            }
            free(key); free(val); free(S); free(p); free(mask);
        }
    }
    return failed;
}

/*
 * Greedy target token per packed row (Appendix A, the arg-max of the target
 * distribution): x[r] = the smallest v attaining max_v logits[r, v].
 * Values are widened exactly, so +0 and -0 compare equal and the lower index
 * wins; inputs are finite by contract.
 */
int oracle_argmax(const uint16_t* logits, int dtype, int T, int V, int32_t* x) {
#pragma omp parallel for schedule(static)
    for (int r = 0; r < T; ++r) {
        const uint16_t* row = logits + (size_t)r * V;
        double best = widen(row[0], dtype);
        int32_t arg = 0;
        for (int v = 1; v < V; ++v) {
            double y = widen(row[v], dtype);
            if (y > best) { best = y; arg = v; }
        }
        x[r] = arg;
    }
    return 0;
}

/*
 * Acceptance length per sample (Appendix A, the acceptance-length equation,
 * and Sec. 3.1: with k drafts between 1 and k+1 tokens are accepted), its
 * running sum, and the accepted target tokens packed sample after sample.
 *
 * Packed row j of sample i carries input token input_ids[cu[i]+j]; row 0 is
 * the last emitted token and rows 1..k_i-1 are the drafts.  x[cu[i]+j] is the
 * target's greedy token after row j.  Draft j+1 is accepted while it equals
 * x[cu[i]+j] and every earlier draft was accepted; the row after the last
 * draft has nothing to be compared with, which ends the run.
 *   accepted[i] = (number of leading accepted drafts) + 1,   0 when k_i = 0.
 */
int oracle_greedy_accept(const int32_t* x, const int32_t* input_ids, const int32_t* cu, int B,
                         int32_t* accepted, int32_t* accepted_cu, int32_t* out_tokens) {
    accepted_cu[0] = 0;
    for (int i = 0; i < B; ++i) {
        const int k = cu[i + 1] - cu[i];
        int tau = 0;
        if (k > 0) {
            int m = 0;
            while (m < k - 1 && x[cu[i] + m] == input_ids[cu[i] + m + 1]) m += 1;
            tau = m + 1;
        }
        accepted[i] = tau;
        accepted_cu[i + 1] = accepted_cu[i] + tau;
        if (out_tokens)
            for (int j = 0; j < tau; ++j) out_tokens[accepted_cu[i] + j] = x[cu[i] + j];
    }
    return 0;
}

/*
 * KV-cache append (Sec. 3.2 "Unpad KV cache": each sample's write location
 * advances by its own accepted count, so no padding row ever enters a cache).
 * The first accepted[i] new rows of sample i are copied, bit for bit, to cache
 * rows kv_start[i]+kv_len[i]+j; kv_len_out[i] = kv_len[i] + accepted[i].
 * Nothing else in the arena is written.
 */
int oracle_kv_append(uint16_t* k_cache, uint16_t* v_cache, int64_t row_stride, int64_t head_stride,
                     const uint16_t* k_new, const uint16_t* v_new,
                     const int32_t* cu, const int32_t* accepted,
                     const int32_t* kv_start, const int32_t* kv_len, int32_t* kv_len_out,
                     int B, int H, int D) {
    for (int i = 0; i < B; ++i) {
        for (int j = 0; j < accepted[i]; ++j) {
            const int64_t dst_row = (int64_t)kv_start[i] + kv_len[i] + j;
            const int64_t src_row = (int64_t)cu[i] + j;
            for (int h = 0; h < H; ++h) {
                for (int d = 0; d < D; ++d) {
                    int64_t dst = dst_row * row_stride + (int64_t)h * head_stride + d;
                    int64_t src = (src_row * H + h) * D + d;
                    k_cache[dst] = k_new[src];
                    v_cache[dst] = v_new[src];
                }
            }
        }
    }
    if (kv_len_out)
        for (int i = 0; i < B; ++i) kv_len_out[i] = kv_len[i] + accepted[i];
    return 0;
}

/*
 * The padded "vanilla" method (Sec. 3.1), kept as the ablation's own definition.
 * Inputs are padded to k_max rows per sample, caches are aligned to l_pad rows per sample
 * (sample i owns arena rows i*cap .. i*cap+l_pad-1) and an attention mask hides padding:
 *   cached key n          visible iff key_mask[i*cap + n] != 0
 *   new key jj of row j   visible iff jj <= j and jj < k_valid[i]
 * Every one of the k_max rows is computed, padding rows included (their values are
 * don't-care; the paper's point is that they cost time and traffic).
 * out is fp64 [B*k_max, H, D].
 */
int oracle_padded_verify_attention(const uint16_t* q_pad, const uint16_t* k_new_pad,
                                   const uint16_t* v_new_pad, const uint16_t* k_cache,
                                   const uint16_t* v_cache, int64_t row_stride, int64_t head_stride,
                                   int64_t cap, const uint8_t* key_mask, const int32_t* k_valid,
                                   double* out, int B, int k_max, int l_pad, int H, int D,
                                   float scale, int dtype) {
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int i = 0; i < B; ++i) {
        for (int h = 0; h < H; ++h) {
            const int N = l_pad + k_max;
            double* S = (double*)malloc(sizeof(double) * (size_t)N);
            double* p = (double*)malloc(sizeof(double) * (size_t)N);
            unsigned char* mask = (unsigned char*)malloc((size_t)N);
            if (!S || !p || !mask) {
#pragma omp atomic write
                failed = 1;
                free(S); free(p); free(mask);
                continue;
            }
            for (int j = 0; j < k_max; ++j) {
                const int64_t qoff = (((int64_t)i * k_max + j) * H + h) * D;
                for (int n = 0; n < N; ++n) {
                    if (n < l_pad) mask[n] = key_mask[(int64_t)i * cap + n] != 0;
                    else mask[n] = (n - l_pad <= j) && (n - l_pad < k_valid[i]);
                }
                double m = -INFINITY;
                for (int n = 0; n < N; ++n) {
                    S[n] = -INFINITY;
                    if (mask[n]) {
                        double dot = 0.0;
                        for (int d = 0; d < D; ++d) {
                            double kv = n < l_pad
                                ? widen(k_cache[((int64_t)i * cap + n) * row_stride + (int64_t)h * head_stride + d], dtype)
                                : widen(k_new_pad[(((int64_t)i * k_max + n - l_pad) * H + h) * D + d], dtype);
                            dot += widen(q_pad[qoff + d], dtype) * kv;
                        }
                        S[n] = (double)scale * dot;
                    }
                    if (S[n] > m) m = S[n];
                }
                double Z = 0.0;
                for (int n = 0; n < N; ++n) {
                    p[n] = mask[n] ? exp(S[n] - m) : 0.0;
                    Z += p[n];
                }
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n) {
                        if (!mask[n]) continue;
                        double vv = n < l_pad
                            ? widen(v_cache[((int64_t)i * cap + n) * row_stride + (int64_t)h * head_stride + d], dtype)
                            : widen(v_new_pad[(((int64_t)i * k_max + n - l_pad) * H + h) * D + d], dtype);
                        acc += p[n] * vv;
                    }
                    out[qoff + d] = acc / Z;
                }
            }
            free(S); free(p); free(mask);
        }
    }
    return failed;
}

/*
 * Vanilla append (Sec. 3.1, Table 1): every sample grows by tau_max = the batch maximum of
 * the accepted counts; sample i's rows j < accepted[i] are real, the other tau_max -
 * accepted[i] rows are padding (written, but masked).  Aligned length becomes l_pad + tau_max.
 */
int oracle_padded_kv_append(uint16_t* k_cache, uint16_t* v_cache, int64_t row_stride,
                            int64_t head_stride, int64_t cap, uint8_t* key_mask,
                            const uint16_t* k_new_pad, const uint16_t* v_new_pad,
                            const int32_t* accepted, int B, int k_max, int l_pad, int tau_max,
                            int H, int D) {
    for (int i = 0; i < B; ++i) {
        for (int j = 0; j < tau_max; ++j) {
            const int64_t dst_row = (int64_t)i * cap + l_pad + j;
            const int64_t src_row = (int64_t)i * k_max + j;
            key_mask[dst_row] = (uint8_t)(j < accepted[i]);
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d) {
                    int64_t dst = dst_row * row_stride + (int64_t)h * head_stride + d;
                    int64_t src = (src_row * H + h) * D + d;
                    k_cache[dst] = k_new_pad[src];
                    v_cache[dst] = v_new_pad[src];
                }
        }
    }
    return 0;
}

/*
 * Paper-order cache write (Sec. 3.2): before attention, the K/V of EVERY new row of sample i
 * is written at the sample's own location, cache rows kv_start[i]+kv_len[i]+j for j < k_i;
 * after verification only the location advances (kv_len += accepted).  Rows at or beyond
 * the advanced length then hold rejected drafts and are don't-care.
 */
int oracle_kv_write_through(uint16_t* k_cache, uint16_t* v_cache, int64_t row_stride,
                            int64_t head_stride, const uint16_t* k_new, const uint16_t* v_new,
                            const int32_t* cu, const int32_t* kv_start, const int32_t* kv_len,
                            int B, int H, int D) {
    for (int i = 0; i < B; ++i) {
        const int k = cu[i + 1] - cu[i];
        for (int j = 0; j < k; ++j)
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d) {
                    int64_t dst = ((int64_t)kv_start[i] + kv_len[i] + j) * row_stride + (int64_t)h * head_stride + d;
                    int64_t src = (((int64_t)cu[i] + j) * H + h) * D + d;
                    k_cache[dst] = k_new[src];
                    v_cache[dst] = v_new[src];
                }
    }
    return 0;
}

/*
 * Tree-structured verification.  The paper names it as the next thing to combine with
 * the multi-sample method (Limitations, item 4; Sec. 2 "Dynamic Tree decoding": several
 * candidate tokens at the same position) and gives no algorithm of its own, so what
 * follows is the usual statement of tree verification, sample by sample.
 *
 * The k_i new rows of sample i form a token tree: row 0 (the last emitted token) is the
 * root and row j > 0 continues the row parent[cu[i]+j], a row of the same sample with a
 * smaller index (parent[cu[i]] = -1).  A root-to-node path is one candidate continuation.
 *
 * Attention: row j sees every cached key of its sample and, among the new rows, itself
 * and its ancestors only:   mask[L + jj] = (jj is j or an ancestor of j).
 * With parent[j] = j-1 (a chain) this is the causal mask of oracle_verify_attention.
 * Returns 0, 1 on memory exhaustion, 2 when parent[] is not a tree in topological order.
 */
int oracle_tree_verify_attention(const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new,
                                 const uint16_t* k_cache, const uint16_t* v_cache,
                                 int64_t row_stride, int64_t head_stride,
                                 const int32_t* cu, const int32_t* parent,
                                 const int32_t* kv_start, const int32_t* kv_len,
                                 double* out, int B, int H, int D, float scale, int dtype) {
    for (int i = 0; i < B; ++i) {
        const int k = cu[i + 1] - cu[i];
        for (int j = 0; j < k; ++j) {
            const int pj = parent[cu[i] + j];
            if (j == 0 ? pj != -1 : (pj < 0 || pj >= j)) return 2;
        }
    }
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int i = 0; i < B; ++i) {
        for (int h = 0; h < H; ++h) {
            const int k = cu[i + 1] - cu[i];
            const int L = kv_len[i];
            const int64_t s = kv_start[i];
            const int N = L + k;
            if (k <= 0) continue;
            double* key = (double*)malloc(sizeof(double) * (size_t)N * D);
            double* val = (double*)malloc(sizeof(double) * (size_t)N * D);
            double* S = (double*)malloc(sizeof(double) * (size_t)N);
            double* p = (double*)malloc(sizeof(double) * (size_t)N);
            unsigned char* mask = (unsigned char*)malloc((size_t)N);
            if (!key || !val || !S || !p || !mask) {
#pragma omp atomic write
                failed = 1;
                free(key); free(val); free(S); free(p); free(mask);
                continue;
            }
            for (int n = 0; n < N; ++n) {
                for (int d = 0; d < D; ++d) {
                    int64_t off = n < L ? (s + n) * row_stride + (int64_t)h * head_stride + d
                                        : ((int64_t)(cu[i] + n - L) * H + h) * D + d;
                    key[(size_t)n * D + d] = widen(n < L ? k_cache[off] : k_new[off], dtype);
                    val[(size_t)n * D + d] = widen(n < L ? v_cache[off] : v_new[off], dtype);
                }
            }
            for (int j = 0; j < k; ++j) {
                const int64_t qoff = ((int64_t)(cu[i] + j) * H + h) * D;
                for (int n = 0; n < N; ++n) mask[n] = (unsigned char)(n < L);
                for (int u = j; u >= 0; u = parent[cu[i] + u]) mask[L + u] = 1;   /* j, then its ancestors */
                double m = -INFINITY;
                for (int n = 0; n < N; ++n) {
                    if (mask[n]) {
                        double dot = 0.0;
                        for (int d = 0; d < D; ++d)
                            dot += widen(q[qoff + d], dtype) * key[(size_t)n * D + d];
                        S[n] = (double)scale * dot;
                    } else {
                        S[n] = -INFINITY;
                    }
                    if (S[n] > m) m = S[n];
                }
                double Z = 0.0;
                for (int n = 0; n < N; ++n) {
                    p[n] = mask[n] ? exp(S[n] - m) : 0.0;
                    Z += p[n];
                }
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n) acc += p[n] * val[(size_t)n * D + d];
                    out[qoff + d] = acc / Z;
                }
            }
            free(key); free(val); free(S); free(p); free(mask);
        }
    }
    return failed;
}

/*
 * Greedy acceptance along the tree: starting at the root, the target's greedy token after
 * the current row, x[row], is looked for among the tokens of that row's children; the
 * matching child (the lowest-indexed one if several carry the same token) is accepted and
 * becomes the current row; the walk ends at a row none of whose children matches.
 *   accepted[i]      = number of rows on the accepted path (root included), 0 when k_i = 0
 *   out_tokens       = x at the rows of the path, packed sample after sample
 *   accepted_rows    = the packed row index cu[i] + j of every row of the path, same packing
 * With a chain this is oracle_greedy_accept, and accepted_rows = cu[i], cu[i]+1, ...
 */
int oracle_tree_accept(const int32_t* x, const int32_t* input_ids, const int32_t* parent,
                       const int32_t* cu, int B, int32_t* accepted, int32_t* accepted_cu,
                       int32_t* out_tokens, int32_t* accepted_rows) {
    accepted_cu[0] = 0;
    for (int i = 0; i < B; ++i) {
        const int k = cu[i + 1] - cu[i];
        int tau = 0;
        if (k > 0) {
            int u = 0;
            for (;;) {
                if (out_tokens) out_tokens[accepted_cu[i] + tau] = x[cu[i] + u];
                if (accepted_rows) accepted_rows[accepted_cu[i] + tau] = cu[i] + u;
                tau += 1;
                int next = -1;
                for (int c = u + 1; c < k && next < 0; ++c)
                    if (parent[cu[i] + c] == u && input_ids[cu[i] + c] == x[cu[i] + u]) next = c;
                if (next < 0) break;
                u = next;
            }
        }
        accepted[i] = tau;
        accepted_cu[i + 1] = accepted_cu[i] + tau;
    }
    return 0;
}

/*
 * Append of an accepted path: the rows of a path are not contiguous in the packed tensors,
 * so the copy gathers them: cache row kv_start[i]+kv_len[i]+j receives, bit for bit, packed
 * row accepted_rows[accepted_cu[i]+j], j < accepted[i] = accepted_cu[i+1]-accepted_cu[i];
 * kv_len_out[i] = kv_len[i] + accepted[i].  Nothing else in the arena is written
 * (Sec. 3.2 "Unpad KV cache": each sample advances by its own count).
 */
int oracle_kv_append_rows(uint16_t* k_cache, uint16_t* v_cache, int64_t row_stride, int64_t head_stride,
                          const uint16_t* k_new, const uint16_t* v_new,
                          const int32_t* accepted_rows, const int32_t* accepted_cu,
                          const int32_t* kv_start, const int32_t* kv_len, int32_t* kv_len_out,
                          int B, int H, int D) {
    for (int i = 0; i < B; ++i) {
        const int a = accepted_cu[i + 1] - accepted_cu[i];
        for (int j = 0; j < a; ++j) {
            const int64_t dst_row = (int64_t)kv_start[i] + kv_len[i] + j;
            const int64_t src_row = accepted_rows[accepted_cu[i] + j];
            for (int h = 0; h < H; ++h)
                for (int d = 0; d < D; ++d) {
                    int64_t dst = dst_row * row_stride + (int64_t)h * head_stride + d;
                    int64_t src = (src_row * H + h) * D + d;
                    k_cache[dst] = k_new[src];
                    v_cache[dst] = v_new[src];
                }
        }
        if (kv_len_out) kv_len_out[i] = kv_len[i] + a;
    }
    return 0;
}

/*
 * "Unpad input tokens" (Sec. 3.2; Appendix D, Alg. 1): the packed sequence holds the samples'
 * input tokens back to back, without padding, and every sample's count is kept.  Written as
 * a gather: packed slot t holds token t - first_i of the one sample i whose share
 * [first_i, first_i + lens[i]) contains t (first_i = lens[0] + ... + lens[i-1]).  The
 * samples' token lists are the first lens[i] entries of row i of a padded [B, k_max] array.
 * Returns the total number of packed tokens.
 */
int oracle_concatenate_tokens(const int32_t* padded_ids, const int32_t* lens, int B, int k_max,
                              int32_t* packed_ids, int32_t* rows_per_sample) {
    int total = 0;
    for (int i = 0; i < B; ++i) {
        rows_per_sample[i] = lens[i];
        total += lens[i];
    }
    for (int t = 0; t < total; ++t) {
        int i = 0, first = 0;
        while (t >= first + lens[i]) {
            first += lens[i];
            i += 1;
        }
        packed_ids[t] = padded_ids[(size_t)i * k_max + (t - first)];
    }
    return total;
}

/* The same greedy target token for fp32 logits (Appendix A): smallest index of the row maximum. */
int oracle_argmax_f32(const float* logits, int T, int V, int32_t* x) {
#pragma omp parallel for schedule(static)
    for (int r = 0; r < T; ++r) {
        const float* row = logits + (size_t)r * V;
        double best = (double)row[0];
        int32_t arg = 0;
        for (int v = 1; v < V; ++v) {
            double y = (double)row[v];
            if (y > best) { best = y; arg = v; }
        }
        x[r] = arg;
    }
    return 0;
}
