/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 definition of batched grouped-query decode attention over
 * per-sequence contiguous KV ranges.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it; the product path never does.  It
 * shares no code with the GPU path.
 *
 * What it computes (the operator of the paper's section 4.3 "Operator
 * Adaptation": attention that receives each request's starting KV address and
 * lengths instead of a block table; and of section 4.4.1 "MLA Optimization": the
 * m+1 query tokens of a speculative step are multiplied with the same K).  The
 * method re-associates the textbook result exactly (splitting the key range and
 * merging is exact up to rounding order), so the oracle is the textbook
 * definition written out, with two passes over the keys and no online trick:
 *
 *   for sequence b, new query token t in [0,T), query head h:
 *     g   = h / (Hq / Hkv)                         consecutive query heads share a KV head
 *     Lv  = kv_lens[b] - T + t + 1                 keys visible to token t: causal inside the block
 *     s_j = scale * sum_d Q[b,t,h,d] * K_b[j,g,d]  j in [0, Lv)
 *     m   = max_j s_j;  p_j = exp(s_j - m);  Z = sum_j p_j
 *     out[b,t,h,:] = sum_j p_j * V_b[j,g,:] / Z
 *     lse[b,t,h]   = m + ln Z
 *
 * Inputs are bf16 bit patterns (widening bf16 -> fp64 is exact); `scale` is the
 * caller's fp32 value widened to double.  Outputs are unrounded fp64.
 *
 * Pins (tests/test_oracle_pins.py): single key, identical keys, q = 0, dominant
 * key, key-shift invariance, causal block == sequential single-token calls,
 * split + merge identity, GQA == MHA on duplicated KV heads, joint key/value
 * permutation, weights sum to one, scipy softmax/logsumexp, and a pure-Python
 * fsum brute force on tiny inputs.
 *
 * oracle_merge is the aggregation step (section 4.4.3, "Layer 2": partial
 * attention results computed elsewhere are gathered by an aggregation
 * operator): given normalised partial outputs and their log-sum-exps over
 * disjoint key ranges it returns the attention over the union.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_f64(uint16_t bits) {
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * One (b, t, h) row.  weights (may be NULL) receives p_j / Z for j in [0, Lv).
 * scratch must hold Lv doubles.
 */
static void attn_row(const uint16_t* q_row, const uint16_t* K, const uint16_t* V, int Lv, int g, int Hkv,
                     int D, double scale, double* out_row, double* lse_out, double* weights,
                     double* scratch) {
    const size_t row_stride = (size_t)Hkv * (size_t)D;
    double m = -INFINITY;
    for (int j = 0; j < Lv; ++j) {
        const uint16_t* k_row = K + (size_t)j * row_stride + (size_t)g * D;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += bf16_to_f64(q_row[d]) * bf16_to_f64(k_row[d]);
        scratch[j] = scale * dot;
        if (scratch[j] > m) m = scratch[j];
    }
    double Z = 0.0;
    for (int j = 0; j < Lv; ++j) {
        scratch[j] = exp(scratch[j] - m);
        Z += scratch[j];
    }
    for (int d = 0; d < D; ++d) out_row[d] = 0.0;
    for (int j = 0; j < Lv; ++j) {
        const uint16_t* v_row = V + (size_t)j * row_stride + (size_t)g * D;
        const double p = scratch[j];
        for (int d = 0; d < D; ++d) out_row[d] += p * bf16_to_f64(v_row[d]);
    }
    for (int d = 0; d < D; ++d) out_row[d] /= Z;
    if (lse_out) *lse_out = m + log(Z);
    if (weights)
        for (int j = 0; j < Lv; ++j) weights[j] = scratch[j] / Z;
}

/*
 * q       bf16 [batch, q_len, n_q_heads, head_dim]
 * k_ptrs  batch host pointers, each bf16 [kv_lens[b], n_kv_heads, head_dim]; v_ptrs alike
 * kv_lens int32[batch], each >= q_len (prefix plus the q_len new tokens)
 * out     fp64 [batch, q_len, n_q_heads, head_dim];  lse fp64 [batch, q_len, n_q_heads] (may be NULL)
 * Returns 0, or -1 on an argument the definition does not cover.
 */
int oracle_attn(const uint16_t* q, const uint16_t* const* k_ptrs, const uint16_t* const* v_ptrs,
                const int32_t* kv_lens, int batch, int q_len, int n_q_heads, int n_kv_heads, int head_dim,
                float scale, double* out, double* lse) {
    if (!q || !k_ptrs || !v_ptrs || !kv_lens || !out) return -1;
    if (batch < 0 || q_len < 1 || n_q_heads < 1 || n_kv_heads < 1 || head_dim < 1) return -1;
    if (n_q_heads % n_kv_heads) return -1;
    int max_len = 0;
    for (int b = 0; b < batch; ++b) {
        if (kv_lens[b] < q_len) return -1;
        if (kv_lens[b] > max_len) max_len = kv_lens[b];
    }
    const int G = n_q_heads / n_kv_heads;
    const long rows = (long)batch * q_len * n_q_heads;
    int failed = 0;
#pragma omp parallel
    {
        double* scratch = (double*)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        if (!scratch) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long r = 0; r < rows; ++r) {
            if (!scratch) continue;
            const int h = (int)(r % n_q_heads);
            const int t = (int)((r / n_q_heads) % q_len);
            const int b = (int)(r / ((long)n_q_heads * q_len));
            const int Lv = kv_lens[b] - q_len + t + 1;
            attn_row(q + (size_t)r * head_dim, k_ptrs[b], v_ptrs[b], Lv, h / G, n_kv_heads, head_dim,
                     (double)scale, out + (size_t)r * head_dim, lse ? lse + r : NULL, NULL, scratch);
        }
        free(scratch);
    }
    return failed ? -1 : 0;
}

/* The normalised softmax weights p_j / Z of one (b, t, h) row; weights holds kv_lens[b]-q_len+t+1 doubles. */
int oracle_attn_weights(const uint16_t* q, const uint16_t* const* k_ptrs, const uint16_t* const* v_ptrs,
                        const int32_t* kv_lens, int batch, int q_len, int n_q_heads, int n_kv_heads,
                        int head_dim, float scale, int b, int t, int h, double* weights) {
    if (!q || !k_ptrs || !v_ptrs || !kv_lens || !weights) return -1;
    if (b < 0 || b >= batch || t < 0 || t >= q_len || h < 0 || h >= n_q_heads) return -1;
    if (n_q_heads % n_kv_heads || kv_lens[b] < q_len) return -1;
    const int G = n_q_heads / n_kv_heads;
    const int Lv = kv_lens[b] - q_len + t + 1;
    double* scratch = (double*)malloc(sizeof(double) * (size_t)Lv);
    double* out_row = (double*)malloc(sizeof(double) * (size_t)head_dim);
    if (!scratch || !out_row) {
        free(scratch);
        free(out_row);
        return -1;
    }
    const size_t r = ((size_t)b * q_len + t) * n_q_heads + h;
    attn_row(q + r * head_dim, k_ptrs[b], v_ptrs[b], Lv, h / G, n_kv_heads, head_dim, (double)scale, out_row,
             NULL, weights, scratch);
    free(scratch);
    free(out_row);
    return 0;
}

/*
 * Aggregation of partial attention results over disjoint key ranges:
 *   LSE = ln sum_s exp(lse_s)      (computed around the largest lse_s)
 *   out = sum_s exp(lse_s - LSE) * out_s
 * out_parts fp64 [n_parts, rows, head_dim], lse_parts fp64 [n_parts, rows]; a part whose range was
 * empty carries lse = -inf and is ignored.  out fp64 [rows, head_dim], lse fp64 [rows].
 */
int oracle_merge(const double* out_parts, const double* lse_parts, int n_parts, long rows, int head_dim,
                 double* out, double* lse) {
    if (!out_parts || !lse_parts || !out || n_parts < 1 || rows < 0 || head_dim < 1) return -1;
    for (long r = 0; r < rows; ++r) {
        double M = -INFINITY;
        for (int s = 0; s < n_parts; ++s)
            if (lse_parts[(size_t)s * rows + r] > M) M = lse_parts[(size_t)s * rows + r];
        double Z = 0.0;
        for (int s = 0; s < n_parts; ++s) {
            const double l = lse_parts[(size_t)s * rows + r];
            if (l > -INFINITY) Z += exp(l - M);
        }
        const double L = M + log(Z);
        for (int d = 0; d < head_dim; ++d) out[(size_t)r * head_dim + d] = 0.0;
        for (int s = 0; s < n_parts; ++s) {
            const double l = lse_parts[(size_t)s * rows + r];
            if (!(l > -INFINITY)) continue;
            const double w = exp(l - L);
            const double* o = out_parts + ((size_t)s * rows + r) * head_dim;
            for (int d = 0; d < head_dim; ++d) out[(size_t)r * head_dim + d] += w * o[d];
        }
        if (lse) lse[r] = L;
    }
    return 0;
}

/*
 * Address identity of section 4.3 (the unnumbered equation after "On-demand Memory Mapping"):
 * a byte at virtual address va of a range starting at va_start lives in physical page
 * floor((va - va_start) / page_size) of that range, at offset (va - va_start) mod page_size.
 */
void oracle_page_of(uint64_t va, uint64_t va_start, uint64_t page_size, uint64_t* page_idx, uint64_t* offset) {
    *page_idx = (va - va_start) / page_size;
    *offset = (va - va_start) % page_size;
}

/*
 * write_kvcache (section 4.3, "Operator Adaptation"): the q_len new K/V rows of sequence b go to rows
 * [kv_lens[b] - q_len, kv_lens[b]) of its K and V ranges; kv_lens are the lengths after the append.
 * k_new, v_new: bf16 [batch, q_len, row_elems]; k_ptrs[b], v_ptrs[b]: bf16 [>= kv_lens[b], row_elems].
 */
int oracle_write_kvcache(const uint16_t* k_new, const uint16_t* v_new, uint16_t* const* k_ptrs,
                         uint16_t* const* v_ptrs, const int32_t* kv_lens, int batch, int q_len, int row_elems) {
    if (!k_new || !v_new || !k_ptrs || !v_ptrs || !kv_lens || batch < 0 || q_len < 1 || row_elems < 1) return -1;
    for (int b = 0; b < batch; ++b) {
        if (kv_lens[b] < q_len) return -1;
        for (int t = 0; t < q_len; ++t) {
            const size_t dst = (size_t)(kv_lens[b] - q_len + t) * (size_t)row_elems;
            const size_t src = ((size_t)b * q_len + t) * (size_t)row_elems;
            for (int e = 0; e < row_elems; ++e) {
                k_ptrs[b][dst + e] = k_new[src + e];
                v_ptrs[b][dst + e] = v_new[src + e];
            }
        }
    }
    return 0;
}

/*
 * Latent-KV (MLA-shaped) decode attention: the operator the paper itself adapts (section 4.3 "Operator
 * Adaptation", section 4.4.1 "MLA Optimization").  Every head of a sequence reads the SAME cached row
 * per token: the first d_v values of the row are the value vector, all d_qk values are the key
 *     s_j = scale * sum_{d < d_qk} Q[b,t,h,d] * C_b[j,d]        j in [0, Lv),  Lv = kv_lens[b] - T + t + 1
 *     out[b,t,h,:] = sum_j softmax(s)_j * C_b[j, 0:d_v]           lse = ln sum_j exp(s_j)
 * q bf16 [batch, q_len, n_heads, d_qk]; c_ptrs[b] bf16 [>= kv_lens[b], d_qk]; out fp64 [batch, q_len,
 * n_heads, d_v]; lse fp64 [batch, q_len, n_heads] (may be NULL).  Written out on its own (it does not
 * call oracle_attn), two passes, fp64.
 */
int oracle_mla(const uint16_t* q, const uint16_t* const* c_ptrs, const int32_t* kv_lens, int batch, int q_len,
               int n_heads, int d_qk, int d_v, float scale, double* out, double* lse) {
    if (!q || !c_ptrs || !kv_lens || !out) return -1;
    if (batch < 0 || q_len < 1 || n_heads < 1 || d_qk < 1 || d_v < 1 || d_v > d_qk) return -1;
    int max_len = 0;
    for (int b = 0; b < batch; ++b) {
        if (kv_lens[b] < q_len) return -1;
        if (kv_lens[b] > max_len) max_len = kv_lens[b];
    }
    const long rows = (long)batch * q_len * n_heads;
    int failed = 0;
#pragma omp parallel
    {
        double* p = (double*)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
        if (!p) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long r = 0; r < rows; ++r) {
            if (!p) continue;
            const int t = (int)((r / n_heads) % q_len);
            const int b = (int)(r / ((long)n_heads * q_len));
            const int Lv = kv_lens[b] - q_len + t + 1;
            const uint16_t* q_row = q + (size_t)r * d_qk;
            const uint16_t* C = c_ptrs[b];
            double m = -INFINITY;
            for (int j = 0; j < Lv; ++j) {
                double dot = 0.0;
                for (int d = 0; d < d_qk; ++d) dot += bf16_to_f64(q_row[d]) * bf16_to_f64(C[(size_t)j * d_qk + d]);
                p[j] = (double)scale * dot;
                if (p[j] > m) m = p[j];
            }
            double Z = 0.0;
            for (int j = 0; j < Lv; ++j) {
                p[j] = exp(p[j] - m);
                Z += p[j];
            }
            double* o = out + (size_t)r * d_v;
            for (int d = 0; d < d_v; ++d) o[d] = 0.0;
            for (int j = 0; j < Lv; ++j)
                for (int d = 0; d < d_v; ++d) o[d] += p[j] * bf16_to_f64(C[(size_t)j * d_qk + d]);
            for (int d = 0; d < d_v; ++d) o[d] /= Z;
            if (lse) lse[r] = m + log(Z);
        }
        free(p);
    }
    return failed ? -1 : 0;
}
