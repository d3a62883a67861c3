/*
 * CPU oracle for mixed-batch attention over a paged KV cache, and for the KV-cache append.
 *
 * THIS IS TEST INFRASTRUCTURE, not the product: only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the GPU library.
 *
 * What it computes is the plain definition, written out in fp64 with no blocking, fusion or
 * reordering:
 *
 *   - Scaled dot-product self-attention, softmax(Q K^T / sqrt(d_k)) V, per head
 *     (paper Sec. 2.1, the self-attention equation; heads are independent and concatenated).
 *   - A query token attends to the keys of all previous tokens of its own sequence and to
 *     itself (Sec. 2.1 "all the keys of previous tokens"; auto-regressive generation, Sec. 1):
 *     the row at absolute position p sees keys 0..p inclusive.
 *   - A prompt chunk is rows prior..prior+q_len-1 of one sequence, processed against all
 *     earlier KV of that sequence (Sec. 2.3 chunking; Sec. 4.2 dynamic chunking); a generation
 *     task is the case q_len = 1.
 *   - K and V live in fixed-size token blocks that need not be contiguous (Sec. 2.2, block-based
 *     KVC allocation): token t of sequence i is at block_table[i][t / bs], offset t % bs.
 *   - The append stores the K/V of the iteration's new tokens in the cache (Sec. 2.2 "KVC
 *     allocation": the KV values of all tokens of a step are stored in the KVC).
 *
 *   - Query heads may share K/V heads (grouped-query attention, as in the Llama-3-70B model the
 *     paper also serves, Sec. 6.1): with HK K/V heads, query head h reads K/V head h / (H/HK).
 *     HK == H is ordinary multi-head attention.
 *
 * Inputs are 16-bit floating-point bit patterns, bf16 (dtype 1: the upper half of an IEEE single)
 * or fp16 (dtype 2: IEEE half, the precision of the paper's own experiments, Sec. 5), widened
 * exactly to double; outputs stay in double.
 * Layouts: q [T,H,D]; k_new/v_new [T,HK,D]; caches [NB,HK,bs,D]; block_table [S,stride].
 *
 * Pins (tests/test_oracle_pins.py): dense brute force with an explicit masked score matrix,
 * closed forms (single key, zero query, constant V, dominant key), a library causal SDPA in
 * fp64, and the invariants chunked == one-shot, generation row == last prompt row, physical
 * block permutation, batch independence, poison independence.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC mpa_oracle.c -o libmpa_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 1, ORACLE_FP16 = 2 };

/* The value of a 16-bit pattern.  fp16: 1 sign, 5 exponent (bias 15), 10 fraction bits;
 * exponent 0 = subnormal (fraction * 2^-24), 31 = infinity / NaN. */
static double widen(uint16_t b, int dtype)
{
    if (dtype == ORACLE_FP16) {
        const int sign = b >> 15, e = (b >> 10) & 31, f = b & 1023;
        double v;
        if (e == 0) v = ldexp((double)f, -24);
        else if (e == 31) v = f ? NAN : INFINITY;
        else v = ldexp(1.0 + (double)f / 1024.0, e - 15);
        return sign ? -v : v;
    }
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* For the pins: out[i] = value of in[i]. */
void mpa_oracle_widen(const uint16_t *in, int64_t n, int dtype, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = widen(in[i], dtype);
}

int mpa_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* For every token t with slot_map[t] >= 0 and every K/V head (H of them here): copy the D-vector
 * of K and of V to cache[slot / bs][h][slot % bs][:].  Byte copy, hence exact. */
void mpa_oracle_kv_append(const uint16_t *k_new, const uint16_t *v_new, const int64_t *slot_map,
                          int T, int H, int D, int bs, uint16_t *k_cache, uint16_t *v_cache)
{
    for (int t = 0; t < T; ++t) {
        int64_t slot = slot_map[t];
        if (slot < 0) continue;
        int64_t blk = slot / bs, off = slot % bs;
        for (int h = 0; h < H; ++h) {
            size_t src = ((size_t)t * H + h) * D;
            size_t dst = (((size_t)blk * H + h) * bs + off) * D;
            memcpy(k_cache + dst, k_new + src, (size_t)D * sizeof(uint16_t));
            memcpy(v_cache + dst, v_new + src, (size_t)D * sizeof(uint16_t));
        }
    }
}

/* One output row: query row `row` of q (belonging to sequence i, absolute position p), head h. */
static void one_row(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                    const int32_t *table_i, int row, int p, int h, int H, int HK, int D, int bs,
                    double scale, int dtype, double *s, double *out_row)
{
    const uint16_t *qv = q + ((size_t)row * H + h) * D;
    const int hk = h / (H / HK); /* the K/V head this query head reads */
    double m = -INFINITY;
    for (int t = 0; t <= p; ++t) {
        const uint16_t *kv = k_cache + (((size_t)table_i[t / bs] * HK + hk) * bs + t % bs) * D;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += widen(qv[d], dtype) * widen(kv[d], dtype);
        s[t] = scale * dot;
        if (s[t] > m) m = s[t];
    }
    double Z = 0.0;
    for (int t = 0; t <= p; ++t) {
        s[t] = exp(s[t] - m);
        Z += s[t];
    }
    for (int d = 0; d < D; ++d) out_row[d] = 0.0;
    for (int t = 0; t <= p; ++t) {
        const uint16_t *vv = v_cache + (((size_t)table_i[t / bs] * HK + hk) * bs + t % bs) * D;
        for (int d = 0; d < D; ++d) out_row[d] += s[t] * widen(vv[d], dtype);
    }
    for (int d = 0; d < D; ++d) out_row[d] /= Z;
}

/* All rows of the batch.  out is [T,H,D] double.  Returns 0, or -1 on a malformed batch. */
int mpa_oracle_attention(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                         const int32_t *block_table, int stride, const int32_t *chunk_starts,
                         const int32_t *context_lens, int S, int H, int HK, int D, int bs,
                         double scale, int dtype, double *out)
{
    int max_ctx = 0;
    if (HK < 1 || H % HK != 0 || (dtype != ORACLE_BF16 && dtype != ORACLE_FP16)) return -1;
    for (int i = 0; i < S; ++i) {
        int q_len = chunk_starts[i + 1] - chunk_starts[i];
        if (q_len < 1 || context_lens[i] < q_len) return -1;
        if (context_lens[i] > max_ctx) max_ctx = context_lens[i];
    }
    int T = chunk_starts[S];
    /* row -> sequence */
    int *seq_of = (int *)malloc(sizeof(int) * (size_t)(T > 0 ? T : 1));
    for (int i = 0; i < S; ++i)
        for (int r = chunk_starts[i]; r < chunk_starts[i + 1]; ++r) seq_of[r] = i;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(max_ctx > 0 ? max_ctx : 1));
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int row = 0; row < T; ++row)
            for (int h = 0; h < H; ++h) {
                int i = seq_of[row];
                int q_len = chunk_starts[i + 1] - chunk_starts[i];
                int prior = context_lens[i] - q_len;
                int p = prior + (row - chunk_starts[i]);
                one_row(q, k_cache, v_cache, block_table + (size_t)i * stride, row, p, h, H, HK, D,
                        bs, scale, dtype, s, out + ((size_t)row * H + h) * D);
            }
        free(s);
    }
    free(seq_of);
    return 0;
}

/* Selected (row, head) outputs only: out is [n, D] double. */
int mpa_oracle_attention_rows(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                              const int32_t *block_table, int stride, const int32_t *chunk_starts,
                              const int32_t *context_lens, int S, int H, int HK, int D, int bs,
                              double scale, int dtype, const int32_t *rows, const int32_t *heads, int n,
                              double *out)
{
    int max_ctx = 0;
    if (HK < 1 || H % HK != 0 || (dtype != ORACLE_BF16 && dtype != ORACLE_FP16)) return -1;
    for (int i = 0; i < S; ++i) {
        int q_len = chunk_starts[i + 1] - chunk_starts[i];
        if (q_len < 1 || context_lens[i] < q_len) return -1;
        if (context_lens[i] > max_ctx) max_ctx = context_lens[i];
    }
    for (int x = 0; x < n; ++x)
        if (rows[x] < 0 || rows[x] >= chunk_starts[S] || heads[x] < 0 || heads[x] >= H) return -1;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(max_ctx > 0 ? max_ctx : 1));
#pragma omp for schedule(dynamic, 1)
        for (int x = 0; x < n; ++x) {
            int row = rows[x], i = 0;
            while (chunk_starts[i + 1] <= row) ++i;
            int q_len = chunk_starts[i + 1] - chunk_starts[i];
            int p = context_lens[i] - q_len + (row - chunk_starts[i]);
            one_row(q, k_cache, v_cache, block_table + (size_t)i * stride, row, p, heads[x], H, HK,
                    D, bs, scale, dtype, s, out + (size_t)x * D);
        }
        free(s);
    }
    return 0;
}
