/*
 * CPU oracle for the HATA decode-attention path -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the path computes,
 * written from the paper's definitions.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product (the HIP library)
 * shares no code with this file and never routes through it.
 *
 * All floating-point arithmetic is fp64 on the exact bf16 / fp32 inputs.
 * No blocking, fusion or reordering beyond what the definitions state.
 *
 * What follows which passage of the paper:
 *   oracle_hash_encode        Alg. 2 (HashEncode): Sign(MatMul(x, W_H)) then BitPack;
 *                             hash function h(x) = sign(x W_H) of Sec. 3.1.1
 *   oracle_hamming_score      Alg. 3 "Calculate distance in Hamming space":
 *                             S = bitcount(bitwise_xor(Q_H, K_H^cache)), and the
 *                             aggregation over query heads that share one KV cache
 *                             (Sec. 3.2, decode-stage paragraph)
 *   oracle_topk               Alg. 3 "Select top-k key-value pairs": Idx = TopK(S, N)
 *   oracle_attention_rows     Alg. 3 Gather + Attention over the gathered rows;
 *                             third line of Eq. 2 with the 1/sqrt(d) scale of Eq. 1
 *   oracle_dense_attention    Eq. 1 for one query row
 *   *_batch                   the same per (sequence, KV head) unit over the cache layout
 *
 * Readings taken where the paper is silent (listed in the design notes too):
 *   - sign(0): bit = 1 iff projection >= 0;
 *   - BitPack: 32-bit words, bit j of a code -> word j/32, bit position j%32;
 *   - one W_H per KV head, used by every query head of its group;
 *   - aggregation over a group = SUM of the per-head Hamming distances;
 *   - TopK keeps the k SMALLEST distances (= most matching bits);
 *     equal distances: lower cache index wins; Idx is returned ascending;
 *   - k >= L selects every row.
 *
 * Pins: tests/test_oracle_*.py (closed forms, brute force, invariants).
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC hata_oracle.c -o libhata_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* bf16 bit pattern -> double, exact (bf16 is the upper half of an fp32). */
static double bf16_to_double(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* double -> bf16 bit pattern, round to nearest even, done on the double's own
 * value (no intermediate fp32 rounding): find the two neighbouring bf16 values. */
static uint16_t double_to_bf16(double v) {
    if (v != v) return 0x7FC0;
    uint16_t sign = (v < 0.0 || (v == 0.0 && 1.0 / v < 0.0)) ? 0x8000 : 0;
    double av = fabs(v);
    float f = (float)av; /* only to get a nearby bit pattern to start from */
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t lo = (uint16_t)(u >> 16);     /* bf16 at or just below |v| ... */
    if ((lo & 0x7F80) == 0x7F80) return (uint16_t)(sign | 0x7F80); /* inf */
    /* ... unless the float rounding stepped up over a bf16 boundary */
    if (bf16_to_double(lo) > av) lo = (uint16_t)(lo - 1);
    uint16_t hi = (uint16_t)(lo + 1);      /* next bf16 above (positive patterns are monotone) */
    double el = av - bf16_to_double(lo), eh = bf16_to_double(hi) - av;
    uint16_t pick;
    if (el < eh) pick = lo;
    else if (eh < el) pick = hi;
    else pick = (lo & 1) ? hi : lo;
    return (uint16_t)(sign | pick);
}

void oracle_round_bf16(const double* in, int64_t n, uint16_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = double_to_bf16(in[i]);
}

/* ------------------------------------------------------------------ */
/* Alg. 2: HashEncode                                                  */
/* ------------------------------------------------------------------ */
/*
 * x        n vectors of d bf16 values, vector i starts at x + i*x_stride
 * W        [d, r] fp32, row-major (r fastest)
 * codes    [n, r/32] packed bits (output)
 * near     [n, r/32] or NULL: bit set where |projection| < band (so a harness
 *          can exclude those bits from bit-exact comparison)
 * proj     [n, r] doubles or NULL: the projections themselves
 */
void oracle_hash_encode(const uint16_t* x, int64_t n, int64_t d, int64_t x_stride,
                        const float* W, int64_t r,
                        uint32_t* codes, uint32_t* near, double band, double* proj) {
    int64_t words = r / 32;
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t w = 0; w < words; ++w) {
            codes[v * words + w] = 0;
            if (near) near[v * words + w] = 0;
        }
        for (int64_t j = 0; j < r; ++j) {
            double y = 0.0;
            for (int64_t i = 0; i < d; ++i)
                y += bf16_to_double(x[v * x_stride + i]) * (double)W[i * r + j];
            if (proj) proj[v * r + j] = y;
            if (y >= 0.0) codes[v * words + (j >> 5)] |= (uint32_t)1 << (j & 31);
            if (near && fabs(y) < band) near[v * words + (j >> 5)] |= (uint32_t)1 << (j & 31);
        }
    }
}

/* ------------------------------------------------------------------ */
/* Alg. 3: Hamming score with aggregation over the query group         */
/* ------------------------------------------------------------------ */
static int bitcount32(uint32_t v) {
    int c = 0;
    for (int b = 0; b < 32; ++b) c += (int)((v >> b) & 1u);
    return c;
}

/* scores[n] = sum over g < G of bitcount(xor(qcodes[g], codes[n])) */
void oracle_hamming_score(const uint32_t* qcodes, int64_t G, const uint32_t* codes,
                          int64_t L, int64_t words, int32_t* scores) {
    for (int64_t n = 0; n < L; ++n) {
        int32_t s = 0;
        for (int64_t g = 0; g < G; ++g)
            for (int64_t w = 0; w < words; ++w)
                s += bitcount32(qcodes[g * words + w] ^ codes[n * words + w]);
        scores[n] = s;
    }
}

/* ------------------------------------------------------------------ */
/* Alg. 3: TopK(S, N) -- k smallest distances, lower index wins ties    */
/* ------------------------------------------------------------------ */
typedef struct { int32_t score; int32_t index; } pair_t;

static int cmp_pair(const void* a, const void* b) {
    const pair_t* p = (const pair_t*)a;
    const pair_t* q = (const pair_t*)b;
    if (p->score != q->score) return p->score < q->score ? -1 : 1;
    if (p->index != q->index) return p->index < q->index ? -1 : 1;
    return 0;
}
static int cmp_i32(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

/* Writes min(k, L) indices (ascending) into idx and returns that count. */
int64_t oracle_topk(const int32_t* scores, int64_t L, int64_t k, int32_t* idx) {
    if (L <= 0 || k <= 0) return 0;
    pair_t* p = (pair_t*)malloc((size_t)L * sizeof(pair_t));
    for (int64_t n = 0; n < L; ++n) { p[n].score = scores[n]; p[n].index = (int32_t)n; }
    qsort(p, (size_t)L, sizeof(pair_t), cmp_pair);
    int64_t cnt = k < L ? k : L;
    for (int64_t t = 0; t < cnt; ++t) idx[t] = p[t].index;
    free(p);
    qsort(idx, (size_t)cnt, sizeof(int32_t), cmp_i32);
    return cnt;
}

/* ------------------------------------------------------------------ */
/* Attention over a list of rows (Eq. 2 third line, scale of Eq. 1)    */
/* ------------------------------------------------------------------ */
/*
 * q [d] bf16; K, V: row n starts at K + n*row_stride; idx[count] row numbers
 * (idx == NULL means rows 0..count-1); out [d] doubles.
 * count == 0 gives zeros.
 */
void oracle_attention_rows(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                           int64_t row_stride, const int32_t* idx, int64_t count,
                           int64_t d, double scale, double* out) {
    for (int64_t c = 0; c < d; ++c) out[c] = 0.0;
    if (count <= 0) return;
    double* s = (double*)malloc((size_t)count * sizeof(double));
    double m = -INFINITY;
    for (int64_t t = 0; t < count; ++t) {
        int64_t n = idx ? idx[t] : t;
        double dot = 0.0;
        for (int64_t c = 0; c < d; ++c)
            dot += bf16_to_double(q[c]) * bf16_to_double(K[n * row_stride + c]);
        s[t] = dot * scale;
        if (s[t] > m) m = s[t];
    }
    double denom = 0.0;
    for (int64_t t = 0; t < count; ++t) { s[t] = exp(s[t] - m); denom += s[t]; }
    for (int64_t t = 0; t < count; ++t) {
        int64_t n = idx ? idx[t] : t;
        double p = s[t] / denom;
        for (int64_t c = 0; c < d; ++c) out[c] += p * bf16_to_double(V[n * row_stride + c]);
    }
    free(s);
}

/* ================================================================== */
/* Batch drivers over the cache layout                                 */
/*   q      [B, Hq, d]            bf16                                  */
/*   K, V   [B, Hkv, L_cap, d]    bf16                                  */
/*   W_H    [Hkv, d, r]           fp32                                  */
/*   codes  [B, Hkv, L_cap, r/32] u32                                   */
/*   qcodes [B, Hq, r/32]         u32                                   */
/*   scores [B, Hkv, L_cap]       i32 (rows >= seq_len[b] untouched)    */
/*   idx    [B, Hkv, k_max]       i32 (entries past the count = -1)     */
/* One (sequence, KV head) pair is one independent unit of work.       */
/* ================================================================== */

/* HashEncode of cache rows [start[b], start[b]+n_new[b]) of every unit. */
void oracle_encode_keys_batch(const uint16_t* K, const float* W_H,
                              const int32_t* start, const int32_t* n_new,
                              int64_t B, int64_t Hkv, int64_t L_cap, int64_t d, int64_t r,
                              uint32_t* codes, uint32_t* near, double band) {
    int64_t words = r / 32;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < Hkv; ++h) {
            int64_t unit = b * Hkv + h;
            int64_t s = start[b], n = n_new[b];
            if (n <= 0) continue;
            oracle_hash_encode(K + (unit * L_cap + s) * d, n, d, d, W_H + h * d * r, r,
                               codes + (unit * L_cap + s) * words,
                               near ? near + (unit * L_cap + s) * words : NULL, band, NULL);
        }
    }
}

/* Same, but parallel over blocks of keys (for one long prefill). */
void oracle_encode_keys_bulk(const uint16_t* K, const float* W_H,
                             const int32_t* start, const int32_t* n_new,
                             int64_t B, int64_t Hkv, int64_t L_cap, int64_t d, int64_t r,
                             uint32_t* codes, uint32_t* near, double band) {
    int64_t words = r / 32;
    const int64_t blk = 256;
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < Hkv; ++h) {
            int64_t unit = b * Hkv + h;
            int64_t s = start[b], n = n_new[b];
            if (n <= 0) continue;
            int64_t nblk = (n + blk - 1) / blk;
#pragma omp parallel for schedule(dynamic, 1)
            for (int64_t ib = 0; ib < nblk; ++ib) {
                int64_t r0 = s + ib * blk;
                int64_t cnt = (ib + 1) * blk <= n ? blk : n - ib * blk;
                oracle_hash_encode(K + (unit * L_cap + r0) * d, cnt, d, d, W_H + h * d * r, r,
                                   codes + (unit * L_cap + r0) * words,
                                   near ? near + (unit * L_cap + r0) * words : NULL, band, NULL);
            }
        }
    }
}

/* HashEncode of every query head with the weights of its KV head. */
void oracle_encode_query_batch(const uint16_t* q, const float* W_H,
                               int64_t B, int64_t Hq, int64_t Hkv, int64_t d, int64_t r,
                               uint32_t* qcodes, uint32_t* near, double band) {
    int64_t words = r / 32, G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t hq = 0; hq < Hq; ++hq) {
            int64_t i = b * Hq + hq;
            oracle_hash_encode(q + i * d, 1, d, d, W_H + (hq / G) * d * r, r,
                               qcodes + i * words, near ? near + i * words : NULL, band, NULL);
        }
    }
}

void oracle_score_batch(const uint32_t* qcodes, const uint32_t* codes, const int32_t* seq_len,
                        int64_t B, int64_t Hq, int64_t Hkv, int64_t L_cap, int64_t r,
                        int32_t* scores) {
    int64_t words = r / 32, G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < Hkv; ++h) {
            int64_t unit = b * Hkv + h;
            oracle_hamming_score(qcodes + (b * Hq + h * G) * words, G,
                                 codes + unit * L_cap * words, seq_len[b], words,
                                 scores + unit * L_cap);
        }
    }
}

void oracle_topk_batch(const int32_t* scores, const int32_t* seq_len, const int32_t* k,
                       int64_t B, int64_t Hkv, int64_t L_cap, int64_t k_max, int32_t* idx) {
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < Hkv; ++h) {
            int64_t unit = b * Hkv + h;
            int64_t kk = k[b] < k_max ? k[b] : k_max;
            int64_t cnt = oracle_topk(scores + unit * L_cap, seq_len[b], kk, idx + unit * k_max);
            for (int64_t t = cnt; t < k_max; ++t) idx[unit * k_max + t] = -1;
        }
    }
}

/* Attention of every query head over the rows listed for its KV head
 * (the leading non-negative entries of the unit's idx row). */
void oracle_sparse_decode_batch(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                                const int32_t* idx, int64_t B, int64_t Hq, int64_t Hkv,
                                int64_t L_cap, int64_t d, int64_t k_max, double scale,
                                double* out) {
    int64_t G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t hq = 0; hq < Hq; ++hq) {
            int64_t unit = b * Hkv + hq / G;
            const int32_t* row = idx + unit * k_max;
            int64_t cnt = 0;
            while (cnt < k_max && row[cnt] >= 0) ++cnt;
            oracle_attention_rows(q + (b * Hq + hq) * d, K + unit * L_cap * d,
                                  V + unit * L_cap * d, d, row, cnt, d, scale,
                                  out + (b * Hq + hq) * d);
        }
    }
}

/* Eq. 1 for every query head over rows 0..seq_len[b]-1 of its KV head. */
void oracle_dense_decode_batch(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                               const int32_t* seq_len, int64_t B, int64_t Hq, int64_t Hkv,
                               int64_t L_cap, int64_t d, double scale, double* out) {
    int64_t G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t hq = 0; hq < Hq; ++hq) {
            int64_t unit = b * Hkv + hq / G;
            oracle_attention_rows(q + (b * Hq + hq) * d, K + unit * L_cap * d,
                                  V + unit * L_cap * d, d, NULL, seq_len[b], d, scale,
                                  out + (b * Hq + hq) * d);
        }
    }
}

/*
 * One whole decode step (Alg. 3 in its stated order), given that the new K/V
 * row of each sequence already sits at cache row seq_len[b]-1:
 *   encode that key row into the code cache (if append != 0), encode q,
 *   score all seq_len[b] cached codes, select, attend.
 * scores / idx / qcodes are scratch outputs the caller provides (and may inspect).
 */
void oracle_decode_step(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                        const float* W_H, uint32_t* codes, const int32_t* seq_len,
                        const int32_t* k, int append,
                        int64_t B, int64_t Hq, int64_t Hkv, int64_t L_cap, int64_t d,
                        int64_t r, int64_t k_max, double scale,
                        uint32_t* qcodes, int32_t* scores, int32_t* idx, double* out) {
    if (append) {
        int32_t* st = (int32_t*)malloc((size_t)B * sizeof(int32_t));
        int32_t* nn = (int32_t*)malloc((size_t)B * sizeof(int32_t));
        for (int64_t b = 0; b < B; ++b) { st[b] = seq_len[b] - 1; nn[b] = 1; }
        oracle_encode_keys_batch(K, W_H, st, nn, B, Hkv, L_cap, d, r, codes, NULL, 0.0);
        free(st); free(nn);
    }
    oracle_encode_query_batch(q, W_H, B, Hq, Hkv, d, r, qcodes, NULL, 0.0);
    oracle_score_batch(qcodes, codes, seq_len, B, Hq, Hkv, L_cap, r, scores);
    oracle_topk_batch(scores, seq_len, k, B, Hkv, L_cap, k_max, idx);
    oracle_sparse_decode_batch(q, K, V, idx, B, Hq, Hkv, L_cap, d, k_max, scale, out);
}
