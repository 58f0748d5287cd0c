/*
 * hata_train.h -- C ABI of the MI355X (gfx950) learning-to-hash trainer of HATA: one SGD step on
 * the hash weights W_H of one attention head (paper: Sec. 3.1 "Learning-to-Hash for Top-k
 * Attention", the final multi-query hashing model; App. B.2 training setup).
 *
 * For a batch of N triplets (q_n, k_n, s_n) -- a query, a key and their similarity label -- with
 *   h(x) = 2 Sigmoid(sigma x W_H) - 1,
 * the loss is
 *   L = eps * scale_sim * sum_n s_n ||h(q_n) - h(k_n)||^2                  (similarity)
 *     + eta * scale_bal * sum_j || sum_{n in query j} h(k_n) ||^2          (bit balance, per query)
 *     + lam * || W_H^T W_H - I_r ||_F                                      (uncorrelation)
 * and a step is  g = dL/dW_H + weight_decay * W_H;  v = momentum * v + g;  W_H -= lr * v.
 * scale_sim / scale_bal are not in the paper: 1 gives the sums as printed, 1/N and 1/N^2 the mean
 * forms.  The balance term is summed per sampled query j, as the final hashing model prints it:
 * the triplets of one query occupy whole blocks of HATA_TRAIN_BLOCK consecutive triplets (a query
 * whose count is not a multiple is padded with all-zero rows q = k = 0, s = 0, which add nothing
 * to any term or to the gradient), and `block_query` names the query of every block.  Without
 * names the whole batch counts as one query (stored batches are shuffled and carry no query
 * index, App. B.1).
 *
 * Rules as in hata.h: every data pointer is a DEVICE pointer owned by the caller unless marked
 * "host"; nothing is allocated or freed (scratch lives in the caller's workspace); `stream` is a
 * hipStream_t passed as void*; calls only enqueue work; calls that share a context must be
 * ordered on one stream; status codes are hata_status.
 *
 * Layouts:  Q, K  [n, d] bf16 (16-bit patterns), contiguous, d = 128
 *           s     [n]    fp32
 *           W, v  [d, r] fp32, contiguous, updated in place (v: the momentum buffer)
 *           grad  [d, r] fp32 (optional output: dL/dW_H of this batch, without the weight decay)
 *           loss  [3]    fp32 (optional output: the three terms in the order above)
 *           block_query [ceil(n / HATA_TRAIN_BLOCK)] int32: query id of each block, 0 <= id < n_queries
 */
#ifndef HATA_TRAIN_H
#define HATA_TRAIN_H

#include <stddef.h>
#include <stdint.h>

#include "hata.h"

#ifdef __cplusplus
extern "C" {
#endif

#define HATA_TRAIN_BLOCK 128 /* triplets per block: the granularity of the per-query balance term */

typedef struct {
    int32_t d;     /* head dimension; must be 128 */
    int32_t r;     /* hash bits; 32, 64, 128 or 256 */
    int32_t n_max; /* largest batch (triplets) any call will pass; >= 1 */
} hata_train_config;

typedef struct { /* host struct, read at call time (App. B.2 hyper-parameter table for the defaults) */
    float sigma, eps, eta, lam;
    float scale_sim, scale_bal;
    float lr, momentum, weight_decay;
} hata_train_hparams;

typedef struct hata_train_ctx hata_train_ctx; /* opaque, host memory */

/* Workspace size (bytes) for a context of that shape.  cfg, out: host pointers. */
int hata_train_workspace_bytes(const hata_train_config* cfg, size_t* out);

/* Creates a context over `workspace` (device, 256-byte aligned, >= hata_train_workspace_bytes()
 * bytes, owned by the caller, must outlive the context). */
int hata_train_create(hata_train_ctx** ctx_out, const hata_train_config* cfg, void* workspace,
                      size_t workspace_bytes);

int hata_train_destroy(hata_train_ctx* ctx);

/* One SGD step on W (and v) from the n triplets (Q[i], K[i], s[i]), 1 <= n <= n_max.
 * block_query (device, may be NULL = one query) and n_queries (1 <= n_queries <= number of blocks;
 * ignored when block_query is NULL) select the per-query balance term; ids outside [0, n_queries)
 * count as the nearest valid id.  hp: host pointer.  grad and loss may be NULL.  Six small
 * launches on `stream`; the projections and the weight-gradient contraction run on the matrix
 * cores (bf16 MFMA over exact three-way bf16 splits of the fp32 operands, fp32 accumulation). */
int hata_train_step(hata_train_ctx* ctx, const void* Q, const void* K, const float* s, int32_t n,
                    const int32_t* block_query, int32_t n_queries, float* W, float* v,
                    const hata_train_hparams* hp, float* grad, float* loss, void* stream);

/* Training-data construction of App. B.1 (steps 3-4) for ONE sampled query: the qk scores of the
 * query against m keys (accumulated in fp64), the best floor(m / 10) pairs (at least one) labelled
 * 20 .. 1 in equal steps by rank -- the earlier key first on equal scores -- and the others -1.
 *   q [d] bf16, K [m, d] bf16, s [m] fp32 (output), 1 <= m <= n_max; two launches on `stream`. */
int hata_train_make_labels(hata_train_ctx* ctx, const void* q, const void* K, int32_t m, float* s,
                           void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HATA_TRAIN_H */
