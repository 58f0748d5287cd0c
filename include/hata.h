/*
 * hata.h -- C ABI of the MI355X (gfx950) implementation of the HATA decode-attention
 * hot path: hash-aware top-k attention for one decode step (paper: "HATA: Trainable and
 * Hardware-Efficient Hash-Aware Top-k Attention", Sec. 3.2 and Sec. 4).
 *
 * One decode step (Alg. 3 of the paper), per (sequence, KV head) unit:
 *   1. HashEncode the query heads and the newly cached key (Alg. 2),
 *   2. score every cached key code by Hamming distance to the query codes,
 *      summed over the query heads that share the KV head,
 *   3. select the k keys with the smallest distance,
 *   4. run softmax attention over only those k K/V rows.
 *
 * General rules of every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller unless a comment says
 *     "host".  The library never allocates or frees device memory: all scratch lives in
 *     the workspace the caller hands to hata_create().
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; they never synchronise the device.  Calls that share one context
 *     must be issued on one stream (or be otherwise ordered): they share the workspace.
 *   - Return value: HATA_OK (0) or a negative hata_status.  Nothing is enqueued after a
 *     validation failure.  No exception or abort crosses this boundary.
 *   - bf16 tensors are passed as void* to 16-bit patterns (upper half of an IEEE fp32).
 *   - Per-sequence integers (seq_len, k, start, n_new) are device arrays, read by the
 *     kernels; the host never waits for them.
 *
 * Tensor layouts (B sequences, Hq query heads, Hkv KV heads, G = Hq / Hkv, d = 128,
 * r hash bits, Wd = r / 32 words, "unit" u = b * Hkv + h):
 *   q, out    [B, Hq, d]            bf16, contiguous
 *   out_f32   [B, Hq, d]            fp32, contiguous (optional copy of the un-rounded output)
 *   K, V      row n of unit (b, h) starts at  base + b*kv_stride_b + h*kv_stride_h + n*kv_stride_n
 *             (strides in elements; the d values of a row are contiguous; every row 16-byte aligned)
 *   W_H       [Hkv, d, r]           fp32, contiguous; query head hq uses W_H[hq / G]
 *   codes     [B, Hkv, L_cap, Wd]   uint32, contiguous; bit j of a code = bit (j % 32) of word j / 32,
 *             set iff the j-th projection is >= 0
 *   qcodes    [B, Hq, Wd]           uint32
 *   scores    [B, Hkv, L_cap]       uint16, Hamming distance summed over the G heads (0 .. G*r)
 *   idx       [B, Hkv, k_max]       int32, the selected cache rows in ascending order,
 *                                   entries past min(k[b], seq_len[b]) are -1
 *   seq_len   [B] int32             number of cached rows of sequence b, INCLUDING the token
 *                                   appended in this step (Alg. 3 appends before it scores)
 *   k         [B] int32             token budget of sequence b (clamped to [0, k_max] on device)
 */
#ifndef HATA_H
#define HATA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HATA_OK = 0,
    HATA_EINVAL = -1,       /* NULL pointer, B out of range, bad stride/alignment, ... */
    HATA_EUNSUPPORTED = -2, /* a shape this build has no kernel for */
    HATA_EWORKSPACE = -3,   /* workspace NULL, misaligned or too small */
    HATA_EHIP = -4,         /* a HIP runtime call failed (launch error, no device, ...) */
    HATA_ETIMEOUT = -5,     /* hata_check(): a single-launch decode step gave up its bounded in-kernel wait */
    HATA_ETOOLARGE = -6     /* hata_sparse_decode_static(): the shape needs more scratch than its static buffer holds */
} hata_status;

typedef struct {
    int32_t B_max;   /* largest batch any call will pass */
    int32_t Hq;      /* query heads */
    int32_t Hkv;     /* KV heads; Hq % Hkv == 0, Hq / Hkv <= 16 */
    int32_t d;       /* head dimension; must be 128 */
    int32_t r;       /* hash bits; multiple of 32, 32..256; (Hq/Hkv) * r <= 4096 */
    int32_t L_cap;   /* rows allocated per (sequence, KV head) in K, V and codes */
    int32_t k_max;   /* largest token budget; 1 <= k_max <= L_cap */
    int64_t kv_stride_b, kv_stride_h, kv_stride_n; /* K/V strides in elements; stride_n >= d, % 8 == 0 */
} hata_config;

typedef struct hata_ctx hata_ctx; /* opaque, host memory; owns nothing but its own struct */

/* Static message for a status code (host pointer, never NULL). */
const char* hata_strerror(int status);

/* Validates `cfg` and writes the workspace size (bytes) a context of that shape needs.
 * cfg, out: host pointers. */
int hata_workspace_bytes(const hata_config* cfg, size_t* out);

/* Creates a context.  `workspace` is device memory (256-byte aligned, at least
 * hata_workspace_bytes() bytes) that stays owned by the caller and must outlive the
 * context; its control words are cleared here with a synchronous hipMemset on the
 * current device.  ctx_out, cfg: host pointers. */
int hata_create(hata_ctx** ctx_out, const hata_config* cfg, void* workspace, size_t workspace_bytes);

/* Launch-shape choices a caller may fix instead of taking the defaults (sweeps over launch
 * shapes; tests of the batch slicing on small inputs; a device that is not the caller's alone).
 * A zero-initialised struct, or a NULL pointer, means "all defaults". */
typedef struct {
    int32_t chunk;         /* cached keys per scoring workgroup: 0 = default (the single-launch step then picks, per
                            * call, the size that needs the fewest launches for the batch), else 1024, 2048,
                            * 4096 or 8192 for every kernel, or 16384 / 32768 for the single-launch step alone
                            * (the other kernels keep their default) */
    int32_t attn_rows;     /* selected rows per attention workgroup of the three-launch form: 0 = default, else a power of two in 16..256 */
    int32_t par_merge;     /* single-launch form, merge of a unit's partials: -1 = default, 0 = by the last workgroup to arrive, 1 = a query head per workgroup (taken for launches with more than four chunks per unit; the default when a group has two heads or more) */
    int32_t shared_device; /* != 0: other work may run on the device beside the step, so the context starts in step mode 3 (see hata_set_step_mode) */
} hata_tuning;

/* hata_workspace_bytes / hata_create with the launch shapes of `tuning` (host pointer, may be
 * NULL): the chunk size changes the workspace size, so both calls must be given the same values.
 * HATA_EINVAL for a value outside the sets above. */
int hata_workspace_bytes_tuned(const hata_config* cfg, const hata_tuning* tuning, size_t* out);
int hata_create_tuned(hata_ctx** ctx_out, const hata_config* cfg, const hata_tuning* tuning,
                      void* workspace, size_t workspace_bytes);

/* Frees the host-side context (the workspace is the caller's). */
int hata_destroy(hata_ctx* ctx);

/*
 * Key-code writer (the key-code fill of Alg. 1 in bulk; Alg. 3 "Update code cache" for one appended key):
 *   codes[b, h, n, :] = BitPack(Sign(K[b, h, n, :] . W_H[h]))   for start[b] <= n < start[b] + n_new[b].
 * `max_new` (host value) is an upper bound of n_new[b] and sizes the launch; rows outside the
 * range, and rows >= L_cap, are not touched.  Small max_new (<= 8) uses an fp64-accumulating
 * kernel; larger uses the matrix-core projection kernel (r in {32, 64, 128, 256}: bf16 MFMA over an
 * exact three-way bf16 split of W_H, fp32 accumulation; other r: fp32 vector kernel), where a bit may
 * differ from an exact evaluation only if |projection| is below about 1e-4.
 */
int hata_encode_keys(hata_ctx* ctx, const void* K, const float* W_H,
                     const int32_t* start, const int32_t* n_new, int32_t B, int32_t max_new,
                     uint32_t* codes, void* stream);

/* Prepares the hash weights for the matrix-core key-code writer (the weights of HashEncode, Alg. 2,
 * are fixed once trained, Sec. 3.1): W_H [Hkv, d, r] fp32 becomes two fp16 planes per tile of 32 hash
 * columns -- hi = fp16(W S), lo = fp16(W S - hi), S a power of two that brings the tile's largest
 * weight below 2^14, so no sign changes -- laid out as the kernels' operand fragments, in the workspace.
 * Afterwards hata_encode_keys, hata_prefill_write and hata_prefill_write_paged calls of this context
 * that are given the SAME pointer W_H read the prepared planes instead of splitting the weights into
 * three bf16 planes in every workgroup: two matrix-core instructions per fragment instead of three.
 * The prepared form evaluates the projection to within 2^-22 of sum_c |K_c W_c| (about 5e-6 here), so,
 * like the unprepared form, its code bits can differ from an exact evaluation only where |projection|
 * is below about 1e-4; inside that band the two forms need not agree with each other.  The caller
 * promises that the tensor at W_H does not change until the next hata_prepare_weights call of this
 * context; W_H == NULL forgets the prepared tensor.  Enqueues one small kernel on `stream`; the calls
 * that use the planes must be ordered after it. */
int hata_prepare_weights(hata_ctx* ctx, const float* W_H, void* stream);

/* Prefill cache fill in one pass (Alg. 1: KCache <- K, VCache <- V, K_H = HashEncode(K)): the rows
 *   K_new[b, h, i, :], V_new[b, h, i, :], i < n_new[b]   (bf16, layout [B, Hkv, max_new, d], contiguous)
 * are written to cache rows start[b] + i of K and V (strides of the context) while their key codes
 * go to `codes` -- the keys are read once.  Same numerics as hata_encode_keys' matrix-core kernel;
 * r must be 32, 64, 128 or 256 (HATA_EUNSUPPORTED otherwise).  Rows >= L_cap are not touched. */
int hata_prefill_write(hata_ctx* ctx, const void* K_new, const void* V_new, const int32_t* start,
                       const int32_t* n_new, int32_t B, int32_t max_new, void* K, void* V,
                       uint32_t* codes, const float* W_H, void* stream);

/* Query-code writer (Alg. 3 "HashEncode(Q)"): qcodes[b, hq, :] = BitPack(Sign(q[b, hq, :] . W_H[hq / G])).
 * fp64 accumulation. */
int hata_encode_query(hata_ctx* ctx, const void* q, const float* W_H, int32_t B,
                      uint32_t* qcodes, void* stream);

/* Hamming scores (Alg. 3 "Calculate distance in Hamming space", with the aggregation over
 * query heads sharing a KV cache):
 *   scores[b, h, n] = sum_{g < G} bitcount(qcodes[b, h*G + g, :] xor codes[b, h, n, :])   for n < seq_len[b].
 * Entries n >= seq_len[b] are not written. */
int hata_hamming_score(hata_ctx* ctx, const uint32_t* qcodes, const uint32_t* codes,
                       const int32_t* seq_len, int32_t B, uint16_t* scores, void* stream);

/* Selection (Alg. 3 "Idx = TopK(S, N)"): the min(k[b], seq_len[b]) rows n < seq_len[b] with the
 * smallest (scores[n], n) in lexicographic order, i.e. smallest distance first and the lower
 * row on equal distance; written ascending, the rest of the idx row set to -1.
 * Scores above G*r are treated as G*r. */
int hata_topk(hata_ctx* ctx, const uint16_t* scores, const int32_t* seq_len, const int32_t* k,
              int32_t B, int32_t* idx, void* stream);

/* Attention over the gathered rows (Alg. 3 Gather + Attention; Eq. 2 third line):
 *   out[b, hq, :] = softmax_t( sm_scale * q[b, hq] . K[b, h, idx_t] ) . V[b, h, idx_t],  h = hq / G,
 * over the first min(k[b], k_max) entries of idx[b, h, :], skipping negative entries.
 * The gather is fused: no K_sparse / V_sparse is materialised.  bf16 inputs, fp32 accumulation.
 * A unit with no valid row gives zeros.  out_f32 may be NULL. */
int hata_sparse_decode(hata_ctx* ctx, const void* q, const void* K, const void* V,
                       const int32_t* idx, const int32_t* k, int32_t B, float sm_scale,
                       void* out, float* out_f32, void* stream);

/* The gather of Alg. 3 ("K_sparse, V_sparse = Gather(K, V, Idx)") materialised, for the offloading
 * variant (Sec. 5.3: the KV cache in host memory, the selected rows prefetched over the bus): copies
 * the selected rows into contiguous staging buffers
 *   K_stage, V_stage  [B, Hkv, k_max, d] bf16 (device memory, caller-owned):
 *   K_stage[b, h, t, :] = K[b, h, idx[b, h, t], :]   for t < min(k[b], k_max), likewise V.
 * K and V follow the context's strides and may be pinned, mapped host memory
 * (hata_host_device_pointer).  Negative or out-of-range index entries, and rows t past the budget,
 * leave their staged rows untouched.  Issued on a stream of its own it overlaps other layers'
 * work; attention over the staged rows is hata_sparse_decode on a context whose cache is the
 * staging buffer (L_cap = k_max, contiguous strides) with the index list 0, 1, 2, ...
 * max_workgroups (host value): 0 = one workgroup per block of 64 rows (caches in device memory);
 * n > 0 = at most n workgroups, each with 32 KB of reads outstanding.  With a cache in host
 * memory every outstanding read also delays whatever else crosses the bus, the launches of other
 * streams included: 32 is what kept the bus busy without stalling the other stream on the box
 * this was measured on. */
int hata_gather_rows(hata_ctx* ctx, const void* K, const void* V, const int32_t* idx, const int32_t* k,
                     int32_t B, int32_t max_workgroups, void* K_stage, void* V_stage, void* stream);

/* hata_sparse_decode for callers that cannot allocate device memory or keep a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (the shape is passed as the config itself, host pointer; no context), same kernels, same
 * results bit for bit; the attention partials and their arrival counters live in a buffer that
 * is part of the library's device image: 8 MiB per device, held until the process ends.
 * Limit: align256(B_max * Hq * 4) + B_max * Hq * splits * 520 bytes <= 8 MiB, where splits is the
 * number of row slices the launch plan cuts k_max into (at most 256); larger shapes return
 * HATA_ETOOLARGE and enqueue nothing.  The call allocates nothing, frees nothing, and only
 * enqueues kernels (a small fill kernel clears the counters first, so it may be captured).
 * Every call on a device uses that device's one buffer: calls that overlap in time on one device
 * (different streams, different threads) race and must be serialised by the caller. */
int hata_sparse_decode_static(const hata_config* cfg, const void* q, const void* K, const void* V,
                              const int32_t* idx, const int32_t* k, int32_t B, float sm_scale,
                              void* out, float* out_f32, void* stream);

/* Dense decode attention over the whole cache (Eq. 1), rows 0 .. seq_len[b]-1: the baseline the
 * sparse path is compared with.  Same numerics and outputs as hata_sparse_decode. */
int hata_dense_decode(hata_ctx* ctx, const void* q, const void* K, const void* V,
                      const int32_t* seq_len, int32_t B, float sm_scale,
                      void* out, float* out_f32, void* stream);

/* One whole decode step in the order of Alg. 3.  The caller has already copied the new K/V row
 * of each sequence to cache row seq_len[b]-1 (static pre-allocated cache).  If `append` != 0
 * that row is hash-encoded into `codes` first; then the query is encoded, all seq_len[b] codes
 * are scored, the budget is selected and attention runs over the selected rows.
 * Intermediate qcodes / idx (and scores, see hata_keep_step_scores) live in the workspace
 * (see hata_step_buffers).
 *
 * Launches (see hata_step_plan): for r in {32, 64, 128, 256} and Hq/Hkv in {1, 2, 4, 5, 8}, or 16
 * with r <= 128, a budget k_max of at most 65535 rows, and when the workgroups of at least one sequence
 * can be resident on the device at once,
 * the step is ONE kernel launch whose workgroups each take a chunk of 1024 to 32768 cached keys of
 * one (sequence, KV head) unit -- per call the chunk size that lets the fewest resident launches
 * cover the batch, the smallest such; a batch too large to be resident even at the largest chunk
 * goes as one launch per slice of it: hata_step_sub_batches, hata_step_plan -- and hand the query codes, the selection threshold and the attention partials to each
 * other through the workspace, waiting for one another inside the kernel.  Every such wait is
 * bounded: a workgroup that gives up raises a flag in the workspace and runs to its end; the
 * outputs of every (sequence, KV head) unit one of whose workgroups gave up are then overwritten
 * with NaN (out: bf16 0x7fc0, out_f32: NaN), so the failure shows in the data itself (the idx
 * rows of such a step are unspecified: -1 where the unit could still be marked, else whatever its
 * workgroups wrote), and the next hata_check() returns HATA_ETIMEOUT.  Otherwise
 * the step is three launches (encode; score + threshold; select + attend) with no in-kernel wait.
 * The residency test assumes the device runs nothing else at that moment and that the context is
 * used on the device that was current in hata_create(): a process that overlaps other kernels
 * with the step (other streams, other processes) should create the context with
 * hata_tuning.shared_device set (or call hata_set_step_mode(ctx, 3)), or watch hata_check().
 * Both forms select the same rows and agree on the output to rounding.  Either form may be
 * recorded into a HIP graph and replayed (no memset nodes, no host-side state a replay depends
 * on: the single-launch kernel retires the words its workgroups publish before it ends);
 * hata_check() is a synchronising call and stays outside the capture. */
int hata_decode_step(hata_ctx* ctx, const void* q, const void* K, const void* V, const float* W_H,
                     uint32_t* codes, const int32_t* seq_len, const int32_t* k, int32_t B,
                     int32_t append, float sm_scale, void* out, float* out_f32, void* stream);

/* The selection half of hata_decode_step alone (Alg. 3 from "Update code cache" to "Select
 * top-k"): the appended key (if `append` != 0; K is read for that row only and may be NULL
 * otherwise) and the query are hash-encoded, all seq_len[b] codes are scored, and the budget is
 * selected into
 *   idx  [B, Hkv, k_max] int32 (caller-owned device memory): ascending cache rows, -1 past the budget.
 * For the offloading variant (Sec. 5.3), where the selected rows are then fetched with
 * hata_gather_rows while another layer computes.  ONE launch of the single-launch kernel of
 * hata_decode_step, stopped after the selection, with the same residency rule, bounded waits and
 * hata_check() reporting (the lists of a unit whose workgroup gave up are unspecified);
 * HATA_EUNSUPPORTED for the shapes and batches whose step takes three launches. */
int hata_select_step(hata_ctx* ctx, const void* q, const void* K, const float* W_H, uint32_t* codes,
                     const int32_t* seq_len, const int32_t* k, int32_t B, int32_t append, int32_t* idx,
                     void* stream);

/*
 * Paged (block-table) cache layout: the serving-side layout in which sequences grow page by page
 * out of shared pools instead of owning L_cap rows each.
 *   K_pool, V_pool  [n_pages, Hkv, page_rows, d]  bf16, contiguous (the context's K/V strides are not used)
 *   codes_pool      [n_pages, Hkv, page_rows, r/32] uint32
 *   block_table     [B, max_blocks] int32 (device): row n of sequence b is row n % page_rows of
 *                   page block_table[b, n / page_rows]
 * page_rows is a power of two >= 16 (256 or more keeps a page's codes a multi-KB contiguous read);
 * max_blocks * page_rows <= 2^30; n_pages * Hkv * page_rows < 2^31.  Sequence lengths are clamped to
 * min(L_cap, max_blocks * page_rows); L_cap still sizes the workspace and the launch.  Page numbers
 * read from the table are clamped to [0, n_pages) (a wrong entry gives wrong results, never an
 * access outside the pools); entries past a sequence's last block are not read.  Two sequences
 * may share pages for reading; the page that holds an appended row must belong to one sequence.
 *
 * hata_decode_step_paged: hata_decode_step on that layout, same outputs (Idx holds LOGICAL row
 * numbers).  It exists in the single-launch form only: HATA_EUNSUPPORTED when the shape does not
 * fit it (see hata_decode_step; hata_set_step_mode does not apply).
 */
int hata_decode_step_paged(hata_ctx* ctx, const void* q, const void* K_pool, const void* V_pool,
                           const float* W_H, uint32_t* codes_pool, const int32_t* block_table,
                           int32_t max_blocks, int32_t page_rows, int32_t n_pages,
                           const int32_t* seq_len, const int32_t* k, int32_t B, int32_t append,
                           float sm_scale, void* out, float* out_f32, void* stream);

/* hata_prefill_write into the paged layout above (Alg. 1 in one pass): row start[b] + i of
 * sequence b goes to the page its block-table entry names; the blocks that cover rows
 * start[b] .. start[b] + n_new[b] - 1 must be assigned in the table before the call. */
int hata_prefill_write_paged(hata_ctx* ctx, const void* K_new, const void* V_new, const int32_t* start,
                             const int32_t* n_new, int32_t B, int32_t max_new, void* K_pool, void* V_pool,
                             uint32_t* codes_pool, const int32_t* block_table, int32_t max_blocks,
                             int32_t page_rows, int32_t n_pages, const float* W_H, void* stream);

/* Host-side query of how hata_decode_step() runs a batch of B sequences; nothing is enqueued.
 * *n_launches: 1 (single-launch form) or 3 (three-launch form); *chunk: cached keys per scoring
 * workgroup for a batch of this size; *n_chunks: scoring workgroups per (sequence, KV head).  Any
 * output pointer (host) may be NULL. */
int hata_step_plan(const hata_ctx* ctx, int32_t B, int32_t* n_launches, int32_t* chunk, int32_t* n_chunks);

/* A batch with more (sequence, KV head) units than one launch can keep resident still runs in the
 * single-launch form, as consecutive launches over equal slices of the batch (each a whole step
 * for its sequences).  *n_sub (host): the number of such launches for a batch of B, 1 when the
 * batch fits one launch, 0 when hata_decode_step() uses the three-launch form. */
int hata_step_sub_batches(const hata_ctx* ctx, int32_t B, int32_t* n_sub);

/* mode 0 (default): hata_decode_step() uses the single-launch form whenever it fits, a batch too
 *   large to be resident as consecutive launches over slices of it;
 * mode 1: as mode 0, but a batch of any size goes in ONE launch.  Its workgroups then become
 *   resident in the order of their indices as earlier ones retire.  The workgroups of a unit lie
 *   within a span of 8 * chunks-per-unit consecutive indices when the number of units is a
 *   multiple of eight (eight units are interleaved, one per L2), chunks-per-unit otherwise; the
 *   mode is taken only when such a span fits the device at once (else the batch goes in slices as
 *   in mode 0), so the units with the lowest indices still at work are always resident as a whole
 *   and finish -- which is how the hardware dispatches a grid, not a guarantee of the
 *   programming model: should a wait ever give up, hata_check() reports it (HATA_ETIMEOUT) and
 *   the step must be repeated in mode 0 or 3;
 * mode 3: always the three-launch form (no in-kernel waits). */
int hata_set_step_mode(hata_ctx* ctx, int32_t mode);

/* The Hamming scores of a step are an intermediate: the single-launch form keeps them on chip and
 * writes the score region of the workspace only if asked to (keep != 0; default off, which saves
 * 2 bytes of HBM writes per cached key).  The three-launch form always writes it (its second
 * launch reads it back). */
int hata_keep_step_scores(hata_ctx* ctx, int32_t keep);

/* Bound of every in-kernel wait of the single-launch form, in polls (0 restores the default, 2^18:
 * far longer than any step).  A tiny bound makes the waits give up at once -- the kernel still runs
 * to its end, writes nothing out of bounds, and hata_check() then returns HATA_ETIMEOUT -- which is
 * how the error path is exercised in the tests. */
int hata_set_wait_limit(hata_ctx* ctx, int32_t polls);

/* Waits for `stream` (hipStreamSynchronize), then reports whether a single-launch decode step of
 * this context gave up an in-kernel wait since the last check: HATA_OK, or HATA_ETIMEOUT (the
 * flag and the workspace's control words are cleared; the outputs of the steps since the last
 * check must be discarded).  The only synchronous call of the library besides hata_create();
 * never needed for the three-launch form. */
int hata_check(hata_ctx* ctx, void* stream);

/* KV cache in host memory (the paper's offloading variant, Sec. 5.3: hash codes stay on the GPU,
 * K and V live in pinned host memory and only the selected rows cross the bus).  Every K / V
 * argument above may be the device-side address of PINNED, MAPPED host memory (hipHostMalloc):
 * the attention kernels then gather the selected rows over the bus themselves, nothing is staged.
 * This helper returns that address for a host pointer (*dev_out; host pointers in and out) or
 * HATA_EINVAL if the memory is not pinned and mapped -- pass nothing else to a kernel. */
int hata_host_device_pointer(void* host, void** dev_out);

/* Device pointers of the workspace regions hata_decode_step() writes (layouts as above, sized
 * for B_max); valid until the workspace is released.  Any output pointer may be NULL. */
int hata_step_buffers(hata_ctx* ctx, uint32_t** qcodes, uint16_t** scores, int32_t** idx);

/* Diagnostic (no part of the method; used by bench.py --overlap-probe): one launch of 256 workgroups
 * in which four waves per workgroup issue mfma_iters x 16 bf16 matrix-core instructions on operands
 * taken from the first 10 KB of buf (mode bit 0) and four waves read the workgroup's 1/256 share of
 * buf [bytes] with 16-byte loads (mode bit 1).  buf: device memory, 16-byte aligned, at least 4 MiB,
 * read only; fill it with values like the workload's (the matrix cores' rate depends on them).  The
 * caller times mode 1, mode 2 and mode 3 to see whether the two overlap on the device at hand.
 * Returns HATA_EINVAL for bad arguments; enqueues on `stream` and returns. */
int hata_probe_mfma_stream(const void* buf, size_t bytes, int32_t mfma_iters, int32_t mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HATA_H */
