// Host-side internals of libhata: the context and the per-stage launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hata.h"

// Words between the arrival counters of consecutive units in the single-launch step (128 bytes:
// the workgroups of different units then never queue their arrivals on one cache line).  The
// three-launch kernels index the same arrays densely.
#define HATA_COUNTER_STRIDE 32
// 64-bit words between the records of consecutive chunks (two are used): a cache line per chunk, so
// that the workgroups polling for their records do not all read the same lines
#define HATA_REC_STRIDE 8

struct hata_ctx {
    hata_config cfg;
    int G;            // query heads per KV head
    int Wd;           // 32-bit words per code
    int NB;           // number of score values: G*r + 1
    int NBP;          // NB rounded up to a multiple of 8 (row pitch of the chunk histograms)
    int chunk;        // cached keys handled by one scoring / selection workgroup
    int n_chunks;     // ceil(L_cap / chunk)
    int HT;           // query heads of a group handled together by one attention workgroup
    // keys per workgroup the single-launch step may use (ascending; [0] = chunk unless the caller fixed
    // another size) and how many of its workgroups are resident at once with each (0 = unusable); a
    // call takes the size that needs the fewest launches for its batch, the smallest such
    int coop_opts, coop_opt_chunk[4], coop_opt_cap[4];
    int sparse_rows;  // selected rows per attention workgroup
    int sparse_splits;
    int dense_rows;   // cache rows per dense-attention workgroup
    int dense_splits;
    // regions of the caller's workspace
    uint32_t* qcodes;      // [B_max, Hq, Wd]
    uint16_t* scores;      // [B_max, Hkv, L_cap]
    int32_t* idx;          // [B_max, Hkv, k_max]
    uint16_t* chunk_hist;  // [B_max*Hkv, n_chunks, NBP]
    int32_t* chunk_info;   // [B_max*Hkv, n_chunks + 1, 2] = {output offset, ties taken}
    int32_t* unit_info;    // [B_max*Hkv, 2] = {threshold, selected count}
    uint32_t* unit_counter;  // [B_max*Hkv (* HATA_COUNTER_STRIDE in the cooperative step)] scored chunks of a unit (self-resetting)
    uint32_t* unit_hist;     // [B_max*Hkv, NB] total histogram of a unit (self-clearing)
    uint32_t* attn_counter;  // [B_max*Hq (cooperative step: per unit, HATA_COUNTER_STRIDE apart)] finished attention slices (self-resetting)
    unsigned long long* coop_rec;  // [B_max*Hkv, n_chunks, HATA_REC_STRIDE] epoch-stamped chunk records, two words used (cooperative step)
    unsigned long long* coop_qrec; // [B_max*Hkv, n_chunks, G*Wd] epoch-stamped query code words, one copy per chunk (cooperative step)
    uint32_t* error_word;    // [1] set by a cooperative launch that gave up waiting
    uint32_t epoch;          // launch counter of the cooperative step
    int spin_limit;          // polls an in-kernel wait makes before it gives up (0 = the default)
    int keep_scores;         // single-launch step also writes the score array
    int par_merge;           // single-launch step merges the heads of a unit in several workgroups
    int step_mode;           // 0 = single launch when it fits, 3 = always three launches
    int cus;                 // compute units of the device that was current in hata_create
    int coop_opt_cap_paged[4];  // the same for the block-table variant of the kernel
    float* partials;       // [B_max*Hq, max(sparse_splits, dense_splits), d + 2]
    void* wplanes;               // [Hkv, r/32, 8, 2, 64] 16-byte fragments: the two scaled fp16 planes of the hash weights (prefill key encode)
    const float* prepared_W_H;   // the weight tensor those planes were made from (nullptr: none)
    size_t control_bytes;  // bytes from chunk_info up to the partials: the control words, cleared at creation and after a give-up
};

namespace hata {

// Block table of a paged cache (table == nullptr: the contiguous layout).  Page p of the pools
// holds 1 << shift rows of every KV head -- K, V [n_pages, Hkv, page_rows, d], codes [n_pages,
// Hkv, page_rows, Wd] -- and row n of sequence b lives in page table[b * max_blocks + (n >> shift)]
// at row n & (page_rows - 1).  Device code clamps the page numbers it reads to [0, n_pages).
struct PageView {
    const int32_t* table;
    int max_blocks, shift, n_pages;
};

// every launcher returns hipGetLastError() of its launches
hipError_t launch_encode_vectors(const hata_ctx* c, const void* q, uint32_t* qcodes,
                                 const void* K, const int32_t* start, const int32_t* n_new,
                                 int max_new, int from_seq_len, uint32_t* codes,
                                 const float* W_H, int B, hipStream_t s);
// K_new .. V_out non-null: fused cache fill (rows read from K_new / V_new [B, Hkv, max_new, d],
// written to the caches K_out / V_out while the key codes are computed)
hipError_t launch_encode_bulk(const hata_ctx* c, const void* K, const float* W_H,
                              const int32_t* start, const int32_t* n_new, int B, int max_new,
                              uint32_t* codes, hipStream_t s, const void* K_new = nullptr,
                              const void* V_new = nullptr, void* K_out = nullptr, void* V_out = nullptr,
                              const PageView* pages = nullptr);
hipError_t launch_split_weights(const hata_ctx* c, const float* W_H, hipStream_t s);
hipError_t launch_score(const hata_ctx* c, const uint32_t* qcodes, const uint32_t* codes,
                        const int32_t* seq_len, int B, uint16_t* scores, const int32_t* kbud,
                        hipStream_t s);
hipError_t launch_topk(const hata_ctx* c, const uint16_t* scores, const int32_t* seq_len,
                       const int32_t* k, int B, int32_t* idx, hipStream_t s);
// mode: 0 = rows from idx, 1 = dense, 2 = select on the fly (writes idx)
hipError_t launch_attention(const hata_ctx* c, int mode, const void* q, const void* K,
                            const void* V, int32_t* idx, const int32_t* count_src,
                            const int32_t* seq_len, int B, float sm_scale, void* out,
                            float* out_f32, hipStream_t s);

hipError_t launch_gather_rows(const hata_ctx* c, const void* K, const void* V, const int32_t* idx,
                              const int32_t* k, int B, int max_workgroups, void* K_stage, void* V_stage,
                              hipStream_t s);

// encode + score + select + attend in one cooperative launch; returns hipErrorNotSupported if
// this shape has no cooperative kernel
hipError_t launch_coop_step(hata_ctx* c, const void* q, const void* K, const void* V,
                            const float* W_H, uint32_t* codes, int append, const int32_t* seq_len,
                            const int32_t* k, int B, float sm_scale, void* out, float* out_f32, hipStream_t s,
                            int chunk, const PageView* pages = nullptr, int b0 = 0, int32_t* idx_only = nullptr);
// (chunk: keys per workgroup, one of the context's coop_opt_chunk; idx_only != nullptr: the launch
// stops once the index lists are written, into idx_only [B, Hkv, k_max] instead of the workspace;
// V, out and out_f32 are not touched)
int coop_capacity(const hata_ctx* c, bool paged, int chunk);

}  // namespace hata
