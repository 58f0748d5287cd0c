// C-ABI entry points of libhata: argument validation, workspace carving, launch-shape
// selection and the stage sequence of one decode step (Alg. 3 of the paper).
#include <mutex>
#include <new>
#include <string.h>

#include "hata_internal.h"
#include "hata_trace.h"

#ifdef HATA_TRACE
__device__ unsigned long long g_hata_trace[HATA_TRACE_WGS * 32];
// host_out: HATA_TRACE_WGS * 32 words (host)
extern "C" int hata_debug_trace(unsigned long long* host_out) {
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_hata_trace), sizeof(unsigned long long) * HATA_TRACE_WGS * 32);
}
extern "C" int hata_debug_trace_reset(void) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_hata_trace)) != hipSuccess) return -1;
    return (int)hipMemset(p, 0, sizeof(unsigned long long) * HATA_TRACE_WGS * 32);
}
#endif

// Scratch of hata_sparse_decode_static(): attention partials and their arrival counters for callers
// that cannot hand over a workspace.  One copy per device the library runs on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress(); kernels are
// given the per-device address looked up below.
#define HATA_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[HATA_STATIC_SCRATCH_BYTES];

// fills n words with zero (used instead of a memset node so that the call may be captured in a graph)
__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t* p, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0u;
}

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxDevices = 64;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
    int G, Wd, NB, NBP, chunk, n_chunks, coop_chunk, HT, sparse_rows, sparse_splits, dense_rows, dense_splits;
    size_t off_qcodes, off_scores, off_idx, off_hist, off_cinfo, off_uinfo, off_ucnt, off_acnt, off_uflag, off_qrec, off_err, off_uhist, off_partials, off_wplanes, total;
};

int validate_config(const hata_config* f) {
    if (!f) return HATA_EINVAL;
    if (f->B_max < 1 || f->Hq < 1 || f->Hkv < 1 || f->L_cap < 1 || f->k_max < 1) return HATA_EINVAL;
    if (f->Hq % f->Hkv != 0) return HATA_EINVAL;
    if (f->k_max > f->L_cap) return HATA_EINVAL;
    if (f->r < 32 || f->r % 32 != 0) return HATA_EINVAL;
    if (f->kv_stride_n < f->d || f->kv_stride_n % 8 != 0 || f->kv_stride_h % 8 != 0 ||
        f->kv_stride_b % 8 != 0 || f->kv_stride_h < 0 || f->kv_stride_b < 0)
        return HATA_EINVAL;
    if (f->d != 128) return HATA_EUNSUPPORTED;
    if (f->r > 256) return HATA_EUNSUPPORTED;
    const int G = f->Hq / f->Hkv;
    if (G > 16 || (int64_t)G * f->r > 4096) return HATA_EUNSUPPORTED;
    if ((int64_t)f->B_max * f->Hkv > 65535 || f->B_max > 65535) return HATA_EUNSUPPORTED;
    return HATA_OK;
}

// Launch shapes.
int make_plan(const hata_config* f, const hata_tuning* t, Plan* p) {
    int rc = validate_config(f);
    if (rc != HATA_OK) return rc;
    p->G = f->Hq / f->Hkv;
    p->Wd = f->r / 32;
    p->NB = p->G * f->r + 1;
    p->NBP = (p->NB + 7) / 8 * 8;
    const int64_t units = (int64_t)f->B_max * f->Hkv;
    // chunks of at most 4096 keys (larger only if the cache is so long that a unit would otherwise
    // exceed 1024 chunks), halved while that keeps the grid within two workgroups per CU: measured
    // with the single-launch step, more and smaller chunks win until then (cfg 2: 20.5 / 17.3 /
    // 16.9 us at 4096 / 2048 / 1024 keys), and a grid that size is resident for every kernel variant
    const int64_t max_wgs = 512;
    int chunk = 4096;
    while (chunk > 1024 && units * ((f->L_cap + chunk / 2 - 1) / (chunk / 2)) <= max_wgs) chunk >>= 1;
    while (chunk < 8192 && (f->L_cap + chunk - 1) / chunk > 1024) chunk <<= 1;
    // the single-launch step can give a workgroup more keys than the other kernels' chunk (its scores
    // stay in LDS, up to 32768 of them): fewer workgroups per unit, fewer exchanges between them
    int coop_chunk = 0;
    if (t && t->chunk != 0) {  // the caller's choice (launch-shape sweeps, tests of the batch slicing)
        const int v = t->chunk;
        if (v == 16384 || v == 32768) {
            coop_chunk = v;  // the single-launch step only; the other kernels keep the choice made above
        } else {
            if (!(v == 1024 || v == 2048 || v == 4096 || v == 8192) || (f->L_cap + v - 1) / v > 1024) return HATA_EINVAL;
            chunk = v;
        }
    }
    p->chunk = chunk;
    p->n_chunks = (f->L_cap + chunk - 1) / chunk;
    if (p->n_chunks > 1024) return HATA_EUNSUPPORTED;  // L_cap above 8M rows
    p->coop_chunk = (t && t->chunk != 0) ? (coop_chunk > chunk ? coop_chunk : chunk) : 0;  // 0: chosen per call
    const int G = p->G;
    // (16 heads as two tiles of 8: measured faster than one tile of 16 for the stand-alone kernels)
    p->HT = (G % 8 == 0) ? 8 : (G % 5 == 0) ? 5 : (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1;
    const int64_t attn_units = units * (G / p->HT);
    // selected rows per attention workgroup: halved from 256 towards 512 workgroups, but not below 64
    // (measured with hata_sparse_decode alone: at B = 1 slices of 16-32 rows cost more in partials and
    // merge than they gain in parallelism -- cfg 2 10.0 us at 16 rows, 8.0 at 64; cfg 4 18.7 at 32, 10.8 at 64)
    int rows = 256;
    while (rows > 64 && attn_units * ((f->k_max + rows - 1) / rows) < 512) rows >>= 1;
    if (t && t->attn_rows != 0) {
        const int v = t->attn_rows;
        if (v < 16 || v > 256 || (v & (v - 1)) != 0) return HATA_EINVAL;
        rows = v;
    }
    while (rows < 256 && (f->k_max + rows - 1) / rows > 256) rows <<= 1;
    p->sparse_rows = rows;
    p->sparse_splits = (f->k_max + rows - 1) / rows;
    if (p->sparse_splits > 256) return HATA_EUNSUPPORTED;  // budget above 65536 rows
    int drows = 4096;
    // (measured: with few units, 512 workgroups -- more slices make the last workgroup's merge the
    // long pole, 39 -> 53 us at B = 1, L = 32K; with 32 units and more, 1024: 240 -> 209 us at B = 4, G = 8, L = 64K)
    const int64_t dense_wgs = attn_units >= 32 ? 1024 : 512;
    while (drows > 512 && attn_units * ((f->L_cap + drows - 1) / drows) < dense_wgs) drows >>= 1;
    while ((f->L_cap + drows - 1) / drows > 256) drows <<= 1;  // the merge handles <= 256 slices
    p->dense_rows = drows;
    p->dense_splits = (f->L_cap + drows - 1) / drows;
    int max_splits = p->sparse_splits > p->dense_splits ? p->sparse_splits : p->dense_splits;
    if (p->n_chunks > max_splits) max_splits = p->n_chunks;  // the cooperative step: one slice per chunk

    size_t o = 0;
    p->off_qcodes = o;   o = align_up(o + (size_t)f->B_max * f->Hq * p->Wd * 4);
    p->off_scores = o;   o = align_up(o + (size_t)units * f->L_cap * 2);
    p->off_idx = o;      o = align_up(o + (size_t)units * f->k_max * 4);
    p->off_hist = o;     o = align_up(o + (size_t)units * p->n_chunks * p->NBP * 2);
    p->off_cinfo = o;    o = align_up(o + (size_t)units * (p->n_chunks + 1) * 2 * 4);
    p->off_uinfo = o;    o = align_up(o + (size_t)units * 2 * 4);
    // (the single-launch step keeps each unit's two arrival counters on a cache line of their own)
    p->off_ucnt = o;     o = align_up(o + (size_t)units * HATA_COUNTER_STRIDE * 4);
    p->off_acnt = o;     o = align_up(o + (size_t)f->B_max * f->Hq * HATA_COUNTER_STRIDE * 4);
    p->off_uflag = o;    o = align_up(o + (size_t)units * p->n_chunks * HATA_REC_STRIDE * 8);
    p->off_qrec = o;     o = align_up(o + (size_t)f->B_max * f->Hq * p->Wd * p->n_chunks * 8);
    p->off_err = o;      o = align_up(o + 4);
    p->off_uhist = o;    o = align_up(o + (size_t)units * p->NB * 4);
    p->off_partials = o; o = align_up(o + (size_t)f->B_max * f->Hq * max_splits * (128 + 2) * 4);
    p->off_wplanes = o;  o = align_up(o + (size_t)f->Hkv * 2 * 128 * f->r * 2);  // two fp16 planes
    p->total = o;
    return HATA_OK;
}

inline bool f_has_mfma_width(int r) { return r == 32 || r == 64 || r == 128 || r == 256; }

inline int check_call(const hata_ctx* c, int B) {
    if (!c) return HATA_EINVAL;
    if (B < 1 || B > c->cfg.B_max) return HATA_EINVAL;
    return HATA_OK;
}
// the cooperative kernel needs its whole grid resident (its workgroups wait for one another) and
// merges at most 256 attention partials per unit
// Single-launch form of the step: the number of launches a batch of B sequences is cut into -- every
// launch must be resident as a whole, so a batch with more (sequence, KV head) units than that
// allows goes in equal slices, one launch each -- or 0 when the form is not available.
inline int coop_sub_batches(const hata_ctx* c, int B, bool paged, int* chunk_out = nullptr) {
    if (c->step_mode == 3) return 0;
    // the oversubscribed grid of mode 1 uses the first size only
    const int n_opts = c->step_mode == 1 ? 1 : c->coop_opts;
    int best = 0, best_chunk = 0;
    for (int o = 0; o < n_opts; ++o) {
        const int chunk = c->coop_opt_chunk[o];
        const int n_chunks = (c->cfg.L_cap + chunk - 1) / chunk;
        const int cap = paged ? c->coop_opt_cap_paged[o] : c->coop_opt_cap[o];
        const int64_t per_seq = (int64_t)n_chunks * c->cfg.Hkv;
        if (n_chunks > 256 || cap <= 0 || per_seq > cap) continue;
        int ns;
        // mode 1: the whole batch in one grid, whatever its size, if the workgroups of the units that
        // are at work together -- eight units interleaved when their number is a multiple of eight,
        // else one -- fit the device at once; otherwise in slices, as in mode 0
        if (c->step_mode == 1 && ((int64_t)B * c->cfg.Hkv % 8 == 0 ? 8 : 1) * (int64_t)n_chunks <= cap) {
            ns = 1;
        } else {
            const int per_launch = (int)(cap / per_seq);
            ns = (B + per_launch - 1) / per_launch;
        }
        if (best == 0 || ns < best) { best = ns; best_chunk = chunk; }
    }
    if (chunk_out) *chunk_out = best_chunk;
    return best;
}
inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Validates a block-table description and fills the view the launchers take.
inline int make_page_view(const hata_ctx* c, const int32_t* block_table, int32_t max_blocks,
                          int32_t page_rows, int32_t n_pages, hata::PageView* pv) {
    if (!block_table || max_blocks < 1 || n_pages < 1) return HATA_EINVAL;
    if (page_rows < 16 || page_rows > (1 << 20) || (page_rows & (page_rows - 1)) != 0) return HATA_EINVAL;
    if ((int64_t)max_blocks * page_rows > (1ll << 30)) return HATA_EINVAL;
    // rows of the pools are indexed with 32-bit integers on the device
    if ((int64_t)n_pages * c->cfg.Hkv * page_rows > 0x7fffffffll) return HATA_EINVAL;
    int shift = 0;
    while ((1 << shift) < page_rows) ++shift;
    pv->table = block_table; pv->max_blocks = max_blocks; pv->shift = shift; pv->n_pages = n_pages;
    return HATA_OK;
}
inline int hip_rc(hipError_t e) { return e == hipSuccess ? HATA_OK : HATA_EHIP; }

}  // namespace

extern "C" {

const char* hata_strerror(int status) {
    switch (status) {
        case HATA_OK: return "ok";
        case HATA_EINVAL: return "invalid argument";
        case HATA_EUNSUPPORTED: return "unsupported shape";
        case HATA_EWORKSPACE: return "workspace missing, misaligned or too small";
        case HATA_EHIP: return "HIP runtime error";
        case HATA_ETIMEOUT: return "a single-launch decode step gave up an in-kernel wait";
        case HATA_ETOOLARGE: return "shape needs more scratch than the static buffer of the allocation-free entry point holds";
        default: return "unknown status";
    }
}

int hata_workspace_bytes_tuned(const hata_config* cfg, const hata_tuning* tuning, size_t* out) {
    if (!out) return HATA_EINVAL;
    Plan p;
    int rc = make_plan(cfg, tuning, &p);
    if (rc != HATA_OK) return rc;
    *out = p.total;
    return HATA_OK;
}

int hata_workspace_bytes(const hata_config* cfg, size_t* out) { return hata_workspace_bytes_tuned(cfg, nullptr, out); }

int hata_create_tuned(hata_ctx** ctx_out, const hata_config* cfg, const hata_tuning* tuning, void* workspace,
                      size_t workspace_bytes) {
    if (!ctx_out) return HATA_EINVAL;
    *ctx_out = nullptr;
    if (tuning && (tuning->par_merge < -1 || tuning->par_merge > 1)) return HATA_EINVAL;
    Plan p;
    int rc = make_plan(cfg, tuning, &p);
    if (rc != HATA_OK) return rc;
    if (!workspace || !aligned(workspace, kAlign) || workspace_bytes < p.total) return HATA_EWORKSPACE;
    hata_ctx* c = new (std::nothrow) hata_ctx;
    if (!c) return HATA_EINVAL;
    c->cfg = *cfg;
    c->G = p.G; c->Wd = p.Wd; c->NB = p.NB; c->NBP = p.NBP;
    c->chunk = p.chunk; c->n_chunks = p.n_chunks; c->HT = p.HT;
    c->sparse_rows = p.sparse_rows; c->sparse_splits = p.sparse_splits;
    c->dense_rows = p.dense_rows; c->dense_splits = p.dense_splits;
    char* w = (char*)workspace;
    c->qcodes = (uint32_t*)(w + p.off_qcodes);
    c->scores = (uint16_t*)(w + p.off_scores);
    c->idx = (int32_t*)(w + p.off_idx);
    c->chunk_hist = (uint16_t*)(w + p.off_hist);
    c->chunk_info = (int32_t*)(w + p.off_cinfo);
    c->unit_info = (int32_t*)(w + p.off_uinfo);
    c->unit_counter = (uint32_t*)(w + p.off_ucnt);
    c->attn_counter = (uint32_t*)(w + p.off_acnt);
    c->unit_hist = (uint32_t*)(w + p.off_uhist);
    c->coop_rec = (unsigned long long*)(w + p.off_uflag);
    c->coop_qrec = (unsigned long long*)(w + p.off_qrec);
    c->error_word = (uint32_t*)(w + p.off_err);
    c->epoch = 0;
    c->coop_opts = 0;
    c->partials = (float*)(w + p.off_partials);
    c->wplanes = (f_has_mfma_width(cfg->r)) ? (void*)(w + p.off_wplanes) : nullptr;
    c->prepared_W_H = nullptr;
    c->control_bytes = p.off_partials - p.off_cinfo;
    // control words and the self-resetting arrival counters start from zero
    if (hipMemset(c->chunk_info, 0, c->control_bytes) != hipSuccess) {
        delete c;
        return HATA_EHIP;
    }
    // the device's size is looked up once, here: no launch queries the runtime
    int dev = 0;
    c->cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&c->cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        c->cus = 0;
    // Chunk sizes of the single-launch step.  The caller's, if one was given; else the plan's and,
    // for batches too large to be resident at that size, up to three larger ones: with 16384 keys
    // per workgroup B = 32 at L = 32K is ONE resident launch of 512 workgroups instead of two of 1024
    // (measured 58 against 75 us), while small batches are fastest at the plan's size.
    if (p.coop_chunk) {
        c->coop_opts = 1;
        c->coop_opt_chunk[0] = p.coop_chunk;
    } else {
        c->coop_opt_chunk[c->coop_opts++] = p.chunk;
        for (int v = 8192; v <= 32768 && c->coop_opts < 4; v <<= 1)
            if (v > p.chunk && v < 2 * cfg->L_cap) c->coop_opt_chunk[c->coop_opts++] = v;
    }
    for (int o = 0; o < c->coop_opts; ++o) {
        c->coop_opt_cap[o] = hata::coop_capacity(c, false, c->coop_opt_chunk[o]);
        c->coop_opt_cap_paged[o] = hata::coop_capacity(c, true, c->coop_opt_chunk[o]);
    }
    // a device shared with other work cannot promise that a whole grid is resident: three launches
    c->step_mode = (tuning && tuning->shared_device) ? 3 : 0;
    c->spin_limit = 0;
    c->keep_scores = 0;
    // with more than one query head per KV head the merge is spread over the unit's workgroups,
    // a head each (measured: never slower, 1-5 us faster with many slices or heads; with one head
    // the last arriver merging alone is 0.6 us faster)
    c->par_merge = c->G >= 2 ? 1 : 0;
    if (tuning && tuning->par_merge >= 0) c->par_merge = tuning->par_merge;
    *ctx_out = c;
    return HATA_OK;
}

int hata_create(hata_ctx** ctx_out, const hata_config* cfg, void* workspace, size_t workspace_bytes) {
    return hata_create_tuned(ctx_out, cfg, nullptr, workspace, workspace_bytes);
}

int hata_destroy(hata_ctx* ctx) {
    delete ctx;
    return HATA_OK;
}

int hata_encode_keys(hata_ctx* ctx, const void* K, const float* W_H, const int32_t* start,
                     const int32_t* n_new, int32_t B, int32_t max_new, uint32_t* codes,
                     void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!K || !W_H || !start || !n_new || !codes) return HATA_EINVAL;
    if (max_new < 0 || max_new > ctx->cfg.L_cap) return HATA_EINVAL;
    if (!aligned(K, 16) || !aligned(codes, 16) || !aligned(W_H, 16)) return HATA_EINVAL;
    if (max_new == 0) return HATA_OK;
    hipStream_t s = (hipStream_t)stream;
    if (max_new <= 8)
        return hip_rc(hata::launch_encode_vectors(ctx, nullptr, nullptr, K, start, n_new, max_new,
                                                  0, codes, W_H, B, s));
    return hip_rc(hata::launch_encode_bulk(ctx, K, W_H, start, n_new, B, max_new, codes, s));
}

int hata_prepare_weights(hata_ctx* ctx, const float* W_H, void* stream) {
    if (!ctx) return HATA_EINVAL;
    if (!W_H) {  // forget the prepared tensor
        ctx->prepared_W_H = nullptr;
        return HATA_OK;
    }
    if (!aligned(W_H, 16)) return HATA_EINVAL;
    if (!ctx->wplanes) return HATA_OK;  // widths without a matrix-core kernel have nothing to prepare
    if (hata::launch_split_weights(ctx, W_H, (hipStream_t)stream) != hipSuccess) return HATA_EHIP;
    ctx->prepared_W_H = W_H;
    return HATA_OK;
}

int hata_prefill_write(hata_ctx* ctx, const void* K_new, const void* V_new, const int32_t* start,
                       const int32_t* n_new, int32_t B, int32_t max_new, void* K, void* V,
                       uint32_t* codes, const float* W_H, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!K_new || !V_new || !start || !n_new || !K || !V || !codes || !W_H) return HATA_EINVAL;
    if (max_new < 0 || max_new > ctx->cfg.L_cap) return HATA_EINVAL;
    if (!aligned(K_new, 16) || !aligned(V_new, 16) || !aligned(K, 16) || !aligned(V, 16) ||
        !aligned(codes, 16) || !aligned(W_H, 16))
        return HATA_EINVAL;
    const int r = ctx->cfg.r;
    if (r != 32 && r != 64 && r != 128 && r != 256) return HATA_EUNSUPPORTED;
    if (max_new == 0) return HATA_OK;
    return hip_rc(hata::launch_encode_bulk(ctx, K, W_H, start, n_new, B, max_new, codes,
                                           (hipStream_t)stream, K_new, V_new, K, V));
}

int hata_prefill_write_paged(hata_ctx* ctx, const void* K_new, const void* V_new, const int32_t* start,
                             const int32_t* n_new, int32_t B, int32_t max_new, void* K_pool, void* V_pool,
                             uint32_t* codes_pool, const int32_t* block_table, int32_t max_blocks,
                             int32_t page_rows, int32_t n_pages, const float* W_H, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!K_new || !V_new || !start || !n_new || !K_pool || !V_pool || !codes_pool || !W_H) return HATA_EINVAL;
    if (max_new < 0 || max_new > ctx->cfg.L_cap) return HATA_EINVAL;
    if (!aligned(K_new, 16) || !aligned(V_new, 16) || !aligned(K_pool, 16) || !aligned(V_pool, 16) ||
        !aligned(codes_pool, 16) || !aligned(W_H, 16) || !aligned(block_table, 4))
        return HATA_EINVAL;
    hata::PageView pv;
    rc = make_page_view(ctx, block_table, max_blocks, page_rows, n_pages, &pv);
    if (rc != HATA_OK) return rc;
    const int r = ctx->cfg.r;
    if (r != 32 && r != 64 && r != 128 && r != 256) return HATA_EUNSUPPORTED;
    if (max_new == 0) return HATA_OK;
    return hip_rc(hata::launch_encode_bulk(ctx, K_pool, W_H, start, n_new, B, max_new, codes_pool,
                                           (hipStream_t)stream, K_new, V_new, K_pool, V_pool, &pv));
}

int hata_encode_query(hata_ctx* ctx, const void* q, const float* W_H, int32_t B, uint32_t* qcodes,
                      void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!q || !W_H || !qcodes) return HATA_EINVAL;
    if (!aligned(q, 16) || !aligned(qcodes, 4) || !aligned(W_H, 16)) return HATA_EINVAL;
    return hip_rc(hata::launch_encode_vectors(ctx, q, qcodes, nullptr, nullptr, nullptr, 0, 0,
                                              nullptr, W_H, B, (hipStream_t)stream));
}

int hata_hamming_score(hata_ctx* ctx, const uint32_t* qcodes, const uint32_t* codes,
                       const int32_t* seq_len, int32_t B, uint16_t* scores, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!qcodes || !codes || !seq_len || !scores) return HATA_EINVAL;
    if (!aligned(qcodes, 4) || !aligned(codes, 16) || !aligned(scores, 2)) return HATA_EINVAL;
    // the chunk histograms are written too (into the workspace), as in the fused decode step
    return hip_rc(hata::launch_score(ctx, qcodes, codes, seq_len, B, scores, nullptr,
                                     (hipStream_t)stream));
}

int hata_topk(hata_ctx* ctx, const uint16_t* scores, const int32_t* seq_len, const int32_t* k,
              int32_t B, int32_t* idx, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!scores || !seq_len || !k || !idx) return HATA_EINVAL;
    if (!aligned(scores, 2) || !aligned(idx, 4)) return HATA_EINVAL;
    return hip_rc(hata::launch_topk(ctx, scores, seq_len, k, B, idx, (hipStream_t)stream));
}

int hata_sparse_decode(hata_ctx* ctx, const void* q, const void* K, const void* V,
                       const int32_t* idx, const int32_t* k, int32_t B, float sm_scale, void* out,
                       float* out_f32, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!q || !K || !V || !idx || !k || !out) return HATA_EINVAL;
    if (!aligned(q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 2)) return HATA_EINVAL;
    return hip_rc(hata::launch_attention(ctx, 0, q, K, V, const_cast<int32_t*>(idx), k, nullptr, B,
                                         sm_scale, out, out_f32, (hipStream_t)stream));
}

int hata_gather_rows(hata_ctx* ctx, const void* K, const void* V, const int32_t* idx, const int32_t* k,
                     int32_t B, int32_t max_workgroups, void* K_stage, void* V_stage, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!K || !V || !idx || !k || !K_stage || !V_stage || max_workgroups < 0) return HATA_EINVAL;
    if (!aligned(K, 16) || !aligned(V, 16) || !aligned(K_stage, 16) || !aligned(V_stage, 16) || !aligned(idx, 4))
        return HATA_EINVAL;
    return hip_rc(hata::launch_gather_rows(ctx, K, V, idx, k, B, max_workgroups, K_stage, V_stage, (hipStream_t)stream));
}

int hata_dense_decode(hata_ctx* ctx, const void* q, const void* K, const void* V,
                      const int32_t* seq_len, int32_t B, float sm_scale, void* out, float* out_f32,
                      void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!q || !K || !V || !seq_len || !out) return HATA_EINVAL;
    if (!aligned(q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 2)) return HATA_EINVAL;
    return hip_rc(hata::launch_attention(ctx, 1, q, K, V, nullptr, seq_len, seq_len, B, sm_scale,
                                         out, out_f32, (hipStream_t)stream));
}

int hata_sparse_decode_static(const hata_config* cfg, const void* q, const void* K, const void* V,
                              const int32_t* idx, const int32_t* k, int32_t B, float sm_scale, void* out,
                              float* out_f32, void* stream) {
    Plan p;
    int rc = make_plan(cfg, nullptr, &p);
    if (rc != HATA_OK) return rc;
    if (B < 1 || B > cfg->B_max) return HATA_EINVAL;
    if (!q || !K || !V || !idx || !k || !out) return HATA_EINVAL;
    if (!aligned(q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 2)) return HATA_EINVAL;
    // layout inside the scratch: [arrival counters of B_max * Hq head tiles][partials]
    const size_t counter_bytes = align_up((size_t)cfg->B_max * cfg->Hq * 4);
    const size_t partial_bytes = (size_t)cfg->B_max * cfg->Hq * p.sparse_splits * (128 + 2) * 4;
    if (counter_bytes + partial_bytes > HATA_STATIC_SCRATCH_BYTES) return HATA_ETOOLARGE;
    // the device copy of `scratch` that belongs to the current device, looked up once per device
    static std::mutex mu;
    static void* dev_ptr[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HATA_EHIP;
    void* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!dev_ptr[dev]) {
            void* sym = nullptr;
            if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return HATA_EHIP;
            dev_ptr[dev] = sym;
        }
        base = dev_ptr[dev];
    }
    hata_ctx c = {};
    c.cfg = *cfg;
    c.G = p.G; c.Wd = p.Wd; c.NB = p.NB; c.NBP = p.NBP; c.chunk = p.chunk; c.n_chunks = p.n_chunks; c.HT = p.HT;
    c.sparse_rows = p.sparse_rows; c.sparse_splits = p.sparse_splits;
    c.dense_rows = p.dense_rows; c.dense_splits = p.dense_splits;
    c.attn_counter = (uint32_t*)base;
    c.partials = (float*)((char*)base + counter_bytes);
    hipStream_t s = (hipStream_t)stream;
    // the counters must start at zero whatever an earlier call left behind
    const int n_cnt = cfg->B_max * cfg->Hq;
    hipLaunchKernelGGL(zero_words_kernel, dim3((n_cnt + 255) / 256), dim3(256), 0, s, c.attn_counter, n_cnt);
    if (hipGetLastError() != hipSuccess) return HATA_EHIP;
    return hip_rc(hata::launch_attention(&c, 0, q, K, V, const_cast<int32_t*>(idx), k, nullptr, B, sm_scale, out,
                                         out_f32, s));
}

int hata_decode_step(hata_ctx* ctx, const void* q, const void* K, const void* V, const float* W_H,
                     uint32_t* codes, const int32_t* seq_len, const int32_t* k, int32_t B,
                     int32_t append, float sm_scale, void* out, float* out_f32, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!q || !K || !V || !W_H || !codes || !seq_len || !k || !out) return HATA_EINVAL;
    if (!aligned(q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(codes, 16) ||
        !aligned(W_H, 16) || !aligned(out, 2))
        return HATA_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    // Cooperative path: encoding, scoring, selection and attention in ONE launch (workgroups of a
    // unit wait for the unit's threshold inside the kernel), when every workgroup can be resident
    // at once.
    int step_chunk = 0;
    if (const int ns = coop_sub_batches(ctx, B, false, &step_chunk)) {
        hipError_t e = hipSuccess;
        for (int i = 0; i < ns && e == hipSuccess; ++i) {
            const int b0 = (int)((int64_t)i * B / ns), b1 = (int)((int64_t)(i + 1) * B / ns);
            e = hata::launch_coop_step(ctx, q, K, V, W_H, codes, append, seq_len, k, b1 - b0, sm_scale, out,
                                       out_f32, s, step_chunk, nullptr, b0);
        }
        if (e == hipSuccess) return HATA_OK;
        if (e != hipErrorNotSupported) return HATA_EHIP;  // (not supported: no kernel for this shape, nothing was launched)
    }
    // Alg. 3: HashEncode(Q), HashEncode(K_new) and the code-cache update, in one launch
    hipError_t e = hata::launch_encode_vectors(ctx, q, ctx->qcodes, append ? K : nullptr, seq_len,
                                               nullptr, 1, 1, codes, W_H, B, s);
    if (e != hipSuccess) return HATA_EHIP;
    // Three-launch path.  Hamming distances of every cached code (the new one included), chunk
    // histograms, and -- by the last workgroup of each unit -- the selection threshold and offsets
    e = hata::launch_score(ctx, ctx->qcodes, codes, seq_len, B, ctx->scores, k, s);
    if (e != hipSuccess) return HATA_EHIP;
    // TopK(S, N) compaction fused with the attention over the selected rows (gather fused too)
    e = hata::launch_attention(ctx, 2, q, K, V, ctx->idx, k, seq_len, B, sm_scale, out, out_f32, s);
    return hip_rc(e);
}

int hata_select_step(hata_ctx* ctx, const void* q, const void* K, const float* W_H, uint32_t* codes,
                     const int32_t* seq_len, const int32_t* k, int32_t B, int32_t append, int32_t* idx,
                     void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!q || !W_H || !codes || !seq_len || !k || !idx || (append && !K)) return HATA_EINVAL;
    if (!aligned(q, 16) || !aligned(K, 16) || !aligned(codes, 16) || !aligned(W_H, 16) || !aligned(idx, 4))
        return HATA_EINVAL;
    int step_chunk = 0;
    const int ns = coop_sub_batches(ctx, B, false, &step_chunk);
    if (ns == 0) return HATA_EUNSUPPORTED;
    hipError_t e = hipSuccess;
    for (int i = 0; i < ns && e == hipSuccess; ++i) {
        const int b0 = (int)((int64_t)i * B / ns), b1 = (int)((int64_t)(i + 1) * B / ns);
        e = hata::launch_coop_step(ctx, q, K, nullptr, W_H, codes, append, seq_len, k, b1 - b0, 0.f, nullptr,
                                   nullptr, (hipStream_t)stream, step_chunk, nullptr, b0, idx);
    }
    if (e == hipErrorNotSupported) return HATA_EUNSUPPORTED;
    return hip_rc(e);
}

int hata_decode_step_paged(hata_ctx* ctx, const void* q, const void* K_pool, const void* V_pool,
                           const float* W_H, uint32_t* codes_pool, const int32_t* block_table,
                           int32_t max_blocks, int32_t page_rows, int32_t n_pages,
                           const int32_t* seq_len, const int32_t* k, int32_t B, int32_t append,
                           float sm_scale, void* out, float* out_f32, void* stream) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!q || !K_pool || !V_pool || !W_H || !codes_pool || !seq_len || !k || !out) return HATA_EINVAL;
    if (!aligned(q, 16) || !aligned(K_pool, 16) || !aligned(V_pool, 16) || !aligned(codes_pool, 16) ||
        !aligned(W_H, 16) || !aligned(out, 2) || !aligned(block_table, 4))
        return HATA_EINVAL;
    hata::PageView pv;
    rc = make_page_view(ctx, block_table, max_blocks, page_rows, n_pages, &pv);
    if (rc != HATA_OK) return rc;
    // the block table is read by the single-launch kernel only
    const int mode = ctx->step_mode;
    ctx->step_mode = 0;  // (hata_set_step_mode does not apply here)
    int step_chunk = 0;
    const int ns = coop_sub_batches(ctx, B, true, &step_chunk);
    ctx->step_mode = mode;
    if (ns == 0) return HATA_EUNSUPPORTED;
    hipError_t e = hipSuccess;
    for (int i = 0; i < ns && e == hipSuccess; ++i) {
        const int b0 = (int)((int64_t)i * B / ns), b1 = (int)((int64_t)(i + 1) * B / ns);
        e = hata::launch_coop_step(ctx, q, K_pool, V_pool, W_H, codes_pool, append, seq_len, k, b1 - b0, sm_scale,
                                   out, out_f32, (hipStream_t)stream, step_chunk, &pv, b0);
    }
    if (e == hipErrorNotSupported) return HATA_EUNSUPPORTED;
    return hip_rc(e);
}

int hata_step_plan(const hata_ctx* ctx, int32_t B, int32_t* n_launches, int32_t* chunk, int32_t* n_chunks) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    int step_chunk = 0;
    const bool single = coop_sub_batches(ctx, B, false, &step_chunk) != 0;
    if (!single) step_chunk = ctx->chunk;
    if (n_launches) *n_launches = single ? 1 : 3;
    if (chunk) *chunk = step_chunk;
    if (n_chunks) *n_chunks = (ctx->cfg.L_cap + step_chunk - 1) / step_chunk;
    return HATA_OK;
}

int hata_step_sub_batches(const hata_ctx* ctx, int32_t B, int32_t* n_sub) {
    int rc = check_call(ctx, B);
    if (rc != HATA_OK) return rc;
    if (!n_sub) return HATA_EINVAL;
    *n_sub = coop_sub_batches(ctx, B, false);
    return HATA_OK;
}

int hata_set_step_mode(hata_ctx* ctx, int32_t mode) {
    if (!ctx || (mode != 0 && mode != 1 && mode != 3)) return HATA_EINVAL;
    ctx->step_mode = mode;
    return HATA_OK;
}

int hata_keep_step_scores(hata_ctx* ctx, int32_t keep) {
    if (!ctx) return HATA_EINVAL;
    ctx->keep_scores = keep ? 1 : 0;
    return HATA_OK;
}

int hata_set_wait_limit(hata_ctx* ctx, int32_t polls) {
    if (!ctx || polls < 0) return HATA_EINVAL;
    ctx->spin_limit = polls;
    return HATA_OK;
}

int hata_check(hata_ctx* ctx, void* stream) {
    if (!ctx) return HATA_EINVAL;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return HATA_EHIP;
    uint32_t w = 0;
    if (hipMemcpy(&w, ctx->error_word, sizeof(w), hipMemcpyDeviceToHost) != hipSuccess) return HATA_EHIP;
    if (!w) return HATA_OK;
    // a step that gave up may have left counters and published words half-way: start clean again
    // (the stream is idle here)
    if (hipMemset(ctx->chunk_info, 0, ctx->control_bytes) != hipSuccess) return HATA_EHIP;
    return HATA_ETIMEOUT;
}

int hata_host_device_pointer(void* host, void** dev_out) {
    if (!host || !dev_out) return HATA_EINVAL;
    *dev_out = nullptr;
    void* d = nullptr;
    if (hipHostGetDevicePointer(&d, host, 0) != hipSuccess || !d) {
        (void)hipGetLastError();  // not pinned / not mapped: leave no sticky error behind
        return HATA_EINVAL;
    }
    *dev_out = d;
    return HATA_OK;
}

int hata_step_buffers(hata_ctx* ctx, uint32_t** qcodes, uint16_t** scores, int32_t** idx) {
    if (!ctx) return HATA_EINVAL;
    if (qcodes) *qcodes = ctx->qcodes;
    if (scores) *scores = ctx->scores;
    if (idx) *idx = ctx->idx;
    return HATA_OK;
}

}  // extern "C"
