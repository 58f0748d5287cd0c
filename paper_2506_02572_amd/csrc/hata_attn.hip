// Decode attention over a list of cache rows (Alg. 3 of the paper: Gather + Attention, with
// the gather fused into the attention kernel; Eq. 2 third line, scale of Eq. 1), and the
// dense variant over the whole cache (Eq. 1) that serves as the comparison baseline.
//
// One kernel template, three row sources:
//   ROWS_IDX     rows come from an index list in memory            (hata_sparse_decode)
//   ROWS_DENSE   rows 0 .. seq_len-1                               (hata_dense_decode)
//   ROWS_SELECT  rows are selected on the fly from the stored scores, the unit threshold and
//                the per-chunk offsets (ordered compaction of just the chunks that hold this
//                workgroup's slice of the index list); the index list is written as a
//                by-product                                         (hata_decode_step)
//
// Split over the rows: every workgroup handles a slice of a unit's rows for HT query heads of
// the group at once (each K/V row is read once for all of them), keeps an online-softmax
// state per wave, and writes one partial (max, sum, weighted V) per query head; the last
// workgroup of a (unit, head tile) to finish merges the partials and writes the output, so no
// separate merge launch is needed.  A row is 256 B = 16 lanes x 128-bit, so a wave reads
// four whole rows per load instruction.  bf16 inputs, fp32 softmax and accumulation.
#include "hata_device.h"
#include "hata_internal.h"
#include "hata_select.h"
#include "hata_attn_core.h"
#include "hata_trace.h"

namespace hata {

#define HATA_MAX_ROWS_PER_WG 256

enum { ROWS_IDX = 0, ROWS_DENSE = 1, ROWS_SELECT = 2 };

struct AttnArgs {
    const uint16_t* q;
    const uint16_t* K;
    const uint16_t* V;
    const int32_t* idx_in;      // ROWS_IDX
    int32_t* idx_out;           // ROWS_SELECT
    const int32_t* count_src;   // ROWS_IDX: k[B]; ROWS_DENSE: seq_len[B]
    const uint16_t* scores;     // ROWS_SELECT ...
    const int32_t* seq_len;
    const int32_t* chunk_info;
    const int32_t* unit_info;
    int chunk, n_chunks;
    float* partials;
    uint32_t* counter;
    uint16_t* out;
    float* out_f32;
    int Hq, Hkv, G, L_cap, k_max, rows_per_wg, n_splits;
    int64_t sb, sh, sn;
    float scale_log2;
};

// grid = (splits, Hkv * (G / HT), B); 256 threads.
template <int HT, int MODE>
__global__ __launch_bounds__(256) void attn_kernel(const AttnArgs a) {
    constexpr bool MFMA = HT >= 4;  // matrix-core form of the attention core
    __shared__ __attribute__((aligned(16))) AttnLds<HT> S;
    __shared__ __attribute__((aligned(16))) uint16_t s_vt[MFMA ? HATA_VT_ELEMS : 8];
    __shared__ int s_rows[MODE == ROWS_SELECT ? HATA_MAX_ROWS_PER_WG : 1];
    __shared__ uint32_t scan4[4];
    __shared__ int s_clo, s_chi, s_last;
    const int tid = threadIdx.x;
    const int split = blockIdx.x;
    const int tiles = a.G / HT;
    const int h = blockIdx.y / tiles;
    const int ht = blockIdx.y % tiles;
    const int b = blockIdx.z;
    const int64_t u = (int64_t)b * a.Hkv + h;
    const int hq0 = h * a.G + ht * HT;
#define TA(i) HATA_TRACE_AT(i, MODE == ROWS_SELECT && u == 0 && ht == 0 && split == 0)
#define TL(i) HATA_TRACE_AT(i, MODE == ROWS_SELECT && u == 0 && ht == 0)
    TA(20);
    int count;
    if (MODE == ROWS_DENSE) count = clampi(a.count_src[b], 0, a.L_cap);
    else if (MODE == ROWS_IDX) count = clampi(a.count_src[b], 0, a.k_max);
    else count = clampi(a.unit_info[u * 2 + 1], 0, a.k_max);
    const int row_begin = split * a.rows_per_wg;
    uint16_t* outp = a.out + ((int64_t)b * a.Hq + hq0) * HATA_D;
    float* outp32 = a.out_f32 ? a.out_f32 + ((int64_t)b * a.Hq + hq0) * HATA_D : nullptr;
    if (MODE == ROWS_SELECT && ht == 0) {
        // slots of the index list past the selected count hold -1
        const int p0 = max(count, row_begin), p1 = min(row_begin + a.rows_per_wg, a.k_max);
        for (int p = p0 + tid; p < p1; p += 256) a.idx_out[u * a.k_max + p] = -1;
    }
    if (row_begin >= count) {
        if (count == 0 && split == 0) {  // no row at all: the output is zero
            for (int i = tid; i < HT * HATA_D; i += 256) {
                outp[i] = 0;
                if (outp32) outp32[i] = 0.f;
            }
        }
        return;
    }
    const int row_end = min(row_begin + a.rows_per_wg, count);
    const uint16_t* Kb = a.K + b * a.sb + h * a.sh;
    const uint16_t* Vb = a.V + b * a.sb + h * a.sh;
    const int32_t* ip = (MODE == ROWS_IDX) ? a.idx_in + u * a.k_max : nullptr;
    // query fragments first: nothing below depends on them until the rows are known
    uint32_t qr[MFMA ? 1 : HT][4];
    uint4 qb[4];
    if constexpr (MFMA) attn_load_q_mfma<HT>(a.q + ((int64_t)b * a.Hq + hq0) * HATA_D, qb);
    else attn_load_q<HT>(a.q + ((int64_t)b * a.Hq + hq0) * HATA_D, qr);

    if constexpr (MODE == ROWS_SELECT) {
        // ordered compaction of the chunks that hold positions [row_begin, row_end)
        const int L = clampi(a.seq_len[b], 0, a.L_cap);
        const int nc = (L + a.chunk - 1) / a.chunk;
        const int T = a.unit_info[u * 2 + 0];
        const int32_t* ci = a.chunk_info + u * (a.n_chunks + 1) * 2;
        TA(21);
        if (tid == 0) { s_clo = nc; s_chi = -1; }
        __syncthreads();
        for (int c = tid; c < nc; c += 256) {
            const int o0 = ci[2 * c], o1 = ci[2 * c + 2];
            if (o0 < row_end && o1 > row_begin) { atomicMin(&s_clo, c); atomicMax(&s_chi, c); }
        }
        __syncthreads();
        const int c_lo = s_clo, c_hi = s_chi;
        TA(22);
        const uint16_t* sp = a.scores + u * a.L_cap;
        int32_t* io = a.idx_out + u * a.k_max;
        for (int c = c_lo; c <= c_hi; ++c) {
            const int off = ci[2 * c], take = ci[2 * c + 1];
            if (ci[2 * c + 2] == off) continue;
            const int base = c * a.chunk;
            const int end = min(base + a.chunk, L);
            compact_chunk_any(a.chunk / 256, sp, base, end, T, off, take, scan4,
                              [&](int pos, int n) {
                                  if (pos >= row_begin && pos < row_end) {
                                      s_rows[pos - row_begin] = n;
                                      if (ht == 0) io[pos] = n;
                                  }
                              });
        }
        __syncthreads();
    }
    TA(23);
    auto row_of = [&](int row) {
        if (MODE == ROWS_DENSE) return row;
        if (MODE == ROWS_IDX) return (int)ip[row];
        return s_rows[row - row_begin];
    };
    if constexpr (MFMA)
        attn_rows_mfma<HT, (MODE == ROWS_DENSE ? 2 : 1), false>(qb, Kb, Vb, a.sn, a.L_cap, row_begin, row_end,
                                                         a.scale_log2, row_of, S, s_vt);
    else
        attn_rows<HT, 4>(qr, Kb, Vb, a.sn, a.L_cap, row_begin, row_end, a.scale_log2, row_of, S);
    TA(24);
    const int ns = (count + a.rows_per_wg - 1) / a.rows_per_wg;  // workgroups that contribute
    const int64_t head_stride = (int64_t)a.n_splits * HATA_PSTRIDE;
    float* part0 = a.partials + ((int64_t)b * a.Hq + hq0) * head_stride;
    attn_emit<HT>(S, ns == 1, outp, outp32, part0 + (int64_t)split * HATA_PSTRIDE, head_stride);
    if (ns == 1) return;
    // count the finished slices; the last workgroup merges them (partials are written with
    // write-through stores and read back with device-coherent loads)
    TA(25);
    wait_stores();
    __syncthreads();
    if (tid == 0) {
        uint32_t* cnt = a.counter + u * tiles + ht;
        const uint32_t done = atomicAdd(cnt, 1u);
        const int last = (done == (uint32_t)(ns - 1));
        if (last) *cnt = 0;
        s_last = last;
    }
    __syncthreads();
    TA(27);
    if (!s_last) return;
    TL(30);
    attn_merge<HT>(S, part0, head_stride, ns, outp, outp32);
    TL(31);
#undef TA
#undef TL
}

template <int HT>
static void launch_mode(int mode, const AttnArgs& a, dim3 grid, hipStream_t s) {
    switch (mode) {
        case ROWS_DENSE: hipLaunchKernelGGL((attn_kernel<HT, ROWS_DENSE>), grid, dim3(256), 0, s, a); break;
        case ROWS_SELECT: hipLaunchKernelGGL((attn_kernel<HT, ROWS_SELECT>), grid, dim3(256), 0, s, a); break;
        default: hipLaunchKernelGGL((attn_kernel<HT, ROWS_IDX>), grid, dim3(256), 0, s, a); break;
    }
}

// mode 0: rows from idx (count from k); 1: dense (count from seq_len); 2: select on the fly
// from the workspace's scores / thresholds (idx is written)
hipError_t launch_attention(const hata_ctx* c, int mode, const void* q, const void* K,
                            const void* V, int32_t* idx, const int32_t* count_src,
                            const int32_t* seq_len, int B, float sm_scale, void* out,
                            float* out_f32, hipStream_t s) {
    const hata_config& f = c->cfg;
    AttnArgs a;
    a.q = (const uint16_t*)q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V;
    a.idx_in = idx; a.idx_out = idx; a.count_src = count_src;
    a.scores = c->scores; a.seq_len = seq_len; a.chunk_info = c->chunk_info;
    a.unit_info = c->unit_info; a.chunk = c->chunk; a.n_chunks = c->n_chunks;
    a.partials = c->partials; a.counter = c->attn_counter;
    a.out = (uint16_t*)out; a.out_f32 = out_f32;
    a.Hq = f.Hq; a.Hkv = f.Hkv; a.G = c->G; a.L_cap = f.L_cap; a.k_max = f.k_max;
    const bool dense = (mode == ROWS_DENSE);
    a.rows_per_wg = dense ? c->dense_rows : c->sparse_rows;
    a.n_splits = dense ? c->dense_splits : c->sparse_splits;
    a.sb = f.kv_stride_b; a.sh = f.kv_stride_h; a.sn = f.kv_stride_n;
    a.scale_log2 = sm_scale * 1.4426950408889634f;
    switch (c->HT) {
        case 8: launch_mode<8>(mode, a, dim3(a.n_splits, f.Hkv * (c->G / 8), B), s); break;
        case 5: launch_mode<5>(mode, a, dim3(a.n_splits, f.Hkv * (c->G / 5), B), s); break;
        case 4: launch_mode<4>(mode, a, dim3(a.n_splits, f.Hkv * (c->G / 4), B), s); break;
        case 2: launch_mode<2>(mode, a, dim3(a.n_splits, f.Hkv * (c->G / 2), B), s); break;
        default: launch_mode<1>(mode, a, dim3(a.n_splits, f.Hkv * c->G, B), s); break;
    }
    return hipGetLastError();
}

}  // namespace hata
