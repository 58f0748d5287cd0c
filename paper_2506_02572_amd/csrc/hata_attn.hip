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
#include "hata_trace.h"

namespace hata {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

#define HATA_NEG_INF (-__builtin_huge_valf())
// 2^x for x <= 0 in one instruction (v_exp_f32, ~1 ulp; results below the normal range flush to 0,
// which is what a vanishing softmax weight should do; 2^-inf = 0)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// partial layout per (query head, split): [0] = running max (log2 domain), [1] = sum, [2..2+d) = acc
#define HATA_PSTRIDE (HATA_D + 2)
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

// grid = (splits, Hkv * (G / HT), B); 256 threads = 4 waves; lane = (row group rg = lane / 16,
// sub = lane % 16 -> elements [8 sub, 8 sub + 8) of a row).
template <int HT, int MODE>
__global__ __launch_bounds__(256) void attn_kernel(const AttnArgs a) {
    __shared__ float sm_m[4][HT];
    __shared__ float sm_l[4][HT];
    __shared__ float sm_acc[4][HT][HATA_D];
    __shared__ int s_rows[MODE == ROWS_SELECT ? HATA_MAX_ROWS_PER_WG : 1];
    __shared__ uint32_t scan4[4];
    __shared__ int s_clo, s_chi, s_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane & 15, rg = lane >> 4;
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
    if (MODE == ROWS_SELECT && ht == 0) {
        // slots of the index list past the selected count hold -1
        const int p0 = max(count, row_begin), p1 = min(row_begin + a.rows_per_wg, a.k_max);
        for (int p = p0 + tid; p < p1; p += 256) a.idx_out[u * a.k_max + p] = -1;
    }
    if (row_begin >= count) {
        if (count == 0 && split == 0) {  // no row at all: the output is zero
            for (int i = tid; i < HT * HATA_D; i += 256) {
                const int64_t o = ((int64_t)b * a.Hq + hq0) * HATA_D + i;
                a.out[o] = 0;
                if (a.out_f32) a.out_f32[o] = 0.f;
            }
        }
        return;
    }
    const int row_end = min(row_begin + a.rows_per_wg, count);
    const uint16_t* Kb = a.K + b * a.sb + h * a.sh;
    const uint16_t* Vb = a.V + b * a.sb + h * a.sh;
    const int32_t* ip = (MODE == ROWS_IDX) ? a.idx_in + u * a.k_max : nullptr;

    // this lane's 8 query elements of each head, kept as packed bf16 pairs (loaded
    // first: nothing below depends on them until the rows are known)
    uint32_t qr[HT][4];
#pragma unroll
    for (int g = 0; g < HT; ++g) {
        const uint4 v = *reinterpret_cast<const uint4*>(a.q + ((int64_t)b * a.Hq + hq0 + g) * HATA_D + sub * 8);
        qr[g][0] = v.x; qr[g][1] = v.y; qr[g][2] = v.z; qr[g][3] = v.w;
    }

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
    float m_run[HT], l_run[HT], acc[HT][8];
#pragma unroll
    for (int g = 0; g < HT; ++g) {
        m_run[g] = HATA_NEG_INF; l_run[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }

    constexpr int IT = 4;  // 4 iterations x 16 rows = 64 rows per tile
    for (int tile = row_begin; tile < row_end; tile += 16 * IT) {
        uint4 kv[IT], vv[IT];
        bool ok[IT];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int row = tile + it * 16 + wave * 4 + rg;
            ok[it] = row < row_end;
            int n = 0;
            if (ok[it]) {
                if (MODE == ROWS_DENSE) n = row;
                else if (MODE == ROWS_IDX) n = ip[row];
                else n = s_rows[row - row_begin];
            }
            ok[it] = ok[it] && n >= 0 && n < a.L_cap;
            kv[it] = make_uint4(0, 0, 0, 0);
            vv[it] = make_uint4(0, 0, 0, 0);
            if (ok[it]) {
                const int64_t o = (int64_t)n * a.sn + sub * 8;
                kv[it] = *reinterpret_cast<const uint4*>(Kb + o);
                vv[it] = *reinterpret_cast<const uint4*>(Vb + o);
            }
        }
        float s[IT][HT];
        float m_tile[HT];
#pragma unroll
        for (int g = 0; g < HT; ++g) m_tile[g] = HATA_NEG_INF;
#pragma unroll
        for (int it = 0; it < IT; ++it) {
#pragma unroll
            for (int g = 0; g < HT; ++g) {
                float d = dot2_bf16(qr[g][0], kv[it].x, 0.f);
                d = dot2_bf16(qr[g][1], kv[it].y, d);
                d = dot2_bf16(qr[g][2], kv[it].z, d);
                d = dot2_bf16(qr[g][3], kv[it].w, d);
                d = row_sum16(d);
                s[it][g] = ok[it] ? d * a.scale_log2 : HATA_NEG_INF;
                m_tile[g] = fmaxf(m_tile[g], s[it][g]);
            }
        }
#pragma unroll
        for (int g = 0; g < HT; ++g) {
            m_tile[g] = rows_max4(m_tile[g]);
            const float m_new = fmaxf(m_run[g], m_tile[g]);
            // m_new == -inf only while no valid row has been seen: keep the state untouched
            const float alpha = (m_new == HATA_NEG_INF) ? 1.f : fast_exp2(m_run[g] - m_new);
            l_run[g] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
            m_run[g] = m_new;
        }
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            float vf[8];
            vf[0] = bf16_lo(vv[it].x); vf[1] = bf16_hi(vv[it].x);
            vf[2] = bf16_lo(vv[it].y); vf[3] = bf16_hi(vv[it].y);
            vf[4] = bf16_lo(vv[it].z); vf[5] = bf16_hi(vv[it].z);
            vf[6] = bf16_lo(vv[it].w); vf[7] = bf16_hi(vv[it].w);
#pragma unroll
            for (int g = 0; g < HT; ++g) {
                const float p = ok[it] ? fast_exp2(s[it][g] - m_run[g]) : 0.f;
                l_run[g] += p;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
            }
        }
    }
    TA(24);
    // combine the four row groups of the wave (all share m_run)
#pragma unroll
    for (int g = 0; g < HT; ++g) {
        l_run[g] = rows_sum4(l_run[g]);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = rows_sum4(acc[g][e]);
    }
    if (rg == 0) {
#pragma unroll
        for (int g = 0; g < HT; ++g) {
            if (sub == 0) { sm_m[wave][g] = m_run[g]; sm_l[wave][g] = l_run[g]; }
#pragma unroll
            for (int e = 0; e < 8; ++e) sm_acc[wave][g][sub * 8 + e] = acc[g][e];
        }
    }
    __syncthreads();
    const int ns = (count + a.rows_per_wg - 1) / a.rows_per_wg;  // workgroups that contribute
    // combine the four waves: thread -> (head, channel)
    for (int i = tid; i < HT * HATA_D; i += 256) {
        const int g = i / HATA_D, ch = i % HATA_D;
        const float m0 = sm_m[0][g], m1 = sm_m[1][g], m2 = sm_m[2][g], m3 = sm_m[3][g];
        const float M = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
        float av = 0.f, l = 0.f;
        if (M != HATA_NEG_INF) {
            const float f0 = fast_exp2(m0 - M), f1 = fast_exp2(m1 - M), f2 = fast_exp2(m2 - M), f3 = fast_exp2(m3 - M);
            av = f0 * sm_acc[0][g][ch] + f1 * sm_acc[1][g][ch] + f2 * sm_acc[2][g][ch] + f3 * sm_acc[3][g][ch];
            l = f0 * sm_l[0][g] + f1 * sm_l[1][g] + f2 * sm_l[2][g] + f3 * sm_l[3][g];
        }
        if (ns == 1) {  // single slice: this is the result
            const float o = l > 0.f ? av / l : 0.f;
            const int64_t oo = ((int64_t)b * a.Hq + hq0 + g) * HATA_D + ch;
            a.out[oo] = (uint16_t)f32_to_bf16(o);
            if (a.out_f32) a.out_f32[oo] = o;
        } else {
            float* pp = a.partials + (((int64_t)b * a.Hq + hq0 + g) * a.n_splits + split) * HATA_PSTRIDE;
            st_dev(pp + 2 + ch, av);
            if (ch == 0) { st_dev(pp, M); st_dev(pp + 1, l); }
        }
    }
    if (ns == 1) return;
    // count the finished slices; the last workgroup merges them (partials are written with
    // write-through stores and read back with device-coherent loads)
    TA(25);
    wait_stores();
    TA(26);
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
    // Merge.  Every load of the merge is issued before the first wait: each thread pulls the
    // first 16 slices of its NO output channels into registers (later slices, ns > 16, batch by
    // batch), while one wave per head turns the (max, sum) pairs of the slices into normalised
    // weights w[g][s] = exp2(m_s - M) / sum_s' exp2(m_s' - M) l_s' in LDS.
    constexpr int NO = (HT * HATA_D + 255) / 256;  // outputs (head, channel) per thread
    float* sm_w = &sm_acc[0][0][0];                // [HT][nsp], nsp <= 256
    const int nsp = (ns + 3) & ~3;
    float av[NO][16];
#pragma unroll
    for (int r = 0; r < NO; ++r) {
        const int i = min(tid + 256 * r, HT * HATA_D - 1);
        const int g = i / HATA_D, ch = i % HATA_D;
        const float* pp = a.partials + ((int64_t)b * a.Hq + hq0 + g) * a.n_splits * HATA_PSTRIDE + 2 + ch;
#pragma unroll
        for (int j = 0; j < 16; ++j) av[r][j] = ld_dev(pp + (int64_t)min(j, ns - 1) * HATA_PSTRIDE);
    }
    for (int g = wave; g < HT; g += 4) {
        const float* pp = a.partials + ((int64_t)b * a.Hq + hq0 + g) * a.n_splits * HATA_PSTRIDE;
        float m_loc = HATA_NEG_INF;
        for (int s2 = lane; s2 < ns; s2 += 64) m_loc = fmaxf(m_loc, ld_dev(pp + (int64_t)s2 * HATA_PSTRIDE));
        const float M = wave_max64(m_loc);
        float l_loc = 0.f;
        for (int s2 = lane; s2 < ns; s2 += 64) {
            const float w = (M == HATA_NEG_INF) ? 0.f : fast_exp2(ld_dev(pp + (int64_t)s2 * HATA_PSTRIDE) - M);
            sm_w[g * nsp + s2] = w;
            l_loc = fmaf(w, ld_dev(pp + (int64_t)s2 * HATA_PSTRIDE + 1), l_loc);
        }
        const float Lsum = wave_sum64(l_loc);
        const float inv = Lsum > 0.f ? 1.f / Lsum : 0.f;
        for (int s2 = lane; s2 < nsp; s2 += 64) sm_w[g * nsp + s2] = (s2 < ns) ? sm_w[g * nsp + s2] * inv : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < NO; ++r) {
        const int i = tid + 256 * r;
        if (i < HT * HATA_D) {
            const int g = i / HATA_D, ch = i % HATA_D;
            const float4* w4 = reinterpret_cast<const float4*>(sm_w + g * nsp);
            float A = 0.f;
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                if (j4 * 4 < nsp) {  // weights of slices >= ns are zero
                    const float4 w = w4[j4];
                    A = fmaf(w.x, av[r][4 * j4], A); A = fmaf(w.y, av[r][4 * j4 + 1], A);
                    A = fmaf(w.z, av[r][4 * j4 + 2], A); A = fmaf(w.w, av[r][4 * j4 + 3], A);
                }
            }
            const float* pp = a.partials + ((int64_t)b * a.Hq + hq0 + g) * a.n_splits * HATA_PSTRIDE + 2 + ch;
            for (int s0 = 16; s0 < ns; s0 += 16) {
                float bv[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) bv[j] = ld_dev(pp + (int64_t)min(s0 + j, ns - 1) * HATA_PSTRIDE);
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (s0 + j < ns) A = fmaf(sm_w[g * nsp + s0 + j], bv[j], A);
            }
            const int64_t oo = ((int64_t)b * a.Hq + hq0 + g) * HATA_D + ch;
            a.out[oo] = (uint16_t)f32_to_bf16(A);
            if (a.out_f32) a.out_f32[oo] = A;
        }
    }
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
