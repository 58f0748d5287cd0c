// Learning-to-hash trainer: one SGD step on the hash weights of one attention head (Sec. 3.1 of
// the paper, the final multi-query hashing model; App. B.2 for the optimiser).
//
//   L = c_sim sum_n s_n ||h(q_n) - h(k_n)||^2 + c_bal sum_j ||sum_{n in query j} h(k_n)||^2
//       + lam ||W^T W - I||_F,      h(x) = 2 Sigmoid(sigma x W) - 1 = tanh(sigma x W / 2)
// (the balance term per query j, as the final hashing model prints it: the triplets of a query fill
// whole blocks of TR_ROWS rows and every block names its query; without names the batch is one query)
//
// The two projections X W ([n,128] x [128,r]) and the weight-gradient contraction X^T dZ
// ([128,n] x [n,r]) are dense contractions and run on MFMA (v_mfma_f32_32x32x16_bf16).  q and k are
// bf16 already; fp32 operands (W, dZ) are split exactly into three bf16 planes, so every product is
// exact and only the fp32 accumulation rounds.
//
// Launches of a step:
//   1. train_colsum_kernel   h(k) of every key -> per-workgroup column sums (the balance term
//                            couples every row to the sum of h(k) over its query, so those sums
//                            come first);
//      train_colreduce_kernel adds them up per query
//   2. train_grad_kernel     forward of q and k again, dL/dz elementwise in the MFMA result
//                            registers, then X^T dZ with those registers as the B operand (the
//                            contraction index -- the row -- may be enumerated in any order, so the
//                            32x32 result layout is used as it stands; only X is read transposed,
//                            from the LDS tile it was staged in) -> per-workgroup partial dW
//   3. train_gram_kernel     P = W^T W - I and its squared Frobenius norm (r x r, tiny)
//   4. train_assemble_kernel dL/dW = sigma sum partials + 2 lam W P / ||P||_F, and the loss terms
//   5. train_update_kernel   weight decay, momentum, step
#include <new>

#include "hata_device.h"
#include "../../include/hata_train.h"

struct hata_train_ctx {
    hata_train_config cfg;
    int n_wgs_max;
    float* colsum_part;  // [n_wgs_max, r]
    float* colsum;       // [queries (<= n_wgs_max), r]  sum of h(k_n) over the triplets of a query
    double* scores;      // [n_max] qk scores of the label builder
    float* dw_part;      // [n_wgs_max, d, r]
    float* loss_part;    // [column groups (<= 2), n_wgs_max]
    float* P;            // [r, r]
    float* fro_part;     // [r]
    float* G;            // [d, r]
};

namespace hata {

typedef __attribute__((ext_vector_type(8))) __bf16 tr_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float tr_f32x16_t;
#define TR_ROWS 128   // triplets per workgroup (one LDS stage)
#define TR_PITCH 136  // LDS row pitch in bf16 elements (272 B: conflict-free 16-B and transposed reads)

// fp32 -> three bf16 terms whose sum carries all 24 mantissa bits (each term is the remainder
// truncated to its upper 8 significant bits, so both subtractions are exact)
__device__ __forceinline__ void split3(float x, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    const uint32_t hb = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(hb);
    const uint32_t mb = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(mb);
    hi = hb >> 16;
    mid = mb >> 16;
    lo = __float_as_uint(r2) >> 16;
}

// h = 2 Sigmoid(z) - 1
__device__ __forceinline__ float relaxed_sign(float z) { return fmaf(2.f, __builtin_amdgcn_rcpf(1.f + __expf(-z)), -1.f); }

// Weight fragments of hash column `col` as the B operand:
// frag[plane][kk] holds W[16 kk + 8 half + e][col], e = 0..7
template <int R>
__device__ __forceinline__ void load_weight_planes(const float* __restrict__ W, int col, int half,
                                                   tr_bf16x8_t (&frag)[3][8]) {
    const float* wp = W + col;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        uint32_t hi[4], mid[4], lo[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            uint32_t ph[2], pm[2], pl[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) split3(wp[(int64_t)(kk * 16 + 8 * half + 2 * e2 + q) * R], ph[q], pm[q], pl[q]);
            hi[e2] = ph[0] | (ph[1] << 16);
            mid[e2] = pm[0] | (pm[1] << 16);
            lo[e2] = pl[0] | (pl[1] << 16);
        }
        frag[0][kk] = __builtin_bit_cast(tr_bf16x8_t, make_uint4(hi[0], hi[1], hi[2], hi[3]));
        frag[1][kk] = __builtin_bit_cast(tr_bf16x8_t, make_uint4(mid[0], mid[1], mid[2], mid[3]));
        frag[2][kk] = __builtin_bit_cast(tr_bf16x8_t, make_uint4(lo[0], lo[1], lo[2], lo[3]));
    }
}

// rows [row0, row0 + TR_ROWS) of X [n, 128] into an LDS tile (zeros past n)
template <int THREADS>
__device__ __forceinline__ void stage_rows(const uint16_t* __restrict__ X, int row0, int n, uint16_t* tile) {
    for (int i = threadIdx.x; i < TR_ROWS * 16; i += THREADS) {
        const int row = i >> 4, sub = i & 15;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row0 + row < n) v = *reinterpret_cast<const uint4*>(X + (int64_t)(row0 + row) * HATA_D + sub * 8);
        *reinterpret_cast<uint4*>(&tile[row * TR_PITCH + sub * 8]) = v;
    }
}

// Z tile t (32 rows x the wave's 32 columns) = X_tile . W: result register ri of lane (m, half)
// holds row 8 (ri / 4) + 4 half + ri % 4 of the tile, column 32 w + m
__device__ __forceinline__ tr_f32x16_t project_tile(const uint16_t* tile, int t, int m, int half,
                                                    const tr_bf16x8_t (&wfrag)[3][8]) {
    tr_f32x16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        const tr_bf16x8_t x = *reinterpret_cast<const tr_bf16x8_t*>(&tile[(t * 32 + m) * TR_PITCH + kk * 16 + 8 * half]);
#pragma unroll
        for (int p = 0; p < 3; ++p) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, wfrag[p][kk], acc, 0, 0, 0);
    }
    return acc;
}

// grid = (workgroups of TR_ROWS triplets, groups of up to 128 hash columns); a wave owns 32 columns
template <int R>
__global__ __launch_bounds__((R < 128 ? R : 128) * 2) void train_colsum_kernel(
    const uint16_t* __restrict__ K, const float* __restrict__ W, int n, float sigma,
    float* __restrict__ colsum_part) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[TR_ROWS * TR_PITCH];
    constexpr int THREADS = (R < 128 ? R : 128) * 2;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 31, half = lane >> 5;
    const int col = blockIdx.y * 128 + w * 32 + m;
    tr_bf16x8_t wfrag[3][8];
    load_weight_planes<R>(W, col, half, wfrag);
    stage_rows<THREADS>(K, blockIdx.x * TR_ROWS, n, tile);
    __syncthreads();
    float cs = 0.f;
#pragma unroll
    for (int t = 0; t < TR_ROWS / 32; ++t) {
        const tr_f32x16_t z = project_tile(tile, t, m, half, wfrag);
#pragma unroll
        for (int i = 0; i < 16; ++i) cs += relaxed_sign(sigma * z[i]);  // (rows past n are zero: h = 0)
    }
    cs += __shfl_xor(cs, 32, 64);
    if (half == 0) colsum_part[(int64_t)blockIdx.x * R + col] = cs;
}

// the query a block of TR_ROWS triplets belongs to (no names: everything is query 0; a name outside
// [0, n_groups) counts as the nearest valid one, so no access leaves the arrays)
__device__ __forceinline__ int block_query(const int32_t* __restrict__ block_group, int wg, int n_groups) {
    return block_group ? clampi(block_group[wg], 0, n_groups - 1) : 0;
}

// sum of the per-workgroup column sums of one query: one workgroup per (hash column, query)
__global__ __launch_bounds__(256) void train_colreduce_kernel(const float* __restrict__ colsum_part, int r,
                                                              int n_wgs, const int32_t* __restrict__ block_group,
                                                              int n_groups, float* __restrict__ colsum) {
    __shared__ float red[4];
    const int j = blockIdx.x, q = blockIdx.y, tid = threadIdx.x;
    float acc = 0.f;
    for (int g = tid; g < n_wgs; g += 256)
        if (block_query(block_group, g, n_groups) == q) acc += colsum_part[(int64_t)g * r + j];
    acc = wave_sum64(acc);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) colsum[(int64_t)q * r + j] = red[0] + red[1] + red[2] + red[3];
}

template <int R>
__global__ __launch_bounds__((R < 128 ? R : 128) * 2) void train_grad_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const float* __restrict__ s,
    const float* __restrict__ W, int n, float sigma, float c_sim2, float c_bal2,
    const float* __restrict__ colsum, const int32_t* __restrict__ block_group, int n_groups,
    float* __restrict__ dw_part, float* __restrict__ loss_part) {
    constexpr int THREADS = (R < 128 ? R : 128) * 2;
    __shared__ __attribute__((aligned(16))) uint16_t tile_q[TR_ROWS * TR_PITCH];
    __shared__ __attribute__((aligned(16))) uint16_t tile_k[TR_ROWS * TR_PITCH];
    __shared__ float s_lab[TR_ROWS];
    __shared__ float s_col[R];          // sum of h(k_n) over this block's query, per hash column
    __shared__ float s_loss[THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 31, half = lane >> 5;
    const int row0 = blockIdx.x * TR_ROWS;
    const int col = blockIdx.y * 128 + w * 32 + m;
    tr_bf16x8_t wfrag[3][8];
    load_weight_planes<R>(W, col, half, wfrag);
    const float* colsum_q = colsum + (int64_t)block_query(block_group, blockIdx.x, n_groups) * R;
    for (int j = tid; j < R; j += THREADS) s_col[j] = colsum_q[j];
    for (int i = tid; i < TR_ROWS; i += THREADS) s_lab[i] = (row0 + i < n) ? s[row0 + i] : 0.f;
    stage_rows<THREADS>(Q, row0, n, tile_q);
    stage_rows<THREADS>(K, row0, n, tile_k);
    __syncthreads();
    const float colk = c_bal2 * s_col[col];
    tr_f32x16_t dw[4];  // dw[ct][ri]: channel 32 ct + 8 (ri / 4) + 4 half + ri % 4, this lane's column
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) dw[ct][i] = 0.f;
    float lsim = 0.f;
#pragma unroll 1
    for (int t = 0; t < TR_ROWS / 32; ++t) {
        const tr_f32x16_t zq = project_tile(tile_q, t, m, half, wfrag);
        const tr_f32x16_t zk = project_tile(tile_k, t, m, half, wfrag);
        float da[16], db[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = t * 32 + 8 * (i / 4) + 4 * half + (i % 4);
            const float hq = relaxed_sign(sigma * zq[i]), hk = relaxed_sign(sigma * zk[i]);
            const float diff = hq - hk, sl = s_lab[row];
            const float dhq = c_sim2 * sl * diff;
            const float dhk = colk - dhq;
            da[i] = dhq * (1.f - hq * hq) * 0.5f;
            db[i] = dhk * (1.f - hk * hk) * 0.5f;
            lsim = fmaf(sl * diff, diff, lsim);
        }
        // X^T dZ over the tile's 32 rows, 16 per MFMA: the B operand is dZ as it sits in the
        // registers (slot (half, j) of step ks <-> row 16 ks + 8 (j / 4) + 4 half + j % 4), the A
        // operand X read from the LDS tile in that same row order
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            tr_bf16x8_t bq[3], bk[3];
            {
                uint32_t pq[3][4], pk[3][4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    uint32_t h0, m0, l0, h1, m1, l1;
                    split3(da[8 * ks + 2 * e2], h0, m0, l0);
                    split3(da[8 * ks + 2 * e2 + 1], h1, m1, l1);
                    pq[0][e2] = h0 | (h1 << 16); pq[1][e2] = m0 | (m1 << 16); pq[2][e2] = l0 | (l1 << 16);
                    split3(db[8 * ks + 2 * e2], h0, m0, l0);
                    split3(db[8 * ks + 2 * e2 + 1], h1, m1, l1);
                    pk[0][e2] = h0 | (h1 << 16); pk[1][e2] = m0 | (m1 << 16); pk[2][e2] = l0 | (l1 << 16);
                }
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    bq[p] = __builtin_bit_cast(tr_bf16x8_t, make_uint4(pq[p][0], pq[p][1], pq[p][2], pq[p][3]));
                    bk[p] = __builtin_bit_cast(tr_bf16x8_t, make_uint4(pk[p][0], pk[p][1], pk[p][2], pk[p][3]));
                }
            }
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
                uint32_t aq[4], ak[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    // slots j = 2 e2, 2 e2 + 1 -> rows 16 ks + 8 (j / 4) + 4 half + j % 4
                    const int j0 = 2 * e2;
                    const int r0 = t * 32 + 16 * ks + 8 * (j0 / 4) + 4 * half + (j0 % 4);
                    const int o = r0 * TR_PITCH + 32 * ct + m;
                    aq[e2] = (uint32_t)tile_q[o] | ((uint32_t)tile_q[o + TR_PITCH] << 16);
                    ak[e2] = (uint32_t)tile_k[o] | ((uint32_t)tile_k[o + TR_PITCH] << 16);
                }
                const tr_bf16x8_t xq = __builtin_bit_cast(tr_bf16x8_t, make_uint4(aq[0], aq[1], aq[2], aq[3]));
                const tr_bf16x8_t xk = __builtin_bit_cast(tr_bf16x8_t, make_uint4(ak[0], ak[1], ak[2], ak[3]));
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    dw[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xq, bq[p], dw[ct], 0, 0, 0);
                    dw[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xk, bk[p], dw[ct], 0, 0, 0);
                }
            }
        }
    }
    float* out = dw_part + (int64_t)blockIdx.x * HATA_D * R;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ch = 32 * ct + 8 * (i / 4) + 4 * half + (i % 4);
            out[(int64_t)ch * R + col] = dw[ct][i];
        }
    lsim = wave_sum64(lsim);
    if (lane == 0) s_loss[w] = lsim;
    __syncthreads();
    if (tid == 0) {  // (the similarity partial of column group y; the groups are summed later)
        float t = 0.f;
        for (int i = 0; i < THREADS / 64; ++i) t += s_loss[i];
        loss_part[blockIdx.y * gridDim.x + blockIdx.x] = t;
    }
}

// P = W^T W - I (column j per workgroup) and the squared Frobenius norm of that column
__global__ __launch_bounds__(256) void train_gram_kernel(const float* __restrict__ W, int r,
                                                         float* __restrict__ P, float* __restrict__ fro_part) {
    __shared__ float red[4];
    const int j = blockIdx.x, i = threadIdx.x;
    float sq = 0.f;
    if (i < r) {
        float acc = 0.f;
#pragma unroll 16
        for (int c = 0; c < HATA_D; ++c) acc = fmaf(W[(int64_t)c * r + i], W[(int64_t)c * r + j], acc);
        acc -= (i == j) ? 1.f : 0.f;
        P[(int64_t)i * r + j] = acc;
        sq = acc * acc;
    }
    sq = wave_sum64(sq);
    if ((i & 63) == 0) red[i >> 6] = sq;
    __syncthreads();
    if (i == 0) fro_part[j] = red[0] + red[1] + red[2] + red[3];
}

// dL/dW = sigma * sum of the partials + 2 lam W P / ||P||_F; block 0 also writes the loss terms
__global__ __launch_bounds__(256) void train_assemble_kernel(
    const float* __restrict__ W, int r, int n_wgs, float sigma, float lam, float c_sim, float c_bal,
    const float* __restrict__ dw_part, const float* __restrict__ P, const float* __restrict__ fro_part,
    const float* __restrict__ colsum, int n_groups, const float* __restrict__ loss_part,
    float* __restrict__ G, float* __restrict__ grad, float* __restrict__ loss) {
    __shared__ float s_fro;
    __shared__ float red[4];
    const int tid = threadIdx.x;
    {
        float f = 0.f;
        for (int j = tid; j < r; j += 256) f += fro_part[j];
        f = wave_sum64(f);
        if ((tid & 63) == 0) red[tid >> 6] = f;
        __syncthreads();
        if (tid == 0) s_fro = sqrtf(red[0] + red[1] + red[2] + red[3]);
        __syncthreads();
    }
    const float fro = s_fro;
    // 64 elements per workgroup; wave w sums a quarter of the partials (and a quarter of the W P
    // row-column product) of each, the four quarters meet in LDS in a fixed order
    __shared__ float quart[4][64];
    const int el = tid & 63, sl = tid >> 6;
    const int e = blockIdx.x * 64 + el;
    float g = 0.f;
    if (e < HATA_D * r) {
        const int c = e / r, j = e % r;
        // (eight independent chains: the loads of a chain step are in flight together)
        float gp[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int wg = (int)((int64_t)sl * n_wgs / 4);
        const int wg_end = (int)((int64_t)(sl + 1) * n_wgs / 4);
        for (; wg + 8 <= wg_end; wg += 8) {
#pragma unroll
            for (int u = 0; u < 8; ++u) gp[u] += dw_part[(int64_t)(wg + u) * HATA_D * r + e];
        }
        for (; wg < wg_end; ++wg) gp[0] += dw_part[(int64_t)wg * HATA_D * r + e];
        g = (((gp[0] + gp[1]) + (gp[2] + gp[3])) + ((gp[4] + gp[5]) + (gp[6] + gp[7]))) * sigma;
        if (fro > 0.f) {
            float wp = 0.f;
            const int i0 = sl * (r / 4), i1 = i0 + r / 4;  // (r is a multiple of 32)
#pragma unroll 8
            for (int i = i0; i < i1; ++i) wp = fmaf(W[(int64_t)c * r + i], P[(int64_t)i * r + j], wp);
            g += lam * 2.f * wp / fro;
        }
    }
    quart[sl][el] = g;
    __syncthreads();
    if (sl == 0 && e < HATA_D * r) {
        g = (quart[0][el] + quart[1][el]) + (quart[2][el] + quart[3][el]);
        G[e] = g;
        if (grad) grad[e] = g;
    }
    if (blockIdx.x == 0 && loss) {
        // similarity: sum of the workgroup partials; balance: squared norm of the column sums
        float ls = 0.f, lb = 0.f;
        for (int wg = tid; wg < n_wgs * ((r + 127) / 128); wg += 256) ls += loss_part[wg];
        for (int j = tid; j < r * n_groups; j += 256) lb = fmaf(colsum[j], colsum[j], lb);
        ls = wave_sum64(ls);
        lb = wave_sum64(lb);
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = ls;
        __syncthreads();
        const float ls_all = red[0] + red[1] + red[2] + red[3];
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = lb;
        __syncthreads();
        if (tid == 0) {
            loss[0] = c_sim * ls_all;
            loss[1] = c_bal * (red[0] + red[1] + red[2] + red[3]);
            loss[2] = lam * fro;
        }
    }
}

// Label builder (App. B.1, steps 3-4).  qk scores of one query against m keys, in fp64 (every product
// of two bf16 values is exact there): a row per 16 lanes, 8 channels per lane.
__global__ __launch_bounds__(256) void train_scores_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ K,
                                                           int m, double* __restrict__ scores) {
    const int sub = threadIdx.x & 15;
    const int row = blockIdx.x * 16 + (threadIdx.x >> 4);
    double acc = 0.0;
    if (row < m) {
        const uint4 kv = *reinterpret_cast<const uint4*>(K + (int64_t)row * HATA_D + sub * 8);
        const uint4 qv = *reinterpret_cast<const uint4*>(q + sub * 8);
        const uint32_t kw[4] = {kv.x, kv.y, kv.z, kv.w}, qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc = fma((double)bf16_lo(kw[i]), (double)bf16_lo(qw[i]), acc);
            acc = fma((double)bf16_hi(kw[i]), (double)bf16_hi(qw[i]), acc);
        }
    }
    // sum over the 16 lanes of the row, in a fixed order
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 16);
    if (row < m && sub == 0) scores[row] = acc;
}

// rank of every pair by counting (pairs with a larger score, or an equal score and a lower index,
// come first); the first n_pos ranks get 20 .. 1 in equal steps, the others -1
__global__ __launch_bounds__(256) void train_labels_kernel(const double* __restrict__ scores, int m, int n_pos,
                                                           float* __restrict__ s) {
    __shared__ double tile[256];
    const int i = blockIdx.x * 256 + threadIdx.x;
    const double mine = i < m ? scores[i] : 0.0;
    int rank = 0;
    for (int j0 = 0; j0 < m; j0 += 256) {
        __syncthreads();
        tile[threadIdx.x] = (j0 + threadIdx.x < m) ? scores[j0 + threadIdx.x] : 0.0;
        __syncthreads();
        const int nj = min(256, m - j0);
        for (int j = 0; j < nj; ++j) {
            const double o = tile[j];
            rank += (o > mine || (o == mine && j0 + j < i)) ? 1 : 0;
        }
    }
    if (i < m) {
        float lab = -1.f;
        if (rank < n_pos) lab = (float)(n_pos == 1 ? 20.0 : 20.0 - 19.0 * (double)rank / (double)(n_pos - 1));
        s[i] = lab;
    }
}

__global__ __launch_bounds__(256) void train_update_kernel(float* __restrict__ W, float* __restrict__ v,
                                                           const float* __restrict__ G, int count, float lr,
                                                           float momentum, float weight_decay) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e < count) {
        const float g = fmaf(weight_decay, W[e], G[e]);
        const float vn = fmaf(momentum, v[e], g);
        v[e] = vn;
        W[e] = fmaf(-lr, vn, W[e]);
    }
}

}  // namespace hata

namespace {
constexpr size_t kAlignT = 256;
inline size_t align_up_t(size_t x) { return (x + kAlignT - 1) / kAlignT * kAlignT; }
struct TrainPlan { int n_wgs_max; size_t off_colsum, off_cs, off_dw, off_loss, off_P, off_fro, off_G, off_scores, total; };
int make_train_plan(const hata_train_config* f, TrainPlan* p) {
    if (!f) return HATA_EINVAL;
    if (f->n_max < 1) return HATA_EINVAL;
    if (f->d != 128) return HATA_EUNSUPPORTED;
    if (f->r != 32 && f->r != 64 && f->r != 128 && f->r != 256) return HATA_EUNSUPPORTED;
    p->n_wgs_max = (f->n_max + TR_ROWS - 1) / TR_ROWS;
    if (p->n_wgs_max > 65535) return HATA_EUNSUPPORTED;
    size_t o = 0;
    p->off_colsum = o; o = align_up_t(o + (size_t)p->n_wgs_max * f->r * 4);
    p->off_cs = o;     o = align_up_t(o + (size_t)p->n_wgs_max * f->r * 4);
    p->off_dw = o;     o = align_up_t(o + (size_t)p->n_wgs_max * f->d * f->r * 4);
    p->off_loss = o;   o = align_up_t(o + (size_t)p->n_wgs_max * 2 * 4);
    p->off_P = o;      o = align_up_t(o + (size_t)f->r * f->r * 4);
    p->off_fro = o;    o = align_up_t(o + (size_t)f->r * 4);
    p->off_G = o;      o = align_up_t(o + (size_t)f->d * f->r * 4);
    p->off_scores = o; o = align_up_t(o + (size_t)f->n_max * 8);
    p->total = o;
    return HATA_OK;
}
}  // namespace

extern "C" {

int hata_train_workspace_bytes(const hata_train_config* cfg, size_t* out) {
    if (!out) return HATA_EINVAL;
    TrainPlan p;
    const int rc = make_train_plan(cfg, &p);
    if (rc != HATA_OK) return rc;
    *out = p.total;
    return HATA_OK;
}

int hata_train_create(hata_train_ctx** ctx_out, const hata_train_config* cfg, void* workspace,
                      size_t workspace_bytes) {
    if (!ctx_out) return HATA_EINVAL;
    *ctx_out = nullptr;
    TrainPlan p;
    const int rc = make_train_plan(cfg, &p);
    if (rc != HATA_OK) return rc;
    if (!workspace || ((uintptr_t)workspace % kAlignT) != 0 || workspace_bytes < p.total) return HATA_EWORKSPACE;
    hata_train_ctx* c = new (std::nothrow) hata_train_ctx;
    if (!c) return HATA_EINVAL;
    c->cfg = *cfg;
    c->n_wgs_max = p.n_wgs_max;
    char* w = (char*)workspace;
    c->colsum_part = (float*)(w + p.off_colsum);
    c->colsum = (float*)(w + p.off_cs);
    c->dw_part = (float*)(w + p.off_dw);
    c->loss_part = (float*)(w + p.off_loss);
    c->P = (float*)(w + p.off_P);
    c->fro_part = (float*)(w + p.off_fro);
    c->G = (float*)(w + p.off_G);
    c->scores = (double*)(w + p.off_scores);
    *ctx_out = c;
    return HATA_OK;
}

int hata_train_destroy(hata_train_ctx* ctx) {
    delete ctx;
    return HATA_OK;
}

int hata_train_step(hata_train_ctx* ctx, const void* Q, const void* K, const float* s, int32_t n,
                    const int32_t* block_query, int32_t n_queries, float* W, float* v,
                    const hata_train_hparams* hp, float* grad, float* loss, void* stream) {
    if (!ctx || !Q || !K || !s || !W || !v || !hp) return HATA_EINVAL;
    if (n < 1 || n > ctx->cfg.n_max) return HATA_EINVAL;
    if (!block_query) n_queries = 1;
    if (n_queries < 1 || n_queries > (n + TR_ROWS - 1) / TR_ROWS || ((uintptr_t)block_query % 4)) return HATA_EINVAL;
    if (((uintptr_t)Q % 16) || ((uintptr_t)K % 16) || ((uintptr_t)W % 16) || ((uintptr_t)v % 4) || ((uintptr_t)s % 4))
        return HATA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const int r = ctx->cfg.r;
    const int n_wgs = (n + TR_ROWS - 1) / TR_ROWS;
    const float c_sim = hp->eps * hp->scale_sim, c_bal = hp->eta * hp->scale_bal;
    const uint16_t* q = (const uint16_t*)Q;
    const uint16_t* k = (const uint16_t*)K;
#define HATA_TRAIN_LAUNCH(RR)                                                                          \
    hipLaunchKernelGGL((hata::train_colsum_kernel<RR>), dim3(n_wgs, (RR + 127) / 128),                 \
                       dim3((RR < 128 ? RR : 128) * 2), 0, st, k, W, n, hp->sigma, ctx->colsum_part);  \
    hipLaunchKernelGGL(hata::train_colreduce_kernel, dim3(RR, n_queries), dim3(256), 0, st,            \
                       ctx->colsum_part, RR, n_wgs, block_query, n_queries, ctx->colsum);              \
    hipLaunchKernelGGL((hata::train_grad_kernel<RR>), dim3(n_wgs, (RR + 127) / 128),                   \
                       dim3((RR < 128 ? RR : 128) * 2), 0, st, q, k, s, W, n, hp->sigma,               \
                       2.f * c_sim, 2.f * c_bal, ctx->colsum, block_query, n_queries, ctx->dw_part,     \
                       ctx->loss_part)
    switch (r) {
        case 32: HATA_TRAIN_LAUNCH(32); break;
        case 64: HATA_TRAIN_LAUNCH(64); break;
        case 128: HATA_TRAIN_LAUNCH(128); break;
        default: HATA_TRAIN_LAUNCH(256); break;
    }
#undef HATA_TRAIN_LAUNCH
    hipLaunchKernelGGL(hata::train_gram_kernel, dim3(r), dim3(256), 0, st, W, r, ctx->P, ctx->fro_part);
    const int count = ctx->cfg.d * r;
    hipLaunchKernelGGL(hata::train_assemble_kernel, dim3((count + 63) / 64), dim3(256), 0, st, W, r,
                       n_wgs, hp->sigma, hp->lam, c_sim, c_bal, ctx->dw_part, ctx->P, ctx->fro_part,
                       ctx->colsum, n_queries, ctx->loss_part, ctx->G, grad, loss);
    hipLaunchKernelGGL(hata::train_update_kernel, dim3((count + 255) / 256), dim3(256), 0, st, W, v,
                       ctx->G, count, hp->lr, hp->momentum, hp->weight_decay);
    return hipGetLastError() == hipSuccess ? HATA_OK : HATA_EHIP;
}

int hata_train_make_labels(hata_train_ctx* ctx, const void* q, const void* K, int32_t m, float* s,
                           void* stream) {
    if (!ctx || !q || !K || !s) return HATA_EINVAL;
    if (m < 1 || m > ctx->cfg.n_max) return HATA_EINVAL;
    if (((uintptr_t)q % 16) || ((uintptr_t)K % 16) || ((uintptr_t)s % 4)) return HATA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    int n_pos = m / 10;
    if (n_pos < 1) n_pos = 1;
    hipLaunchKernelGGL(hata::train_scores_kernel, dim3((m + 15) / 16), dim3(256), 0, st, (const uint16_t*)q,
                       (const uint16_t*)K, m, ctx->scores);
    hipLaunchKernelGGL(hata::train_labels_kernel, dim3((m + 255) / 256), dim3(256), 0, st, ctx->scores, m, n_pos, s);
    return hipGetLastError() == hipSuccess ? HATA_OK : HATA_EHIP;
}

}  // extern "C"
