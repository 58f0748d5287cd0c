// Decode attention over a list of cache rows (Alg. 3 of the paper: Gather + Attention, with
// the gather fused into the attention kernel; Eq. 2 third line, scale of Eq. 1), and the
// dense variant over the whole cache (Eq. 1) that serves as the comparison baseline.
//
// Split over the rows: every workgroup handles a slice of a unit's rows for HT query heads of
// the group at once (each K/V row is read once for all of them), keeps an online-softmax
// state per wave, and writes one partial (max, sum, weighted V) per query head; a small merge
// kernel combines the partials.  A row is 256 B = 16 lanes x 128-bit, so a wave reads four
// whole rows per load instruction.  bf16 inputs, fp32 softmax and accumulation.
#include "hata_device.h"
#include "hata_internal.h"

namespace hata {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

#define HATA_NEG_INF (-__builtin_huge_valf())

// partial layout per (query head, split): [0] = running max (log2 domain), [1] = sum, [2..2+d) = acc
#define HATA_PSTRIDE (HATA_D + 2)

// grid = (splits, Hkv * (G / HT), B); 256 threads = 4 waves; lane = (row group rg = lane / 16,
// sub = lane % 16 -> elements [8 sub, 8 sub + 8) of a row).
template <int HT, bool DENSE>
__global__ __launch_bounds__(256) void attn_partial_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K,
    const uint16_t* __restrict__ V, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ count_src, float* __restrict__ partials,
    int Hq, int Hkv, int G, int L_cap, int k_max, int rows_per_wg, int n_splits,
    int64_t sb, int64_t sh, int64_t sn, float scale_log2) {
    __shared__ float sm_m[4][HT];
    __shared__ float sm_l[4][HT];
    __shared__ float sm_acc[4][HT][HATA_D];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane & 15, rg = lane >> 4;
    const int split = blockIdx.x;
    const int tiles_per_group = G / HT;
    const int h = blockIdx.y / tiles_per_group;
    const int ht = blockIdx.y % tiles_per_group;
    const int b = blockIdx.z;
    const int count = DENSE ? clampi(count_src[b], 0, L_cap) : clampi(count_src[b], 0, k_max);
    const int row_begin = split * rows_per_wg;
    if (row_begin >= count) return;
    const int row_end = min(row_begin + rows_per_wg, count);
    const int64_t u = (int64_t)b * Hkv + h;
    const int hq0 = h * G + ht * HT;
    const uint16_t* Kb = K + b * sb + h * sh;
    const uint16_t* Vb = V + b * sb + h * sh;
    const int32_t* ip = DENSE ? nullptr : idx + u * k_max;

    // this lane's 8 query elements of each head, kept as packed bf16 pairs
    uint32_t qr[HT][4];
#pragma unroll
    for (int g = 0; g < HT; ++g) {
        uint4 v = *reinterpret_cast<const uint4*>(q + ((int64_t)b * Hq + hq0 + g) * HATA_D + sub * 8);
        qr[g][0] = v.x; qr[g][1] = v.y; qr[g][2] = v.z; qr[g][3] = v.w;
    }
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
            if (ok[it]) n = DENSE ? row : ip[row];
            ok[it] = ok[it] && n >= 0 && n < L_cap;
            kv[it] = make_uint4(0, 0, 0, 0);
            vv[it] = make_uint4(0, 0, 0, 0);
            if (ok[it]) {
                const int64_t o = (int64_t)n * sn + sub * 8;
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
                d += __shfl_xor(d, 1, 64);
                d += __shfl_xor(d, 2, 64);
                d += __shfl_xor(d, 4, 64);
                d += __shfl_xor(d, 8, 64);
                s[it][g] = ok[it] ? d * scale_log2 : HATA_NEG_INF;
                m_tile[g] = fmaxf(m_tile[g], s[it][g]);
            }
        }
#pragma unroll
        for (int g = 0; g < HT; ++g) {
            m_tile[g] = fmaxf(m_tile[g], __shfl_xor(m_tile[g], 16, 64));
            m_tile[g] = fmaxf(m_tile[g], __shfl_xor(m_tile[g], 32, 64));
            const float m_new = fmaxf(m_run[g], m_tile[g]);
            // m_new == -inf only while no valid row has been seen: keep the state untouched
            const float alpha = (m_new == HATA_NEG_INF) ? 1.f : exp2f(m_run[g] - m_new);
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
                const float p = ok[it] ? exp2f(s[it][g] - m_run[g]) : 0.f;
                l_run[g] += p;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
            }
        }
    }
    // combine the four row groups of the wave (all share m_run)
#pragma unroll
    for (int g = 0; g < HT; ++g) {
        l_run[g] += __shfl_xor(l_run[g], 16, 64);
        l_run[g] += __shfl_xor(l_run[g], 32, 64);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            acc[g][e] += __shfl_xor(acc[g][e], 16, 64);
            acc[g][e] += __shfl_xor(acc[g][e], 32, 64);
        }
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
    // combine the four waves and write the partial: thread -> (head, channel)
    for (int i = tid; i < HT * HATA_D; i += 256) {
        const int g = i / HATA_D, ch = i % HATA_D;
        const float m0 = sm_m[0][g], m1 = sm_m[1][g], m2 = sm_m[2][g], m3 = sm_m[3][g];
        const float M = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
        float a = 0.f, l = 0.f;
        if (M != HATA_NEG_INF) {
            const float f0 = exp2f(m0 - M), f1 = exp2f(m1 - M), f2 = exp2f(m2 - M), f3 = exp2f(m3 - M);
            a = f0 * sm_acc[0][g][ch] + f1 * sm_acc[1][g][ch] + f2 * sm_acc[2][g][ch] + f3 * sm_acc[3][g][ch];
            l = f0 * sm_l[0][g] + f1 * sm_l[1][g] + f2 * sm_l[2][g] + f3 * sm_l[3][g];
        }
        float* pp = partials + (((int64_t)b * Hq + hq0 + g) * n_splits + split) * HATA_PSTRIDE;
        pp[2 + ch] = a;
        if (ch == 0) { pp[0] = M; pp[1] = l; }
    }
}

// grid = B*Hq, 128 threads (one per channel)
__global__ __launch_bounds__(128) void attn_merge_kernel(
    const float* __restrict__ partials, const int32_t* __restrict__ count_src,
    uint16_t* __restrict__ out, float* __restrict__ out_f32, int Hq, int count_cap,
    int rows_per_wg, int n_splits) {
    const int ch = threadIdx.x;
    const int bh = blockIdx.x;
    const int b = bh / Hq;
    const int count = clampi(count_src[b], 0, count_cap);
    const int ns = (count + rows_per_wg - 1) / rows_per_wg;
    const float* pp = partials + (int64_t)bh * n_splits * HATA_PSTRIDE;
    float M = HATA_NEG_INF;
    for (int s = 0; s < ns; ++s) M = fmaxf(M, pp[s * HATA_PSTRIDE]);
    float a = 0.f, l = 0.f;
    if (M != HATA_NEG_INF) {
        for (int s = 0; s < ns; ++s) {
            const float f = exp2f(pp[s * HATA_PSTRIDE] - M);
            a = fmaf(f, pp[s * HATA_PSTRIDE + 2 + ch], a);
            l = fmaf(f, pp[s * HATA_PSTRIDE + 1], l);
        }
    }
    const float o = l > 0.f ? a / l : 0.f;
    out[(int64_t)bh * HATA_D + ch] = (uint16_t)f32_to_bf16(o);
    if (out_f32) out_f32[(int64_t)bh * HATA_D + ch] = o;
}

template <int HT>
static void launch_partial(const hata_ctx* c, bool dense, const void* q, const void* K,
                           const void* V, const int32_t* idx, const int32_t* count_src, int B,
                           float scale_log2, hipStream_t s) {
    const hata_config& f = c->cfg;
    const int rows = dense ? c->dense_rows : c->sparse_rows;
    const int splits = dense ? c->dense_splits : c->sparse_splits;
    const dim3 grid(splits, f.Hkv * (c->G / HT), B);
    if (dense)
        hipLaunchKernelGGL((attn_partial_kernel<HT, true>), grid, dim3(256), 0, s,
                           (const uint16_t*)q, (const uint16_t*)K, (const uint16_t*)V, idx,
                           count_src, c->partials, f.Hq, f.Hkv, c->G, f.L_cap, f.k_max, rows,
                           splits, f.kv_stride_b, f.kv_stride_h, f.kv_stride_n, scale_log2);
    else
        hipLaunchKernelGGL((attn_partial_kernel<HT, false>), grid, dim3(256), 0, s,
                           (const uint16_t*)q, (const uint16_t*)K, (const uint16_t*)V, idx,
                           count_src, c->partials, f.Hq, f.Hkv, c->G, f.L_cap, f.k_max, rows,
                           splits, f.kv_stride_b, f.kv_stride_h, f.kv_stride_n, scale_log2);
}

hipError_t launch_attention(const hata_ctx* c, bool dense, const void* q, const void* K,
                            const void* V, const int32_t* idx, const int32_t* count_src, int B,
                            float sm_scale, void* out, float* out_f32, hipStream_t s) {
    const hata_config& f = c->cfg;
    const float scale_log2 = sm_scale * 1.4426950408889634f;
    switch (c->HT) {
        case 8: launch_partial<8>(c, dense, q, K, V, idx, count_src, B, scale_log2, s); break;
        case 5: launch_partial<5>(c, dense, q, K, V, idx, count_src, B, scale_log2, s); break;
        case 4: launch_partial<4>(c, dense, q, K, V, idx, count_src, B, scale_log2, s); break;
        case 2: launch_partial<2>(c, dense, q, K, V, idx, count_src, B, scale_log2, s); break;
        default: launch_partial<1>(c, dense, q, K, V, idx, count_src, B, scale_log2, s); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_merge_kernel, dim3(B * f.Hq), dim3(128), 0, s, c->partials, count_src,
                       (uint16_t*)out, out_f32, f.Hq, dense ? f.L_cap : f.k_max,
                       dense ? c->dense_rows : c->sparse_rows,
                       dense ? c->dense_splits : c->sparse_splits);
    return hipGetLastError();
}

}  // namespace hata
