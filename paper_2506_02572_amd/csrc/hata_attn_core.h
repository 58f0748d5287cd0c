// Device-side core of decode attention over a list of cache rows (Alg. 3 of the paper: Gather +
// Attention with the gather fused; Eq. 2 third line, scale of Eq. 1), shared by the stand-alone
// attention kernels and the cooperative decode-step kernel.
//
// A workgroup of 256 threads (4 waves) handles a slice of a unit's rows for HT query heads of the
// group at once, so each K/V row is read once for all of them.  A row is 256 B = 16 lanes x 128-bit:
// lane = (row group rg = lane / 16, sub = lane % 16 -> elements [8 sub, 8 sub + 8) of a row), a wave
// reads four whole rows per load instruction.  q.k uses v_dot2_f32_bf16; reductions over the 16
// lanes of a row use DPP, over the 4 row groups the lane-swap instructions.  Every wave keeps its
// own online-softmax state (no workgroup barrier inside the row loop); the four states are combined
// through LDS at the end.  bf16 inputs, fp32 softmax and accumulation.
#pragma once
#include "hata_device.h"

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
// partial layout per (query head, slice): [0] = running max (log2 domain), [1] = sum, [2..2+d) = acc
#define HATA_PSTRIDE (HATA_D + 2)

// (the accumulator rows are padded by 4 floats so that the 128-bit stores of the matrix-core path,
// one head per lane, spread over the LDS banks)
template <int HT>
struct AttnLds {
    float m[4][HT];
    float l[4][HT];
    float acc[4][HT][HATA_D + 4];  // reused by the merge for the slice weights
};

// this lane's 8 query elements of each of the HT heads starting at q0 (packed bf16 pairs)
template <int HT>
__device__ __forceinline__ void attn_load_q(const uint16_t* __restrict__ q0, uint32_t (&qr)[HT][4]) {
    const int sub = threadIdx.x & 15;
#pragma unroll
    for (int g = 0; g < HT; ++g) {
        const uint4 v = *reinterpret_cast<const uint4*>(q0 + (int64_t)g * HATA_D + sub * 8);
        qr[g][0] = v.x; qr[g][1] = v.y; qr[g][2] = v.z; qr[g][3] = v.w;
    }
}

// Attention of the HT heads over rows [row_begin, row_end): row_of(row) gives the cache row (< 0 or
// >= L_cap: skipped).  On return (after a workgroup barrier) S holds the four waves' states.
// Must be called by all 256 threads.
// IT: 16-row load iterations per tile (a tile of 16 IT rows is in flight per workgroup).
template <int HT, int IT, typename RowOf>
__device__ __forceinline__ void attn_rows(
    const uint32_t (&qr)[HT][4], const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb,
    int64_t sn, int L_cap, int row_begin, int row_end, float scale_log2, RowOf row_of,
    AttnLds<HT>& S) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane & 15, rg = lane >> 4;
    float m_run[HT], l_run[HT], acc[HT][8];
#pragma unroll
    for (int g = 0; g < HT; ++g) {
        m_run[g] = HATA_NEG_INF; l_run[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }
    for (int tile = row_begin; tile < row_end; tile += 16 * IT) {
        uint4 kv[IT], vv[IT];
        bool ok[IT];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int row = tile + it * 16 + wave * 4 + rg;
            ok[it] = row < row_end;
            int n = 0;
            if (ok[it]) n = row_of(row);
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
                d = row_sum16(d);
                s[it][g] = ok[it] ? d * scale_log2 : HATA_NEG_INF;
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
            if (sub == 0) { S.m[wave][g] = m_run[g]; S.l[wave][g] = l_run[g]; }
#pragma unroll
            for (int e = 0; e < 8; ++e) S.acc[wave][g][sub * 8 + e] = acc[g][e];
        }
    }
    __syncthreads();
}

// ---- the same step on the matrix cores, for 4 <= HT <= 16 heads ----
// With 8 heads the VALU form above is instruction-bound (every lane repeats the softmax of its row
// for all heads, and each q.k needs a 16-lane reduction), so the two contractions go to MFMA with the
// heads padded to 16:
//   S[row][head]   = K_tile[16 rows][128] . Q^T[128][16 heads]     4 x v_mfma_f32_16x16x32_bf16
//   O^T[ch][head] += V_tile^T[16 ch][16 rows] . P[16 rows][16 heads]   per 16-channel tile, P split
//                    into two bf16 terms (hi + lo) so its rounding stays below 2^-16
// A wave owns a tile of 16 rows.  Lane = (n = lane % 16, kg = lane / 16): for the loads n is the row
// and kg selects 8 of every 32 channels (one 128-bit load per 32 channels, straight into the MFMA
// operand layout); in S and in the accumulators n is the HEAD, so the online-softmax state (max,
// sum) is one scalar per lane, and the 4 rows a lane holds of S (rows 4 kg .. 4 kg + 3) are exactly
// the k-slice of P the second contraction wants from it.  Only V needs a transpose (its operand
// wants 4 rows of one channel per lane): the tile goes through a wave-private LDS buffer, rows
// padded to 264 B so that the 2-byte transposed reads are bank-conflict free.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define HATA_VT_PITCH 132                    // uint16 per staged V row (264 B)
#define HATA_VT_WAVE (16 * HATA_VT_PITCH)    // uint16 per wave
#define HATA_VT_ELEMS (4 * HATA_VT_WAVE)     // uint16 of LDS a workgroup needs for attn_rows_mfma

// Q as the B operand: lane (n, kg) holds q[head n][32 s + 8 kg, + 8) for s < 4; heads >= HT are zero
template <int HT>
__device__ __forceinline__ void attn_load_q_mfma(const uint16_t* __restrict__ q0, uint4 (&qb)[4]) {
    const int lane = threadIdx.x & 63, n = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        qb[s] = make_uint4(0, 0, 0, 0);
        if (n < HT) qb[s] = *reinterpret_cast<const uint4*>(q0 + (int64_t)n * HATA_D + 32 * s + 8 * kg);
    }
}

// Same contract as attn_rows (state of the four waves in S after a workgroup barrier).  IT: 16-row
// tiles per wave whose loads are in flight together; PF: software pipeline -- the loads of the
// next IT tiles are issued before the current ones are consumed (measured on the dense baseline:
// no faster than IT = 2 without it, so no caller turns it on).  vt: HATA_VT_ELEMS uint16 of LDS.
template <int HT, int IT, bool PF, typename RowOf>
__device__ __forceinline__ void attn_rows_mfma(
    const uint4 (&qb)[4], const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb, int64_t sn,
    int L_cap, int row_begin, int row_end, float scale_log2, RowOf row_of, AttnLds<HT>& S,
    uint16_t* vt_all) {
    static_assert(HT >= 1 && HT <= 16, "heads are padded to one 16-wide MFMA tile");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kg = lane >> 4;
    uint16_t* vt = vt_all + wave * HATA_VT_WAVE;
    float m_run = HATA_NEG_INF, l_run = 0.f;
    f32x4_t acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    struct Stage { uint4 kr[IT][4], vr[IT][4]; bool ok[IT]; };
    // loads of the IT tiles of this wave in the 64 * IT rows from tile0 (lane: row n, channels 8 kg + 32 s)
    auto load_stage = [&](int tile0, Stage& st) {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int row = tile0 + (it * 4 + wave) * 16 + n;
            st.ok[it] = row < row_end;
            int idx = 0;
            if (st.ok[it]) idx = row_of(row);
            st.ok[it] = st.ok[it] && idx >= 0 && idx < L_cap;
#pragma unroll
            for (int s = 0; s < 4; ++s) { st.kr[it][s] = make_uint4(0, 0, 0, 0); st.vr[it][s] = make_uint4(0, 0, 0, 0); }
            if (st.ok[it]) {
                const int64_t o = (int64_t)idx * sn + 8 * kg;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    st.kr[it][s] = *reinterpret_cast<const uint4*>(Kb + o + 32 * s);
                    st.vr[it][s] = *reinterpret_cast<const uint4*>(Vb + o + 32 * s);
                }
            }
        }
    };
    auto compute_stage = [&](int tile0, const Stage& st) {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            if (tile0 + (it * 4 + wave) * 16 >= row_end) break;  // wave-uniform: no row in this tile
            const unsigned long long okmask = __builtin_amdgcn_ballot_w64(st.ok[it]);  // bits 0..15: the tile's rows
            f32x4_t sacc = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, st.kr[it][s]),
                                                               __builtin_bit_cast(bf16x8_t, qb[s]), sacc, 0, 0, 0);
            // stage V (row n, channels 32 s + 8 kg) for the transposed reads below
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uint2* d = reinterpret_cast<uint2*>(vt + n * HATA_VT_PITCH + 32 * s + 8 * kg);
                d[0] = make_uint2(st.vr[it][s].x, st.vr[it][s].y);
                d[1] = make_uint2(st.vr[it][s].z, st.vr[it][s].w);
            }
            // online softmax of head n over the rows 4 kg .. 4 kg + 3 this lane holds
            float sv[4], m_tile = HATA_NEG_INF;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool valid = (okmask >> (4 * kg + r)) & 1ull;
                sv[r] = valid ? sacc[r] * scale_log2 : HATA_NEG_INF;
                m_tile = fmaxf(m_tile, sv[r]);
            }
            m_tile = rows_max4(m_tile);
            const float m_new = fmaxf(m_run, m_tile);
            const float alpha = (m_new == HATA_NEG_INF) ? 1.f : fast_exp2(m_run - m_new);
            float p[4], psum = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[r] = (sv[r] == HATA_NEG_INF) ? 0.f : fast_exp2(sv[r] - m_new);
                psum += p[r];
            }
            l_run = fmaf(l_run, alpha, psum);
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0ull) {
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[c] *= alpha;
            }
            // P as two bf16 terms: hi = p truncated to bf16, lo = (p - hi) truncated to bf16
            uint32_t hb[4], lb[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                hb[r] = __float_as_uint(p[r]) & 0xffff0000u;
                lb[r] = __float_as_uint(p[r] - __uint_as_float(hb[r]));
            }
            const uint2 ph = make_uint2((hb[0] >> 16) | hb[1], (hb[2] >> 16) | hb[3]);
            const uint2 pl = make_uint2((lb[0] >> 16) | (lb[1] & 0xffff0000u), (lb[2] >> 16) | (lb[3] & 0xffff0000u));
            const s16x4_t phv = __builtin_bit_cast(s16x4_t, ph), plv = __builtin_bit_cast(s16x4_t, pl);
            __builtin_amdgcn_wave_barrier();  // (LDS serves a wave's accesses in order: the staged tile is visible)
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const uint16_t* src = vt + (4 * kg) * HATA_VT_PITCH + 16 * c + n;
                const uint32_t v0 = src[0], v1 = src[HATA_VT_PITCH], v2 = src[2 * HATA_VT_PITCH], v3 = src[3 * HATA_VT_PITCH];
                const s16x4_t av = __builtin_bit_cast(s16x4_t, make_uint2(v0 | (v1 << 16), v2 | (v3 << 16)));
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, phv, acc[c], 0, 0, 0);
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, plv, acc[c], 0, 0, 0);
            }
            __builtin_amdgcn_wave_barrier();
        }
    };
    if constexpr (PF) {
        Stage cur, nxt;
        load_stage(row_begin, cur);
        for (int tile0 = row_begin; tile0 < row_end; tile0 += 64 * IT) {
            const bool more = tile0 + 64 * IT < row_end;  // workgroup-uniform
            if (more) load_stage(tile0 + 64 * IT, nxt);
            compute_stage(tile0, cur);
            if (more) cur = nxt;
        }
    } else {
        for (int tile0 = row_begin; tile0 < row_end; tile0 += 64 * IT) {
            Stage st;
            load_stage(tile0, st);
            compute_stage(tile0, st);
        }
    }
    // lanes of the 4 row groups hold partial sums of the same head
    l_run = rows_sum4(l_run);
    if (n < HT) {
        if (kg == 0) { S.m[wave][n] = m_run; S.l[wave][n] = l_run; }
#pragma unroll
        for (int c = 0; c < 8; ++c)  // acc[c][r] = O[head n][channel 16 c + 4 kg + r]
            *reinterpret_cast<float4*>(&S.acc[wave][n][16 * c + 4 * kg]) = make_float4(acc[c][0], acc[c][1], acc[c][2], acc[c][3]);
    }
    __syncthreads();
}

// Combine the four wave states in S (thread -> (head, channel)).  final: write the attention
// output of head g to out[g * 128 + ch]; otherwise write the slice's partial (max, sum, acc) for
// head g at part + g * head_stride with write-through stores.
template <int HT>
__device__ __forceinline__ void attn_emit(
    const AttnLds<HT>& S, bool final, uint16_t* __restrict__ out, float* __restrict__ out_f32,
    float* __restrict__ part, int64_t head_stride) {
    for (int i = threadIdx.x; i < HT * HATA_D; i += 256) {
        const int g = i / HATA_D, ch = i % HATA_D;
        const float m0 = S.m[0][g], m1 = S.m[1][g], m2 = S.m[2][g], m3 = S.m[3][g];
        const float M = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
        float av = 0.f, l = 0.f;
        if (M != HATA_NEG_INF) {
            const float f0 = fast_exp2(m0 - M), f1 = fast_exp2(m1 - M), f2 = fast_exp2(m2 - M), f3 = fast_exp2(m3 - M);
            av = f0 * S.acc[0][g][ch] + f1 * S.acc[1][g][ch] + f2 * S.acc[2][g][ch] + f3 * S.acc[3][g][ch];
            l = f0 * S.l[0][g] + f1 * S.l[1][g] + f2 * S.l[2][g] + f3 * S.l[3][g];
        }
        if (final) {
            const float o = l > 0.f ? av / l : 0.f;
            out[i] = (uint16_t)f32_to_bf16(o);
            if (out_f32) out_f32[i] = o;
        } else {
            float* pp = part + g * head_stride;
            st_dev(pp + 2 + ch, av);
            if (ch == 0) { st_dev(pp, M); st_dev(pp + 1, l); }
        }
    }
}

// Merge ns slices (written by other workgroups of this launch with attn_emit) into the output of
// the HT heads: part0 = partial of head 0, slice 0; slices are HATA_PSTRIDE apart, heads
// head_stride apart.  Every load is issued before the first wait: the (max, sum) pairs of the heads
// a wave prepares, then the first 16-32 slices of each thread's NO output channels (later slices batch
// by batch); one wave per head turns the pairs into normalised weights in LDS (S.acc is reused;
// ns <= 256).
// Must be called by all 256 threads, after a barrier that follows the last use of S.
template <int HT, int NJ>
__device__ __forceinline__ void attn_merge_nj(
    AttnLds<HT>& S, const float* __restrict__ part0, int64_t head_stride, int ns,
    uint16_t* __restrict__ out, float* __restrict__ out_f32) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NO = (HT * HATA_D + 255) / 256;  // outputs (head, channel) per thread
    constexpr int HPW = (HT + 3) / 4;              // heads whose weights one wave prepares
    float* sm_w = &S.acc[0][0][0];                 // [HT][nsp]
    const int nsp = (ns + 3) & ~3;
    // the (max, sum) pairs first -- they head the longest dependent chain -- lane l takes slices
    // l, l + 64, ... (ns <= 256)
    float mv[HPW][4], lv[HPW][4];
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
        const float* pp = part0 + min(wave + 4 * hh, HT - 1) * head_stride;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            mv[hh][t] = HATA_NEG_INF;
            lv[hh][t] = 0.f;
            if (t * 64 < ns) {
                const int s2 = min(lane + 64 * t, ns - 1);
                mv[hh][t] = ld_dev(pp + (int64_t)s2 * HATA_PSTRIDE);
                lv[hh][t] = ld_dev(pp + (int64_t)s2 * HATA_PSTRIDE + 1);
            }
        }
    }
    // first NJ slices of every output of this thread, all loads in flight
    float av[NO][NJ];
#pragma unroll
    for (int r = 0; r < NO; ++r) {
        const int i = min(tid + 256 * r, HT * HATA_D - 1);
        const int g = i / HATA_D, ch = i % HATA_D;
        const float* pp = part0 + g * head_stride + 2 + ch;
#pragma unroll
        for (int j = 0; j < NJ; ++j) av[r][j] = (j < ns) ? ld_dev(pp + (int64_t)j * HATA_PSTRIDE) : 0.f;
    }
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
        const int g = wave + 4 * hh;
        if (g < HT) {
            float m_loc = HATA_NEG_INF;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (lane + 64 * t >= ns) { mv[hh][t] = HATA_NEG_INF; lv[hh][t] = 0.f; }
                m_loc = fmaxf(m_loc, mv[hh][t]);
            }
            const float M = wave_max64(m_loc);
            float wt[4], l_loc = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                wt[t] = (mv[hh][t] == HATA_NEG_INF) ? 0.f : fast_exp2(mv[hh][t] - M);
                l_loc = fmaf(wt[t], lv[hh][t], l_loc);
            }
            const float Lsum = wave_sum64(l_loc);
            const float inv = Lsum > 0.f ? 1.f / Lsum : 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (lane + 64 * t < nsp) sm_w[g * nsp + lane + 64 * t] = wt[t] * inv;  // 0 past ns
        }
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
            for (int j4 = 0; j4 < NJ / 4; ++j4) {
                if (j4 * 4 < nsp) {  // weights of slices >= ns are zero
                    const float4 w = w4[j4];
                    A = fmaf(w.x, av[r][4 * j4], A); A = fmaf(w.y, av[r][4 * j4 + 1], A);
                    A = fmaf(w.z, av[r][4 * j4 + 2], A); A = fmaf(w.w, av[r][4 * j4 + 3], A);
                }
            }
            const float* pp = part0 + g * head_stride + 2 + ch;
            for (int s0 = NJ; s0 < ns; s0 += 16) {
                float bv[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) bv[j] = (s0 + j < ns) ? ld_dev(pp + (int64_t)(s0 + j) * HATA_PSTRIDE) : 0.f;
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (s0 + j < ns) A = fmaf(sm_w[g * nsp + s0 + j], bv[j], A);
            }
            out[i] = (uint16_t)f32_to_bf16(A);
            if (out_f32) out_f32[i] = A;
        }
    }
}

// The same merge for ONE head by a whole workgroup (the heads of a unit can then be merged by
// different workgroups side by side).  pp = the head's partial of slice 0; thread -> (channel
// tid % 128, slices of parity tid / 128), so 2 * NJ slices are in flight at once; the two halves
// meet in LDS.  sm: 384 floats of LDS nobody else uses until the call returns.  Must be called by
// all 256 threads, after a barrier that follows the last use of sm.
template <int NJ>
__device__ __forceinline__ void attn_merge_head(
    float* __restrict__ sm, const float* __restrict__ pp, int ns, uint16_t* __restrict__ out,
    float* __restrict__ out_f32) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ch = tid & 127, par = tid >> 7;
    float* sm_w = sm;           // [256] normalised slice weights (ns <= 256)
    float* sm_half = sm + 256;  // [128] the odd slices' sums
    float mv[4], lv[4];
    if (wave == 0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            mv[t] = HATA_NEG_INF;
            lv[t] = 0.f;
            if (t * 64 < ns) {
                const int s2 = min(lane + 64 * t, ns - 1);
                mv[t] = ld_dev(pp + (int64_t)s2 * HATA_PSTRIDE);
                lv[t] = ld_dev(pp + (int64_t)s2 * HATA_PSTRIDE + 1);
            }
        }
    }
    const float* pc = pp + 2 + ch;
    float av[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int s2 = par + 2 * j;
        av[j] = (s2 < ns) ? ld_dev(pc + (int64_t)s2 * HATA_PSTRIDE) : 0.f;
    }
    if (wave == 0) {
        float m_loc = HATA_NEG_INF;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (lane + 64 * t >= ns) { mv[t] = HATA_NEG_INF; lv[t] = 0.f; }
            m_loc = fmaxf(m_loc, mv[t]);
        }
        const float M = wave_max64(m_loc);
        float wt[4], l_loc = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            wt[t] = (mv[t] == HATA_NEG_INF) ? 0.f : fast_exp2(mv[t] - M);
            l_loc = fmaf(wt[t], lv[t], l_loc);
        }
        const float Lsum = wave_sum64(l_loc);
        const float inv = Lsum > 0.f ? 1.f / Lsum : 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) sm_w[lane + 64 * t] = wt[t] * inv;  // 0 past ns
    }
    __syncthreads();
    float A = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; ++j) A = fmaf(sm_w[min(par + 2 * j, 255)], av[j], A);  // (av is 0 past ns)
    for (int s0 = 2 * NJ; s0 < ns; s0 += 2 * NJ) {
        float bv[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int s2 = s0 + par + 2 * j;
            bv[j] = (s2 < ns) ? ld_dev(pc + (int64_t)s2 * HATA_PSTRIDE) : 0.f;
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) A = fmaf(sm_w[min(s0 + par + 2 * j, 255)], bv[j], A);
    }
    if (par) sm_half[ch] = A;
    __syncthreads();
    if (!par) {
        A += sm_half[ch];
        out[ch] = (uint16_t)f32_to_bf16(A);
        if (out_f32) out_f32[ch] = A;
    }
}

// NJ (slices whose loads are in flight together) by the number of slices: a second batch costs a
// memory round trip, registers bound the first (80 per thread at most)
template <int HT>
__device__ __forceinline__ void attn_merge(
    AttnLds<HT>& S, const float* __restrict__ part0, int64_t head_stride, int ns,
    uint16_t* __restrict__ out, float* __restrict__ out_f32) {
    constexpr int NO = (HT * HATA_D + 255) / 256;
    constexpr int NJ_BIG = NO <= 2 ? 32 : (NO <= 4 ? 20 : 16);
    if (NJ_BIG > 16 && ns > 16) attn_merge_nj<HT, NJ_BIG>(S, part0, head_stride, ns, out, out_f32);
    else attn_merge_nj<HT, 16>(S, part0, head_stride, ns, out, out_f32);
}

}  // namespace hata
