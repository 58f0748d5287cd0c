// HashEncode kernels (Alg. 2 of the paper): codes = BitPack(Sign(x . W_H)).
//
//   encode_vectors_kernel  one workgroup per vector (query heads, appended keys);
//                          fp64 accumulation, so the sign agrees with an exact
//                          evaluation unless |projection| is below ~1e-13.
//   encode_bulk_kernel     64 keys per workgroup, fp32 accumulation (prefill, the key-code fill of Alg. 1).
#include "hata_device.h"
#include "hata_internal.h"

namespace hata {

// Bit j of a code goes to word j/32, bit position j%32; bit = (projection >= 0).
// 1024 threads = (column j, part p): every thread sums 128 / parts channels with all its W_H
// loads in flight at once, so the kernel costs about one memory round trip.
#define HATA_ENC_THREADS 1024
__global__ __launch_bounds__(HATA_ENC_THREADS) void encode_vectors_kernel(
    const uint16_t* __restrict__ q, uint32_t* __restrict__ qcodes, int nq_blocks,
    const uint16_t* __restrict__ K, const int32_t* __restrict__ start,
    const int32_t* __restrict__ n_new, int max_new, int from_seq_len,
    uint32_t* __restrict__ codes, const float* __restrict__ W_H,
    int Hq, int Hkv, int G, int r, int Wd, int L_cap,
    int64_t sb, int64_t sh, int64_t sn) {
    __shared__ float xs[HATA_D];
    __shared__ double part[HATA_ENC_THREADS];
    const int tid = threadIdx.x;
    int blk = blockIdx.x;
    const uint16_t* x;
    uint32_t* dst;
    int h;
    if (blk < nq_blocks) {
        const int hq = blk % Hq;
        h = hq / G;
        x = q + (int64_t)blk * HATA_D;
        dst = qcodes + (int64_t)blk * Wd;
    } else {
        blk -= nq_blocks;
        const int t = blk % max_new;
        const int u = blk / max_new;
        const int b = u / Hkv;
        h = u % Hkv;
        int n, cnt;
        if (from_seq_len) { n = start[b] - 1; cnt = 1; }
        else { n = start[b] + t; cnt = n_new[b]; }
        if (t >= cnt || n < 0 || n >= L_cap) return;  // uniform over the workgroup
        x = K + b * sb + h * sh + n * sn;
        dst = codes + ((int64_t)u * L_cap + n) * Wd;
    }
    const int parts = HATA_ENC_THREADS / r;       // r <= 256 -> parts >= 4
    const int per = (HATA_D + parts - 1) / parts; // channels per part (<= 32)
    const int j = tid % r, p = tid / r;
    // issue the weight loads before waiting for x
    float wv[32];
    const int i0 = p * per;
    const bool active = p < parts;
    {
        const float* w = W_H + (int64_t)h * HATA_D * r + j;
#pragma unroll
        for (int t = 0; t < 32; ++t)
            wv[t] = (active && t < per && i0 + t < HATA_D) ? w[(int64_t)(i0 + t) * r] : 0.f;
    }
    if (tid < HATA_D) xs[tid] = __uint_as_float((uint32_t)x[tid] << 16);
    __syncthreads();
    double acc = 0.0;
#pragma unroll
    for (int t = 0; t < 32; ++t)
        if (t < per && i0 + t < HATA_D) acc += (double)xs[i0 + t] * (double)wv[t];
    part[tid] = acc;
    __syncthreads();
    bool bit = false;
    if (tid < r) {
        double y = 0.0;
        for (int pp = 0; pp < parts; ++pp) y += part[pp * r + tid];
        bit = (y >= 0.0);
    }
    const unsigned long long mask = __ballot(bit);
    const int wave = tid >> 6;
    if ((tid & 63) == 0 && wave * 64 < r) {
        dst[2 * wave] = (uint32_t)mask;
        if (2 * wave + 1 < Wd) dst[2 * wave + 1] = (uint32_t)(mask >> 32);
    }
}

// One workgroup per (sequence, KV head) unit: the G query heads of the group and, optionally,
// the key appended in this step share one pass over W_H[h] (each weight is loaded once and used
// for every vector).  1024 threads = (column j, part p); fp64 accumulation; the partial sums of
// the parts are combined in a fixed order, so the result is deterministic.
// grid = B * Hkv.  R = hash bits (128 or 256).
template <int R>
__global__ __launch_bounds__(HATA_ENC_THREADS) void encode_unit_kernel(
    const uint16_t* __restrict__ q, uint32_t* __restrict__ qcodes,
    const uint16_t* __restrict__ K, const int32_t* __restrict__ seq_len, int append,
    uint32_t* __restrict__ codes, const float* __restrict__ W_H,
    int Hq, int Hkv, int G, int L_cap, int64_t sb, int64_t sh, int64_t sn) {
    constexpr int PARTS = HATA_ENC_THREADS / R;
    constexpr int PER = HATA_D / PARTS;
    constexpr int WD = R / 32;
    constexpr int VG = 4;  // vectors reduced per round
    __shared__ float xs[17][HATA_D];
    __shared__ double part[PARTS][VG][R];
    const int tid = threadIdx.x;
    const int u = blockIdx.x;
    const int b = u / Hkv, h = u % Hkv;
    const int j = tid % R, p = tid / R;
    // weights first: PER independent loads per thread
    float wv[PER];
    {
        const float* w = W_H + (int64_t)h * HATA_D * R + (int64_t)p * PER * R + j;
#pragma unroll
        for (int t = 0; t < PER; ++t) wv[t] = w[(int64_t)t * R];
    }
    int n_key = -1;
    if (append) {
        n_key = seq_len[b] - 1;
        if (n_key < 0 || n_key >= L_cap) n_key = -1;
    }
    const int nv = G + (n_key >= 0 ? 1 : 0);
    for (int i = tid; i < nv * HATA_D; i += HATA_ENC_THREADS) {
        const int v = i / HATA_D, ch = i % HATA_D;
        const uint16_t* x = (v < G) ? q + ((int64_t)b * Hq + (int64_t)h * G + v) * HATA_D
                                    : K + b * sb + h * sh + (int64_t)n_key * sn;
        xs[v][ch] = __uint_as_float((uint32_t)x[ch] << 16);
    }
    __syncthreads();
    for (int v0 = 0; v0 < nv; v0 += VG) {
        double acc[VG];
#pragma unroll
        for (int i = 0; i < VG; ++i) acc[i] = 0.0;
#pragma unroll
        for (int t = 0; t < PER; ++t) {
            const double wd = (double)wv[t];
#pragma unroll
            for (int i = 0; i < VG; ++i)  // rows past nv are read (stale LDS) but never used
                acc[i] += (double)xs[min(v0 + i, 16)][p * PER + t] * wd;
        }
#pragma unroll
        for (int i = 0; i < VG; ++i) part[p][i][j] = acc[i];
        __syncthreads();
        if (tid < VG * R) {
            const int i = tid / R;  // uniform over a wave (R >= 64)
            const int v = v0 + i;
            double y = 0.0;
#pragma unroll
            for (int pp = 0; pp < PARTS; ++pp) y += part[pp][i][j];
            const unsigned long long mask = __ballot(y >= 0.0);
            if ((tid & 63) == 0 && v < nv) {
                uint32_t* dst = (v < G) ? qcodes + ((int64_t)b * Hq + (int64_t)h * G + v) * WD
                                        : codes + ((int64_t)u * L_cap + n_key) * WD;
                const int w0 = (j >> 6) * 2;
                dst[w0] = (uint32_t)mask;
                dst[w0 + 1] = (uint32_t)(mask >> 32);
            }
        }
        __syncthreads();
    }
}

// 64 keys per workgroup; thread = (key, word group).  The word group is uniform over a
// wave, so the W_H reads are wave-uniform.  grid = (tiles, Hkv, B).
__global__ __launch_bounds__(256) void encode_bulk_kernel(
    const uint16_t* __restrict__ K, const float* __restrict__ W_H,
    const int32_t* __restrict__ start, const int32_t* __restrict__ n_new,
    uint32_t* __restrict__ codes, int Hkv, int r, int Wd, int L_cap,
    int64_t sb, int64_t sh, int64_t sn) {
    __shared__ float xs[64][HATA_D + 1];
    const int tid = threadIdx.x;
    const int h = blockIdx.y, b = blockIdx.z;
    const int first = start[b];
    const int cnt = n_new[b];
    const int t0 = blockIdx.x * 64;
    if (t0 >= cnt) return;
    const int64_t u = (int64_t)b * Hkv + h;
    // stage the tile: 16 lanes per row, 16 B (8 bf16) per lane
    for (int it = 0; it < 4; ++it) {
        const int row = it * 16 + (tid >> 4);
        const int n = first + t0 + row;
        const int sub = tid & 15;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (t0 + row < cnt && n >= 0 && n < L_cap)
            v = *reinterpret_cast<const uint4*>(K + b * sb + h * sh + (int64_t)n * sn + sub * 8);
        float* dstp = &xs[row][sub * 8];
        dstp[0] = bf16_lo(v.x); dstp[1] = bf16_hi(v.x);
        dstp[2] = bf16_lo(v.y); dstp[3] = bf16_hi(v.y);
        dstp[4] = bf16_lo(v.z); dstp[5] = bf16_hi(v.z);
        dstp[6] = bf16_lo(v.w); dstp[7] = bf16_hi(v.w);
    }
    __syncthreads();
    const int key = tid & 63;
    const int n = first + t0 + key;
    const bool live = (t0 + key < cnt) && n >= 0 && n < L_cap;
    const int wg = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int w = wg; w < Wd; w += 4) {
        float acc[32];
#pragma unroll
        for (int c = 0; c < 32; ++c) acc[c] = 0.f;
        const float* wp = W_H + (int64_t)h * HATA_D * r + w * 32;
        for (int i = 0; i < HATA_D; ++i) {
            const float xv = xs[key][i];
#pragma unroll
            for (int c = 0; c < 32; ++c) acc[c] = fmaf(xv, wp[(int64_t)i * r + c], acc[c]);
        }
        uint32_t word = 0;
#pragma unroll
        for (int c = 0; c < 32; ++c) word |= (acc[c] >= 0.f ? 1u : 0u) << c;
        if (live) codes[(u * L_cap + n) * Wd + w] = word;
    }
}

// ---------------------------------------------------------------------------------------
// Prefill key-code writer on the matrix cores (Alg. 1: K_H = HashEncode(K) during the prefill).
//
// The projection [keys, 128] x [128, r] is a dense contraction, so it runs on MFMA
// (v_mfma_f32_32x32x16_bf16).  K is bf16 already; the fp32 weights are split exactly into
// three bf16 planes (hi + mid + lo carries all 24 mantissa bits), every bf16 x bf16 product is
// exact in fp32, and only the fp32 accumulation rounds (~1e-6 relative) -- which is what keeps
// the sign bits equal to an exact evaluation outside a |projection| < ~1e-5 band.
//
// Mapping: M = 32 hash columns (wave w owns columns [32 w, 32 w + 32), i.e. code word w),
// N = 32 keys, K = channels.  A wave keeps its weight fragments (3 planes x 8 channel steps) in
// registers for the whole launch; key rows are staged through LDS 128 at a time with coalesced
// 128-bit loads (next stage prefetched into registers) and read back in the operand layout
// (lane = key, 16 B of consecutive channels).  In the 32x32 result a lane holds 16 hash columns of
// ONE key, so the sign bits are packed inside the lane and joined with the other half-wave.
// grid = (key blocks, Hkv, B); R / 32 waves per workgroup (r = 32, 64, 128 or 256).
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
#define HATA_MFMA_PITCH 136   // LDS row pitch in bf16 elements (272 B: rows shift by 4 banks)


// fp32 weight pair -> the three bf16 planes (hi, mid, lo) whose sum is the weight exactly; two weights per dword
__device__ __forceinline__ void split_weight_pair(float w0, float w1, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    uint32_t ph[2], pm[2], pl[2];
    const float wv2[2] = {w0, w1};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const float wv = wv2[q];
        ph[q] = f32_to_bf16(wv);
        const float r1 = wv - __uint_as_float(ph[q] << 16);
        pm[q] = f32_to_bf16(r1);
        const float r2 = r1 - __uint_as_float(pm[q] << 16);
        pl[q] = f32_to_bf16(r2);
    }
    hi = ph[0] | (ph[1] << 16);
    mid = pm[0] | (pm[1] << 16);
    lo = pl[0] | (pl[1] << 16);
}

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;

// eight bf16 values (one 16-byte operand fragment) -> fp16
__device__ __forceinline__ f16x8_t bf16x8_to_f16(const uint4 v) {
    const uint32_t x[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_lo(x[i]), bf16_hi(x[i])));
    return __builtin_bit_cast(f16x8_t, make_uint4(o[0], o[1], o[2], o[3]));
}

// PRESPLIT: the weights come from the planes hata_prepare_weights made, and they are the two scaled
// fp16 planes described at encode_dma_kernel below (two MFMAs per fragment instead of three; the key
// fragments are converted to fp16 on their way from LDS)
template <int R, bool PAGED, bool PRESPLIT>
__global__ __launch_bounds__(R * 2) void encode_mfma_kernel(
    const uint16_t* __restrict__ K, const float* __restrict__ W_H, const uint4* __restrict__ planes,
    const int32_t* __restrict__ start, const int32_t* __restrict__ n_new,
    uint32_t* __restrict__ codes, int Hkv, int L_cap, int keys_per_wg,
    int64_t sb, int64_t sh, int64_t sn,
    // fused cache fill (all null otherwise): the keys are read from K_new [B, Hkv, max_new, d] and
    // written to the cache K as they pass through; V_new is copied to V alongside
    const uint16_t* __restrict__ K_new, const uint16_t* __restrict__ V_new,
    uint16_t* __restrict__ K_out, uint16_t* __restrict__ V_out, int max_new,
    // block table of the destination (PAGED instantiation, fused fill only).  Paged pools are
    // [n_pages, Hkv, page_rows, d] / [n_pages, Hkv, page_rows, WD].
    const PageView pv) {
    constexpr int THREADS = R * 2;
    constexpr int WD = R / 32;
    constexpr int STAGE = R >= 64 ? 128 : 64;              // keys per LDS stage
    constexpr int NT = STAGE / 32;                         // 32-key MFMA tiles per stage
    constexpr int ROWS_PER_IT = THREADS / 16;              // rows staged per load instruction
    constexpr int NIT = STAGE / ROWS_PER_IT;               // load instructions per stage and thread
    __shared__ __attribute__((aligned(16))) uint16_t tile[STAGE * HATA_MFMA_PITCH];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 31, half = lane >> 5;
    const int h = blockIdx.y, b = blockIdx.z;
    const int first = start[b];
    constexpr bool paged = PAGED;
    int cnt = min(n_new[b], (paged ? min(L_cap, pv.max_blocks << pv.shift) : L_cap) - first);
    if (K_new != nullptr) cnt = min(cnt, max_new);  // the source holds max_new rows per unit
    const int kb0 = blockIdx.x * keys_per_wg;
    if (first < 0 || kb0 >= cnt) return;
    const int kb1 = min(kb0 + keys_per_wg, cnt);
    const int64_t u = (int64_t)b * Hkv + h;
    const uint16_t* Kb = K + b * sb + h * sh + (int64_t)first * sn;
    uint32_t* cb = codes + (u * L_cap + first) * WD;
    const bool fill = K_new != nullptr;
    const uint16_t* Ksrc = fill ? K_new + u * (int64_t)max_new * HATA_D : nullptr;
    const uint16_t* Vsrc = fill ? V_new + u * (int64_t)max_new * HATA_D : nullptr;
    uint16_t* Kdst = fill ? K_out + b * sb + h * sh + (int64_t)first * sn : nullptr;
    uint16_t* Vdst = fill ? V_out + b * sb + h * sh + (int64_t)first * sn : nullptr;
    // paged destination: row (first + key) of sequence b -> row of the pools, in rows of one head
    auto pool_row = [&](int key) -> int64_t {
        const int n = first + key;
        const int p = clampi(pv.table[(int64_t)b * pv.max_blocks + (n >> pv.shift)], 0, pv.n_pages - 1);
        return (((int64_t)p * Hkv + h) << pv.shift) + (n & ((1 << pv.shift) - 1));
    };

    // stage loader: thread -> (row = it * ROWS_PER_IT + tid / 16, 16-byte piece tid % 16)
    const int lrow = tid >> 4, lsub = tid & 15;
    uint4 pre[NIT];
    auto load_stage = [&](int k0) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int key = k0 + it * ROWS_PER_IT + lrow;
            pre[it] = make_uint4(0, 0, 0, 0);
            if (key < kb1) {
                if (fill) {
                    pre[it] = *reinterpret_cast<const uint4*>(Ksrc + (int64_t)key * HATA_D + lsub * 8);
                    const uint4 vv = *reinterpret_cast<const uint4*>(Vsrc + (int64_t)key * HATA_D + lsub * 8);
                    if constexpr (paged) {
                        const int64_t o = pool_row(key) * HATA_D + lsub * 8;
                        *reinterpret_cast<uint4*>(K_out + o) = pre[it];
                        *reinterpret_cast<uint4*>(V_out + o) = vv;
                    } else {
                        *reinterpret_cast<uint4*>(Kdst + (int64_t)key * sn + lsub * 8) = pre[it];
                        *reinterpret_cast<uint4*>(Vdst + (int64_t)key * sn + lsub * 8) = vv;
                    }
                } else {
                    pre[it] = *reinterpret_cast<const uint4*>(Kb + (int64_t)key * sn + lsub * 8);
                }
            }
        }
    };
    // the first stage of keys is on its way while the weight fragments arrive
    load_stage(kb0);

    // weight fragments: a[plane][kk] holds W_H[h][kk*16 + 8*half + e][32 w + m], e = 0..7
    bf16x8_t afrag[PRESPLIT ? 1 : 3][PRESPLIT ? 1 : 8];
    f16x8_t afrag16[PRESPLIT ? 2 : 1][PRESPLIT ? 8 : 1];
    if constexpr (PRESPLIT) {
        // prepared once per weight tensor (hata_prepare_weights): 16 coalesced 16-byte loads
        const uint4* src = planes + ((int64_t)(h * (R / 32) + w) * 8 * 2) * 64 + lane;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int p = 0; p < 2; ++p) afrag16[p][kk] = __builtin_bit_cast(f16x8_t, src[(kk * 2 + p) * 64]);
    } else {
        const float* wp = W_H + (int64_t)h * HATA_D * R + w * 32 + m;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            uint32_t hi[4], mid[4], lo[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2)
                split_weight_pair(wp[(int64_t)(kk * 16 + 8 * half + 2 * e2) * R],
                                  wp[(int64_t)(kk * 16 + 8 * half + 2 * e2 + 1) * R], hi[e2], mid[e2], lo[e2]);
            afrag[0][kk] = __builtin_bit_cast(bf16x8_t, make_uint4(hi[0], hi[1], hi[2], hi[3]));
            afrag[1][kk] = __builtin_bit_cast(bf16x8_t, make_uint4(mid[0], mid[1], mid[2], mid[3]));
            afrag[2][kk] = __builtin_bit_cast(bf16x8_t, make_uint4(lo[0], lo[1], lo[2], lo[3]));
        }
    }
    for (int k0 = kb0; k0 < kb1; k0 += STAGE) {
        __syncthreads();  // the previous stage has been consumed
#pragma unroll
        for (int it = 0; it < NIT; ++it)
            *reinterpret_cast<uint4*>(&tile[(it * ROWS_PER_IT + lrow) * HATA_MFMA_PITCH + lsub * 8]) = pre[it];
        __syncthreads();
        if (k0 + STAGE < kb1) load_stage(k0 + STAGE);  // overlaps the MFMAs below

        f32x16_t acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
        // Key fragments come from LDS one channel step ahead: as soon as the three planes of a tile
        // have been issued for step kk, the tile's fragment for step kk + 1 is requested into the same
        // registers, so its LDS latency is covered by the nine MFMAs of the other tiles.
        uint4 bfrag[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
            bfrag[t] = *reinterpret_cast<const uint4*>(&tile[(t * 32 + m) * HATA_MFMA_PITCH + 8 * half]);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if constexpr (PRESPLIT) {
                    const f16x8_t b16 = bf16x8_to_f16(bfrag[t]);
#pragma unroll
                    for (int p = 0; p < 2; ++p)
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afrag16[p][kk], b16, acc[t], 0, 0, 0);
                } else {
#pragma unroll
                    for (int p = 0; p < 3; ++p)
                        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[p][kk], __builtin_bit_cast(bf16x8_t, bfrag[t]), acc[t], 0, 0, 0);
                }
                if (kk + 1 < 8)
                    bfrag[t] = *reinterpret_cast<const uint4*>(
                        &tile[(t * 32 + m) * HATA_MFMA_PITCH + (kk + 1) * 16 + 8 * half]);
            }
        }
        // sign bits: this lane holds hash columns 8*(i/4) + 4*half + i%4 of key t*32 + m
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            // (the bit is "projection >= 0": the complement of the sign bit; a sum of exact products
            // that starts from +0 is never -0)
            uint32_t neg = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                neg |= (__float_as_uint(acc[t][i]) >> 31) << (8 * (i / 4) + (i % 4));
            uint32_t word = (~neg & 0x0f0f0f0fu) << (4 * half);
            word |= (uint32_t)__shfl_xor((int)word, 32, 64);
            const int key = k0 + t * 32 + m;
            if (half == 0 && key < kb1) {
                if constexpr (paged) codes[pool_row(key) * WD + w] = word;
                else cb[(int64_t)key * WD + w] = word;
            }
        }
    }
}

// ---- key encode with fp16 weight planes -------------------------------------------------------
// The projection for keys that already lie in a contiguous cache (no fused fill), with weights
// prepared by hata_prepare_weights.  Two things differ from encode_mfma_kernel.
//
// (1) Two fp16 planes instead of three bf16 planes.  With realistic operand values the matrix cores
// of the whole chip sustain about 55 cycles per v_mfma_f32_32x32x16 and SIMD, not 32 (measured with a
// loop of nothing but MFMAs: the rate depends on the values, i.e. on power), and the three-plane kernel's
// stage loop runs at exactly that rate -- so what shortens the kernel is fewer MFMAs.  Per hash-column
// tile (32 columns) the weights are scaled by a power of two S so that max |W S| < 2^14 (signs and
// therefore code bits are unchanged), hi = fp16(W S), lo = fp16(W S - hi): |W S - hi - lo| <= 2^-22 |W S|.
// A bf16 key channel converts to fp16 exactly for 2^-14 <= |x| <= 65504 (eight significant bits);
// smaller values lose at most 2^-25 absolutely, larger ones saturate at 65504.  Every product of two
// fp16 values is exact in the fp32 accumulator.  The projection therefore differs from the exact one by
// at most 2^-22 * sum_c |x_c W_c| (about 5e-6 for the workloads here) plus the fp32 summation error the
// bf16 form has as well: far inside the band of 1e-4 in which code bits may differ from an exact evaluation.
//
// (2) The key rows are staged by the memory pipeline itself: global_load_lds_dwordx4 moves 16 bytes
// per lane from memory straight into LDS (lane l of a wave lands at the instruction's LDS base + 16 l),
// so a stage costs no registers and several stages can be on their way while one is being multiplied.
// A workgroup cycles through DMA_NBUF tiles of DMA_STAGE keys: in turn s it waits for tile s, passes the
// one barrier of the turn, requests tile s + DMA_NBUF - 1 into the buffer that turn s - 1 has just
// finished with, and multiplies tile s.
// LDS tile: row r at byte 256 r, unpadded; its 16-byte piece c sits in slot c ^ (r & 15), which makes
// the operand reads (32 rows, one piece index) conflict-free.  A lane of a DMA instruction therefore
// fetches piece slot ^ (row & 15) of its row: 16 lanes still read one whole 256-byte row.
// Every wave converts the key fragments it reads to fp16 itself (three VALU instructions per dword, in
// the shadow of the MFMAs).  The code words of a stage go through a small LDS array and leave as
// 16-byte stores one turn later.
#define DMA_STAGE 64
#define DMA_NBUF 4

// Fragment order of the fp16 planes: for KV head h, wave w (hash columns 32 w .. 32 w + 31), channel
// step kk and plane p (0 = hi, 1 = lo) the 64 lanes' 16-byte fragments lie one after the other:
//   uint4 index = (((h * (R / 32) + w) * 8 + kk) * 2 + p) * 64 + lane
// grid = (R / 32, Hkv); 64 threads: one wave scales and splits its 32 columns
__global__ __launch_bounds__(64) void split_weights_f16_kernel(const float* __restrict__ W_H, uint4* __restrict__ planes, int R) {
    const int lane = threadIdx.x, w = blockIdx.x, h = blockIdx.y;
    const int m = lane & 31, half = lane >> 5;
    const float* wp = W_H + (int64_t)h * HATA_D * R + w * 32 + m;
    float wv[8][8];
    float mx = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            wv[kk][e] = wp[(int64_t)(kk * 16 + 8 * half + e) * R];
            mx = fmaxf(mx, fabsf(wv[kk][e]));  // (fmaxf drops NaN)
        }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    int ex = 14;  // scale 1 for an all-zero or non-finite tile
    if (mx > 0.f && mx < __builtin_inff()) (void)frexpf(mx, &ex);  // mx = f 2^ex, 0.5 <= f < 1
    const int sh = 14 - ex;                                        // max |W| 2^sh < 2^14
    uint4* dst = planes + ((int64_t)(h * (R / 32) + w) * 8 * 2) * 64 + lane;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        f16x8_t hi, lo;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float ws = ldexpf(wv[kk][e], sh);
            hi[e] = (_Float16)ws;                 // round to nearest even
            lo[e] = (_Float16)(ws - (float)hi[e]);  // (the difference is exact in fp32)
        }
        dst[(kk * 2 + 0) * 64] = __builtin_bit_cast(uint4, hi);
        dst[(kk * 2 + 1) * 64] = __builtin_bit_cast(uint4, lo);
    }
}

template <int R>
__global__ __launch_bounds__(R * 2) void encode_dma_kernel(
    const uint16_t* __restrict__ K, const uint4* __restrict__ planes,
    const int32_t* __restrict__ start, const int32_t* __restrict__ n_new, uint32_t* __restrict__ codes,
    int Hkv, int L_cap, int keys_per_wg, int64_t sb, int64_t sh, int64_t sn) {
    constexpr int WAVES = R / 32, WD = R / 32;
    constexpr int NT = DMA_STAGE / 32;                 // 32-key MFMA tiles per stage
    constexpr int INSTR = DMA_STAGE / (WAVES * 4);     // DMA instructions per wave and stage (4 rows each)
    static_assert(INSTR >= 1 && INSTR * WAVES * 4 == DMA_STAGE, "a stage is a whole number of DMA instructions per wave");
    __shared__ __attribute__((aligned(16))) uint4 tile[DMA_NBUF][DMA_STAGE * 16];
    __shared__ __attribute__((aligned(16))) uint32_t cbuf[2][DMA_STAGE * WD];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m = lane & 31, half = lane >> 5;
    const int h = blockIdx.y, b = blockIdx.z;
    const int first = start[b];
    const int cnt = min(n_new[b], L_cap - first);
    const int kb0 = blockIdx.x * keys_per_wg;
    if (first < 0 || kb0 >= cnt) return;
    const int kb1 = min(kb0 + keys_per_wg, cnt);
    const int64_t u = (int64_t)b * Hkv + h;
    const uint16_t* Kb = K + b * sb + h * sh + (int64_t)first * sn;
    uint32_t* cb = codes + (u * L_cap + first) * WD;
    const int n_stages = (kb1 - kb0 + DMA_STAGE - 1) / DMA_STAGE;

    // rows past the end of the range are fetched from the range's last row (valid memory; their code
    // words are never stored)
    const int drow = lane >> 4, dslot = lane & 15;
    auto request = [&](int s) {
        const int k0 = kb0 + s * DMA_STAGE;
        uint4* dst = &tile[s % DMA_NBUF][0];
#pragma unroll
        for (int it = 0; it < INSTR; ++it) {
            const int r0 = (it * WAVES + w) * 4;
            const int row = r0 + drow;
            const int key = min(k0 + row, kb1 - 1);
            const uint16_t* g = Kb + (int64_t)key * sn + ((dslot ^ (row & 15)) * 8);
            // (written as an instruction: given the compiler's builtin for it, every later LDS read is
            // made to wait for ALL requests outstanding, which is the one thing this kernel must not do;
            // the waits are the explicit ones in the stage loop)
            const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
                (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(dst + r0 * 16));
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                         :: "s"(lds_base), "v"(g) : "memory", "m0");
        }
    };
    // weight fragments first (they are needed for as long as the kernel runs), then the first tiles
    f16x8_t afrag[2][8];
    {
        const uint4* src = planes + ((int64_t)(h * (R / 32) + w) * 8 * 2) * 64 + lane;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
#pragma unroll
            for (int p = 0; p < 2; ++p) afrag[p][kk] = __builtin_bit_cast(f16x8_t, src[(kk * 2 + p) * 64]);
    }
#pragma unroll
    for (int s = 0; s < DMA_NBUF - 1; ++s)
        if (s < n_stages) request(s);
    // the weight fragments are there before the loop starts (said explicitly, or the compiler guards
    // their every use inside the loop with a count of outstanding loads that fits the first turn only)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

    // 16-byte pieces of the previous stage's code words that this thread stores (none for most threads)
    constexpr int CODE_VEC = DMA_STAGE * WD / 4;
    auto flush_codes = [&](int s) {  // code words of stage s, staged in cbuf[s & 1]
        const int k0 = kb0 + s * DMA_STAGE;
        if constexpr (WD >= 4) {  // (a key's code is 16 bytes or more: every piece is aligned)
            if (tid < CODE_VEC && k0 + (tid * 4) / WD < kb1)
                reinterpret_cast<uint4*>(cb + (int64_t)k0 * WD)[tid] = reinterpret_cast<const uint4*>(&cbuf[s & 1][0])[tid];
        } else {
            if (tid < DMA_STAGE * WD && k0 + tid / WD < kb1) cb[(int64_t)k0 * WD + tid] = cbuf[s & 1][tid];
        }
    };
    for (int s = 0; s < n_stages; ++s) {
        // tile s has landed once at most the requests made after it are outstanding: those of the
        // DMA_NBUF - 2 tiles that follow (stores of code words, if any, only make this wait longer)
        if (s + DMA_NBUF - 2 < n_stages) __builtin_amdgcn_s_waitcnt(0x0F70 | (((DMA_NBUF - 2) * INSTR) & 15) | ((((DMA_NBUF - 2) * INSTR) >> 4) << 14));
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();  // every wave's part of tile s is there; everybody is done with tile s - 1
        if (s + DMA_NBUF - 1 < n_stages) request(s + DMA_NBUF - 1);
        if (s > 0) flush_codes(s - 1);
        const uint4* tl = &tile[s % DMA_NBUF][0];
        f32x16_t acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
        // Key fragments: the raw bf16 pieces are read from LDS two channel steps ahead and converted one
        // step ahead, so that neither the LDS latency nor the conversion stands in front of an MFMA (the
        // scheduler is told to keep the steps apart: left alone it moves each read down to its first use)
        auto piece = [&](int kk, int t) { return tl[(t * 32 + m) * 16 + ((2 * kk + half) ^ (m & 15))]; };
        uint4 raw[NT];
        f16x8_t bcur[NT], bnext[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) raw[t] = piece(0, t);
#pragma unroll
        for (int t = 0; t < NT; ++t) bcur[t] = bf16x8_to_f16(raw[t]);
#pragma unroll
        for (int t = 0; t < NT; ++t) raw[t] = piece(1, t);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            __builtin_amdgcn_sched_barrier(0);
            if (kk + 1 < 8) {
#pragma unroll
                for (int t = 0; t < NT; ++t) bnext[t] = bf16x8_to_f16(raw[t]);
            }
            if (kk + 2 < 8) {
#pragma unroll
                for (int t = 0; t < NT; ++t) raw[t] = piece(kk + 2, t);
            }
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(afrag[p][kk], bcur[t], acc[t], 0, 0, 0);
            // one MFMA, then a quarter of the step's conversions in its shadow
#pragma unroll
            for (int q = 0; q < 2 * NT; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);           // MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 12 / 2, 0);      // VALU
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < NT; ++t) bcur[t] = bnext[t];
        }
        // sign bits: this lane holds hash columns 8*(i/4) + 4*half + i%4 of key t*32 + m
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            uint32_t neg = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                neg |= (__float_as_uint(acc[t][i]) >> 31) << (8 * (i / 4) + (i % 4));
            uint32_t word = (~neg & 0x0f0f0f0fu) << (4 * half);
            word |= (uint32_t)__shfl_xor((int)word, 32, 64);
            if (half == 0) cbuf[s & 1][(t * 32 + m) * WD + w] = word;
        }
    }
    __syncthreads();
    flush_codes(n_stages - 1);
}

hipError_t launch_encode_vectors(const hata_ctx* c, const void* q, uint32_t* qcodes,
                                 const void* K, const int32_t* start, const int32_t* n_new,
                                 int max_new, int from_seq_len, uint32_t* codes,
                                 const float* W_H, int B, hipStream_t s) {
    const hata_config& f = c->cfg;
    // queries (+ the key at seq_len - 1) of a unit in one workgroup when a kernel for r exists
    if (q && (!K || from_seq_len) && c->G <= 16 && (f.r == 128 || f.r == 256)) {
        const int append = K ? 1 : 0;
        if (f.r == 128)
            hipLaunchKernelGGL((encode_unit_kernel<128>), dim3(B * f.Hkv), dim3(HATA_ENC_THREADS), 0, s,
                               (const uint16_t*)q, qcodes, (const uint16_t*)K, start, append, codes,
                               W_H, f.Hq, f.Hkv, c->G, f.L_cap, f.kv_stride_b, f.kv_stride_h,
                               f.kv_stride_n);
        else
            hipLaunchKernelGGL((encode_unit_kernel<256>), dim3(B * f.Hkv), dim3(HATA_ENC_THREADS), 0, s,
                               (const uint16_t*)q, qcodes, (const uint16_t*)K, start, append, codes,
                               W_H, f.Hq, f.Hkv, c->G, f.L_cap, f.kv_stride_b, f.kv_stride_h,
                               f.kv_stride_n);
        return hipGetLastError();
    }
    const int nq = q ? B * f.Hq : 0;
    const int nk = K ? B * f.Hkv * max_new : 0;
    if (nq + nk == 0) return hipSuccess;
    hipLaunchKernelGGL(encode_vectors_kernel, dim3(nq + nk), dim3(HATA_ENC_THREADS), 0, s,
                       (const uint16_t*)q, qcodes, nq, (const uint16_t*)K, start, n_new,
                       max_new > 0 ? max_new : 1, from_seq_len, codes, W_H, f.Hq, f.Hkv, c->G,
                       f.r, c->Wd, f.L_cap, f.kv_stride_b, f.kv_stride_h, f.kv_stride_n);
    return hipGetLastError();
}

hipError_t launch_encode_bulk(const hata_ctx* c, const void* K, const float* W_H,
                              const int32_t* start, const int32_t* n_new, int B, int max_new,
                              uint32_t* codes, hipStream_t s, const void* K_new, const void* V_new,
                              void* K_out, void* V_out, const PageView* pages) {
    const hata_config& f = c->cfg;
    const PageView pv = pages ? *pages : PageView{nullptr, 0, 0, 0};
    if (pages && !K_new) return hipErrorNotSupported;  // the block table addresses the fused fill only
    if (max_new <= 0 || B <= 0) return hipSuccess;
    const uint16_t* kn = (const uint16_t*)K_new;
    const uint16_t* vn = (const uint16_t*)V_new;
    uint16_t* ko = (uint16_t*)K_out;
    uint16_t* vo = (uint16_t*)V_out;
    if (f.r == 32 || f.r == 64 || f.r == 128 || f.r == 256) {
        // key blocks of 512..4096 keys: at least ~512 workgroups when the prefill is long enough
        int kpw = 4096;
        while (kpw > 512 && (int64_t)((max_new + kpw - 1) / kpw) * f.Hkv * B < 512) kpw >>= 1;
        const dim3 grid((max_new + kpw - 1) / kpw, f.Hkv, B);
        // the weight planes prepared for exactly this weight tensor, if any (hata_prepare_weights)
        const uint4* planes = (c->prepared_W_H == W_H && c->wplanes) ? (const uint4*)c->wplanes : nullptr;
        if (!kn && !pages && planes) {
            // keys already in a contiguous cache, weights prepared: the kernel that stages with LDS-direct loads
            const uint4* p16 = planes;
#define HATA_LAUNCH_DMA(R_)                                                                                   \
    hipLaunchKernelGGL((encode_dma_kernel<R_>), grid, dim3(R_ * 2), 0, s, (const uint16_t*)K, p16, start, n_new, \
                       codes, f.Hkv, f.L_cap, kpw, f.kv_stride_b, f.kv_stride_h, f.kv_stride_n)
            if (f.r == 32) HATA_LAUNCH_DMA(32);
            else if (f.r == 64) HATA_LAUNCH_DMA(64);
            else if (f.r == 128) HATA_LAUNCH_DMA(128);
            else HATA_LAUNCH_DMA(256);
#undef HATA_LAUNCH_DMA
            return hipGetLastError();
        }
#define HATA_LAUNCH_MFMA(R_, P_)                                                                           \
    do {                                                                                                   \
        if (planes)                                                                                        \
            hipLaunchKernelGGL((encode_mfma_kernel<R_, P_, true>), grid, dim3(R_ * 2), 0, s,               \
                               (const uint16_t*)K, W_H, planes, start, n_new, codes, f.Hkv, f.L_cap, kpw,  \
                               f.kv_stride_b, f.kv_stride_h, f.kv_stride_n, kn, vn, ko, vo, max_new, pv);  \
        else                                                                                               \
            hipLaunchKernelGGL((encode_mfma_kernel<R_, P_, false>), grid, dim3(R_ * 2), 0, s,              \
                               (const uint16_t*)K, W_H, planes, start, n_new, codes, f.Hkv, f.L_cap, kpw,  \
                               f.kv_stride_b, f.kv_stride_h, f.kv_stride_n, kn, vn, ko, vo, max_new, pv);  \
    } while (0)
        if (pages) {
            if (f.r == 32) HATA_LAUNCH_MFMA(32, true);
            else if (f.r == 64) HATA_LAUNCH_MFMA(64, true);
            else if (f.r == 128) HATA_LAUNCH_MFMA(128, true);
            else HATA_LAUNCH_MFMA(256, true);
        } else {
            if (f.r == 32) HATA_LAUNCH_MFMA(32, false);
            else if (f.r == 64) HATA_LAUNCH_MFMA(64, false);
            else if (f.r == 128) HATA_LAUNCH_MFMA(128, false);
            else HATA_LAUNCH_MFMA(256, false);
        }
#undef HATA_LAUNCH_MFMA
        return hipGetLastError();
    }
    if (kn) return hipErrorNotSupported;  // the fused cache fill exists for the MFMA widths only
    const int tiles = (max_new + 63) / 64;
    hipLaunchKernelGGL(encode_bulk_kernel, dim3(tiles, f.Hkv, B), dim3(256), 0, s,
                       (const uint16_t*)K, W_H, start, n_new, codes, f.Hkv, f.r, c->Wd, f.L_cap,
                       f.kv_stride_b, f.kv_stride_h, f.kv_stride_n);
    return hipGetLastError();
}

// Split of the fp32 hash weights into two scaled fp16 planes in the operand-fragment order of the key encoders
hipError_t launch_split_weights(const hata_ctx* c, const float* W_H, hipStream_t s) {
    const hata_config& f = c->cfg;
    hipLaunchKernelGGL(split_weights_f16_kernel, dim3(f.r / 32, f.Hkv), dim3(64), 0, s, W_H, (uint4*)c->wplanes, f.r);
    return hipGetLastError();
}

}  // namespace hata
