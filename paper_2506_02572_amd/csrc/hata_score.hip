// Hamming-score kernel (Alg. 3 of the paper: S = bitcount(xor(Q_H, K_H^cache)), summed
// over the query heads of a GQA group so that the group shares ONE pass over the codes).
//
// Bandwidth-bound streaming: each lane owns one cached key per iteration and pulls its
// whole packed code with 128-bit loads (a wave reads 1 KB or 2 KB of consecutive bytes);
// the G query codes are wave-uniform and sit in scalar registers.  Optionally the
// workgroup also histograms its chunk's scores in LDS and writes the histogram out, which
// is what the selection stage needs (a counting select over the <= G*r+1 score values).
// In the fused decode step (SELECT = true) the workgroup that scores the LAST chunk of a unit
// to finish goes on to compute the unit's selection threshold and the per-chunk output
// offsets, so no separate launch is needed for that.
#include "hata_device.h"
#include "hata_internal.h"
#include "hata_select.h"
#include "hata_trace.h"

namespace hata {

template <int WD>
struct CodeVec { uint32_t w[WD]; };

template <int WD>
__device__ __forceinline__ CodeVec<WD> load_code(const uint32_t* p) {
    CodeVec<WD> c;
    if constexpr (WD % 4 == 0) {
#pragma unroll
        for (int i = 0; i < WD / 4; ++i) {
            uint4 v = reinterpret_cast<const uint4*>(p)[i];
            c.w[4 * i] = v.x; c.w[4 * i + 1] = v.y; c.w[4 * i + 2] = v.z; c.w[4 * i + 3] = v.w;
        }
    } else if constexpr (WD % 2 == 0) {
#pragma unroll
        for (int i = 0; i < WD / 2; ++i) {
            uint2 v = reinterpret_cast<const uint2*>(p)[i];
            c.w[2 * i] = v.x; c.w[2 * i + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < WD; ++i) c.w[i] = p[i];
    }
    return c;
}

template <int WD, int G, bool SELECT>
__global__ __launch_bounds__(256) void score_kernel(
    const uint32_t* __restrict__ qcodes, const uint32_t* __restrict__ codes,
    const int32_t* __restrict__ seq_len, uint16_t* __restrict__ scores,
    uint16_t* __restrict__ chunk_hist, int Hq, int Hkv, int L_cap, int chunk, int n_chunks,
    int NB, int NBP, const int32_t* __restrict__ kbud, int k_max,
    int32_t* __restrict__ chunk_info, int32_t* __restrict__ unit_info,
    uint32_t* __restrict__ unit_counter, uint32_t* __restrict__ unit_hist) {
    extern __shared__ uint32_t hist[];  // NB bins when chunk_hist != nullptr
    __shared__ ThresholdLds S;
    __shared__ int last_flag;
    const int tid = threadIdx.x;
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    // wave-uniform query codes (as bit-count planes for the larger groups); their loads do not depend on
    // the sequence length and go out together with it
    constexpr bool PLANES = HammingSum<WD, G>::PLANES;
    HammingSum<WD, G> dist;
    uint32_t qc[PLANES ? 1 : G][WD];
    const uint32_t* qp = qcodes + ((int64_t)b * Hq + (int64_t)h * G) * WD;
    if constexpr (PLANES) {
        dist.init(qp);
    } else {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int w = 0; w < WD; ++w) qc[g][w] = __builtin_amdgcn_readfirstlane(qp[g * WD + w]);
    }
    const int L = clampi(seq_len[b], 0, L_cap);
    const int base = c * chunk;
    const int64_t u = (int64_t)b * Hkv + h;
    if (base >= L) {
        if (SELECT && L == 0 && c == 0 && tid == 0) {  // empty sequence: nothing selected
            unit_info[u * 2 + 0] = 0;
            unit_info[u * 2 + 1] = 0;
            chunk_info[u * (n_chunks + 1) * 2 + 0] = 0;
            chunk_info[u * (n_chunks + 1) * 2 + 1] = 0;
        }
        return;
    }
    const int end = min(base + chunk, L);
    HATA_TRACE_AT(0, SELECT && u == 0 && c == 0);
    const bool do_hist = chunk_hist != nullptr;
    if (do_hist) {
        for (int i = tid; i < NB; i += 256) hist[i] = 0;
        __syncthreads();
    }
    const uint32_t* cp = codes + u * L_cap * WD;
    uint16_t* sp = scores + u * L_cap;
    constexpr int UNR = (WD <= 4) ? 8 : 4;  // 128 B of codes in flight per lane (256 B measured: 0.3-1 us slower)
    for (int n0 = base + tid; n0 < end; n0 += 256 * UNR) {
        CodeVec<WD> kc[UNR];
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            const int n = n0 + j * 256;
            if (n < end) kc[j] = load_code<WD>(cp + (int64_t)n * WD);
        }
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            const int n = n0 + j * 256;
            if (n < end) {
                uint32_t s = 0;
                if constexpr (PLANES) {
                    s = dist(kc[j].w);
                } else {
#pragma unroll
                    for (int g = 0; g < G; ++g)
#pragma unroll
                        for (int w = 0; w < WD; ++w) s += __popc(qc[g][w] ^ kc[j].w[w]);
                }
                sp[n] = (uint16_t)s;
                if (do_hist) atomicAdd(&hist[s], 1u);
            }
        }
    }
    HATA_TRACE_AT(1, SELECT && u == 0 && c == 0);
    if (do_hist) {
        __syncthreads();
        write_chunk_hist(chunk_hist + (u * n_chunks + c) * NBP, hist, NB, NBP);
    }
    if constexpr (SELECT) {
        const int keff = min(clampi(kbud[b], 0, k_max), L);
        finish_unit(u, (L + chunk - 1) / chunk, keff, chunk_hist + u * n_chunks * NBP, NB, NBP,
                    n_chunks, chunk_info, unit_info, unit_counter, unit_hist, hist, S, &last_flag);
    }
}

// Generic fallback: any WD <= 8 and G <= 16, query codes in LDS.
__global__ __launch_bounds__(256) void score_kernel_generic(
    const uint32_t* __restrict__ qcodes, const uint32_t* __restrict__ codes,
    const int32_t* __restrict__ seq_len, uint16_t* __restrict__ scores,
    uint16_t* __restrict__ chunk_hist, int Hq, int Hkv, int G, int WD, int L_cap, int chunk,
    int n_chunks, int NB, int NBP, int select, const int32_t* __restrict__ kbud, int k_max,
    int32_t* __restrict__ chunk_info, int32_t* __restrict__ unit_info,
    uint32_t* __restrict__ unit_counter, uint32_t* __restrict__ unit_hist) {
    extern __shared__ uint32_t hist[];
    __shared__ uint32_t qc[16 * 8];
    __shared__ ThresholdLds S;
    __shared__ int last_flag;
    const int tid = threadIdx.x;
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = clampi(seq_len[b], 0, L_cap);
    const int base = c * chunk;
    const int64_t u = (int64_t)b * Hkv + h;
    if (base >= L) {
        if (select && L == 0 && c == 0 && tid == 0) {
            unit_info[u * 2 + 0] = 0;
            unit_info[u * 2 + 1] = 0;
            chunk_info[u * (n_chunks + 1) * 2 + 0] = 0;
            chunk_info[u * (n_chunks + 1) * 2 + 1] = 0;
        }
        return;
    }
    const int end = min(base + chunk, L);
    for (int i = tid; i < NB; i += 256) hist[i] = 0;
    if (tid < G * WD) qc[tid] = qcodes[((int64_t)b * Hq + (int64_t)h * G) * WD + tid];
    __syncthreads();
    const uint32_t* cp = codes + u * L_cap * WD;
    uint16_t* sp = scores + u * L_cap;
    for (int n = base + tid; n < end; n += 256) {
        uint32_t s = 0;
        for (int w = 0; w < WD; ++w) {
            const uint32_t kw = cp[(int64_t)n * WD + w];
            for (int g = 0; g < G; ++g) s += __popc(qc[g * WD + w] ^ kw);
        }
        sp[n] = (uint16_t)s;
        atomicAdd(&hist[s], 1u);
    }
    __syncthreads();
    write_chunk_hist(chunk_hist + (u * n_chunks + c) * NBP, hist, NB, NBP);
    if (select) {
        const int keff = min(clampi(kbud[b], 0, k_max), L);
        finish_unit(u, (L + chunk - 1) / chunk, keff, chunk_hist + u * n_chunks * NBP, NB, NBP,
                    n_chunks, chunk_info, unit_info, unit_counter, unit_hist, hist, S, &last_flag);
    }
}

template <int WD, int G>
static void launch_t(const hata_ctx* c, const uint32_t* qcodes, const uint32_t* codes,
                     const int32_t* seq_len, int B, uint16_t* scores, const int32_t* kbud,
                     hipStream_t s) {
    const hata_config& f = c->cfg;
    const size_t lds = (size_t)c->NB * 4;
    const dim3 grid(c->n_chunks, f.Hkv, B);
    if (kbud)
        hipLaunchKernelGGL((score_kernel<WD, G, true>), grid, dim3(256), lds, s, qcodes, codes,
                           seq_len, scores, c->chunk_hist, f.Hq, f.Hkv, f.L_cap, c->chunk,
                           c->n_chunks, c->NB, c->NBP, kbud, f.k_max, c->chunk_info,
                           c->unit_info, c->unit_counter, c->unit_hist);
    else
        hipLaunchKernelGGL((score_kernel<WD, G, false>), grid, dim3(256), lds, s, qcodes, codes,
                           seq_len, scores, c->chunk_hist, f.Hq, f.Hkv, f.L_cap, c->chunk,
                           c->n_chunks, c->NB, c->NBP, kbud, f.k_max, c->chunk_info,
                           c->unit_info, c->unit_counter, c->unit_hist);
}

// kbud == nullptr: scores (+ chunk histograms) only.  kbud != nullptr: the fused-step variant,
// which also leaves the unit thresholds and chunk offsets of the selection in the workspace.
hipError_t launch_score(const hata_ctx* c, const uint32_t* qcodes, const uint32_t* codes,
                        const int32_t* seq_len, int B, uint16_t* scores, const int32_t* kbud,
                        hipStream_t s) {
    const hata_config& f = c->cfg;
    const int key = c->Wd * 100 + c->G;
    switch (key) {
#define HATA_CASE(WD, GG) case WD * 100 + GG: launch_t<WD, GG>(c, qcodes, codes, seq_len, B, scores, kbud, s); break;
        HATA_CASE(4, 1) HATA_CASE(4, 2) HATA_CASE(4, 4) HATA_CASE(4, 5) HATA_CASE(4, 8)
        HATA_CASE(8, 1) HATA_CASE(8, 2) HATA_CASE(8, 4) HATA_CASE(8, 5) HATA_CASE(8, 8)
        HATA_CASE(2, 1) HATA_CASE(2, 2) HATA_CASE(2, 4) HATA_CASE(2, 5) HATA_CASE(2, 8)
        HATA_CASE(1, 1) HATA_CASE(1, 2) HATA_CASE(1, 4) HATA_CASE(1, 5) HATA_CASE(1, 8)
        HATA_CASE(1, 16) HATA_CASE(2, 16) HATA_CASE(4, 16) HATA_CASE(8, 16)
#undef HATA_CASE
        default:
            hipLaunchKernelGGL(score_kernel_generic, dim3(c->n_chunks, f.Hkv, B), dim3(256),
                               (size_t)c->NB * 4, s, qcodes, codes, seq_len, scores, c->chunk_hist,
                               f.Hq, f.Hkv, c->G, c->Wd, f.L_cap, c->chunk, c->n_chunks, c->NB,
                               c->NBP, kbud ? 1 : 0, kbud, f.k_max, c->chunk_info, c->unit_info,
                               c->unit_counter, c->unit_hist);
    }
    return hipGetLastError();
}

}  // namespace hata
