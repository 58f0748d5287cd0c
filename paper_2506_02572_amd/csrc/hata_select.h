// Device-side pieces of the selection stage (Alg. 3 of the paper: Idx = TopK(S, N)), shared by
// the stand-alone top-k kernels, the scoring kernel (which finishes a unit's threshold as soon
// as its last chunk is scored) and the fused select-and-attend kernel.
//
// Selection is a counting select over the <= G*r + 1 possible score values:
//   chunk histograms -> unit threshold T, ties still needed -> per-chunk output offsets,
// then an ordered compaction, so equal scores are granted in cache order (lower row wins)
// and the index list comes out ascending.  No atomic decides an output position.
#pragma once
#include "hata_device.h"

namespace hata {

#define HATA_MAX_CHUNKS 1024

// LDS a workgroup needs to run unit_threshold()
struct ThresholdLds {
    uint32_t scan4[4];
    int T, need;
    uint32_t c_lt[HATA_MAX_CHUNKS];
    uint32_t c_eq[HATA_MAX_CHUNKS];
};

// One workgroup of 256 threads computes, for unit u:
//   unit_info[u]       = {T, keff}: keys with score < T are all selected, keff = min(k, L)
//   chunk_info[u][c]   = {first output position of chunk c, ties (score == T) chunk c may take},
//                        c = 0 .. nc (entry nc = {keff, 0} closes the list)
// from the nc chunk histograms of the unit (`hp`, pitch NBP, uint16 counts).
// COHERENT: the histograms were written by other workgroups of this launch (device-coherent loads).
// `tot` is NB words of LDS.  Must be called by all 256 threads.
template <bool COHERENT>
__device__ __forceinline__ uint2 load_bins4(const uint16_t* p) {
    if constexpr (COHERENT) return ld_dev_u2(p);
    else return *reinterpret_cast<const uint2*>(p);
}

template <bool COHERENT>
__device__ __forceinline__ void unit_threshold(
    const uint16_t* __restrict__ hp, int nc, int keff, int NB, int NBP,
    int32_t* __restrict__ chunk_info_u, int32_t* __restrict__ unit_info_u, uint32_t* tot,
    ThresholdLds& S) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // total histogram: thread -> 4 consecutive bins (one 8-byte load per chunk)
    const int ncol = NBP / 4;
    for (int col = tid; col < ncol; col += 256) {
        uint32_t a0 = 0, a1 = 0, a2 = 0, a3 = 0;
        const uint16_t* p = hp + col * 4;
#pragma unroll 8
        for (int c = 0; c < nc; ++c) {
            const uint2 v = load_bins4<COHERENT>(p + (int64_t)c * NBP);
            a0 += v.x & 0xffffu; a1 += v.x >> 16;
            a2 += v.y & 0xffffu; a3 += v.y >> 16;
        }
        const int b0 = col * 4;
        if (b0 + 0 < NB) tot[b0 + 0] = a0;
        if (b0 + 1 < NB) tot[b0 + 1] = a1;
        if (b0 + 2 < NB) tot[b0 + 2] = a2;
        if (b0 + 3 < NB) tot[b0 + 3] = a3;
    }
    if (tid == 0) { S.T = (keff > 0) ? NB : 0; S.need = 0; }
    __syncthreads();
    // T = smallest score value whose inclusive prefix count reaches keff
    const int seg = (NB + 255) / 256;
    const int s0 = tid * seg, s1 = min(NB, s0 + seg);
    uint32_t local = 0;
    for (int i = s0; i < s1; ++i) local += tot[i];
    uint32_t total;
    const uint32_t before = block_excl_scan_256(local, S.scan4, &total);
    if (keff > 0 && before < (uint32_t)keff && before + local >= (uint32_t)keff) {
        uint32_t run = before;
        for (int i = s0; i < s1; ++i) {
            if (run + tot[i] >= (uint32_t)keff) { S.T = i; S.need = keff - (int)run; break; }
            run += tot[i];
        }
    }
    __syncthreads();
    const int T = S.T, need = S.need;
    // per chunk: keys below T and keys equal to T (one wave per chunk, 4 bins per lane and load)
    for (int c = wave; c < nc; c += 4) {
        const uint16_t* row = hp + (int64_t)c * NBP;
        uint32_t lt = 0;
        for (int col = lane; col * 4 < T; col += 64) {
            const uint2 v = load_bins4<COHERENT>(row + col * 4);
            const int b0 = col * 4;
            lt += (b0 + 0 < T ? v.x & 0xffffu : 0u) + (b0 + 1 < T ? v.x >> 16 : 0u);
            lt += (b0 + 2 < T ? v.y & 0xffffu : 0u) + (b0 + 3 < T ? v.y >> 16 : 0u);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) lt += __shfl_xor(lt, o, 64);
        if (lane == 0) {
            uint32_t eq = 0;
            if (T < NB) {
                const uint2 v = load_bins4<COHERENT>(row + (T & ~3));
                const uint32_t w = (T & 2) ? v.y : v.x;
                eq = (T & 1) ? (w >> 16) : (w & 0xffffu);
            }
            S.c_lt[c] = lt;
            S.c_eq[c] = eq;
        }
    }
    __syncthreads();
    // ordered offsets: ties are granted to chunks in cache order.  thread t owns chunks
    // [t*cpt, (t+1)*cpt)
    const int cpt = (nc + 255) / 256;
    const int c0 = min(nc, tid * cpt), c1 = min(nc, c0 + cpt);
    uint32_t eq_loc = 0;
    for (int c = c0; c < c1; ++c) eq_loc += S.c_eq[c];
    uint32_t eq_before = block_excl_scan_256(eq_loc, S.scan4, &total);
    uint32_t sel_loc = 0;
    {
        uint32_t eqb = eq_before;
        for (int c = c0; c < c1; ++c) {
            const uint32_t can = (uint32_t)need > eqb ? (uint32_t)need - eqb : 0u;
            const uint32_t take = min(can, S.c_eq[c]);
            sel_loc += S.c_lt[c] + take;
            eqb += S.c_eq[c];
        }
    }
    uint32_t off = block_excl_scan_256(sel_loc, S.scan4, &total);
    {
        uint32_t eqb = eq_before;
        for (int c = c0; c < c1; ++c) {
            const uint32_t can = (uint32_t)need > eqb ? (uint32_t)need - eqb : 0u;
            const uint32_t take = min(can, S.c_eq[c]);
            chunk_info_u[c * 2 + 0] = (int32_t)off;
            chunk_info_u[c * 2 + 1] = (int32_t)take;
            off += S.c_lt[c] + take;
            eqb += S.c_eq[c];
        }
    }
    if (tid == 0) {
        chunk_info_u[nc * 2 + 0] = keff;
        chunk_info_u[nc * 2 + 1] = 0;
        unit_info_u[0] = T;
        unit_info_u[1] = keff;
    }
}

// Ordered compaction of one block of 1024 consecutive keys [n0, n0 + 1024) by 256 threads
// (4 keys each).  `run_lt`, `run_eq` count the selected-below-T and equal-to-T keys of the
// chunk seen before this block; they are advanced.  For every selected key, emit(pos, n) is
// called with pos = its position in the unit's index list.  Must be called by all 256 threads.
template <typename Emit>
__device__ __forceinline__ void compact_block_1024(
    const uint16_t* __restrict__ sp, int n0, int L, int T, int off, int take,
    uint32_t& run_lt, uint32_t& run_eq, uint32_t* scan4, Emit emit) {
    const int tid = threadIdx.x;
    const int n = n0 + tid * 4;
    uint32_t sv[4];
    if (n + 4 <= L && (reinterpret_cast<uintptr_t>(sp + n) & 7) == 0) {
        const uint2 v = *reinterpret_cast<const uint2*>(sp + n);
        sv[0] = v.x & 0xffffu; sv[1] = v.x >> 16; sv[2] = v.y & 0xffffu; sv[3] = v.y >> 16;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[i] = (n + i < L) ? (uint32_t)sp[n + i] : 0xffffffffu;
    }
    uint32_t lt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool live = n + i < L;
        lt += (live && (int)sv[i] < T) ? 1u : 0u;
        eq += (live && (int)sv[i] == T) ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t before = block_excl_scan_256(lt | (eq << 16), scan4, &total);
    uint32_t lt_b = run_lt + (before & 0xffffu), eq_b = run_eq + (before >> 16);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool live = n + i < L;
        if (live && (int)sv[i] < T) {
            emit(off + (int)lt_b + (int)min(eq_b, (uint32_t)take), n + i);
            ++lt_b;
        } else if (live && (int)sv[i] == T) {
            if (eq_b < (uint32_t)take) emit(off + (int)lt_b + (int)eq_b, n + i);
            ++eq_b;
        }
    }
    run_lt += total & 0xffffu;
    run_eq += total >> 16;
}

}  // namespace hata
