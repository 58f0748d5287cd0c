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
#include "hata_internal.h"
#include "hata_trace.h"

namespace hata {

#define HATA_MAX_CHUNKS 1024

// LDS a workgroup needs to run unit_threshold()
struct ThresholdLds {
    uint32_t scan4[4];
    uint32_t wtot[4];
    float wlow[4];
    int T, need, bmin;
    uint32_t c_lt[HATA_MAX_CHUNKS];
    uint32_t c_eq[HATA_MAX_CHUNKS];
};

// One workgroup of 256 threads computes, for unit u:
//   unit_info[u]       = {T, keff}: keys with score < T are all selected, keff = min(k, L)
//   chunk_info[u][c]   = {first output position of chunk c, ties (score == T) chunk c may take},
//                        c = 0 .. nc (entry nc = {keff, 0} closes the list)
// from the nc chunk histograms of the unit (`hp`, pitch NBP, uint16 counts) and the unit's total
// histogram `unit_hist` (NB words) that the workgroups of this launch accumulated with atomics; it
// is read with device-coherent loads and cleared for the next launch.  `tot` is unused.
// Must be called by all 256 threads.
//
// Only the few 8-bin columns between the lowest occupied score and T matter for the per-chunk
// counts (the selected keys are the low tail of the distribution), so the second pass reads
// just those columns of every chunk row.
struct Bins8 { uint32_t w[4]; };  // 8 uint16 counts

template <bool COHERENT>
__device__ __forceinline__ Bins8 load_bins8(const uint16_t* p) {
    Bins8 r;
    if constexpr (COHERENT) {
        const uint2 a = ld_dev_u2(p), b = ld_dev_u2(p + 4);
        r.w[0] = a.x; r.w[1] = a.y; r.w[2] = b.x; r.w[3] = b.y;
    } else {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
    }
    return r;
}
__device__ __forceinline__ uint32_t bin_of(const Bins8& v, int e) {
    const uint32_t w = v.w[e >> 1];
    return (e & 1) ? (w >> 16) : (w & 0xffffu);
}

template <int MAXSEG = 17>
__device__ __forceinline__ void unit_threshold(
    const uint16_t* __restrict__ hp, uint32_t* __restrict__ unit_hist_u, int nc, int keff, int NB,
    int NBP, int32_t* __restrict__ chunk_info_u, int32_t* __restrict__ unit_info_u, uint32_t* tot,
    ThresholdLds& S, unsigned long long* __restrict__ rec_u = nullptr, uint32_t epoch = 0,
    int spec_bmin = -1) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { S.T = (keff > 0) ? NB : 0; S.need = 0; }
    for (int c = tid; c < nc; c += 256) { S.c_lt[c] = 0; S.c_eq[c] = 0; }
    // Total histogram of the unit, held in registers: thread t owns the seg consecutive score
    // values from t * seg (seg <= MAXSEG; NB <= 4097 needs 17); all loads are in flight together.
    const int seg = (NB + 255) / 256;
    const int s0 = tid * seg;
    uint32_t x[MAXSEG];
    // Speculation (spec_bmin = lowest score of the caller's own chunk, or -1): the per-chunk counts
    // below need columns [bmin / 8, T / 8] of every chunk row, which are only known after T -- a
    // second dependent round trip.  T sits in the low tail, a few columns above the lowest score
    // of any chunk, so SPEC_COLS columns starting a little below the caller's own lowest score are
    // fetched together with the unit histogram and used if they turn out to cover the range
    // (3 columns below: the unit's lowest score is a little lower than one chunk's).
    constexpr int SPEC_COLS = 8, SPEC_IT = 4;
    const bool spec = spec_bmin >= 0 && nc * SPEC_COLS <= 256 * SPEC_IT && NBP / 8 >= SPEC_COLS;
    const int colA = spec ? min(max(spec_bmin / 8 - 3, 0), NBP / 8 - SPEC_COLS) : 0;
    Bins8 sx[SPEC_IT];
    {
#pragma unroll
        for (int j = 0; j < MAXSEG; ++j)  // clamped index: unconditional loads
            if (j < seg)
                x[j] = __hip_atomic_load(unit_hist_u + min(s0 + j, NB - 1), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
        if (spec) {
#pragma unroll
            for (int j = 0; j < SPEC_IT; ++j) {
                if (j * 256 < nc * SPEC_COLS) {
                    const int i = min(tid + j * 256, nc * SPEC_COLS - 1);
                    sx[j] = load_bins8<true>(hp + (int64_t)(i / SPEC_COLS) * NBP + (colA + i % SPEC_COLS) * 8);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < MAXSEG; ++j) {
            if (j < seg && s0 + j < NB) {
                if (x[j]) unit_hist_u[s0 + j] = 0;  // left clean for the next launch
            } else {
                x[j] = 0;
            }
        }
    }
    uint32_t local = 0;
    int first_nz = NB;
#pragma unroll
    for (int j = MAXSEG - 1; j >= 0; --j) {
        local += x[j];
        if (x[j]) first_nz = s0 + j;
    }
    // T = smallest score value whose inclusive prefix count reaches keff; bmin = lowest occupied
    // score (values <= 4097 are exact in the float lane reductions)
    const uint32_t incl_w = wave_incl_scan(local);
    const float low_w = wave_max64(-(float)first_nz);
    if (lane == 63) { S.wtot[wave] = incl_w; S.wlow[wave] = low_w; }
    __syncthreads();
    HATA_TRACE_AT(26, true);
    {
        const uint32_t w0 = S.wtot[0], w1 = S.wtot[1], w2 = S.wtot[2];
        const uint32_t before = (wave > 0 ? w0 : 0u) + (wave > 1 ? w1 : 0u) + (wave > 2 ? w2 : 0u) + incl_w - local;
        if (keff > 0 && before < (uint32_t)keff && before + local >= (uint32_t)keff) {
            uint32_t run = before;
            bool found = false;
#pragma unroll
            for (int j = 0; j < MAXSEG; ++j) {
                if (!found && run + x[j] >= (uint32_t)keff) {
                    S.T = s0 + j;
                    S.need = keff - (int)run;
                    found = true;
                }
                run += x[j];
            }
        }
        if (tid == 0)
            S.bmin = (int)(-fmaxf(fmaxf(S.wlow[0], S.wlow[1]), fmaxf(S.wlow[2], S.wlow[3])));
    }
    __syncthreads();
    const int T = S.T, need = S.need;
    HATA_TRACE_AT(27, true);
    // per chunk: keys below T and keys equal to T, from columns [bmin / 8, T / 8] of its row
    auto count_item = [&](const Bins8& v, int c, int col) {
        uint32_t lt = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t cnt = bin_of(v, e);
            lt += (col * 8 + e < T) ? cnt : 0u;
            if (col * 8 + e == T) S.c_eq[c] = cnt;  // one item per chunk holds bin T
        }
        if (lt) atomicAdd(&S.c_lt[c], lt);
    };
    if (T < NB && spec && min(S.bmin, T) / 8 >= colA && T / 8 < colA + SPEC_COLS) {
        // the speculative columns cover [bmin / 8, T / 8]: no second round trip
        const int col0 = min(S.bmin, T) / 8, col1 = T / 8;
#pragma unroll
        for (int j = 0; j < SPEC_IT; ++j) {
            const int i = tid + j * 256;
            if (i < nc * SPEC_COLS) {
                const int c = i / SPEC_COLS, col = colA + i % SPEC_COLS;
                if (col >= col0 && col <= col1) count_item(sx[j], c, col);
            }
        }
    } else if (T < NB) {
        const int col0 = min(S.bmin, T) / 8;
        const int ncols = T / 8 - col0 + 1;
        const int items = nc * ncols;
        for (int i0 = tid; i0 < items; i0 += 256 * 4) {
            Bins8 x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = min(i0 + j * 256, items - 1);
                const int c = i / ncols, col = col0 + (i - c * ncols);
                x[j] = load_bins8<true>(hp + (int64_t)c * NBP + col * 8);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j * 256;
                if (i < items) {
                    const int c = i / ncols, col = col0 + (i - c * ncols);
                    count_item(x[j], c, col);
                }
            }
        }
    }
    __syncthreads();
    HATA_TRACE_AT(28, true);
    // ordered offsets: ties are granted to chunks in cache order.  One wave: lane l owns chunks
    // [l*cpl, (l+1)*cpl); two wave scans (ties seen so far, then selected so far), no barrier.
    if (tid < 64) {
        const int cpl = (nc + 63) / 64;
        const int c0 = min(nc, tid * cpl), c1 = min(nc, c0 + cpl);
        uint32_t eq_loc = 0;
        for (int c = c0; c < c1; ++c) eq_loc += S.c_eq[c];
        const uint32_t eq_before = wave_incl_scan(eq_loc) - eq_loc;
        uint32_t sel_loc = 0;
        {
            uint32_t eqb = eq_before;
            for (int c = c0; c < c1; ++c) {
                const uint32_t can = (uint32_t)need > eqb ? (uint32_t)need - eqb : 0u;
                sel_loc += S.c_lt[c] + min(can, S.c_eq[c]);
                eqb += S.c_eq[c];
            }
        }
        uint32_t off = wave_incl_scan(sel_loc) - sel_loc;
        uint32_t eqb = eq_before;
        for (int c = c0; c < c1; ++c) {
            const uint32_t can = (uint32_t)need > eqb ? (uint32_t)need - eqb : 0u;
            const uint32_t take = min(can, S.c_eq[c]);
            if (!rec_u) {  // (the single-launch step reads the records below instead)
                st_dev(reinterpret_cast<uint32_t*>(chunk_info_u) + c * 2 + 0, off);
                st_dev(reinterpret_cast<uint32_t*>(chunk_info_u) + c * 2 + 1, take);
            } else {
                // two self-validating words per chunk (each carries the launch epoch in its upper
                // half, so a waiting workgroup needs no separate flag): {off, selected count}, 16 bits
                // each (the caller runs this form only for budgets below 65536 rows), and
                // {ties granted, T}, 19 and 13 bits
                const uint32_t cnt_c = S.c_lt[c] + take;
                __hip_atomic_store(rec_u + HATA_REC_STRIDE * c, ((unsigned long long)epoch << 32) | (off << 16) | cnt_c,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(rec_u + HATA_REC_STRIDE * c + 1, ((unsigned long long)epoch << 32) | (take << 13) | (uint32_t)T,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            off += S.c_lt[c] + take;
            eqb += S.c_eq[c];
        }
    }
    HATA_TRACE_AT(29, true);
    if (tid == 0 && !rec_u) {
        // (write-through: the next launch's workgroups read these)
        st_dev(reinterpret_cast<uint32_t*>(chunk_info_u) + nc * 2 + 0, (uint32_t)keff);
        st_dev(reinterpret_cast<uint32_t*>(chunk_info_u) + nc * 2 + 1, 0u);
        st_dev(reinterpret_cast<uint32_t*>(unit_info_u) + 0, (uint32_t)T);
        st_dev(reinterpret_cast<uint32_t*>(unit_info_u) + 1, (uint32_t)keff);
    }
}

// LDS histogram (NB words) -> the chunk's row of uint16 counts, two bins per write-through store
__device__ __forceinline__ void write_chunk_hist(uint16_t* hp, const uint32_t* hist, int NB, int NBP) {
    uint32_t* hp32 = reinterpret_cast<uint32_t*>(hp);
    for (int i = threadIdx.x; i < NBP / 2; i += 256) {
        const uint32_t lo = (2 * i < NB) ? hist[2 * i] : 0u;
        const uint32_t hi = (2 * i + 1 < NB) ? hist[2 * i + 1] : 0u;
        st_dev(hp32 + i, lo | (hi << 16));
    }
}

// Tail of a scoring workgroup in the fused step: publish the chunk histogram, count the unit's
// finished chunks, and let the last one compute the unit's threshold.  `hist` (NB words of LDS)
// is reused as the total histogram.
__device__ __forceinline__ void finish_unit(
    int64_t u, int nc, int keff, const uint16_t* __restrict__ chunk_hist_u, int NB, int NBP,
    int n_chunks, int32_t* __restrict__ chunk_info, int32_t* __restrict__ unit_info,
    uint32_t* __restrict__ unit_counter, uint32_t* __restrict__ unit_hist, uint32_t* hist,
    ThresholdLds& S, int* flag) {
    HATA_TRACE_AT(2, u == 0);
    // add this chunk's histogram to the unit's total (only occupied bins)
    for (int i = threadIdx.x; i < NB; i += 256) {
        const uint32_t hv = hist[i];
        if (hv) atomicAdd(&unit_hist[u * NB + i], hv);
    }
    HATA_TRACE_AT(3, u == 0);
    wait_stores();    // this thread's write-through stores and atomics have completed
    HATA_TRACE_AT(4, u == 0);
    __syncthreads();  // ... and so have those of the whole workgroup
    if (threadIdx.x == 0) {
        const uint32_t done = atomicAdd(&unit_counter[u], 1u);
        const int last = (done == (uint32_t)(nc - 1));
        if (last) unit_counter[u] = 0;  // ready for the next launch
        *flag = last;
    }
    __syncthreads();
    if (!*flag) return;
    HATA_TRACE_AT(5, u == 0);
    // the other workgroups' histograms are read with device-coherent loads
    unit_threshold(chunk_hist_u, unit_hist + u * NB, nc, keff, NB, NBP, chunk_info + u * (n_chunks + 1) * 2,
                   unit_info + u * 2, hist, S);
    HATA_TRACE_AT(6, u == 0);
}

// Ordered compaction of one whole chunk of 256 * KPT consecutive keys [n0, n0 + 256*KPT) by 256
// threads (KPT consecutive keys each, all score loads in flight together).  For every selected
// key, emit(pos, n) is called with pos = its position in the unit's index list.
// Must be called by all 256 threads.
template <int KPT, typename Emit>
__device__ __forceinline__ void compact_chunk(
    const uint16_t* __restrict__ sp, int n0, int L, int T, int off, int take, uint32_t* scan4,
    Emit emit) {
    const int tid = threadIdx.x;
    const int n = n0 + tid * KPT;
    uint32_t sv[KPT];
    if (n + KPT <= L && (reinterpret_cast<uintptr_t>(sp + n) & 7) == 0) {
#pragma unroll
        for (int i = 0; i < KPT / 4; ++i) {
            const uint2 v = reinterpret_cast<const uint2*>(sp + n)[i];
            sv[4 * i + 0] = v.x & 0xffffu; sv[4 * i + 1] = v.x >> 16;
            sv[4 * i + 2] = v.y & 0xffffu; sv[4 * i + 3] = v.y >> 16;
        }
    } else {
#pragma unroll
        for (int i = 0; i < KPT; ++i) sv[i] = (n + i < L) ? (uint32_t)sp[n + i] : 0xffffffffu;
    }
    uint32_t lt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const bool live = n + i < L;
        lt += (live && (int)sv[i] < T) ? 1u : 0u;
        eq += (live && (int)sv[i] == T) ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t before = block_excl_scan_256(lt | (eq << 16), scan4, &total);
    uint32_t lt_b = before & 0xffffu, eq_b = before >> 16;
    if (lt == 0 && (eq == 0 || eq_b >= (uint32_t)take)) return;  // nothing of this thread is selected
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const bool live = n + i < L;
        if (live && (int)sv[i] < T) {
            emit(off + (int)lt_b + (int)min(eq_b, (uint32_t)take), n + i);
            ++lt_b;
        } else if (live && (int)sv[i] == T) {
            if (eq_b < (uint32_t)take) emit(off + (int)lt_b + (int)eq_b, n + i);
            ++eq_b;
        }
    }
}

// chunk = 256 * kpt keys, kpt in {4, 8, 16, 32}
template <typename Emit>
__device__ __forceinline__ void compact_chunk_any(
    int kpt, const uint16_t* __restrict__ sp, int n0, int L, int T, int off, int take,
    uint32_t* scan4, Emit emit) {
    switch (kpt) {
        case 4: compact_chunk<4>(sp, n0, L, T, off, take, scan4, emit); break;
        case 8: compact_chunk<8>(sp, n0, L, T, off, take, scan4, emit); break;
        case 16: compact_chunk<16>(sp, n0, L, T, off, take, scan4, emit); break;
        default: compact_chunk<32>(sp, n0, L, T, off, take, scan4, emit); break;
    }
}

}  // namespace hata
