// Selection kernels (Alg. 3 of the paper: Idx = TopK(S, N)).
//
// The paper names no algorithm.  Scores are small integers (0 .. G*r), so selection is
// a counting select: per-chunk histograms -> per-unit threshold T and the number of
// keys with score == T still needed -> ordered compaction, so that among equal scores
// the LOWER cache row wins and Idx comes out ascending.  Everything is deterministic
// (no atomics decide an output position).
//
//   hist_kernel       chunk histogram from stored scores (stand-alone top-k only; the
//                     fused decode step gets the histograms from the scoring kernel)
//   threshold_kernel  one workgroup per unit: total histogram, T, per-chunk output offsets
//   compact_kernel    one workgroup per chunk: writes the selected rows at their final place
#include "hata_device.h"
#include "hata_internal.h"

namespace hata {

#define HATA_MAX_CHUNKS 1024

__global__ __launch_bounds__(256) void hist_kernel(
    const uint16_t* __restrict__ scores, const int32_t* __restrict__ seq_len,
    uint16_t* __restrict__ chunk_hist, int Hkv, int L_cap, int chunk, int n_chunks, int NB,
    int NBP) {
    extern __shared__ uint32_t hist[];
    const int tid = threadIdx.x;
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = clampi(seq_len[b], 0, L_cap);
    const int base = c * chunk;
    if (base >= L) return;
    const int end = min(base + chunk, L);
    const int64_t u = (int64_t)b * Hkv + h;
    for (int i = tid; i < NB; i += 256) hist[i] = 0;
    __syncthreads();
    const uint16_t* sp = scores + u * L_cap;
    for (int n = base + tid; n < end; n += 256) atomicAdd(&hist[min((int)sp[n], NB - 1)], 1u);
    __syncthreads();
    uint16_t* hp = chunk_hist + (u * n_chunks + c) * NBP;
    for (int i = tid; i < NB; i += 256) hp[i] = (uint16_t)hist[i];
}

// grid = B*Hkv units, 256 threads.
__global__ __launch_bounds__(256) void threshold_kernel(
    const uint16_t* __restrict__ chunk_hist, const int32_t* __restrict__ seq_len,
    const int32_t* __restrict__ kbud, int32_t* __restrict__ chunk_info,
    int32_t* __restrict__ unit_info, int Hkv, int L_cap, int k_max, int chunk, int n_chunks,
    int NB, int NBP) {
    extern __shared__ uint32_t tot[];          // NB bins
    __shared__ uint32_t scan4[4];
    __shared__ int sh_T, sh_need;
    __shared__ uint32_t c_lt[HATA_MAX_CHUNKS], c_eq[HATA_MAX_CHUNKS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = blockIdx.x;
    const int b = u / Hkv;
    const int L = clampi(seq_len[b], 0, L_cap);
    const int keff = min(clampi(kbud[b], 0, k_max), L);
    const int nc = (L + chunk - 1) / chunk;
    const uint16_t* hp = chunk_hist + (int64_t)u * n_chunks * NBP;

    // total histogram of the unit
    for (int i = tid; i < NB; i += 256) {
        uint32_t t = 0;
        for (int c = 0; c < nc; ++c) t += hp[(int64_t)c * NBP + i];
        tot[i] = t;
    }
    if (tid == 0) { sh_T = NB; sh_need = 0; }
    __syncthreads();

    // T = smallest score value whose inclusive prefix count reaches keff
    const int seg = (NB + 255) / 256;
    const int s0 = tid * seg, s1 = min(NB, s0 + seg);
    uint32_t local = 0;
    for (int i = s0; i < s1; ++i) local += tot[i];
    uint32_t total;
    uint32_t before = block_excl_scan_256(local, scan4, &total);
    if (keff > 0 && before < (uint32_t)keff && before + local >= (uint32_t)keff) {
        uint32_t run = before;
        for (int i = s0; i < s1; ++i) {
            if (run + tot[i] >= (uint32_t)keff) { sh_T = i; sh_need = keff - (int)run; break; }
            run += tot[i];
        }
    }
    if (keff == 0 && tid == 0) { sh_T = 0; sh_need = 0; }
    __syncthreads();
    const int T = sh_T, need = sh_need;

    // per chunk: keys below T and keys equal to T
    for (int c = wave; c < nc; c += 4) {
        const uint16_t* row = hp + (int64_t)c * NBP;
        uint32_t lt = 0;
        for (int i = lane; i < T; i += 64) lt += row[i];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) lt += __shfl_xor(lt, o, 64);
        if (lane == 0) { c_lt[c] = lt; c_eq[c] = (T < NB) ? row[T] : 0u; }
    }
    __syncthreads();
    // ordered offsets: ties are granted to chunks in cache order
    if (tid == 0) {
        uint32_t off = 0, eq_seen = 0;
        for (int c = 0; c < nc; ++c) {
            uint32_t can = (uint32_t)need > eq_seen ? (uint32_t)need - eq_seen : 0u;
            uint32_t take = min(can, c_eq[c]);
            chunk_info[((int64_t)u * n_chunks + c) * 2 + 0] = (int32_t)off;
            chunk_info[((int64_t)u * n_chunks + c) * 2 + 1] = (int32_t)take;
            off += c_lt[c] + take;
            eq_seen += c_eq[c];
        }
        unit_info[u * 2 + 0] = T;
        unit_info[u * 2 + 1] = keff;
    }
}

// grid = (n_chunks, Hkv, B), 256 threads; thread t owns chunk/256 consecutive keys.
template <int KPT>
__global__ __launch_bounds__(256) void compact_kernel(
    const uint16_t* __restrict__ scores, const int32_t* __restrict__ seq_len,
    const int32_t* __restrict__ chunk_info, const int32_t* __restrict__ unit_info,
    int32_t* __restrict__ idx, int Hkv, int L_cap, int k_max, int n_chunks) {
    __shared__ uint32_t scan4[4];
    const int tid = threadIdx.x;
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    constexpr int chunk = KPT * 256;
    const int L = clampi(seq_len[b], 0, L_cap);
    const int64_t u = (int64_t)b * Hkv + h;
    const int T = unit_info[u * 2 + 0];
    const int keff = unit_info[u * 2 + 1];
    int32_t* out = idx + u * k_max;
    if (c == 0)  // pad the row
        for (int i = keff + tid; i < k_max; i += 256) out[i] = -1;
    const int base = c * chunk;
    if (base >= L) return;
    const int off = chunk_info[(u * n_chunks + c) * 2 + 0];
    const int take = chunk_info[(u * n_chunks + c) * 2 + 1];
    const int n0 = base + tid * KPT;
    const uint16_t* sp = scores + u * L_cap;
    uint32_t sv[KPT];
    if (n0 + KPT <= L && (reinterpret_cast<uintptr_t>(sp + n0) & 7) == 0) {
        // 8-byte loads of four scores
        const uint2* p = reinterpret_cast<const uint2*>(sp + n0);
#pragma unroll
        for (int i = 0; i < KPT / 4; ++i) {
            uint2 v = p[i];
            sv[4 * i + 0] = v.x & 0xffffu; sv[4 * i + 1] = v.x >> 16;
            sv[4 * i + 2] = v.y & 0xffffu; sv[4 * i + 3] = v.y >> 16;
        }
    } else {
#pragma unroll
        for (int i = 0; i < KPT; ++i) sv[i] = (n0 + i < L) ? (uint32_t)sp[n0 + i] : 0xffffffffu;
    }
    uint32_t lt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const bool live = n0 + i < L;
        lt += (live && (int)sv[i] < T) ? 1u : 0u;
        eq += (live && (int)sv[i] == T) ? 1u : 0u;
    }
    uint32_t total;
    uint32_t before = block_excl_scan_256(lt | (eq << 16), scan4, &total);
    uint32_t lt_b = before & 0xffffu, eq_b = before >> 16;
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const bool live = n0 + i < L;
        if (live && (int)sv[i] < T) {
            const int pos = off + (int)lt_b + (int)min(eq_b, (uint32_t)take);
            if (pos < k_max) out[pos] = n0 + i;
            ++lt_b;
        } else if (live && (int)sv[i] == T) {
            if (eq_b < (uint32_t)take) {
                const int pos = off + (int)lt_b + (int)eq_b;
                if (pos < k_max) out[pos] = n0 + i;
            }
            ++eq_b;
        }
    }
}

hipError_t launch_topk(const hata_ctx* c, const uint16_t* scores, const int32_t* seq_len,
                       const int32_t* k, int B, int32_t* idx, bool have_hist, hipStream_t s) {
    const hata_config& f = c->cfg;
    const dim3 grid(c->n_chunks, f.Hkv, B);
    const size_t lds = (size_t)c->NB * 4;
    if (!have_hist)
        hipLaunchKernelGGL(hist_kernel, grid, dim3(256), lds, s, scores, seq_len, c->chunk_hist,
                           f.Hkv, f.L_cap, c->chunk, c->n_chunks, c->NB, c->NBP);
    hipLaunchKernelGGL(threshold_kernel, dim3(B * f.Hkv), dim3(256), lds, s, c->chunk_hist,
                       seq_len, k, c->chunk_info, c->unit_info, f.Hkv, f.L_cap, f.k_max,
                       c->chunk, c->n_chunks, c->NB, c->NBP);
#define HATA_COMPACT(KPT)                                                                     \
    hipLaunchKernelGGL((compact_kernel<KPT>), grid, dim3(256), 0, s, scores, seq_len,         \
                       c->chunk_info, c->unit_info, idx, f.Hkv, f.L_cap, f.k_max, c->n_chunks)
    switch (c->chunk / 256) {
        case 4: HATA_COMPACT(4); break;
        case 8: HATA_COMPACT(8); break;
        case 16: HATA_COMPACT(16); break;
        case 32: HATA_COMPACT(32); break;
        default: return hipErrorInvalidValue;
    }
#undef HATA_COMPACT
    return hipGetLastError();
}

}  // namespace hata
