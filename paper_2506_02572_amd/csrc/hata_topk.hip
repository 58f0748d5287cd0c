// Stand-alone selection kernels (Alg. 3 of the paper: Idx = TopK(S, N)) for scores that are
// already stored: chunk histograms and, by the last workgroup of each unit, the unit threshold ->
// ordered compaction (two launches).  The fused decode
// step does not use these launches (its scoring kernel produces the histograms and the
// threshold, its attention kernel compacts on the fly); the arithmetic is the shared code of
// hata_select.h either way.
#include "hata_device.h"
#include "hata_internal.h"
#include "hata_select.h"

namespace hata {

// grid = (n_chunks, Hkv, B), 256 threads: histogram of one chunk of stored scores; the last workgroup
// of a unit to finish goes on to the unit's threshold and chunk offsets (finish_unit), as the scoring
// kernel of the three-launch step does.
__global__ __launch_bounds__(256) void hist_kernel(
    const uint16_t* __restrict__ scores, const int32_t* __restrict__ seq_len,
    const int32_t* __restrict__ kbud, uint16_t* __restrict__ chunk_hist, int Hkv, int L_cap, int k_max,
    int chunk, int n_chunks, int NB, int NBP, int32_t* __restrict__ chunk_info,
    int32_t* __restrict__ unit_info, uint32_t* __restrict__ unit_counter, uint32_t* __restrict__ unit_hist) {
    extern __shared__ uint32_t hist[];
    __shared__ ThresholdLds S;
    __shared__ int last_flag;
    const int tid = threadIdx.x;
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = clampi(seq_len[b], 0, L_cap);
    const int base = c * chunk;
    const int64_t u = (int64_t)b * Hkv + h;
    if (base >= L) {
        if (L == 0 && c == 0 && tid == 0) {  // empty sequence: nothing selected
            unit_info[u * 2 + 0] = 0;
            unit_info[u * 2 + 1] = 0;
            chunk_info[u * (n_chunks + 1) * 2 + 0] = 0;
            chunk_info[u * (n_chunks + 1) * 2 + 1] = 0;
        }
        return;
    }
    const int end = min(base + chunk, L);
    for (int i = tid; i < NB; i += 256) hist[i] = 0;
    __syncthreads();
    const uint16_t* sp = scores + u * L_cap;
    for (int n = base + tid; n < end; n += 256) atomicAdd(&hist[min((int)sp[n], NB - 1)], 1u);
    __syncthreads();
    write_chunk_hist(chunk_hist + (u * n_chunks + c) * NBP, hist, NB, NBP);
    const int keff = min(clampi(kbud[b], 0, k_max), L);
    finish_unit(u, (L + chunk - 1) / chunk, keff, chunk_hist + u * n_chunks * NBP, NB, NBP, n_chunks, chunk_info,
                unit_info, unit_counter, unit_hist, hist, S, &last_flag);
}

// grid = (n_chunks, Hkv, B), 256 threads: ordered compaction of one chunk into the index list.
__global__ __launch_bounds__(256) void compact_kernel(
    const uint16_t* __restrict__ scores, const int32_t* __restrict__ seq_len,
    const int32_t* __restrict__ chunk_info, const int32_t* __restrict__ unit_info,
    int32_t* __restrict__ idx, int Hkv, int L_cap, int k_max, int chunk, int n_chunks) {
    __shared__ uint32_t scan4[4];
    const int tid = threadIdx.x;
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = clampi(seq_len[b], 0, L_cap);
    const int64_t u = (int64_t)b * Hkv + h;
    const int T = unit_info[u * 2 + 0];
    const int keff = unit_info[u * 2 + 1];
    int32_t* out = idx + u * k_max;
    if (c == 0)  // pad the row
        for (int i = keff + tid; i < k_max; i += 256) out[i] = -1;
    const int base = c * chunk;
    if (base >= L) return;
    const int32_t* ci = chunk_info + (u * (n_chunks + 1) + c) * 2;
    const int off = ci[0], take = ci[1];
    if (ci[2] == off) return;  // nothing selected in this chunk
    const uint16_t* sp = scores + u * L_cap;
    const int end = min(base + chunk, L);
    compact_chunk_any(chunk / 256, sp, base, end, T, off, take, scan4,
                      [&](int pos, int n) { if (pos < k_max) out[pos] = n; });
}

hipError_t launch_topk(const hata_ctx* c, const uint16_t* scores, const int32_t* seq_len,
                       const int32_t* k, int B, int32_t* idx, hipStream_t s) {
    const hata_config& f = c->cfg;
    const dim3 grid(c->n_chunks, f.Hkv, B);
    const size_t lds = (size_t)c->NB * 4;
    hipLaunchKernelGGL(hist_kernel, grid, dim3(256), lds, s, scores, seq_len, k, c->chunk_hist,
                       f.Hkv, f.L_cap, f.k_max, c->chunk, c->n_chunks, c->NB, c->NBP, c->chunk_info,
                       c->unit_info, c->unit_counter, c->unit_hist);
    hipLaunchKernelGGL(compact_kernel, grid, dim3(256), 0, s, scores, seq_len, c->chunk_info,
                       c->unit_info, idx, f.Hkv, f.L_cap, f.k_max, c->chunk, c->n_chunks);
    return hipGetLastError();
}

}  // namespace hata
