// Stand-alone selection kernels (Alg. 3 of the paper: Idx = TopK(S, N)) for scores that are
// already stored: chunk histograms -> unit threshold -> ordered compaction.  The fused decode
// step does not use these launches (its scoring kernel produces the histograms and the
// threshold, its attention kernel compacts on the fly); the arithmetic is the shared code of
// hata_select.h either way.
#include "hata_device.h"
#include "hata_internal.h"
#include "hata_select.h"

namespace hata {

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
    extern __shared__ uint32_t tot[];  // NB words
    __shared__ ThresholdLds S;
    const int u = blockIdx.x;
    const int b = u / Hkv;
    const int L = clampi(seq_len[b], 0, L_cap);
    const int keff = min(clampi(kbud[b], 0, k_max), L);
    const int nc = (L + chunk - 1) / chunk;
    unit_threshold<false>(chunk_hist + (int64_t)u * n_chunks * NBP, nullptr, nc, keff, NB, NBP,
                   chunk_info + (int64_t)u * (n_chunks + 1) * 2, unit_info + u * 2, tot, S);
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
    hipLaunchKernelGGL(hist_kernel, grid, dim3(256), lds, s, scores, seq_len, c->chunk_hist,
                       f.Hkv, f.L_cap, c->chunk, c->n_chunks, c->NB, c->NBP);
    hipLaunchKernelGGL(threshold_kernel, dim3(B * f.Hkv), dim3(256), lds, s, c->chunk_hist,
                       seq_len, k, c->chunk_info, c->unit_info, f.Hkv, f.L_cap, f.k_max,
                       c->chunk, c->n_chunks, c->NB, c->NBP);
    hipLaunchKernelGGL(compact_kernel, grid, dim3(256), 0, s, scores, seq_len, c->chunk_info,
                       c->unit_info, idx, f.Hkv, f.L_cap, f.k_max, c->chunk, c->n_chunks);
    return hipGetLastError();
}

}  // namespace hata
