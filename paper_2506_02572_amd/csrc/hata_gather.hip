// Gather of the selected K / V rows into a contiguous staging buffer (Alg. 3 of the paper: the
// "Gather" line, materialised): for the offloading variant of Sec. 5.3, where K and V live in pinned
// host memory, the rows a layer will attend over are fetched over the bus ahead of time -- on a
// stream of their own, while another layer computes -- and attention then reads device memory.
//
// staged K / V: [B, Hkv, k_max, d] bf16; row t of unit (b, h) = cache row idx[b, h, t].  Entries
// t >= min(k[b], k_max) and negative or out-of-range index entries leave their staged row untouched.
// A row is 256 B = 16 lanes x 128 bit; a workgroup of 256 threads moves blocks of 64 rows of K and of
// V, every load of a block in flight before its first store (bus latency, not bandwidth, is what a
// thread waits for).  The blocks are dealt out to a grid the caller may cap: every read of host
// memory that is outstanding also stands in front of whatever else crosses the bus -- the command
// processor's fetches of the kernel launches of other streams included -- so with the whole 2 MB of
// a step's rows in flight at once the step a pipeline wants to overlap waits for the fetch
// (measured: 32 workgroups, 1 MB in flight, keep the bus at 48 GB/s and a 32-layer pipeline at 55 us
// per layer; 64 workgroups 60 us, 16 workgroups 71 us).
#include "hata_device.h"
#include "hata_internal.h"

namespace hata {

#define HATA_GATHER_IT 4  // passes whose loads are in flight together (64 rows per block)

__global__ __launch_bounds__(256) void gather_rows_kernel(
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ kbud, uint16_t* __restrict__ Ks, uint16_t* __restrict__ Vs, int Hkv, int L_cap,
    int k_max, int blocks_per_unit, int n_blocks, int64_t sb, int64_t sh, int64_t sn) {
    const int tid = threadIdx.x, sub = tid & 15, r = tid >> 4;
    for (int blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
        const int64_t u = blk / blocks_per_unit;
        const int t0 = (blk % blocks_per_unit) * (16 * HATA_GATHER_IT);
        const int b = (int)(u / Hkv), h = (int)(u % Hkv);
        const int cnt = clampi(kbud[b], 0, k_max);
        if (t0 >= cnt) continue;
        const int32_t* ip = idx + u * k_max;
        const uint16_t* Kb = K + b * sb + h * sh;
        const uint16_t* Vb = V + b * sb + h * sh;
        uint4 kv[HATA_GATHER_IT], vv[HATA_GATHER_IT];
        bool ok[HATA_GATHER_IT];
#pragma unroll
        for (int it = 0; it < HATA_GATHER_IT; ++it) {
            const int t = t0 + it * 16 + r;
            int n = -1;
            if (t < cnt) n = ip[t];
            ok[it] = n >= 0 && n < L_cap;
            if (ok[it]) {
                const int64_t o = (int64_t)n * sn + sub * 8;
                kv[it] = *reinterpret_cast<const uint4*>(Kb + o);
                vv[it] = *reinterpret_cast<const uint4*>(Vb + o);
            }
        }
#pragma unroll
        for (int it = 0; it < HATA_GATHER_IT; ++it) {
            const int t = t0 + it * 16 + r;
            if (ok[it]) {
                const int64_t o = (u * k_max + t) * HATA_D + sub * 8;
                *reinterpret_cast<uint4*>(Ks + o) = kv[it];
                *reinterpret_cast<uint4*>(Vs + o) = vv[it];
            }
        }
    }
}

hipError_t launch_gather_rows(const hata_ctx* c, const void* K, const void* V, const int32_t* idx,
                              const int32_t* k, int B, int max_workgroups, void* K_stage, void* V_stage,
                              hipStream_t s) {
    const hata_config& f = c->cfg;
    const int per_block = 16 * HATA_GATHER_IT;
    const int blocks_per_unit = (f.k_max + per_block - 1) / per_block;
    const int64_t n_blocks = (int64_t)blocks_per_unit * f.Hkv * B;
    if (n_blocks > 0x7fffffffll) return hipErrorInvalidValue;
    int64_t grid = n_blocks;
    if (max_workgroups > 0 && grid > max_workgroups) grid = max_workgroups;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)grid), dim3(256), 0, s, (const uint16_t*)K,
                       (const uint16_t*)V, idx, k, (uint16_t*)K_stage, (uint16_t*)V_stage, f.Hkv, f.L_cap, f.k_max,
                       blocks_per_unit, (int)n_blocks, f.kv_stride_b, f.kv_stride_h, f.kv_stride_n);
    return hipGetLastError();
}

}  // namespace hata
