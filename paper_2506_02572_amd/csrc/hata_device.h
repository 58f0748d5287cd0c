// Device-side helpers shared by the HATA kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define HATA_WAVE 64
#define HATA_D 128  // head dimension every kernel is written for

namespace hata {

// bf16 pair packed in one dword -> two fp32 values (bf16 is the upper half of an fp32)
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (inf/nan pass through)
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return u >> 16;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Device-coherent accesses for data that one workgroup writes and another workgroup of the SAME
// launch reads (last-arriver patterns).  The stores write through the XCD-local L2 and the loads
// bypass it, so no L2 write-back / invalidate fence is needed around the arrival counter: the
// writer only waits for its stores to complete (wait_stores) before it bumps the counter.
__device__ __forceinline__ void st_dev(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint2 ld_dev_u2(const void* p) {
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint2((uint32_t)v, (uint32_t)(v >> 32));
}
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// ---- cross-lane reductions in the VALU (no LDS traffic) ----
// A wave is 4 rows of 16 lanes.  row_sum16: every lane gets the sum over its row (DPP quad
// permutes and row mirrors).  xor16 / xor32 exchanges use the lane-swap instructions: with both
// operands equal to v, swapping the odd rows of one copy with the even rows of the other leaves
// {v[row ^ 1 ... even source], v[odd source]}, whose sum (or max) is the all-reduce over row
// pairs; likewise for the two 32-lane halves.
#define HATA_DPP(v, ctrl) \
    __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (v)), (ctrl), 0xf, 0xf, true))
__device__ __forceinline__ float row_sum16(float v) {
    v += HATA_DPP(v, 0xB1);   // quad_perm [1,0,3,2]
    v += HATA_DPP(v, 0x4E);   // quad_perm [2,3,0,1]
    v += HATA_DPP(v, 0x141);  // row_half_mirror
    v += HATA_DPP(v, 0x140);  // row_mirror
    return v;
}
// (written as inline asm: the instruction rewrites BOTH of its registers, and the compiler
// builtin of this toolchain returns the first register for both results; the s_nop cover the
// VALU-write -> lane-swap read hazard the compiler would otherwise handle)
__device__ __forceinline__ float row_max16(float v) {
    v = fmaxf(v, HATA_DPP(v, 0xB1));
    v = fmaxf(v, HATA_DPP(v, 0x4E));
    v = fmaxf(v, HATA_DPP(v, 0x141));
    v = fmaxf(v, HATA_DPP(v, 0x140));
    return v;
}
__device__ __forceinline__ void swap16(float v, float& a, float& b) {
    a = v; b = v;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap32(float v, float& a, float& b) {
    a = v; b = v;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
// all-reduce over the 4 rows of the wave (lane-wise): every lane gets the sum / max of the four
// lanes with the same position in their row
__device__ __forceinline__ float rows_sum4(float v) {
    float a, b;
    swap16(v, a, b); v = a + b;
    swap32(v, a, b); return a + b;
}
__device__ __forceinline__ float rows_max4(float v) {
    float a, b;
    swap16(v, a, b); v = fmaxf(a, b);
    swap32(v, a, b); return fmaxf(a, b);
}

// all-reduce over the whole wave
__device__ __forceinline__ float wave_sum64(float v) { return rows_sum4(row_sum16(v)); }
__device__ __forceinline__ float wave_max64(float v) { return rows_max4(row_max16(v)); }

// wave-level inclusive scan (sum) over 64 lanes, in the VALU: Hillis-Steele inside each row of
// 16 lanes with DPP row shifts, then the row totals are carried across rows with the two
// row-broadcast controls (lane 15 of a row into the next row; lane 31 into the upper half)
#define HATA_DPP_U(v, ctrl, rows) \
    (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(v), (ctrl), (rows), 0xf, false)
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    v += HATA_DPP_U(v, 0x111, 0xf);  // row_shr:1
    v += HATA_DPP_U(v, 0x112, 0xf);  // row_shr:2
    v += HATA_DPP_U(v, 0x114, 0xf);  // row_shr:4
    v += HATA_DPP_U(v, 0x118, 0xf);  // row_shr:8
    v += HATA_DPP_U(v, 0x142, 0xa);  // row_bcast:15 into rows 1 and 3
    v += HATA_DPP_U(v, 0x143, 0xc);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Block-wide exclusive scan for blockDim.x == 256 (4 waves).  `lds4` is 4 words of LDS.
// Returns the exclusive prefix of v; *total receives the block sum.
__device__ __forceinline__ uint32_t block_excl_scan_256(uint32_t v, uint32_t* lds4, uint32_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = wave_incl_scan(v);
    if (lane == 63) lds4[wave] = inc;
    __syncthreads();
    uint32_t w0 = lds4[0], w1 = lds4[1], w2 = lds4[2], w3 = lds4[3];
    uint32_t base = (wave > 0 ? w0 : 0u) + (wave > 1 ? w1 : 0u) + (wave > 2 ? w2 : 0u);
    *total = w0 + w1 + w2 + w3;
    __syncthreads();
    return base + inc - v;
}

// ---- summed Hamming distance of one key code to the G query codes of a group ----
// (Alg. 3 of the paper, "distance in Hamming space", with the aggregation over the query heads
// that share a KV cache: S = sum_g bitcount(xor(q_g, k)).)
// Direct form (written out in the kernels): G * WD (xor, popcount-accumulate) pairs per key.  For
// G >= 5 this helper rearranges the sum
// per BIT: a key bit that is 0 disagrees with the heads whose bit is 1, a key bit that is 1 with
// the d heads whose bit is 0, so with d[bit] = number of heads with a 0 there,
//   S = C0 + sum_{bits set in k} (2 d[bit] - G),   C0 = sum_g bitcount(q_g),
// and with d held bit-sliced in NP = ceil(log2(G + 1)) planes D_p (wave-uniform, like the codes),
//   S = C0 + 2 sum_p 2^p bitcount(k & D_p) - G bitcount(k):
// WD * (2 NP + 1) operations instead of 2 G WD (36 instead of 64 at G = 8, r = 128).
template <int WD, int G>
struct HammingSum {
    // (below five heads the direct form is as short; with 256-bit codes and four heads it needs 32
    // scalar registers for the query codes against 24 for the planes, and one instruction in eight less)
    static constexpr bool PLANES = G >= 5 || (G >= 4 && WD >= 8);
    static constexpr int NP = G >= 16 ? 5 : G >= 8 ? 4 : 3;  // G <= 31
    uint32_t d[NP][WD];
    uint32_t c0;

    // qp: the G * WD code words of the group (the same for every lane)
    __device__ __forceinline__ void init(const uint32_t* qp) {
        static_assert(G >= 1 && G <= 31, "plane count");
        c0 = 0;
#pragma unroll
        for (int w = 0; w < WD; ++w) {
            uint32_t pl[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p) pl[p] = 0;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const uint32_t qw = __builtin_amdgcn_readfirstlane(qp[g * WD + w]);
                c0 += __popc(qw);
                uint32_t carry = ~qw;  // add one to the counters of the bits where this head has a 0
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    const uint32_t t = pl[p] & carry;
                    pl[p] ^= carry;
                    carry = t;
                }
            }
#pragma unroll
            for (int p = 0; p < NP; ++p) d[p][w] = pl[p];
        }
    }

    __device__ __forceinline__ uint32_t operator()(const uint32_t (&k)[WD]) const {
        uint32_t pk = 0, a[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) a[p] = 0;
#pragma unroll
        for (int w = 0; w < WD; ++w) {
            pk += __popc(k[w]);
#pragma unroll
            for (int p = 0; p < NP; ++p) a[p] += __popc(k[w] & d[p][w]);
        }
        uint32_t t = a[NP - 1];
#pragma unroll
        for (int p = NP - 2; p >= 0; --p) t = 2 * t + a[p];
        return c0 + 2 * t - G * pk;
    }
};

}  // namespace hata
