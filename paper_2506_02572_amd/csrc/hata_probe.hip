// Diagnostic, not part of the method: do the matrix cores and an HBM stream run at full rate at the
// same time on this device?  One launch of 256 workgroups of 8 waves: waves 0-3 of a workgroup (one
// per SIMD) issue nothing but v_mfma_f32_32x32x16_bf16 on operands taken from the caller's buffer,
// waves 4-7 read the workgroup's share of the buffer with 16-byte loads.  The caller times the launch
// with either half switched off and with both on.  (On the MI355X boxes this was written on the
// combined time is the SUM of the two: a kernel that needs both pays for both, which is why the
// prefill key encoder is priced by its MFMA count plus its bytes.)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hata.h"

namespace hata {

typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16_t;

__global__ __launch_bounds__(512) void probe_mfma_stream_kernel(const uint4* __restrict__ buf, size_t n16_per_wg,
                                                                int mfma_iters, int mode, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float s = 0.f;
    if (wave < 4) {
        if (!(mode & 1)) return;
        probe_bf16x8_t a[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = __builtin_bit_cast(probe_bf16x8_t, buf[i * 64 + lane]);
        const probe_bf16x8_t b0 = __builtin_bit_cast(probe_bf16x8_t, buf[512 + lane]);
        const probe_bf16x8_t b1 = __builtin_bit_cast(probe_bf16x8_t, buf[576 + lane]);
        probe_f32x16_t c0 = {}, c1 = {};
        for (int i = 0; i < mfma_iters; ++i) {
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {  // 16 MFMAs per turn, two independent accumulators
                c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], b0, c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], b1, c1, 0, 0, 0);
            }
        }
        s = c0[0] + c1[1];
    } else {
        if (!(mode & 2)) return;
        const uint4* p = buf + (size_t)blockIdx.x * n16_per_wg;
        uint32_t acc = 0;
        for (size_t i = threadIdx.x - 256; i < n16_per_wg; i += 256 * 8) {
            uint4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (i + j * 256 < n16_per_wg) ? p[i + j * 256] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc += v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
        }
        s = (float)acc;
    }
    if (s == 12345.678f && sink) sink[blockIdx.x] = s;  // (keeps the work alive; practically never taken)
}

}  // namespace hata

extern "C" int hata_probe_mfma_stream(const void* buf, size_t bytes, int32_t mfma_iters, int32_t mode, void* stream) {
    if (!buf || ((uintptr_t)buf & 15) || bytes < (size_t)256 * 16384 || mfma_iters < 0 || mode < 1 || mode > 3)
        return HATA_EINVAL;
    const size_t n16_per_wg = bytes / 16 / 256;
    hipLaunchKernelGGL(hata::probe_mfma_stream_kernel, dim3(256), dim3(512), 0, (hipStream_t)stream,
                       (const uint4*)buf, n16_per_wg, (int)mfma_iters, (int)mode, (float*)nullptr);
    return hipGetLastError() == hipSuccess ? HATA_OK : HATA_EHIP;
}
