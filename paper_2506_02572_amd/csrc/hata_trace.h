// Optional in-kernel timestamps for tuning (compiled only with -DHATA_TRACE -fgpu-rdc; the
// normal build contains none of this).  HATA_TRACE_AT(slot, cond) stores the 100 MHz wall clock
// into slot `slot` of a device array when thread 0 of a workgroup satisfies `cond`.
#pragma once
#ifdef HATA_TRACE
extern __device__ unsigned long long g_hata_trace[64];
#define HATA_TRACE_AT(slot, cond) \
    do { if (threadIdx.x == 0 && (cond)) g_hata_trace[slot] = wall_clock64(); } while (0)
#else
#define HATA_TRACE_AT(slot, cond) do { } while (0)
#endif
