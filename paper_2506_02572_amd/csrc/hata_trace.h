// Optional in-kernel timestamps for tuning (compiled only with -DHATA_TRACE -fgpu-rdc; the
// normal build contains none of this).  HATA_TRACE_AT(slot, cond): thread 0 of every workgroup
// (up to HATA_TRACE_WGS of them) that satisfies `cond` stores the 100 MHz wall clock into its own
// row of a device array, column slot % 32 -- plain stores, nothing shared between workgroups, so
// the instrument does not serialise them.  The host clears the array between launches
// (hata_debug_trace_reset), reads it back (hata_debug_trace) and forms, per checkpoint, when the
// first, the median and the last workgroup of the grid passed it.
#pragma once
#ifdef HATA_TRACE
#define HATA_TRACE_WGS 4096
extern __device__ unsigned long long g_hata_trace[HATA_TRACE_WGS * 32];
#define HATA_TRACE_AT(slot, cond)                                                          \
    do {                                                                                   \
        if (threadIdx.x == 0 && (cond) && blockIdx.x < HATA_TRACE_WGS)                     \
            g_hata_trace[blockIdx.x * 32 + ((slot) & 31)] = wall_clock64();                \
    } while (0)
#else
#define HATA_TRACE_AT(slot, cond) do { } while (0)
#endif
