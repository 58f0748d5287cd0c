// Cooperative decode step: Hamming scoring, top-k selection and attention over the selected rows
// (Alg. 3 of the paper from "Calculate distance in Hamming space" to the sparse attention output)
// in ONE launch.
//
// grid = n_chunks * Hkv * B workgroups; the workgroup of (unit u, chunk c)
//   0. hash-encodes its share of the unit's query vectors, publishes the code words and collects
//      the others' (the owner of the appended row also encodes that key);
//   1. scores its chunk of cached key codes (as score_kernel does), keeps the scores in LDS,
//      publishes the chunk histogram and adds it to the unit histogram, then ARRIVES at the unit;
//   2. the last workgroup of the unit to arrive computes the unit's threshold and the ordered
//      chunk offsets (unit_threshold) and publishes an epoch flag; the others WAIT for that flag --
//      and meanwhile list their chunk's candidates (the keys up to a score taken from the chunk's own
//      histogram), so that the selection is a filter over a short list once the threshold is there;
//   3. compacts its own chunk (ordered, from the LDS scores) -- writing its part of Idx -- and
//      attends over exactly the rows it selected, for all query heads of the group;
//   4. writes its partial (max, sum, weighted V) and arrives; the first min(G, nc) workgroups of the
//      unit wait for all arrivals and merge one query head each (with one head per KV head: the
//      last workgroup to arrive merges).
// So the scores never make a round trip through memory for the selection, and the only serial
// pieces are the threshold tail and the merge.
// What workgroups poll or bump lives on cache lines of its own per unit / per chunk (counters,
// records, one copy of the query code words per chunk): polls and arrivals that share lines across
// units queue behind each other at the memory side.
//
// The waits need every workgroup of a unit to be running; the host launches this kernel
// only when the whole grid can be resident at once.  The wait is bounded anyway: a workgroup that
// gives up sets the context's error word and runs to its end, so every wave always terminates.
#include "hata_attn_core.h"
#include "hata_device.h"
#include "hata_internal.h"
#include "hata_select.h"
#include "hata_trace.h"

namespace hata {

#define HATA_COOP_MAX_CHUNK 32768        // keys per workgroup: their scores stay in LDS (2 bytes each)
#define HATA_COOP_SUB 4096               // chunks above this size run the BIG instantiation (more than 16 keys per thread in the compaction)
#define HATA_COOP_SPIN_LIMIT (1 << 18)  // default bound of every in-kernel wait (polls, ~0.1 us apart at least)

struct CoopArgs {
    const uint16_t* q;
    const uint16_t* K;
    const uint16_t* V;
    const float* W_H;
    uint32_t* qcodes;
    uint32_t* codes;
    const int32_t* seq_len;
    const int32_t* kbud;
    uint16_t* scores;
    int32_t* idx;
    uint16_t* chunk_hist;
    int32_t* chunk_info;
    int32_t* unit_info;
    uint32_t* unit_counter;
    uint32_t* unit_hist;
    unsigned long long* rec;
    unsigned long long* qrec;
    uint32_t* attn_counter;
    uint32_t* error_word;
    float* partials;
    uint16_t* out;
    float* out_f32;
    int Hq, Hkv, L_cap, k_max, chunk, n_chunks, NB, NBP, units;
    int64_t sb, sh, sn;
    float scale_log2;
    uint32_t epoch;
    int append;
    int spin_limit;
    int prefetch;     // fetch the first batch of key codes before the query codes are known
    int keep_scores;  // also write the score array (a by-product the kernel itself never reads back)
    int par_merge;    // the heads of a unit are merged side by side by several of its workgroups
    int cmajor;       // workgroup order: chunk-major (every unit's chunk 0 first) instead of unit-major
    int select_only;  // stop after the index lists are written (no attention, no output)
    hata::PageView pv;  // block table (used by the PAGED instantiations only)
};

// the kernel's argument block as it lies in memory (the only argument of the kernel is a CoopArgs)
__device__ __forceinline__ const CoopArgs* coop_args_in_memory() {
#if defined(__HIP_DEVICE_COMPILE__)
    return (const CoopArgs*)__builtin_amdgcn_kernarg_segment_ptr();
#else
    return nullptr;
#endif
}

template <int WD>
struct CodeW { uint32_t w[WD]; };

template <int WD>
__device__ __forceinline__ CodeW<WD> coop_load_code(const uint32_t* p) {
    CodeW<WD> c;
    if constexpr (WD == 1) {
        c.w[0] = p[0];
    } else if constexpr (WD == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        c.w[0] = v.x; c.w[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < WD / 4; ++i) {
            const uint4 v = reinterpret_cast<const uint4*>(p)[i];
            c.w[4 * i] = v.x; c.w[4 * i + 1] = v.y; c.w[4 * i + 2] = v.z; c.w[4 * i + 3] = v.w;
        }
    }
    return c;
}


// x + y across a lane pair that differs in lane bit 5 (swap32) or bit 4 (swap16): the lane with the
// bit clear gets the pair's total of x, the lane with the bit set the pair's total of y (one
// lane-swap per dword instead of two moves, and the number of live values halves).
__device__ __forceinline__ double swapadd32(double x, double y) {
    uint32_t xl = (uint32_t)__double2loint(x), xh = (uint32_t)__double2hiint(x);
    uint32_t yl = (uint32_t)__double2loint(y), yh = (uint32_t)__double2hiint(y);
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_permlane32_swap_b32 %2, %3\n\ts_nop 1"
                 : "+v"(xl), "+v"(yl), "+v"(xh), "+v"(yh));
    return __hiloint2double((int)xh, (int)xl) + __hiloint2double((int)yh, (int)yl);
}
__device__ __forceinline__ double swapadd16(double x, double y) {
    uint32_t xl = (uint32_t)__double2loint(x), xh = (uint32_t)__double2hiint(x);
    uint32_t yl = (uint32_t)__double2loint(y), yh = (uint32_t)__double2hiint(y);
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\tv_permlane16_swap_b32 %2, %3\n\ts_nop 1"
                 : "+v"(xl), "+v"(yl), "+v"(xh), "+v"(yh));
    return __hiloint2double((int)xh, (int)xl) + __hiloint2double((int)yh, (int)yl);
}
// x + (x of the lane N positions further round the same row of 16 lanes); N = 8, then 4, then 2
// sums over the lanes that agree in the low bits
template <int N>
__device__ __forceinline__ double rotadd(double x) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), 0x120 + N, 0xf, 0xf, false);  // row_ror:N
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), 0x120 + N, 0xf, 0xf, false);
    return x + __hiloint2double(hi, lo);
}

// HashEncode (Alg. 2: Sign(x . W_H), BitPack) of ONE 128-channel bf16 vector x against a KV head's
// weights Wh [128][r], by the whole workgroup, accumulating in fp64 (every product of a bf16 and
// an fp32 value is exact in fp64).  s_word: WD code words in LDS, zero on entry, complete after
// the caller's next barrier.  A wave owns r/4 hash columns (one code word at r = 128, two at
// r = 256, half / a quarter of one below); its lanes are (column group of 4 = one 128-bit weight load) x (1024/r parts of the
// channel range), so all loads of a thread are independent and in flight together.  The partial
// sums are combined across the parts with lane swaps, each step halving the live values: lane
// (bit5, bit4) ends up with the total of column 4 cg + bit4 + 2 bit5.
template <int WD>
struct EncodeLoads {  // what coop_encode_vec needs before its first FMA
    static constexpr int CP = HATA_D / (64 / (WD * 2));  // channels per part: 4, 8, 16, 32 for r = 32 .. 256
    static constexpr int NW = CP < 16 ? CP : 16;
    float4 w[NW];         // first (up to) 16 weight rows of this lane's channel part
    uint32_t xw[CP / 2];  // the part's channels of x, bf16 pairs
};
template <int WD>
__device__ __forceinline__ void coop_encode_load(const float* __restrict__ Wh,
                                                 const uint16_t* __restrict__ x, EncodeLoads<WD>& e) {
    constexpr int R = WD * 32, CG = R / 16, P = 64 / CG, CP = HATA_D / P;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cg = lane % CG, p = lane / CG;
    const float* wp = Wh + (int64_t)(p * CP) * R + wave * (R / 4) + 4 * cg;
    if constexpr (CP == 4) {
        const uint2 v = *reinterpret_cast<const uint2*>(x + p * CP);
        e.xw[0] = v.x; e.xw[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < CP / 8; ++i) {
            const uint4 v = reinterpret_cast<const uint4*>(x + p * CP)[i];
            e.xw[4 * i] = v.x; e.xw[4 * i + 1] = v.y; e.xw[4 * i + 2] = v.z; e.xw[4 * i + 3] = v.w;
        }
    }
#pragma unroll
    for (int j = 0; j < EncodeLoads<WD>::NW; ++j) e.w[j] = *reinterpret_cast<const float4*>(wp + (int64_t)j * R);
}
// the channels of x alone (for a further vector once the weight part is in registers: NW == CP)
template <int WD>
__device__ __forceinline__ void coop_encode_load_x(const uint16_t* __restrict__ x, uint32_t* xw) {
    constexpr int R = WD * 32, CG = R / 16, P = 64 / CG, CP = HATA_D / P;
    const int p = (threadIdx.x & 63) / CG;
    if constexpr (CP == 4) {
        const uint2 v = *reinterpret_cast<const uint2*>(x + p * CP);
        xw[0] = v.x; xw[1] = v.y;
    } else {
#pragma unroll
        for (int i = 0; i < CP / 8; ++i) {
            const uint4 v = reinterpret_cast<const uint4*>(x + p * CP)[i];
            xw[4 * i] = v.x; xw[4 * i + 1] = v.y; xw[4 * i + 2] = v.z; xw[4 * i + 3] = v.w;
        }
    }
}
template <int WD>
__device__ __forceinline__ void coop_encode_vec(const float* __restrict__ Wh, const EncodeLoads<WD>& e,
                                                uint32_t* s_word) {
    constexpr int R = WD * 32, CG = R / 16, P = 64 / CG, CP = HATA_D / P;  // CP = 4 .. 32 channels
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cg = lane % CG, p = lane / CG;
    const float* wp = Wh + (int64_t)(p * CP) * R + wave * (R / 4) + 4 * cg;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    auto fma_row = [&](const float4& w, int ch) {
        const uint32_t pair = e.xw[ch >> 1];
        const double xd = (double)((ch & 1) ? bf16_hi(pair) : bf16_lo(pair));
        a0 = fma((double)w.x, xd, a0);
        a1 = fma((double)w.y, xd, a1);
        a2 = fma((double)w.z, xd, a2);
        a3 = fma((double)w.w, xd, a3);
    };
#pragma unroll
    for (int j = 0; j < EncodeLoads<WD>::NW; ++j) fma_row(e.w[j], j);
    // r = 256: the part's other 16 weight rows, 8 at a time (registers)
#pragma unroll
    for (int c0 = 16; c0 < CP; c0 += 8) {
        float4 w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = *reinterpret_cast<const float4*>(wp + (int64_t)(c0 + j) * R);
#pragma unroll
        for (int j = 0; j < 8; ++j) fma_row(w[j], c0 + j);
    }
    const int b5 = lane >> 5, b4 = (lane >> 4) & 1;
    const int col = wave * (R / 4) + 4 * cg + b4 + 2 * b5;  // hash column this lane ends up with
    const double ev = swapadd32(a0, a2);  // column 0 + 2 b5
    const double od = swapadd32(a1, a3);  // column 1 + 2 b5
    double t = swapadd16(ev, od);
    // the remaining part bits (lane bits 3, 2, 1 for r = 128, 64, 32) by rotations inside the row
    if (P >= 8) t = rotadd<8>(t);
    if (P >= 16) t = rotadd<4>(t);
    if (P >= 32) t = rotadd<2>(t);
    if (t >= 0.0) atomicOr(&s_word[col >> 5], 1u << (col & 31));
}

// WD in {1, 2, 4, 8} (r = 32, 64, 128, 256); G in {1, 2, 4, 5, 8, 16} (all heads of the group in one
// attention tile; 16 only up to r = 128: one wave collects the G * WD <= 64 query code words)
// BIG: chunks of more than HATA_COOP_SUB keys (a thread of the ordered compaction then holds up to 128
// keys as eight mask words; kept out of the other instantiation, whose registers are tighter)
// (registers: at least three workgroups per CU, two with sixteen heads; at r = 256 also at most
// three -- with the scores in dynamic LDS the compiler would otherwise squeeze that form into the
// registers of a fourth, which costs it 1.3 us; the narrower forms fit four as they are, and a batch of
// 128 units at 4096 keys per chunk needs the four)
template <int WD, int G, bool PAGED, bool BIG = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((G >= 16 ? 2 : 3), (WD >= 8 ? 3 : 4))))
void decode_step_coop_kernel(const CoopArgs a) {
    static_assert(G * WD <= 64, "query code words of a unit are collected by one wave");
    // dynamic LDS: the chunk's scores (2 bytes per key; later the selected rows as offsets in the
    // chunk) at a fixed address, then NB words of histogram (the chunk's, later the unit's total)
    extern __shared__ __attribute__((aligned(16))) uint16_t s_sc[];
    uint32_t* const hist = reinterpret_cast<uint32_t*>(s_sc + a.chunk);
    constexpr bool MFMA = G >= 4;  // matrix-core form of the attention core
    // the threshold search (last arriver only) is over before the attention stages V tiles
    __shared__ __attribute__((aligned(16))) union {
        ThresholdLds ts;
        uint16_t vt[MFMA ? HATA_VT_ELEMS : 8];
    } U;
    ThresholdLds& TS = U.ts;
    __shared__ __attribute__((aligned(16))) AttnLds<G> S;
    __shared__ uint32_t scan4[4];
    __shared__ int s_flag;
    __shared__ uint32_t s_rec[2];
    __shared__ int s_low;  // lowest score of this chunk
    __shared__ int s_bad;  // this workgroup gave up a wait: the unit's outputs are invalid
    __shared__ uint32_t s_codes[(G + 1) * WD];  // codes of the G query heads and of the appended key
    // PAGED: where the pages of this chunk's rows start (pages of 16 rows or more: at most chunk / 16 + 1)
    __shared__ int s_page[PAGED ? (BIG ? HATA_COOP_MAX_CHUNK : HATA_COOP_SUB) / 16 + 2 : 1];
    const int tid = threadIdx.x;
    HATA_TRACE_AT(39, true);
    // Workgroup -> (unit, chunk).  Consecutive workgroup ids go to consecutive XCDs (8 of them, each
    // with its own L2); when the unit count allows, all chunks of a unit get ids that are equal
    // mod 8, so one L2 serves the unit's hash weights and the data its workgroups exchange.  Within
    // an XCD the order is chunk-major when the whole grid is resident: workgroups start in index
    // order, so every unit's chunk 0 .. G-1 -- the ones that encode the query vectors everybody waits
    // for -- start first, and the chunks past the end of short sequences, which return at once,
    // start last (measured against unit-major: 2 us per step with 32 and with 128 units).
    int64_t u;
    int c;
    if (a.units % 8 == 0) {
        const int j = blockIdx.x >> 3;
        if (a.cmajor) {
            const int ug = a.units >> 3;  // groups of 8 units
            u = (int64_t)(j % ug) * 8 + (blockIdx.x & 7);
            c = j / ug;
        } else {
            u = (int64_t)(j / a.n_chunks) * 8 + (blockIdx.x & 7);
            c = j % a.n_chunks;
        }
    } else {
        u = blockIdx.x / a.n_chunks;
        c = blockIdx.x % a.n_chunks;
    }
    const int b = (int)(u / a.Hkv), h = (int)(u % a.Hkv);
    // the query vector this workgroup will encode first (vector c, if c < G) does not depend on the
    // sequence length: its loads go out before anything else
    const uint16_t* qv = a.q + ((int64_t)b * a.Hq + h * G) * HATA_D;
    const float* Wh = a.W_H + (int64_t)h * HATA_D * (WD * 32);
    EncodeLoads<WD> el;
    constexpr bool EARLY = WD <= 4;  // (at r = 256 the second half of the weights needs the registers)
    if (EARLY && c < G) coop_encode_load<WD>(Wh, qv + c * HATA_D, el);
    const int base = c * a.chunk;
    const int blk0 = PAGED ? base >> a.pv.shift : 0;  // first block of the sequence this chunk touches
    // PAGED: the chunk's block-table entries are fetched alongside the sequence length (one entry
    // per thread covers every case: at most MAX_CHUNK / 16 = 256 blocks when pages are small and
    // therefore aligned with the chunk, a handful when they are large)
    int nblk = 0, my_page = 0;
    if constexpr (PAGED) {
        nblk = min(((base + a.chunk - 1) >> a.pv.shift) + 1, a.pv.max_blocks) - blk0;
        if (threadIdx.x < nblk) my_page = a.pv.table[(int64_t)b * a.pv.max_blocks + blk0 + threadIdx.x];
    }
    const int L = clampi(a.seq_len[b], 0, PAGED ? min(a.L_cap, a.pv.max_blocks << a.pv.shift) : a.L_cap);
    // Row n of the unit (a row of this chunk when PAGED) -> its row in the code array, in rows of
    // one (sequence or page, head): the contiguous cache is [B, Hkv, L_cap], the pools are
    // [n_pages, Hkv, page_rows] with K and V rows of exactly d elements.
    // (s_page holds, per block, the pool row at which this head's part of the page starts: a
    // 32-bit number, the host has checked that the pools have fewer than 2^31 rows)
    auto row_in_page = [&](int page_row0, int n) -> int64_t {
        return (int64_t)(page_row0 + (n & ((1 << a.pv.shift) - 1)));
    };
    auto cache_row = [&](int n) -> int64_t {
        if constexpr (PAGED) return row_in_page(s_page[(n >> a.pv.shift) - blk0], n);
        else return u * a.L_cap + n;
    };
    const int hq0 = h * G;
    uint16_t* outp = a.out + ((int64_t)b * a.Hq + hq0) * HATA_D;
    float* outp32 = a.out_f32 ? a.out_f32 + ((int64_t)b * a.Hq + hq0) * HATA_D : nullptr;
    if (base >= L && c != 0) return;  // chunk 0 always runs the encoding (it publishes the query codes)
#define TC(i) HATA_TRACE_AT(i, true)
#define TU(i) HATA_TRACE_AT(i, true)
    TC(40);
    const int end = min(base + a.chunk, L);
    // ---- 0. HashEncode(Q) and HashEncode(K_new).  The G query vectors of the unit are dealt out
    // to its nc workgroups (vector v to chunk v mod nc), each published as epoch-stamped words
    // that every workgroup of the unit then picks up; the workgroup whose chunk holds the
    // appended row L - 1 also encodes that key, updates the code cache and scores the row from
    // the code it just computed.
    const int nc = (L + a.chunk - 1) / a.chunk;
    const bool own = a.append && L > 0 && base <= L - 1 && L - 1 < base + a.chunk;
    const int end_main = own ? L - 1 : end;  // the owner scores row L - 1 from the code it computes
    constexpr int UNR = (WD <= 2) ? 16 : (WD <= 4) ? 8 : 4;  // 64-128 B of codes in flight per lane
    CodeW<WD> kc[UNR];
    // codes of rows n0, n0 + 256, ... (those below `stop`) into kc; PAGED: all page lookups first,
    // so that the loads go out together instead of one per LDS round trip
    auto load_codes = [&](int n0, int stop) {
        if constexpr (PAGED) {
            int pg[UNR];
#pragma unroll
            for (int j = 0; j < UNR; ++j)
                pg[j] = s_page[(max(min(n0 + j * 256, stop - 1), base) >> a.pv.shift) - blk0];
#pragma unroll
            for (int j = 0; j < UNR; ++j) {
                const int n = n0 + j * 256;
                if (n < stop) kc[j] = coop_load_code<WD>(a.codes + row_in_page(pg[j], n) * WD);
            }
        } else {
#pragma unroll
            for (int j = 0; j < UNR; ++j) {
                const int n = n0 + j * 256;
                if (n < stop) kc[j] = coop_load_code<WD>(a.codes + cache_row(n) * WD);
            }
        }
    };
    {
        // every chunk of the unit has its own copy of the G * WD published words (the encoders write
        // all copies, a workgroup polls -- and afterwards clears -- only its own)
        unsigned long long* qrec_u = a.qrec + u * a.n_chunks * (G * WD);
        unsigned long long* qrec = qrec_u + c * (G * WD);
        if (tid < (G + 1) * WD) s_codes[tid] = 0;
        if (tid == 0) { s_low = a.NB; s_bad = 0; }
        for (int i = tid; i < a.NB; i += 256) hist[i] = 0;
        if constexpr (PAGED) {
            if (tid < nblk) s_page[tid] = (clampi(my_page, 0, a.pv.n_pages - 1) * a.Hkv + h) << a.pv.shift;
            for (int i = tid + 256; i < nblk; i += 256)
                s_page[i] = (clampi(a.pv.table[(int64_t)b * a.pv.max_blocks + blk0 + i], 0, a.pv.n_pages - 1) * a.Hkv + h)
                            << a.pv.shift;
        }
        __syncthreads();
        auto publish = [&](int v) {
            __syncthreads();
            for (int i = tid; i < WD * max(nc, 1); i += 256)
                __hip_atomic_store(qrec_u + (i / WD) * (G * WD) + v * WD + i % WD,
                                   ((unsigned long long)a.epoch << 32) | s_codes[v * WD + i % WD],
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        const uint16_t* kx = !own ? nullptr
                             : PAGED ? a.K + cache_row(L - 1) * HATA_D
                                     : a.K + b * a.sb + h * a.sh + (int64_t)(L - 1) * a.sn;
        if constexpr (BIG && EncodeLoads<WD>::NW == EncodeLoads<WD>::CP) {
            // Large chunks mean few chunks per unit, so a workgroup has several vectors to encode (fewer
            // chunks than heads in the group, and the appended key on top).  The lane's weight part stays
            // in registers (r <= 128): the workgroup loads the weights once, and the channels of the
            // NEXT vector while it works on the current one.
            // Items: query vectors c, c + nc, ... < G, then the appended key (index G) if it is ours.
            const int stepv = max(nc, 1);
            int v = c < G ? c : (own ? G : G + 1);
            if (v <= G && !(EARLY && c < G)) coop_encode_load<WD>(Wh, v < G ? qv + v * HATA_D : kx, el);
#pragma clang loop unroll(disable)
            while (v <= G) {
                const int vn = v == G ? G + 1 : (v + stepv < G ? v + stepv : (own ? G : G + 1));
                uint32_t xn[EncodeLoads<WD>::CP / 2];
                if (vn <= G) coop_encode_load_x<WD>(vn < G ? qv + vn * HATA_D : kx, xn);
                // (the weights are loop-invariant: without this the compiler keeps their fp64 conversions,
                // twice the registers, across the loop)
#pragma unroll
                for (int j = 0; j < EncodeLoads<WD>::NW; ++j)
                    asm volatile("" : "+v"(el.w[j].x), "+v"(el.w[j].y), "+v"(el.w[j].z), "+v"(el.w[j].w));
                coop_encode_vec<WD>(Wh, el, &s_codes[v * WD]);
                if (v < G) publish(v);
                if (vn <= G) {
#pragma unroll
                    for (int i = 0; i < EncodeLoads<WD>::CP / 2; ++i) el.xw[i] = xn[i];
                }
                v = vn;
            }
        } else {
            for (int v = c; v < G; v += max(nc, 1)) {
                if (!EARLY || v != c) coop_encode_load<WD>(Wh, qv + v * HATA_D, el);
                coop_encode_vec<WD>(Wh, el, &s_codes[v * WD]);
                publish(v);
            }
            if (own) {
                coop_encode_load<WD>(Wh, kx, el);
                coop_encode_vec<WD>(Wh, el, &s_codes[G * WD]);
            }
        }
        // Small grids (at most one workgroup per CU: the step is a chain of latencies, not a stream):
        // the first batch of the chunk's key codes is fetched while the query codes are collected.
        // With more workgroups per CU these loads would only queue in front of the encoders' own.
        if (a.prefetch) {
            __builtin_amdgcn_sched_barrier(0);
            load_codes(base + tid, end_main);
        }
        if (tid < 64) {  // one wave collects the G * WD (<= 64) query code words of the unit
            const int i = min(tid, G * WD - 1);
            int budget = a.spin_limit;
            unsigned long long r;
            for (;;) {
                r = __hip_atomic_load(qrec + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const bool miss = (uint32_t)(r >> 32) != a.epoch;
                if (__builtin_amdgcn_ballot_w64(miss) == 0ull) break;
                if (--budget <= 0) { if (tid == 0) { a.error_word[0] = 1u; s_bad = 1; } break; }  // gave up: results invalid
                __builtin_amdgcn_s_sleep(1);
            }
            if (tid < G * WD) {
                s_codes[tid] = (uint32_t)r;
                // retired at once: a later launch that carries the SAME epoch (a replay of a captured
                // HIP graph freezes the kernel arguments) must not mistake these words for its own
                qrec[tid] = 0ull;
            }
        }
        __syncthreads();
    }
    if (c == 0)
        for (int i = tid; i < G * WD; i += 256) a.qcodes[((int64_t)b * a.Hq + hq0) * WD + i] = s_codes[i];
    if (own && tid < WD) a.codes[cache_row(L - 1) * WD + tid] = s_codes[G * WD + tid];
    if (base >= L) {  // empty sequence: nothing selected, zero output
        for (int i = tid; i < (a.select_only ? 0 : G * HATA_D); i += 256) {
            outp[i] = 0;
            if (outp32) outp32[i] = 0.f;
        }
        for (int p = tid; p < a.k_max; p += 256) a.idx[u * a.k_max + p] = -1;
        return;
    }
    TC(50);
    const int keff = min(clampi(a.kbud[b], 0, a.k_max), L);
    // ---- 1. score the chunk (the appended row from the code just computed, the rest from the cache)
    // wave-uniform query codes: as they are, or as bit-count planes for the larger groups
    constexpr bool PLANES = HammingSum<WD, G>::PLANES;
    HammingSum<WD, G> dist;
    uint32_t qc[PLANES ? 1 : G][WD];
    if constexpr (PLANES) {
        dist.init(s_codes);
    } else {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int w = 0; w < WD; ++w) qc[g][w] = __builtin_amdgcn_readfirstlane(s_codes[g * WD + w]);
    }
    auto distance = [&](const uint32_t (&k)[WD]) {
        if constexpr (PLANES) {
            return dist(k);
        } else {
            uint32_t s = 0;
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int w = 0; w < WD; ++w) s += __popc(qc[g][w] ^ k[w]);
            return s;
        }
    };
    {
        uint16_t* sp = a.scores + u * a.L_cap;
        uint32_t low = 0xffffu;  // lowest score this thread sees
        for (int n0 = base + tid; n0 < end_main; n0 += 256 * UNR) {
            if (!a.prefetch || n0 != base + tid) load_codes(n0, end_main);  // (the first batch may be in the registers already)
#pragma unroll
            for (int j = 0; j < UNR; ++j) {
                const int n = n0 + j * 256;
                if (n < end_main) {
                    const uint32_t s = distance(kc[j].w);
                    if (a.keep_scores) sp[n] = (uint16_t)s;
                    s_sc[n - base] = (uint16_t)s;
                    atomicAdd(&hist[s], 1u);
                    low = min(low, s);
                }
            }
        }
        low = (uint32_t)(-wave_max64(-(float)low));  // (scores <= 4096 are exact in fp32)
        if ((tid & 63) == 0 && low < (uint32_t)a.NB) atomicMin(&s_low, (int)low);
        if (own && tid == 0) {
            uint32_t kw[WD];
#pragma unroll
            for (int w = 0; w < WD; ++w) kw[w] = s_codes[G * WD + w];
            const uint32_t s = distance(kw);
            if (a.keep_scores) sp[L - 1] = (uint16_t)s;
            s_sc[L - 1 - base] = (uint16_t)s;
            atomicAdd(&hist[s], 1u);
            atomicMin(&s_low, (int)s);
        }
    }
    __syncthreads();
    TC(41);
    // ---- 2. publish the histogram, arrive at the unit, threshold by the last arriver
    {
        uint32_t* hp32 = reinterpret_cast<uint32_t*>(a.chunk_hist + (u * a.n_chunks + c) * a.NBP);
        for (int i = tid; i < a.NBP / 2; i += 256) {
            const uint32_t lo = (2 * i < a.NB) ? hist[2 * i] : 0u;
            const uint32_t hi = (2 * i + 1 < a.NB) ? hist[2 * i + 1] : 0u;
            st_dev(hp32 + i, lo | (hi << 16));
        }
        for (int i = tid; i < a.NB; i += 256) {
            const uint32_t hv = hist[i];
            if (hv) atomicAdd(&a.unit_hist[u * a.NB + i], hv);
        }
    }
    TC(42);
    wait_stores();
    __syncthreads();
    TC(43);
    if (tid == 0) {
        const uint32_t done = atomicAdd(&a.unit_counter[u * HATA_COUNTER_STRIDE], 1u);
        const int last = (done == (uint32_t)(nc - 1));
        if (last) a.unit_counter[u * HATA_COUNTER_STRIDE] = 0;
        s_flag = last;
    }
    __syncthreads();
    int32_t* ci_u = a.chunk_info + u * (a.n_chunks + 1) * 2;
    unsigned long long* rec_u = a.rec + u * a.n_chunks * HATA_REC_STRIDE;
    TC(44);
    // query fragments for the attention: in flight across the wait below
    uint32_t qr[MFMA ? 1 : G][4];
    uint4 qb[4];
    if constexpr (MFMA) attn_load_q_mfma<G>(a.q + ((int64_t)b * a.Hq + hq0) * HATA_D, qb);
    else attn_load_q<G>(a.q + ((int64_t)b * a.Hq + hq0) * HATA_D, qr);
    if (s_flag) {
        TU(51);
        unit_threshold<(G * WD * 32) / 256 + 1>(a.chunk_hist + u * a.n_chunks * a.NBP, a.unit_hist + u * a.NB, nc, keff,
                             a.NB, a.NBP, ci_u, a.unit_info + u * 2, hist, TS, rec_u, a.epoch,
                             s_low < a.NB ? s_low : -1);
        TU(52);
    }
    // While the unit's threshold is on its way (the last arriver computes it, everybody else would only
    // wait): an ordered list of the chunk's CANDIDATES, the keys up to a score Tc chosen from the chunk's
    // own histogram so that the list holds about twice the chunk's share of the budget.  If the unit's
    // threshold turns out to be at most Tc -- the rule -- the selection is a filter over this short
    // list instead of a pass over the whole chunk.  The list lives where the last arriver keeps its
    // threshold search and the attention later stages V (neither is in use by this workgroup now).
    constexpr int CAND_MAX = 1024;
    uint32_t* const s_cand = reinterpret_cast<uint32_t*>(&U);
    __shared__ int s_Tc, s_ncand;
    {
        if (tid == 0) { s_Tc = -1; s_ncand = 0; }
        if (!s_flag) {
            const int n_keys = end - base;
            const int want = min(n_keys, (int)(((int64_t)keff * n_keys + L - 1) / L) * 2 + 64);
            // smallest score whose inclusive count reaches `want`: thread t owns seg consecutive bins
            const int seg = (a.NB + 255) / 256;
            uint32_t loc = 0;
            for (int j = 0; j < seg; ++j) loc += (tid * seg + j < a.NB) ? hist[tid * seg + j] : 0u;
            const uint32_t incl = wave_incl_scan(loc);
            if ((tid & 63) == 63) scan4[tid >> 6] = incl;
            __syncthreads();
            const int wv = tid >> 6;
            uint32_t run = (wv > 0 ? scan4[0] : 0u) + (wv > 1 ? scan4[1] : 0u) + (wv > 2 ? scan4[2] : 0u) + incl - loc;
            if (run < (uint32_t)want && run + loc >= (uint32_t)want) {
                for (int j = 0; j < seg; ++j) {
                    const uint32_t hv = (tid * seg + j < a.NB) ? hist[tid * seg + j] : 0u;
                    if (run < (uint32_t)want && run + hv >= (uint32_t)want) { s_Tc = tid * seg + j; s_ncand = (int)(run + hv); }
                    run += hv;
                }
            }
            __syncthreads();
            const int Tc = s_Tc;
            if (Tc >= 0 && s_ncand <= CAND_MAX) {
                if constexpr (BIG) {
                    // (16 keys at a time, as the one-pass compaction of these chunks below)
                    const int kpt = a.chunk / 256;
                    const int n_first = tid * kpt;
                    uint32_t mc[8];
                    uint32_t cn = 0;
#pragma unroll
                    for (int g = 0; g < 8; ++g) {
                        mc[g] = 0;
                        if (g * 16 < kpt) {
                            const uint4 v0 = *reinterpret_cast<const uint4*>(&s_sc[n_first + g * 16]);
                            const uint4 v1 = *reinterpret_cast<const uint4*>(&s_sc[n_first + g * 16 + 8]);
                            const uint32_t w8[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                            uint32_t m = 0;
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                const int sc = (int)((i & 1) ? (w8[i >> 1] >> 16) : (w8[i >> 1] & 0xffffu));
                                m |= (sc <= Tc ? 1u : 0u) << i;
                            }
                            const int nlive = clampi(end - base - n_first - g * 16, 0, 16);
                            mc[g] = m & ((1u << nlive) - 1u);
                            cn += __popc(mc[g]);
                        }
                    }
                    const uint32_t cincl = wave_incl_scan(cn);
                    __syncthreads();  // (scan4 is free again)
                    if ((tid & 63) == 63) scan4[tid >> 6] = cincl;
                    __syncthreads();
                    uint32_t r = (wv > 0 ? scan4[0] : 0u) + (wv > 1 ? scan4[1] : 0u) + (wv > 2 ? scan4[2] : 0u) + cincl - cn;
#pragma unroll
                    for (int g = 0; g < 8; ++g) {
                        uint32_t m = mc[g];
                        while (m) {
                            const int n = n_first + g * 16 + __ffs(m) - 1;
                            m &= m - 1;
                            if (r < (uint32_t)CAND_MAX) s_cand[r] = (uint32_t)n | ((uint32_t)s_sc[n] << 16);
                            ++r;
                        }
                    }
                } else {
                    const int kpt = a.chunk / 256;
                    const int n_first = tid * kpt;
                    uint32_t sv[16];
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        if (i4 * 4 < kpt) {
                            const uint2 v = *reinterpret_cast<const uint2*>(&s_sc[n_first + i4 * 4]);
                            sv[4 * i4 + 0] = v.x & 0xffffu; sv[4 * i4 + 1] = v.x >> 16;
                            sv[4 * i4 + 2] = v.y & 0xffffu; sv[4 * i4 + 3] = v.y >> 16;
                        } else {
                            sv[4 * i4 + 0] = sv[4 * i4 + 1] = sv[4 * i4 + 2] = sv[4 * i4 + 3] = 0xffffffffu;
                        }
                    }
                    const int nlive = clampi(end - base - n_first, 0, kpt);
                    uint32_t m_c = 0;
#pragma unroll
                    for (int i = 0; i < 16; ++i) m_c |= ((int)sv[i] <= Tc ? 1u : 0u) << i;
                    m_c &= (1u << nlive) - 1u;
                    const uint32_t cn = __popc(m_c);
                    const uint32_t cincl = wave_incl_scan(cn);
                    __syncthreads();  // (scan4 is free again)
                    if ((tid & 63) == 63) scan4[tid >> 6] = cincl;
                    __syncthreads();
                    uint32_t r = (wv > 0 ? scan4[0] : 0u) + (wv > 1 ? scan4[1] : 0u) + (wv > 2 ? scan4[2] : 0u) + cincl - cn;
                    while (m_c) {
                        const int i = __ffs(m_c) - 1;
                        m_c &= m_c - 1;
                        if (r < (uint32_t)CAND_MAX) s_cand[r] = (uint32_t)(n_first + i) | (sv[i] << 16);
                        ++r;
                    }
                }
            } else if (tid == 0) {
                s_Tc = -1;
            }
        }
        __syncthreads();
    }
    // every workgroup (the last arriver too) picks up its chunk's record: two words that carry
    // this launch's epoch once the threshold of the unit has been published
    if (tid == 0) {
        int budget = a.spin_limit;
        unsigned long long r0, r1;
        for (;;) {
            r0 = __hip_atomic_load(rec_u + HATA_REC_STRIDE * c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r1 = __hip_atomic_load(rec_u + HATA_REC_STRIDE * c + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (((uint32_t)(r0 >> 32) == a.epoch && (uint32_t)(r1 >> 32) == a.epoch) || --budget <= 0) break;
            __builtin_amdgcn_s_sleep(1);
        }
        if (budget <= 0) { a.error_word[0] = 1u; s_bad = 1; r0 = 0; r1 = 0; }  // gave up: this launch's results are invalid
        s_rec[0] = (uint32_t)r0;
        s_rec[1] = (uint32_t)r1;
        // this workgroup is the record's only reader: retired at once (see the query code words above)
        rec_u[HATA_REC_STRIDE * c] = 0ull;
        rec_u[HATA_REC_STRIDE * c + 1] = 0ull;
    }
    __syncthreads();
    TC(45);
    const int off = clampi((int)(s_rec[0] >> 16), 0, a.k_max);
    const int cnt = clampi((int)(s_rec[0] & 0xffffu), 0, min(a.chunk, a.k_max - off));
    const int take = (int)(s_rec[1] >> 13);
    const int T = (int)(s_rec[1] & 0x1fffu);

    // ---- 3. ordered compaction of the own chunk from the LDS scores
    int32_t* io = a.idx + u * a.k_max;
    if (c == 0)
        for (int p = keff + tid; p < a.k_max; p += 256) io[p] = -1;
    if (s_Tc >= 0 && (T <= s_Tc || cnt == 0)) {
        // the candidate list covers the selection: a thread filters up to four consecutive candidates
        const int n_cand = s_ncand;
        const int cpt = (n_cand + 255) / 256;  // <= 4
        const int j0 = tid * cpt;
        uint32_t cw[4];
        uint32_t m_lt = 0, m_eq = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            cw[i] = (i < cpt && j0 + i < n_cand) ? s_cand[j0 + i] : 0xffff0000u;
            const int sc = (int)(cw[i] >> 16);
            const bool live = i < cpt && j0 + i < n_cand;
            m_lt |= (live && sc < T ? 1u : 0u) << i;
            m_eq |= (live && sc == T ? 1u : 0u) << i;
        }
        const uint32_t lt = __popc(m_lt), eq = __popc(m_eq);
        const uint32_t mine = lt | (eq << 16);
        const uint32_t incl = wave_incl_scan(mine);
        if ((tid & 63) == 63) scan4[tid >> 6] = incl;
        __syncthreads();
        const int wv = tid >> 6;
        const uint32_t before = (wv > 0 ? scan4[0] : 0u) + (wv > 1 ? scan4[1] : 0u) + (wv > 2 ? scan4[2] : 0u) + incl - mine;
        const uint32_t lt_b = before & 0xffffu, eq_b = before >> 16;
        const uint32_t ties_before = min(eq_b, (uint32_t)take);
        const uint32_t avail = min(eq, (uint32_t)take - ties_before);
        uint32_t keep = m_eq;
        while ((uint32_t)__popc(keep) > avail) keep &= ~(0x80000000u >> __clz(keep));
        uint32_t sel = m_lt | keep;
        uint32_t r = lt_b + ties_before;
        while (sel) {
            const int i = __ffs(sel) - 1;
            sel &= sel - 1;
            if (r < (uint32_t)cnt) {
                s_sc[r] = (uint16_t)(cw[i] & 0xffffu);
                io[off + r] = base + (int)(cw[i] & 0xffffu);
            }
            ++r;
        }
    } else if constexpr (BIG) {
        // chunks of 8192 .. 32768 keys: a thread takes kpt = 32 .. 128 consecutive keys, 16 at a time
        // (bits 0..15 of mk[g]: key below the threshold, bits 16..31: key at the threshold), then ONE
        // block-wide scan; the totals stay below 65536, so the packed (lt, eq) pair still fits
        const int kpt = a.chunk / 256;
        const int n_first = tid * kpt;  // offset in the chunk
        uint32_t mk[8];
        uint32_t lt = 0, eq = 0;
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            mk[g] = 0;
            if (g * 16 < kpt) {
                const uint4 v0 = *reinterpret_cast<const uint4*>(&s_sc[n_first + g * 16]);
                const uint4 v1 = *reinterpret_cast<const uint4*>(&s_sc[n_first + g * 16 + 8]);
                const uint32_t w8[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                uint32_t m_lt = 0, m_eq = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int sc = (int)((i & 1) ? (w8[i >> 1] >> 16) : (w8[i >> 1] & 0xffffu));
                    m_lt |= (sc < T ? 1u : 0u) << i;
                    m_eq |= (sc == T ? 1u : 0u) << i;
                }
                const int nlive = clampi(end - base - n_first - g * 16, 0, 16);
                const uint32_t live = (1u << nlive) - 1u;
                m_lt &= live;
                m_eq &= live;
                mk[g] = m_lt | (m_eq << 16);
                lt += __popc(m_lt);
                eq += __popc(m_eq);
            }
        }
        const uint32_t mine = lt | (eq << 16);
        const uint32_t incl = wave_incl_scan(mine);
        if ((tid & 63) == 63) scan4[tid >> 6] = incl;
        __syncthreads();  // (every thread has read its scores: s_sc becomes the row list)
        const int wv = tid >> 6;
        const uint32_t before = (wv > 0 ? scan4[0] : 0u) + (wv > 1 ? scan4[1] : 0u) + (wv > 2 ? scan4[2] : 0u) + incl - mine;
        const uint32_t lt_b = before & 0xffffu, eq_b = before >> 16;
        // ties go to the lowest rows: this thread may keep `ties_left` of its keys at the threshold
        const uint32_t ties_before = min(eq_b, (uint32_t)take);
        uint32_t ties_left = (uint32_t)take - ties_before;
        uint32_t r = lt_b + ties_before;  // local rank of the thread's first selected key
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            if (g * 16 < kpt) {
                uint32_t keep = mk[g] >> 16;
                const uint32_t avail = min((uint32_t)__popc(keep), ties_left);
                while ((uint32_t)__popc(keep) > avail) keep &= ~(0x80000000u >> __clz(keep));  // drop the highest row
                ties_left -= avail;
                uint32_t sel = (mk[g] & 0xffffu) | keep;
                while (sel) {
                    const int i = __ffs(sel) - 1;
                    sel &= sel - 1;
                    if (r < (uint32_t)cnt) {
                        s_sc[r] = (uint16_t)(n_first + g * 16 + i);
                        io[off + r] = base + n_first + g * 16 + i;
                    }
                    ++r;
                }
            }
        }
    } else {
        // chunks of up to HATA_COOP_SUB keys: a thread takes kpt <= 16 consecutive keys
        const int kpt = a.chunk / 256;  // consecutive keys per thread
        const int n_first = tid * kpt;  // offset in the chunk
        // this thread's scores (kpt <= 16 consecutive uint16), read once with 8-byte LDS loads
        uint32_t sv[16];
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            if (i4 * 4 < kpt) {
                const uint2 v = *reinterpret_cast<const uint2*>(&s_sc[n_first + i4 * 4]);
                sv[4 * i4 + 0] = v.x & 0xffffu; sv[4 * i4 + 1] = v.x >> 16;
                sv[4 * i4 + 2] = v.y & 0xffffu; sv[4 * i4 + 3] = v.y >> 16;
            } else {
                sv[4 * i4 + 0] = sv[4 * i4 + 1] = sv[4 * i4 + 2] = sv[4 * i4 + 3] = 0xffffffffu;
            }
        }
        // bit i of m_lt / m_eq: key i of this thread is live and scores below / exactly the threshold
        const int nlive = clampi(end - base - n_first, 0, kpt);
        const uint32_t live = (1u << nlive) - 1u;  // (nlive <= 16)
        uint32_t m_lt = 0, m_eq = 0;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            if (i4 * 4 < kpt) {
#pragma unroll
                for (int i = 4 * i4; i < 4 * i4 + 4; ++i) {
                    m_lt |= ((int)sv[i] < T ? 1u : 0u) << i;
                    m_eq |= ((int)sv[i] == T ? 1u : 0u) << i;
                }
            }
        }
        m_lt &= live;
        m_eq &= live;
        const uint32_t lt = __popc(m_lt), eq = __popc(m_eq);
        // block-wide exclusive scan of (lt, eq) with ONE barrier, which also marks the point where
        // every thread has read its scores, so that s_sc can become the row list
        uint32_t* sc4 = scan4;
        const uint32_t mine = lt | (eq << 16);
        const uint32_t incl = wave_incl_scan(mine);
        if ((tid & 63) == 63) sc4[tid >> 6] = incl;
        __syncthreads();
        const int wv = tid >> 6;
        const uint32_t before = (wv > 0 ? sc4[0] : 0u) + (wv > 1 ? sc4[1] : 0u) + (wv > 2 ? sc4[2] : 0u) + incl - mine;
        const uint32_t lt_b = before & 0xffffu, eq_b = before >> 16;
        // ties go to the lowest rows: this thread keeps the first `avail` of its keys at the threshold
        const uint32_t ties_before = min(eq_b, (uint32_t)take);  // ties taken by the threads before this one
        const uint32_t avail = min(eq, (uint32_t)take - ties_before);
        uint32_t keep = m_eq;
        while ((uint32_t)__popc(keep) > avail) keep &= ~(0x80000000u >> __clz(keep));  // drop the highest row
        uint32_t sel = m_lt | keep;
        uint32_t r = lt_b + ties_before;  // local rank of the thread's first selected key
        while (sel) {  // (a thread holds k / L of its keys on average: mostly zero or one turn)
            const int i = __ffs(sel) - 1;
            sel &= sel - 1;
            if (r < (uint32_t)cnt) {
                s_sc[r] = (uint16_t)(n_first + i);
                io[off + r] = base + n_first + i;
            }
            ++r;
        }
    }
    __syncthreads();
    TC(46);
    if (a.select_only) {
        // (a workgroup that gave up a wait poisons the unit's list as far as it can: peers that did
        // not give up may still write their slices afterwards, hata_check() reports the step)
        if (s_bad)
            for (int p = tid; p < a.k_max; p += 256) io[p] = -1;
        return;
    }
    // ---- 4. attention over the rows this chunk contributes
    if constexpr (PAGED) {  // rows of the pools (the host has checked that their count fits an int)
        auto row_of = [&](int row) { return (int)cache_row(base + (int)s_sc[row]); };
        const int rows = (a.pv.n_pages * a.Hkv) << a.pv.shift;
        if constexpr (MFMA) attn_rows_mfma<G, 1, false>(qb, a.K, a.V, HATA_D, rows, 0, cnt, a.scale_log2, row_of, S, U.vt);
        else attn_rows<G, 4>(qr, a.K, a.V, HATA_D, rows, 0, cnt, a.scale_log2, row_of, S);
    } else {
        const uint16_t* Kb = a.K + b * a.sb + h * a.sh;
        const uint16_t* Vb = a.V + b * a.sb + h * a.sh;
        auto row_of = [&](int row) { return base + (int)s_sc[row]; };
        if constexpr (MFMA) attn_rows_mfma<G, 1, false>(qb, Kb, Vb, a.sn, a.L_cap, 0, cnt, a.scale_log2, row_of, S, U.vt);
        else attn_rows<G, 4>(qr, Kb, Vb, a.sn, a.L_cap, 0, cnt, a.scale_log2, row_of, S);
    }
    TC(47);
    const int64_t head_stride = (int64_t)a.n_chunks * HATA_PSTRIDE;
    float* part0 = a.partials + ((int64_t)b * a.Hq + hq0) * head_stride;
    attn_emit<G>(S, nc == 1, outp, outp32, part0 + (int64_t)c * HATA_PSTRIDE, head_stride);
    // A wait that gave up leaves the unit without valid results.  That is made visible in the data
    // itself: the workgroup that writes a head's output overwrites it with NaN, and whoever writes
    // head 0 also sets the unit's index list to -1 (a caller that never calls hata_check() still
    // cannot mistake the step for a good one).  The arrival counter carries the news: bits 0..9
    // count arrivals, bits 10..19 the arrivals that had given up a wait, bits 20..31 the sign-offs.
    int hw_lo = G, hw_step = 1;  // the heads whose output this workgroup writes: hw_lo, hw_lo + hw_step, ... < G
    if (nc == 1) {
        hw_lo = 0;
    } else {
        TC(48);
        wait_stores();
        __syncthreads();
        uint32_t* cntp = a.attn_counter + u * HATA_COUNTER_STRIDE;
        const uint32_t arrival = 1u + (s_bad ? (1u << 10) : 0u);
        if (a.par_merge) {
            // Many slices x many heads: every workgroup arrives; the first nm = min(G, nc) workgroups
            // of the unit wait for all nc arrivals, sign off ("I no longer look at the counter") and
            // merge one query head each (heads c, c + nm, ...).  Whoever brings the counter to its final
            // value -- nc arrivals, nm sign-offs -- clears it.
            const int nm = min(G, nc);
            auto final_value = [&](uint32_t v) { return (v & 0x3ffu) == (uint32_t)nc && (v >> 20) == (uint32_t)nm; };
            if (tid == 0) {
                uint32_t seen = atomicAdd(cntp, arrival) + arrival;
                if (c >= nm) {
                    if (final_value(seen)) *cntp = 0;  // (possible only after a merging workgroup gave up its wait)
                } else {
                    int budget = a.spin_limit;
                    while ((seen & 0x3ffu) != (uint32_t)nc) {
                        if (--budget <= 0) { a.error_word[0] = 1u; s_bad = 1; break; }  // gave up: results invalid
                        __builtin_amdgcn_s_sleep(1);
                        seen = __hip_atomic_load(cntp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if ((seen >> 10) & 0x3ffu) s_bad = 1;  // some workgroup of the unit gave up a wait
                }
            }
            if (c >= nm) return;
            __syncthreads();
            // the sign-off goes out now and is looked at after the merge (one lane of the last wave: its
            // return value queues behind that lane's own partial loads)
            uint32_t signed_off = 0;
            if (tid == 255) signed_off = atomicAdd(cntp, 1u << 20) + (1u << 20);
            float* sm = &S.acc[0][0][0];
            for (int g = c; g < G; g += nm) {
                if (g != c) __syncthreads();  // the previous head's use of sm
                attn_merge_head<16>(sm, part0 + g * head_stride, nc, outp + g * HATA_D, outp32 ? outp32 + g * HATA_D : nullptr);
            }
            if (tid == 255 && final_value(signed_off)) *cntp = 0;
            hw_lo = c;
            hw_step = nm;
        } else {
            if (tid == 0) {
                const uint32_t done = atomicAdd(cntp, arrival);
                const int last = ((done & 0x3ffu) == (uint32_t)(nc - 1));
                if (last) *cntp = 0;
                if (done >> 10) s_bad = 1;
                s_flag = last;
            }
            __syncthreads();
            TC(49);
            if (!s_flag) return;
            TU(53);
            attn_merge<G>(S, part0, head_stride, nc, outp, outp32);
            hw_lo = 0;
        }
        TU(54);
    }
    if (s_bad) {
        // (a path that is never taken in a good launch: it reads the kernel arguments again from
        // the argument segment instead of keeping them in registers through the whole kernel)
        const CoopArgs* ka = coop_args_in_memory();
        const int u32 = (int)u;  // (at most 65535 units)
        const int b2 = u32 / ka->Hkv, h2 = u32 % ka->Hkv;
        for (int g = hw_lo; g < G; g += hw_step) {
            const int64_t o = ((int64_t)b2 * ka->Hq + h2 * G + g) * HATA_D;
            if (tid < HATA_D) {
                ka->out[o + tid] = 0x7fc0;
                if (ka->out_f32) ka->out_f32[o + tid] = __builtin_nanf("");
            }
            if (g == 0)
                for (int p = tid; p < ka->k_max; p += 256) ka->idx[u * ka->k_max + p] = -1;
        }
    }
#undef TC
#undef TU
}

template <int WD, int G>
static const void* coop_fn(bool paged, bool big) {
    if (paged) return big ? (const void*)&decode_step_coop_kernel<WD, G, true, true> : (const void*)&decode_step_coop_kernel<WD, G, true, false>;
    return big ? (const void*)&decode_step_coop_kernel<WD, G, false, true> : (const void*)&decode_step_coop_kernel<WD, G, false, false>;
}

static const void* coop_kernel_for(int Wd, int G, bool paged, bool big) {
    switch (Wd * 100 + G) {
        case 101: return coop_fn<1, 1>(paged, big);
        case 102: return coop_fn<1, 2>(paged, big);
        case 104: return coop_fn<1, 4>(paged, big);
        case 105: return coop_fn<1, 5>(paged, big);
        case 108: return coop_fn<1, 8>(paged, big);
        case 116: return coop_fn<1, 16>(paged, big);
        case 216: return coop_fn<2, 16>(paged, big);
        case 416: return coop_fn<4, 16>(paged, big);
        case 201: return coop_fn<2, 1>(paged, big);
        case 202: return coop_fn<2, 2>(paged, big);
        case 204: return coop_fn<2, 4>(paged, big);
        case 205: return coop_fn<2, 5>(paged, big);
        case 208: return coop_fn<2, 8>(paged, big);
        case 401: return coop_fn<4, 1>(paged, big);
        case 402: return coop_fn<4, 2>(paged, big);
        case 404: return coop_fn<4, 4>(paged, big);
        case 405: return coop_fn<4, 5>(paged, big);
        case 408: return coop_fn<4, 8>(paged, big);
        case 801: return coop_fn<8, 1>(paged, big);
        case 802: return coop_fn<8, 2>(paged, big);
        case 804: return coop_fn<8, 4>(paged, big);
        case 805: return coop_fn<8, 5>(paged, big);
        case 808: return coop_fn<8, 8>(paged, big);
        default: return nullptr;
    }
}

// chunk sizes the kernel is built for, and the width of the {offset, count} record word
static bool coop_shape_ok(const hata_ctx* c, bool paged, int chunk) {
    return chunk >= 256 && chunk % 256 == 0 && chunk <= HATA_COOP_MAX_CHUNK &&
           c->cfg.k_max <= 65535;
}
static size_t coop_dynamic_lds(const hata_ctx* c, int chunk) { return (size_t)chunk * 2 + (size_t)c->NB * 4; }

// how many workgroups of this context's cooperative kernel fit on the device at once
int coop_capacity(const hata_ctx* c, bool paged, int chunk) {
    const void* fn = coop_kernel_for(c->Wd, c->G, paged, chunk > HATA_COOP_SUB);
    if (!fn || !coop_shape_ok(c, paged, chunk)) return 0;
    int per_cu = 0;
    if (c->cus <= 0) return 0;
    const size_t lds = coop_dynamic_lds(c, chunk);
    // (more than 64 KB of dynamic LDS has to be asked for)
    if (lds > 65536 && hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 256, lds) != hipSuccess) return 0;
    return per_cu * c->cus;
}

hipError_t launch_coop_step(hata_ctx* c, const void* q, const void* K, const void* V,
                            const float* W_H, uint32_t* codes, int append, const int32_t* seq_len,
                            const int32_t* k, int B, float sm_scale, void* out, float* out_f32, hipStream_t s,
                            int chunk, const PageView* pages, int b0, int32_t* idx_only) {
    const hata_config& f = c->cfg;
    const void* fn = coop_kernel_for(c->Wd, c->G, pages != nullptr, chunk > HATA_COOP_SUB);
    if (!fn || !coop_shape_ok(c, pages != nullptr, chunk) || chunk < c->chunk) return hipErrorNotSupported;
    const int n_chunks = (f.L_cap + chunk - 1) / chunk;  // (the workspace regions are sized for c->n_chunks >= n_chunks)
    CoopArgs a;
    a.q = (const uint16_t*)q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V;
    a.W_H = W_H; a.append = append;
    a.spin_limit = c->spin_limit > 0 ? c->spin_limit : HATA_COOP_SPIN_LIMIT;
    a.keep_scores = c->keep_scores;
    // side-by-side merging pays with many slices per unit; with up to four, the workgroups that would
    // wait for the unit's last partial only add a hand-off, and the unit's last arriver merges all heads
    // (measured at L = 32K: B = 32 at two slices 55.1 -> 54.1 us, at four 73.1 -> 72.7, eight: no difference)
    a.par_merge = c->par_merge && n_chunks > 4;
    a.select_only = idx_only ? 1 : 0;
    // chunk-major order needs the whole grid resident (an oversubscribed grid relies on a unit's
    // workgroups having neighbouring indices)
    a.cmajor = (c->step_mode != 1) ? 1 : 0;
    a.pv = pages ? *pages : PageView{nullptr, 0, 0, 0};
    // sequences [b0, b0 + B) of the caller's batch: every per-sequence and per-unit base moves up
    const int64_t u0 = (int64_t)b0 * f.Hkv;
    a.q += (int64_t)b0 * f.Hq * HATA_D;
    if (pages) {
        a.pv.table += (int64_t)b0 * pages->max_blocks;
    } else {
        a.K += b0 * f.kv_stride_b;
        a.V += b0 * f.kv_stride_b;
        codes += u0 * f.L_cap * c->Wd;
    }
    seq_len += b0;
    k += b0;
    if (out) out = (uint16_t*)out + (int64_t)b0 * f.Hq * HATA_D;
    if (out_f32) out_f32 += (int64_t)b0 * f.Hq * HATA_D;
    // small grids (at most one workgroup per CU): the first batch of key codes is fetched ahead
    a.prefetch = (c->cus > 0 && (int64_t)n_chunks * f.Hkv * B <= c->cus) ? 1 : 0;
    a.qcodes = c->qcodes + (int64_t)b0 * f.Hq * c->Wd; a.codes = codes; a.seq_len = seq_len; a.kbud = k;
    a.scores = c->scores + u0 * f.L_cap; a.idx = (idx_only ? idx_only : c->idx) + u0 * f.k_max;
    a.chunk_hist = c->chunk_hist + u0 * n_chunks * c->NBP;
    a.chunk_info = c->chunk_info + u0 * (n_chunks + 1) * 2; a.unit_info = c->unit_info + u0 * 2;
    a.unit_counter = c->unit_counter + u0 * HATA_COUNTER_STRIDE;
    a.unit_hist = c->unit_hist + u0 * c->NB; a.rec = c->coop_rec + u0 * n_chunks * HATA_REC_STRIDE;
    a.qrec = c->coop_qrec + u0 * n_chunks * c->G * c->Wd;
    a.attn_counter = c->attn_counter + u0 * HATA_COUNTER_STRIDE;
    a.error_word = c->error_word;
    a.partials = c->partials + (int64_t)b0 * f.Hq * n_chunks * HATA_PSTRIDE;
    a.out = (uint16_t*)out; a.out_f32 = out_f32;
    a.Hq = f.Hq; a.Hkv = f.Hkv; a.L_cap = f.L_cap; a.k_max = f.k_max; a.chunk = chunk;
    a.n_chunks = n_chunks; a.NB = c->NB; a.NBP = c->NBP; a.units = f.Hkv * B;
    a.sb = f.kv_stride_b; a.sh = f.kv_stride_h; a.sn = f.kv_stride_n;
    a.scale_log2 = sm_scale * 1.4426950408889634f;
    c->epoch += 1;
    if (c->epoch == 0) c->epoch = 1;  // 0 is the cleared state of the flags
    a.epoch = c->epoch;
    void* args[] = {(void*)&a};
    return hipLaunchKernel(fn, dim3((unsigned)(n_chunks * f.Hkv * B)), dim3(256), args, coop_dynamic_lds(c, chunk), s);
}

}  // namespace hata
