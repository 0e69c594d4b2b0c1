// What the two large-batch scan kernels (linr_kernels_dense.hip: int8 rows of 64 bytes; linr_kernels_dense_bf16.hip:
// bf16 rows of 256 bytes) have in common: sizes, the LDS address helper, the per-query state of a workgroup.
#pragma once
#include "linr_scan_common.h"
#include <type_traits>

#define DENSE_CH 128                   // items per chunk, the unit of the sweep plan and of a wave's walk
#define DENSE_SUB 32                   // items per step of a wave (two tiles of 16)
#define DENSE_QCAP 192                 // keys a wave queues in LDS before writing them out
#define DENSE_SLACK LINR_DENSE_SLACK   // room a segment must have beyond k: the queue's keys + what one chunk can add per query
#define DENSE_SCRATCH_WORDS 516        // per wave: queue (keys, query numbers) / compaction histogram / flush prefix
// Stand-in for "no bound" (-) and "no query" (+) among the integer bounds T.  |raw| < 2^20, so raw - T stays within
// +-(2^29 + 2^20) and its difference to a test value in [-2^29 (1 + 2^-11) - 3, 2^28] cannot overflow 32 bits.
#define DENSE_BIG (1 << 29)

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding)
#define DENSE_WAIT_VM(n) (((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

// The ring and the per-query arrays are read with hand-placed LDS instructions: for an LDS access the compiler can
// see, it would wait until every outstanding direct load has landed, i.e. for the memory latency of the step
// requested last.  That a stage's loads have landed is established by the counted wait of the step loop.
__device__ __forceinline__ uint32_t dense_lds_addr(const void* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

__device__ __forceinline__ int dense_floor_to_int(float x)      // floor(x) clamped to +-DENSE_BIG (x may be +-inf)
{
    return (int)fminf(fmaxf(floorf(x), -(float)DENSE_BIG), (float)DENSE_BIG);
}

// running maximum over the four accumulators of a product (two v_max3_i32)
__device__ __forceinline__ int dense_max_acc(int m, const v4i& a)
{
    m = max(max(m, a[0]), a[1]);
    return max(max(m, a[2]), a[3]);
}

// Per-query state of a workgroup in LDS.  Bounds are kept per WAVE (a wave's accumulator inputs and the values its
// survivor path adds back must be the same numbers, and waves refresh at different times); the filters, which never
// change during a launch, per query set.
template <int NQW, bool TS>
struct DenseQ {
    float thr[4 * NQW];                // [wave][query] lower bound of the ranking value (raw ranking: the int32 bound's bits; "none": -inf / INT_MIN)
    int T[4 * NQW];                    // [wave][query] integer bound that enters the accumulators (see the header comment)
    uint32_t fa[4 * NQW], fn[4 * NQW]; // [set][query] compact filter: an item passes the all / none clauses iff (mask & fn) == fa
    uint32_t t0[TS ? 4 * NQW : 1], t1[TS ? 4 * NQW : 1];   // timestamp window
    uint16_t qi[4 * NQW];              // [set][query] index of the query in the batch (0xFFFF: none)
    uint8_t flag[4 * NQW];             // 1: the filter has any-of clauses (read the full record from global memory)
};

