// Issue model of one gfx950 SIMD for the large-batch scan kernel (linr_kernels_dense.hip): how much time a
// v_mfma_i32_16x16x64_i8 takes next to the vector instructions that look at its result, at 1, 2 and 4 waves per SIMD.
// Stand-alone program (no library code): every wave keeps G query fragments in registers, makes G products per
// "tile" against a changing item fragment and post-processes them in one of these ways:
//   chains      no vector work: acc[g] = mfma(a, q[g], acc[g])                          (the matrix pipe by itself)
//   max2        running maximum over the four accumulators: 2 v_max3_i32 per product, one compare per 8 products
//               (what the kernel's tile loop does)
//   test4       per product: maximum of its four values, fused multiply-add, compare, ballot (4 vector instructions;
//               the per-group test of the other scan kernels), on the previous product's result
// Prints time per product per SIMD in cycles at 2.4 GHz.  Usage: mfma_issue_bench
#include <hip/hip_runtime.h>
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

enum { CHAINS = 0, MAX2 = 1, TEST4 = 2 };

template <int MODE, int G, int WAVES_PER_SIMD>
__global__ void __launch_bounds__(256, WAVES_PER_SIMD) loopk(const v4i* src, int* out, int iters, float thr0, float s0)
{
    const int lane = threadIdx.x & 63;
    v4i q[G];
#pragma unroll
    for (int g = 0; g < G; ++g) q[g] = src[lane + g];
    v4i a = src[lane + 64 + (threadIdx.x >> 6)];
    v4i c0 = {0x4B400000, 0x4B400000, 0x4B400000, 0x4B400000};
    asm volatile("" : "+v"(c0));
    float thr[G];
#pragma unroll
    for (int g = 0; g < G; ++g) thr[g] = thr0 + g;
    const float smax = s0 + lane * 1e-6f, umax = smax * 12582910.0f;
    u64 hot = 0;
    unsigned cnt = 0;
    if constexpr (MODE == CHAINS) {
        v4i acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g) acc[g] = c0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, q[g], acc[g], 0, 0, 0);
        }
#pragma unroll
        for (int g = 0; g < G; ++g) cnt += (unsigned)acc[g][0] + (unsigned)acc[g][3];
    } else {
        v4i prev = c0;
        int run = INT_MIN;
        for (int it = 0; it < iters; ++it) {
            a[0] ^= it;                                  // a new item fragment per tile (stand-in for the LDS read)
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const v4i r = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, q[g], c0, 0, 0, 0);
                if constexpr (MODE == TEST4) {
                    const int m = max(max(max(prev[0], prev[1]), prev[2]), prev[3]);
                    const bool h = __builtin_fmaf(__int_as_float(m), smax, -umax) >= thr[(g + G - 1) % G];
                    hot |= __builtin_amdgcn_ballot_w64(h);
                } else {
                    run = max(max(run, prev[0]), prev[1]);
                    run = max(max(run, prev[2]), prev[3]);
                    if ((g & 7) == 7) hot |= __builtin_amdgcn_ballot_w64(run >= (int)thr[g]);
                }
                prev = r;
            }
            if (hot) { cnt += 1; hot = 0; thr[0] += 1.0f; }      // never taken with these inputs; keeps `hot` alive per tile
        }
        cnt += (unsigned)prev[0] ^ (unsigned)run;
    }
    if (cnt == (unsigned)iters * 77u) out[threadIdx.x] = cnt;
}

template <int MODE, int G, int WAVES_PER_SIMD>
static void run(const char* name, const v4i* src, int* out)
{
    const int iters = 20000, grid = 256 * WAVES_PER_SIMD;        // one workgroup of four waves per SIMD quartet, all 256 CUs
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    hipLaunchKernelGGL((loopk<MODE, G, WAVES_PER_SIMD>), dim3(grid), dim3(256), 0, 0, src, out, 100, 1e30f, 1.0f);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((loopk<MODE, G, WAVES_PER_SIMD>), dim3(grid), dim3(256), 0, 0, src, out, iters, 1e30f, 1.0f);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double ops = (double)grid * 4 * iters * G * 2.0 * 16 * 16 * 64;
    const double ns = ms * 1e6 / (iters * (double)G * WAVES_PER_SIMD);
    printf("%-10s %2d fragments, %d waves/SIMD: %8.3f ms  %7.1f TOP/s  %5.1f cycles per product per SIMD at 2.4 GHz\n", name, G,
           WAVES_PER_SIMD, ms, ops / ms / 1e9, ns * 2.4);
    fflush(stdout);
}

int main()
{
    v4i* src;
    int* out;
    CK(hipMalloc(&src, 4096 * sizeof(v4i)));
    CK(hipMemset(src, 0x11, 4096 * sizeof(v4i)));
    CK(hipMalloc(&out, 4096));
    run<CHAINS, 8, 1>("chains", src, out); run<MAX2, 16, 1>("max2", src, out); run<TEST4, 16, 1>("test4", src, out);
    run<CHAINS, 8, 2>("chains", src, out); run<MAX2, 16, 2>("max2", src, out); run<TEST4, 16, 2>("test4", src, out);
    run<CHAINS, 8, 4>("chains", src, out); run<MAX2, 8, 4>("max2", src, out);  run<TEST4, 8, 4>("test4", src, out);
    return 0;
}
