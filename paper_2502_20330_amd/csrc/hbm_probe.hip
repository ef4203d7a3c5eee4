// Streaming-read probe: what read bandwidth the device delivers when nothing else
// limits the kernel.  Not part of the method; it gives the benchmark a measured
// ceiling to set next to the published 8 TB/s.  It moves memory exactly the way the
// attention kernel does (HBM -> LDS, 1 KiB per instruction, streaming hint, every
// wave on its own contiguous range, a two-slot ring of 16 KiB blocks per wave) and
// does no arithmetic on it.
#include "rapid_internal.h"

namespace {

constexpr int kBlock = 16384;      // bytes per ring slot
constexpr int kWaves = 4;

// Workgroups 2i and 2i + 1 share the blocks of pair i; the first takes (32 + skew)/64 of them (skew = 0:
// equal shares).  Inside a workgroup every wave streams its own contiguous quarter.
__global__ void __launch_bounds__(kWaves * 64) hbm_read_stream(const char* buf, int64_t nblock, int skew, uint32_t* sink)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t npair = (gridDim.x + 1) / 2, pair = blockIdx.x >> 1;
    const int64_t p0 = nblock * pair / npair, p1 = nblock * (pair + 1) / npair;        // the pair's blocks
    const bool alone = 2 * pair + 1 >= gridDim.x;                                      // an odd grid's last workgroup
    const int64_t cut = alone ? p1 : p0 + (p1 - p0) * (32 + skew) / 64;
    const int64_t g0 = (blockIdx.x & 1) ? cut : p0, g1 = (blockIdx.x & 1) ? p1 : cut;  // this workgroup's blocks
    const int64_t b0 = g0 + (g1 - g0) * wave / kWaves, b1 = g0 + (g1 - g0) * (wave + 1) / kWaves;
    const int n = (int)(b1 - b0);
    if (n <= 0) return;
    const char* base = buf + b0 * kBlock;
    const uint32_t ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + wave * 2 * kBlock;
    auto issue = [&](int t) {
        const char* bp = base + (int64_t)t * kBlock;
#pragma unroll
        for (int e = 0; e < kBlock / 1024; ++e) {
            const uint32_t off = e * 1024 + lane * 16;
            const uint32_t dst = ring + (t & 1) * kBlock + e * 1024;
            asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                         :
                         : "v"(off), "s"(bp), "s"(dst)
                         : "memory", "m0");
        }
    };
    issue(0);
    uint32_t acc = 0;
    for (int t = 0; t < n; ++t) {
        if (t + 1 < n) {
            issue(t + 1);
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");          // block t has landed
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        acc ^= *reinterpret_cast<const uint32_t*>(smem + wave * 2 * kBlock + (t & 1) * kBlock + lane * 4);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (acc == 0x9E3779B9u && sink) *sink = acc;                       // keeps the reads alive
}

}  // namespace

hipError_t configure_hbm_read_probe()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(hbm_read_stream),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kWaves * 2 * kBlock);
}

hipError_t launch_hbm_read_probe(const rapid_ctx* ctx, const void* buf, size_t bytes, uint32_t* sink, hipStream_t stream)
{
    const int64_t nblock = (int64_t)(bytes / kBlock);
    hipLaunchKernelGGL(hbm_read_stream, dim3(ctx->n_cu), dim3(kWaves * 64), kWaves * 2 * kBlock, stream,
                       static_cast<const char*>(buf), nblock, ctx->probe_skew, sink);
    return hipGetLastError();
}
