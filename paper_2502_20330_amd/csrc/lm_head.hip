// Output head of the target model for the verification rows, for gfx950 (MI355X):
//     z[r][v] = sum_k h[r][k] * W[v][k]          ("LogitsOf", Alg. 1)
// for the rows of a verification step (gamma+1 rows of one sequence, or of a batch: up to 96),
// with the per-chunk softmax statistics of every row (max z, sum exp((z - max)/T)) produced in
// the epilogue, so that the acceptance pass does not have to form them from the logits.
//
// With so few rows every weight is used 2 x rows times, so the kernel is bound by streaming W
// (vocab x hidden bf16, about 1 GB for a 128K vocabulary) from HBM, which is read once whatever
// the row count.  NR = number of 16-row blocks of h (1..6).
//
//  * One workgroup owns up to 512 consecutive vocabulary rows (4 MiB of W at hidden = 4096); the
//    host picks the row count (a multiple of 16) so that the grid fills the chip in whole rounds:
//    501 rows x 251 workgroups would leave a second round of 41 workgroups that cannot saturate
//    HBM, 304 rows x 501 workgroups does not.
//  * The four waves split the vocabulary range: wave w takes the 16-row blocks w, w + 4, ... (eight
//    at most) and runs over the whole hidden dimension for them, one slab of SK = 256 or 128 hidden
//    elements at a time.  Its accumulators (8 blocks x NR row blocks x 4 registers) stay in
//    registers across all slabs, and the logits leave straight from them: no exchange between
//    waves except four (max, sum) pairs per row at the very end.  (A first version split the
//    hidden dimension over the waves and met in LDS; its accumulators then limited a workgroup to
//    512 / NR vocabulary rows and the grid to NR times as many short-lived workgroups, each ending
//    in that exchange: 456 us at 72 rows where this one takes 202 us, and no faster at 9 rows.)
//  * W travels HBM -> LDS directly (global_load_lds_dwordx4, 1 KiB per instruction) in tiles of
//    16 rows x SK (8 KiB / 4 KiB) through a 32 KiB ring per wave, three / seven tiles ahead of the
//    math; the wave counts its own outstanding loads, so the main loop has no workgroup barrier.
//  * The matching slab of h (NR tiles of 16 rows; rows past the last real one repeat it) comes
//    through the same ring at the head of every slab (from cache: every wave of every workgroup
//    reads the same h) and is then held in registers as the B operand of
//    v_mfma_f32_16x16x32_bf16 for the W tiles that follow.
//  * A 16-byte-chunk XOR swizzle applied by the load addressing makes the operand reads
//    (ds_read_b128, 16 rows of 512 / 256 B) bank-conflict free without padding.
//  * Epilogue: fp32 logits from the accumulators (16-byte stores where the row stride allows);
//    per row the wave's own (max, sum exp) over its blocks, combined over the four waves by the
//    first threads of the workgroup.
#include "rapid_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kWaves = 4;
constexpr int kNB = 32;                      // 16-row vocabulary blocks per workgroup
constexpr int kRing = 32768;                 // LDS ring per wave
// Tile geometry for a slab width of SK hidden elements (256, or 128 for hidden sizes
// that are a multiple of 128 but not of 256).
template <int SK>
struct Tile {
    static constexpr int BYTES = 16 * SK * 2;          // 8 KiB / 4 KiB
    static constexpr int NLD = BYTES / 1024;           // 1 KiB load instructions per tile
    static constexpr int RPI = 1024 / (SK * 2);        // rows moved by one instruction
    static constexpr int CPR = SK * 2 / 16;            // 16-byte chunks per row
    static constexpr int KS = SK / 32;                 // MFMA k-steps per tile
    static constexpr int SLOTS = kRing / BYTES;        // 4 / 8
    static constexpr int AHEAD = SLOTS - 1;            // tiles requested ahead of the math
};
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ void dma16(const char* base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(byte_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
// h is re-read by every workgroup: no streaming hint, it should stay in cache
__device__ __forceinline__ void dma16_keep(const char* base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(byte_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void lds_reads_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

constexpr int kNBW = kNB / kWaves;                      // vocabulary blocks per wave at most
constexpr int lds_bytes() { return kWaves * kRing + kWaves * 96 * 2 * 4; }   // rings + (max, sum) of 96 rows per wave

template <int SK, int NR>
__global__ void __launch_bounds__(kWaves * 64) lm_head_stream(LmHeadLaunch a)
{
    using T = Tile<SK>;
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;
    const int nb = a.nb;                                 // 16-row vocabulary blocks per workgroup (<= 32)
    const int nbw = (nb + kWaves - 1 - wave) / kWaves;   // blocks of this wave: wave, wave + 4, ...
    const int v0 = blockIdx.x * nb * 16;
    const uint32_t row_bytes = (uint32_t)a.hidden * 2u;
    const int nslab = a.hidden / SK;
    char* ring = smem + wave * kRing;
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + wave * kRing;

    // Per-lane byte offsets of the loads of a tile, relative to the tile's first row and first k:
    // instruction e moves RPI consecutive rows; lane i writes LDS bytes [16 i, 16 i + 16) of that
    // 1 KiB and fetches the chunk the swizzle assigns there.
    uint32_t woff[T::NLD], coff[T::NLD];
    int rrow[T::NLD];
#pragma unroll
    for (int e = 0; e < T::NLD; ++e) {
        rrow[e] = T::RPI * e + lane / T::CPR;
        coff[e] = (uint32_t)((lane % T::CPR) ^ (rrow[e] & 15)) * 16u;
        woff[e] = (uint32_t)rrow[e] * row_bytes + coff[e];
    }
    // first vocabulary row of the wave's block jj as loaded: a block that reaches past the vocabulary
    // reads the last 16 rows instead (the epilogue drops the rows that belong to the block before)
    auto block_row0 = [&](int jj) { return min(v0 + (jj * kWaves + wave) * 16, a.vocab - 16); };

    // tile j of slab s: j = 0..NR-1 the row blocks of the h slab, j = NR.. the wave's W blocks
    auto issue = [&](int s, int j, int slot) {
        const int64_t kbyte = (int64_t)s * SK * 2;
        const uint32_t dst = ring_lds + slot * T::BYTES;
        if (j < NR) {
            const char* base = reinterpret_cast<const char*>(a.h) + kbyte;
#pragma unroll
            for (int e = 0; e < T::NLD; ++e)
                dma16_keep(base, (uint32_t)min(j * 16 + rrow[e], a.n_rows - 1) * row_bytes + coff[e], dst + e * 1024);
            return;
        }
        const char* base = reinterpret_cast<const char*>(a.w) + (int64_t)block_row0(j - NR) * row_bytes + kbyte;
#pragma unroll
        for (int e = 0; e < T::NLD; ++e) dma16(base, woff[e], dst + e * 1024);
    };

    floatx4 acc[kNBW][NR];
#pragma unroll
    for (int j = 0; j < kNBW; ++j)
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) acc[j][rb] = floatx4{0.f, 0.f, 0.f, 0.f};

    if (nbw > 0) {                                       // (a wave without blocks: ranges of fewer than four blocks)
        int ps = 0, pj = 0, pt = 0;                      // next tile to request: slab, index, linear number
        auto request_next = [&]() {
            const int sl = pt & (T::SLOTS - 1);
            if (ps < nslab) issue(ps, pj, sl);
            else issue(nslab - 1, 0, sl);                // past the end: a cached h tile keeps the count uniform
            ++pt;
            if (++pj >= NR + nbw) { pj = 0; ++ps; }
        };
#pragma unroll
        for (int j = 0; j < T::AHEAD; ++j) request_next();

        bf16x8 hreg[NR][T::KS];
        const int rd_row = ln * (SK * 2);
        const int rd_swz = ln & 15;
        int t = 0;
        for (int s = 0; s < nslab; ++s) {
#pragma unroll
            for (int j = 0; j < NR + kNBW; ++j) {
                if (j < NR + nbw) {
                    wait_loads<(T::AHEAD - 1) * T::NLD>();     // tile (s, j) has landed
                    request_next();
                    const char* tile = ring + (t & (T::SLOTS - 1)) * T::BYTES;
                    ++t;
                    if (j < NR) {
#pragma unroll
                        for (int ks = 0; ks < T::KS; ++ks)
                            hreg[j < NR ? j : 0][ks] = *reinterpret_cast<const bf16x8*>(tile + rd_row + (((ks * 4 + lg) ^ rd_swz) * 16));
                    } else {
#pragma unroll
                        for (int ks = 0; ks < T::KS; ++ks) {
                            bf16x8 wa = *reinterpret_cast<const bf16x8*>(tile + rd_row + (((ks * 4 + lg) ^ rd_swz) * 16));
#pragma unroll
                            for (int rb = 0; rb < NR; ++rb)
                                acc[j >= NR ? j - NR : 0][rb] =
                                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, hreg[rb][ks], acc[j >= NR ? j - NR : 0][rb], 0, 0, 0);
                        }
                    }
                    lds_reads_done();
                }
            }
        }
        wait_loads<0>();
    }

    // ---- epilogue.  acc[jj][rb]: lane (ln, lg) holds, for row rb*16 + ln of h, the four vocabulary
    // entries block_row0(jj) + lg*4 .. +3.  Logits go out from the registers; the chunk statistics
    // are formed per wave (own maximum) and combined over the four waves by the first threads.
    const float c = a.inv_T * kLog2e;
    float* red = reinterpret_cast<float*>(smem + kWaves * kRing);          // [kWaves][NR*16][2]
    const bool vec_ok = (a.ldz & 3) == 0 && (reinterpret_cast<uintptr_t>(a.logits) & 15) == 0;
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int hrow = rb * 16 + ln;
        const bool row_ok = hrow < a.n_rows;
        float m = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < kNBW; ++jj) {
            const int nominal = v0 + (jj * kWaves + wave) * 16;
            if (jj < nbw && nominal < a.vocab && row_ok) {
                const int vi = block_row0(jj) + lg * 4;
                float* dst = a.logits + (int64_t)hrow * a.ldz + vi;
                if (vec_ok && vi >= nominal && (vi & 3) == 0) {
                    *reinterpret_cast<floatx4*>(dst) = acc[jj][rb];
#pragma unroll
                    for (int i = 0; i < 4; ++i) m = fmaxf(m, acc[jj][rb][i]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (vi + i >= nominal) { dst[i] = acc[jj][rb][i]; m = fmaxf(m, acc[jj][rb][i]); }
                }
            }
        }
        if (!a.stats) continue;                                // uniform
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        float sum = 0.f;
        if (m > -INFINITY) {
#pragma unroll
            for (int jj = 0; jj < kNBW; ++jj) {
                const int nominal = v0 + (jj * kWaves + wave) * 16;
                if (jj < nbw && nominal < a.vocab && row_ok) {
                    const int vi = block_row0(jj) + lg * 4;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (vi + i >= nominal) sum += __builtin_amdgcn_exp2f((acc[jj][rb][i] - m) * c);
                }
            }
        }
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        if (lg == 0) {
            red[((wave * NR * 16) + hrow) * 2 + 0] = m;
            red[((wave * NR * 16) + hrow) * 2 + 1] = sum;
        }
    }
    if (!a.stats) return;
    __syncthreads();
    if (tid < a.n_rows) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, red[((w * NR * 16) + tid) * 2]);
        float S = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = red[((w * NR * 16) + tid) * 2], sw = red[((w * NR * 16) + tid) * 2 + 1];
            if (sw > 0.f) S += sw * __builtin_amdgcn_exp2f((mw - M) * c);
        }
        a.stats[((int64_t)tid * gridDim.x + blockIdx.x) * 2 + 0] = M;
        a.stats[((int64_t)tid * gridDim.x + blockIdx.x) * 2 + 1] = S;
    }
}

}  // namespace

namespace {
template <int SK, int NR>
hipError_t configure_one()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(lm_head_stream<SK, NR>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes());
}
template <int SK, int NR>
void launch_one(const LmHeadLaunch& a, int nwg, hipStream_t stream)
{
    hipLaunchKernelGGL((lm_head_stream<SK, NR>), dim3(nwg), dim3(kWaves * 64), lds_bytes(), stream, a);
}
}  // namespace

hipError_t configure_lm_head()
{
    hipError_t e;
    if ((e = configure_one<256, 1>()) != hipSuccess) return e;
    if ((e = configure_one<128, 1>()) != hipSuccess) return e;
    if ((e = configure_one<256, 2>()) != hipSuccess) return e;
    if ((e = configure_one<128, 2>()) != hipSuccess) return e;
    if ((e = configure_one<128, 3>()) != hipSuccess) return e;
    if ((e = configure_one<128, 4>()) != hipSuccess) return e;
    if ((e = configure_one<128, 5>()) != hipSuccess) return e;
    if ((e = configure_one<128, 6>()) != hipSuccess) return e;
    if ((e = configure_one<256, 3>()) != hipSuccess) return e;
    if ((e = configure_one<256, 4>()) != hipSuccess) return e;
    if ((e = configure_one<256, 5>()) != hipSuccess) return e;
    return configure_one<256, 6>();
}

// Row blocks of 16 rows of h; the 256-wide slab when the hidden size allows (at six row blocks its h
// operands and the accumulators take 384 of the 512 registers), else the 128-wide one.
hipError_t launch_lm_head(const LmHeadLaunch& a, hipStream_t stream)
{
    const int nwg = (a.vocab + a.nb * 16 - 1) / (a.nb * 16);
    const int nr = (a.n_rows + 15) / 16;
    if (a.hidden % 128 != 0 || nr < 1 || nr > 6 || a.nb < 1 || a.nb > kNB) return hipErrorInvalidValue;
    const bool wide_slab = a.hidden % 256 == 0;
    switch (nr) {
        case 1: wide_slab ? launch_one<256, 1>(a, nwg, stream) : launch_one<128, 1>(a, nwg, stream); break;
        case 2: wide_slab ? launch_one<256, 2>(a, nwg, stream) : launch_one<128, 2>(a, nwg, stream); break;
        case 3: wide_slab ? launch_one<256, 3>(a, nwg, stream) : launch_one<128, 3>(a, nwg, stream); break;
        case 4: wide_slab ? launch_one<256, 4>(a, nwg, stream) : launch_one<128, 4>(a, nwg, stream); break;
        case 5: wide_slab ? launch_one<256, 5>(a, nwg, stream) : launch_one<128, 5>(a, nwg, stream); break;
        default: wide_slab ? launch_one<256, 6>(a, nwg, stream) : launch_one<128, 6>(a, nwg, stream); break;
    }
    return hipGetLastError();
}
