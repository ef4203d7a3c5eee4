// Output head of the target model for the verification rows, for gfx950 (MI355X):
//     z[r][v] = sum_k h[r][k] * W[v][k]          ("LogitsOf", Alg. 1)
// for the rows of a verification step (gamma+1 rows of one sequence, or of a batch: up to 96),
// with the per-chunk
// softmax statistics of every row (max z, sum exp((z - max)/T)) produced in the
// epilogue, so that the acceptance pass does not have to read the logits once more
// to form them.
//
// With so few rows this is a matrix-vector problem: every weight is used 2 x rows
// times, so the kernel is bound by streaming W (vocab x hidden bf16, about 1 GB for a
// 128K vocabulary) from HBM, which is read once whatever the row count.  Design (NR = number of
// 16-row blocks of h; the description is for NR = 1, more row blocks shrink the vocabulary range
// of a workgroup to 512 / NR rows so that the accumulators still fit the register file, use the
// narrower slab, and send NR h tiles ahead of every slab):
//
//  * One workgroup owns up to 512 consecutive vocabulary rows (4 MiB of W at hidden =
//    4096); the host picks the row count (a multiple of 16) so that the grid fills the
//    chip in whole rounds: 501 rows x 251 workgroups would leave a second round of 41
//    workgroups that cannot saturate HBM, 304 rows x 501 workgroups does not.
//    Its four waves split the hidden dimension in quarters: a wave reads 2*hidden/4
//    contiguous bytes of every row, 512 B at a time.
//  * W travels HBM -> LDS directly (global_load_lds_dwordx4, 1 KiB per instruction)
//    in tiles of 16 rows x 256 k (8 KiB) through a four-slot ring per wave, three tiles
//    ahead of the math (16 rows x 128 k, eight slots, seven ahead when the hidden size
//    is a multiple of 512 only); the wave counts its own outstanding loads, so the main loop has
//    no workgroup barrier.
//  * The matching 256-k slab of h (16 rows, rows past the last real one repeat it)
//    comes through the same ring as one more tile at the head of every slab and is
//    then held in registers as the B operand of v_mfma_f32_16x16x32_bf16 for the 32
//    W tiles that follow; the accumulators of all 32 row blocks (128 registers) stay in
//    registers across slabs.
//  * A 16-byte-chunk XOR swizzle applied by the load addressing makes the operand reads
//    (ds_read_b128, 16 rows of 512 B) bank-conflict free without padding.
//  * Epilogue: the four K-quarter partial sums meet in LDS, are added in a fixed
//    order, stored as fp32 logits, and reduced to the chunk's (max, sum exp) per row.
#include "rapid_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kWaves = 4;
constexpr int kNB = 32;                      // 16-row vocabulary blocks per workgroup
constexpr int kVB = kNB * 16;                // vocabulary rows per workgroup (= statistics chunk)
constexpr int kRing = 32768;                 // LDS ring per wave
// Tile geometry for a slab width of SK hidden elements (256, or 128 for hidden sizes
// that are a multiple of 512 but not of 1024, e.g. 3584).
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


constexpr int lds_bytes()
{
    constexpr int ring = kWaves * kRing;
    constexpr int epi = kWaves * 16 * (kVB + 4) * 4 + 2 * kWaves * 16 * 4;   // the widest epilogue buffer (NR = 1)
    return ring > epi ? ring : epi;
}

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

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <int SK, int NR>
__global__ void __launch_bounds__(kWaves * 64) lm_head_stream(LmHeadLaunch a)
{
    using T = Tile<SK>;
    constexpr int NBM = kNB / NR;                       // vocabulary blocks per workgroup at most
    constexpr int VBM = NBM * 16;                       // vocabulary rows per workgroup at most
    constexpr int VBP = VBM + 4;                        // padded row of the epilogue buffer (floats)
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;
    const int nb = a.nb;                                 // 16-row vocabulary blocks per workgroup (<= NBM)
    const int v0 = blockIdx.x * nb * 16;
    const uint32_t row_bytes = (uint32_t)a.hidden * 2u;
    const int kq = wave * (a.hidden / kWaves);          // first hidden element of this wave's quarter
    const int nslab = a.hidden / (kWaves * SK);
    char* ring = smem + wave * kRing;
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + wave * kRing;

    // Per-lane byte offsets of the loads of a tile, relative to the tile's first row and
    // first k: instruction e moves RPI consecutive rows; lane i writes LDS bytes
    // [16 i, 16 i + 16) of that 1 KiB and fetches the chunk the swizzle assigns there.
    uint32_t woff[T::NLD], coff[T::NLD];
    int rrow[T::NLD];
#pragma unroll
    for (int e = 0; e < T::NLD; ++e) {
        rrow[e] = T::RPI * e + lane / T::CPR;
        coff[e] = (uint32_t)((lane % T::CPR) ^ (rrow[e] & 15)) * 16u;
        woff[e] = (uint32_t)rrow[e] * row_bytes + coff[e];
    }

    // tile j of slab s: j = 0..NR-1 are the row blocks of the h slab (rows past the last real one
    // repeat it), j = NR.. the W row blocks
    auto issue = [&](int s, int j, int slot) {
        const int64_t kbyte = (int64_t)(kq + s * SK) * 2;
        const uint32_t dst = ring_lds + slot * T::BYTES;
        if (j < NR) {
            const char* base = reinterpret_cast<const char*>(a.h) + kbyte;
#pragma unroll
            for (int e = 0; e < T::NLD; ++e)
                dma16_keep(base, (uint32_t)min(j * 16 + rrow[e], a.n_rows - 1) * row_bytes + coff[e], dst + e * 1024);
            return;
        }
        // A block that reaches past the vocabulary reads the last 16 rows instead: its
        // rows are then shifted against the block's nominal ones, which the epilogue
        // undoes; a block wholly past the end is never stored.
        const int row0 = min(v0 + (j - NR) * 16, a.vocab - 16);
        const char* base = reinterpret_cast<const char*>(a.w) + (int64_t)row0 * row_bytes + kbyte;
#pragma unroll
        for (int e = 0; e < T::NLD; ++e) dma16(base, woff[e], dst + e * 1024);
    };

    // The wave's tiles form one sequence: slab 0 (NR h tiles, then nb W tiles), slab 1, ...
    // (ps, pj) walks that sequence AHEAD tiles in front of the math; past the end it keeps
    // re-requesting a cached h tile so that the count of outstanding loads stays uniform.
    int ps = 0, pj = 0, pt = 0;                          // next tile to request: slab, index, linear number
    auto request_next = [&]() {
        const int sl = pt & (T::SLOTS - 1);
        if (ps < nslab) issue(ps, pj, sl);
        else issue(nslab - 1, 0, sl);
        ++pt;
        if (++pj >= NR + nb) { pj = 0; ++ps; }
    };
#pragma unroll
    for (int j = 0; j < T::AHEAD; ++j) request_next();

    floatx4 acc[NBM][NR];
#pragma unroll
    for (int j = 0; j < NBM; ++j)
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) acc[j][rb] = floatx4{0.f, 0.f, 0.f, 0.f};
    bf16x8 hreg[NR][T::KS];
    // operand read: lane (ln, lg) takes row ln, chunk 4 ks + lg of the chunks of a row
    const int rd_row = ln * (SK * 2);
    const int rd_swz = ln & 15;

    int t = 0;                                           // linear number of the tile being consumed
    for (int s = 0; s < nslab; ++s) {
#pragma unroll
        for (int j = 0; j < NR + NBM; ++j) {
            if (j < NR + nb) {                                 // this workgroup's slabs have NR + nb tiles
                wait_loads<(T::AHEAD - 1) * T::NLD>();         // tile (s, j) has landed
                request_next();                                // into the slot whose reads finished last iteration
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
    __syncthreads();                                           // the ring is dead from here on

    // ---- the four K quarters meet, one block of 16 h rows at a time: zbuf[wave][row n][vocabulary entry]
    float* zbuf = reinterpret_cast<float*>(smem);
    float* red = zbuf + kWaves * 16 * VBP;                     // [2][kWaves][16]
    constexpr int kPer = (VBM + kWaves * 64 - 1) / (kWaves * 64);   // vocabulary entries per thread
    int col[kPer];                                             // where this thread's entries sit in zbuf
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int vl = tid + u * (kWaves * 64);
        const int nominal = v0 + (vl & ~15);                   // first row of the entry's block
        col[u] = vl + max(0, nominal - (a.vocab - 16));        // shifted block at the end of the vocabulary
    }
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int rows_here = min(16, a.n_rows - rb * 16);     // real rows of this block (uniform)
        if (rows_here <= 0) break;
        if (rb > 0) __syncthreads();                           // the previous block's zbuf / red are still being read
#pragma unroll
        for (int j = 0; j < NBM; ++j)
            if (j < nb) *reinterpret_cast<floatx4*>(zbuf + (wave * 16 + ln) * VBP + j * 16 + lg * 4) = acc[j][rb];
        __syncthreads();

        float z[16][kPer];
        float mx[16];
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            mx[n] = -INFINITY;
            if (n < rows_here) {
#pragma unroll
                for (int u = 0; u < kPer; ++u) {
                    const int vl = tid + u * (kWaves * 64);
                    float x = 0.f;
                    if (vl < nb * 16 && v0 + vl < a.vocab) {
                        x = zbuf[(0 * 16 + n) * VBP + col[u]];
#pragma unroll
                        for (int w = 1; w < kWaves; ++w) x += zbuf[(w * 16 + n) * VBP + col[u]];
                        a.logits[(int64_t)(rb * 16 + n) * a.ldz + v0 + vl] = x;
                        mx[n] = fmaxf(mx[n], x);
                    }
                    z[n][u] = x;
                }
                mx[n] = wave_max(mx[n]);
            }
        }
        if (!a.stats) continue;                                // uniform
        if (lane < 16) {
            float m = -INFINITY;
#pragma unroll
            for (int n = 0; n < 16; ++n) m = lane == n ? mx[n] : m;
            red[wave * 16 + lane] = m;
        }
        __syncthreads();
        float sm[16];
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            sm[n] = 0.f;
            if (n < rows_here) {
                const float M = fmaxf(fmaxf(red[n], red[16 + n]), fmaxf(red[32 + n], red[48 + n]));
                mx[n] = M;
                float sacc = 0.f;
#pragma unroll
                for (int u = 0; u < kPer; ++u)
                    if (tid + u * (kWaves * 64) < nb * 16 && v0 + tid + u * (kWaves * 64) < a.vocab)
                        sacc += __builtin_amdgcn_exp2f((z[n][u] - M) * a.inv_T * kLog2e);
                sm[n] = wave_sum(sacc);
            }
        }
        float* red2 = red + kWaves * 16;
        if (lane < 16) {
            float sv = 0.f;
#pragma unroll
            for (int n = 0; n < 16; ++n) sv = lane == n ? sm[n] : sv;
            red2[wave * 16 + lane] = sv;
        }
        __syncthreads();
        if (tid < rows_here) {
            float M = -INFINITY;
#pragma unroll
            for (int n = 0; n < 16; ++n) M = tid == n ? mx[n] : M;
            const float S = (red2[tid] + red2[16 + tid]) + (red2[32 + tid] + red2[48 + tid]);
            a.stats[((int64_t)(rb * 16 + tid) * gridDim.x + blockIdx.x) * 2 + 0] = M;
            a.stats[((int64_t)(rb * 16 + tid) * gridDim.x + blockIdx.x) * 2 + 1] = S;
        }
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
    return configure_one<128, 6>();
}

// Row blocks of 16 rows of h; one and two blocks use the 256-wide slab when the hidden size allows,
// more blocks always the 128-wide one (the h operands of a slab must fit the register file next to
// the accumulators).
hipError_t launch_lm_head(const LmHeadLaunch& a, hipStream_t stream)
{
    const int nwg = (a.vocab + a.nb * 16 - 1) / (a.nb * 16);
    const int nr = (a.n_rows + 15) / 16;
    if (a.hidden % 512 != 0 || nr < 1 || nr > 6 || a.nb > kNB / nr) return hipErrorInvalidValue;
    const bool wide_slab = a.hidden % 1024 == 0;
    switch (nr) {
        case 1: wide_slab ? launch_one<256, 1>(a, nwg, stream) : launch_one<128, 1>(a, nwg, stream); break;
        case 2: wide_slab ? launch_one<256, 2>(a, nwg, stream) : launch_one<128, 2>(a, nwg, stream); break;
        case 3: launch_one<128, 3>(a, nwg, stream); break;
        case 4: launch_one<128, 4>(a, nwg, stream); break;
        case 5: launch_one<128, 5>(a, nwg, stream); break;
        default: launch_one<128, 6>(a, nwg, stream); break;
    }
    return hipGetLastError();
}
