// Split-KV verification attention for gfx950 (MI355X).
//
// What it computes (Sec. 2.1 / Alg. 1 of the RAPID paper: the target model scores
// all gamma drafted positions in one forward pass over the full context): causal
// grouped-query softmax attention of the Q = gamma+1 verification positions
// against the whole KV cache.  The paper gives no kernel; this design is for
// CDNA4:
//
//  * The R = Q*G query rows that share one KV head (G query heads x Q positions)
//    are packed into the N side of bf16 MFMA tiles, so every K/V byte is read
//    from HBM once and used by all R rows.
//  * One workgroup = one (sequence, kv head, KV split).  Its four waves run
//    independent software pipelines over interleaved 32-token tiles: coalesced
//    128-bit global loads two tiles ahead into registers, a private LDS staging
//    tile per wave (no workgroup barrier in the main loop), MFMA 16x16x32 bf16
//    for S^T = K Q^T and O^T = V^T P^T with fp32 accumulators.
//  * Scores are produced transposed (tokens on M, query rows on N): a query
//    row's running max/sum then lives in one lane column, so the online softmax
//    needs two cross-lane steps per tile instead of a butterfly per row.
//  * V is stored token-major but the PV product reduces over tokens; the LDS V
//    tile is XOR-swizzled so the per-lane column gathers are conflict free.
//  * Waves combine (m, l, O) through LDS in a fixed order; the workgroup writes
//    one fp32 partial.  A second small kernel merges the splits with the
//    log-sum-exp rule and rounds to bf16.
#include "rapid_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int kTile = 32;          // tokens per wave tile
constexpr int kWaves = 4;          // waves per workgroup
constexpr int kChunkQuantum = kTile * kWaves;
constexpr float kRescaleLog2 = 8.0f;   // lazy rescale threshold (log2 units)

template <int D>
struct Geo {
    static constexpr int KS = D / 32;             // MFMA k-steps of the QK product
    static constexpr int DB = D / 16;             // 16-wide blocks of the head dim (PV M side)
    static constexpr int CPR = D * 2 / 16;        // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;          // rows covered by one wave-wide 16-byte load
    static constexpr int NLD = kTile / RPI;       // loads per tile per tensor
    static constexpr int KROW = D * 2 + 16;       // padded LDS row of the K tile (bytes)
    static constexpr int VROW = D * 2;            // LDS row of the swizzled V tile (bytes)
    static constexpr int WAVE_LDS = kTile * (KROW + VROW);
};

template <int D, int RB>
constexpr int attn_lds_bytes()
{
    constexpr int tiles = kWaves * Geo<D>::WAVE_LDS;
    constexpr int merge = (D * (RB * 16 + 1) + kWaves * RB * 16 * 2) * 4;
    return tiles > merge ? tiles : merge;
}

template <int D>
struct TileRegs {
    u32x4 k[Geo<D>::NLD];
    u32x4 v[Geo<D>::NLD];
};

// Where the rows of this (sequence, kv head) start.  Contiguous caches are addressed
// as a wave-uniform base plus a 32-bit byte offset per lane (the host checks that a
// sequence spans less than 4 GiB); paged caches look the page up per row.
struct RowAddr {
    const char* kbase;
    const char* vbase;
    const int32_t* pages;      // page table row of this sequence (paged only)
    uint32_t tok_bytes;        // bytes between consecutive tokens
    int64_t page_bytes;        // bytes between pages
    int page_shift, page_mask;
};

template <bool PAGED>
__device__ __forceinline__ RowAddr make_row_addr(const AttnLaunch& a, int b, int hkv)
{
    RowAddr r;
    int64_t head = (int64_t)hkv * a.hstride + (PAGED ? 0 : (int64_t)b * a.bstride);
    r.kbase = reinterpret_cast<const char*>(a.k + head);
    r.vbase = reinterpret_cast<const char*>(a.v + head);
    r.pages = PAGED ? a.page_table + (int64_t)b * a.max_pages : nullptr;
    r.tok_bytes = (uint32_t)(a.tstride * 2);
    r.page_bytes = a.pstride * 2;
    r.page_shift = a.page_shift;
    r.page_mask = a.page_mask;
    return r;
}

// Issue the global loads of one 32-token tile (K and V rows of this kv head).
// Rows past `last_tok` are clamped to it; the softmax masks them.
template <int D, bool PAGED>
__device__ __forceinline__ void load_tile(TileRegs<D>& r, const RowAddr& ra, int t0, int last_tok, int lane)
{
    using G = Geo<D>;
    const uint32_t lane_off = (lane % G::CPR) * 16;
#pragma unroll
    for (int e = 0; e < G::NLD; ++e) {
        int tok = min(t0 + e * G::RPI + lane / G::CPR, last_tok);
        if (PAGED) {
            int64_t off = (int64_t)ra.pages[tok >> ra.page_shift] * ra.page_bytes
                        + (uint32_t)(tok & ra.page_mask) * ra.tok_bytes + lane_off;
            r.k[e] = *reinterpret_cast<const u32x4*>(ra.kbase + off);
            r.v[e] = *reinterpret_cast<const u32x4*>(ra.vbase + off);
        } else {
            uint32_t off = (uint32_t)tok * ra.tok_bytes + lane_off;
            r.k[e] = *reinterpret_cast<const u32x4*>(ra.kbase + off);
            r.v[e] = *reinterpret_cast<const u32x4*>(ra.vbase + off);
        }
    }
}

// V tile swizzle: the 32-byte column unit `u` of row `row` is stored at unit
// u ^ ((row ^ (row >> 2)) & 3), which spreads both "rows r, r+4, r+8, r+12" and
// "rows r..r+3" over distinct bank groups.
__device__ __forceinline__ int v_swz(int row) { return (row ^ (row >> 2)) & 3; }

template <int D>
__device__ __forceinline__ void store_tile(const TileRegs<D>& r, char* kt, char* vt, int lane)
{
    using G = Geo<D>;
#pragma unroll
    for (int e = 0; e < G::NLD; ++e) {
        int row = e * G::RPI + lane / G::CPR;
        int c = lane % G::CPR;
        *reinterpret_cast<u32x4*>(kt + row * G::KROW + c * 16) = r.k[e];
        int pu = (c >> 1) ^ v_swz(row);
        *reinterpret_cast<u32x4*>(vt + row * G::VROW + ((pu << 1) | (c & 1)) * 16) = r.v[e];
    }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int RB>
struct WaveState {
    float m[RB];                     // running max per query row, log2 units (score*scale*log2e)
    float l[RB];                     // running sum, this lane group's tokens only
    floatx4 acc[Geo<D>::DB][RB];     // O^T: d = 16*db + 4*(lane/16) + i, row = 16*rb + lane%16
};

// One 32-token tile already staged in this wave's LDS region.
template <int D, int RB>
__device__ __forceinline__ void compute_tile(WaveState<D, RB>& st, const bf16x8 (&qf)[RB][Geo<D>::KS],
                                             const char* kt, char* vt, int t0, bool masked,
                                             const int (&lim)[RB], float c, int lane)
{
    using G = Geo<D>;
    const int ln = lane & 15, lg = lane >> 4;
    floatx4 s[2][RB];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) s[tb][rb] = floatx4{0.f, 0.f, 0.f, 0.f};

    // S^T[token][row] = sum_d K[token][d] Q[row][d]
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
        for (int ks = 0; ks < G::KS; ++ks) {
            bf16x8 ka = *reinterpret_cast<const bf16x8*>(kt + (tb * 16 + ln) * G::KROW + ks * 64 + lg * 16);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                s[tb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qf[rb][ks], s[tb][rb], 0, 0, 0);
        }
    }
    if (masked) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int tok = t0 + tb * 16 + lg * 4 + i;
                    if (tok > lim[rb]) s[tb][rb][i] = -INFINITY;
                }
    }

    float alpha[RB];
    bool changed = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        float mx = fmaxf(fmaxf(fmaxf(s[0][rb][0], s[0][rb][1]), fmaxf(s[0][rb][2], s[0][rb][3])),
                         fmaxf(fmaxf(s[1][rb][0], s[1][rb][1]), fmaxf(s[1][rb][2], s[1][rb][3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // the reference max only moves when the tile max exceeds it by kRescaleLog2;
        // until then p = 2^(s - ref) <= 2^kRescaleLog2, exact in the final ratio
        float m_new = (mx * c > st.m[rb] + kRescaleLog2) ? mx * c : st.m[rb];
        float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        alpha[rb] = fast_exp2(st.m[rb] - m_use);
        changed |= (m_new != st.m[rb]);
        st.m[rb] = m_new;
        float sum = 0.f;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float p = fast_exp2(fmaf(s[tb][rb][i], c, -m_use));
                s[tb][rb][i] = p;
                sum += p;
            }
        st.l[rb] = st.l[rb] * alpha[rb] + sum;
    }
    if (__any(changed)) {
#pragma unroll
        for (int db = 0; db < G::DB; ++db)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                for (int i = 0; i < 4; ++i) st.acc[db][rb][i] *= alpha[rb];
    }

    // P^T as the B operand: k-slot j of lane group lg is token 16*(j/4) + 4*lg + j%4,
    // exactly the tokens this lane holds in s[j/4][rb][j%4].
    bf16x8 pb[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < 8; ++j) pb[rb][j] = (__bf16)s[j >> 2][rb][j & 3];

    // O^T[d][row] += sum_token V[token][d] P[row][token].  The A operand needs, per lane,
    // eight tokens of one head-dim column; ds_read_b64_tr_b16 delivers four of them per
    // read: inside a 16-lane group, lane i supplies the address of row i/4, columns
    // 4*(i%4)..+3, and receives column i of rows 0..3.
#pragma unroll
    for (int db = 0; db < G::DB; ++db) {
        s16x4 half[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int row = h * 16 + lg * 4 + (ln >> 2);
            int pu = db ^ v_swz(row);
            half[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(vt + row * G::VROW + pu * 32 + (ln & 3) * 8));
        }
        s16x8 both = __builtin_shufflevector(half[0], half[1], 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 va = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            st.acc[db][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[rb], st.acc[db][rb], 0, 0, 0);
    }
}

template <int D, int RB, bool PAGED>
__global__ void __launch_bounds__(kWaves * 64) verify_attn_split(AttnLaunch a)
{
    using G = Geo<D>;
    constexpr int RP = RB * 16;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
    const int L = a.ctx_lens[b];
    const int c0 = split * a.chunk;
    if (c0 >= L) return;                             // this split holds no token of sequence b
    const int c1 = min(c0 + a.chunk, L);
    const int Q = (a.gammas ? a.gammas[b] : a.gamma) + 1;
    const int R = Q * a.G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;

    // Q^T as the B operand of the score product, kept in registers for the whole split.
    bf16x8 qf[RB][G::KS];
    int lim[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        int row = rb * 16 + ln;
        bool real = row < R;
        int qi = real ? row / a.G : 0, qg = real ? row % a.G : 0;
        lim[rb] = min(real ? L - Q + qi : L - 1, c1 - 1);   // last key this row may see in this split
        const uint16_t* qrow = a.q + (((int64_t)b * a.Qmax + qi) * a.Hq + hkv * a.G + qg) * D;
#pragma unroll
        for (int ks = 0; ks < G::KS; ++ks) {
            u32x4 raw = real ? *reinterpret_cast<const u32x4*>(qrow + ks * 32 + lg * 8) : u32x4{0, 0, 0, 0};
            qf[rb][ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    WaveState<D, RB> st;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        st.m[rb] = -INFINITY;
        st.l[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < G::DB; ++db) st.acc[db][rb] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    char* kt = smem + wave * G::WAVE_LDS;
    char* vt = kt + kTile * G::KROW;
    const int ntile = (c1 - c0 + kTile - 1) / kTile;
    const int nt = ntile > wave ? (ntile - wave + kWaves - 1) / kWaves : 0;   // tiles of this wave
    const int last_tok = c1 - 1;
    const float c = a.scale_log2e;
    const int first_masked_t0 = min(L - Q, c1) - (kTile - 1);   // tiles with t0 >= this hold masked keys
    auto tile_t0 = [&](int it) { return c0 + (wave + it * kWaves) * kTile; };

    // Two tiles are always in flight.  Prefetches are unconditional (rows past the
    // split are clamped to its last row and masked) and tiles go in pairs (a wave
    // with an odd count runs one fully masked tile), so that the loop body has no
    // branch and the load counters stay exact.
    const RowAddr addr = make_row_addr<PAGED>(a, b, hkv);
    if (nt > 0) {
        TileRegs<D> ra, rb2;
        load_tile<D, PAGED>(ra, addr, tile_t0(0), last_tok, lane);
        load_tile<D, PAGED>(rb2, addr, tile_t0(1), last_tok, lane);
        for (int it = 0; it < nt; it += 2) {
            store_tile<D>(ra, kt, vt, lane);
            load_tile<D, PAGED>(ra, addr, tile_t0(it + 2), last_tok, lane);
            __builtin_amdgcn_wave_barrier();
            compute_tile<D, RB>(st, qf, kt, vt, tile_t0(it), tile_t0(it) >= first_masked_t0, lim, c, lane);
            __builtin_amdgcn_wave_barrier();
            store_tile<D>(rb2, kt, vt, lane);
            load_tile<D, PAGED>(rb2, addr, tile_t0(it + 3), last_tok, lane);
            __builtin_amdgcn_wave_barrier();
            compute_tile<D, RB>(st, qf, kt, vt, tile_t0(it + 1), tile_t0(it + 1) >= first_masked_t0, lim, c, lane);
            __builtin_amdgcn_wave_barrier();
        }
    }

    // Row sums were kept per lane group; make them whole.
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        st.l[rb] += __shfl_xor(st.l[rb], 16);
        st.l[rb] += __shfl_xor(st.l[rb], 32);
    }

    // ---- combine the four waves (fixed order) and write the split's partial
    __syncthreads();                                  // staging tiles are dead from here on
    float* obuf = reinterpret_cast<float*>(smem);     // [D][RP+1]
    float* mlbuf = obuf + D * (RP + 1);               // [kWaves][RP][2]
    if (lg == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            mlbuf[(wave * RP + rb * 16 + ln) * 2 + 0] = st.m[rb];
            mlbuf[(wave * RP + rb * 16 + ln) * 2 + 1] = st.l[rb];
        }
    }
    __syncthreads();
    float m_all[RB], l_all[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        int row = rb * 16 + ln;
        float mm = -INFINITY;
        for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, mlbuf[(w * RP + row) * 2]);
        float m_use = (mm == -INFINITY) ? 0.f : mm;
        float ll = 0.f;
        for (int w = 0; w < kWaves; ++w)
            ll += mlbuf[(w * RP + row) * 2 + 1] * fast_exp2(mlbuf[(w * RP + row) * 2] - m_use);
        float f = fast_exp2(st.m[rb] - m_use);
        m_all[rb] = mm;
        l_all[rb] = ll;
#pragma unroll
        for (int db = 0; db < G::DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) st.acc[db][rb][i] *= f;
    }
    for (int w = 0; w < kWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int db = 0; db < G::DB; ++db)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        int idx = (db * 16 + lg * 4 + i) * (RP + 1) + rb * 16 + ln;
                        if (w == 0) obuf[idx] = st.acc[db][rb][i];
                        else obuf[idx] += st.acc[db][rb][i];
                    }
        }
        __syncthreads();
    }
    const int64_t pbase = (((int64_t)b * a.Hkv + hkv) * a.nsplit + split) * RP;
    float* po = a.part_o + pbase * D;
    for (int idx = tid; idx < R * D; idx += kWaves * 64) {
        int row = idx / D, d = idx % D;
        po[idx] = obuf[d * (RP + 1) + row];
    }
    if (wave == 0 && lg == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            int row = rb * 16 + ln;
            if (row < R) {
                a.part_ml[(pbase + row) * 2 + 0] = m_all[rb];
                a.part_ml[(pbase + row) * 2 + 1] = l_all[rb];
            }
        }
    }
}

// Merge the splits of one (sequence, kv head): out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
template <int D>
__global__ void __launch_bounds__(256) verify_attn_merge(AttnLaunch a)
{
    constexpr int ROWS = 256 / D;
    const int hkv = blockIdx.y, b = blockIdx.z;
    const int row = blockIdx.x * ROWS + threadIdx.x / D, d = threadIdx.x % D;
    const int Rmax = a.Qmax * a.G;
    if (row >= Rmax) return;
    const int L = a.ctx_lens[b];
    const int Q = (a.gammas ? a.gammas[b] : a.gamma) + 1;
    const int R = Q * a.G, RP = a.RB * 16;
    const int qi = row / a.G, qg = row % a.G;
    const int h = hkv * a.G + qg;
    uint16_t* dst = a.out + (((int64_t)b * a.Qmax + qi) * a.Hq + h) * D + d;
    if (row >= R) {                                   // query rows this sequence does not have
        *dst = 0;
        if (a.lse_out && d == 0) a.lse_out[((int64_t)b * a.Hq + h) * a.Qmax + qi] = 0.f;
        return;
    }
    const int ns = min((L + a.chunk - 1) / a.chunk, a.nsplit);
    const int64_t pbase = ((int64_t)b * a.Hkv + hkv) * a.nsplit * RP;
    float M = -INFINITY;
    for (int s = 0; s < ns; ++s) M = fmaxf(M, a.part_ml[(pbase + (int64_t)s * RP + row) * 2]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < ns; ++s) {
        int64_t pr = pbase + (int64_t)s * RP + row;
        float w = fast_exp2(a.part_ml[pr * 2] - M);
        den += w * a.part_ml[pr * 2 + 1];
        num += w * a.part_o[pr * D + d];
    }
    float o = den > 0.f ? num / den : 0.f;
    __bf16 ob = (__bf16)o;
    *dst = __builtin_bit_cast(uint16_t, ob);
    if (a.lse_out && d == 0)
        a.lse_out[((int64_t)b * a.Hq + h) * a.Qmax + qi] = (M + log2f(den)) * 0.6931471805599453f;
}

template <int D, int RB, bool PAGED>
hipError_t launch_split(const AttnLaunch& a, hipStream_t stream)
{
    constexpr int lds = attn_lds_bytes<D, RB>();
    static bool configured[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    auto fn = verify_attn_split<D, RB, PAGED>;
    if (dev < 64 && !configured[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        configured[dev] = true;
    }
    dim3 grid(a.nsplit, a.Hkv, a.B), block(kWaves * 64);
    hipLaunchKernelGGL(fn, grid, block, lds, stream, a);
    return hipGetLastError();
}

template <int D, bool PAGED>
hipError_t dispatch_rb(const AttnLaunch& a, hipStream_t stream)
{
    switch (a.RB) {
        case 1: return launch_split<D, 1, PAGED>(a, stream);
        case 2: return launch_split<D, 2, PAGED>(a, stream);
        case 3: return launch_split<D, 3, PAGED>(a, stream);
        case 4: return launch_split<D, 4, PAGED>(a, stream);
        case 5: return launch_split<D, 5, PAGED>(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace

size_t attn_workspace_bytes(int B, int Hkv, int nsplit, int RB, int D)
{
    size_t rows = (size_t)B * Hkv * nsplit * RB * 16;
    size_t o = rows * D * sizeof(float), ml = rows * 2 * sizeof(float);
    return ((o + 255) / 256) * 256 + ((ml + 255) / 256) * 256;
}

hipError_t launch_verify_attn(const AttnLaunch& a, hipStream_t stream)
{
    hipError_t e;
    const bool paged = a.page_shift >= 0;
    if (a.D == 128) e = paged ? dispatch_rb<128, true>(a, stream) : dispatch_rb<128, false>(a, stream);
    else if (a.D == 64) e = paged ? dispatch_rb<64, true>(a, stream) : dispatch_rb<64, false>(a, stream);
    else return hipErrorInvalidValue;
    if (e != hipSuccess) return e;
    const int rows_per_block = 256 / a.D;
    dim3 grid((a.Qmax * a.G + rows_per_block - 1) / rows_per_block, a.Hkv, a.B);
    if (a.D == 128) hipLaunchKernelGGL(verify_attn_merge<128>, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(verify_attn_merge<64>, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}
