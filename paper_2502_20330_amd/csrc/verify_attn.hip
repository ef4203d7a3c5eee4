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
//    independent pipelines, each over its own contiguous quarter of the split in
//    32-token tiles.  K and V tiles travel
//    HBM -> LDS directly (global_load_lds_dwordx4, 1 KiB per instruction, no
//    staging registers) into a private two-slot ring per wave, two tiles ahead of
//    the math; the wave waits on its own load counter, so the main loop has no
//    workgroup barrier.
//  * The lane -> global-chunk assignment of those loads applies an XOR swizzle,
//    so that the later LDS reads (128-bit rows for K, transposed 64-bit reads for
//    V) spread over all 64 banks without padding.
//  * Scores are produced transposed (S^T = K Q^T: tokens on M, query rows on N): a
//    query row's running max/sum then lives in one lane column, so the online
//    softmax needs two cross-lane steps per tile instead of a butterfly per row.
//    The running max is only moved when it grows by more than 2^8, so the
//    accumulator rescale almost never runs.
//  * V is token-major in memory but the PV product reduces over tokens:
//    ds_read_b64_tr_b16 delivers the transposed MFMA operand straight from LDS.
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

constexpr int kTile = 32;              // tokens per wave tile
constexpr int kWaves = 4;              // waves per workgroup
constexpr float kRescaleLog2 = 8.0f;   // lazy rescale threshold (log2 units)

template <int D>
struct Geo {
    static constexpr int KS = D / 32;             // MFMA k-steps of the QK product
    static constexpr int DB = D / 16;             // 16-wide blocks of the head dim (PV M side)
    static constexpr int ROWB = D * 2;            // bytes of one K or V row
    static constexpr int CPR = ROWB / 16;         // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;          // rows moved by one wave-wide 1 KiB load
    static constexpr int NLD = kTile / RPI;       // load instructions per tile per tensor
    static constexpr int SLOT = kTile * ROWB;     // bytes of one K or V tile
    static constexpr int WAVE_LDS = 4 * SLOT;     // K ring (2 slots) + V ring (2 slots)
};

template <int D, int RB>
constexpr int attn_lds_bytes()
{
    constexpr int tiles = kWaves * Geo<D>::WAVE_LDS + RB * 16 * Geo<D>::ROWB;   // rings + the Q block
    constexpr int merge = (2 * RB * 16 * (D + 4) + kWaves * RB * 16 * 2) * 4;
    return tiles > merge ? tiles : merge;
}

// LDS swizzles (16-byte chunk index within a row).  The LDS of this chip serves 64 banks of
// 4 bytes per cycle: 16 lanes of a 128-bit read, 32 lanes of a 64-bit read.  Rows are unpadded
// (256 B at d = 128, 128 B at d = 64), so without a swizzle all rows of an operand read would
// hit the same banks.
//   K / Q (ds_read_b128: 16 consecutive rows, same logical chunk): chunk c of row r is stored at
//      c ^ (r & 15) for 256-byte rows; 128-byte rows pair up per 256 bytes, so there the row
//      pair index does the work: c ^ ((r >> 1) & 7).
//   V (transposed 64-bit reads: 8 consecutive rows, each lane group of four reading 32 bytes):
//      the 32-byte unit u = c / 2 of row r is stored at u ^ (r & 7), i.e. c ^ 2 (r & 7);
//      128-byte rows: c ^ 2 ((r >> 1) & 3).
template <int D> __device__ __forceinline__ int k_swz(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D> __device__ __forceinline__ int v_swz(int row) { return D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1); }

// Where the rows of this (sequence, kv head) start.  A wave-uniform base pointer
// plus a 32-bit byte offset per lane (the host checks that a sequence, or a page,
// spans less than 4 GiB); paged caches add a uniform page base per load.
struct RowAddr {
    const char* kbase;
    const char* vbase;
    // page table row of this sequence (paged only), read through the constant address
    // space so that the uniform lookups become scalar loads
    const __attribute__((address_space(4))) int32_t* pages;
    uint32_t tok_bytes;        // bytes between consecutive tokens
    int64_t page_bytes;        // bytes between pages
    int page_shift, page_mask;
    int page_hi;               // page ids (device data) are clamped to [0, page_hi]
};

template <bool PAGED>
__device__ __forceinline__ RowAddr make_row_addr(const AttnLaunch& a, int b, int hkv)
{
    RowAddr r;
    int64_t head = (int64_t)hkv * a.hstride + (PAGED ? 0 : (int64_t)b * a.bstride);
    r.kbase = reinterpret_cast<const char*>(a.k + head);
    r.vbase = reinterpret_cast<const char*>(a.v + head);
    r.pages = PAGED ? (const __attribute__((address_space(4))) int32_t*)(a.page_table + (int64_t)b * a.max_pages) : nullptr;
    r.tok_bytes = (uint32_t)(a.tstride * 2);
    r.page_bytes = a.pstride * 2;
    r.page_shift = a.page_shift;
    r.page_mask = a.page_mask;
    r.page_hi = a.page_hi;
    return r;
}

// Issue the HBM -> LDS loads of one 32-token tile of K or of V into `slot`
// (wave-uniform LDS address).  Each instruction moves RPI whole rows: lane i
// writes LDS bytes [16 i, 16 i + 16) of that 1 KiB block and fetches the global
// chunk that the swizzle assigns to that position.  Rows past `last_tok` are
// clamped to it (always a valid address); the softmax masks them.
//
// The instruction is written as inline assembly on purpose: the wave keeps its own
// account of outstanding loads (wait_loads<N>() below).  Issued through the
// compiler's builtin, every later LDS read would be preceded by a compiler-inserted
// wait for ALL outstanding loads, which serialises the pipeline.  `nt` marks the
// data as streaming (read once): measured +5..10 % bandwidth over the default policy.
__device__ __forceinline__ void dma16(const char* base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(byte_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
// The same load without the streaming hint, for data that other workgroups read again (Q).
__device__ __forceinline__ void dma16_keep(const char* base, uint32_t byte_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(byte_off), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}

template <int D, bool PAGED, bool IS_V>
__device__ __forceinline__ void dma_tile(const RowAddr& ra, uint32_t slot, int t0, int last_tok, int lane)
{
    using G = Geo<D>;
    const char* base = IS_V ? ra.vbase : ra.kbase;
    const int r_local = lane / G::CPR, cpos = lane % G::CPR;
#pragma unroll
    for (int e = 0; e < G::NLD; ++e) {
        const int row = e * G::RPI + r_local;
        const int c = cpos ^ (IS_V ? v_swz<D>(row) : k_swz<D>(row));
        const int tok = min(t0 + row, last_tok);
        if (PAGED) {
            // the RPI rows of one instruction lie in one page (pages hold >= 16 tokens)
            const int tok0 = min(t0 + e * G::RPI, last_tok);
            const int64_t pg = min(max(ra.pages[tok0 >> ra.page_shift], 0), ra.page_hi);
            dma16(base + pg * ra.page_bytes, (uint32_t)(tok & ra.page_mask) * ra.tok_bytes + (uint32_t)c * 16u,
                  slot + e * 1024);
        } else {
            dma16(base, (uint32_t)tok * ra.tok_bytes + (uint32_t)c * 16u, slot + e * 1024);
        }
    }
}

// Wait until at most N of this wave's vector-memory loads are outstanding.  The
// loads complete in order, so this guarantees everything older has landed in LDS.
template <int N>
__device__ __forceinline__ void wait_loads()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// All LDS reads issued so far have returned: the slot they read may be refilled.
__device__ __forceinline__ void lds_reads_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D, int RB>
struct WaveState {
    float m[RB];                     // reference max per query row, log2 units (score*scale*log2e)
    float l[RB];                     // running sum, this lane group's tokens only
    floatx4 acc[Geo<D>::DB][RB];     // O^T: d = 16*db + 4*(lane/16) + i, row = 16*rb + lane%16
};

// S^T[token][row] = sum_d K[token][d] Q[row][d] for the 32 tokens in `kt`.
template <int D, int RB>
__device__ __forceinline__ void score_tile(floatx4 (&s)[2][RB], const bf16x8 (&qf)[RB][Geo<D>::KS],
                                           const char* kt, int lane)
{
    using G = Geo<D>;
    const int ln = lane & 15, lg = lane >> 4;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) s[tb][rb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < G::KS; ++ks) {
            const int row = tb * 16 + ln;
            const int c = (ks * 4 + lg) ^ k_swz<D>(row);
            bf16x8 ka = *reinterpret_cast<const bf16x8*>(kt + row * G::ROWB + c * 16);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                s[tb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qf[rb][ks], s[tb][rb], 0, 0, 0);
        }
    }
}

// Mask, online softmax with lazy rescale; leaves P^T packed as the B operand of PV.
template <int D, int RB>
__device__ __forceinline__ void softmax_tile(WaveState<D, RB>& st, floatx4 (&s)[2][RB], bf16x8 (&pb)[RB],
                                             int t0, bool masked, const int (&lim)[RB], float c, int lane)
{
    using G = Geo<D>;
    const int lg = lane >> 4;
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
    // k-slot j of lane group lg is token 16*(j/4) + 4*lg + j%4: exactly the tokens this
    // lane holds in s[j/4][rb][j%4].
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < 8; ++j) pb[rb][j] = (__bf16)s[j >> 2][rb][j & 3];
}

// O^T[d][row] += sum_token V[token][d] P[row][token].  The A operand needs, per lane,
// eight tokens of one head-dim column; ds_read_b64_tr_b16 delivers four of them per
// read: inside a 16-lane group, lane i supplies the address of row i/4, columns
// 4*(i%4)..+3, and receives column i of rows 0..3.
template <int D, int RB>
__device__ __forceinline__ void pv_tile(WaveState<D, RB>& st, const bf16x8 (&pb)[RB], char* vt, int lane)
{
    using G = Geo<D>;
    const int ln = lane & 15, lg = lane >> 4;
#pragma unroll
    for (int db = 0; db < G::DB; ++db) {
        s16x4 half[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int row = h * 16 + lg * 4 + (ln >> 2);
            const int c = (db * 2) ^ v_swz<D>(row);                // chunk pair of the 32-byte column unit
            half[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(vt + row * G::ROWB + c * 16 + (ln & 3) * 8));
        }
        s16x8 both = __builtin_shufflevector(half[0], half[1], 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 va = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            st.acc[db][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[rb], st.acc[db][rb], 0, 0, 0);
    }
}

// Query positions of sequence b (gamma_b + 1); device data, so clamped to the rows q / out hold.
__device__ __forceinline__ int seq_queries(const AttnLaunch& a, int b)
{
    return min(max(a.gammas ? a.gammas[b] : a.gamma, 0), a.Qmax - 1) + 1;
}

// Token range of split s of kv head h.  Splits come in pairs that cover 2*chunk
// tokens; the member of a pair that runs on an even dispatch slot takes chunk + skew
// tokens, the other chunk - skew (see the slot -> head mapping in the kernel).  An
// unpaired last split keeps `chunk`.
__device__ __forceinline__ int split_begin(const AttnLaunch& a, int s, int h)
{
    int t = (s >> 1) * 2 * a.chunk;
    if (s & 1) t += a.chunk + ((h & 1) ? -a.skew : a.skew);
    return t;
}
__device__ __forceinline__ int split_end(const AttnLaunch& a, int s, int h)
{
    return s + 1 < a.nsplit ? split_begin(a, s + 1, h) : a.nsplit * a.chunk;
}

template <int D, int RB, bool PAGED>
__global__ void __launch_bounds__(kWaves * 64) verify_attn_split(AttnLaunch a)
{
    using G = Geo<D>;
    constexpr int RP = RB * 16;
    constexpr int kAhead = 3 * G::NLD;     // loads issued after the tile a wait is for
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    // With rotation, dispatch slot x = blockIdx.x serves kv head (x + split) mod Hkv.
    // Workgroups go to the chip's eight dies round robin in dispatch order, so the
    // splits of one head are then spread over all dies (and all L2s) instead of
    // sitting on one, and the parity of x is the parity of the die.  Without it,
    // the heads of one token range sit next to each other in dispatch order, which
    // suits caches whose heads interleave inside a token row.
    const int split = blockIdx.y, b = blockIdx.z;
    const int hkv = a.rot ? (int)((blockIdx.x + split) % a.Hkv) : (int)blockIdx.x;
    const int L = min(a.ctx_lens[b], a.max_ctx);        // device data: never address past the planned range
    const int c0 = split_begin(a, split, hkv);
    if (c0 >= L) return;                             // this split holds no token of sequence b
    const int c1 = min(split_end(a, split, hkv), L);
    const int Q = seq_queries(a, b);
    const int R = Q * a.G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 15, lg = lane >> 4;

    const int ntile = (c1 - c0 + kTile - 1) / kTile;
    // each wave streams its own contiguous quarter of the split
    const int ntq = (ntile + kWaves - 1) / kWaves;
    const int nt = max(0, min(ntq, ntile - wave * ntq));                      // tiles of this wave
    // last token this wave may load: prefetches past its range are clamped to this row
    const int last_tok = min(c1, c0 + (wave + 1) * ntq * kTile) - 1;
    auto tile_t0 = [&](int it) { return c0 + (wave * ntq + it) * kTile; };
    const RowAddr addr = make_row_addr<PAGED>(a, b, hkv);
    char* kring = smem + wave * G::WAVE_LDS;
    char* vring = kring + 2 * G::SLOT;
    const uint32_t kring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + wave * G::WAVE_LDS;
    const uint32_t vring_lds = kring_lds + 2 * G::SLOT;

    // Q block of this kv head: RP rows of D bf16, HBM -> LDS once per workgroup, each wave
    // fetching a share.  These loads are issued BEFORE the first K/V tiles: loads return in
    // order, so Q is complete as soon as only the tile loads are still outstanding, and the
    // math can start on tile 0 while tile 1 is still in flight.  (Waiting for everything
    // here would let all 1024 waves of the grid drain the memory pipeline at the same
    // moment, right after the start.)  Rows past the real ones repeat a valid row and are
    // zeroed when read.
    char* qlds = smem + kWaves * G::WAVE_LDS;
    {
        const uint32_t q_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + kWaves * G::WAVE_LDS;
        constexpr int QI = RP / G::RPI;                  // 1 KiB loads that make up the block
        const int last_row = a.Qmax * a.G - 1;
        for (int e = wave; e < QI; e += kWaves) {
            const int row = e * G::RPI + lane / G::CPR;
            const int rr = min(row, last_row);
            const int qi = rr / a.G, qg = rr % a.G;
            const int c = (lane % G::CPR) ^ k_swz<D>(row);
            const uint32_t off = (uint32_t)(((((int64_t)b * a.Qmax + qi) * a.Hq + hkv * a.G + qg) * D) * 2) + c * 16;
            dma16_keep(reinterpret_cast<const char*>(a.q), off, q_lds + e * 1024);
        }
    }

    // Start the pipeline: tiles 0 and 1 of this wave.
    if (nt > 0) {
        dma_tile<D, PAGED, false>(addr, kring_lds, tile_t0(0), last_tok, lane);
        dma_tile<D, PAGED, true>(addr, vring_lds, tile_t0(0), last_tok, lane);
        dma_tile<D, PAGED, false>(addr, kring_lds + G::SLOT, tile_t0(1), last_tok, lane);
        dma_tile<D, PAGED, true>(addr, vring_lds + G::SLOT, tile_t0(1), last_tok, lane);
        wait_loads<4 * G::NLD>();                       // everything older than the four tiles: Q
    } else {
        wait_loads<0>();
    }
    __syncthreads();                                     // the whole Q block is in LDS

    // Q^T as the B operand of the score product, kept in registers for the whole split.
    bf16x8 qf[RB][G::KS];
    int lim[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = rb * 16 + ln;
        const bool real = row < R;
        const int qi = real ? row / a.G : 0;
        lim[rb] = min(real ? L - Q + qi : L - 1, c1 - 1);   // last key this row may see in this split
#pragma unroll
        for (int ks = 0; ks < G::KS; ++ks) {
            const int c = (ks * 4 + lg) ^ k_swz<D>(row);
            u32x4 raw = *reinterpret_cast<const u32x4*>(qlds + row * G::ROWB + c * 16);
            if (!real) raw = u32x4{0, 0, 0, 0};
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
    const float c = a.scale_log2e;
    const int first_masked_t0 = min(L - Q, c1) - (kTile - 1);   // tiles with t0 >= this hold masked keys

    // Steady state, oldest load first: K(it) V(it) K(it+1) V(it+1).  Prefetches are
    // unconditional (tiles past the split are clamped to its last row), so the
    // number of loads behind the one being waited for is always 3*NLD.
    for (int it = 0; it < nt; ++it) {
        char* kt = kring + (it & 1) * G::SLOT;
        char* vt = vring + (it & 1) * G::SLOT;
        const int t0 = tile_t0(it);
        floatx4 s[2][RB];
        bf16x8 pb[RB];

        wait_loads<kAhead>();                        // K(it) has landed
        score_tile<D, RB>(s, qf, kt, lane);
        lds_reads_done();
        dma_tile<D, PAGED, false>(addr, kring_lds + (it & 1) * G::SLOT, tile_t0(it + 2), last_tok, lane);

        softmax_tile<D, RB>(st, s, pb, t0, t0 >= first_masked_t0, lim, c, lane);

        wait_loads<kAhead>();                        // V(it) has landed
        pv_tile<D, RB>(st, pb, vt, lane);
        lds_reads_done();
        dma_tile<D, PAGED, true>(addr, vring_lds + (it & 1) * G::SLOT, tile_t0(it + 2), last_tok, lane);
    }
    wait_loads<0>();                                 // no load may land after the ring is reused below

    // Row sums were kept per lane group; make them whole.
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        st.l[rb] += __shfl_xor(st.l[rb], 16);
        st.l[rb] += __shfl_xor(st.l[rb], 32);
    }

    // ---- combine the four waves and write the split's partial.
    // Waves 2 and 3 park their accumulators in LDS; waves 0 and 1 fold their partner's
    // into their own (both brought to the workgroup's reference max) and write the
    // pair sums back; then all threads add the two pair sums and store coalesced.
    // The order of the additions is fixed, so results do not depend on timing.
    __syncthreads();                                  // all rings are dead from here on
    constexpr int OROW = D + 4;                       // padded row of the exchange buffers (floats)
    float* obuf = reinterpret_cast<float*>(smem);     // [2][RP][OROW]
    float* mlbuf = obuf + 2 * RP * OROW;              // [kWaves][RP][2]
    if (lg == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            mlbuf[(wave * RP + rb * 16 + ln) * 2 + 0] = st.m[rb];
            mlbuf[(wave * RP + rb * 16 + ln) * 2 + 1] = st.l[rb];
        }
    }
    float* mine = obuf + (wave & 1) * RP * OROW;
    if (wave >= 2) {
#pragma unroll
        for (int db = 0; db < G::DB; ++db)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                *reinterpret_cast<floatx4*>(mine + (rb * 16 + ln) * OROW + db * 16 + lg * 4) = st.acc[db][rb];
    }
    __syncthreads();
    float m_all[RB], l_all[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = rb * 16 + ln;
        float mw[kWaves];
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            mw[w] = mlbuf[(w * RP + row) * 2];
            mm = fmaxf(mm, mw[w]);
        }
        const float m_use = (mm == -INFINITY) ? 0.f : mm;
        float ll = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) ll += mlbuf[(w * RP + row) * 2 + 1] * fast_exp2(mw[w] - m_use);
        m_all[rb] = mm;
        l_all[rb] = ll;
        if (wave < 2) {
            const float f_own = fast_exp2(mw[wave] - m_use), f_par = fast_exp2(mw[wave + 2] - m_use);
#pragma unroll
            for (int db = 0; db < G::DB; ++db) {
                float* cell = mine + row * OROW + db * 16 + lg * 4;
                floatx4 other = *reinterpret_cast<const floatx4*>(cell);
                *reinterpret_cast<floatx4*>(cell) = st.acc[db][rb] * f_own + other * f_par;
            }
        }
    }
    __syncthreads();
    const int64_t pbase = (((int64_t)b * a.Hkv + hkv) * a.nsplit + split) * RP;
    floatx4* po = reinterpret_cast<floatx4*>(a.part_o + pbase * D);
    for (int f = tid; f < R * (D / 4); f += kWaves * 64) {
        const int row = f / (D / 4), d4 = f % (D / 4);
        const floatx4 x = *reinterpret_cast<const floatx4*>(obuf + row * OROW + d4 * 4);
        const floatx4 y = *reinterpret_cast<const floatx4*>(obuf + (RP + row) * OROW + d4 * 4);
        po[f] = x + y;
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

// ---------------------------------------------------------------- wide row counts: two row teams
// Above 64 packed rows (five or six row blocks) one wave per SIMD is nearly compute bound: the MFMA
// work and the softmax of a tile leave no slack to hide LDS and wait latency.  The wide kernel runs
// eight waves: wave (team, p) = (wave / 4, wave % 4).  The two waves of pair p share the K/V ring of
// token quarter p and each takes RBT of the 2*RBT row blocks, so every K/V byte is still fetched once
// per workgroup and each SIMD holds two waves that fill each other's stalls.  Each wave of a pair
// issues half of the load instructions of every tile and waits on its own counter; two workgroup
// barriers per tile make the halves visible to the partner and tell it when a slot may be refilled:
//     wait own K(it) | barrier A | issue V(it+1) | scores, softmax | wait own V(it) | barrier B |
//     issue K(it+2) | PV
// Barrier A: K(it) is complete, and everybody has finished PV(it-1), so V slot (it+1)&1 is free.
// Barrier B: V(it) is complete, and everybody has finished the scores of it, so K slot it&1 is free.
template <int D, bool PAGED, bool IS_V>
__device__ __forceinline__ void dma_half_tile(const RowAddr& ra, uint32_t slot, int t0, int last_tok, int lane, int half)
{
    using G = Geo<D>;
    const char* base = IS_V ? ra.vbase : ra.kbase;
    const int r_local = lane / G::CPR, cpos = lane % G::CPR;
#pragma unroll
    for (int h = 0; h < G::NLD / 2; ++h) {
        const int e = half * (G::NLD / 2) + h;
        const int row = e * G::RPI + r_local;
        const int c = cpos ^ (IS_V ? v_swz<D>(row) : k_swz<D>(row));
        const int tok = min(t0 + row, last_tok);
        if (PAGED) {
            const int tok0 = min(t0 + e * G::RPI, last_tok);
            const int64_t pg = min(max(ra.pages[tok0 >> ra.page_shift], 0), ra.page_hi);
            dma16(base + pg * ra.page_bytes, (uint32_t)(tok & ra.page_mask) * ra.tok_bytes + (uint32_t)c * 16u,
                  slot + e * 1024);
        } else {
            dma16(base, (uint32_t)tok * ra.tok_bytes + (uint32_t)c * 16u, slot + e * 1024);
        }
    }
}

template <int D, int RB0, int RB1>
constexpr int attn_wide_lds_bytes()
{
    constexpr int RBM = RB0 > RB1 ? RB0 : RB1;
    constexpr int tiles = kWaves * Geo<D>::WAVE_LDS + (RB0 + RB1) * 16 * Geo<D>::ROWB;          // four rings + the Q block
    constexpr int merge = (2 * (RB0 + RB1) * 16 * (D + 4) + 2 * kWaves * RBM * 16 * 2) * 4;   // two teams' exchange buffers
    return tiles > merge ? tiles : merge;
}

// What a wave of the wide kernel knows before its team's part begins.
struct WideWave {
    RowAddr addr;
    char *kring, *vring, *qlds;
    uint32_t kring_lds, vring_lds;
    int b, hkv, split, L, Q, R, c0, c1, ntq, last_tok;
    int lane, wave, team, pr;
};

// One team's share of the wide kernel: RBT row blocks starting at packed row `row0`, from the Q
// fragments to the team's partial in LDS (obuf: [2][RBT * 16][D + 4] floats; mlbuf: [8 waves][MLS][2]).
// Both teams execute the same sequence of workgroup barriers (two per tile, three afterwards), so the
// two instantiations of a kernel with unequal teams may sit in the two arms of a wave-uniform branch.
template <int D, int RBT, int MLS, bool PAGED>
__device__ __forceinline__ void wide_team(const AttnLaunch& a, const WideWave& w, char* smem, int row0, float* obuf,
                                          float* mlbuf, int64_t pbase)
{
    using G = Geo<D>;
    constexpr int RPT = RBT * 16;          // rows of this team
    constexpr int kWait = G::NLD;          // own loads issued after the tile a wait is for (two half tiles)
    const int lane = w.lane, wave = w.wave, team = w.team, pr = w.pr;
    const int ln = lane & 15, lg = lane >> 4;
    const int L = w.L, Q = w.Q, R = w.R, c0 = w.c0, c1 = w.c1, ntq = w.ntq, last_tok = w.last_tok;
    auto tile_t0 = [&](int it) { return c0 + (pr * ntq + it) * kTile; };

    bf16x8 qf[RBT][G::KS];
    int lim[RBT];
#pragma unroll
    for (int rb = 0; rb < RBT; ++rb) {
        const int row = row0 + rb * 16 + ln;
        const bool real = row < R;
        const int qi = real ? row / a.G : 0;
        lim[rb] = min(real ? L - Q + qi : L - 1, c1 - 1);
#pragma unroll
        for (int ks = 0; ks < G::KS; ++ks) {
            const int c = (ks * 4 + lg) ^ k_swz<D>(row);
            u32x4 raw = *reinterpret_cast<const u32x4*>(w.qlds + row * G::ROWB + c * 16);
            if (!real) raw = u32x4{0, 0, 0, 0};
            qf[rb][ks] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    WaveState<D, RBT> st;
#pragma unroll
    for (int rb = 0; rb < RBT; ++rb) {
        st.m[rb] = -INFINITY;
        st.l[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < G::DB; ++db) st.acc[db][rb] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    const float c = a.scale_log2e;
    const int first_masked_t0 = min(L - Q, c1) - (kTile - 1);
    // (tiles of this quarter past the end of the split start at t0 >= c1: every key of theirs is masked)

    for (int it = 0; it < ntq; ++it) {
        char* kt = w.kring + (it & 1) * G::SLOT;
        char* vt = w.vring + (it & 1) * G::SLOT;
        const int t0 = tile_t0(it);
        floatx4 s[2][RBT];
        bf16x8 pb[RBT];

        wait_loads<kWait>();                         // own half of K(it) has landed
        __syncthreads();                             // barrier A
        dma_half_tile<D, PAGED, true>(w.addr, w.vring_lds + ((it + 1) & 1) * G::SLOT, tile_t0(it + 1), last_tok, lane, team);
        score_tile<D, RBT>(s, qf, kt, lane);
        softmax_tile<D, RBT>(st, s, pb, t0, t0 >= first_masked_t0, lim, c, lane);

        wait_loads<kWait>();                         // own half of V(it) has landed
        lds_reads_done();
        __syncthreads();                             // barrier B
        dma_half_tile<D, PAGED, false>(w.addr, w.kring_lds + (it & 1) * G::SLOT, tile_t0(it + 2), last_tok, lane, team);
        pv_tile<D, RBT>(st, pb, vt, lane);
        lds_reads_done();
    }
    wait_loads<0>();

#pragma unroll
    for (int rb = 0; rb < RBT; ++rb) {
        st.l[rb] += __shfl_xor(st.l[rb], 16);
        st.l[rb] += __shfl_xor(st.l[rb], 32);
    }

    // ---- combine the four waves of the team (fixed order)
    __syncthreads();                                  // all rings are dead from here on
    constexpr int OROW = D + 4;
    if (lg == 0) {
#pragma unroll
        for (int rb = 0; rb < RBT; ++rb) {
            mlbuf[(wave * MLS + rb * 16 + ln) * 2 + 0] = st.m[rb];
            mlbuf[(wave * MLS + rb * 16 + ln) * 2 + 1] = st.l[rb];
        }
    }
    float* mine = obuf + (pr & 1) * RPT * OROW;
    if (pr >= 2) {
#pragma unroll
        for (int db = 0; db < G::DB; ++db)
#pragma unroll
            for (int rb = 0; rb < RBT; ++rb)
                *reinterpret_cast<floatx4*>(mine + (rb * 16 + ln) * OROW + db * 16 + lg * 4) = st.acc[db][rb];
    }
    __syncthreads();
    float m_all[RBT], l_all[RBT];
#pragma unroll
    for (int rb = 0; rb < RBT; ++rb) {
        const int row = rb * 16 + ln;
        float mw[kWaves];
        float mm = -INFINITY;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) {
            mw[v] = mlbuf[((team * kWaves + v) * MLS + row) * 2];
            mm = fmaxf(mm, mw[v]);
        }
        const float m_use = (mm == -INFINITY) ? 0.f : mm;
        float ll = 0.f;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) ll += mlbuf[((team * kWaves + v) * MLS + row) * 2 + 1] * fast_exp2(mw[v] - m_use);
        m_all[rb] = mm;
        l_all[rb] = ll;
        if (pr < 2) {
            const float f_own = fast_exp2(mw[pr] - m_use), f_par = fast_exp2(mw[pr + 2] - m_use);
#pragma unroll
            for (int db = 0; db < G::DB; ++db) {
                float* cell = mine + row * OROW + db * 16 + lg * 4;
                floatx4 other = *reinterpret_cast<const floatx4*>(cell);
                *reinterpret_cast<floatx4*>(cell) = st.acc[db][rb] * f_own + other * f_par;
            }
        }
    }
    __syncthreads();
    if (pr == 0 && lg == 0) {
#pragma unroll
        for (int rb = 0; rb < RBT; ++rb) {
            const int row = row0 + rb * 16 + ln;
            if (row < R) {
                a.part_ml[(pbase + row) * 2 + 0] = m_all[rb];
                a.part_ml[(pbase + row) * 2 + 1] = l_all[rb];
            }
        }
    }
}

// Team 0 takes RB0 row blocks, team 1 the next RB1 (RB0 >= RB1): five row blocks run as 3 + 2, so that
// no wave spends a third of its matrix and softmax work on rows that do not exist.
template <int D, int RB0, int RB1, bool PAGED>
__global__ void __launch_bounds__(2 * kWaves * 64) verify_attn_split_wide(AttnLaunch a)
{
    using G = Geo<D>;
    constexpr int RPT0 = RB0 * 16, RPT1 = RB1 * 16;
    constexpr int RP = RPT0 + RPT1;        // rows of the workgroup (= a.RB * 16)
    constexpr int MLS = RPT0 > RPT1 ? RPT0 : RPT1;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    WideWave w;
    w.split = blockIdx.y;
    w.b = blockIdx.z;
    w.hkv = a.rot ? (int)((blockIdx.x + w.split) % a.Hkv) : (int)blockIdx.x;
    w.L = min(a.ctx_lens[w.b], a.max_ctx);
    w.c0 = split_begin(a, w.split, w.hkv);
    if (w.c0 >= w.L) return;
    w.c1 = min(split_end(a, w.split, w.hkv), w.L);
    w.Q = seq_queries(a, w.b);
    w.R = w.Q * a.G;
    const int tid = threadIdx.x;
    w.lane = tid & 63;
    w.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    w.team = w.wave >> 2;                                // row team
    w.pr = w.wave & 3;                                   // token quarter
    const int lane = w.lane, team = w.team, pr = w.pr;

    const int ntile = (w.c1 - w.c0 + kTile - 1) / kTile;
    w.ntq = (ntile + kWaves - 1) / kWaves;                                      // tiles per quarter (uniform)
    w.last_tok = min(w.c1, w.c0 + (pr + 1) * w.ntq * kTile) - 1;
    auto tile_t0 = [&](int it) { return w.c0 + (pr * w.ntq + it) * kTile; };
    w.addr = make_row_addr<PAGED>(a, w.b, w.hkv);
    w.kring = smem + pr * G::WAVE_LDS;
    w.vring = w.kring + 2 * G::SLOT;
    w.kring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + pr * G::WAVE_LDS;
    w.vring_lds = w.kring_lds + 2 * G::SLOT;

    // Q block: RP rows, HBM -> LDS once per workgroup, the eight waves sharing the loads; issued
    // before the first tiles so that it is complete when only tile loads are outstanding.
    w.qlds = smem + kWaves * G::WAVE_LDS;
    {
        const uint32_t q_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + kWaves * G::WAVE_LDS;
        constexpr int QI = RP / G::RPI;
        const int last_row = a.Qmax * a.G - 1;
        for (int e = w.wave; e < QI; e += 2 * kWaves) {
            const int row = e * G::RPI + lane / G::CPR;
            const int rr = min(row, last_row);
            const int qi = rr / a.G, qg = rr % a.G;
            const int c = (lane % G::CPR) ^ k_swz<D>(row);
            const uint32_t off = (uint32_t)(((((int64_t)w.b * a.Qmax + qi) * a.Hq + w.hkv * a.G + qg) * D) * 2) + c * 16;
            dma16_keep(reinterpret_cast<const char*>(a.q), off, q_lds + e * 1024);
        }
    }
    // Pipeline start: K(0), V(0), K(1) (V(1) follows barrier A of the first iteration).  Every wave runs
    // all ntq iterations, also over tiles past the end of the split (their loads are clamped, their
    // keys masked), so that all eight waves meet at every barrier.
    dma_half_tile<D, PAGED, false>(w.addr, w.kring_lds, tile_t0(0), w.last_tok, lane, team);
    dma_half_tile<D, PAGED, true>(w.addr, w.vring_lds, tile_t0(0), w.last_tok, lane, team);
    dma_half_tile<D, PAGED, false>(w.addr, w.kring_lds + G::SLOT, tile_t0(1), w.last_tok, lane, team);
    wait_loads<3 * (G::NLD / 2)>();                      // everything older than the three half tiles: Q
    __syncthreads();

    constexpr int OROW = D + 4;
    float* mlbuf = reinterpret_cast<float*>(smem) + 2 * RP * OROW;              // [8 waves][MLS][2]
    const int64_t pbase = (((int64_t)w.b * a.Hkv + w.hkv) * a.nsplit + w.split) * RP;
    if (RB0 == RB1 || team == 0)
        wide_team<D, RB0, MLS, PAGED>(a, w, smem, team * RPT0, reinterpret_cast<float*>(smem) + team * 2 * RPT0 * OROW,
                                      mlbuf, pbase);
    else
        wide_team<D, RB1, MLS, PAGED>(a, w, smem, RPT0, reinterpret_cast<float*>(smem) + 2 * RPT0 * OROW, mlbuf, pbase);

    // ---- the split's partial: per row the sum of the team's two halves
    floatx4* po = reinterpret_cast<floatx4*>(a.part_o + pbase * D);
    const float* oall = reinterpret_cast<const float*>(smem);
    for (int f = tid; f < w.R * (D / 4); f += 2 * kWaves * 64) {
        const int row = f / (D / 4), d4 = f % (D / 4);
        const bool t1 = row >= RPT0;
        const int lr = t1 ? row - RPT0 : row, rpt = t1 ? RPT1 : RPT0;
        const float* ob = oall + (t1 ? 2 * RPT0 * OROW : 0);
        const floatx4 x = *reinterpret_cast<const floatx4*>(ob + lr * OROW + d4 * 4);
        const floatx4 y = *reinterpret_cast<const floatx4*>(ob + (rpt + lr) * OROW + d4 * 4);
        po[f] = x + y;
    }
}

// Merge the splits of one query row: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// One workgroup of D threads per (sequence, kv head, packed row), splits taken 32 at a
// time.  The kernel is latency bound, so every thread issues the loads of its column
// for a whole block of splits before anything else, next to the (m, l) loads; the
// weights are formed while they are in flight.
template <int D>
__global__ void __launch_bounds__(D) verify_attn_merge(AttnLaunch a)
{
    constexpr int SB = 32;                             // splits per block
    __shared__ float wgt[SB];
    __shared__ float red[2][4];
    const int row = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
    const int d = threadIdx.x;
    const int Q = seq_queries(a, b);
    const int R = Q * a.G, RP = a.RB * 16;
    const int qi = row / a.G, qg = row % a.G;
    const int h = hkv * a.G + qg;
    uint16_t* dst = a.out + (((int64_t)b * a.Qmax + qi) * a.Hq + h) * D + d;
    if (row >= R) {                                   // query rows this sequence does not have
        *dst = 0;
        if (a.lse_out && d == 0) a.lse_out[((int64_t)b * a.Hq + h) * a.Qmax + qi] = 0.f;
        return;
    }
    const int64_t pbase = ((int64_t)b * a.Hkv + hkv) * a.nsplit * RP;
    float M = -INFINITY, den = 0.f, num = 0.f;
    int ns = a.nsplit;                                 // refined below, once the length has arrived
    for (int s0 = 0; s0 < ns; s0 += SB) {
        // The loads of a block do not wait for the sequence length: every split slot of the
        // workspace is addressable, and the slots of splits that hold no token (stale or
        // never written) are discarded after the fact.  The length is one more dependent
        // memory round trip that this way overlaps with the loads.
        const int nsb = min(SB, a.nsplit - s0);
        const float* po = a.part_o + (pbase + (int64_t)s0 * RP + row) * D + d;
        float o[SB];
#pragma unroll
        for (int j = 0; j < SB; ++j) o[j] = j < nsb ? po[(int64_t)j * RP * D] : 0.f;
        float ms = -INFINITY, ls = 0.f;
        if (d < nsb) {
            const float* ml = a.part_ml + (pbase + (int64_t)(s0 + d) * RP + row) * 2;
            ms = ml[0];
            ls = ml[1];
        }
        if (s0 == 0) {
            const int L = min(a.ctx_lens[b], a.max_ctx);
            ns = min(L / a.chunk + 2, a.nsplit);      // splits that hold a token of this sequence
            while (ns > 0 && split_begin(a, ns - 1, hkv) >= L) --ns;
        }
        const int nb = min(SB, ns - s0);
#pragma unroll
        for (int j = 0; j < SB; ++j) o[j] = j < nb ? o[j] : 0.f;
        if (d >= nb) { ms = -INFINITY; ls = 0.f; }
        float mb = ms;                                 // D >= 64 > SB: the first wave holds them all
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) mb = fmaxf(mb, __shfl_xor(mb, off));
        if (d == 0) red[0][0] = mb;
        __syncthreads();
        mb = red[0][0];
        const float Mn = fmaxf(M, mb);
        const float Mu = (Mn == -INFINITY) ? 0.f : Mn;
        const float resc = fast_exp2(M - Mu);
        M = Mn;
        float w = fast_exp2(ms - Mu), dl = w * ls;     // threads >= nb: w = 0
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) dl += __shfl_xor(dl, off);
        if (d < SB) wgt[d] = w;
        if (d == 0) red[1][0] = dl;
        __syncthreads();
        den = den * resc + red[1][0];
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int j = 0; j < SB; j += 2) {
            acc0 = fmaf(wgt[j], o[j], acc0);
            acc1 = fmaf(wgt[j + 1], o[j + 1], acc1);
        }
        num = num * resc + (acc0 + acc1);
        __syncthreads();                               // wgt/red are rewritten by the next block
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
    auto fn = verify_attn_split<D, RB, PAGED>;
    dim3 grid(a.Hkv, a.nsplit, a.B), block(kWaves * 64);
    hipLaunchKernelGGL(fn, grid, block, lds, stream, a);
    return hipGetLastError();
}

template <int D, int RB0, int RB1, bool PAGED>
hipError_t launch_split_wide(const AttnLaunch& a, hipStream_t stream)
{
    constexpr int lds = attn_wide_lds_bytes<D, RB0, RB1>();
    auto fn = verify_attn_split_wide<D, RB0, RB1, PAGED>;
    dim3 grid(a.Hkv, a.nsplit, a.B), block(2 * kWaves * 64);
    hipLaunchKernelGGL(fn, grid, block, lds, stream, a);
    return hipGetLastError();
}
template <int D, int RB0, int RB1, bool PAGED>
hipError_t configure_split_wide()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(verify_attn_split_wide<D, RB0, RB1, PAGED>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, attn_wide_lds_bytes<D, RB0, RB1>());
}

// The split kernels use more dynamic LDS than the default limit allows; raise it once
// per device, ahead of any launch (and so outside any stream capture).
template <int D, int RB, bool PAGED>
hipError_t configure_split()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(verify_attn_split<D, RB, PAGED>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, attn_lds_bytes<D, RB>());
}
template <int D, bool PAGED>
hipError_t configure_rb()
{
    hipError_t e;
    if ((e = configure_split<D, 1, PAGED>()) != hipSuccess) return e;
    if ((e = configure_split<D, 2, PAGED>()) != hipSuccess) return e;
    if ((e = configure_split<D, 3, PAGED>()) != hipSuccess) return e;
    if ((e = configure_split<D, 4, PAGED>()) != hipSuccess) return e;
    if ((e = configure_split<D, 5, PAGED>()) != hipSuccess) return e;
    if ((e = configure_split_wide<D, 2, 2, PAGED>()) != hipSuccess) return e;
    if ((e = configure_split_wide<D, 3, 2, PAGED>()) != hipSuccess) return e;
    return configure_split_wide<D, 3, 3, PAGED>();
}

template <int D, bool PAGED>
hipError_t dispatch_rb(const AttnLaunch& a, hipStream_t stream)
{
    if (a.wide) {                                    // a.RB row blocks over two teams
        if (a.RB == 4) return launch_split_wide<D, 2, 2, PAGED>(a, stream);
        if (a.RB == 5) return launch_split_wide<D, 3, 2, PAGED>(a, stream);
        if (a.RB == 6) return launch_split_wide<D, 3, 3, PAGED>(a, stream);
        return hipErrorInvalidValue;
    }
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

hipError_t configure_verify_attn()
{
    hipError_t e;
    if ((e = configure_rb<128, false>()) != hipSuccess) return e;
    if ((e = configure_rb<128, true>()) != hipSuccess) return e;
    if ((e = configure_rb<64, false>()) != hipSuccess) return e;
    return configure_rb<64, true>();
}

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
    dim3 grid(a.Qmax * a.G, a.Hkv, a.B);
    if (a.D == 128) hipLaunchKernelGGL(verify_attn_merge<128>, grid, dim3(128), 0, stream, a);
    else hipLaunchKernelGGL(verify_attn_merge<64>, grid, dim3(64), 0, stream, a);
    return hipGetLastError();
}
