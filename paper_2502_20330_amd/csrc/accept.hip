// Acceptance pass of RAPID's validation loop (Alg. 1) for gfx950 (MI355X).
//
// Per sequence b and drafted position k the paper defines
//   p = softmax(z/T), q = softmax(z_q/T)                       (Alg. 1)
//   p_hat = softmax(z/T + eta (q - p))                         (Eq. new_target)
//   p_hat(v) <- p(v) where p_hat(v) < alpha * max p_hat        (tail rule, Sec. 2.4)
//   accept x' iff r <= min(1, p_hat(x')/q(x'))                 (Alg. 1)
//   first reject: x ~ norm(max(p - p_hat, p - q, 0)); none: x ~ p of the next row.
//
// The accept test of a position needs p, q, p_hat only at the one drafted token, given three
// log-normalisers per row; only the row where the draw happens needs an elementwise pass.
// Two launches:
//
//   accept_rows   reads every logit ONCE.  A row pair (target row k, draft row k) is cut into
//       slices of 2048*NV entries; one workgroup of 512 threads holds its slice of both rows in
//       registers.  It publishes the slice's (max, sum exp) of either row, picks up the
//       publications of the other workgroups of the row pair, and with the row normalisers
//       forms d = z/T + eta (q - p) for its slice (still in registers) and publishes
//       (max d, sum exp(d - max)).  The workgroup of slice 0 then collects all slices of its row,
//       combines them in fp64 and runs the accept test of the drafted token.
//
//   accept_draw_row   n = first rejected position; the draw weights of row n (the residual,
//       or p of the bonus row) are formed entirely in fp64 -- exponentials, normalisers,
//       running sums -- because their prefix sums decide an integer; three small exchanges
//       between the workgroups of the row (normalisers of p and q; normaliser and maximum
//       of p_hat; weight totals), then the workgroup whose range holds u*W finds the token.
//
// Exchange between workgroups.  A publication is a group of 64-bit words, each written with a
// device-scope atomic store: 32 bits of payload below a 32-bit tag.  The two tags (even and odd
// words) belong to the call: they are derived from a counter in the workspace that the other
// kernel of the pass advances, so it is constant while a kernel runs and differs from every
// earlier execution's, also when a captured graph replays the launches.  A reader polls the
// words with device-scope atomic loads until every tag is the call's.  An earlier call's
// publications never carry them; whatever else a workspace holds when it is first used is taken
// for a publication only if both tags of a pair match, 2^-64 for unrelated bits.  Nothing has to
// be cleared before the pass, hence no third launch; in return the caller must leave the
// workspace alone between calls (or zero all of it).  Every wait is
// bounded (wall-clock ticks): when a word stays unpublished, the waiting workgroup computes that
// slice's publication itself from the logits in memory -- same code, same order of operations,
// hence the same bits -- stores it, and goes on.  No workgroup ever depends on another one for
// termination, and results do not depend on timing.
//
// Numerics: per-slice sums in fp32, combined in fp32 for the elementwise pass of accept_rows
// and in fp64 for every decision; the accept ratio therefore carries ~1e-7 relative error
// (decisions within 1e-5 of the uniform are near-ties by the definition of the benchmark).
// The draw is fp64 throughout and differs from a sequential fp64 evaluation by summation
// order only.  Statistics are kept relative to the raw row maximum so that dividing by T
// costs no absolute precision.
#include "rapid_internal.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

// Per-phase timestamps for development builds (-DRAPID_ACCEPT_STAMPS); absent from normal builds.
#ifdef RAPID_ACCEPT_STAMPS
__device__ unsigned long long g_dbg[8192 * 16];
#define STAMP(i) do { if (threadIdx.x == 0) { int _l = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z); \
    if (_l < 8192) g_dbg[_l * 16 + (i)] = wall_clock64(); } } while (0)
#define STAMP_AT(l, i) do { if (threadIdx.x == 0 && (l) < 8192) g_dbg[(l) * 16 + (i)] = wall_clock64(); } while (0)
extern "C" int rapid_debug_read(void* dst) { return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_dbg), sizeof(g_dbg)); }
#else
#define STAMP(i) do { } while (0)
#define STAMP_AT(l, i) do { } while (0)
#endif

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kDrawSlice = kThreads * 8;            // smallest slice of accept_draw_row (8 entries per thread)
constexpr int kMinSlice = kThreads * 4 * 2;         // smallest slice of accept_rows (NV = 2)
constexpr float kLog2e = 1.4426950408889634f;
constexpr double kLn2 = 0.6931471805599453;

__device__ __forceinline__ float fexp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Wave-wide inclusive scan through the DPP lane-permute path (no LDS traffic): shifts by 1, 2, 4, 8
// inside each row of 16 lanes, then the row broadcasts of this architecture (lane 15 of a row into
// the next row, lane 31 into the upper half).  Lanes whose source does not exist read `id`.  Lane 63
// ends up with the reduction over the wave; the order of the operations is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float id, float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(id), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_move(double id, double v)
{
    const long long i = __double_as_longlong(id), x = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp((int)i, (int)x, CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp((int)(i >> 32), (int)(x >> 32), CTRL, ROW_MASK, 0xf, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
template <class T, class Op>
__device__ __forceinline__ T wave_scan(T v, Op op)
{
    const T id = Op::id();
    v = op(v, dpp_move<0x111, 0xf>(id, v));      // row_shr:1
    v = op(v, dpp_move<0x112, 0xf>(id, v));      // row_shr:2
    v = op(v, dpp_move<0x114, 0xf>(id, v));      // row_shr:4
    v = op(v, dpp_move<0x118, 0xf>(id, v));      // row_shr:8
    v = op(v, dpp_move<0x142, 0xa>(id, v));      // row_bcast:15 into rows 1 and 3
    v = op(v, dpp_move<0x143, 0xc>(id, v));      // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ double lane_value(double v, int lane)
{
    const long long x = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)x, lane), hi = __builtin_amdgcn_readlane((int)(x >> 32), lane);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
struct OpMaxF { __device__ float operator()(float x, float y) const { return fmaxf(x, y); } static __device__ float id() { return -INFINITY; } };
struct OpAddF { __device__ float operator()(float x, float y) const { return x + y; } static __device__ float id() { return 0.f; } };
struct OpMaxD { __device__ double operator()(double x, double y) const { return fmax(x, y); } static __device__ double id() { return -INFINITY; } };
struct OpAddD { __device__ double operator()(double x, double y) const { return x + y; } static __device__ double id() { return 0.0; } };
template <class T, class Op>
__device__ __forceinline__ T wave_reduce(T v, Op op) { return lane_value(wave_scan(v, op), 63); }
__device__ __forceinline__ float wave_max(float v) { return wave_reduce(v, OpMaxF()); }
__device__ __forceinline__ float wave_sum(float v) { return wave_reduce(v, OpAddF()); }
__device__ __forceinline__ double wave_max(double v) { return wave_reduce(v, OpMaxD()); }
__device__ __forceinline__ double wave_sum(double v) { return wave_reduce(v, OpAddD()); }

// Block-wide reductions over kThreads threads of two values at once; results go to every thread.
// `sh` holds two banks of 2*kWaves slots used alternately (`bank` flips on every call), so one
// barrier per reduction is enough: a wave can only be two reductions ahead of another one after
// that one has passed the barrier in between, i.e. after it has finished reading the bank.
// Fixed order: the wave scan above, then waves 0..7.
template <class T, class OpA, class OpB>
__device__ __forceinline__ void block_reduce2(T& a, T& b, T* sh, int& bank, OpA opa, OpB opb)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    a = wave_scan(a, opa);
    b = wave_scan(b, opb);
    T* s = sh + bank * 2 * kWaves;
    bank ^= 1;
    if (lane == 63) { s[wave] = a; s[kWaves + wave] = b; }
    __syncthreads();
    a = s[0];
    b = s[kWaves];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) { a = opa(a, s[w]); b = opb(b, s[kWaves + w]); }
}

// Four consecutive logits of a row starting at index i (i % 4 == 0); entries at or past V
// come back as -inf.  `vec` says the row base is 16-byte aligned (V a multiple of 4 keeps all
// rows aligned; otherwise the loads are scalar, which is slower but reads the same values).
__device__ __attribute__((noinline)) floatx4 load4_edge(const float* row, int64_t i, int V)
{
    floatx4 r = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    for (int j = 0; j < 4; ++j)
        if (i + j < V) r[j] = row[i + j];
    return r;
}
__device__ __forceinline__ floatx4 load4(const float* row, int64_t i, int V, bool vec)
{
    if (__builtin_expect(vec && i + 3 < V, 1)) return *reinterpret_cast<const floatx4*>(row + i);
    return load4_edge(row, i, V);
}

// Drafts of sequence b; device data, so clamped to the range the buffers were sized for.
__device__ __forceinline__ int seq_gamma(const AcceptLaunch& a, int b)
{
    return a.gammas ? min(max(a.gammas[b], 0), a.gmax) : a.gmax;
}

// ---------------------------------------------------------------- workspace
struct Ws {
    int32_t* status;  // [64]: [0] positions rejected because the draft id was outside [0, V)
                      //       [1] exchange waits that gave up and recomputed the missing slice
                      //       [kCntRows] / [kCntDraw] call counters read by accept_rows / accept_draw_row
                      //       [kGiveRows], [kGiveRows + 1] give-ups of accept_rows: count, tag of the call
    u64* slot_t;      // [B][gmax+1][wmax][2]  (raw max, sum exp((z-max)/T)) per slice of a target row
    u64* slot_d;      // [B][gmax][wmax][2]
    u64* slot_h;      // [B][gmax][wmax][2]    (max d, sum exp2(d - max)), d in log2 units relative to zmax_t/T
    u64* slot_b;      // [B][3][w2][4]         two fp64 values per slice and phase of accept_draw_row
    double* rows;     // [B][gmax+1][4]: zmax_t, zmax_d (raw maxima, exact)
    int32_t* flags;   // [B][gmax]: 1 = draft k passed its accept test, 2 = its id was outside [0, V)
    int wmax;         // slots per row (slices of the smallest slice size)
    int w2;           // workgroups per sequence in accept_draw_row
    size_t bytes;
};
constexpr int kCntRows = 8, kCntDraw = 9, kGiveRows = 10;

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

__host__ __device__ inline Ws carve(void* base, int B, int gmax, int V)
{
    Ws w;
    const int gd = gmax > 0 ? gmax : 1;
    w.wmax = (V + kMinSlice - 1) / kMinSlice;
    w.w2 = (V + kDrawSlice - 1) / kDrawSlice;
    char* p = static_cast<char*>(base);
    w.status = reinterpret_cast<int32_t*>(p); p += 256;
    w.slot_t = reinterpret_cast<u64*>(p); p += align256((size_t)B * (gmax + 1) * w.wmax * 2 * sizeof(u64));
    w.slot_d = reinterpret_cast<u64*>(p); p += align256((size_t)B * gd * w.wmax * 2 * sizeof(u64));
    w.slot_h = reinterpret_cast<u64*>(p); p += align256((size_t)B * gd * w.wmax * 2 * sizeof(u64));
    w.slot_b = reinterpret_cast<u64*>(p); p += align256((size_t)B * w.w2 * 12 * sizeof(u64));
    w.rows = reinterpret_cast<double*>(p); p += align256((size_t)B * (gmax + 1) * 4 * sizeof(double));
    w.flags = reinterpret_cast<int32_t*>(p); p += align256((size_t)B * gd * sizeof(int32_t));
    w.bytes = (size_t)(p - static_cast<char*>(base));
    return w;
}

// ---------------------------------------------------------------- exchange primitives
__device__ __forceinline__ u64 slot_load(const u64* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void slot_store(u64* p, u64 v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The call's tags: words at even offsets of a slot array carry t0, words at odd offsets t1.  Each is
// one-to-one (odd multiplier) in the call counter kept in the workspace, which moves by one with every
// execution of the pass, replays of a captured graph included: no two executions within 2^32 on one
// workspace share either tag.  A zero-filled workspace (counter 0, tags 0 in every slot) is safe too:
// neither tag of counter 0 is zero.
struct Tags { uint32_t t0, t1; };
__device__ __forceinline__ Tags make_tags(uint32_t counter)
{
    return Tags{counter * 0x9E3779B1u + 0x7F4A7C15u, (counter * 0x85EBCA77u) ^ 0xC2B2AE3Du};
}
// the tag of word i (by its parity), without indexing into the pair
__device__ __forceinline__ uint32_t tag_of(int i, const Tags& t) { return t.t0 ^ ((t.t0 ^ t.t1) & (0u - (uint32_t)(i & 1))); }
__device__ __forceinline__ bool word_ok(u64 v, int i, const Tags& t) { return (uint32_t)(v >> 32) == tag_of(i, t); }
__device__ __forceinline__ u64 tagged(uint32_t payload, uint32_t tag) { return (u64)payload | ((u64)tag << 32); }
__device__ __forceinline__ float lo_f(u64 v) { return __uint_as_float((uint32_t)v); }
// Two floats = one slot of two words; p must be an even offset into its array.
__device__ __forceinline__ void publish2f(u64* p, float a, float b, const Tags& t)
{
    slot_store(p, tagged(__float_as_uint(a), t.t0));
    slot_store(p + 1, tagged(__float_as_uint(b), t.t1));
}
// One double = two words (high half first).
__device__ __forceinline__ void put_d(u64* p, double d, const Tags& t, bool global)
{
    const u64 x = (u64)__double_as_longlong(d);
    const u64 hi = tagged((uint32_t)(x >> 32), t.t0), lo = tagged((uint32_t)x, t.t1);
    if (global) { slot_store(p, hi); slot_store(p + 1, lo); }
    else { p[0] = hi; p[1] = lo; }
}
__device__ __forceinline__ double get_d(const u64* p)
{
    return __longlong_as_double((long long)(((p[0] & 0xffffffffull) << 32) | (p[1] & 0xffffffffull)));
}
// Rarely taken: count a give-up of accept_rows in a (count, tag) pair that needs no clearing.
__device__ __forceinline__ void count_giveup(int32_t* status, const Tags& t)
{
    u64* p = reinterpret_cast<u64*>(status + kGiveRows);
    u64 old = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {
        const u64 nw = (uint32_t)(old >> 32) == t.t0 ? old + 1 : tagged(1u, t.t0);
        if (__hip_atomic_compare_exchange_strong(p, &old, nw, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
    }
}

// Compact fp64 exponential (about twenty instructions, inlined where used): exp(x) with ~2e-16
// relative error for x <= 700; anything below -745 (also -inf and NaN) gives 0.  The decisions
// need fp64 but each workgroup runs its code exactly once, so instruction count matters more
// here than in a loop: the library routine is several times longer.
__device__ __forceinline__ double exp_c(double x)
{
    x = fmax(x, -746.0);
    const double k = rint(x * 1.4426950408889634);
    double r = fma(k, -6.93147180369123816490e-01, x);        // k ln2 in two parts
    r = fma(k, -1.90821492927058770002e-10, r);
    double p = 1.0 / 6227020800.0;                           // Taylor to r^13 / 13!, |r| <= 0.347
    p = fma(p, r, 1.0 / 479001600.0);
    p = fma(p, r, 1.0 / 39916800.0);
    p = fma(p, r, 1.0 / 3628800.0);
    p = fma(p, r, 1.0 / 362880.0);
    p = fma(p, r, 1.0 / 40320.0);
    p = fma(p, r, 1.0 / 5040.0);
    p = fma(p, r, 1.0 / 720.0);
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)k);
}
// Wave 0: poll the words addr(lo) .. addr(hi - 1) into dst[lo .. hi) until every one carries its
// tag or `wait_ticks` have passed; *nmiss = words still unpublished (dst then holds what was there).
// lo and hi are even and addr(i) has the parity of i.  Two words per lane and round.
template <class Addr>
__device__ __forceinline__ void poll_into(Addr addr, int lo, int hi, u64* dst, int* nmiss, int64_t wait_ticks, const Tags& tg)
{
    const int lane = threadIdx.x;
    const int64_t t0 = (int64_t)wall_clock64();
    const uint32_t want = tag_of(lane, tg);               // every word of this lane has the lane's parity
    int miss = 0;
    for (int i0 = lo; i0 < hi; i0 += 128) {
        const int ia = i0 + lane, ib = ia + 64;
        u64 va = 0, vb = 0;
        bool pa = ia < hi, pb = ib < hi;
        for (;;) {
            if (pa) {
                va = slot_load(addr(ia));
                pa = (uint32_t)(va >> 32) != want;
            }
            if (pb) {
                vb = slot_load(addr(ib));
                pb = (uint32_t)(vb >> 32) != want;
            }
            if (!__any(pa || pb)) break;
            if ((int64_t)wall_clock64() - t0 >= wait_ticks) break;
            __builtin_amdgcn_s_sleep(2);
        }
        if (ia < hi) dst[ia] = va;
        if (ib < hi) dst[ib] = vb;
        miss += __popcll(__ballot(pa)) + __popcll(__ballot(pb));
    }
    if (lane == 0) *nmiss = miss;
}

// ---------------------------------------------------------------- accept_rows: per-slice arithmetic
// The statistics of a slice are written once, as templates over the way a thread gets at its
// NV float4 of a row: from registers (the workgroup's own slice) or from memory (a slice whose
// publication did not arrive in time).  Same operations in the same order either way; this file
// is compiled without implicit multiply-add contraction so that the two instantiations round alike.
// UNROLL: the register path unrolls (its arrays need constant indices); the memory path keeps its
// loops rolled, it is code that normally never runs and should stay small.
template <int NV, bool UNROLL, class GetT, class GetD>
__device__ __forceinline__ void slice_stats(GetT gt, GetD gd, bool do_t, bool do_d, float c, float* sh, int& bank,
                                            float& mt, float& st, float& md, float& sd)
{
    mt = -INFINITY;
    md = -INFINITY;
    if (do_t)
#pragma unroll UNROLL ? NV : 1
        for (int v = 0; v < NV; ++v) {
            const floatx4 x = gt(v);
            mt = fmaxf(mt, fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])));
        }
    if (do_d)
#pragma unroll UNROLL ? NV : 1
        for (int v = 0; v < NV; ++v) {
            const floatx4 y = gd(v);
            md = fmaxf(md, fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])));
        }
    block_reduce2(mt, md, sh, bank, OpMaxF(), OpMaxF());
    st = 0.f;
    sd = 0.f;
    if (do_t && mt > -INFINITY)
#pragma unroll UNROLL ? NV : 1
        for (int v = 0; v < NV; ++v) {
            const floatx4 x = gt(v);
#pragma unroll
            for (int j = 0; j < 4; ++j) st += fexp2((x[j] - mt) * c);
        }
    if (do_d && md > -INFINITY)
#pragma unroll UNROLL ? NV : 1
        for (int v = 0; v < NV; ++v) {
            const floatx4 y = gd(v);
#pragma unroll
            for (int j = 0; j < 4; ++j) sd += fexp2((y[j] - md) * c);
        }
    block_reduce2(st, sd, sh, bank, OpAddF(), OpAddF());
}

// Row normalisers in the form the elementwise pass uses (log2 units).
struct PairNorm { float Mt, l2St, Md, l2Sd; };

// d = z/T + eta (q - p) of one entry, in log2 units relative to zmax_t/T.  Entries past V were
// loaded as -inf: p = q = 0 and d = -inf.
__device__ __forceinline__ float shifted(float zt, float zd, const PairNorm& r, float c, float eta_l2)
{
    const float at = (zt - r.Mt) * c;
    const float p = fexp2(at - r.l2St);
    const float q = fexp2((zd - r.Md) * c - r.l2Sd);
    return fmaf(eta_l2, q - p, at);
}

// (max d, sum exp2(d - max)) of a slice; d_first(v) yields d of the thread's v-th float4 (the register
// path also stores it), d_again(v) yields it again (from the registers, or recomputed: same value).
template <int NV, bool UNROLL, class GetFirst, class GetAgain>
__device__ __forceinline__ void shifted_stats(GetFirst d_first, GetAgain d_again, float* sh, int& bank, float& mh,
                                              float& shs)
{
    mh = -INFINITY;
    float unused = -INFINITY;
#pragma unroll UNROLL ? NV : 1
    for (int v = 0; v < NV; ++v) {
        const floatx4 d = d_first(v);
        mh = fmaxf(mh, fmaxf(fmaxf(d[0], d[1]), fmaxf(d[2], d[3])));
    }
    block_reduce2(mh, unused, sh, bank, OpMaxF(), OpMaxF());
    shs = 0.f;
    unused = 0.f;
    if (mh > -INFINITY)
#pragma unroll UNROLL ? NV : 1
        for (int v = 0; v < NV; ++v) {
            const floatx4 d = d_again(v);
#pragma unroll
            for (int j = 0; j < 4; ++j) shs += fexp2(d[j] - mh);
        }
    block_reduce2(shs, unused, sh, bank, OpAddF(), OpAddF());
}

// Wave 0: combine n (max, sum) pairs, maxima raw logits, sums of exp((z - max)/T):
// M = max, S = sum_i s_i 2^((m_i - M) c); fp32, fixed order.  Result valid in every lane of wave 0.
template <class Pair>
__device__ __forceinline__ void wave_combine_f32(Pair pair, int n, float c, float& M, float& l2S)
{
    const int lane = threadIdx.x & 63;
    float m = -INFINITY;
    for (int i = lane; i < n; i += 64) m = fmaxf(m, pair(i).x);
    M = wave_max(m);
    float s = 0.f;
    for (int i = lane; i < n; i += 64) {
        const float2 v = pair(i);
        if (v.y > 0.f) s += v.y * fexp2((v.x - M) * c);
    }
    l2S = __log2f(wave_sum(s));
}
// The same in fp64 (decisions); `scale` multiplies the difference of maxima (1/T for raw logits,
// ln 2 for maxima kept in log2 units).
template <class Pair>
__device__ __forceinline__ void wave_combine_f64(Pair pair, int n, double scale, double& M, double& S)
{
    const int lane = threadIdx.x & 63;
    double m = -INFINITY;
    for (int i = lane; i < n; i += 64) m = fmax(m, (double)pair(i).x);
    M = wave_max(m);
    double s = 0.0;
    for (int i = lane; i < n; i += 64) {
        const float2 v = pair(i);
        if (v.y > 0.f) s += (double)v.y * exp_c(((double)v.x - M) * scale);
    }
    S = wave_sum(s);
}

struct LdsA {
    double dec[4];        // Mt, St, Md, Sd of the row in fp64 (deciding workgroup)
    float red[4 * kWaves];
    PairNorm norm;
    int nmiss;
    u64 slots[];          // 6 W words: two per slice of the target row, the draft row, the shifted row
};

// ---------------------------------------------------------------- accept_rows
// One workgroup per work item (sequence b, row k, slice w), slice index fastest in dispatch order, so
// the slices of one row pair are worked on by different workgroups at about the same time.
template <int NV>
__global__ void __launch_bounds__(kThreads, 4) accept_rows(AcceptLaunch a, Ws ws, int W, int n_items)
{
    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    LdsA& lds = *reinterpret_cast<LdsA*>(smem_raw);
    constexpr int kSlice = kThreads * 4 * NV;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int V = a.V, rows = a.gmax + 1;
    int bank = 0;
    const float c = a.inv_T * kLog2e, eta_l2 = a.eta * kLog2e;

    // Item id -> (w, k, b); g = drafts of its sequence (a device value, read one item ahead).
    auto row_t = [&](int b, int k) { return a.zt + ((int64_t)b * rows + k) * V; };
    auto row_d = [&](int b, int k) { return a.zd + ((int64_t)b * a.gmax + k) * V; };

    // Issue the loads of item `id` into x / y (nothing for rows past the sequence's drafts).
    auto issue = [&](int id, int g, floatx4 (&x)[NV], floatx4 (&y)[NV]) {
        const int w = id % W, k = (id / W) % rows, b = id / (W * rows);
        if (k > g) return;
        const bool pair = k < g;
        const float* zt = row_t(b, k);
        const float* zd = pair ? row_d(b, k) : nullptr;
        const bool vec_t = (reinterpret_cast<uintptr_t>(zt) & 15) == 0;
        const bool vec_d = (reinterpret_cast<uintptr_t>(zd) & 15) == 0;
        if (vec_t && (!pair || vec_d) && (int64_t)(w + 1) * kSlice <= V) {
            // the whole slice exists and both rows are aligned: plain 128-bit loads (uniform branch)
            const floatx4* pt = reinterpret_cast<const floatx4*>(zt + (int64_t)w * kSlice) + tid;
#pragma unroll
            for (int v = 0; v < NV; ++v) x[v] = pt[v * kThreads];
            if (pair) {
                const floatx4* pd = reinterpret_cast<const floatx4*>(zd + (int64_t)w * kSlice) + tid;
#pragma unroll
                for (int v = 0; v < NV; ++v) y[v] = pd[v * kThreads];
            }
        } else {
#pragma unroll
            for (int v = 0; v < NV; ++v) x[v] = load4(zt, (int64_t)w * kSlice + (v * kThreads + tid) * 4, V, vec_t);
            if (pair) {
#pragma unroll
                for (int v = 0; v < NV; ++v) y[v] = load4(zd, (int64_t)w * kSlice + (v * kThreads + tid) * 4, V, vec_d);
            }
        }
    };

    // Everything after the loads of one item.
    auto process = [&](int id, int g, floatx4 (&x)[NV], floatx4 (&y)[NV], const Tags& tg) {
        const int w = id % W, k = (id / W) % rows, b = id / (W * rows);
        if (k > g) return;
        STAMP_AT(id, 1);
        const bool pair = k < g;                              // row g has a target row only (the bonus position)
        const float* zt = row_t(b, k);
        const float* zd = pair ? row_d(b, k) : nullptr;
        const bool vec_t = (reinterpret_cast<uintptr_t>(zt) & 15) == 0;
        const bool vec_d = (reinterpret_cast<uintptr_t>(zd) & 15) == 0;
        const bool own_t = a.ext_t == nullptr, own_d = pair && a.ext_d == nullptr;
        u64* slot_t = ws.slot_t + ((int64_t)b * rows + k) * ws.wmax * 2;
        u64* slot_d = ws.slot_d + ((int64_t)b * a.gmax + (pair ? k : 0)) * ws.wmax * 2;
        u64* slot_h = ws.slot_h + ((int64_t)b * a.gmax + (pair ? k : 0)) * ws.wmax * 2;
        auto reg_t = [&](int v) { return x[v]; };
        auto reg_d = [&](int v) { return y[v]; };
        // slice s of either row straight from memory (a slice another workgroup owns)
        auto mem_slice = [&](const float* row, bool vec, int s) {
            return [row, vec, s, tid, V](int v) { return load4(row, (int64_t)s * kSlice + (v * kThreads + tid) * 4, V, vec); };
        };

        // ---- statistics of the own slice
        if (own_t || own_d) {
            float mt, st, md, sd;
            slice_stats<NV, true>(reg_t, reg_d, own_t, own_d, c, lds.red, bank, mt, st, md, sd);
            if (tid == 0) {
                if (own_t) publish2f(slot_t + 2 * w, mt, st, tg);
                if (own_d) publish2f(slot_d + 2 * w, md, sd, tg);
            }
        }
        STAMP_AT(id, 2);

        // ---- publications of all slices of the row (pair): lds.slots[0..2W) target, [2W..4W) draft.
        // A slice that stays unpublished past the bound is computed here (and published for the others).
        u64* got = lds.slots;
        const int W2w = 2 * W;
        auto have = [&](const u64* g2, int s) { return word_ok(g2[2 * s], 0, tg) && word_ok(g2[2 * s + 1], 1, tg); };
        auto keep2f = [&](u64* g2, int s, float m, float sum) {
            g2[2 * s] = tagged(__float_as_uint(m), tg.t0);
            g2[2 * s + 1] = tagged(__float_as_uint(sum), tg.t1);
        };
        auto gather = [&](bool need_t, bool need_d) {
            const int lo = need_t ? 0 : W2w, hi = need_d ? 2 * W2w : W2w;
            if (tid < 64) poll_into([&](int i) { return i < W2w ? slot_t + i : slot_d + (i - W2w); }, lo, hi, got, &lds.nmiss,
                                    a.wait_ticks, tg);
            __syncthreads();
            if (__builtin_expect(lds.nmiss != 0, 0)) {
                for (int s = 0; s < W; ++s) {
                    const bool miss_t = need_t && !have(got, s), miss_d = need_d && !have(got + W2w, s);
                    if (!miss_t && !miss_d) continue;
                    float mt, st, md, sd;
                    slice_stats<NV, false>(mem_slice(zt, vec_t, s), mem_slice(zd, vec_d, s), miss_t, miss_d, c, lds.red, bank, mt, st, md, sd);
                    if (tid == 0) {
                        if (miss_t) { keep2f(got, s, mt, st); publish2f(slot_t + 2 * s, mt, st, tg); }
                        if (miss_d) { keep2f(got + W2w, s, md, sd); publish2f(slot_d + 2 * s, md, sd, tg); }
                        count_giveup(ws.status, tg);
                    }
                    __syncthreads();
                }
            }
        };
        // (max, sum) pair i of the target / draft row: a slot, or the caller's statistics
        const float2* ext_t = a.ext_t ? reinterpret_cast<const float2*>(a.ext_t) + ((int64_t)b * rows + k) * a.nch_t : nullptr;
        const float2* ext_d = (pair && a.ext_d) ? reinterpret_cast<const float2*>(a.ext_d) + ((int64_t)b * a.gmax + k) * a.nch_d : nullptr;
        auto pair_t = [&](int i) { return ext_t ? ext_t[i] : make_float2(lo_f(got[2 * i]), lo_f(got[2 * i + 1])); };
        auto pair_d = [&](int i) { return ext_d ? ext_d[i] : make_float2(lo_f(got[W2w + 2 * i]), lo_f(got[W2w + 2 * i + 1])); };
        const int n_t = ext_t ? a.nch_t : W, n_d = ext_d ? a.nch_d : W;

        if (pair) {
            gather(own_t, own_d);
            STAMP_AT(id, 3);
            if (ext_t || ext_d) {
                // The caller's statistics are hundreds of pairs per row in memory: all eight waves fetch them at
                // once (one round trip) and two block reductions combine them (a side without supplied statistics
                // brings its W gathered pairs the same way); every workgroup of the row pair gets the same bits.
                float2 vt[2], vd[2];                          // pairs tid and tid + kThreads; beyond: the loops below
                float mt = -INFINITY, md = -INFINITY;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int i = tid + j * kThreads;
                    vt[j] = i < n_t ? pair_t(i) : make_float2(-INFINITY, 0.f);
                    vd[j] = i < n_d ? pair_d(i) : make_float2(-INFINITY, 0.f);
                    mt = fmaxf(mt, vt[j].x);
                    md = fmaxf(md, vd[j].x);
                }
                for (int i = tid + 2 * kThreads; i < n_t; i += kThreads) mt = fmaxf(mt, pair_t(i).x);
                for (int i = tid + 2 * kThreads; i < n_d; i += kThreads) md = fmaxf(md, pair_d(i).x);
                block_reduce2(mt, md, lds.red, bank, OpMaxF(), OpMaxF());
                float st = 0.f, sd = 0.f;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (vt[j].y > 0.f) st += vt[j].y * fexp2((vt[j].x - mt) * c);
                    if (vd[j].y > 0.f) sd += vd[j].y * fexp2((vd[j].x - md) * c);
                }
                for (int i = tid + 2 * kThreads; i < n_t; i += kThreads) {
                    const float2 v = pair_t(i);
                    if (v.y > 0.f) st += v.y * fexp2((v.x - mt) * c);
                }
                for (int i = tid + 2 * kThreads; i < n_d; i += kThreads) {
                    const float2 v = pair_d(i);
                    if (v.y > 0.f) sd += v.y * fexp2((v.x - md) * c);
                }
                block_reduce2(st, sd, lds.red, bank, OpAddF(), OpAddF());
                if (tid == 0) lds.norm = PairNorm{mt, __log2f(st), md, __log2f(sd)};
            } else if (tid < 64) {
                PairNorm r;
                wave_combine_f32(pair_t, n_t, c, r.Mt, r.l2St);
                wave_combine_f32(pair_d, n_d, c, r.Md, r.l2Sd);
                if (tid == 0) lds.norm = r;
            }
            __syncthreads();
            const PairNorm r = lds.norm;
            // ---- d for the own slice (kept in x), its statistics
            float mh, shs;
            auto d_first = [&](int v) {
#pragma unroll
                for (int j = 0; j < 4; ++j) x[v][j] = shifted(x[v][j], y[v][j], r, c, eta_l2);
                return x[v];
            };
            shifted_stats<NV, true>(d_first, reg_t, lds.red, bank, mh, shs);
            if (tid == 0) publish2f(slot_h + 2 * w, mh, shs, tg);
            STAMP_AT(id, 4);
        }

        // ---- the workgroup of slice 0 decides the row once all slices have reported
        STAMP_AT(id, 5);
        if (w == 0) {
            // Wave 0 first fetches the drafted token's two logits (a dependent chain that overlaps the polls).
            int xtok = -1;
            float zx_t = 0.f, zx_d = 0.f;
            if (pair && tid < 64) {
                xtok = a.tokens[(int64_t)b * a.gmax + k];
                if (xtok >= 0 && xtok < V) { zx_t = zt[xtok]; zx_d = zd[xtok]; }
            }
            u64* got_h = lds.slots + 2 * W2w;
            if (!pair) {
                gather(own_t, false);                         // (a pair's workgroups all gathered above)
            } else {
                // while wave 0 waits for the shifted statistics, waves 1 and 2 combine the row's two
                // normalisers in fp64 (their slices were gathered before the shift)
                if (wave == 1 || wave == 2) {
                    double M, S;
                    if (wave == 1) wave_combine_f64(pair_t, n_t, a.inv_T_exact, M, S);
                    else wave_combine_f64(pair_d, n_d, a.inv_T_exact, M, S);
                    if (lane == 0) { lds.dec[2 * (wave - 1)] = M; lds.dec[2 * (wave - 1) + 1] = S; }
                }
                if (tid < 64) poll_into([&](int i) { return slot_h + i; }, 0, W2w, got_h, &lds.nmiss, a.wait_ticks, tg);
                __syncthreads();
                if (__builtin_expect(lds.nmiss != 0, 0)) {
                    const PairNorm r = lds.norm;
                    for (int s = 0; s < W; ++s) {
                        if (have(got_h, s)) continue;
                        auto gt = mem_slice(zt, vec_t, s);
                        auto gd = mem_slice(zd, vec_d, s);
                        auto d_mem = [&](int v) {
                            floatx4 t4 = gt(v);
                            const floatx4 d4 = gd(v);
#pragma unroll
                            for (int j = 0; j < 4; ++j) t4[j] = shifted(t4[j], d4[j], r, c, eta_l2);
                            return t4;
                        };
                        float mh, shs;
                        shifted_stats<NV, false>(d_mem, d_mem, lds.red, bank, mh, shs);
                        if (tid == 0) { keep2f(got_h, s, mh, shs); publish2f(slot_h + 2 * s, mh, shs, tg); count_giveup(ws.status, tg); }
                        __syncthreads();
                    }
                }
            }
            STAMP_AT(id, 6);
            if (tid < 64) {
                // one wave: fp64 combine of the row's statistics and the accept test of its drafted token
                double Mt, St, Md = 0, Sd = 1, Mh = 0, Sh = 1;
                if (pair) {
                    Mt = lds.dec[0]; St = lds.dec[1]; Md = lds.dec[2]; Sd = lds.dec[3];
                    auto pair_h = [&](int i) { return make_float2(lo_f(got_h[2 * i]), lo_f(got_h[2 * i + 1])); };
                    wave_combine_f64(pair_h, W, kLn2, Mh, Sh);
                } else {
                    wave_combine_f64(pair_t, n_t, a.inv_T_exact, Mt, St);
                }
                if (tid == 0) {
                    double* rec = ws.rows + ((int64_t)b * rows + k) * 4;
                    rec[0] = Mt;                             // raw maxima: exact, reused by the draw
                    rec[1] = Md;
                    if (pair) {
                        double rho = 0.0;
                        bool ok = false;
                        const bool in_range = xtok >= 0 && xtok < V;
                        if (in_range) {
                            // p = e^at / St, q = e^ad / Sd, p_hat = e^(at + eta (q - p) - Mh ln2) / Sh, max p_hat = 1 / Sh
                            const double invT = a.inv_T_exact;
                            const double at = ((double)zx_t - Mt) * invT;
                            const double p = exp_c(at) / St, q = exp_c(((double)zx_d - Md) * invT) / Sd;
                            double ph = exp_c(at + (double)a.eta * (q - p) - Mh * kLn2) / Sh;
                            if (ph < (double)a.tail_alpha / Sh) ph = p;
                            rho = q > 0.0 ? ph / q : INFINITY;
                            const double u = (double)a.uniforms[(int64_t)b * rows + k];
                            ok = u <= fmin(1.0, rho);
                        }
                        if (a.ratio) a.ratio[(int64_t)b * a.gmax + k] = (float)rho;
                        // an id outside the vocabulary is rejected, and counted by accept_draw_row
                        ws.flags[(int64_t)b * a.gmax + k] = in_range ? (ok ? 1 : 0) : 2;
                    }
                }
            }
            STAMP_AT(id, 7);
        }
        __syncthreads();                                      // lds.slots / lds.norm are reused by the next item
    };

    floatx4 x[NV], y[NV];
    const int id = blockIdx.x;
    if (id >= n_items) return;
    const int g = seq_gamma(a, id / (W * rows));
    STAMP_AT(id, 0);
    issue(id, g, x, y);
    // The call's tags (the counter is constant while this kernel runs: accept_draw_row advances it).
    const Tags tg = make_tags((uint32_t)ws.status[kCntRows]);
    if (id == 0 && tid == 0) {
        // This kernel adds to neither status word; accept_draw_row does, after this kernel is done.
        ws.status[0] = 0;
        ws.status[1] = 0;
        ws.status[kCntDraw] += 1;                             // read only by accept_draw_row
    }
    process(id, g, x, y, tg);
}

// Number of accepted drafts: index of the first failed accept test, or g.  Every wave reads the flags of
// all gmax positions, one per lane, without waiting for the sequence's own count g (one dependent memory
// round trip less); positions >= g hold whatever an earlier call left and are cut off by the min.
__device__ __forceinline__ int first_reject(const Ws& ws, int b, int gmax, int g)
{
    const int lane = threadIdx.x & 63;
    int n = 0x7fffffff;
    for (int k0 = 0; k0 < gmax; k0 += 64) {
        const int k = k0 + lane;
        const int f = k < gmax ? ws.flags[(int64_t)b * gmax + k] : 1;
        const unsigned long long rejected = __ballot(f != 1);
        if (rejected && n == 0x7fffffff) n = k0 + __ffsll((long long)rejected) - 1;
    }
    return min(n, g);
}

// ---------------------------------------------------------------- accept_draw_row (fp64)
// Thread t of workgroup w owns the NE consecutive entries  w*512*NE + t*NE + i  (i = 0..NE-1), so
// vocabulary order inside a workgroup is thread order.
//
// Phase 1: e_t = exp((z - zmax)/T), e_d likewise; sums -> p = e_t/S_t, q = e_d/S_d.
// Phase 2: f = e_t exp(eta (q - p)) (p_hat up to its normaliser); sum and max of f -> p_hat = f/S_h
//          and the tail threshold alpha max p_hat.
// Phase 3: the residual weights max(p - p_hat', p - q, 0) and p; their sums per slice.
// The bonus row (all drafts accepted) draws from p: phase 1 only, weights e_t.
struct DrawNorm { double iSt, iSd, iSh, thr, eta; };

struct LdsB {
    double red[4 * kWaves];
    int nmiss;
    u64 slots[];          // 4 W2 words: the two fp64 values of every slice for the current phase
};

// The three quantities of one entry that the phases are made of.
__device__ __forceinline__ double draw_f(double et, double ed, const DrawNorm& nm)
{
    return et * exp_c(nm.eta * (ed * nm.iSd - et * nm.iSt));
}
// f = draw_f(et, ed, nm): the register path kept it from phase 2, the memory path forms it again (same bits).
__device__ __forceinline__ double draw_weight(double et, double ed, double f, const DrawNorm& nm, double& p)
{
    p = et * nm.iSt;
    const double q = ed * nm.iSd;
    double ph = f * nm.iSh;
    if (ph < nm.thr) ph = p;
    return fmax(fmax(p - ph, p - q), 0.0);
}
// Accumulates entry (et, ed) into the two running values of `phase`; the entries of a thread are
// taken in index order both by the register path and by the memory path.
__device__ __forceinline__ void draw_accumulate(int phase, double et, double ed, const DrawNorm& nm, double& a0, double& a1)
{
    if (phase == 1) {
        a0 += et;
        a1 += ed;
    } else if (phase == 2) {
        const double f = draw_f(et, ed, nm);
        a0 += f;
        a1 = fmax(a1, f);
    } else {
        double p;
        a0 += draw_weight(et, ed, draw_f(et, ed, nm), nm, p);
        a1 += p;
    }
}

// OCC = waves per SIMD the kernel is compiled for: 4 (two workgroups per compute unit, 128 registers,
// a few spilled) for grids of several rounds, 2 (256 registers, no spills) when every workgroup has a
// compute unit to itself anyway.
template <int NE, int OCC>
__global__ void __launch_bounds__(kThreads, OCC) accept_draw_row(AcceptLaunch a, Ws ws, int W2)
{
    extern __shared__ __attribute__((aligned(16))) char smem_raw[];
    LdsB& lds = *reinterpret_cast<LdsB*>(smem_raw);
    constexpr int kSlice = kThreads * NE;
    const int w = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    STAMP(8);
    const int g = seq_gamma(a, b);
    const int n = first_reject(ws, b, a.gmax, g);
    const double u = (double)a.uniforms[(int64_t)b * (a.gmax + 1) + a.gmax];
    if (w == 0) {
        // accepted drafts, then -1 (the draw fills slot n)
        for (int k = tid; k <= a.gmax; k += kThreads)
            if (k != n) a.out_tokens[(int64_t)b * (a.gmax + 1) + k] = k < n ? a.tokens[(int64_t)b * a.gmax + k] : -1;
        if (tid == 0) {
            a.n_accepted[b] = n;
            int bad = 0;                                      // drafted ids outside the vocabulary
            for (int k = 0; k < g; ++k) bad += ws.flags[(int64_t)b * a.gmax + k] == 2;
            if (bad) atomicAdd(ws.status + 0, bad);
            if (b == 0) {
                // give-ups of accept_rows (counted under that kernel's tag), then its counter moves on
                const Tags ta = make_tags((uint32_t)ws.status[kCntRows]);
                if ((uint32_t)ws.status[kGiveRows + 1] == ta.t0) atomicAdd(ws.status + 1, ws.status[kGiveRows]);
                ws.status[kCntRows] += 1;
            }
        }
    }
    const Tags tg = make_tags(~(uint32_t)ws.status[kCntDraw]);
    const int V = a.V;
    int bank = 0;
    const bool bonus = n >= g;
    const float* zt = a.zt + ((int64_t)b * (a.gmax + 1) + n) * V;
    const float* zd = bonus ? nullptr : a.zd + ((int64_t)b * a.gmax + n) * V;
    const bool vec_t = (reinterpret_cast<uintptr_t>(zt) & 15) == 0;
    const bool vec_d = (reinterpret_cast<uintptr_t>(zd) & 15) == 0;
    const double* rec = ws.rows + ((int64_t)b * (a.gmax + 1) + n) * 4;
    const double Mt = rec[0], Md = rec[1], invT = a.inv_T_exact;

    // own slice: e_t, e_d of the thread's entries, kept in registers for all phases; wgt holds
    // f = e_t exp(eta (q - p)) after phase 2 and the draw weight after phase 3
    double et[NE], ed[NE], wgt[NE];
    const int64_t first = (int64_t)w * kSlice + (int64_t)tid * NE;
#pragma unroll
    for (int v = 0; v < NE / 4; ++v) {
        const floatx4 t4 = load4(zt, first + v * 4, V, vec_t);
        floatx4 d4 = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (!bonus) d4 = load4(zd, first + v * 4, V, vec_d);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            et[v * 4 + j] = exp_c(((double)t4[j] - Mt) * invT);
            ed[v * 4 + j] = bonus ? 0.0 : exp_c(((double)d4[j] - Md) * invT);
            wgt[v * 4 + j] = 0.0;
        }
    }
    STAMP(9);
    DrawNorm nm{1.0, 0.0, 0.0, 0.0, (double)a.eta};
    u64* my_slots = ws.slot_b + (int64_t)b * ws.w2 * 12;

    // Reduction of word `word` (0 / 1) of the current phase over all slices, in a fixed order (the
    // same in every workgroup): lanes take slices lane, lane + 64, ...; then the wave reduction.
    auto all_sum = [&](int word) {
        double s = 0.0;
        for (int i = lane; i < W2; i += 64) s += get_d(lds.slots + 4 * i + 2 * word);
        return wave_sum(s);
    };
    auto all_max = [&](int word) {
        double s = -INFINITY;
        for (int i = lane; i < W2; i += 64) s = fmax(s, get_d(lds.slots + 4 * i + 2 * word));
        return wave_max(s);
    };

    const int nphase = bonus ? 1 : 3;
    for (int phase = 1; phase <= nphase; ++phase) {
        double a0 = 0.0, a1 = phase == 2 ? -INFINITY : 0.0;
#pragma unroll
        for (int i = 0; i < NE; ++i) {
            if (phase == 2) {                                 // f is kept for phase 3 (no second exponential)
                wgt[i] = draw_f(et[i], ed[i], nm);
                a0 += wgt[i];
                a1 = fmax(a1, wgt[i]);
            } else if (phase == 3) {                          // the weights are kept for the token search
                double p;
                wgt[i] = draw_weight(et[i], ed[i], wgt[i], nm, p);
                a0 += wgt[i];
                a1 += p;
            } else {
                draw_accumulate(phase, et[i], ed[i], nm, a0, a1);
            }
        }
        if (phase == 2) block_reduce2(a0, a1, lds.red, bank, OpAddD(), OpMaxD());
        else block_reduce2(a0, a1, lds.red, bank, OpAddD(), OpAddD());
        u64* base = my_slots + (phase - 1) * 4 * W2;         // slice s: words base[4 s .. 4 s + 3]
        if (tid == 0) { put_d(base + 4 * w, a0, tg, true); put_d(base + 4 * w + 2, a1, tg, true); }
        if (tid < 64) poll_into([&](int i) { return base + i; }, 0, 4 * W2, lds.slots, &lds.nmiss, a.wait_ticks, tg);
        __syncthreads();
        if (__builtin_expect(lds.nmiss != 0, 0)) {
            // a slice whose sums did not arrive: the same sums from the logits in memory
            for (int s = 0; s < W2; ++s) {
                const u64* have = lds.slots + 4 * s;
                if (word_ok(have[0], 0, tg) && word_ok(have[1], 1, tg) && word_ok(have[2], 0, tg) && word_ok(have[3], 1, tg)) continue;
                double m0 = 0.0, m1 = phase == 2 ? -INFINITY : 0.0;
#pragma unroll 1
                for (int i = 0; i < NE; ++i) {
                    const int64_t e = (int64_t)s * kSlice + (int64_t)tid * NE + i;
                    const double met = e < V ? exp_c(((double)zt[e] - Mt) * invT) : 0.0;
                    const double med = (!bonus && e < V) ? exp_c(((double)zd[e] - Md) * invT) : 0.0;
                    draw_accumulate(phase, met, med, nm, m0, m1);
                }
                if (phase == 2) block_reduce2(m0, m1, lds.red, bank, OpAddD(), OpMaxD());
                else block_reduce2(m0, m1, lds.red, bank, OpAddD(), OpAddD());
                if (tid == 0) {
                    put_d(lds.slots + 4 * s, m0, tg, false);
                    put_d(lds.slots + 4 * s + 2, m1, tg, false);
                    put_d(base + 4 * s, m0, tg, true);
                    put_d(base + 4 * s + 2, m1, tg, true);
                    atomicAdd(ws.status + 1, 1);
                }
                __syncthreads();
            }
        }
        STAMP(9 + phase);
        if (phase == 1 && !bonus) {
            nm.iSt = 1.0 / all_sum(0);
            nm.iSd = 1.0 / all_sum(1);
        } else if (phase == 2) {
            nm.iSh = 1.0 / all_sum(0);
            nm.thr = (double)a.tail_alpha * (all_max(1) * nm.iSh);   // alpha * max p_hat
        }
        if (phase < nphase) __syncthreads();                  // lds.slots are rewritten by the next phase
    }

    // ---- which slice holds the crossing.  Inclusive prefix sums over the slices in slice order
    // (chunks of 64 slices, a wave scan per chunk): every workgroup computes the same values.
    // Weights: the residual (word 0) unless it is empty, then p (word 1); bonus row: e_t (word 0).
    int word = 0;
    auto prefix_pass = [&](double t, bool search, int& owner, double& owner_excl) {
        double carry = 0.0;
        owner = -1;
        owner_excl = 0.0;
        for (int i0 = 0; i0 < W2; i0 += 64) {
            const int i = i0 + lane;
            const double v = i < W2 ? get_d(lds.slots + 4 * i + 2 * word) : 0.0;
            const double inc = carry + wave_scan(v, OpAddD());
            if (search && owner < 0) {
                const unsigned long long hit = __ballot(i < W2 && inc > t);
                if (hit) {
                    const int l = __ffsll((long long)hit) - 1;
                    owner = i0 + l;
                    owner_excl = lane_value(inc - v, l);
                }
            }
            carry = lane_value(inc, 63);
        }
        return carry;                                        // the total
    };
    int owner;
    double excl;
    double Wtot = prefix_pass(0.0, false, owner, excl);
    if (!bonus && !(Wtot > 0.0)) {                            // empty residual: draw from p instead
        word = 1;
        Wtot = prefix_pass(0.0, false, owner, excl);
    }
    const double t = u * Wtot;
    prefix_pass(t, true, owner, excl);
    STAMP(13);
    if (owner < 0) {                                          // no weight anywhere (NaN / infinite logits): any valid id
        if (w == 0 && tid == 0) a.out_tokens[(int64_t)b * (a.gmax + 1) + n] = 0;
        return;
    }
    if (owner != w) return;

    // ---- this workgroup's range holds the crossing: running sums in vocabulary order = thread order
    double seg = 0.0;
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        if (bonus) wgt[i] = et[i];
        else if (word == 1) wgt[i] = et[i] * nm.iSt;           // (else: the residual weight from phase 3)
        seg += wgt[i];
    }
    const double incl = wave_scan(seg, OpAddD());
    if (lane == 63) lds.red[wave] = incl;
    __syncthreads();
    double run = excl + (incl - seg);
    for (int s = 0; s < wave; ++s) run += lds.red[s];
    int my_lo = 0x7fffffff, my_hi = -1;
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        const double nxt = run + wgt[i];
        if (wgt[i] > 0.0) {
            my_hi = (int)first + i;
            if (nxt > t) my_lo = min(my_lo, (int)first + i);
        }
        run = nxt;
    }
    // entries are in thread order: the first thread with a hit holds the smallest index, the last
    // thread with weight the largest (ballots instead of atomics on one LDS word)
    const unsigned long long hit = __ballot(my_lo != 0x7fffffff), any = __ballot(my_hi >= 0);
    const int lo_w = hit ? __shfl(my_lo, __ffsll((long long)hit) - 1) : 0x7fffffff;
    const int hi_w = any ? __shfl(my_hi, 63 - __clzll((long long)any)) : -1;
    int* picks = reinterpret_cast<int*>(lds.red + 2 * kWaves);    // [kWaves][2], past the wave totals above
    if (lane == 0) { picks[2 * wave] = lo_w; picks[2 * wave + 1] = hi_w; }
    __syncthreads();
    if (tid == 0) {
        int lo = 0x7fffffff, hi = -1;
        for (int s = 0; s < kWaves; ++s) { lo = min(lo, picks[2 * s]); hi = max(hi, picks[2 * s + 1]); }
        const int tok = lo != 0x7fffffff ? lo : hi;           // hi: rounding at the slice's end
        a.out_tokens[(int64_t)b * (a.gmax + 1) + n] = tok;
    }
    STAMP(14);
}

}  // namespace

size_t accept_workspace_bytes(int B, int gmax, int V)
{
    return carve(nullptr, B, gmax, V).bytes;
}

hipError_t launch_accept(const AcceptLaunch& a, hipStream_t stream)
{
    Ws ws = carve(a.workspace, a.B, a.gmax, a.V);
    // Slice size of accept_rows: the largest of 16384 / 8192 / 4096 entries that still gives two
    // workgroups per compute unit; small batches take the smallest so that the chip is used at all.
    const int64_t rows = (int64_t)a.B * (a.gmax + 1);
    int nv = 2;
    for (int cand = 8; cand >= 2; cand >>= 1) {
        const int64_t Wc = ((int64_t)a.V + 2048 * cand - 1) / (2048 * cand);
        if (cand == 2 || rows * Wc >= 2 * (int64_t)a.n_cu) { nv = cand; break; }
    }
    if (a.force_nv == 2 || a.force_nv == 4 || a.force_nv == 8) nv = a.force_nv;
    const int W = (a.V + 2048 * nv - 1) / (2048 * nv);
    const int64_t n_items = rows * W;
    const int grid = (int)n_items;
    const size_t lds_a = sizeof(LdsA) + (size_t)6 * W * sizeof(u64);
    const dim3 blk(kThreads);
    if (nv == 8) hipLaunchKernelGGL(accept_rows<8>, dim3(grid), blk, lds_a, stream, a, ws, W, (int)n_items);
    else if (nv == 4) hipLaunchKernelGGL(accept_rows<4>, dim3(grid), blk, lds_a, stream, a, ws, W, (int)n_items);
    else hipLaunchKernelGGL(accept_rows<2>, dim3(grid), blk, lds_a, stream, a, ws, W, (int)n_items);
    const size_t lds_b = sizeof(LdsB) + (size_t)4 * ws.w2 * sizeof(u64);
    if ((int64_t)ws.w2 * a.B <= a.n_cu)
        hipLaunchKernelGGL((accept_draw_row<8, 2>), dim3(ws.w2, a.B), blk, lds_b, stream, a, ws, ws.w2);
    else
        hipLaunchKernelGGL((accept_draw_row<8, 4>), dim3(ws.w2, a.B), blk, lds_b, stream, a, ws, ws.w2);
    return hipGetLastError();
}
