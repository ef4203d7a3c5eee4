// Acceptance pass of RAPID's validation loop (Alg. 1) for gfx950 (MI355X).
//
// Per sequence b and drafted position k the paper defines
//   p = softmax(z/T), q = softmax(z_q/T)                       (Alg. 1)
//   p_hat = softmax(z/T + eta (q - p))                         (Eq. new_target)
//   p_hat(v) <- p(v) where p_hat(v) < alpha * max p_hat        (tail rule, Sec. 2.4)
//   accept x' iff r <= min(1, p_hat(x')/q(x'))                 (Alg. 1)
//   first reject: x ~ norm(max(p - p_hat, p - q, 0)); none: x ~ p of the next row.
//
// The accept test at a position needs p, q, p_hat only at the one drafted token,
// given three log-normalisers per row; only the row where the draw happens needs
// an elementwise pass.  So the work is organised as reductions over the
// vocabulary, chunked over many workgroups so the logits stream at HBM rate:
//
//   K1 row_stats      : per chunk of 4096 entries (max z, sum exp((z - max)/T)) of every target and draft row
//   K2 shifted_stats  : per chunk (max, sum exp) of d = (z - zmax)/T + eta (q - p)
//   K3 decide         : one wave per row: combine chunks -> log-normalisers (double), accept
//                       test in double at the drafted token -> pass/fail flag, ratio
//   K4 residual_sums  : n = first failed flag; per chunk sum of the draw weights of row n (double);
//                       n_accepted and the accepted prefix of out_tokens
//   K5 draw           : locate the chunk and the token where the running sum passes u*W
//
// Sums over the vocabulary run in fp32 per thread and are combined in fp64;
// everything that decides an integer (accept test, draw) is evaluated in fp64.
// Statistics are kept relative to the raw row maximum so that dividing by T
// costs no absolute precision.
#include "rapid_internal.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kVec = 4;                 // 128-bit loads per thread and chunk
constexpr int kChunk = kThreads * 4 * kVec;   // vocabulary entries per workgroup (4096)
constexpr int kSub = 256;                // entries per draw-weight partial sum (one wave x one 128-bit load)
constexpr int kSubs = kChunk / kSub;     // partial sums per chunk
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float fexp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }

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
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ double wave_max(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o));
    return v;
}

// Block-wide reductions over kThreads threads; `sh` has >= 4 slots; the result
// is returned to every thread.
#define RAPID_BLOCK_REDUCE(NAME, T, WAVE_OP, COMBINE)                      \
    __device__ __forceinline__ T NAME(T v, T* sh)                          \
    {                                                                      \
        v = WAVE_OP(v);                                                    \
        __syncthreads();                                                   \
        if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;             \
        __syncthreads();                                                   \
        T r = sh[0];                                                       \
        for (int w = 1; w < kThreads / 64; ++w) r = COMBINE(r, sh[w]);     \
        return r;                                                          \
    }
#define RAPID_ADD(a, b) ((a) + (b))
RAPID_BLOCK_REDUCE(block_max, float, wave_max, fmaxf)
RAPID_BLOCK_REDUCE(block_sum, float, wave_sum, RAPID_ADD)
RAPID_BLOCK_REDUCE(block_max, double, wave_max, fmax)
RAPID_BLOCK_REDUCE(block_sum, double, wave_sum, RAPID_ADD)

// Four consecutive logits of a row starting at index i (i % 4 == 0); entries at or
// past V come back as -inf.  `vec` says the row base is 16-byte aligned.
__device__ __forceinline__ floatx4 load4(const float* row, int i, int V, bool vec)
{
    floatx4 r = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (vec && i + 3 < V) return *reinterpret_cast<const floatx4*>(row + i);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (i + j < V) r[j] = row[i + j];
    return r;
}

// Drafts of sequence b; device data, so clamped to the range the buffers were sized for.
__device__ __forceinline__ int seq_gamma(const AcceptLaunch& a, int b)
{
    return a.gammas ? min(max(a.gammas[b], 0), a.gmax) : a.gmax;
}

struct Ws {
    float2* st_t;     // [B][gmax+1][nch]  (raw max, sum exp((z-max)/T))
    float2* st_d;     // [B][gmax][nch]
    float2* st_h;     // [B][gmax][nch]    (max d, sum exp(d - max d)), d relative to the target row max / T
    double* rows;     // [B][gmax+1][8]: zmax_t, lse_p, zmax_d, lse_q, lse_h, 1/S_h (= max p_hat), -, -
    double* wsum;     // [B][nch*kSubs][2]: per 256 entries, sum of residual weights and sum of p (fallback)
    int32_t* flags;   // [B][gmax]: 1 = draft k passed its accept test
    int nch;          // chunks of kChunk entries (st_h, wsum)
    int nch_t, nch_d; // chunks of st_t / st_d: nch, or the caller's when the statistics come from outside
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

__host__ __device__ inline Ws carve(void* base, int B, int gmax, int V)
{
    Ws w;
    w.nch = (V + kChunk - 1) / kChunk;
    w.nch_t = w.nch_d = w.nch;
    char* p = static_cast<char*>(base);
    w.st_t = reinterpret_cast<float2*>(p); p += align256((size_t)B * (gmax + 1) * w.nch * sizeof(float2));
    w.st_d = reinterpret_cast<float2*>(p); p += align256((size_t)B * (gmax > 0 ? gmax : 1) * w.nch * sizeof(float2));
    w.st_h = reinterpret_cast<float2*>(p); p += align256((size_t)B * (gmax > 0 ? gmax : 1) * w.nch * sizeof(float2));
    w.rows = reinterpret_cast<double*>(p); p += align256((size_t)B * (gmax + 1) * 8 * sizeof(double));
    w.wsum = reinterpret_cast<double*>(p); p += align256((size_t)B * w.nch * kSubs * 2 * sizeof(double));
    w.flags = reinterpret_cast<int32_t*>(p); p += align256((size_t)B * (gmax > 0 ? gmax : 1) * sizeof(int32_t));
    return w;
}

// ---------------------------------------------------------------- K1
__global__ void __launch_bounds__(kThreads) accept_row_stats(AcceptLaunch a, Ws ws)
{
    __shared__ float sh[8];
    const int ch = blockIdx.x, y = blockIdx.y, b = blockIdx.z;
    const int g = seq_gamma(a, b);
    const bool is_t = y <= a.gmax;
    const int k = is_t ? y : y - (a.gmax + 1);
    if (is_t ? (k > g) : (k >= g)) return;
    if (is_t ? a.ext_t != nullptr : a.ext_d != nullptr) return;    // this side's statistics were supplied
    const float* row = is_t ? a.zt + ((int64_t)b * (a.gmax + 1) + k) * a.V
                            : a.zd + ((int64_t)b * a.gmax + k) * a.V;
    const bool vec = ((reinterpret_cast<uintptr_t>(row) & 15) == 0);
    floatx4 x[kVec];
    float m = -INFINITY;
#pragma unroll
    for (int v = 0; v < kVec; ++v) {
        x[v] = load4(row, ch * kChunk + (v * kThreads + threadIdx.x) * 4, a.V, vec);
        m = fmaxf(m, fmaxf(fmaxf(x[v][0], x[v][1]), fmaxf(x[v][2], x[v][3])));
    }
    m = block_max(m, sh);
    float s = 0.f;
    if (m > -INFINITY) {
#pragma unroll
        for (int v = 0; v < kVec; ++v)
#pragma unroll
            for (int j = 0; j < 4; ++j) s += fexp((x[v][j] - m) * a.inv_T);
    }
    s = block_sum(s, sh);
    if (threadIdx.x == 0) {
        float2* dst = is_t ? ws.st_t + ((int64_t)b * (a.gmax + 1) + k) * ws.nch
                           : ws.st_d + ((int64_t)b * a.gmax + k) * ws.nch;
        dst[ch] = make_float2(m, s);
    }
}

// Combine per-chunk (max, sum) pairs of a row: returns the row max and
// S = sum_i s_i exp((m_i - max) * inv_T) (inv_T = 1 when the maxima are already scaled).
__device__ __forceinline__ void combine_row(const float2* st, int nch, double inv_T, double* shd,
                                            double& M, double& S)
{
    double m = -INFINITY;
    for (int i = threadIdx.x; i < nch; i += kThreads) m = fmax(m, (double)st[i].x);
    M = block_max(m, shd);
    double s = 0.0;
    for (int i = threadIdx.x; i < nch; i += kThreads) {
        float2 v = st[i];
        if (v.y > 0.f) s += (double)v.y * exp(((double)v.x - M) * inv_T);
    }
    S = block_sum(s, shd);
}

// ---------------------------------------------------------------- K2
// Row statistics of the target and the draft row, combined in fp32 by every workgroup
// (enough for the elementwise pass; the decisions later use the fp64 combine of K3).
__device__ __forceinline__ void combine_pair_f32(const float2* st_t, int nt, const float2* st_d, int nd, float inv_T,
                                                 float* sh, float& Mt, float& lnSt, float& Md, float& lnSd)
{
    float mt = -INFINITY, md = -INFINITY;
    for (int i = threadIdx.x; i < nt; i += kThreads) mt = fmaxf(mt, st_t[i].x);
    for (int i = threadIdx.x; i < nd; i += kThreads) md = fmaxf(md, st_d[i].x);
    mt = wave_max(mt);
    md = wave_max(md);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sh[threadIdx.x >> 6] = mt; sh[4 + (threadIdx.x >> 6)] = md; }
    __syncthreads();
    Mt = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
    Md = fmaxf(fmaxf(sh[4], sh[5]), fmaxf(sh[6], sh[7]));
    float st = 0.f, sd = 0.f;
    for (int i = threadIdx.x; i < nt; i += kThreads) {
        float2 t = st_t[i];
        if (t.y > 0.f) st += t.y * fexp((t.x - Mt) * inv_T);
    }
    for (int i = threadIdx.x; i < nd; i += kThreads) {
        float2 d = st_d[i];
        if (d.y > 0.f) sd += d.y * fexp((d.x - Md) * inv_T);
    }
    st = wave_sum(st);
    sd = wave_sum(sd);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sh[threadIdx.x >> 6] = st; sh[4 + (threadIdx.x >> 6)] = sd; }
    __syncthreads();
    lnSt = __logf((sh[0] + sh[1]) + (sh[2] + sh[3]));
    lnSd = __logf((sh[4] + sh[5]) + (sh[6] + sh[7]));
}

__global__ void __launch_bounds__(kThreads) accept_shifted_stats(AcceptLaunch a, Ws ws)
{
    __shared__ float sh[8];
    const int ch = blockIdx.x, k = blockIdx.y, b = blockIdx.z;
    const int g = seq_gamma(a, b);
    if (k >= g) return;
    const float* zt = a.zt + ((int64_t)b * (a.gmax + 1) + k) * a.V;
    const float* zd = a.zd + ((int64_t)b * a.gmax + k) * a.V;
    const bool vec = ((reinterpret_cast<uintptr_t>(zt) & 15) == 0) && ((reinterpret_cast<uintptr_t>(zd) & 15) == 0);
    floatx4 x[kVec], y[kVec];                     // in flight while the row statistics combine
#pragma unroll
    for (int v = 0; v < kVec; ++v) {
        const int i0 = ch * kChunk + (v * kThreads + threadIdx.x) * 4;
        x[v] = load4(zt, i0, a.V, vec);
        y[v] = load4(zd, i0, a.V, vec);
    }
    float zmax_t, lnS_t, zmax_d, lnS_d;
    combine_pair_f32(ws.st_t + ((int64_t)b * (a.gmax + 1) + k) * ws.nch_t, ws.nch_t,
                     ws.st_d + ((int64_t)b * a.gmax + k) * ws.nch_d, ws.nch_d, a.inv_T, sh, zmax_t, lnS_t, zmax_d, lnS_d);
    float m = -INFINITY;
#pragma unroll
    for (int v = 0; v < kVec; ++v)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float at = (x[v][j] - zmax_t) * a.inv_T;          // z/T relative to the row max
            float ad = (y[v][j] - zmax_d) * a.inv_T;
            float p = fexp(at - lnS_t), q = fexp(ad - lnS_d);
            // entries past V were loaded as -inf: at = -inf, p = q = 0 -> d = -inf
            x[v][j] = fmaf(a.eta, q - p, at);
            m = fmaxf(m, x[v][j]);
        }
    m = block_max(m, sh);
    float s = 0.f;
    if (m > -INFINITY) {
#pragma unroll
        for (int v = 0; v < kVec; ++v)
#pragma unroll
            for (int j = 0; j < 4; ++j) s += fexp(x[v][j] - m);
    }
    s = block_sum(s, sh);
    if (threadIdx.x == 0) ws.st_h[((int64_t)b * a.gmax + k) * ws.nch + ch] = make_float2(m, s);
}

// ---------------------------------------------------------------- K3
// One wave per (sequence, row): combine the row's per-chunk statistics in fp64 and
// run the accept test of that row's drafted token.
__device__ __forceinline__ void wave_combine(const float2* st, int nch, double inv_T, double& M, double& S)
{
    const int lane = threadIdx.x & 63;
    double m = -INFINITY;
    for (int i = lane; i < nch; i += 64) m = fmax(m, (double)st[i].x);
    M = wave_max(m);
    double s = 0.0;
    for (int i = lane; i < nch; i += 64) {
        float2 v = st[i];
        if (v.y > 0.f) s += (double)v.y * exp(((double)v.x - M) * inv_T);
    }
    S = wave_sum(s);
}

__global__ void __launch_bounds__(64) accept_decide(AcceptLaunch a, Ws ws)
{
    const int k = blockIdx.x, b = blockIdx.y;
    const int g = seq_gamma(a, b);
    if (k > g) return;
    // the drafted token's two logits are fetched while the statistics combine
    int x = -1;
    float zx_t = 0.f, zx_d = 0.f;
    if (k < g) {
        x = a.tokens[(int64_t)b * a.gmax + k];
        if (x >= 0 && x < a.V) {
            zx_t = a.zt[((int64_t)b * (a.gmax + 1) + k) * a.V + x];
            zx_d = a.zd[((int64_t)b * a.gmax + k) * a.V + x];
        }
    }
    double Mt, St, Md = 0, Sd = 1, Mh = 0, Sh = 1;
    wave_combine(ws.st_t + ((int64_t)b * (a.gmax + 1) + k) * ws.nch_t, ws.nch_t, a.inv_T_exact, Mt, St);
    if (k < g) {
        wave_combine(ws.st_d + ((int64_t)b * a.gmax + k) * ws.nch_d, ws.nch_d, a.inv_T_exact, Md, Sd);
        wave_combine(ws.st_h + ((int64_t)b * a.gmax + k) * ws.nch, ws.nch, 1.0, Mh, Sh);
    }
    if (threadIdx.x != 0) return;
    double* r = ws.rows + ((int64_t)b * (a.gmax + 1) + k) * 8;
    const double lnS_t = log(St), lnS_d = log(Sd), lse_h = Mh + log(Sh), pmax = 1.0 / Sh;
    r[0] = Mt;                                   // raw max of the target row
    r[1] = lnS_t;                                // lse_p = r[0]/T + r[1]
    r[2] = Md;
    r[3] = lnS_d;
    r[4] = lse_h;                                // lse_h = r[0]/T + r[4]
    r[5] = pmax;                                 // max p_hat
    if (k >= g) return;
    double rho = 0.0;
    bool ok = false;
    if (x >= 0 && x < a.V) {
        const double invT = a.inv_T_exact;
        double at = ((double)zx_t - Mt) * invT;
        double ad = ((double)zx_d - Md) * invT;
        double p = exp(at - lnS_t), q = exp(ad - lnS_d);
        double ph = exp(at + (double)a.eta * (q - p) - lse_h);
        if (ph < (double)a.tail_alpha * pmax) ph = p;
        rho = q > 0.0 ? ph / q : INFINITY;
        double u = (double)a.uniforms[(int64_t)b * (a.gmax + 1) + k];
        ok = u <= fmin(1.0, rho);
    }
    if (a.ratio) a.ratio[(int64_t)b * a.gmax + k] = (float)rho;
    ws.flags[(int64_t)b * a.gmax + k] = ok ? 1 : 0;
}

// Number of accepted drafts: index of the first failed accept test, or g.
__device__ __forceinline__ int first_reject(const Ws& ws, int b, int gmax, int g)
{
    int n = g;
    for (int k = g - 1; k >= 0; --k)
        if (ws.flags[(int64_t)b * gmax + k] == 0) n = k;
    return n;
}

// Draw weight of vocabulary entry v of row n (fp64): the residual
// max(p - p_hat', p - q, 0) when n < g, p itself for the bonus row n = g.
struct RowCtx {
    const float* zt;
    const float* zd;
    double zmax_t, lnS_t, zmax_d, lnS_d, lse_h_rel, tail_thr, eta, invT;
    bool bonus;
};
__device__ __forceinline__ RowCtx make_row_ctx(const AcceptLaunch& a, const Ws& ws, int b, int n, int g)
{
    RowCtx c;
    const double* r = ws.rows + ((int64_t)b * (a.gmax + 1) + n) * 8;
    c.zt = a.zt + ((int64_t)b * (a.gmax + 1) + n) * a.V;
    c.zd = n < g ? a.zd + ((int64_t)b * a.gmax + n) * a.V : nullptr;
    c.zmax_t = r[0]; c.lnS_t = r[1]; c.zmax_d = r[2]; c.lnS_d = r[3]; c.lse_h_rel = r[4];
    c.tail_thr = (double)a.tail_alpha * r[5];
    c.eta = (double)a.eta;
    c.invT = (double)a.inv_T_exact;
    c.bonus = n >= g;
    return c;
}
__device__ __forceinline__ void weights(const RowCtx& c, int v, double& w, double& p)
{
    double at = ((double)c.zt[v] - c.zmax_t) * c.invT;
    p = exp(at - c.lnS_t);
    if (c.bonus) { w = p; return; }
    double ad = ((double)c.zd[v] - c.zmax_d) * c.invT;
    double q = exp(ad - c.lnS_d);
    double ph = exp(at + c.eta * (q - p) - c.lse_h_rel);
    if (ph < c.tail_thr) ph = p;
    w = fmax(fmax(p - ph, p - q), 0.0);
}

// ---------------------------------------------------------------- K4
__global__ void __launch_bounds__(kThreads) accept_residual_sums(AcceptLaunch a, Ws ws)
{
    const int ch = blockIdx.x, b = blockIdx.y;
    const int g = seq_gamma(a, b);
    const int n = first_reject(ws, b, a.gmax, g);
    if (ch == 0) {
        // accepted drafts, then -1 (the draw fills slot n later)
        for (int k = threadIdx.x; k <= a.gmax; k += kThreads)
            a.out_tokens[(int64_t)b * (a.gmax + 1) + k] = k < n ? a.tokens[(int64_t)b * a.gmax + k] : -1;
        if (threadIdx.x == 0) a.n_accepted[b] = n;
    }
    RowCtx c = make_row_ctx(a, ws, b, n, g);
    // one partial sum per wave: a run of 256 consecutive entries (the fp64 exponentials make
    // this kernel ALU-heavy, so it uses four times more workgroups than the statistics kernels)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i0 = (ch * kThreads + threadIdx.x) * 4;
    double sw = 0.0, sp = 0.0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (i0 + j < a.V) {
            double w, p;
            weights(c, i0 + j, w, p);
            sw += w;
            sp += p;
        }
    }
    sw = wave_sum(sw);
    sp = wave_sum(sp);
    if (lane == 0) {
        const int64_t sub = (int64_t)b * ws.nch * kSubs + ch * (kThreads / 64) + wave;
        ws.wsum[sub * 2 + 0] = sw;
        ws.wsum[sub * 2 + 1] = sp;
    }
}

// ---------------------------------------------------------------- K5
// Prefix sums over the kThreads threads of a block (fp64); `sh` has >= 4 slots.
// Returns the exclusive prefix; `incl` gets the inclusive one and `total` the block
// sum.  incl of thread j and the exclusive prefix of thread j+1 are the same
// floating-point value, so "first prefix above t" has exactly one owner.
__device__ __forceinline__ double block_scan(double v, double* sh, double& incl, double& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    double iw = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        double y = __shfl_up(iw, o);
        if (lane >= o) iw += y;
    }
    double ew = __shfl_up(iw, 1);
    if (lane == 0) ew = 0.0;
    __syncthreads();
    if (lane == 63) sh[wave] = iw;
    __syncthreads();
    double off = 0.0, tot = 0.0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        if (w < wave) off += sh[w];
        tot += sh[w];
    }
    total = tot;
    incl = off + iw;
    return off + ew;
}

__global__ void __launch_bounds__(kThreads) accept_draw(AcceptLaunch a, Ws ws)
{
    __shared__ double shd[8];
    __shared__ int pick_chunk, last_chunk, pick_lo, pick_hi;
    __shared__ double chunk_base;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int g = seq_gamma(a, b);
    const int n = first_reject(ws, b, a.gmax, g);
    RowCtx c = make_row_ctx(a, ws, b, n, g);
    const int nsub = ws.nch * kSubs;             // partial sums of 256 entries, in vocabulary order
    const double* cs = ws.wsum + (int64_t)b * nsub * 2;
    if (tid == 0) { pick_chunk = -1; last_chunk = 0; pick_lo = 0x7fffffff; pick_hi = -1; }

    // every thread owns `per` consecutive chunks
    const int per = (nsub + kThreads - 1) / kThreads;
    const int cbeg = min(tid * per, nsub), cend = min(cbeg + per, nsub);
    double tw = 0.0, tp = 0.0;
    for (int i = cbeg; i < cend; ++i) { tw += cs[i * 2]; tp += cs[i * 2 + 1]; }
    double Wres, Wp, in_w, in_p;
    const double ex_w = block_scan(tw, shd, in_w, Wres);
    const double ex_p = block_scan(tp, shd, in_p, Wp);
    const int col = Wres > 0.0 ? 0 : 1;          // empty residual: draw from p instead
    const double W = col == 0 ? Wres : Wp;
    const double t = (double)a.uniforms[(int64_t)b * (a.gmax + 1) + a.gmax] * W;

    // chunk whose inclusive running sum first exceeds t (chunks in vocabulary order)
    {
        const double excl = col == 0 ? ex_w : ex_p, incl = col == 0 ? in_w : in_p;
        int lastpos = -1;
        for (int i = cbeg; i < cend; ++i) if (cs[i * 2 + col] > 0.0) lastpos = i;
        if (lastpos >= 0) atomicMax(&last_chunk, lastpos);
        if (excl <= t && incl > t) {             // the crossing lies in this thread's chunks
            double run = excl;
            for (int i = cbeg; i < cend; ++i) {
                double v = cs[i * 2 + col];
                if (run + v > t || i == cend - 1) { pick_chunk = i; chunk_base = run; break; }
                run += v;
            }
        }
    }
    __syncthreads();
    if (pick_chunk < 0) {                         // t rounded up to W: last chunk with weight
        __syncthreads();
        if (tid == 0) {
            double base = 0.0;
            for (int i = 0; i < last_chunk; ++i) base += cs[i * 2 + col];
            pick_chunk = last_chunk;
            chunk_base = base;
        }
        __syncthreads();
    }
    constexpr int kPer = kSub / kThreads;           // entries per thread inside the chosen run
    const int i0 = pick_chunk * kSub + tid * kPer;
    double w[kPer], local = 0.0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        w[j] = 0.0;
        if (i0 + j < a.V) {
            double ww, pp;
            weights(c, i0 + j, ww, pp);
            w[j] = col == 0 ? ww : pp;
        }
        local += w[j];
    }
    double chunk_total, local_incl;
    double run = chunk_base + block_scan(local, shd, local_incl, chunk_total);
    int my_lo = 0x7fffffff, my_hi = -1;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        double nxt = run + w[j];
        if (w[j] > 0.0) {
            my_hi = i0 + j;
            if (nxt > t) my_lo = min(my_lo, i0 + j);
        }
        run = nxt;
    }
    if (my_hi >= 0) atomicMax(&pick_hi, my_hi);
    if (my_lo != 0x7fffffff) atomicMin(&pick_lo, my_lo);
    __syncthreads();
    if (tid == 0) {
        int tok = pick_lo != 0x7fffffff ? pick_lo : pick_hi;   // pick_hi: rounding at the chunk's end
        a.out_tokens[(int64_t)b * (a.gmax + 1) + n] = tok;
    }
}

}  // namespace

size_t accept_workspace_bytes(int B, int gmax, int V)
{
    Ws w = carve(nullptr, B, gmax, V);
    return reinterpret_cast<size_t>(w.flags) + align256((size_t)B * (gmax > 0 ? gmax : 1) * sizeof(int32_t));
}

hipError_t launch_accept(const AcceptLaunch& a, hipStream_t stream)
{
    Ws ws = carve(a.workspace, a.B, a.gmax, a.V);
    if (a.ext_t) { ws.st_t = reinterpret_cast<float2*>(const_cast<float*>(a.ext_t)); ws.nch_t = a.nch_t; }
    if (a.ext_d) { ws.st_d = reinterpret_cast<float2*>(const_cast<float*>(a.ext_d)); ws.nch_d = a.nch_d; }
    dim3 blk(kThreads);
    if (!a.ext_t || (a.gmax > 0 && !a.ext_d))
        hipLaunchKernelGGL(accept_row_stats, dim3(ws.nch, 2 * a.gmax + 1, a.B), blk, 0, stream, a, ws);
    if (a.gmax > 0)
        hipLaunchKernelGGL(accept_shifted_stats, dim3(ws.nch, a.gmax, a.B), blk, 0, stream, a, ws);
    hipLaunchKernelGGL(accept_decide, dim3(a.gmax + 1, a.B), dim3(64), 0, stream, a, ws);
    hipLaunchKernelGGL(accept_residual_sums, dim3(ws.nch * kVec, a.B), blk, 0, stream, a, ws);
    hipLaunchKernelGGL(accept_draw, dim3(a.B), blk, 0, stream, a, ws);
    return hipGetLastError();
}
