// The greedy limit T -> 0 of RAPID's validation loop (Alg. 1) for gfx950.
//
// As T -> 0, p and q become one-hot on the arg-max of their logits, the mixing term
// eta T (q - p) of Eq. new_target vanishes, and the ratio of the accept test behaves like
// exp(((z_x' - max z) - (zq_x' - max zq)) / T): it tends to infinity, 1 or 0 as the target's
// gap at the drafted token is above, equal to or below the drafter's gap.  A rejection and the
// bonus position emit the target's arg-max of that row (the limit of the residual for a draft
// that is the drafter's own arg-max, which is what a drafter proposes at T -> 0).  Equal maxima:
// the lowest index.  The accept test stays the literal r <= min(1, limit of the ratio).
//
// Two launches, every logit read once:
//   greedy_slice_argmax  per 4096-entry slice of every row: (max, lowest index of the max)
//   greedy_decide        one workgroup per sequence: rows combined, gaps compared in fp64 (the
//                        difference of two fp32 numbers is exact there), prefix length, token
#include "rapid_internal.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kSlice = kThreads * 16;

struct GreedyWs {
    int32_t* status;      // same place and meaning as in the general accept pass
    float* smax;          // [B][2 gmax + 1][W]
    int32_t* sidx;        // [B][2 gmax + 1][W]
    int W;
    size_t bytes;
};
__host__ __device__ inline size_t galign(size_t x) { return (x + 255) / 256 * 256; }
__host__ __device__ inline GreedyWs gcarve(void* base, int B, int gmax, int V)
{
    GreedyWs w;
    w.W = (V + kSlice - 1) / kSlice;
    char* p = static_cast<char*>(base);
    w.status = reinterpret_cast<int32_t*>(p); p += 256;
    const size_t n = (size_t)B * (2 * gmax + 1) * w.W;
    w.smax = reinterpret_cast<float*>(p); p += galign(n * sizeof(float));
    w.sidx = reinterpret_cast<int32_t*>(p); p += galign(n * sizeof(int32_t));
    w.bytes = (size_t)(p - static_cast<char*>(base));
    return w;
}

__device__ __forceinline__ int seq_gamma(const AcceptLaunch& a, int b)
{
    return a.gammas ? min(max(a.gammas[b], 0), a.gmax) : a.gmax;
}
// (value, index) pairs ordered by larger value, then lower index
__device__ __forceinline__ void take_better(float& m, int& i, float m2, int i2)
{
    if (m2 > m || (m2 == m && i2 < i)) { m = m2; i = i2; }
}

// Row y of sequence b: y <= gmax the target rows, then the draft rows.
__global__ void __launch_bounds__(kThreads) greedy_slice_argmax(AcceptLaunch a, GreedyWs ws)
{
    __shared__ float shm[kThreads / 64];
    __shared__ int shi[kThreads / 64];
    const int w = blockIdx.x, y = blockIdx.y, b = blockIdx.z;
    // only the two status words: the words behind them are the general pass's call counters, which persist
    if (w == 0 && y == 0 && b == 0 && threadIdx.x < 2) ws.status[threadIdx.x] = 0;
    const int g = seq_gamma(a, b);
    const bool is_t = y <= a.gmax;
    const int k = is_t ? y : y - (a.gmax + 1);
    if (is_t ? (k > g) : (k >= g)) return;
    const float* row = is_t ? a.zt + ((int64_t)b * (a.gmax + 1) + k) * a.V : a.zd + ((int64_t)b * a.gmax + k) * a.V;
    const bool vec = (reinterpret_cast<uintptr_t>(row) & 15) == 0;
    float m = -INFINITY;
    int idx = 0x7fffffff;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int i0 = w * kSlice + (v * kThreads + threadIdx.x) * 4;
        if (vec && i0 + 3 < a.V) {
            const floatx4 x = *reinterpret_cast<const floatx4*>(row + i0);
#pragma unroll
            for (int j = 0; j < 4; ++j) take_better(m, idx, x[j], i0 + j);
        } else {
            for (int j = 0; j < 4; ++j)
                if (i0 + j < a.V) take_better(m, idx, row[i0 + j], i0 + j);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) take_better(m, idx, __shfl_xor(m, o), __shfl_xor(idx, o));
    if ((threadIdx.x & 63) == 0) { shm[threadIdx.x >> 6] = m; shi[threadIdx.x >> 6] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int s = 1; s < kThreads / 64; ++s) take_better(m, idx, shm[s], shi[s]);
        const int64_t slot = ((int64_t)b * (2 * a.gmax + 1) + y) * ws.W + w;
        ws.smax[slot] = m;
        ws.sidx[slot] = idx;
    }
}

// One wave combines the slices of row y of sequence b; the result is valid in every lane.
__device__ __forceinline__ void row_argmax(const GreedyWs& ws, int64_t row, float& m, int& idx)
{
    const int lane = threadIdx.x & 63;
    m = -INFINITY;
    idx = 0x7fffffff;
    const int64_t base = row * ws.W;
    for (int s = lane; s < ws.W; s += 64) take_better(m, idx, ws.smax[base + s], ws.sidx[base + s]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) take_better(m, idx, __shfl_xor(m, o), __shfl_xor(idx, o));
}

__global__ void __launch_bounds__(kThreads) greedy_decide(AcceptLaunch a, GreedyWs ws)
{
    __shared__ int first_fail;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = seq_gamma(a, b);
    const int nrows = 2 * a.gmax + 1;
    if (tid == 0) first_fail = g;
    __syncthreads();
    // accept tests: one wave per drafted position
    for (int k = wave; k < g; k += kThreads / 64) {
        float mt, md;
        int it, id;
        row_argmax(ws, (int64_t)b * nrows + k, mt, it);
        row_argmax(ws, (int64_t)b * nrows + a.gmax + 1 + k, md, id);
        if (lane == 0) {
            const int x = a.tokens[(int64_t)b * a.gmax + k];
            double rho = 0.0;
            bool ok = false;
            if (x >= 0 && x < a.V) {
                // gaps of the drafted token to the row maxima; differences of fp32 values are exact in fp64
                const double gap_t = (double)a.zt[((int64_t)b * (a.gmax + 1) + k) * a.V + x] - (double)mt;
                const double gap_d = (double)a.zd[((int64_t)b * a.gmax + k) * a.V + x] - (double)md;
                rho = gap_t > gap_d ? INFINITY : (gap_t < gap_d ? 0.0 : 1.0);
                const double u = (double)a.uniforms[(int64_t)b * (a.gmax + 1) + k];
                ok = u <= fmin(1.0, rho);
            } else {
                atomicAdd(ws.status + 0, 1);                  // id outside the vocabulary: rejected, and counted
            }
            if (a.ratio) a.ratio[(int64_t)b * a.gmax + k] = (float)rho;
            if (!ok) atomicMin(&first_fail, k);
        }
    }
    __syncthreads();
    const int n = first_fail;
    if (wave == 0) {
        float m;
        int tok;
        row_argmax(ws, (int64_t)b * nrows + n, m, tok);       // target row n: rejection or bonus position
        if (lane == 0) {
            if (tok < 0 || tok >= a.V) tok = 0;               // a row of NaNs has no arg-max: any valid id
            a.out_tokens[(int64_t)b * (a.gmax + 1) + n] = tok;
            a.n_accepted[b] = n;
        }
    }
    for (int k = tid; k <= a.gmax; k += kThreads)
        if (k != n) a.out_tokens[(int64_t)b * (a.gmax + 1) + k] = k < n ? a.tokens[(int64_t)b * a.gmax + k] : -1;
}

}  // namespace

size_t accept_greedy_workspace_bytes(int B, int gmax, int V)
{
    return gcarve(nullptr, B, gmax, V).bytes;
}

hipError_t launch_accept_greedy(const AcceptLaunch& a, hipStream_t stream)
{
    GreedyWs ws = gcarve(a.workspace, a.B, a.gmax, a.V);
    hipLaunchKernelGGL(greedy_slice_argmax, dim3(ws.W, 2 * a.gmax + 1, a.B), dim3(kThreads), 0, stream, a, ws);
    hipLaunchKernelGGL(greedy_decide, dim3(a.B), dim3(kThreads), 0, stream, a, ws);
    return hipGetLastError();
}
