// Chunk selection of the RAG drafter (Sec. 2.2; "RAG Setup", Sec. 3) for gfx950:
// cosine similarity of every chunk embedding with the query embedding, the top-k
// chunks, those below the similarity threshold dropped, the rest reported in
// document order.  At most a few hundred chunks (128K tokens / 512) of dimension
// ~1024: a megabyte of input, run once per request, so the design goal is only to
// keep it on the device and to one pass over the embeddings:
//   K1: one wave per chunk, 16-byte loads, fp32 dot product and squared norm (the
//       query's norm is recomputed per wave from the same loads' companion);
//   K2: one workgroup ranks the similarities by counting (rank = number of chunks
//       that come first in "larger similarity, then lower index"), keeps rank <
//       top_k and sim >= threshold, and compacts the survivors in index order
//       with a block prefix sum.
#include "rapid_internal.h"

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__global__ void __launch_bounds__(256) retrieve_similarity(RetrieveLaunch a)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= a.n) return;
    const float* e = a.emb + (int64_t)i * a.dim;
    float dot = 0.f, en = 0.f, qn = 0.f;
    for (int c = lane * 4; c < a.dim; c += 256) {
        const floatx4 x = *reinterpret_cast<const floatx4*>(e + c);
        const floatx4 q = *reinterpret_cast<const floatx4*>(a.query + c);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            dot = fmaf(x[j], q[j], dot);
            en = fmaf(x[j], x[j], en);
            qn = fmaf(q[j], q[j], qn);
        }
    }
    dot = wave_sum(dot);
    en = wave_sum(en);
    qn = wave_sum(qn);
    if (lane == 0) a.sim[i] = (en > 0.f && qn > 0.f) ? dot / (sqrtf(en) * sqrtf(qn)) : 0.f;
}

constexpr int kMaxChunks = 1024;

__global__ void __launch_bounds__(256) retrieve_select(RetrieveLaunch a)
{
    __shared__ float s[kMaxChunks];
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < a.n; i += 256) s[i] = a.sim[i];
    __syncthreads();
    // thread t owns chunks 4t .. 4t+3 (consecutive, so that compaction keeps index order)
    int keep[4], cnt = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = tid * 4 + u;
        keep[u] = 0;
        if (i < a.n) {
            const float si = s[i];
            int rank = 0;
            for (int j = 0; j < a.n; ++j) {
                const float sj = s[j];
                rank += (sj > si || (sj == si && j < i)) ? 1 : 0;
            }
            keep[u] = (rank < a.top_k && si >= a.threshold) ? 1 : 0;
        }
        cnt += keep[u];
    }
    // exclusive prefix of cnt over the block
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int off = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (w < wave) off += wave_tot[w];
        total += wave_tot[w];
    }
    int pos = off + incl - cnt;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (keep[u]) a.selected[pos++] = tid * 4 + u;
    for (int p = total + tid; p < a.top_k; p += 256) a.selected[p] = -1;
    if (tid == 0) *a.n_selected = total;
}

}  // namespace

hipError_t launch_retrieve(const RetrieveLaunch& a, hipStream_t stream)
{
    hipLaunchKernelGGL(retrieve_similarity, dim3((a.n + 3) / 4), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(retrieve_select, dim3(1), dim3(256), 0, stream, a);
    return hipGetLastError();
}
