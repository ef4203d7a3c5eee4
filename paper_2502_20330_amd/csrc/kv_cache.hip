// Cache bookkeeping around one validation round of Alg. 1 (gfx950).
//
// Before the target model validates gamma drafts, the keys and values of the gamma+1
// verification positions (the last committed token and the drafts) become the last
// gamma+1 tokens of the cache; after n drafts are accepted the sequence has grown by
// n+1 tokens, the newest of which has no key/value yet, so the cache keeps the first
// 1+n of those positions.  Both steps are tiny (36 KB per layer at 8 kv heads, d = 128,
// gamma = 8) and launch-bound; they exist so that a caller can run the whole round
// without a host round trip: lengths, gammas and the accepted counts stay on the device.
#include "rapid_internal.h"

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

// One workgroup per (query row i, sequence b): copies the Hkv * d elements of K and of V
// in 16-byte pieces to token ctx_lens[b] - (gamma_b+1) + i.
__global__ void __launch_bounds__(256) kv_append_rows(KvAppendLaunch a)
{
    const int i = blockIdx.x, b = blockIdx.y;
    // device data: clamped to the rows k_new / v_new hold
    const int Q = min(max(a.gammas ? a.gammas[b] : a.gamma, 0), a.Qmax - 1) + 1;
    if (i >= Q) return;
    const int64_t tok = (int64_t)min(a.ctx_lens[b], a.max_ctx) - Q + i;
    if (tok < 0) return;                                   // malformed length: nothing to write
    int64_t base;
    if (a.page_shift >= 0) {
        const int64_t pg = min(max(a.page_table[(int64_t)b * a.max_pages + (tok >> a.page_shift)], 0), a.page_hi);
        base = pg * a.pstride + (tok & a.page_mask) * a.tstride;
    } else {
        base = (int64_t)b * a.bstride + tok * a.tstride;
    }
    const int cpr = a.D / 8;                               // 16-byte pieces per (token, head)
    const int64_t src0 = ((int64_t)b * a.Qmax + i) * a.Hkv * a.D;
    for (int f = threadIdx.x; f < a.Hkv * cpr; f += blockDim.x) {
        const int h = f / cpr, c = f % cpr;
        const int64_t src = src0 + (int64_t)h * a.D + c * 8;
        const int64_t dst = base + (int64_t)h * a.hstride + c * 8;
        *reinterpret_cast<u32x4*>(a.k_cache + dst) = *reinterpret_cast<const u32x4*>(a.k_new + src);
        *reinterpret_cast<u32x4*>(a.v_cache + dst) = *reinterpret_cast<const u32x4*>(a.v_new + src);
    }
}

__global__ void __launch_bounds__(256) kv_commit_lengths(int B, int gamma, const int32_t* gammas,
                                                         const int32_t* n_accepted, int32_t* ctx_lens)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int g = gamma;
    if (gammas) {                                           // device data: kept inside the range the caller states
        g = max(gammas[b], 0);
        if (gamma > 0) g = min(g, gamma);
    }
    const int n = min(max(n_accepted[b], 0), g);
    ctx_lens[b] = ctx_lens[b] - (g + 1) + (1 + n);
}

// One thread per sequence: the length update, and the page-table slots that lie wholly past the
// committed length (at most a handful: the verification positions span few pages).
__global__ void __launch_bounds__(256) kv_commit_pages(KvCommitPagesLaunch a)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    const int g = min(max(a.gammas ? a.gammas[b] : a.gamma, 0), a.Qmax - 1);
    const int n = min(max(a.n_accepted[b], 0), g);
    const int l_old = min(max(a.ctx_lens[b], 0), a.max_ctx);
    const int l_new = max(l_old - (g + 1) + (1 + n), 0);
    const int ps = 1 << a.page_shift;
    const int first = (l_new + ps - 1) >> a.page_shift, end = min((l_old + ps - 1) >> a.page_shift, a.max_pages);
    int cnt = 0;
    for (int j = first; j < end && cnt < a.cap; ++j)
        a.released[(int64_t)b * a.cap + cnt++] = min(max(a.page_table[(int64_t)b * a.max_pages + j], 0), a.page_hi);
    a.n_released[b] = cnt;
    for (int j = cnt; j < a.cap; ++j) a.released[(int64_t)b * a.cap + j] = -1;
    a.ctx_lens[b] = l_new;
}

}  // namespace

hipError_t launch_kv_append(const KvAppendLaunch& a, hipStream_t stream)
{
    hipLaunchKernelGGL(kv_append_rows, dim3(a.Qmax, a.B), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_kv_commit_pages(const KvCommitPagesLaunch& a, hipStream_t stream)
{
    hipLaunchKernelGGL(kv_commit_pages, dim3((a.B + 255) / 256), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_kv_commit(int B, int gamma, const int32_t* gammas, const int32_t* n_accepted, int32_t* ctx_lens,
                            hipStream_t stream)
{
    hipLaunchKernelGGL(kv_commit_lengths, dim3((B + 255) / 256), dim3(256), 0, stream, B, gamma, gammas, n_accepted,
                       ctx_lens);
    return hipGetLastError();
}
