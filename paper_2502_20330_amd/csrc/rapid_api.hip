// C ABI of librapid.so: argument checking, split planning, kernel dispatch.
#include <new>

#include "rapid_internal.h"

// Scratch memory of the allocation-free entry point (rapid_verify_attn_static): one copy per
// GPU that loads this library, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; the device address is looked up once per context
// (rapid_create, with the context's device current) and kept in rapid_ctx::static_scratch.
static __device__ __align__(256) unsigned char scratch[RAPID_STATIC_SCRATCH_BYTES];

namespace {

// Makes the context's device current for the duration of a call and restores the caller's.
struct DeviceScope {
    int prev = -1;
    bool switched = false;
    hipError_t err = hipSuccess;
    explicit DeviceScope(int device)
    {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != device) {
            err = hipSetDevice(device);
            switched = err == hipSuccess;
        }
    }
    ~DeviceScope() { if (switched) (void)hipSetDevice(prev); }
};

// Largest page id a kernel may use: ids are device data and are clamped to [0, page_hi].
int page_hi_of(const rapid_attn_shape* s) { return s->n_pages > 0 ? s->n_pages - 1 : 0x7fffffff; }

#ifndef RAPID_WIDE_FROM
#define RAPID_WIDE_FROM 5
#endif
constexpr int kWideFromBlocks = RAPID_WIDE_FROM;    // row blocks from which the two-team attention kernel is used

// Row blocks of 16 packed query rows that the partials of a shape are laid out in.  Five and six
// blocks run on the two-team kernel (teams of 3 + 2 and 3 + 3 blocks).
int attn_row_blocks(const rapid_attn_shape* s, int* wide)
{
    const int G = s->n_q_heads / s->n_kv_heads;
    const int rb = (s->q_max * G + 15) / 16;
    if (wide) *wide = (rb >= kWideFromBlocks && rb >= 4) ? 1 : 0;
    return rb;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int hip_fail(rapid_ctx* ctx, hipError_t e)
{
    if (ctx) ctx->last_hip_error = (int)e;
    return RAPID_EHIP;
}

int check_attn_shape(const rapid_attn_shape* s)
{
    if (!s) return RAPID_EINVAL;
    if (s->batch < 1 || s->q_max < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->max_ctx < 1) return RAPID_EINVAL;
    if (s->n_q_heads % s->n_kv_heads) return RAPID_EINVAL;
    if (s->gamma < 0 || s->gamma >= s->q_max || s->max_ctx < s->q_max) return RAPID_EINVAL;
    if (!(s->softmax_scale > 0.f)) return RAPID_EINVAL;
    if (s->chunk_tokens < 0 || s->ctx_sum_hint < 0 || s->n_pages < 0) return RAPID_EINVAL;
    if (s->head_dim != 64 && s->head_dim != 128) return RAPID_EUNSUPPORTED;
    if (s->batch > 65535) return RAPID_EUNSUPPORTED;                       // grid z dimension
    const int G = s->n_q_heads / s->n_kv_heads;
    if ((int64_t)s->q_max * G > 96) return RAPID_EUNSUPPORTED;
    if (s->page_size != 0) {
        if (s->page_size < 16 || (s->page_size & (s->page_size - 1))) return RAPID_EUNSUPPORTED;
        if (s->max_pages < 1 || (int64_t)s->max_pages * s->page_size < s->max_ctx) return RAPID_EINVAL;
        if (s->kv_page_stride % 8) return RAPID_EALIGN;
    } else if (s->kv_batch_stride % 8) {
        return RAPID_EALIGN;
    }
    if (s->kv_token_stride < s->head_dim || s->kv_token_stride % 8 || s->kv_head_stride % 8) return RAPID_EALIGN;
    // rows of one (sequence, head) are addressed with 32-bit byte offsets
    const int64_t span_tokens = s->page_size ? s->page_size : s->max_ctx;
    if (s->kv_token_stride * 2 * span_tokens >= (int64_t)1 << 32) return RAPID_EUNSUPPORTED;
    // and so are the rows of q
    if ((int64_t)s->batch * s->q_max * s->n_q_heads * s->head_dim * 2 >= (int64_t)1 << 32) return RAPID_EUNSUPPORTED;
    return RAPID_OK;
}

// Tokens per KV split, a multiple of 128, never below 256 (two tiles per wave).
// Measured on uniform and ragged batches of 2..64 sequences: a workgroup costs about 8 us
// besides its streaming time, so for sequences of equal length one workgroup per compute
// unit (a single round of long splits) beats any finer grid by 5..15 %.  When the lengths
// differ, a single round leaves compute units idle behind the short sequences; two rounds
// let the dispatcher back-fill.  The host cannot see the lengths (device data), so it
// plans for equal lengths unless the caller passes their sum: then the split is sized so
// that the non-empty workgroups fill at most two rounds.
int plan_chunk(const rapid_ctx* ctx, const rapid_attn_shape* s)
{
    const int quantum = 128;
    if (s->chunk_tokens > 0) return (s->chunk_tokens + quantum - 1) / quantum * quantum;
    const int64_t n_cu = ctx ? ctx->n_cu : 256;
    const int64_t units = (int64_t)s->batch * s->n_kv_heads;
    const int64_t full = (int64_t)s->batch * s->max_ctx;
    const bool ragged = s->batch > 1 && s->ctx_sum_hint > 0 && s->ctx_sum_hint * 10 < full * 9;
    const int64_t tokens = (s->ctx_sum_hint > 0 && s->ctx_sum_hint < full) ? s->ctx_sum_hint : full;
    // workgroups that may hold tokens: every (sequence, head) wastes less than one split, so
    // sum_b ceil(L_b / chunk) * Hkv <= tokens * Hkv / chunk + units stays within two full rounds
    // (a third round of a few stragglers, each limited to one compute unit's bandwidth, is the
    // worst case)
    int64_t wgs = ragged ? 2 * n_cu - units : n_cu;
    if (wgs < units) wgs = units;
    int64_t chunk = (tokens * s->n_kv_heads + wgs - 1) / wgs;
    chunk = (chunk + quantum - 1) / quantum * quantum;
    if (chunk < 256) chunk = 256;
    const int64_t cap = ((int64_t)s->max_ctx + quantum - 1) / quantum * quantum;
    if (chunk > cap) chunk = cap;
    return (int)chunk;
}

// How the splits are laid over the chip (measured on MI355X, 128K context):
//  * rotate: when the rows of one head are contiguous in the cache (head stride above
//    token stride), spreading each head's splits over all dies is worth 4 % on
//    batches; when heads interleave inside a token row it costs 2.5 %, because the
//    workgroups that share those rows no longer run side by side.
//  * skew: with a single wave of workgroups (one per compute unit) the dies on odd
//    dispatch slots finish 10..15 % later than the even ones.  Moving about a tenth of a
//    split from each odd-slot workgroup to its even-slot pair partner evens that out
//    (2..3 % on the whole call).  With several workgroups per compute unit the
//    dispatcher balances by itself and the skew only hurts.
// The skew is a multiple of 128 tokens so both partners keep whole tiles per wave.
void plan_layout(const rapid_ctx* ctx, AttnLaunch& a)
{
    a.rot = a.hstride > a.tstride && a.Hkv > 1;
    a.skew = 0;
    const int64_t wgs = (int64_t)a.B * a.Hkv * a.nsplit;
    // measured: 3/32 of the split for the one-team kernel (config 3: 88.2 us with 384 tokens, 89.5 with 256,
    // 91.1 with none), 1/16 for the two-team kernel, which runs all waves through the same number of tiles
    // (70B shape: 93-94 us with 256 tokens, 96.5 with 384)
    if (a.rot && a.Hkv % 2 == 0 && a.nsplit >= 2 && wgs <= ctx->n_cu)
        a.skew = a.wide ? a.chunk / 16 / 128 * 128 : (a.chunk * 3 / 32 + 64) / 128 * 128;
}

}  // namespace

extern "C" {

int rapid_create(rapid_ctx** out, int device)
{
    if (!out) return RAPID_EINVAL;
    *out = nullptr;
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess) return RAPID_EHIP;
    if (device < 0 || device >= n) return RAPID_EINVAL;
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, device);
    if (e != hipSuccess) return RAPID_EHIP;
    // Kernels that need more dynamic LDS than the default limit are configured here, once
    // per context, on the context's device: no launch path changes function attributes, so
    // every entry point may be recorded into a stream capture.
    int prev = 0;
    if ((e = hipGetDevice(&prev)) != hipSuccess) return RAPID_EHIP;
    if ((e = hipSetDevice(device)) != hipSuccess) return RAPID_EHIP;
    hipError_t ec = configure_verify_attn();
    if (ec == hipSuccess) ec = configure_lm_head();
    if (ec == hipSuccess) ec = configure_hbm_read_probe();
    void* scratch_ptr = nullptr;                      // this device's copy of `scratch`
    if (ec == hipSuccess) ec = hipGetSymbolAddress(&scratch_ptr, HIP_SYMBOL(scratch));
    (void)hipSetDevice(prev);
    if (ec != hipSuccess || !scratch_ptr) return RAPID_EHIP;
    rapid_ctx* c = new (std::nothrow) rapid_ctx;
    if (!c) return RAPID_EINVAL;
    c->device = device;
    c->static_scratch = scratch_ptr;
    c->accept_wait_ticks = 100 * 100;                 // 100 us
    c->accept_slice = 0;
    c->probe_skew = 0;
    c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    c->last_hip_error = 0;
    *out = c;
    return RAPID_OK;
}

void rapid_destroy(rapid_ctx* ctx) { delete ctx; }

const char* rapid_strerror(int status)
{
    switch (status) {
        case RAPID_OK: return "ok";
        case RAPID_EINVAL: return "invalid argument";
        case RAPID_EALIGN: return "pointer or stride not aligned";
        case RAPID_EUNSUPPORTED: return "shape not supported";
        case RAPID_EWORKSPACE: return "workspace missing, misaligned or too small";
        case RAPID_EHIP: return "HIP runtime error";
        case RAPID_ETOOLARGE: return "shape needs more scratch memory than the allocation-free entry point holds";
    }
    return "unknown status";
}

int rapid_last_hip_error(const rapid_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

int rapid_set_option(rapid_ctx* ctx, int option, int64_t value)
{
    if (!ctx) return RAPID_EINVAL;
    switch (option) {
        case RAPID_OPT_ACCEPT_WAIT_US:
            if (value < 0 || value > 10 * 1000 * 1000) return RAPID_EINVAL;
            ctx->accept_wait_ticks = value * 100;         // the wall clock of the device ticks at 100 MHz
            return RAPID_OK;
        case RAPID_OPT_ACCEPT_SLICE:
            if (value != 0 && value != 4096 && value != 8192 && value != 16384) return RAPID_EINVAL;
            ctx->accept_slice = (int)value;
            return RAPID_OK;
        case RAPID_OPT_PROBE_SKEW:
            if (value < 0 || value > 16) return RAPID_EINVAL;
            ctx->probe_skew = (int)value;
            return RAPID_OK;
    }
    return RAPID_EINVAL;
}

int rapid_verify_attn_chunk(const rapid_ctx* ctx, const rapid_attn_shape* shape)
{
    int rc = check_attn_shape(shape);
    if (rc != RAPID_OK) return rc;
    return plan_chunk(ctx, shape);
}

size_t rapid_verify_attn_workspace_bytes(const rapid_ctx* ctx, const rapid_attn_shape* shape)
{
    if (check_attn_shape(shape) != RAPID_OK) return 0;
    const int chunk = plan_chunk(ctx, shape);
    const int nsplit = (shape->max_ctx + chunk - 1) / chunk;
    const int RB = attn_row_blocks(shape, nullptr);
    return attn_workspace_bytes(shape->batch, shape->n_kv_heads, nsplit, RB, shape->head_dim);
}

int rapid_verify_attn(rapid_ctx* ctx, const rapid_attn_shape* shape,
                      const void* q, const void* k_cache, const void* v_cache,
                      const int32_t* ctx_lens, const int32_t* gammas, const int32_t* page_table,
                      void* out, float* lse_out,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ctx) return RAPID_EINVAL;
    int rc = check_attn_shape(shape);
    if (rc != RAPID_OK) return rc;
    if (!q || !k_cache || !v_cache || !ctx_lens || !out) return RAPID_EINVAL;
    if (shape->page_size != 0 && !page_table) return RAPID_EINVAL;
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16)) return RAPID_EALIGN;
    const size_t need = rapid_verify_attn_workspace_bytes(ctx, shape);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < need) return RAPID_EWORKSPACE;

    AttnLaunch a{};
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k_cache);
    a.v = static_cast<const uint16_t*>(v_cache);
    a.ctx_lens = ctx_lens;
    a.gammas = gammas;
    a.page_table = shape->page_size ? page_table : nullptr;
    a.out = static_cast<uint16_t*>(out);
    a.lse_out = lse_out;
    a.B = shape->batch;
    a.Qmax = shape->q_max;
    a.Hq = shape->n_q_heads;
    a.Hkv = shape->n_kv_heads;
    a.G = a.Hq / a.Hkv;
    a.D = shape->head_dim;
    a.gamma = shape->gamma;
    a.max_ctx = shape->max_ctx;
    a.chunk = plan_chunk(ctx, shape);
    a.nsplit = (shape->max_ctx + a.chunk - 1) / a.chunk;
    a.RB = attn_row_blocks(shape, &a.wide);
    a.bstride = shape->kv_batch_stride;
    a.tstride = shape->kv_token_stride;
    a.hstride = shape->kv_head_stride;
    a.pstride = shape->kv_page_stride;
    a.max_pages = shape->max_pages;
    a.page_shift = -1;
    a.page_mask = 0;
    if (shape->page_size) {
        int sh = 0;
        while ((1 << sh) < shape->page_size) ++sh;
        a.page_shift = sh;
        a.page_mask = shape->page_size - 1;
    }
    a.page_hi = page_hi_of(shape);
    a.scale_log2e = shape->softmax_scale * 1.4426950408889634f;
    plan_layout(ctx, a);
    const size_t rows = (size_t)a.B * a.Hkv * a.nsplit * a.RB * 16;
    const size_t o_bytes = (rows * a.D * sizeof(float) + 255) / 256 * 256;
    a.part_o = static_cast<float*>(workspace);
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + o_bytes);

    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    hipError_t e = launch_verify_attn(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

int rapid_verify_attn_static(rapid_ctx* ctx, const rapid_attn_shape* shape,
                             const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* ctx_lens, const int32_t* gammas, const int32_t* page_table,
                             void* out, float* lse_out, void* stream)
{
    if (!ctx) return RAPID_EINVAL;
    const int rc = check_attn_shape(shape);
    if (rc != RAPID_OK) return rc;
    if (rapid_verify_attn_workspace_bytes(ctx, shape) > (size_t)RAPID_STATIC_SCRATCH_BYTES) return RAPID_ETOOLARGE;
    // same kernels, same argument checks; the split partials go to this device's static array
    return rapid_verify_attn(ctx, shape, q, k_cache, v_cache, ctx_lens, gammas, page_table, out, lse_out,
                             ctx->static_scratch, (size_t)RAPID_STATIC_SCRATCH_BYTES, stream);
}

size_t rapid_accept_workspace_bytes(const rapid_ctx*, int batch, int gamma_max, int vocab)
{
    if (batch < 1 || gamma_max < 0 || vocab < 1) return 0;
    const size_t general = accept_workspace_bytes(batch, gamma_max, vocab);
    const size_t greedy = accept_greedy_workspace_bytes(batch, gamma_max, vocab);
    return general > greedy ? general : greedy;
}

int rapid_accept_prestats(rapid_ctx* ctx, int batch, int gamma_max, int vocab,
                          const float* target_logits, const float* draft_logits,
                          const int32_t* draft_tokens, const int32_t* gammas,
                          float eta, float temperature, float tail_alpha,
                          const float* uniforms,
                          const float* target_stats, int target_chunks,
                          const float* draft_stats, int draft_chunks,
                          int32_t* n_accepted, int32_t* out_tokens, float* accept_ratio,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ctx || batch < 1 || gamma_max < 0 || vocab < 1) return RAPID_EINVAL;
    if (!target_logits || !uniforms || !n_accepted || !out_tokens) return RAPID_EINVAL;
    if (gamma_max > 0 && (!draft_logits || !draft_tokens)) return RAPID_EINVAL;
    if (!(eta >= 0.f) || !(temperature >= 0.f) || !(tail_alpha >= 0.f)) return RAPID_EINVAL;
    if ((target_stats && target_chunks < 1) || (draft_stats && draft_chunks < 1)) return RAPID_EINVAL;
    const bool greedy = temperature == 0.f;                 // the limit T -> 0; row statistics have no meaning there
    if (greedy && (target_stats || draft_stats)) return RAPID_EINVAL;
    if (batch > 65535 || gamma_max > 32767) return RAPID_EUNSUPPORTED;      // grid y / z dimensions
    if ((int64_t)batch * (gamma_max + 1) * (((int64_t)vocab + 4095) / 4096) >= ((int64_t)1 << 31)) return RAPID_EUNSUPPORTED;
    if (vocab > (1 << 22)) return RAPID_EUNSUPPORTED;                        // exchange slots of a row are staged in LDS
    if (!aligned(target_logits, 4) || !aligned(draft_logits, 4)) return RAPID_EALIGN;
    if (!aligned(target_stats, 8) || !aligned(draft_stats, 8)) return RAPID_EALIGN;
    const size_t need = rapid_accept_workspace_bytes(ctx, batch, gamma_max, vocab);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < need) return RAPID_EWORKSPACE;

    AcceptLaunch a{};
    a.zt = target_logits;
    a.zd = draft_logits;
    a.tokens = draft_tokens;
    a.gammas = gammas;
    a.uniforms = uniforms;
    a.n_accepted = n_accepted;
    a.out_tokens = out_tokens;
    a.ratio = accept_ratio;
    a.workspace = workspace;
    a.B = batch;
    a.gmax = gamma_max;
    a.V = vocab;
    a.eta = eta;
    a.inv_T_exact = greedy ? 0.0 : 1.0 / (double)temperature;
    a.inv_T = (float)a.inv_T_exact;
    a.tail_alpha = tail_alpha;
    a.ext_t = target_stats;
    a.nch_t = target_chunks;
    a.ext_d = gamma_max > 0 ? draft_stats : nullptr;
    a.nch_d = draft_chunks;
    a.wait_ticks = ctx->accept_wait_ticks;
    a.n_cu = ctx->n_cu;
    a.force_nv = ctx->accept_slice / 2048;
    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    hipError_t e = greedy ? launch_accept_greedy(a, static_cast<hipStream_t>(stream))
                          : launch_accept(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

int rapid_accept(rapid_ctx* ctx, int batch, int gamma_max, int vocab,
                 const float* target_logits, const float* draft_logits,
                 const int32_t* draft_tokens, const int32_t* gammas,
                 float eta, float temperature, float tail_alpha,
                 const float* uniforms,
                 int32_t* n_accepted, int32_t* out_tokens, float* accept_ratio,
                 void* workspace, size_t workspace_bytes, void* stream)
{
    return rapid_accept_prestats(ctx, batch, gamma_max, vocab, target_logits, draft_logits, draft_tokens, gammas,
                                 eta, temperature, tail_alpha, uniforms, nullptr, 0, nullptr, 0,
                                 n_accepted, out_tokens, accept_ratio, workspace, workspace_bytes, stream);
}

// Vocabulary rows per workgroup of the output head: the grid should fill the chip in whole
// rounds (one workgroup per compute unit and round), with at most 512 rows per workgroup.
static int lm_head_blocks(const rapid_ctx* ctx, int vocab, int /*n_rows*/)
{
    const int64_t nbmax = 32;
    const int64_t blocks = ((int64_t)vocab + 15) / 16;
    const int64_t n_cu = ctx ? ctx->n_cu : 256;
    const int64_t rounds = (blocks + nbmax * n_cu - 1) / (nbmax * n_cu);
    int64_t nb = (blocks + rounds * n_cu - 1) / (rounds * n_cu);
    if (nb < 1) nb = 1;
    if (nb > nbmax) nb = nbmax;
    return (int)nb;
}

int rapid_lm_head_chunk(const rapid_ctx* ctx, int vocab, int n_rows)
{
    return (vocab < 1 || n_rows < 1 || n_rows > 96) ? 0 : 16 * lm_head_blocks(ctx, vocab, n_rows);
}

int rapid_lm_head_stat_chunks(const rapid_ctx* ctx, int vocab, int n_rows)
{
    if (vocab < 1 || n_rows < 1 || n_rows > 96) return 0;
    const int chunk = 16 * lm_head_blocks(ctx, vocab, n_rows);
    return (vocab + chunk - 1) / chunk;
}

int rapid_lm_head(rapid_ctx* ctx, int n_rows, int hidden, int vocab,
                  const void* h, const void* w, float temperature,
                  float* logits, int64_t logits_row_stride, float* stats, void* stream)
{
    if (!ctx || !h || !w || !logits) return RAPID_EINVAL;
    if (n_rows < 1 || hidden < 1 || vocab < 1 || logits_row_stride < vocab || !(temperature > 0.f)) return RAPID_EINVAL;
    if (n_rows > 96 || hidden % 128 || vocab < 16) return RAPID_EUNSUPPORTED;
    if (!aligned(h, 16) || !aligned(w, 16) || !aligned(logits, 4) || !aligned(stats, 8)) return RAPID_EALIGN;
    LmHeadLaunch a{};
    a.h = static_cast<const uint16_t*>(h);
    a.w = static_cast<const uint16_t*>(w);
    a.logits = logits;
    a.stats = stats;
    a.n_rows = n_rows;
    a.hidden = hidden;
    a.vocab = vocab;
    a.ldz = logits_row_stride;
    a.nb = lm_head_blocks(ctx, vocab, n_rows);
    a.inv_T = (float)(1.0 / (double)temperature);
    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    hipError_t e = launch_lm_head(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

int rapid_kv_append(rapid_ctx* ctx, const rapid_attn_shape* shape, const void* k_new, const void* v_new,
                    const int32_t* ctx_lens, const int32_t* gammas, const int32_t* page_table,
                    void* k_cache, void* v_cache, void* stream)
{
    if (!ctx) return RAPID_EINVAL;
    int rc = check_attn_shape(shape);
    if (rc != RAPID_OK) return rc;
    if (!k_new || !v_new || !ctx_lens || !k_cache || !v_cache) return RAPID_EINVAL;
    if (shape->page_size != 0 && !page_table) return RAPID_EINVAL;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16)) return RAPID_EALIGN;
    KvAppendLaunch a{};
    a.k_new = static_cast<const uint16_t*>(k_new);
    a.v_new = static_cast<const uint16_t*>(v_new);
    a.ctx_lens = ctx_lens;
    a.gammas = gammas;
    a.page_table = shape->page_size ? page_table : nullptr;
    a.k_cache = static_cast<uint16_t*>(k_cache);
    a.v_cache = static_cast<uint16_t*>(v_cache);
    a.B = shape->batch;
    a.Qmax = shape->q_max;
    a.Hkv = shape->n_kv_heads;
    a.D = shape->head_dim;
    a.gamma = shape->gamma;
    a.max_ctx = shape->max_ctx;
    a.bstride = shape->kv_batch_stride;
    a.tstride = shape->kv_token_stride;
    a.hstride = shape->kv_head_stride;
    a.pstride = shape->kv_page_stride;
    a.max_pages = shape->max_pages;
    a.page_shift = -1;
    a.page_mask = 0;
    if (shape->page_size) {
        int sh = 0;
        while ((1 << sh) < shape->page_size) ++sh;
        a.page_shift = sh;
        a.page_mask = shape->page_size - 1;
    }
    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    a.page_hi = page_hi_of(shape);
    hipError_t e = launch_kv_append(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

int rapid_kv_commit(rapid_ctx* ctx, int batch, int gamma, const int32_t* gammas, const int32_t* n_accepted,
                    int32_t* ctx_lens, void* stream)
{
    if (!ctx || batch < 1 || gamma < 0 || !n_accepted || !ctx_lens) return RAPID_EINVAL;
    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    hipError_t e = launch_kv_commit(batch, gamma, gammas, n_accepted, ctx_lens, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

int rapid_kv_commit_pages(rapid_ctx* ctx, const rapid_attn_shape* shape, const int32_t* gammas,
                          const int32_t* n_accepted, const int32_t* page_table, int32_t* ctx_lens,
                          int32_t* released_pages, int release_cap, int32_t* n_released, void* stream)
{
    if (!ctx) return RAPID_EINVAL;
    const int rc = check_attn_shape(shape);
    if (rc != RAPID_OK) return rc;
    if (shape->page_size == 0 || !n_accepted || !page_table || !ctx_lens || !released_pages || !n_released) return RAPID_EINVAL;
    if (release_cap < (shape->q_max + shape->page_size - 2) / shape->page_size + 1) return RAPID_EINVAL;
    KvCommitPagesLaunch a{};
    a.gammas = gammas;
    a.n_accepted = n_accepted;
    a.page_table = page_table;
    a.ctx_lens = ctx_lens;
    a.released = released_pages;
    a.n_released = n_released;
    a.B = shape->batch;
    a.Qmax = shape->q_max;
    a.gamma = shape->gamma;
    a.max_ctx = shape->max_ctx;
    a.max_pages = shape->max_pages;
    a.cap = release_cap;
    a.page_hi = page_hi_of(shape);
    int sh = 0;
    while ((1 << sh) < shape->page_size) ++sh;
    a.page_shift = sh;
    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    hipError_t e = launch_kv_commit_pages(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

int rapid_retrieve(rapid_ctx* ctx, int n_chunks, int dim, const float* chunk_emb, const float* query_emb,
                   int top_k, float threshold, float* similarity, int32_t* selected, int32_t* n_selected, void* stream)
{
    if (!ctx || !chunk_emb || !query_emb || !similarity || !selected || !n_selected) return RAPID_EINVAL;
    if (n_chunks < 1 || dim < 1 || top_k < 1 || !(threshold == threshold)) return RAPID_EINVAL;
    if (n_chunks > 1024 || dim % 4) return RAPID_EUNSUPPORTED;
    if (!aligned(chunk_emb, 16) || !aligned(query_emb, 16)) return RAPID_EALIGN;
    RetrieveLaunch a{};
    a.emb = chunk_emb;
    a.query = query_emb;
    a.sim = similarity;
    a.selected = selected;
    a.n_selected = n_selected;
    a.n = n_chunks;
    a.dim = dim;
    a.top_k = top_k;
    a.threshold = threshold;
    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    hipError_t e = launch_retrieve(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

int rapid_hbm_read_probe(rapid_ctx* ctx, const void* buf, size_t bytes, void* sink, void* stream)
{
    if (!ctx || !buf) return RAPID_EINVAL;
    if (bytes < 16384 || bytes % 16384 || bytes >= ((size_t)1 << 46)) return RAPID_EINVAL;
    if (!aligned(buf, 16) || (sink && !aligned(sink, 4))) return RAPID_EALIGN;
    DeviceScope dev(ctx->device);
    if (dev.err != hipSuccess) return hip_fail(ctx, dev.err);
    hipError_t e = launch_hbm_read_probe(ctx, buf, bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return RAPID_OK;
}

}  // extern "C"
