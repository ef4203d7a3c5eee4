/*
 * rapid.h -- C ABI of the MI355X (gfx950) verification step of RAPID,
 * retrieval-augmented speculative decoding.
 *
 * Two operations make up the step the target model performs on gamma drafted
 * tokens (Alg. 1, validation loop):
 *
 *   rapid_verify_attn  attention of the gamma+1 verification positions against
 *                      the whole long-context KV cache: the memory-bound part
 *                      of the target's logits for all drafted positions, which
 *                      the target computes in one pass (Sec. 2.1, Alg. 1);
 *   rapid_accept       p, q, the retrieval-augmented target p_hat
 *                      (Eq. new_target / Eq. delta), the tail rule (Sec. 2.4),
 *                      the accept test and the residual / bonus draw (Alg. 1).
 *
 * Around them: rapid_lm_head (the logits of the verification rows with the
 * statistics rapid_accept_prestats consumes), rapid_kv_append / rapid_kv_commit
 * (cache bookkeeping of a validation round), rapid_retrieve (the RAG drafter's
 * chunk selection, Sec. 2.2) and rapid_hbm_read_probe (a measurement aid).
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless it says "host".  The caller
 *     owns all buffers; the library allocates no device memory, keeps no
 *     pointer after a call returns, and only enqueues kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream).  Calls are
 *     asynchronous: synchronise the stream before reading results.
 *   - Shapes and strides are host values.  bf16 tensors are raw 16-bit words.
 *   - Every function returns 0 or a negative rapid_status; nothing aborts or
 *     prints.  After RAPID_EHIP, rapid_last_hip_error() gives the HIP code.
 *   - Two calls that share a workspace must not overlap in time.
 *   - rapid_create raises the dynamic-LDS limit of the kernels that need it; no other
 *     call changes device or function state, so all of them may be stream-captured.
 */
#ifndef RAPID_H
#define RAPID_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rapid_status {
    RAPID_OK = 0,
    RAPID_EINVAL = -1,        /* NULL pointer, non-positive size, gamma/ctx out of range, eta < 0, T < 0 */
    RAPID_EALIGN = -2,        /* q/k/v/out not 16-byte aligned, or a stride not a multiple of 8 elements  */
    RAPID_EUNSUPPORTED = -3,  /* head_dim not 64/128, (gamma+1)*group > 96, page size not a power of two >= 16 */
    RAPID_EWORKSPACE = -4,    /* workspace NULL, misaligned or smaller than the *_workspace_bytes() answer */
    RAPID_EHIP = -5,          /* a HIP runtime call failed */
    RAPID_ETOOLARGE = -6      /* rapid_verify_attn_static: the shape needs more than RAPID_STATIC_SCRATCH_BYTES */
} rapid_status;

typedef struct rapid_ctx rapid_ctx;   /* opaque; caches device properties, owns no device memory */

/* Create a context for HIP device `device`.  `*out` is host memory. */
int rapid_create(rapid_ctx** out, int device);
void rapid_destroy(rapid_ctx* ctx);
const char* rapid_strerror(int status);
int rapid_last_hip_error(const rapid_ctx* ctx);

/*
 * Tuning / test knobs of a context (host call, takes effect for later calls on this context).
 *   RAPID_OPT_ACCEPT_WAIT_US  The kernels of rapid_accept exchange partial results between
 *       workgroups; a workgroup waits at most this many microseconds for another one and then
 *       computes the missing piece itself (same arithmetic, same result).  Default 100; 0 = never
 *       wait (every exchange takes the recomputation path; for tests).  0 <= value <= 10^7.
 *   RAPID_OPT_ACCEPT_SLICE    Vocabulary entries per workgroup of rapid_accept's row pass:
 *       0 = chosen from the batch size (default), or 4096, 8192, 16384.  Results of the accept
 *       tests may differ in the last bits of accept_ratio between slice sizes (fp32 sums).
 *   RAPID_OPT_PROBE_SKEW      rapid_hbm_read_probe only: of every two consecutive workgroups the
 *       first reads (32 + value)/32 and the second (32 - value)/32 of the mean share, as
 *       rapid_verify_attn splits the tokens of a pair of KV splits unevenly when its grid is one
 *       workgroup per compute unit.  0 <= value <= 16; default 0 (equal shares).
 * Returns RAPID_EINVAL for an unknown option or a value out of range.
 */
typedef enum rapid_option {
    RAPID_OPT_ACCEPT_WAIT_US = 1,
    RAPID_OPT_ACCEPT_SLICE = 2,
    RAPID_OPT_PROBE_SKEW = 3
} rapid_option;
int rapid_set_option(rapid_ctx* ctx, int option, int64_t value);

/*
 * Shape of one rapid_verify_attn call (host struct).
 *
 * KV cache addressing, in ELEMENTS (bf16 words); element (b, token j, kv head h, c):
 *   contiguous (page_size == 0):  b*kv_batch_stride + j*kv_token_stride + h*kv_head_stride + c
 *   paged (page_size > 0):        page_table[b][j / page_size]*kv_page_stride
 *                                 + (j % page_size)*kv_token_stride + h*kv_head_stride + c
 * The head_dim elements of one (token, head) are contiguous.  K and V use the
 * same strides.  The natural layouts are [B, max_ctx, Hkv, d] and
 * [n_pages, page_size, Hkv, d].
 */
typedef struct rapid_attn_shape {
    int32_t batch;            /* B >= 1                                                        */
    int32_t q_max;            /* Qmax = max_b gamma_b + 1: query rows per sequence in q / out  */
    int32_t n_q_heads;        /* Hq                                                            */
    int32_t n_kv_heads;       /* Hkv, divides Hq; query head h reads kv head h / (Hq/Hkv)      */
    int32_t head_dim;         /* d: 64 or 128                                                  */
    int32_t max_ctx;          /* upper bound of ctx_lens[b]; sizes the grid and the workspace  */
    int32_t gamma;            /* drafts per sequence when gammas == NULL (0 <= gamma < q_max)  */
    float   softmax_scale;    /* > 0; scores are softmax_scale * <q, k>                        */
    int64_t kv_batch_stride;
    int64_t kv_token_stride;
    int64_t kv_head_stride;
    int64_t kv_page_stride;
    int32_t page_size;        /* 0 = contiguous cache, else a power of two >= 16               */
    int32_t max_pages;        /* row length of page_table                                      */
    int32_t chunk_tokens;     /* tokens per KV split; 0 = let the library choose               */
    int32_t n_pages;          /* pages in the pool, 0 = unknown: page_table entries (device data) are  */
                              /* clamped to [0, n_pages) before use; with 0 only negative entries are  */
                              /* clamped and larger ones are the caller's responsibility                */
    int64_t ctx_sum_hint;     /* sum of ctx_lens[b] if the host knows it (a scheduler usually  */
                              /* does), else 0: only used to size the KV splits of ragged      */
                              /* batches; results never depend on it                           */
} rapid_attn_shape;

/* Tokens per KV split the library will use for `shape` (multiple of 128), and
 * through it the number of splits per (sequence, kv head): ceil(max_ctx / chunk). */
int rapid_verify_attn_chunk(const rapid_ctx* ctx, const rapid_attn_shape* shape);

/* Bytes of device workspace rapid_verify_attn needs for `shape` (0 on a bad shape). */
size_t rapid_verify_attn_workspace_bytes(const rapid_ctx* ctx, const rapid_attn_shape* shape);

/*
 * Causal grouped-query attention of the verification positions (Sec. 2.1: the
 * target scores all gamma drafted positions in one forward pass; Alg. 1: the
 * target's logits at position j are conditioned on the context and the drafts before j).
 *
 * For sequence b let L = ctx_lens[b], Q = gamma_b + 1.  The cache already holds
 * K/V of the Q verification positions as its LAST Q valid tokens (L counts
 * them).  Query row i (0 <= i < Q) of head h attends keys 0 .. L-Q+i:
 *     out[b,i,h,:] = softmax_j(softmax_scale * <q[b,i,h,:], k[b,j,h/G,:]>) . v[b,j,h/G,:]
 * computed with fp32 accumulation from bf16 inputs, result rounded to bf16.
 * Rows i >= Q are written as zeros.  Rotary embedding etc. are the caller's.
 *
 *   q          bf16 [B, Qmax, Hq, d], contiguous
 *   k_cache    bf16, see rapid_attn_shape
 *   v_cache    bf16, same addressing as k_cache
 *   ctx_lens   int32 [B], gamma_b+1 <= ctx_lens[b] <= max_ctx; device data, so not checked: larger
 *              values are clamped to max_ctx, a sequence of length 0 yields zeros
 *   gammas     int32 [B] or NULL (-> shape->gamma for all), 0 <= gamma_b < Qmax (clamped to that range)
 *   page_table int32 [B, max_pages] when page_size > 0, else NULL
 *   out        bf16 [B, Qmax, Hq, d]
 *   lse_out    fp32 [B, Hq, Qmax] natural-log sum-exp of the scaled scores, or NULL
 *   workspace  >= rapid_verify_attn_workspace_bytes(), 256-byte aligned
 */
int rapid_verify_attn(rapid_ctx* ctx, const rapid_attn_shape* shape,
                      const void* q, const void* k_cache, const void* v_cache,
                      const int32_t* ctx_lens, const int32_t* gammas,
                      const int32_t* page_table,
                      void* out, float* lse_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * rapid_verify_attn for callers that cannot allocate device memory at all: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels,
 * same argument rules and results as rapid_verify_attn, but the split partials go to a static
 * device array inside the library (RAPID_STATIC_SCRATCH_BYTES per GPU, held from the moment the
 * library is loaded until the process ends) instead of a caller-supplied workspace; the call
 * allocates and frees nothing.
 *   - A shape whose rapid_verify_attn_workspace_bytes() exceeds RAPID_STATIC_SCRATCH_BYTES is
 *     refused with RAPID_ETOOLARGE (all other errors as for rapid_verify_attn).  The limit covers
 *     every configuration this library is benchmarked on (the largest, eight ragged 128K-token
 *     sequences, needs 21 MB).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU
 *     (different streams, or different contexts on that GPU) race.  Calls on one stream are safe.
 *   - The array keeps whatever the previous call left; nothing in it has to start at zero (slots of
 *     splits that hold no token are never read), so the call clears nothing.
 */
#define RAPID_STATIC_SCRATCH_BYTES (32u << 20)
int rapid_verify_attn_static(rapid_ctx* ctx, const rapid_attn_shape* shape,
                             const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* ctx_lens, const int32_t* gammas,
                             const int32_t* page_table,
                             void* out, float* lse_out, void* stream);

/* Bytes of device workspace rapid_accept needs (0 on bad sizes). */
size_t rapid_accept_workspace_bytes(const rapid_ctx* ctx, int batch, int gamma_max, int vocab);

/*
 * Accept / reject / resample for `batch` sequences (Alg. 1, validation loop).
 * For sequence b with g = gamma_b drafts, rows k = 0..g-1, temperature T:
 *     p_k  = softmax(z_k / T),  q_k = softmax(zq_k / T)
 *     ph_k = softmax(z_k / T + eta (q_k - p_k))                 (Eq. new_target)
 *     ph_k(v) <- p_k(v) where ph_k(v) < tail_alpha * max ph_k   (tail rule; mask from the
 *                                                                unreplaced ph_k, no renormalising)
 *     draft k accepted iff uniforms[b,k] <= min(1, ph_k(x_k) / q_k(x_k))
 *     n = index of the first rejected draft, or g
 *     n < g : token ~ norm(max(p_n - ph_n, p_n - q_n, 0))       (Alg. 1 residual)
 *     n = g : token ~ p_g  (target row g, the position after the last draft)
 * The draw is the inverse CDF in vocabulary order driven by uniforms[b, gamma_max]:
 * the smallest v whose running sum of weights exceeds u * (total weight).
 *
 *   target_logits fp32 [B, gamma_max+1, V]
 *   draft_logits  fp32 [B, gamma_max,   V]
 *   draft_tokens  int32 [B, gamma_max]; an id outside [0, V) rejects that position
 *   gammas        int32 [B] or NULL (-> gamma_max), 0 <= gamma_b <= gamma_max
 *   eta >= 0, temperature > 0, tail_alpha >= 0 (0 disables the tail rule; the paper uses 0.1)
 *   temperature == 0 selects the greedy limit T -> 0 of the same loop: p and q become one-hot on
 *       the arg-max of their rows (lowest index among equal maxima), the mixing term vanishes, and
 *       the ratio tends to infinity / 1 / 0 as the target's gap z[x_k] - max z is above / equal to /
 *       below the drafter's gap zq[x_k] - max zq; the test stays uniforms[b,k] <= min(1, that
 *       limit); a rejection and the bonus position emit the arg-max of target row n.  eta,
 *       tail_alpha and uniforms[b, gamma_max] are not used.  accept_ratio holds the limit.
 *   uniforms      fp32 [B, gamma_max+1] in [0, 1)
 *   n_accepted    int32 [B]
 *   out_tokens    int32 [B, gamma_max+1]: accepted drafts, the drawn token, then -1
 *   accept_ratio  fp32 [B, gamma_max] ph_k(x_k)/q_k(x_k) of every row k < gamma_b
 *                 (also after the first reject), or NULL
 *   workspace     >= rapid_accept_workspace_bytes(), 256-byte aligned.  Its first words are a
 *                 status block the caller may read once the stream is synchronised (int32):
 *                   [RAPID_ACCEPT_STATUS_BAD_IDS]  drafted positions of this call that were
 *                       rejected because the id was outside [0, V)
 *                   [RAPID_ACCEPT_STATUS_GIVEUPS]  diagnostics: exchange waits of this call that
 *                       ran into RAPID_OPT_ACCEPT_WAIT_US (results are unaffected)
 *                 Ownership: the workspace may hold anything when it is first used and is never
 *                 cleared by the library, but between two calls that use it the caller must either
 *                 leave all of it untouched or fill all of it with zeros: its head also holds a
 *                 counter that moves with every execution (replays of a captured HIP graph
 *                 included), and a call recognises what its own workgroups exchanged through the
 *                 workspace by tags derived from that counter.  Two calls that share a workspace
 *                 must not overlap in time.
 * vocab <= 2^22.  Logit rows whose address is not 16-byte aligned (vocab not a multiple of 4)
 * are read with scalar loads: same results, lower bandwidth.
 */
#define RAPID_ACCEPT_STATUS_BAD_IDS 0
#define RAPID_ACCEPT_STATUS_GIVEUPS 1
int rapid_accept(rapid_ctx* ctx, int batch, int gamma_max, int vocab,
                 const float* target_logits, const float* draft_logits,
                 const int32_t* draft_tokens, const int32_t* gammas,
                 float eta, float temperature, float tail_alpha,
                 const float* uniforms,
                 int32_t* n_accepted, int32_t* out_tokens, float* accept_ratio,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Vocabulary entries per statistics chunk of rapid_lm_head for this device, vocabulary and row count (a
 * multiple of 16, at most 512: one chunk per workgroup, sized so that the grid fills the chip in whole
 * rounds; it may depend on the row count), and the number of chunks per row, ceil(vocab / chunk).
 * 0 on bad sizes. */
int rapid_lm_head_chunk(const rapid_ctx* ctx, int vocab, int n_rows);
int rapid_lm_head_stat_chunks(const rapid_ctx* ctx, int vocab, int n_rows);

/*
 * Output head for the verification rows: what Alg. 1 calls LogitsOf(p(. | [C; x_<j])),
 * taken as the final hidden state times the output embedding (no bias; the final
 * normalisation layer is the caller's):
 *     logits[r][v] = sum_k h[r][k] * w[v][k]      bf16 inputs, fp32 accumulation
 * (the weights are read once whatever the row count) and, when `stats` is given, per row and per chunk c of
 * rapid_lm_head_chunk() consecutive entries
 *     stats[r][c] = ( max_v logits[r][v], sum_v exp((logits[r][v] - max) / temperature) )
 * which is what rapid_accept_prestats consumes (the pieces of softmax(z/T), Alg. 1).
 *
 *   n_rows       1..96 (the gamma+1 rows of one sequence or of a batch, ordered [sequence][position])
 *   hidden       a multiple of 128 (multiples of 256 take the faster path)
 *   vocab        >= 16
 *   h            bf16 [n_rows, hidden], contiguous, 16-byte aligned
 *   w            bf16 [vocab, hidden], contiguous, 16-byte aligned
 *   temperature  > 0 (used only for the statistics)
 *   logits       fp32, row r at logits + r * logits_row_stride (elements, >= vocab)
 *   stats        fp32 [n_rows, rapid_lm_head_stat_chunks(ctx, vocab, n_rows), 2] or NULL
 * No workspace.  RAPID_EUNSUPPORTED for row counts or hidden sizes outside the above.
 */
int rapid_lm_head(rapid_ctx* ctx, int n_rows, int hidden, int vocab,
                  const void* h, const void* w, float temperature,
                  float* logits, int64_t logits_row_stride, float* stats, void* stream);

/*
 * rapid_accept with the (max, sum exp) statistics of the rows supplied by the caller
 * instead of being formed from the logits by a first pass (same results up to the
 * rounding order of the fp32 sums inside a chunk):
 *   target_stats fp32 [B*(gamma_max+1), target_chunks, 2] or NULL; row b*(gamma_max+1)+k
 *   draft_stats  fp32 [B*gamma_max,     draft_chunks,  2] or NULL
 * each pair = (max of the raw logits of the chunk, sum exp((z - max)/temperature)) for ANY
 * partition of the vocabulary into chunks (an empty chunk: sum 0); the temperature must be the
 * one passed here.  A NULL side is computed from the logits as in rapid_accept.  Everything
 * else, including the workspace size, is as for rapid_accept.
 */
int rapid_accept_prestats(rapid_ctx* ctx, int batch, int gamma_max, int vocab,
                          const float* target_logits, const float* draft_logits,
                          const int32_t* draft_tokens, const int32_t* gammas,
                          float eta, float temperature, float tail_alpha,
                          const float* uniforms,
                          const float* target_stats, int target_chunks,
                          const float* draft_stats, int draft_chunks,
                          int32_t* n_accepted, int32_t* out_tokens, float* accept_ratio,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cache bookkeeping around one validation round (implied by Alg. 1: the target scores
 * [C; x_<j] for every drafted position j; its index i advances to j+1 with every accepted
 * draft and by one more after the residual draw).
 *
 * rapid_kv_append: row i (0 <= i <= gamma_b) of k_new / v_new becomes token
 * ctx_lens[b] - (gamma_b+1) + i of sequence b's cache; ctx_lens already counts the
 * appended positions, exactly as rapid_verify_attn expects them.  Rows i > gamma_b and
 * every other cache element are left untouched.  Rotary embedding etc. are the caller's.
 *   shape        the same struct as for rapid_verify_attn (layout, batch, q_max, gamma)
 *   k_new, v_new bf16 [B, Qmax, Hkv, d], contiguous, 16-byte aligned
 *   ctx_lens, gammas, page_table   device arrays as for rapid_verify_attn
 *   k_cache, v_cache               written in place
 *
 * rapid_kv_commit: of the gamma_b+1 verification positions the cache keeps the committed
 * token and the n_accepted[b] accepted drafts (the newly drawn token has no key/value yet):
 *     ctx_lens[b] <- ctx_lens[b] - (gamma_b + 1) + (1 + n_accepted[b])
 * in place, on the device (n_accepted is rapid_accept's output; values outside
 * [0, gamma_b] are clamped).  gammas == NULL: `gamma` for every sequence; otherwise gammas[b]
 * (device data) is clamped to >= 0 and, when gamma > 0, to <= gamma.
 *
 * rapid_kv_commit_pages: the same length update for a paged cache, and the bookkeeping a page
 * allocator needs after the roll-back: the pages of sequence b that held verification positions
 * only and lie wholly past the committed length can be handed back.  With L_old = ctx_lens[b] on
 * entry and L_new the committed length, these are the page-table slots j with
 *     ceil(L_new / page_size) <= j < ceil(L_old / page_size);
 * their page ids are written in ascending slot order to released_pages[b], the rest of the row is
 * -1, and n_released[b] is their number.  The page table itself is not modified (the caller
 * decides when to reuse the pages).  gamma_b is clamped to [0, q_max - 1] and L_old to max_ctx.
 *   shape           as for rapid_verify_attn (page_size > 0 required)
 *   released_pages  int32 [B, release_cap]; release_cap >= (q_max + page_size - 2) / page_size + 1
 *                   (RAPID_EINVAL if smaller)
 *   n_released      int32 [B]
 */
int rapid_kv_append(rapid_ctx* ctx, const rapid_attn_shape* shape, const void* k_new, const void* v_new,
                    const int32_t* ctx_lens, const int32_t* gammas, const int32_t* page_table,
                    void* k_cache, void* v_cache, void* stream);
int rapid_kv_commit(rapid_ctx* ctx, int batch, int gamma, const int32_t* gammas, const int32_t* n_accepted,
                    int32_t* ctx_lens, void* stream);
int rapid_kv_commit_pages(rapid_ctx* ctx, const rapid_attn_shape* shape, const int32_t* gammas,
                          const int32_t* n_accepted, const int32_t* page_table, int32_t* ctx_lens,
                          int32_t* released_pages, int release_cap, int32_t* n_released, void* stream);

/*
 * Chunk selection of the RAG drafter (Sec. 2.2; "RAG Setup" in Sec. 3): the long context is
 * cut into chunks, every chunk and the query are embedded by the caller, and the drafter's
 * context is made of the top_k chunks by cosine similarity with the query, without those whose
 * similarity is below `threshold` (the paper uses 512-token chunks and 0.3):
 *     similarity[i] = <e_i, q> / (|e_i| |q|)      (0 if either norm is 0), fp32
 *     selected      = { i : rank(i) < top_k and similarity[i] >= threshold }, ascending i,
 * where rank orders by larger similarity first and lower index first among equal values (the
 * order of the output and the tie rule are conventions of this library).
 *
 *   chunk_emb   fp32 [n_chunks, dim], contiguous, 16-byte aligned; n_chunks <= 1024, dim % 4 == 0
 *   query_emb   fp32 [dim], 16-byte aligned
 *   similarity  fp32 [n_chunks]
 *   selected    int32 [top_k]: the kept chunk indices in document order, then -1
 *   n_selected  int32 [1]
 * All pointers are device memory.  No workspace.
 */
int rapid_retrieve(rapid_ctx* ctx, int n_chunks, int dim, const float* chunk_emb, const float* query_emb,
                   int top_k, float threshold, float* similarity, int32_t* selected, int32_t* n_selected, void* stream);

/*
 * Measurement aid, not part of the method: reads `bytes` bytes of device memory at
 * `buf` once, with the load path of rapid_verify_attn (HBM -> LDS, streaming hint)
 * and no arithmetic, so that a benchmark can time the read bandwidth this device
 * actually delivers and quote kernel rates against it as well as against the
 * published peak.
 *
 *   buf    device memory, 16-byte aligned, not written
 *   bytes  a multiple of 16384, at least 16384 and below 2^46
 *   sink   4 bytes of device memory or NULL; written only if the XOR of the words
 *          the kernel inspects equals one particular constant (this keeps the loads
 *          observable), so treat its content as unspecified
 * Returns RAPID_EINVAL / RAPID_EALIGN on bad arguments, RAPID_EHIP on launch failure.
 */
int rapid_hbm_read_probe(rapid_ctx* ctx, const void* buf, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RAPID_H */
