/*
 * rapid_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, float64 CPU statement of what the RAPID verification step
 * computes.  It exists so that the GPU library can be checked against
 * something that can be compared with the paper by eye.  It shares no code,
 * header, table or helper with the GPU library; only tests, the smoke check
 * and the CPU-baseline leg of the benchmark may call it.
 *
 * Functions:
 *
 *   oracle_verify_attn  -- the target model's attention for the gamma+1
 *       verification positions against the whole KV cache (Sec. 2.1: the
 *       target scores all drafted positions in one forward pass; Alg. 1: the
 *       step that takes the target's logits at position j).  The paper gives no formula
 *       for attention itself: this is the textbook definition of causal,
 *       grouped-query softmax attention written out per (sequence, query
 *       position, query head) with a two-pass softmax.  No tiling, no online
 *       rescaling, no splitting.
 *
 *   oracle_accept       -- Alg. 1, the body of the validation loop and the
 *       residual draw, in the paper's order and notation:
 *         p  = softmax(z/T), q = softmax(z_q/T)          (Alg. 1; Sec. 2.3)
 *         zh = z + eta*T*(q - p)                         (Eq. "delta")
 *         ph = softmax(zh/T)                             (Eq. "new_target")
 *         ph_v <- p_v where ph_v < alpha * max_j ph_j    (tail rule, Sec. 2.4)
 *         accept x' iff r <= min(1, ph(x')/q(x'))        (Alg. 1 accept test)
 *         on first reject: x ~ norm(max(p-ph, p-q, 0))   (Alg. 1 residual)
 *         all accepted:    x ~ p of the next position    (Sec. 2.1 background)
 *       How a uniform number is turned into a token (inverse CDF in index
 *       order) is an interface convention of this build, not the paper's.
 *
 *   oracle_accept_greedy -- the T -> 0 limit of the same loop (see the function).
 *
 *   oracle_lm_head      -- what "LogitsOf" (Alg. 1) means for a decoder
 *       language model: the logits of a position are its final hidden state
 *       times the output embedding, z[r][v] = sum_k h[r][k] * W[v][k] (no
 *       bias; the final normalisation is the caller's).  The paper does not
 *       spell this out; it is the standard head of the models it uses.
 *   oracle_chunk_stats  -- per block of `chunk` consecutive vocabulary entries,
 *       max_v z and sum_v exp((z - max)/T): the pieces from which
 *       softmax(z/T) of Alg. 1 is normalised.
 *
 *   oracle_kv_append / oracle_kv_commit -- the cache bookkeeping Alg. 1 implies
 *       around a validation round: the keys/values of the gamma+1 verification
 *       positions become the last gamma+1 tokens of the cache before the target
 *       runs; after n drafts are accepted the sequence has grown by n+1 tokens
 *       (Alg. 1: the index i moves to j+1 with every accepted draft and by one
 *       more after the residual draw), of which the last has no key/value yet, so the cache keeps the
 *       first 1+n verification positions.
 *
 *   oracle_retrieve     -- chunk selection of the RAG drafter (Sec. 2.2; "RAG
 *       Setup" in Sec. 3): cosine similarity of every chunk embedding with the
 *       query embedding, the top-k chunks, those below the similarity threshold
 *       dropped.  Output order (document order) and tie handling (lower index
 *       first) are this build's conventions; the paper does not state them.
 *
 * Pins: every function here is pinned by tests that do not call it to check
 * itself (dense torch attention on tiny inputs, closed forms, the eta = 0
 * reduction to textbook speculative sampling, chi-square against the
 * analytically derived output law, finite differences of Proposition 1).
 *
 * All floating point is double.  bf16 inputs are widened exactly.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* bf16 (upper half of an IEEE binary32) -> double, exact.             */
static double bf16_to_double(uint16_t bits)
{
    uint32_t w = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* Where token j of sequence b lives: element offset of (token, kv head, 0). */
typedef struct {
    int64_t batch_stride;   /* contiguous cache: elements between sequences        */
    int64_t token_stride;   /* elements between consecutive tokens (in a page too) */
    int64_t head_stride;    /* elements between kv heads of one token              */
    int32_t page_size;      /* tokens per page, used only when page_table != NULL  */
    int64_t page_stride;    /* elements between pages                              */
    int32_t max_pages;      /* row length of page_table                            */
} oracle_kv_layout;

static int64_t kv_offset(const oracle_kv_layout* lay, const int32_t* page_table,
                         int b, int64_t j, int hkv)
{
    if (page_table) {
        int64_t page = page_table[(int64_t)b * lay->max_pages + j / lay->page_size];
        int64_t slot = j % lay->page_size;
        return page * lay->page_stride + slot * lay->token_stride + hkv * lay->head_stride;
    }
    return b * lay->batch_stride + j * lay->token_stride + hkv * lay->head_stride;
}

/*
 * Causal GQA attention of the verification positions.
 *
 * q    : bf16 bits [B, Qmax, Hq, d]
 * k, v : bf16 bits, addressed through `lay` (+ page_table when paged)
 * ctx_lens[b] : number of valid tokens in the cache of sequence b, INCLUDING
 *               the gamma_b+1 verification positions, which are its last ones
 * gammas[b]   : number of draft tokens of sequence b (NULL -> gamma for all)
 * out  : double [B, Qmax, Hq, d]; rows i > gamma_b are set to 0
 * lse  : double [B, Hq, Qmax] natural-log sum-exp of the scaled scores, or NULL
 *
 * Query position i of sequence b sees keys 0 .. L-Q+i (L = ctx_lens[b],
 * Q = gamma_b+1): the whole earlier context plus verification positions <= i.
 * Query head h reads kv head h / (Hq/Hkv).
 * Returns 0, or -1 on an invalid argument.
 */
int oracle_verify_attn(int B, int Qmax, int Hq, int Hkv, int d, double scale,
                       const uint16_t* q, const uint16_t* k, const uint16_t* v,
                       const oracle_kv_layout* lay, const int32_t* page_table,
                       const int32_t* ctx_lens, const int32_t* gammas, int gamma,
                       double* out, double* lse)
{
    if (B < 0 || Qmax <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
    const int G = Hq / Hkv;
    for (int b = 0; b < B; ++b) {
        int g = gammas ? gammas[b] : gamma;
        if (g < 0 || g + 1 > Qmax || ctx_lens[b] < g + 1) return -1;
    }
    int64_t units = (int64_t)B * Qmax * Hq;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        int h = (int)(u % Hq);
        int i = (int)((u / Hq) % Qmax);
        int b = (int)(u / ((int64_t)Hq * Qmax));
        int Q = (gammas ? gammas[b] : gamma) + 1;
        int64_t L = ctx_lens[b];
        double* o = out + u * d;
        if (i >= Q) {
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            if (lse) lse[((int64_t)b * Hq + h) * Qmax + i] = 0.0;
            continue;
        }
        int hkv = h / G;
        int64_t nvis = L - Q + i + 1;           /* keys 0 .. L-Q+i */
        double* s = (double*)malloc(sizeof(double) * (size_t)nvis);
        double* qd = (double*)malloc(sizeof(double) * (size_t)d);
        if (!s || !qd) { bad = 1; free(s); free(qd); continue; }
        for (int c = 0; c < d; ++c)
            qd[c] = bf16_to_double(q[u * d + c]);
        /* pass 1: scores and their maximum */
        double m = -INFINITY;
        for (int64_t j = 0; j < nvis; ++j) {
            const uint16_t* kr = k + kv_offset(lay, page_table, b, j, hkv);
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += qd[c] * bf16_to_double(kr[c]);
            s[j] = scale * acc;
            if (s[j] > m) m = s[j];
        }
        /* pass 2: weights, their sum, weighted sum of values */
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        double denom = 0.0;
        for (int64_t j = 0; j < nvis; ++j) {
            double w = exp(s[j] - m);
            denom += w;
            const uint16_t* vr = v + kv_offset(lay, page_table, b, j, hkv);
            for (int c = 0; c < d; ++c) o[c] += w * bf16_to_double(vr[c]);
        }
        for (int c = 0; c < d; ++c) o[c] /= denom;
        if (lse) lse[((int64_t)b * Hq + h) * Qmax + i] = m + log(denom);
        free(s);
        free(qd);
    }
    return bad ? -2 : 0;
}

/* ------------------------------------------------------------------ */
/* softmax(x / T) over n entries, max-subtracted.                      */
static void softmax_T(const double* x, double T, int64_t n, double* out)
{
    double m = -INFINITY;
    for (int64_t v = 0; v < n; ++v) if (x[v] / T > m) m = x[v] / T;
    double sum = 0.0;
    for (int64_t v = 0; v < n; ++v) { out[v] = exp(x[v] / T - m); sum += out[v]; }
    for (int64_t v = 0; v < n; ++v) out[v] /= sum;
}

/*
 * The three distributions of one verified position (Sec. 2.3-2.4).
 *   p  = softmax(z/T)
 *   q  = softmax(zq/T)
 *   zh = z + eta*T*(q-p);  ph = softmax(zh/T)
 *   tail rule: every entry of ph below tail_alpha * max(ph) is replaced by the
 *   entry of p (mask taken from ph before any replacement; no renormalising).
 * z, zq, p, q, ph: double[V].
 */
void oracle_distributions(int64_t V, const double* z, const double* zq,
                          double eta, double T, double tail_alpha,
                          double* p, double* q, double* ph)
{
    softmax_T(z, T, V, p);
    softmax_T(zq, T, V, q);
    double* zh = (double*)malloc(sizeof(double) * (size_t)V);
    for (int64_t v = 0; v < V; ++v) zh[v] = z[v] + eta * T * (q[v] - p[v]);
    softmax_T(zh, T, V, ph);
    free(zh);
    double mx = 0.0;
    for (int64_t v = 0; v < V; ++v) if (ph[v] > mx) mx = ph[v];
    double thr = tail_alpha * mx;
    for (int64_t v = 0; v < V; ++v) if (ph[v] < thr) ph[v] = p[v];
}

/*
 * Inverse-CDF draw from unnormalised non-negative weights w[0..V-1]:
 * W = sum in index order, t = u*W, token = smallest v whose running sum
 * (same order) exceeds t.  *margin = distance of t/W to the nearer edge of the
 * chosen token's interval of the normalised CDF.  Returns -1 if W == 0.
 */
static int64_t draw_inverse_cdf(const double* w, int64_t V, double u, double* margin)
{
    double W = 0.0;
    for (int64_t v = 0; v < V; ++v) W += w[v];
    if (!(W > 0.0)) return -1;
    double t = u * W, run = 0.0;
    int64_t tok = -1;
    double lo = 0.0;
    for (int64_t v = 0; v < V; ++v) {
        lo = run;
        run += w[v];
        if (run > t) { tok = v; break; }
    }
    if (tok < 0) {               /* u*W rounded up to W: last entry with weight */
        for (int64_t v = V - 1; v >= 0; --v) if (w[v] > 0.0) { tok = v; break; }
        if (margin) *margin = 0.0;
        return tok;
    }
    if (margin) {
        double a = (t - lo) / W, c = (run - t) / W;
        *margin = a < c ? a : c;
    }
    return tok;
}

/*
 * Accept / reject / resample for B sequences (Alg. 1, validation loop).
 *
 * target_logits : float [B, gmax+1, V]; row k is the target's logits for the
 *                 position of draft k; row gamma_b is the position after the
 *                 last draft (used only when all drafts are accepted)
 * draft_logits  : float [B, gmax, V]
 * draft_tokens  : int32 [B, gmax]
 * gammas        : int32 [B] or NULL (-> gmax for all)
 * uniforms      : float [B, gmax+1]; entry k < gamma_b drives accept test k,
 *                 entry gmax drives the one draw
 * n_accepted    : int32 [B]
 * out_tokens    : int32 [B, gmax+1]: the accepted drafts, then the drawn
 *                 token, then -1
 * ratio         : double [B, gmax]  ph(x')/q(x') of every position (all rows
 *                 are evaluated, also after the first reject), or NULL
 * accept_margin : double [B, gmax]  |min(1, ratio) - r|, or NULL
 * draw_margin   : double [B]        see draw_inverse_cdf, or NULL
 * Returns 0, -1 on an invalid argument.
 */
int oracle_accept(int B, int gmax, int64_t V,
                  const float* target_logits, const float* draft_logits,
                  const int32_t* draft_tokens, const int32_t* gammas,
                  double eta, double T, double tail_alpha,
                  const float* uniforms,
                  int32_t* n_accepted, int32_t* out_tokens,
                  double* ratio, double* accept_margin, double* draw_margin)
{
    if (B < 0 || gmax < 0 || V <= 0 || !(T > 0.0) || eta < 0.0) return -1;
    for (int b = 0; b < B; ++b) {
        int g = gammas ? gammas[b] : gmax;
        if (g < 0 || g > gmax) return -1;
        for (int k = 0; k < g; ++k) {
            int32_t x = draft_tokens[(int64_t)b * gmax + k];
            if (x < 0 || x >= V) return -1;
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int g = gammas ? gammas[b] : gmax;
        double* z  = (double*)malloc(sizeof(double) * (size_t)V);
        double* zq = (double*)malloc(sizeof(double) * (size_t)V);
        double* p  = (double*)malloc(sizeof(double) * (size_t)V);
        double* q  = (double*)malloc(sizeof(double) * (size_t)V);
        double* ph = (double*)malloc(sizeof(double) * (size_t)V);
        double* w  = (double*)malloc(sizeof(double) * (size_t)V);
        int32_t* toks = out_tokens + (int64_t)b * (gmax + 1);
        for (int k = 0; k <= gmax; ++k) toks[k] = -1;

        int n = g;                       /* number of accepted drafts            */
        for (int k = 0; k < g; ++k) {
            const float* zr  = target_logits + ((int64_t)b * (gmax + 1) + k) * V;
            const float* zqr = draft_logits + ((int64_t)b * gmax + k) * V;
            for (int64_t t = 0; t < V; ++t) { z[t] = zr[t]; zq[t] = zqr[t]; }
            oracle_distributions(V, z, zq, eta, T, tail_alpha, p, q, ph);
            int32_t x = draft_tokens[(int64_t)b * gmax + k];
            double rho = q[x] > 0.0 ? ph[x] / q[x] : INFINITY;
            double r = uniforms[(int64_t)b * (gmax + 1) + k];
            double thr = rho < 1.0 ? rho : 1.0;
            if (ratio) ratio[(int64_t)b * gmax + k] = rho;
            if (accept_margin) accept_margin[(int64_t)b * gmax + k] = fabs(thr - r);
            if (n == g && !(r <= thr)) {
                n = k;                   /* first rejection; rows after it are   */
                /* evaluated only to report their ratios                         */
                for (int64_t t = 0; t < V; ++t) {
                    double a = p[t] - ph[t], c = p[t] - q[t];
                    double m = a > c ? a : c;
                    w[t] = m > 0.0 ? m : 0.0;
                }
                double dm = 0.0;
                int64_t tok = draw_inverse_cdf(w, V, uniforms[(int64_t)b * (gmax + 1) + gmax], &dm);
                if (tok < 0)             /* empty residual: fall back to p       */
                    tok = draw_inverse_cdf(p, V, uniforms[(int64_t)b * (gmax + 1) + gmax], &dm);
                toks[k] = (int32_t)tok;
                if (draw_margin) draw_margin[b] = dm;
                if (!ratio && !accept_margin) break;
            }
        }
        for (int k = 0; k < n; ++k) toks[k] = draft_tokens[(int64_t)b * gmax + k];
        if (n == g) {                    /* every draft accepted: bonus from p   */
            const float* zr = target_logits + ((int64_t)b * (gmax + 1) + g) * V;
            for (int64_t t = 0; t < V; ++t) z[t] = zr[t];
            softmax_T(z, T, V, p);
            double dm = 0.0;
            int64_t tok = draw_inverse_cdf(p, V, uniforms[(int64_t)b * (gmax + 1) + gmax], &dm);
            toks[g] = (int32_t)tok;
            if (draw_margin) draw_margin[b] = dm;
        }
        n_accepted[b] = n;
        free(z); free(zq); free(p); free(q); free(ph); free(w);
    }
    return 0;
}


/*
 * The greedy limit T -> 0 of the validation loop (the paper runs T = 0.1 on one of its
 * benchmarks, Appendix C; at T = 0 the softmaxes of Alg. 1 are no longer defined and the
 * limit is taken instead).  With m = max_v z_v and m_q = max_v zq_v, as T -> 0:
 *   p -> one-hot on argmax z, q -> one-hot on argmax zq, zh = z + eta T (q - p) -> z, so
 *   ph -> p and the tail rule changes nothing;
 *   ph(x')/q(x') = exp(((z_x' - m) - (zq_x' - m_q)) / T) * (bounded factor)
 *        -> infinity if the target's gap z_x' - m is above the drafter's gap zq_x' - m_q,
 *        -> 0 if it is below, -> 1 if the gaps are equal (both 0 when x' is the arg-max of both);
 *   the residual max(p - ph, p - q, 0) -> p - q, positive only on argmax z (when the two
 *   arg-maxima differ), and empty otherwise, where the rule falls back to p: either way the
 *   token emitted on a rejection is argmax z of that row; the bonus token is argmax z of row g.
 *   (This is the limit for a draft that is the drafter's own arg-max, which is what a drafter
 *   emits at T -> 0.  For a rejected draft that is not, the literal limit of the residual also
 *   depends on the runner-up gaps of both rows; such ids have probability 0 under q and the rule
 *   here still emits argmax z.)
 * Equal maxima: the lowest index counts as the arg-max (a convention; ties have probability 0
 * for continuous logits).  The accept test stays the literal r <= min(1, ratio limit).
 * eta and tail_alpha do not enter.  ratio: the limit (0, 1 or infinity); accept_margin as in
 * oracle_accept.  No uniform drives the draw.
 */
int oracle_accept_greedy(int B, int gmax, int64_t V,
                         const float* target_logits, const float* draft_logits,
                         const int32_t* draft_tokens, const int32_t* gammas,
                         const float* uniforms,
                         int32_t* n_accepted, int32_t* out_tokens,
                         double* ratio, double* accept_margin)
{
    if (B < 0 || gmax < 0 || V <= 0) return -1;
    for (int b = 0; b < B; ++b) {
        int g = gammas ? gammas[b] : gmax;
        if (g < 0 || g > gmax) return -1;
        for (int k = 0; k < g; ++k) {
            int32_t x = draft_tokens[(int64_t)b * gmax + k];
            if (x < 0 || x >= V) return -1;
        }
    }
    for (int b = 0; b < B; ++b) {
        const int g = gammas ? gammas[b] : gmax;
        int32_t* toks = out_tokens + (int64_t)b * (gmax + 1);
        for (int k = 0; k <= gmax; ++k) toks[k] = -1;
        int n = g;
        for (int k = 0; k < g; ++k) {
            const float* z  = target_logits + ((int64_t)b * (gmax + 1) + k) * V;
            const float* zq = draft_logits + ((int64_t)b * gmax + k) * V;
            double m = -INFINITY, mq = -INFINITY;
            for (int64_t v = 0; v < V; ++v) { if (z[v] > m) m = z[v]; if (zq[v] > mq) mq = zq[v]; }
            const int32_t x = draft_tokens[(int64_t)b * gmax + k];
            const double gap_t = (double)z[x] - m, gap_d = (double)zq[x] - mq;
            const double rho = gap_t > gap_d ? INFINITY : (gap_t < gap_d ? 0.0 : 1.0);
            const double r = uniforms[(int64_t)b * (gmax + 1) + k];
            const double thr = rho < 1.0 ? rho : 1.0;
            if (ratio) ratio[(int64_t)b * gmax + k] = rho;
            if (accept_margin) accept_margin[(int64_t)b * gmax + k] = fabs(thr - r);
            if (n == g && !(r <= thr)) n = k;
        }
        for (int k = 0; k < n; ++k) toks[k] = draft_tokens[(int64_t)b * gmax + k];
        /* rejection at row n < g, or the bonus position n = g: the target's arg-max of that row */
        const float* z = target_logits + ((int64_t)b * (gmax + 1) + n) * V;
        int64_t best = 0;
        for (int64_t v = 1; v < V; ++v) if (z[v] > z[best]) best = v;      /* strict: lowest index wins */
        toks[n] = (int32_t)best;
        n_accepted[b] = n;
    }
    return 0;
}


/* ------------------------------------------------------------------ */
/* Output head: z[r][v] = sum_k h[r][k] * W[v][k], bf16 inputs widened   */
/* exactly, accumulated in double in index order.                        */
/*   h bf16 [rows][hidden], w bf16 [vocab][hidden], z double [rows][vocab] */
int oracle_lm_head(int rows, int64_t hidden, int64_t vocab,
                   const uint16_t* h, const uint16_t* w, double* z)
{
    if (rows < 1 || hidden < 1 || vocab < 1 || !h || !w || !z) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < vocab; ++v) {
        for (int r = 0; r < rows; ++r) {
            double acc = 0.0;
            for (int64_t k = 0; k < hidden; ++k)
                acc += bf16_to_double(h[(int64_t)r * hidden + k]) * bf16_to_double(w[v * hidden + k]);
            z[(int64_t)r * vocab + v] = acc;
        }
    }
    return 0;
}

/* Per block c of `chunk` consecutive entries of every row:               */
/*   cmax[r][c] = max_v z[r][v],  csum[r][c] = sum_v exp((z[r][v] - cmax)/T) */
/* (the last block may be short).                                         */
int oracle_chunk_stats(int rows, int64_t vocab, int64_t chunk, double T,
                       const double* z, double* cmax, double* csum)
{
    if (rows < 1 || vocab < 1 || chunk < 1 || !(T > 0.0) || !z || !cmax || !csum) return -1;
    const int64_t nch = (vocab + chunk - 1) / chunk;
    for (int r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < nch; ++c) {
            const int64_t v0 = c * chunk, v1 = v0 + chunk < vocab ? v0 + chunk : vocab;
            double m = -INFINITY;
            for (int64_t v = v0; v < v1; ++v)
                if (z[(int64_t)r * vocab + v] > m) m = z[(int64_t)r * vocab + v];
            double s = 0.0;
            for (int64_t v = v0; v < v1; ++v) s += exp((z[(int64_t)r * vocab + v] - m) / T);
            cmax[r * nch + c] = m;
            csum[r * nch + c] = s;
        }
    }
    return 0;
}


/* ------------------------------------------------------------------ */
/* Cache bookkeeping around one validation round.                       */
/*                                                                      */
/* Append: row i (0 <= i <= gamma_b) of k_new/v_new [B, Qmax, Hkv, d]    */
/* becomes token ctx_lens[b] - (gamma_b+1) + i of sequence b's cache     */
/* (ctx_lens already counts the appended positions).  Nothing else is    */
/* written.                                                              */
int oracle_kv_append(int B, int Qmax, int Hkv, int d,
                     const uint16_t* k_new, const uint16_t* v_new,
                     const int32_t* ctx_lens, const int32_t* gammas, int gamma,
                     const oracle_kv_layout* lay, const int32_t* page_table,
                     uint16_t* k_cache, uint16_t* v_cache)
{
    if (B < 1 || Qmax < 1 || Hkv < 1 || d < 1 || !k_new || !v_new || !ctx_lens || !lay || !k_cache || !v_cache)
        return -1;
    for (int b = 0; b < B; ++b) {
        const int g = gammas ? gammas[b] : gamma;
        const int Q = g + 1;
        if (g < 0 || Q > Qmax || ctx_lens[b] < Q) return -2;
        for (int i = 0; i < Q; ++i) {
            const int64_t tok = (int64_t)ctx_lens[b] - Q + i;
            for (int h = 0; h < Hkv; ++h) {
                const int64_t dst = kv_offset(lay, page_table, b, tok, h);
                const int64_t src = (((int64_t)b * Qmax + i) * Hkv + h) * d;
                for (int c = 0; c < d; ++c) {
                    k_cache[dst + c] = k_new[src + c];
                    v_cache[dst + c] = v_new[src + c];
                }
            }
        }
    }
    return 0;
}

/* Commit: of the gamma_b+1 verification positions the cache keeps the    */
/* committed token and the n_b accepted drafts:                           */
/*     ctx_lens[b] <- ctx_lens[b] - (gamma_b + 1) + (1 + n_b)              */
int oracle_kv_commit(int B, const int32_t* gammas, int gamma, const int32_t* n_accepted, int32_t* ctx_lens)
{
    if (B < 1 || !n_accepted || !ctx_lens) return -1;
    for (int b = 0; b < B; ++b) {
        const int g = gammas ? gammas[b] : gamma;
        if (n_accepted[b] < 0 || n_accepted[b] > g || ctx_lens[b] < g + 1) return -2;
        ctx_lens[b] = ctx_lens[b] - (g + 1) + (1 + n_accepted[b]);
    }
    return 0;
}


/* Commit for a paged cache, with the allocator's view of the roll-back:  */
/* after the length update above, the page-table slots j of sequence b    */
/* with ceil(L_new / page) <= j < ceil(L_old / page) hold nothing the     */
/* sequence keeps (only rejected verification positions lived there);     */
/* their page ids are listed in ascending slot order, the row padded      */
/* with -1.  released: int32 [B][cap], n_released: int32 [B].             */
int oracle_kv_commit_pages(int B, const int32_t* gammas, int gamma, const int32_t* n_accepted,
                           const int32_t* page_table, int max_pages, int page_size,
                           int32_t* ctx_lens, int32_t* released, int cap, int32_t* n_released)
{
    if (B < 1 || !n_accepted || !ctx_lens || !page_table || !released || !n_released || page_size < 1 || cap < 0)
        return -1;
    for (int b = 0; b < B; ++b) {
        const int g = gammas ? gammas[b] : gamma;
        if (n_accepted[b] < 0 || n_accepted[b] > g || ctx_lens[b] < g + 1) return -2;
        const int l_old = ctx_lens[b];
        const int l_new = l_old - (g + 1) + (1 + n_accepted[b]);
        int cnt = 0;
        for (int j = 0; j < max_pages; ++j) {
            /* slot j covers tokens j*page .. j*page + page - 1 */
            const int used_before = j * page_size < l_old;
            const int used_after = j * page_size < l_new;
            if (used_before && !used_after) {
                if (cnt >= cap) return -3;
                released[(int64_t)b * cap + cnt++] = page_table[(int64_t)b * max_pages + j];
            }
        }
        n_released[b] = cnt;
        for (int j = cnt; j < cap; ++j) released[(int64_t)b * cap + j] = -1;
        ctx_lens[b] = l_new;
    }
    return 0;
}


/* ------------------------------------------------------------------ */
/* Chunk budget of the drafter's context ("RAG Setup", Sec. 3): the      */
/* retrieved context is at least 4096 tokens and otherwise 1/24 of the   */
/* input, counted in whole chunks of chunk_tokens tokens.                */
int oracle_retrieval_top_k(int64_t ctx_tokens, int chunk_tokens)
{
    if (ctx_tokens < 0 || chunk_tokens < 1) return -1;
    int64_t budget = ctx_tokens / 24;
    if (budget < 4096) budget = 4096;
    return (int)(budget / chunk_tokens);
}

/* Retrieval: which chunks of the long context the drafter gets.        */
/*   emb   float [n][dim] chunk embeddings, query float [dim]            */
/*   sim[i] = <emb_i, query> / (|emb_i| |query|), 0 if either norm is 0  */
/*   keep the top_k chunks by similarity (equal values: lower index      */
/*   first), drop those with sim < threshold, report the rest in         */
/*   ascending index order.  margin = smallest distance of any           */
/*   similarity to a decision boundary (the k-th/k+1-th values and the   */
/*   threshold): callers use it to recognise near-ties.                  */
int oracle_retrieve(int n, int dim, const float* emb, const float* query, int top_k, double threshold,
                    double* sim, int32_t* selected, int32_t* n_selected, double* margin)
{
    if (n < 1 || dim < 1 || top_k < 0 || !emb || !query || !sim || !selected || !n_selected) return -1;
    double qn = 0.0;
    for (int c = 0; c < dim; ++c) qn += (double)query[c] * (double)query[c];
    qn = sqrt(qn);
    for (int i = 0; i < n; ++i) {
        double dot = 0.0, en = 0.0;
        for (int c = 0; c < dim; ++c) {
            dot += (double)emb[(int64_t)i * dim + c] * (double)query[c];
            en += (double)emb[(int64_t)i * dim + c] * (double)emb[(int64_t)i * dim + c];
        }
        en = sqrt(en);
        sim[i] = (en > 0.0 && qn > 0.0) ? dot / (en * qn) : 0.0;
    }
    /* rank of chunk i = number of chunks that come before it in the order   */
    /* "larger similarity first, lower index first among equals"             */
    int count = 0;
    double mg = INFINITY, kth = -INFINITY, next = -INFINITY;
    for (int i = 0; i < n; ++i) {
        int rank = 0;
        for (int j = 0; j < n; ++j)
            if (sim[j] > sim[i] || (sim[j] == sim[i] && j < i)) ++rank;
        if (rank == top_k - 1) kth = sim[i];
        if (rank == top_k) next = sim[i];
        if (rank < top_k && sim[i] >= threshold) selected[count++] = i;   /* i ascending: document order */
        if (fabs(sim[i] - threshold) < mg) mg = fabs(sim[i] - threshold);
    }
    if (top_k >= 1 && top_k < n && kth - next < mg) mg = kth - next;
    *n_selected = count;
    if (margin) *margin = mg;
    return 0;
}
