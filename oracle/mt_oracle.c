/*
 * CPU oracle for the serving forward pass of a merged multi-task (MT) BERT model.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition the GPU library is checked
 * against; it is never part of a product path and shares no code with the GPU sources.
 *
 * What it computes (paper Section 3.3 "Model Merging" and Fig. 1(c)): the single-task student
 * models are merged into one graph so that their frozen bottom layers are evaluated once.  The
 * merged model therefore returns, for every task t, exactly the logits of student t run on its
 * own: embeddings, the first x_t shared layers, the task's y_t own layers, a pooler and a head.
 * Both forms are written out here:
 *   orc_mt_forward  - trunk once, each task continues from the hidden state after layer x_t;
 *   orc_st_forward  - student t alone, from the embeddings up, sharing nothing with the above.
 * The paper's cost measure (Section 4.1, the "Overhead" column of Table 2) is orc_overhead().
 *
 * The paper defers the layer arithmetic to BERT ("12-layer uncased", Section 3).  The readings
 * used here, each a public definition:
 *   - embeddings: word[id] + position[s] + type[0], then LayerNorm;
 *   - encoder layer, post-LN: X1 = LN(X + MHA(X) Wo^T + bo), X' = LN(X1 + gelu(X1 W1^T + b1) W2^T + b2);
 *   - attention scores (q.k)/sqrt(d) plus -10000 on masked keys, softmax with max subtraction;
 *   - LayerNorm with biased variance, eps inside the square root;
 *   - GELU x*Phi(x) with the exact erf form (tanh form selectable);
 *   - pooler tanh(Wp h[first token] + bp), head Wc p + bc, raw logits returned.
 *
 * Precision: every stored tensor is float32; every output element is computed in float64 from
 * float32 inputs (dot products, means, variances, softmax sums all accumulate in float64) and is
 * rounded to float32 once.  Loops are the textbook ones: no blocking, no fusion.  OpenMP only
 * spreads the outermost independent loop over threads.
 *
 * Parameter vectors are flat float32 arrays in this order (every linear is W[out][in], y = W x + b):
 *   trunk: word_emb[V,H] pos_emb[P,H] type_emb[TV,H] emb_ln_g[H] emb_ln_b[H], then per layer
 *          Wq bq Wk bk Wv bv Wo bo ln1_g ln1_b W1[F,H] b1[F] W2[H,F] b2[H] ln2_g ln2_b
 *   task : y_t layers in the same order, then Wp[H,H] bp[H] Wc[C,H] bc[C]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t vocab, hidden, heads, ffn, max_pos, type_vocab;
    int32_t n_trunk_layers;
    int32_t n_tasks;
    int32_t gelu_tanh;   /* 0: exact erf form; 1: tanh approximation */
    float   ln_eps;
} orc_config;

typedef struct {
    int32_t fork_layer;  /* x_t */
    int32_t n_layers;    /* y_t */
    int32_t n_classes;   /* C_t */
    int32_t token_level; /* 0: pooler + head on the first token; 1: a linear head on every token, no pooler */
} orc_task;

#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
void orc_set_num_threads(int n) { if (n >= 1) omp_set_num_threads(n); }
#else
int orc_num_threads(void) { return 1; }
void orc_set_num_threads(int n) { (void)n; }
#endif

/* ---------------------------------------------------------------- elementary operations */

/* y[m][n] = sum_k x[m][k] * W[n][k] + b[n]   (b may be NULL) */
void orc_linear(const float *x, int64_t M, int64_t K, const float *W, const float *b, int64_t N, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *xr = x + m * K;
        for (int64_t n = 0; n < N; ++n) {
            const float *wr = W + n * K;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t k = 0; k < K; ++k)
                acc += (double)xr[k] * (double)wr[k];
            if (b) acc += (double)b[n];
            y[m * N + n] = (float)acc;
        }
    }
}

/* y[m][:] = gamma * (v - mean(v)) / sqrt(var(v) + eps) + beta, v = x[m][:] (+ r[m][:] if r) */
void orc_layernorm(const float *x, const float *r, int64_t M, int64_t H,
                   const float *gamma, const float *beta, float eps, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *xr = x + m * H;
        const float *rr = r ? r + m * H : NULL;
        double mean = 0.0;
        for (int64_t i = 0; i < H; ++i)
            mean += (double)xr[i] + (rr ? (double)rr[i] : 0.0);
        mean /= (double)H;
        double var = 0.0;
        for (int64_t i = 0; i < H; ++i) {
            double d = (double)xr[i] + (rr ? (double)rr[i] : 0.0) - mean;
            var += d * d;
        }
        var /= (double)H;
        double inv = 1.0 / sqrt(var + (double)eps);
        for (int64_t i = 0; i < H; ++i) {
            double v = (double)xr[i] + (rr ? (double)rr[i] : 0.0);
            y[m * H + i] = (float)((double)gamma[i] * ((v - mean) * inv) + (double)beta[i]);
        }
    }
}

/* GELU(x) = x * Phi(x) */
float orc_gelu(float x, int tanh_form)
{
    double v = (double)x;
    if (tanh_form) {
        double u = 0.7978845608028654 * (v + 0.044715 * v * v * v);   /* sqrt(2/pi) */
        return (float)(0.5 * v * (1.0 + tanh(u)));
    }
    return (float)(0.5 * v * (1.0 + erf(v * 0.7071067811865476)));
}

void orc_gelu_array(const float *x, int64_t n, int tanh_form, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = orc_gelu(x[i], tanh_form);
}

/* p = softmax(s) over n entries with max subtraction */
void orc_softmax_row(const float *s, int64_t n, float *p)
{
    float mx = s[0];
    for (int64_t j = 1; j < n; ++j) if (s[j] > mx) mx = s[j];
    double sum = 0.0;
    for (int64_t j = 0; j < n; ++j) sum += exp((double)(s[j] - mx));
    for (int64_t j = 0; j < n; ++j) p[j] = (float)(exp((double)(s[j] - mx)) / sum);
}

/*
 * Multi-head scaled dot-product attention with a key padding mask.
 * q, k, v, ctx: [B][S][H] with head a occupying columns a*d .. a*d+d-1; mask: [B][S], 1 = real token.
 * probs (optional, may be NULL): [B][A][S][S] attention weights.
 */
void orc_attention(const float *q, const float *k, const float *v, const int32_t *mask,
                   int64_t B, int64_t S, int64_t H, int64_t A, float *ctx, float *probs)
{
    const int64_t d = H / A;
    const float scale = 1.0f / sqrtf((float)d);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t a = 0; a < A; ++a) {
            float *s = (float *)malloc(sizeof(float) * (size_t)S);
            float *p = (float *)malloc(sizeof(float) * (size_t)S);
            for (int64_t i = 0; i < S; ++i) {
                const float *qi = q + (b * S + i) * H + a * d;
                for (int64_t j = 0; j < S; ++j) {
                    const float *kj = k + (b * S + j) * H + a * d;
                    double acc = 0.0;
                    for (int64_t c = 0; c < d; ++c) acc += (double)qi[c] * (double)kj[c];
                    float sc = (float)acc * scale;
                    if (!mask[b * S + j]) sc += -10000.0f;
                    s[j] = sc;
                }
                orc_softmax_row(s, S, p);
                if (probs) memcpy(probs + ((b * A + a) * S + i) * S, p, sizeof(float) * (size_t)S);
                for (int64_t c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int64_t j = 0; j < S; ++j)
                        acc += (double)p[j] * (double)v[(b * S + j) * H + a * d + c];
                    ctx[(b * S + i) * H + a * d + c] = (float)acc;
                }
            }
            free(s);
            free(p);
        }
    }
}

/* ---------------------------------------------------------------- parameter bookkeeping */

int64_t orc_layer_param_count(int64_t H, int64_t F)
{
    return 4 * (H * H + H) + 2 * H + (F * H + F) + (H * F + H) + 2 * H;
}

int64_t orc_trunk_param_count(const orc_config *c)
{
    int64_t H = c->hidden;
    return ((int64_t)c->vocab + c->max_pos + c->type_vocab) * H + 2 * H
         + (int64_t)c->n_trunk_layers * orc_layer_param_count(H, c->ffn);
}

int64_t orc_task_param_count(const orc_config *c, const orc_task *t)
{
    int64_t H = c->hidden;
    return (int64_t)t->n_layers * orc_layer_param_count(H, c->ffn) + (t->token_level ? 0 : H * H + H)
         + (int64_t)t->n_classes * H + t->n_classes;
}

typedef struct {
    const float *Wq, *bq, *Wk, *bk, *Wv, *bv, *Wo, *bo, *ln1_g, *ln1_b, *W1, *b1, *W2, *b2, *ln2_g, *ln2_b;
} layer_params;

static layer_params slice_layer(const float *p, int64_t H, int64_t F)
{
    layer_params L;
    L.Wq = p; p += H * H;  L.bq = p; p += H;
    L.Wk = p; p += H * H;  L.bk = p; p += H;
    L.Wv = p; p += H * H;  L.bv = p; p += H;
    L.Wo = p; p += H * H;  L.bo = p; p += H;
    L.ln1_g = p; p += H;   L.ln1_b = p; p += H;
    L.W1 = p; p += F * H;  L.b1 = p; p += F;
    L.W2 = p; p += H * F;  L.b2 = p; p += H;
    L.ln2_g = p; p += H;   L.ln2_b = p;
    return L;
}

/* ---------------------------------------------------------------- model pieces */

/* X0[b][s][:] = LN(word_emb[ids[b][s]] + pos_emb[s] + type_emb[0]) */
/* Embeddings with per-token segment ids: word[id] + pos[s] + type[type_ids[b][s]], then LayerNorm.
 * type_ids == NULL means segment 0 everywhere (single-sentence inputs). */
void orc_embed_typed(const orc_config *c, const float *trunk, const int32_t *ids, const int32_t *type_ids, int64_t B, int64_t S,
                     float *X0);

void orc_embed(const orc_config *c, const float *trunk, const int32_t *ids, int64_t B, int64_t S, float *X0)
{
    orc_embed_typed(c, trunk, ids, NULL, B, S, X0);
}

void orc_embed_typed(const orc_config *c, const float *trunk, const int32_t *ids, const int32_t *type_ids, int64_t B, int64_t S,
                     float *X0)
{
    const int64_t H = c->hidden;
    const float *word = trunk;
    const float *pos = word + (int64_t)c->vocab * H;
    const float *type = pos + (int64_t)c->max_pos * H;
    const float *g = type + (int64_t)c->type_vocab * H;
    const float *bt = g + H;
    float *e = (float *)malloc(sizeof(float) * (size_t)(B * S * H));
    for (int64_t b = 0; b < B; ++b)
        for (int64_t s = 0; s < S; ++s)
            for (int64_t i = 0; i < H; ++i)
                e[(b * S + s) * H + i] = (float)((double)word[(int64_t)ids[b * S + s] * H + i]
                                                 + (double)pos[s * H + i]
                                                 + (double)type[(int64_t)(type_ids ? type_ids[b * S + s] : 0) * H + i]);
    orc_layernorm(e, NULL, B * S, H, g, bt, c->ln_eps, X0);
    free(e);
}

/* One post-LN encoder layer.  X, out: [B][S][H]; lp: the layer's parameters in canonical order. */
void orc_encoder_layer(const orc_config *c, const float *lp, const float *X, const int32_t *mask,
                       int64_t B, int64_t S, float *out)
{
    const int64_t H = c->hidden, F = c->ffn, M = B * S;
    layer_params L = slice_layer(lp, H, F);
    float *q = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *k = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *v = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *ctx = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *ao = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *x1 = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *u = (float *)malloc(sizeof(float) * (size_t)(M * F));
    float *fo = (float *)malloc(sizeof(float) * (size_t)(M * H));

    orc_linear(X, M, H, L.Wq, L.bq, H, q);
    orc_linear(X, M, H, L.Wk, L.bk, H, k);
    orc_linear(X, M, H, L.Wv, L.bv, H, v);
    orc_attention(q, k, v, mask, B, S, H, c->heads, ctx, NULL);
    orc_linear(ctx, M, H, L.Wo, L.bo, H, ao);
    orc_layernorm(X, ao, M, H, L.ln1_g, L.ln1_b, c->ln_eps, x1);
    orc_linear(x1, M, H, L.W1, L.b1, F, u);
    orc_gelu_array(u, M * F, c->gelu_tanh, u);
    orc_linear(u, M, F, L.W2, L.b2, H, fo);
    orc_layernorm(x1, fo, M, H, L.ln2_g, L.ln2_b, c->ln_eps, out);

    free(q); free(k); free(v); free(ctx); free(ao); free(x1); free(u); free(fo);
}

/* Task head: p = tanh(Wp Z[b][0][:] + bp); logits[b][:] = Wc p + bc.  hp points at Wp. */
void orc_head(const orc_config *c, const float *hp, int n_classes, const float *Z, int64_t B, int64_t S,
              float *logits, int64_t ld_logits)
{
    const int64_t H = c->hidden;
    const float *Wp = hp, *bp = Wp + H * H, *Wc = bp + H, *bc = Wc + (int64_t)n_classes * H;
    float *first = (float *)malloc(sizeof(float) * (size_t)(B * H));
    float *pool = (float *)malloc(sizeof(float) * (size_t)(B * H));
    float *lg = (float *)malloc(sizeof(float) * (size_t)(B * n_classes));
    for (int64_t b = 0; b < B; ++b) memcpy(first + b * H, Z + b * S * H, sizeof(float) * (size_t)H);
    orc_linear(first, B, H, Wp, bp, H, pool);
    for (int64_t i = 0; i < B * H; ++i) pool[i] = (float)tanh((double)pool[i]);
    orc_linear(pool, B, H, Wc, bc, n_classes, lg);
    for (int64_t b = 0; b < B; ++b)
        for (int j = 0; j < n_classes; ++j) logits[b * ld_logits + j] = lg[b * n_classes + j];
    free(first); free(pool); free(lg);
}

/*
 * Token-level head (tagging tasks such as entity recognition and slot filling, which Appendix E lists among the
 * deployed tasks): every position's final hidden state goes through one linear layer, as in BERT's token
 * classification set-up; there is no pooler.  logits[(b*S+s)*ld + j] = Wc[j] . Z[b][s] + bc[j], for every
 * position, padded ones included.  hp points at Wc.
 */
void orc_token_head(const orc_config *c, const float *hp, int n_classes, const float *Z, int64_t B, int64_t S,
                    float *logits, int64_t ld_logits)
{
    const int64_t H = c->hidden, M = B * S;
    const float *Wc = hp, *bc = Wc + (int64_t)n_classes * H;
    float *lg = (float *)malloc(sizeof(float) * (size_t)(M * n_classes));
    orc_linear(Z, M, H, Wc, bc, n_classes, lg);
    for (int64_t r = 0; r < M; ++r)
        for (int j = 0; j < n_classes; ++j) logits[r * ld_logits + j] = lg[r * n_classes + j];
    free(lg);
}

/* Total transformer layers evaluated per request: max_t x_t + sum_t y_t (Section 4.1). */
int orc_overhead(const orc_task *tasks, int n_tasks)
{
    int shared = 0, own = 0;
    for (int t = 0; t < n_tasks; ++t) {
        if (tasks[t].fork_layer > shared) shared = tasks[t].fork_layer;
        own += tasks[t].n_layers;
    }
    return shared + own;
}

/*
 * Merged model.  logits: [B][sum of C_t over sequence-level tasks]; token_logits: [B][S][sum of C_t over token-level
 * tasks] (may be NULL when there is no such task).  Inside its row a task's columns start at the sum of C_u over
 * the earlier tasks u of the same kind.
 * hidden_out (optional): [n_trunk_layers+1][B][S][H], the embeddings followed by every trunk layer output.
 * Returns 0, or -1 on an invalid task table or a missing output buffer.
 */
int orc_mt_forward_tokens(const orc_config *c, const orc_task *tasks, const float *trunk, const float *const *task_params,
                          const int32_t *ids, const int32_t *type_ids, const int32_t *mask, int64_t B, int64_t S, float *logits,
                          float *token_logits, float *hidden_out);

int orc_mt_forward_typed(const orc_config *c, const orc_task *tasks, const float *trunk, const float *const *task_params,
                         const int32_t *ids, const int32_t *type_ids, const int32_t *mask, int64_t B, int64_t S, float *logits,
                         float *hidden_out);

int orc_mt_forward(const orc_config *c, const orc_task *tasks, const float *trunk, const float *const *task_params,
                   const int32_t *ids, const int32_t *mask, int64_t B, int64_t S, float *logits, float *hidden_out)
{
    return orc_mt_forward_typed(c, tasks, trunk, task_params, ids, NULL, mask, B, S, logits, hidden_out);
}

/* The same with segment ids (NULL = all 0); values must lie in [0, type_vocab). */
int orc_mt_forward_typed(const orc_config *c, const orc_task *tasks, const float *trunk, const float *const *task_params,
                         const int32_t *ids, const int32_t *type_ids, const int32_t *mask, int64_t B, int64_t S, float *logits,
                         float *hidden_out)
{
    return orc_mt_forward_tokens(c, tasks, trunk, task_params, ids, type_ids, mask, B, S, logits, NULL, hidden_out);
}

int orc_mt_forward_tokens(const orc_config *c, const orc_task *tasks, const float *trunk, const float *const *task_params,
                          const int32_t *ids, const int32_t *type_ids, const int32_t *mask, int64_t B, int64_t S, float *logits,
                          float *token_logits, float *hidden_out)
{
    const int64_t H = c->hidden, F = c->ffn, MH = B * S * H;
    const int D = c->n_trunk_layers;
    int ctot = 0, ctok = 0;
    for (int t = 0; t < c->n_tasks; ++t) {
        if (tasks[t].fork_layer < 0 || tasks[t].fork_layer > D || tasks[t].n_layers < 0 || tasks[t].n_classes < 1) return -1;
        if (tasks[t].token_level) ctok += tasks[t].n_classes;
        else ctot += tasks[t].n_classes;
    }
    if ((ctot > 0 && !logits) || (ctok > 0 && !token_logits)) return -1;
    const float *layers = trunk + ((int64_t)c->vocab + c->max_pos + c->type_vocab) * H + 2 * H;
    const int64_t lsz = orc_layer_param_count(H, F);

    float *taps = (float *)malloc(sizeof(float) * (size_t)(MH * (D + 1)));   /* X^(0..D) */
    orc_embed_typed(c, trunk, ids, type_ids, B, S, taps);
    for (int l = 0; l < D; ++l)
        orc_encoder_layer(c, layers + l * lsz, taps + (int64_t)l * MH, mask, B, S, taps + (int64_t)(l + 1) * MH);
    if (hidden_out) memcpy(hidden_out, taps, sizeof(float) * (size_t)(MH * (D + 1)));

    float *za = (float *)malloc(sizeof(float) * (size_t)MH);
    float *zb = (float *)malloc(sizeof(float) * (size_t)MH);
    int col = 0, tcol = 0;
    for (int t = 0; t < c->n_tasks; ++t) {
        const float *z = taps + (int64_t)tasks[t].fork_layer * MH;
        for (int l = 0; l < tasks[t].n_layers; ++l) {
            float *dst = (l % 2 == 0) ? za : zb;
            orc_encoder_layer(c, task_params[t] + l * lsz, z, mask, B, S, dst);
            z = dst;
        }
        const float *hp = task_params[t] + (int64_t)tasks[t].n_layers * lsz;
        if (tasks[t].token_level) {
            orc_token_head(c, hp, tasks[t].n_classes, z, B, S, token_logits + tcol, ctok);
            tcol += tasks[t].n_classes;
        } else {
            orc_head(c, hp, tasks[t].n_classes, z, B, S, logits + col, ctot);
            col += tasks[t].n_classes;
        }
    }
    free(za); free(zb); free(taps);
    return 0;
}

/* Student model of one task on its own.  logits: [B][C_t], or [B][S][C_t] for a token-level task. */
int orc_st_forward_typed(const orc_config *c, const orc_task *task, const float *trunk, const float *task_param,
                         const int32_t *ids, const int32_t *type_ids, const int32_t *mask, int64_t B, int64_t S, float *logits);

int orc_st_forward(const orc_config *c, const orc_task *task, const float *trunk, const float *task_param,
                   const int32_t *ids, const int32_t *mask, int64_t B, int64_t S, float *logits)
{
    return orc_st_forward_typed(c, task, trunk, task_param, ids, NULL, mask, B, S, logits);
}

int orc_st_forward_typed(const orc_config *c, const orc_task *task, const float *trunk, const float *task_param,
                         const int32_t *ids, const int32_t *type_ids, const int32_t *mask, int64_t B, int64_t S, float *logits)
{
    const int64_t H = c->hidden, F = c->ffn, MH = B * S * H;
    if (task->fork_layer < 0 || task->fork_layer > c->n_trunk_layers || task->n_layers < 0 || task->n_classes < 1) return -1;
    const float *layers = trunk + ((int64_t)c->vocab + c->max_pos + c->type_vocab) * H + 2 * H;
    const int64_t lsz = orc_layer_param_count(H, F);
    float *xa = (float *)malloc(sizeof(float) * (size_t)MH);
    float *xb = (float *)malloc(sizeof(float) * (size_t)MH);
    orc_embed_typed(c, trunk, ids, type_ids, B, S, xa);
    float *cur = xa, *nxt = xb;
    for (int l = 0; l < task->fork_layer; ++l) {
        orc_encoder_layer(c, layers + l * lsz, cur, mask, B, S, nxt);
        float *tmp = cur; cur = nxt; nxt = tmp;
    }
    for (int l = 0; l < task->n_layers; ++l) {
        orc_encoder_layer(c, task_param + l * lsz, cur, mask, B, S, nxt);
        float *tmp = cur; cur = nxt; nxt = tmp;
    }
    if (task->token_level)
        orc_token_head(c, task_param + (int64_t)task->n_layers * lsz, task->n_classes, cur, B, S, logits, task->n_classes);
    else
        orc_head(c, task_param + (int64_t)task->n_layers * lsz, task->n_classes, cur, B, S, logits, task->n_classes);
    free(xa); free(xb);
    return 0;
}
