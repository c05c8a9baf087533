/*
 * mt.h - C ABI of the MI355X (gfx950) serving library for merged multi-task BERT models.
 *
 * The model is the "final multi-task model" of the paper's Fig. 1(c) / Section 3.3 (Model Merging):
 * single-task students that share frozen bottom encoder layers are loaded into ONE graph, so the
 * shared layers (the trunk) run once per batch and every task continues from the trunk layer it
 * forked at with its own few distilled layers, a pooler and a classifier.  One call returns the
 * logits of all enabled tasks (Section 5.2: no task's output is available before all are computed).
 *
 * Conventions
 *   - Every function returns MT_OK (0) or a negative MT_ERR_* code; nothing throws or aborts across
 *     this boundary.  mt_last_error() gives a text for the most recent failure on that model.
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller owns all buffers:
 *     token ids, masks, logits, the weight arena and the workspace arena.  The library owns only
 *     host-side metadata inside mt_model.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  mt_forward only
 *     enqueues work on it: it never synchronises, never allocates, never frees.
 *   - All argument checks are done on the host before anything is enqueued.
 *   - Linear layers are y = W x + b with W stored [out][in] row-major.
 */
#ifndef MT_H_
#define MT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MT_ABI_VERSION 2u

enum {
    MT_OK = 0,
    MT_ERR_NULL = -1,    /* a required pointer is NULL */
    MT_ERR_CONFIG = -2,  /* inconsistent or unsupported configuration */
    MT_ERR_SHAPE = -3,   /* batch / seq / buffer size outside what the model was created or bound for */
    MT_ERR_STATE = -4,   /* call order: forward before bind/load, load before bind, ... */
    MT_ERR_BLOB = -5,    /* malformed weight blob */
    MT_ERR_HIP = -6      /* a HIP runtime call failed */
};

enum { MT_BF16 = 0, MT_FP32_CHECK = 1, MT_FP8_FFN = 2, MT_FP8_LAYER = 3 };     /* mt_config.precision */
enum { MT_GELU_ERF = 0, MT_GELU_TANH = 1 };  /* mt_config.gelu */
enum { MT_HEAD_SEQUENCE = 0, MT_HEAD_TOKEN = 1 };  /* mt_task_desc.head */

typedef struct mt_model mt_model; /* opaque, library-owned host object */

/*
 * One task of the merged model: the (x, y) tuple printed under Table 2 plus its output width.
 *   fork_layer  x_t: the task reads the trunk's hidden state after this many shared layers
 *               (0 = directly after the embeddings); 0 <= x_t <= n_trunk_layers.
 *   n_layers    y_t >= 0 task-specific encoder layers.
 *   n_classes   C_t >= 1 logits (1 = regression output, returned unchanged).
 *   head        MT_HEAD_SEQUENCE: tanh pooler on the first token, then a linear classifier: one row of C_t
 *               logits per sequence (the GLUE-style tasks of Section 4).
 *               MT_HEAD_TOKEN: one linear classifier applied to every token's final hidden state, no pooler:
 *               C_t logits per position (the tagging tasks - entity recognition, slot filling - that
 *               Appendix E lists among the deployed tasks).
 */
typedef struct {
    int32_t fork_layer;
    int32_t n_layers;
    int32_t n_classes;
    int32_t head;
} mt_task_desc;

/*
 * Model description.  struct_size/version guard the layout (sizeof(mt_config), MT_ABI_VERSION).
 * n_trunk_layers must equal max_t fork_layer (the shared depth of the "Layers" column of Table 2).
 * precision MT_BF16: matrices and embedding tables are stored as bfloat16 (round to nearest even
 * from the float32 blob), contractions run on bf16 matrix cores with float32 accumulation; it needs
 * hidden/heads == 64, hidden % 64 == 0, ffn % 64 == 0 and max_seq <= 608 (the attention kernel keeps one
 * sequence's keys and values of a head in the 160 KB LDS).  MT_FP32_CHECK: everything float32 on
 * the vector ALUs, any shape, max_seq <= 4096, meant for validation.
 * MT_FP8_FFN: MT_BF16 with the two feed-forward contractions of every layer that is evaluated on all token rows run
 * in OCP FP8 E4M3 on the FP8 matrix cores (float32 accumulation); a reduced-precision serving variant in the spirit of
 * the deployment note of Appendix E (half precision there).  Every feed-forward matrix W is additionally stored as
 * E4M3(s W) with s the largest power of two that keeps s max|W| <= 448, undone exactly in the epilogue; the
 * LayerNorm output that feeds the first contraction and the GELU output that feeds the second are rounded to E4M3
 * (unit scale, saturating at +-448) instead of bfloat16.  Everything else, including the first-token-only last
 * layer of every branch, is as in MT_BF16.  Needs hidden >= 192 and ffn >= 192 on top of MT_BF16's conditions.
 * MT_FP8_LAYER: MT_FP8_FFN with the other two contractions of such a layer in E4M3 as well: the query/key/value
 * projection (the three matrices stored as one [3H, H] matrix under ONE storage scale; its operand is the layer
 * input's bfloat16 copy rounded to E4M3) and the attention output projection (its operand, the attention context, is
 * written as E4M3 by the attention kernel).  Queries, keys, values, the softmax and the float32 residual stream stay as
 * in MT_BF16.
 * max_batch*max_seq bounds the workspace; max_seq <= max_pos.
 */
typedef struct {
    uint32_t struct_size, version;
    int32_t vocab, hidden, heads, ffn, max_pos, type_vocab;
    int32_t n_trunk_layers;
    int32_t n_tasks;
    const mt_task_desc* tasks; /* host array [n_tasks], copied by mt_create */
    int32_t precision;
    int32_t gelu;
    float ln_eps;
    int32_t max_batch, max_seq;
} mt_config;

/* Validate cfg and build the merged graph's schedule (Section 3.3).  Host only; touches no GPU.
 * On success *out owns a new model (release with mt_destroy).  Errors: NULL, CONFIG. */
int mt_create(const mt_config* cfg, mt_model** out);
void mt_destroy(mt_model* m);

/* Sizes in bytes of the two device arenas the caller must provide to mt_bind. */
size_t mt_weight_bytes(const mt_model* m);
size_t mt_workspace_bytes(const mt_model* m);

/* Attach caller-owned device memory.  Both pointers must be 256-byte aligned and at least as large
 * as the sizes above; they must stay valid until mt_destroy.  Errors: NULL, SHAPE. */
int mt_bind(mt_model* m, void* d_weights, size_t weight_bytes, void* d_workspace, size_t workspace_bytes);

/*
 * Serving replicas (the merged model of Section 3.3 is stateless across batches: weights are only read).
 * `m` must have been created from a configuration equal to `owner`'s and bound to the SAME weight arena
 * with a workspace of its own; it then takes over `owner`'s loaded state without copying anything.
 * mt_forward calls on `m` and on `owner` may then be in flight at the same time on different streams
 * (each writes only its own workspace and its caller's logits), which lets one batch's kernels fill the
 * compute units another batch's kernels leave idle.  Loading weights into either handle afterwards is
 * visible to both arenas-wise, but only the loading handle's state is updated: call mt_share_weights
 * again.  Host only.  Errors: NULL, CONFIG (configurations differ), STATE (not bound to the same
 * weight arena, or owner has nothing loaded).
 */
int mt_share_weights(mt_model* m, const mt_model* owner);

/*
 * Merge one checkpoint into the shared graph (Section 3.3, Model Merging).  scope -1 = embeddings + trunk layers, scope t >= 0 = task t's
 * layers, pooler and classifier; loading one task never touches another's memory (the per-task
 * update of Section 5.1).  h_blob is a little-endian HOST buffer:
 *     char magic[4] = "MTW1"; int32 scope; int32 n_tensors; int32 reserved(0);  then float32 data
 *   trunk scope: word_emb[V,H] pos_emb[P,H] type_emb[TV,H] emb_ln_g[H] emb_ln_b[H], then per layer
 *     Wq[H,H] bq[H] Wk bk Wv bv Wo[H,H] bo ln1_g ln1_b W1[F,H] b1[F] W2[H,F] b2[H] ln2_g ln2_b
 *   task scope : y_t layers in that order, then Wp[H,H] bp[H] Wc[C,H] bc[C]
 *                (MT_HEAD_TOKEN: y_t layers, then Wc[C,H] bc[C] only)
 * The call converts on the host, copies on `hip_stream` and waits for the copy, so h_blob may be
 * released on return.  The copy is ordered only against work on `hip_stream`: a forward pass that reads this scope
 * on another stream (a replica's, say) must have finished, or must have the task masked off, while its weights are
 * replaced.  Errors: NULL, STATE (not bound), BLOB (magic/scope/size mismatch), HIP.
 */
int mt_load_weights(mt_model* m, int32_t scope, const void* h_blob, size_t nbytes, void* hip_stream);

/*
 * The serving forward pass: embeddings, the shared trunk once, then all enabled tasks' branches as
 * grouped launches, then poolers and classifiers.
 *   d_input_ids [batch][seq] int32, clamped into [0, vocab) by the kernel;
 *   d_attn_mask [batch][seq] int32, 1 = real token, 0 = padding; applied to attention keys only;
 *               position 0 of every sequence must be a real token (the pooler reads it);
 *   h_task_mask host array [n_tasks] of 0/1, or NULL for all tasks.  Disabled tasks are not computed
 *               and their logit columns are left untouched; the trunk runs only as deep as the
 *               deepest enabled fork;
 *   d_out_logits [batch][C_tot] float32 row-major, C_tot = sum of n_classes over the MT_HEAD_SEQUENCE tasks,
 *               task t's columns start at mt_logit_offset(m, t).  Raw logits (no softmax).
 * Hidden states at padded positions are unspecified and never influence a real token.
 * Errors: NULL (also: an enabled task has a token-level head, which needs mt_forward_tokens), STATE (not
 * bound / a needed scope not loaded), SHAPE (batch, seq out of range), HIP.
 */
int mt_forward(mt_model* m, const int32_t* d_input_ids, const int32_t* d_attn_mask, int32_t batch, int32_t seq,
               const uint8_t* h_task_mask, float* d_out_logits, void* hip_stream);

/*
 * Validation of the one precondition the forward passes do not check themselves (they never wait for the device):
 * position 0 of every sequence must be a real token, because a sequence-level task head reads the hidden state
 * of position 0 (Section 3: the students are BERT models).  A sequence whose mask starts with 0 is served from its
 * first REAL token instead, and a sequence without any real token gets unspecified logits; other sequences are never
 * affected.  This call counts such sequences on the device, WAITS for the result, writes the count to
 * *h_bad_sequences and returns MT_OK if it is zero, MT_ERR_SHAPE (with a text) otherwise.  For input pipelines under
 * test, not for the serving loop.  Errors: NULL, STATE (not bound), SHAPE, HIP.
 */
int mt_check_mask(mt_model* m, const int32_t* d_attn_mask, int32_t batch, int32_t seq, int32_t* h_bad_sequences, void* hip_stream);

/*
 * Several request batches in ONE forward pass (dynamic batching across requests: Appendix E's deployment serves a
 * stream of requests, and the merged model is the same function of every sequence whoever sent it).  Request r
 * brings its own device arrays h_d_input_ids[r], h_d_attn_mask[r] ([batch][seq] int32 each) and receives its logits
 * in h_d_out_logits[r] ([batch][C_tot] float32); the three tables are HOST arrays of n_requests device pointers,
 * read before the call returns.  The library copies the ids and masks behind one another into its workspace, runs
 * the trunk and all branches once over the n_requests * batch sequences (every contraction then has n_requests
 * times the rows, which is what fills a 256-CU chip at serving batch sizes), and copies each request's logits rows
 * back, the columns of enabled tasks only (others are left untouched, as in mt_forward).  Same shapes for every
 * request; sequences of different requests never interact.  Results equal mt_forward per request up to the
 * rounding differences between launch shapes (the contraction kernel is chosen by row count).
 * Needs 1 <= n_requests <= 64, n_requests * batch <= max_batch, sequence-level heads only, C_tot <= 1024.
 * Enqueues on hip_stream only.  Errors: NULL, SHAPE, CONFIG (token-level task enabled), STATE, HIP.
 */
int mt_forward_multi(mt_model* m, int32_t n_requests, const int32_t* const* h_d_input_ids, const int32_t* const* h_d_attn_mask,
                     int32_t batch, int32_t seq, const uint8_t* h_task_mask, float* const* h_d_out_logits, void* hip_stream);
/* The same with a sequence count of its own per request: h_batch is a HOST array [n_requests], request r's arrays are
 * [h_batch[r]][seq] and [h_batch[r]][C_tot]; the sum of h_batch must not exceed max_batch.  (mt_forward_multi is this
 * call with equal counts.)  Errors as above; an error message names the call it came through. */
int mt_forward_requests(mt_model* m, int32_t n_requests, const int32_t* const* h_d_input_ids, const int32_t* const* h_d_attn_mask,
                        const int32_t* h_batch, int32_t seq, const uint8_t* h_task_mask, float* const* h_d_out_logits,
                        void* hip_stream);

/*
 * mt_forward for callers that cannot allocate device memory or let a library do so on their behalf: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical logits, but the workspace is NOT the arena given to mt_bind: it is a fixed array of
 * MT_STATIC_SCRATCH_BYTES of device memory inside the library's code object (every GPU the library is loaded on
 * holds one copy until the process ends; its address is looked up once per device).  The call makes no
 * hipMalloc / hipFree or other allocating call; mt_bind must still have attached the weight arena (its workspace
 * argument is not touched by this call).
 *   - Limit: mt_workspace_bytes(m) <= MT_STATIC_SCRATCH_BYTES, i.e. create the model with max_batch x max_seq
 *     small enough (at BERT-base width with 8 two-layer tasks on 6 shared layers: 2 x 64 tokens); larger models get
 *     MT_ERR_SHAPE with a message that names both sizes, and nothing is enqueued.
 *   - All calls on one GPU, from every model and every stream, share that GPU's array: calls that overlap on one
 *     GPU race.  Issue them on one stream, or order them yourself.  Nothing in the array needs to start at
 *     zero: each call rewrites what it reads, so contents left by an earlier (larger or smaller) call are harmless.
 *   - mt_read_hidden afterwards reads this call's states from the array.  Per-launch timing must be off
 *     (MT_ERR_STATE otherwise: it creates events).  Sequence-level heads only, no segment ids.
 * Errors: as mt_forward, plus the above.
 */
#define MT_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
int mt_forward_static(mt_model* m, const int32_t* d_input_ids, const int32_t* d_attn_mask, int32_t batch, int32_t seq,
                      const uint8_t* h_task_mask, float* d_out_logits, void* hip_stream);

/*
 * mt_forward with segment (token type) ids for sentence-pair inputs, as in the BERT input representation
 * the student models are built on (Section 3): the embedding of a token adds row d_token_type_ids[b][s]
 * of the type table instead of row 0.  d_token_type_ids: [batch][seq] int32 device array, values clamped
 * into [0, type_vocab) by the kernel, or NULL (then identical to mt_forward).  Everything else as above.
 */
int mt_forward_typed(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask, int32_t batch, int32_t seq,
               const uint8_t* h_task_mask, float* d_out_logits, void* hip_stream);

/*
 * The forward pass of a model that has token-level tasks (MT_HEAD_TOKEN).  As mt_forward_typed, plus
 *   d_out_token_logits [batch][seq][C_tok] float32, C_tok = sum of n_classes over the MT_HEAD_TOKEN tasks, task t's
 *               columns start at mt_token_logit_offset(m, t).  Columns of enabled token-level tasks are written at
 *               every position: the logits where d_attn_mask is 1, zeros where it is 0; columns of disabled
 *               tasks are left untouched.
 * d_out_logits may be NULL when no enabled task has a sequence head, d_out_token_logits when none has a token
 * head.  A token-level task's last layer is evaluated for all tokens, a sequence-level task's for the first only.
 * Errors as mt_forward.
 */
int mt_forward_tokens(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask,
                      int32_t batch, int32_t seq, const uint8_t* h_task_mask, float* d_out_logits, float* d_out_token_logits,
                      void* hip_stream);

/*
 * Per-sequence task routing (Section 5.2 discusses that every task is computed for every request; a serving
 * system that knows which tasks a request needs can skip the rest): h_route is a host array [batch][n_tasks],
 * nonzero = sequence b wants task t.  The trunk runs once for the whole batch, as deep as the deepest wanted
 * fork; tasks wanted by the same set of sequences form a group whose sequences are gathered into a row order of
 * their own, on which the group's branch layers, poolers and classifiers run.  Logits of wanted (b, t) pairs are
 * written to d_out_logits[b][mt_logit_offset(t)..]; all other entries are left untouched.  batch <= 1024.
 * d_token_type_ids may be NULL.  Errors as mt_forward; NULL when a wanted task has a token-level head (that needs
 * mt_forward_routed_tokens).  After this call mt_read_hidden serves trunk taps only.
 * With more than one group the groups run side by side on up to four streams that the model owns (default
 * priority; the first routed call creates them and their events, mt_destroy releases them): they wait for the
 * trunk on hip_stream through an event and hip_stream waits for them before the call's work counts as done, so
 * for the caller everything is still ordered on hip_stream and the call only enqueues.
 */
int mt_forward_routed(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask,
                      int32_t batch, int32_t seq, const uint8_t* h_route, float* d_out_logits, void* hip_stream);

/*
 * mt_forward_routed for models with token-level tasks (Section 5.2 x Appendix E's tagging tasks): as above, plus
 *   d_out_token_logits [batch][seq][C_tok] float32: for every wanted pair (b, t) of a MT_HEAD_TOKEN task, task t's
 *               columns of sequence b are written at every position (logits where d_attn_mask is 1, zeros where it
 *               is 0); columns of unwanted pairs are left untouched.  A routed token-level task evaluates all its
 *               layers on every token of its sequences.
 * d_out_logits may be NULL when no wanted task has a sequence head, d_out_token_logits when none has a token head.
 */
int mt_forward_routed_tokens(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask,
                             int32_t batch, int32_t seq, const uint8_t* h_route, float* d_out_logits, float* d_out_token_logits,
                             void* hip_stream);

/* Column of task t's first logit inside the row of its kind (the per-sequence row for MT_HEAD_SEQUENCE, the
 * per-token row for MT_HEAD_TOKEN), or MT_ERR_SHAPE (task out of range) / MT_ERR_CONFIG (task is of the other
 * kind).  mt_n_logits = C_tot, mt_n_token_logits = C_tok. */
int mt_logit_offset(const mt_model* m, int32_t task);
int mt_n_logits(const mt_model* m);
int mt_token_logit_offset(const mt_model* m, int32_t task);
int mt_n_token_logits(const mt_model* m);

/* The paper's cost measure (Section 4.1, "Overhead" of Table 2): the number of transformer layers
 * evaluated per request, n_trunk_layers + sum_t n_layers. */
int mt_layer_count(const mt_model* m);

/* Sequential layer steps of the wavefront schedule for the enabled tasks (h_task_mask as in mt_forward, NULL =
 * all): trunk layer k+1 and every branch layer whose input exists run together in step k, so the count is
 * max(D', max_t(fork_t + n_layers_t)) with D' the deepest enabled fork (Fig. 1(c)); a schedule that finished the
 * trunk before starting any branch would need D' + max_t n_layers_t.  Host only.  Errors: NULL. */
int mt_schedule_steps(const mt_model* m, const uint8_t* h_task_mask);

/* Text of the last error on this model ("" if none).  mt_error_name maps a code to its name. */
const char* mt_last_error(const mt_model* m);
const char* mt_error_name(int code);

/*
 * Copy the float32 hidden state [batch][seq][hidden] the last mt_forward left for
 *   task < 0 : the trunk after `layer` shared layers (only layers some task forks at are kept);
 *   task >= 0: task's branch output after its last own layer, of which only the first token of every
 *              sequence is computed (the pooler reads nothing else): position 0 holds it, the rest is 0;
 *              for a task without own layers this is its trunk tap (`layer` ignored); for a token-level task
 *              the whole state (padded positions 0)
 * into d_out on `hip_stream`.  For validation.  Errors: NULL, SHAPE, STATE (no forward pass has run; the task
 * was masked off in the last one; the last one stopped the trunk below `layer` because no deeper task was
 * enabled, or had no task enabled at all).
 */
int mt_read_hidden(mt_model* m, int32_t task, int32_t layer, float* d_out, size_t out_bytes, void* hip_stream);

/*
 * Per-kernel timing.  While enabled, mt_forward brackets every launch with HIP events on the
 * forward's stream.  mt_profile_read waits for them, then reports, per kernel class, the number of
 * launches and their summed duration since the last read, and clears the record.
 * MT_K_GEMM_FIRST collects the four one-row-per-sequence contractions (query, output projection and
 * both feed-forward layers) of every branch's last layer; that layer's K|V projection over all rows
 * counts under MT_K_GEMM_QKV.
 */
enum {
    MT_K_EMBED = 0, MT_K_GEMM_QKV, MT_K_ATTN, MT_K_GEMM_OUT, MT_K_LN, MT_K_GEMM_FFN1, MT_K_GEMM_FFN2,
    MT_K_POOL, MT_K_GEMM_FIRST, MT_K_COUNT
};
int mt_profile_enable(mt_model* m, int32_t on);
int mt_profile_read(mt_model* m, float* h_ms /*[MT_K_COUNT]*/, int32_t* h_launches /*[MT_K_COUNT]*/);

/*
 * Single operations on device buffers, the same kernels mt_forward launches, exposed so each can be
 * checked on its own.  `precision` selects the element type of activations/weights named "act":
 * MT_BF16 -> bfloat16, MT_FP32_CHECK -> float32.  All enqueue on hip_stream and return.
 */
/* C[M,N] = epilogue(A[M,K] W[N,K]^T + bias[N]) ; act_kind: 0 none, 1 GELU(erf), 2 GELU(tanh), 3 tanh.
 * d_residual (float32 [M,N]) may be NULL; if given it is added after the activation (bf16 precision:
 * only together with out_f32 != 0, and then act_kind must be 0 - the two forms the model uses).
 * out_f32 != 0 stores float32, else the act type.  lda/ldc in elements. */
int mt_op_linear(int32_t precision, const void* d_A, int64_t lda, const void* d_W, const float* d_bias,
                 const float* d_residual, void* d_C, int64_t ldc, int32_t M, int32_t N, int32_t K,
                 int32_t act_kind, int32_t out_f32, void* hip_stream);
/* The grouped form: G same-shaped problems in one launch, problem g using base pointer + g*stride
 * (strides in elements of the respective type; 0 shares the operand between problems), G <= 32. */
int mt_op_linear_batched(int32_t precision, int32_t G, const void* d_A, int64_t strideA, int64_t lda, const void* d_W,
                         int64_t strideW, const float* d_bias, int64_t strideBias, const float* d_residual,
                         int64_t strideRes, void* d_C, int64_t strideC, int64_t ldc, int32_t M, int32_t N, int32_t K,
                         int32_t act_kind, int32_t out_f32, void* hip_stream);

/* The few-row bf16 contraction with sub-problems, as the first-token attention of a branch's last layer uses
 * it (Section 3.3: only the first token feeds the task head): n_sub equal-shaped problems
 *   C_u[M,N] = A_u[M,K] W_u[N,K]^T + bias_u,   A_u = d_A + u*sub_a, W_u = d_W + u*sub_w, C_u = d_C + u*sub_c,
 *   bias_u = d_bias + u*sub_bias (element offsets; lda/ldw/ldc row strides in elements, ldw 0 = K).
 * With d_sub_row0 / d_sub_rows (device int32 [n_sub], both or neither) problem u instead starts at row
 * d_sub_row0[u] of A and C and has min(M, d_sub_rows[u]) rows (a ragged batch; rows beyond are untouched).
 * bf16 inputs; out_f32 != 0 stores float32, else bf16.  Needs K % 64 == 0, N % 4 == 0, 16-byte aligned rows.
 * Errors: NULL, SHAPE. */
int mt_op_linear_sub(const void* d_A, int64_t lda, const void* d_W, int64_t ldw, const float* d_bias, void* d_C, int64_t ldc,
                     int32_t M, int32_t N, int32_t K, int32_t n_sub, int64_t sub_a, int64_t sub_w, int64_t sub_c,
                     int64_t sub_bias, const int32_t* d_sub_row0, const int32_t* d_sub_rows, int32_t out_f32,
                     void* hip_stream);

/* The softmax and weighted row sum of the first-token attention (Section 3.3 head; see mt_op_linear_sub):
 * for sequence b owning rows d_seq_start[b] .. +d_seq_len[b]-1 of the padding-free row order and head a < heads,
 *   p = softmax_j(d_scores[row_j][a] / sqrt(hidden/heads)),  d_xbar[b][a][:] = sum_j p_j * d_x[row_j][:].
 * d_scores float32 [rows][heads_pad], d_x bf16 [rows][hidden], d_xbar bf16 [batch][heads_pad][hidden] (pad heads
 * are not written); heads <= heads_pad <= 16, heads_pad % 4 == 0, seq * heads_pad * 4 <= 64 KiB.
 * Errors: NULL, SHAPE. */
int mt_op_first_token_pool(const float* d_scores, const void* d_x, void* d_xbar, const int32_t* d_seq_start,
                           const int32_t* d_seq_len, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                           int32_t heads_pad, void* hip_stream);
/* ctx[b,s,a*d:(a+1)*d] = softmax(q k^T / sqrt(d) + mask) v per head; d_qkv is [B*S][3H] act
 * (columns Q | K | V), d_ctx [B*S][H] act. */
int mt_op_attention(int32_t precision, const void* d_qkv, const int32_t* d_mask, void* d_ctx,
                    int32_t batch, int32_t seq, int32_t hidden, int32_t heads, void* hip_stream);
/* out = LayerNorm(x) * gamma + beta per row; x float32 [M,H]; writes float32 d_out_f32 (may be NULL)
 * and bfloat16 d_out_bf16 (may be NULL). */
int mt_op_layernorm(const float* d_x, const float* d_gamma, const float* d_beta, float eps, float* d_out_f32,
                    void* d_out_bf16, int32_t M, int32_t H, void* hip_stream);

/* The FP8 contraction alone, as MT_FP8_FFN uses it: d_A [M][lda] and d_W [N][K] are E4M3 bytes (lda in elements, a
 * multiple of 16), C = act(scale * A W^T + bias) (+ residual); out_kind 0 bfloat16, 1 float32 (d_residual allowed, no
 * activation), 2 E4M3 (the value times out_scale, saturating).  act_kind 0 none, 1 GELU(erf), 2 GELU(tanh).
 * Needs K % 64 == 0, K >= 192, N % 4 == 0.  Errors: NULL, SHAPE, HIP. */
int mt_op_linear_fp8(const void* d_A, int64_t lda, const void* d_W, float scale, const float* d_bias, const float* d_residual,
                     void* d_C, int64_t ldc, int32_t M, int32_t N, int32_t K, int32_t act_kind, int32_t out_kind, float out_scale,
                     void* hip_stream);
/* Host only: the conversion mt_load_weights applies to a feed-forward matrix in MT_FP8_FFN mode.  Returns the storage
 * scale s (largest power of two with s max|w| <= 448; 1 for an all-zero matrix) and, if h_out is not NULL, writes
 * E4M3(s w[i]) (round to nearest even, saturating) to h_out[i]. */
float mt_debug_e4m3_quantize(const float* h_w, size_t n, uint8_t* h_out);

/* Tuning aid for benchmarks: force one bf16 GEMM tile configuration for all later launches in this
 * process (0 = choose by shape, the default; 1..26 except 13 = a fixed tile configuration, 13 = the few-row kernel, 27 = the persistent kernel;
 * any other value resets to 0).  One process-wide setting, not thread-safe: for single-threaded tuning sweeps
 * only, never set while forward passes are being enqueued from other threads.  Returns the previous value. */
int mt_debug_set_gemm_tile(int32_t sel);

/*
 * Measured matrix-core rate (the roofline of the bf16 contractions, Section 3.3's serving cost being all
 * transformer layers): runs back-to-back register-only v_mfma_f32_32x32x16_bf16 on every compute unit of the
 * current device for `iters` x 8 instructions per wavefront and writes the achieved dense bf16 TFLOP/s to
 * *h_tflops (host).  d_scratch: device memory of at least `scratch_bytes` >= 1 MiB, overwritten.  Blocks until
 * the measurement is done.  Errors: NULL, SHAPE (iters < 1 or scratch too small), HIP.
 */
int mt_debug_mfma_peak(int32_t iters, void* d_scratch, size_t scratch_bytes, float* h_tflops, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MT_H_ */
