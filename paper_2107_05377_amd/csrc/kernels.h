// Internal launch interface between the host scheduler and the gfx950 kernels.
// Every launcher only enqueues on `stream`; none allocates or synchronises.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mt {

typedef uint16_t bf16_t;   // raw bfloat16 bits in host-visible interfaces

constexpr int kMaxGroup = 32;   // problems per grouped launch (one per active task)

// Epilogue applied to the fp32 accumulator: v = acc + bias[n]; v = act(v); v += residual[m][n].
enum ActKind : int { ACT_NONE = 0, ACT_GELU_ERF = 1, ACT_GELU_TANH = 2, ACT_TANH = 3 };

// A group of G same-shaped problems C_g[M,N] = epi(A_g[M,K] * W_g[N,K]^T), passed by value as a
// kernel argument so that a change of the active task set needs no device-side table.
struct GemmGroup {
    const void* A[kMaxGroup];
    const void* W[kMaxGroup];
    void* C[kMaxGroup];
    const float* bias[kMaxGroup];       // may be null
    const float* residual[kMaxGroup];   // fp32 [M][ldr], may be null
    int32_t N[kMaxGroup];               // per-problem N (fp32 path only; the MFMA path needs uniform N)
    float scale[kMaxGroup];             // FP8 path only: the accumulator is multiplied by this before the bias is added
};

struct GemmShape {
    int32_t G, M, N, K;     // N = max over the group; M = row bound (grid size), see d_M
    int64_t lda, ldc, ldr;  // row strides in elements
    int32_t act;            // ActKind
    int32_t out_f32;        // 1: C is float32, 0: C has the activation element type (bf16); FP8 path also 2: C is E4M3 bytes
    const int32_t* d_M;     // optional device scalar: rows actually present (<= M); tiles beyond it exit at once
    int32_t splits;         // bf16 path, >= 1: K is cut into `splits` equal ranges, range p of problem g writing its
                            // partial product (float32, no epilogue) to C_g + p * split_stride elements
    int64_t split_stride;
    int64_t ldw;            // row stride of W in elements; 0 = dense (K)
    // Few-row kernel only (launch_gemm_bf16 routes there when n_sub > 1): every problem g consists of n_sub
    // sub-problems of the same shape, sub-problem u using A_g + u*sub_a, W_g + u*sub_w, C_g + u*sub_c and
    // bias_g + u*sub_bias (element offsets); no residual.  With d_sub_row0 / d_sub_rows (device arrays [n_sub])
    // sub-problem u additionally starts at row d_sub_row0[u] of A and C and has d_sub_rows[u] (<= M) rows:
    // a ragged batch, e.g. one sub-problem per sequence of the padding-free row order.
    int32_t n_sub;
    int64_t sub_a, sub_w, sub_c, sub_bias;
    const int32_t* d_sub_row0;
    const int32_t* d_sub_rows;
    float out_scale;        // FP8 path, out_f32 == 2: the value is multiplied by this before it is rounded to E4M3
};

// bf16 x bf16 -> fp32 accumulate on the matrix cores.  Needs K % 64 == 0, lda % 8 == 0, 16-byte aligned A/W rows.
hipError_t launch_gemm_bf16(const GemmGroup& g, const GemmShape& s, hipStream_t stream);
// FP8 (OCP E4M3) x FP8 -> float32 accumulate, both operands one byte per element, K contiguous (lda / ldw in elements =
// bytes, multiples of 16); needs K % 64 == 0 and K >= 192.  C_g = epi(g.scale[g] * A_g W_g^T + bias): out_f32 0 / 1 / 2
// = bf16 / float32 (+ residual) / E4M3 (times out_scale).  Activations: none, GELU(erf), GELU(tanh).
hipError_t launch_gemm_fp8(const GemmGroup& g, const GemmShape& s, hipStream_t stream);
// Persistent variant for launches of many 256x256 tiles (one workgroup per compute unit walks a tile list with
// its load ring never draining); launch_gemm_bf16 routes to it by itself.  gemm_bf16_persist_takes: shape supported.
bool gemm_bf16_persist_takes(const GemmShape& s);
bool gemm_bf16_persist_wants(const GemmShape& s);      // ... and measured faster than the tiled kernel
hipError_t launch_gemm_bf16_persist(const GemmGroup& g, const GemmShape& s, hipStream_t stream);
// Few-row variant (M <= 256), memory-parallel instead of tiled; launch_gemm_bf16 routes to it by itself.
hipError_t launch_gemm_skinny_bf16(const GemmGroup& g, const GemmShape& s, hipStream_t stream);
// Register-only matrix-core rate measurement: n_cu workgroups of 8 wavefronts, `iters` x 8 MFMAs each; d_out needs
// mfma_rate_out_floats(n_cu) floats.  Synchronises on the stream.
hipError_t run_mfma_rate(int iters, int n_cu, float* d_out, hipStream_t stream, float* tflops);
int mfma_rate_out_floats(int n_cu);
// fp32 (A) x {fp32|bf16} (W) on the vector ALUs, any shape.  w_bf16 selects the W element type.
hipError_t launch_gemm_f32(const GemmGroup& g, const GemmShape& s, int w_bf16, hipStream_t stream);

// Token rows of a batch in padding-free order: only positions with mask == 1 are kept, sequence after
// sequence, so every row-wise kernel and every contraction runs on sum_b len_b rows instead of B*S.
struct RowMap {
    int32_t* n_rows;      // [1]  number of kept rows
    int32_t* src;         // [B*S] kept row -> b*S+s
    int32_t* row_of;      // [B*S] b*S+s -> kept row, or -1
    int32_t* seq_start;   // [B]  first kept row of sequence b
    int32_t* seq_len;     // [B]  kept rows of sequence b
};
hipError_t launch_build_row_map(const int32_t* mask, int B, int S, const RowMap& map, hipStream_t stream);
// *count = number of sequences whose position 0 is masked off (mask[b][0] == 0; an all-padding sequence is one of them)
hipError_t launch_count_bad_first_tokens(const int32_t* mask, int B, int S, int32_t* count, hipStream_t stream);
// bfloat16 [M][H] -> E4M3 [M][H] (unit scale, saturating) for up to kMaxGroup arrays in one launch; rows past *d_M are left alone
struct CastGroup {
    const void* src[kMaxGroup];
    void* dst[kMaxGroup];
};
hipError_t launch_cast_bf16_to_e4m3(const CastGroup& g, int G, int M, const int32_t* d_M, int H, hipStream_t stream);
// out[b*S+s][:] = x[row_of[b*S+s]][:] or 0 (float32, H columns)
hipError_t launch_unpack_rows(const float* x, const int32_t* row_of, int n_pos, int H, float* out, hipStream_t stream);

// Longest sequence the bf16 attention kernel takes: the keys and values of one (sequence, head) are staged in
// LDS as a whole, 260 bytes per key (rounded up to 32 keys) within the CU's 160 KB.
constexpr int kAttnBf16MaxSeq = 608;
struct AttnGroup {
    const void* qkv[kMaxGroup];   // [rows][3H]: Q | K | V
    void* ctx[kMaxGroup];         // [rows][H]
};
// Sequence b owns rows seq_start[b] .. +seq_len[b]-1 (all real tokens) when the two arrays are given;
// otherwise rows b*S .. b*S+S-1 with `mask` ([B][S], 1 = real) marking the keys.  S bounds the length.
// ctx_fmt 0: the context is written as bfloat16; 1: as E4M3 at unit scale (one byte per element, same row order)
hipError_t launch_attention_bf16(const AttnGroup& g, int G, const int32_t* mask, const int32_t* seq_start,
                                 const int32_t* seq_len, int B, int S, int H, int A, hipStream_t stream, int ctx_fmt = 0);
hipError_t launch_attention_f32(const AttnGroup& g, int G, const int32_t* mask, const int32_t* seq_start,
                                const int32_t* seq_len, int B, int S, int H, int A, hipStream_t stream);

struct LnGroup {
    const float* x[kMaxGroup];      // [n_parts][M][H] fp32: the row to normalise is sum_p x[p] (+ bias) (+ residual)
    const float* bias[kMaxGroup];      // [H], may be null
    const float* residual[kMaxGroup];  // [M][H] fp32, may be null
    const float* gamma[kMaxGroup];
    const float* beta[kMaxGroup];
    float* out_f32[kMaxGroup];      // may be null
    bf16_t* out_bf16[kMaxGroup];    // may be null
};
// d_M (optional device scalar) = rows actually present (<= M); n_parts partial sums part_stride elements apart
// low_fmt: element type written through out_bf16: 0 bfloat16, 1 OCP FP8 E4M3 (one byte per element, saturating)
hipError_t launch_layernorm(const LnGroup& g, int G, int M, const int32_t* d_M, int H, float eps, int n_parts, int64_t part_stride,
                            hipStream_t stream, int low_fmt = 0);

// X0[r] = LN(word[ids[p]] + pos[p % S] + type[0]) with p = src[r] for the kept rows r < *d_M (p = r and all
// B*S rows when src is null); tables are bf16 (emb_bf16 != 0) or fp32.
hipError_t launch_embed_ln(const int32_t* ids, const int32_t* type_ids /* [B*S] segment ids or NULL */, int type_vocab, const int32_t* src, const int32_t* d_M, int B, int S, int H, int vocab, const void* word, const void* pos,
                           const void* type, int emb_bf16, const float* gamma, const float* beta, float eps,
                           float* out_f32, bf16_t* out_bf16, hipStream_t stream);

// Pooler input for the matrix-core path: row b of problem g is the first token of sequence b of x[g]
// (float32 rows of H; row seq_start[b], or b*rows_per_seq when seq_start is null); it is written as [hi | lo] bfloat16 halves, hi = bf16(v), lo = bf16(v - hi), into
// out[g] ([B][2H]), so that a bf16 contraction against [W | W] reproduces the float32 input to ~2^-17.
struct SplitGroup {
    const float* x[kMaxGroup];
    bf16_t* out[kMaxGroup];
    int32_t compact[kMaxGroup];   // 1: x[g] already holds one row per sequence (row b), ignore seq_start
};
// float32 validation mode: the same first-token rows copied unchanged, out[g] reinterpreted as float [B][H]
hipError_t launch_gather_rows(const SplitGroup& g, int G, int B, int H, const int32_t* seq_start, int rows_per_seq, int max_rows,
                              hipStream_t stream);
hipError_t launch_cls_split(const SplitGroup& g, int G, int B, int H, const int32_t* seq_start, int rows_per_seq, int max_rows,
                            hipStream_t stream);

// First-token rows of every sequence, gathered into compact [B][H] arrays: float32 and/or element-type copies.
struct FirstRowsGroup {
    const float* xf[kMaxGroup];     // [rows][H] fp32 source, may be null
    const void* xa[kMaxGroup];      // [rows][H] activation-type source (bf16 or fp32), may be null
    float* out_f[kMaxGroup];        // [B][H]
    void* out_a[kMaxGroup];         // [B][H]
};
hipError_t launch_gather_first_rows(const FirstRowsGroup& g, int G, int B, int H, int act_bytes, const int32_t* seq_start,
                                    int max_rows, hipStream_t stream);
// out[b][s][:] = (s == 0) ? x[b][:] : 0 for a [B][S][H] float32 output
hipError_t launch_place_first_rows(const float* x, int B, int S, int H, float* out, hipStream_t stream);

// Attention for the first-token query of every sequence only (the last layer of a branch needs nothing else):
// q[g] is [B][H] (one query row per sequence), keys and values come from kv[g] = [rows][3H] (columns H.. and 2H..),
// sequence b owning rows seq_start[b] .. +seq_len[b]-1; ctx[g] is [B][H].  Any head width <= 256.
struct AttnClsGroup {
    const void* q[kMaxGroup];
    const void* kv[kMaxGroup];
    void* ctx[kMaxGroup];
};
hipError_t launch_attention_cls(const AttnClsGroup& g, int G, int is_bf16, const int32_t* seq_start, const int32_t* seq_len,
                                int B, int S, int H, int A, hipStream_t stream);

// First-token attention WITHOUT projected keys and values (bf16 path).  With q~[b][a] = Wk_a^T q[b][a] the
// score of key j is q~[b][a] . x_j (+ a constant per row, which the softmax drops), and the head's context is
// Wv_a (sum_j p_j x_j) + bv_a.  This kernel takes the raw scores[g] = [rows][A_pad] (float32, x_j . q~),
// scales them, takes the softmax over each sequence's rows and writes the probability-weighted sum of the
// layer input rows x[g] = [rows][H] (bf16) per head: xbar[g] = [B][A_pad][H] (bf16).
struct PoolGroup {
    const float* scores[kMaxGroup];
    const void* x[kMaxGroup];
    void* xbar[kMaxGroup];
};
hipError_t launch_first_token_pool(const PoolGroup& g, int G, const int32_t* seq_start, const int32_t* seq_len, int B, int S, int H,
                                   int A, int A_pad, hipStream_t stream);

// logits[g][b][c] = Wc_g[c][:] . pooled_g[b][:] + bc_g[c]; one wavefront per (g, b, c).  Wc bf16 or fp32.
struct ClsGroup {
    const float* pooled[kMaxGroup];   // [B][H]
    const void* Wc[kMaxGroup];        // [C][H]
    const float* bc[kMaxGroup];
    float* out[kMaxGroup];            // first logit column of the task, row stride ldo
    int32_t C[kMaxGroup];
};
// out_row: optional device array [B], logits row of compact row b (per-sequence routing); NULL = row b.
hipError_t launch_classifier(const ClsGroup& g, int G, int B, int H, int maxC, int w_bf16, int64_t ldo, const int32_t* out_row,
                             hipStream_t stream);

// Token-level heads: out[g][p*ldo + c] = Wc[g][c] . x[g][row_of[p]] + bc[g][c] for every position p = b*S+s that is a
// kept row (row_of[p] in [0, *n_rows)), zeros for the positions that are not; positions with row_of[p] == -2 are
// left untouched.  x is float32 in the padding-free order.
struct TokGroup {
    const float* x[kMaxGroup];        // [rows][H]
    const void* Wc[kMaxGroup];        // [C][H]
    const float* bc[kMaxGroup];
    float* out[kMaxGroup];            // first logit column of the task at position 0, position stride ldo
    int32_t C[kMaxGroup];
};
hipError_t launch_token_classifier(const TokGroup& g, int G, int n_pos, int H, int w_bf16, int64_t ldo, const int32_t* row_of,
                                   const int32_t* n_rows, hipStream_t stream);

// Several request batches served by one forward pass: request r's ids and mask ([batch][seq] each) are copied behind
// one another into contiguous staging arrays, and afterwards the logits rows of the combined batch go back to each
// request's own [batch][ldo] array, only the columns whose bit is set in col_on (bit c of word c/32).
constexpr int kMaxRequests = 64;
constexpr int kMaxLogitCols = 1024;
struct RequestPtrs {
    const int32_t* ids[kMaxRequests];
    const int32_t* mask[kMaxRequests];
    float* out[kMaxRequests];
    int32_t first[kMaxRequests + 1];     // request r owns sequences first[r] .. first[r+1]-1 of the combined batch
    uint32_t col_on[kMaxLogitCols / 32];
};
// max_batch: the largest request's sequence count (sizes the grids)
hipError_t launch_gather_requests(const RequestPtrs& rq, int n_req, int max_batch, int seq, int32_t* ids_all, int32_t* mask_all, hipStream_t stream);
hipError_t launch_scatter_logits(const RequestPtrs& rq, int n_req, int max_batch, int n_cols, const float* logits_all, hipStream_t stream);

// Per-sequence task routing: a sub-batch of the sequences, as a padding-free row order of its own.
// idx lists the chosen sequences (ascending batch indices), passed by value with the launch.
constexpr int kMaxRouted = 1024;
struct RouteIdx {
    uint16_t seq[kMaxRouted];
};
// From the batch's row map (g_start, g_len) builds the sub-batch's: c_start/c_len [n_sel], *c_n rows in all,
// c_src[r] = row of the batch order that compact row r copies, c_seq[i] = idx.seq[i] (as int32, for the logits rows).
hipError_t launch_route_map(const RouteIdx& idx, int n_sel, const int32_t* g_start, const int32_t* g_len, int32_t* c_start,
                            int32_t* c_len, int32_t* c_src, int32_t* c_seq, int32_t* c_n, hipStream_t stream);
// c_rowof[b*S+s] for all B*S positions of the batch: the sub-batch's compact row of a real token of a chosen sequence,
// -1 for its padded positions, -2 for positions of sequences outside the sub-batch (launch_token_classifier leaves
// those untouched).  row_of / g_start: the batch's row map; c_start: the sub-batch's sequence starts.
hipError_t launch_route_rowof(const RouteIdx& idx, int n_sel, int B, int S, const int32_t* row_of, const int32_t* g_start,
                              const int32_t* c_start, int32_t* c_rowof, hipStream_t stream);
// out_f[r] = in_f[c_src[r]] (float32 rows) and out_a[r] = in_a[c_src[r]] (act_bytes per element; both optional), r < *c_n <= max_rows.
hipError_t launch_route_gather(const float* in_f, const void* in_a, float* out_f, void* out_a, const int32_t* c_src, const int32_t* c_n,
                               int max_rows, int H, int act_bytes, hipStream_t stream);

}  // namespace mt
