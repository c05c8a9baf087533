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
};

struct GemmShape {
    int32_t G, M, N, K;     // N = max over the group
    int64_t lda, ldc, ldr;  // row strides in elements (W is dense: ldw = K)
    int32_t act;            // ActKind
    int32_t out_f32;        // 1: C is float32, 0: C has the activation element type
};

// bf16 x bf16 -> fp32 accumulate on the matrix cores.  Needs K % 64 == 0, lda % 8 == 0, 16-byte aligned A/W rows.
hipError_t launch_gemm_bf16(const GemmGroup& g, const GemmShape& s, hipStream_t stream);
// fp32 (A) x {fp32|bf16} (W) on the vector ALUs, any shape.  w_bf16 selects the W element type.
hipError_t launch_gemm_f32(const GemmGroup& g, const GemmShape& s, int w_bf16, hipStream_t stream);

struct AttnGroup {
    const void* qkv[kMaxGroup];   // [B*S][3H]: Q | K | V
    void* ctx[kMaxGroup];         // [B*S][H]
};
hipError_t launch_attention_bf16(const AttnGroup& g, int G, const int32_t* mask, int B, int S, int H, int A,
                                 hipStream_t stream);
hipError_t launch_attention_f32(const AttnGroup& g, int G, const int32_t* mask, int B, int S, int H, int A,
                                hipStream_t stream);

struct LnGroup {
    const float* x[kMaxGroup];      // [M][H] fp32, already bias+residual summed
    const float* gamma[kMaxGroup];
    const float* beta[kMaxGroup];
    float* out_f32[kMaxGroup];      // may be null
    bf16_t* out_bf16[kMaxGroup];    // may be null
};
hipError_t launch_layernorm(const LnGroup& g, int G, int M, int H, float eps, hipStream_t stream);

// X0 = LN(word[id] + pos[s] + type[0]); tables are bf16 (emb_bf16 != 0) or fp32.
hipError_t launch_embed_ln(const int32_t* ids, int B, int S, int H, int vocab, const void* word, const void* pos,
                           const void* type, int emb_bf16, const float* gamma, const float* beta, float eps,
                           float* out_f32, bf16_t* out_bf16, hipStream_t stream);

// Pooler input for the matrix-core path: row b of problem g is token 0 of sequence b of x[g] (float32,
// row stride ldx); it is written as [hi | lo] bfloat16 halves, hi = bf16(v), lo = bf16(v - hi), into
// out[g] ([B][2H]), so that a bf16 contraction against [W | W] reproduces the float32 input to ~2^-17.
struct SplitGroup {
    const float* x[kMaxGroup];
    bf16_t* out[kMaxGroup];
};
hipError_t launch_cls_split(const SplitGroup& g, int G, int B, int H, int64_t ldx, hipStream_t stream);

// logits[g][b][c] = Wc_g[c][:] . pooled_g[b][:] + bc_g[c]; one wavefront per (g, b, c).  Wc bf16 or fp32.
struct ClsGroup {
    const float* pooled[kMaxGroup];   // [B][H]
    const void* Wc[kMaxGroup];        // [C][H]
    const float* bc[kMaxGroup];
    float* out[kMaxGroup];            // first logit column of the task, row stride ldo
    int32_t C[kMaxGroup];
};
hipError_t launch_classifier(const ClsGroup& g, int G, int B, int H, int maxC, int w_bf16, int64_t ldo, hipStream_t stream);

}  // namespace mt
