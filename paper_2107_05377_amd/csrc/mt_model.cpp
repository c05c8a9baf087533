// Host side of the library: configuration checks, the merged graph's schedule (paper Section 3.3,
// Fig. 1(c)), arena layouts, checkpoint loading and the enqueue-only forward pass.
//
// Rows.  Every forward first builds the padding-free row order of the batch on the device (only
// positions with mask == 1 are kept); all row-wise kernels and contractions then run on those rows,
// their count being read from device memory so that the host never waits for it.
//
// Schedule.  The trunk (shared frozen layers) runs once up to the deepest fork among the enabled
// tasks; the hidden state after every layer some task forks at is kept (a "tap").  Trunk and branches
// advance as one wavefront of layer steps: step k runs trunk layer k+1 and, for every enabled task that
// forked at or before k, that task's own layer k - fork, all as grouped launches with one problem per
// layer instance, a branch reading its tap at its first own layer and its own state afterwards.
// A task's LAST own layer feeds only the pooler, which reads the first token: that layer is evaluated for
// the first-token rows only.  In bfloat16 mode it projects no keys or values either: the query is folded
// into the key matrix (Wk^T q per head), scores are taken against the layer input rows directly, and the
// value matrix is applied to the probability-weighted row sums (exactly the same attention, up to rounding).
// Finally one grouped pooler launch and one grouped classifier launch write all logits.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/mt.h"
#include "kernels.h"

using namespace mt;

namespace mt {
extern int g_gemm_bf16_tile_override;
}

// Upper bounds on the K split of the two narrow contractions of a layer (tuning knobs).  With 64-row tiles for
// narrow outputs a 2304-row problem already has 216 tiles, and measured throughput is best without any split
// (no float32 partial products for the LayerNorm to re-read); the mechanism stays for other shapes.
#ifndef MT_RESID_IN_GEMM
#define MT_RESID_IN_GEMM 0
#endif
#ifndef MT_MAX_SPLITS_OUT
#define MT_MAX_SPLITS_OUT 1
#endif
#ifndef MT_FEW_TILES
#define MT_FEW_TILES 64
#endif
#ifndef MT_FEW_SPLITS_OUT
#define MT_FEW_SPLITS_OUT 2
#endif
#ifndef MT_FEW_SPLITS_FFN2
#define MT_FEW_SPLITS_FFN2 4
#endif
#ifndef MT_MAX_SPLITS_FFN2
#define MT_MAX_SPLITS_FFN2 1
#endif

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct LayerW {   // byte offsets into the weight arena
    size_t Wqkv, bqkv, Wo, bo, ln1g, ln1b, W1, b1, W2, b2, ln2g, ln2b;
    size_t WkT = 0;   // bf16 mode, a task's last layer only: Wk transposed, [H][H] (first-token attention), else 0
    // FP8 variant: E4M3 copies of the two feed-forward matrices, stored as W * s with s the largest power of two that
    // keeps s * max|W| <= 448; inv_s (set when the checkpoint is loaded) undoes it in the contraction's epilogue
    size_t W1q = 0, W2q = 0;
    float inv_s1 = 1.f, inv_s2 = 1.f;
    // MT_FP8_LAYER: likewise [3H][H] of Wq, Wk, Wv under one scale, and Wo
    size_t Wqkvq = 0, Woq = 0;
    float inv_sqkv = 1.f, inv_so = 1.f;
};
struct TaskW {
    std::vector<LayerW> layers;
    size_t Wp, bp, Wc, bc;   // Wp is [H][2H] = [W | W] in bf16 mode (see launch_cls_split), [H][H] in fp32 mode
    size_t begin, end;   // the task's private region of the arena
};
struct Scratch {   // byte offsets into the workspace; one set for the trunk and one per task
    size_t qkv, ctx, y, x1f, x1b, u;
    int y_parts;   // y holds this many [M][H] float32 partial products (K ranges of a split contraction)
};
struct ClsScratch {   // per task with own layers: compact [max_batch] x ... buffers of its last, first-token-only layer
    size_t in_f, in_a, q, ctx, y, x1f, x1a, u, out_f;
    size_t qt = 0, scores = 0, xbar = 0;   // bf16 mode: Wk^T q [max_batch][A_pad][H], raw scores [M][A_pad], weighted row sums
};
struct RouteMapOff {   // byte offsets of a sub-batch row map (per-sequence routing), one per task
    size_t n, src, start, len, seq;
    size_t rowof;      // position -> compact row, for token-level heads
};
struct ProfRec {
    int klass;
    hipEvent_t t0, t1;
    bool owns_t0;      // false: t0 is the previous record's t1 (one event between back-to-back launches)
};

}  // namespace

struct mt_model {
    mt_config cfg;
    std::vector<mt_task_desc> tasks;
    bool bf16 = true;
    bool fp8 = false;   // MT_FP8_FFN / MT_FP8_LAYER: bf16 everywhere, the two feed-forward contractions of every all-rows layer in E4M3
    bool fp8_attn = false;   // MT_FP8_LAYER: the QKV and attention output projections of such a layer too
    size_t esz = 2;   // bytes per matrix / activation element
    int C_tot = 0, C_tok = 0;            // widths of the per-sequence and of the per-token logit row
    std::vector<int> logit_off;          // task -> first column inside the row of its kind

    // weight arena
    size_t w_word = 0, w_pos = 0, w_type = 0, w_embg = 0, w_embb = 0, w_trunk_end = 0;
    std::vector<LayerW> trunk;
    std::vector<TaskW> taskw;
    size_t weight_bytes = 0;

    // workspace
    size_t Mmax = 0;
    std::vector<int> tap_of_layer;            // layer index 0..D -> tap slot or -1
    std::vector<size_t> tap_f, tap_b;         // per tap slot
    size_t pp_f[2] = {0, 0}, pp_b[2] = {0, 0};
    Scratch trunk_scr{};
    std::vector<Scratch> task_scr;
    std::vector<size_t> task_xf, task_xb;
    std::vector<ClsScratch> task_cls;
    size_t pooled = 0, cls_split = 0;
    size_t rm_n = 0, rm_src = 0, rm_rowof = 0, rm_start = 0, rm_len = 0;   // padding-free row map of the current batch
    size_t chk_count = 0;                                                   // mt_check_mask: one int32
    size_t mr_ids = 0, mr_mask = 0, mr_logits = 0;                          // mt_forward_multi: the combined batch's ids, mask, logits
    size_t workspace_bytes = 0;

    unsigned char* d_w = nullptr;
    unsigned char* d_ws = nullptr;
    unsigned char* ws_act = nullptr;   // workspace of the forward pass being enqueued / enqueued last (d_ws or the static scratch)
    bool trunk_loaded = false;
    std::vector<char> task_loaded;

    int last_B = 0, last_S = 0;
    int last_depth = -1;                 // trunk layers the last forward pass evaluated; -1: it evaluated nothing
    std::vector<char> last_enabled;

    bool profiling = false;
    std::vector<ProfRec> prof;
    std::vector<hipEvent_t> event_pool;
    std::vector<RouteMapOff> route;
    // per-sequence routing: groups of tasks run side by side on streams of the model's own (default priority),
    // forked from and joined back into the caller's stream with events; created by the first routed forward
    std::vector<hipStream_t> aux_streams;
    std::vector<hipEvent_t> aux_join;
    hipEvent_t aux_fork = nullptr;

    std::string err;
};

namespace {

int fail(mt_model* m, int code, const char* fmt, ...)
{
    if (m) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        m->err = buf;
    }
    return code;
}

struct Bump {
    size_t off = 0;
    size_t take(size_t bytes)
    {
        size_t at = off;
        off = align_up(off + bytes);
        return at;
    }
};

LayerW layout_layer(Bump& b, size_t H, size_t F, size_t esz, bool fp8 = false, bool fp8_attn = false)
{
    LayerW L;
    L.Wqkv = b.take(3 * H * H * esz);
    L.bqkv = b.take(3 * H * 4);
    L.Wo = b.take(H * H * esz);
    L.bo = b.take(H * 4);
    L.ln1g = b.take(H * 4);
    L.ln1b = b.take(H * 4);
    L.W1 = b.take(F * H * esz);
    L.b1 = b.take(F * 4);
    L.W2 = b.take(H * F * esz);
    L.b2 = b.take(H * 4);
    L.ln2g = b.take(H * 4);
    L.ln2b = b.take(H * 4);
    if (fp8) {
        L.W1q = b.take(F * H);
        L.W2q = b.take(H * F);
    }
    if (fp8_attn) {
        L.Wqkvq = b.take(3 * H * H);
        L.Woq = b.take(H * H);
    }
    return L;
}

Scratch layout_scratch(Bump& b, size_t M, size_t H, size_t F, size_t esz, bool bf16, int y_parts)
{
    Scratch s;
    s.y_parts = y_parts;
    s.qkv = b.take(M * 3 * H * esz);
    s.ctx = b.take(M * H * esz);
    s.y = b.take((size_t)y_parts * M * H * 4);
    s.x1f = b.take(M * H * 4);
    s.x1b = bf16 ? b.take(M * H * 2) : 0;
    s.u = b.take(M * F * esz);
    return s;
}

inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// float32 -> OCP FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; largest finite value 448, no
// infinities, 0x7F = NaN), round to nearest even, saturating: what a conversion instruction with clamping gives.
inline uint8_t f32_to_e4m3_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    const uint8_t sign = (uint8_t)((u >> 24) & 0x80u);
    const uint32_t a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint8_t)(sign | 0x7Fu);                       // NaN
    float af;
    memcpy(&af, &a, 4);
    if (af >= 448.0f) return (uint8_t)(sign | 0x7Eu);                          // saturate (also +-inf)
    if (af < 0.015625f) {                                                      // below 2^-6: multiples of 2^-9
        const float q = nearbyintf(af * 512.0f);                               // default rounding mode: to nearest even
        return (uint8_t)(sign | (uint8_t)q);                                   // q == 8 is the smallest normal, 0x08
    }
    uint32_t r = a + 0x7FFFFu + ((a >> 20) & 1u);                              // keep 3 mantissa bits
    const int e = (int)(r >> 23) - 127 + 7;                                    // 1 .. 15 here
    const uint32_t mant = (r >> 20) & 7u;
    const uint32_t code = ((uint32_t)e << 3) | mant;
    return (uint8_t)(sign | (code > 0x7Eu ? 0x7Eu : code));
}

// The storage scale of an FP8 weight matrix: the largest power of two s with s * max|W| <= 448 (1 for a zero matrix).
inline float e4m3_scale_for(const float* w, size_t n)
{
    float mx = 0.f;
    for (size_t i = 0; i < n; ++i) {
        const float a = fabsf(w[i]);
        if (a > mx) mx = a;                        // NaNs never compare greater
    }
    if (!(mx > 0.f) || !std::isfinite(mx)) return 1.f;
    int e = (int)floorf(log2f(448.0f / mx));
    e = std::max(-100, std::min(100, e));
    float s = ldexpf(1.0f, e);
    while (s * mx > 448.0f) s *= 0.5f;             // log2f rounding at exact powers of two
    while (s * 2.0f * mx <= 448.0f) s *= 2.0f;
    return s;
}

// Copy n float32 values into the staging image as matrix elements (bf16 or fp32).
void put_matrix(unsigned char* dst, const float* src, size_t n, bool bf16)
{
    if (!bf16) {
        memcpy(dst, src, n * 4);
        return;
    }
    uint16_t* d = reinterpret_cast<uint16_t*>(dst);
    const size_t nthreads = n > (1u << 22) ? std::min<size_t>(8, std::max(1u, std::thread::hardware_concurrency())) : 1;
    if (nthreads <= 1) {
        for (size_t i = 0; i < n; ++i) d[i] = f32_to_bf16_rne(src[i]);
        return;
    }
    std::vector<std::thread> th;
    const size_t per = (n + nthreads - 1) / nthreads;
    for (size_t t = 0; t < nthreads; ++t) {
        const size_t lo = t * per, hi = std::min(n, lo + per);
        if (lo >= hi) break;
        th.emplace_back([=] { for (size_t i = lo; i < hi; ++i) d[i] = f32_to_bf16_rne(src[i]); });
    }
    for (auto& t : th) t.join();
}

// Convert one encoder layer from the blob order into the arena image; returns floats consumed.
size_t stage_layer(const mt_model* m, LayerW& L, const float* p, unsigned char* img, size_t img_base)
{
    const size_t H = m->cfg.hidden, F = m->cfg.ffn;
    const float* p0 = p;
    auto at = [&](size_t off) { return img + (off - img_base); };
    if (L.WkT) {                    // Wk^T for the first-token attention of a task's last layer (bf16 mode)
        const float* wk = p + (H * H + H);
        std::vector<float> col(H);
        for (size_t n = 0; n < H; ++n) {
            for (size_t r = 0; r < H; ++r) col[r] = wk[r * H + n];
            put_matrix(at(L.WkT) + n * H * 2, col.data(), H, true);
        }
    }
    if (L.Wqkvq) {                  // one storage scale over Wq, Wk, Wv: the largest of the three maxima decides
        float sc = e4m3_scale_for(p, H * H);
        sc = std::min(sc, e4m3_scale_for(p + (H * H + H), H * H));
        sc = std::min(sc, e4m3_scale_for(p + 2 * (H * H + H), H * H));
        for (int i = 0; i < 3; ++i) {
            const float* w = p + (size_t)i * (H * H + H);
            uint8_t* q = at(L.Wqkvq) + (size_t)i * H * H;
            for (size_t e = 0; e < H * H; ++e) q[e] = f32_to_e4m3_rne(w[e] * sc);
        }
        L.inv_sqkv = 1.0f / sc;
    }
    for (int i = 0; i < 3; ++i) {   // Wq bq Wk bk Wv bv -> one [3H,H] matrix and one [3H] bias
        put_matrix(at(L.Wqkv) + (size_t)i * H * H * m->esz, p, H * H, m->bf16);
        p += H * H;
        memcpy(at(L.bqkv) + (size_t)i * H * 4, p, H * 4);
        p += H;
    }
    put_matrix(at(L.Wo), p, H * H, m->bf16);
    if (L.Woq) {
        const float sc = e4m3_scale_for(p, H * H);
        uint8_t* q = at(L.Woq);
        for (size_t e = 0; e < H * H; ++e) q[e] = f32_to_e4m3_rne(p[e] * sc);
        L.inv_so = 1.0f / sc;
    }
    p += H * H;
    memcpy(at(L.bo), p, H * 4); p += H;
    memcpy(at(L.ln1g), p, H * 4); p += H;
    memcpy(at(L.ln1b), p, H * 4); p += H;
    auto put_e4m3 = [&](size_t off, const float* w, size_t n) {
        const float sc = e4m3_scale_for(w, n);
        uint8_t* q = at(off);
        for (size_t i = 0; i < n; ++i) q[i] = f32_to_e4m3_rne(w[i] * sc);
        return 1.0f / sc;
    };
    put_matrix(at(L.W1), p, F * H, m->bf16);
    if (L.W1q) L.inv_s1 = put_e4m3(L.W1q, p, F * H);
    p += F * H;
    memcpy(at(L.b1), p, F * 4); p += F;
    put_matrix(at(L.W2), p, H * F, m->bf16);
    if (L.W2q) L.inv_s2 = put_e4m3(L.W2q, p, H * F);
    p += H * F;
    memcpy(at(L.b2), p, H * 4); p += H;
    memcpy(at(L.ln2g), p, H * 4); p += H;
    memcpy(at(L.ln2b), p, H * 4); p += H;
    return (size_t)(p - p0);
}

size_t layer_floats(size_t H, size_t F) { return 4 * (H * H + H) + 2 * H + (F * H + F) + (H * F + H) + 2 * H; }

struct Launcher {
    mt_model* m;
    hipStream_t st;
    hipError_t first_err = hipSuccess;

    bool chained = false;      // the previous launch of this forward left its end event as our start

    bool take_event(hipEvent_t* e)
    {
        if (m->event_pool.empty()) {
            if (hipEventCreate(e) != hipSuccess) { first_err = hipErrorOutOfMemory; return false; }
        } else {
            *e = m->event_pool.back();
            m->event_pool.pop_back();
        }
        return true;
    }
    // Launches of a forward follow one another on one stream, so ONE event separates two of them: a launch's
    // duration runs from the end of the previous launch to its own end (the first one records its own start).
    void begin(int klass)
    {
        if (!m->profiling || first_err != hipSuccess) return;
        ProfRec r;
        r.klass = klass;
        r.owns_t0 = !(chained && !m->prof.empty());
        if (r.owns_t0) {
            if (!take_event(&r.t0)) return;
            (void)hipEventRecord(r.t0, st);
        } else {
            r.t0 = m->prof.back().t1;
        }
        if (!take_event(&r.t1)) return;
        m->prof.push_back(r);
        chained = true;
    }
    void end()
    {
        if (!m->profiling || first_err != hipSuccess || m->prof.empty()) return;
        (void)hipEventRecord(m->prof.back().t1, st);
    }
    void check(hipError_t e)
    {
        if (first_err == hipSuccess && e != hipSuccess) first_err = e;
    }

    void gemm(int klass, const GemmGroup& g, GemmShape s, bool force_f32_kernel)
    {
        begin(klass);
        if (m->bf16 && !force_f32_kernel) check(launch_gemm_bf16(g, s, st));
        else check(launch_gemm_f32(g, s, m->bf16 ? 1 : 0, st));
        end();
    }
};

// One encoder layer for n same-shaped problems (n <= kMaxGroup).
struct LayerIO {
    const float* in_f;
    const void* in_b;      // bf16 copy of the input (bf16 mode)
    const LayerW* w;
    const Scratch* scr;
    float* out_f;
    void* out_b;
};

void run_layer_group(Launcher& L, const std::vector<LayerIO>& io, const RowMap& rm, int B, int S)
{
    mt_model* m = L.m;
    const int H = m->cfg.hidden, F = m->cfg.ffn, A = m->cfg.heads, M = B * S;
    const int n = (int)io.size();
    unsigned char* W = m->d_w;
    unsigned char* ws = m->ws_act;
    const bool bf = m->bf16;
    const int gelu_act = m->cfg.gelu == MT_GELU_TANH ? ACT_GELU_TANH : ACT_GELU_ERF;

    GemmGroup g;
    memset(&g, 0, sizeof g);
    GemmShape s;

    // QKV projection: [M,H] x [3H,H]^T + b -> [M,3H]
    const bool f8a = m->fp8_attn;
    if (f8a) {
        // E4M3 operand copies of the layer inputs, into the head of each problem's FFN buffer u (free until FFN1 writes
        // it); problems that read the same input (branches forking at one tap) share the first one's copy
        CastGroup cg;
        memset(&cg, 0, sizeof cg);
        int n_cast = 0;
        for (int i = 0; i < n; ++i) {
            int same = -1;
            for (int j = 0; j < i && same < 0; ++j)
                if (io[j].in_b == io[i].in_b) same = j;
            if (same >= 0) {
                g.A[i] = g.A[same];
                continue;
            }
            cg.src[n_cast] = io[i].in_b;
            cg.dst[n_cast] = ws + io[i].scr->u;
            g.A[i] = ws + io[i].scr->u;
            ++n_cast;
        }
        L.begin(MT_K_LN);
        L.check(launch_cast_bf16_to_e4m3(cg, n_cast, M, rm.n_rows, H, L.st));
        L.end();
    }
    for (int i = 0; i < n; ++i) {
        if (!f8a) g.A[i] = bf ? io[i].in_b : (const void*)io[i].in_f;
        g.W[i] = W + (f8a ? io[i].w->Wqkvq : io[i].w->Wqkv);
        g.bias[i] = (const float*)(W + io[i].w->bqkv);
        g.residual[i] = nullptr;
        g.C[i] = ws + io[i].scr->qkv;
        g.N[i] = 3 * H;
        g.scale[i] = io[i].w->inv_sqkv;
    }
    s = GemmShape{n, M, 3 * H, H, H, 3 * H, 0, ACT_NONE, bf ? 0 : 1, rm.n_rows, 1, 0};
    if (f8a) {
        L.begin(MT_K_GEMM_QKV);
        L.check(launch_gemm_fp8(g, s, L.st));
        L.end();
    } else {
        L.gemm(MT_K_GEMM_QKV, g, s, false);
    }

    // attention
    AttnGroup ag;
    memset(&ag, 0, sizeof ag);
    for (int i = 0; i < n; ++i) {
        ag.qkv[i] = ws + io[i].scr->qkv;
        ag.ctx[i] = ws + io[i].scr->ctx;
    }
    L.begin(MT_K_ATTN);
    // (MT_FP8_LAYER: the context is written as E4M3, one byte per element, into the same buffer)
    L.check(bf ? launch_attention_bf16(ag, n, nullptr, rm.seq_start, rm.seq_len, B, S, H, A, L.st, f8a ? 1 : 0)
               : launch_attention_f32(ag, n, nullptr, rm.seq_start, rm.seq_len, B, S, H, A, L.st));
    L.end();

    // Option (off): without a K split the contraction's epilogue can add bias and residual itself, so that the
    // LayerNorm reads one operand instead of two.  Measured: LayerNorm gets 30 % faster and the contractions
    // slower by the same time, so the plainer split of work stays the default.
    const bool fuse_res = bf && MT_RESID_IN_GEMM;
    // A contraction with few output tiles (one problem, narrow output) is cut along K into equal
    // ranges whose float32 partial products the following LayerNorm adds up in a fixed order.
    const bool f8 = m->fp8;
    auto pick_splits = [&](int K, int N, int max_splits, int max_splits_few) {
        if (!bf || n != 1 || io[0].scr->y_parts < 2) return 1;
        if ((f8 && K == F) || f8a) return 1;                         // the FP8 contraction has no K split
        const long tiles128 = (long)((M + 127) / 128) * ((N + 127) / 128);
        if (tiles128 >= 256) return 1;
        // a launch of at most MT_FEW_TILES 64x128 tiles leaves most CUs idle: there the K ranges pay
        const long tiles64 = (long)((M + 63) / 64) * ((N + 127) / 128);
        if (tiles64 <= MT_FEW_TILES) max_splits = max_splits_few;
        int sp = std::min(max_splits, io[0].scr->y_parts);
        while (sp > 1 && K % (64 * sp) != 0) sp >>= 1;
        return sp;
    };

    // output projection -> y (fp32 partial products), then LayerNorm(y + bias + residual) -> x1
    const int sp_o = pick_splits(H, H, MT_MAX_SPLITS_OUT, MT_FEW_SPLITS_OUT);
    for (int i = 0; i < n; ++i) {
        g.A[i] = ws + io[i].scr->ctx;
        g.W[i] = W + (f8a ? io[i].w->Woq : io[i].w->Wo);
        g.bias[i] = (fuse_res && sp_o == 1) ? (const float*)(W + io[i].w->bo) : nullptr;
        g.residual[i] = (fuse_res && sp_o == 1) ? io[i].in_f : nullptr;
        g.C[i] = ws + io[i].scr->y;
        g.N[i] = H;
        g.scale[i] = io[i].w->inv_so;
    }
    s = GemmShape{n, M, H, H, H, H, H, ACT_NONE, 1, rm.n_rows, sp_o, (int64_t)m->Mmax * H};
    if (f8a) {
        L.begin(MT_K_GEMM_OUT);
        L.check(launch_gemm_fp8(g, s, L.st));
        L.end();
    } else {
        L.gemm(MT_K_GEMM_OUT, g, s, false);
    }

    LnGroup lg;
    memset(&lg, 0, sizeof lg);
    for (int i = 0; i < n; ++i) {
        lg.x[i] = (const float*)(ws + io[i].scr->y);
        lg.bias[i] = (fuse_res && sp_o == 1) ? nullptr : (const float*)(W + io[i].w->bo);
        lg.residual[i] = (fuse_res && sp_o == 1) ? nullptr : io[i].in_f;
        lg.gamma[i] = (const float*)(W + io[i].w->ln1g);
        lg.beta[i] = (const float*)(W + io[i].w->ln1b);
        lg.out_f32[i] = (float*)(ws + io[i].scr->x1f);
        lg.out_bf16[i] = bf ? (bf16_t*)(ws + io[i].scr->x1b) : nullptr;
    }
    L.begin(MT_K_LN);
    // (FP8 variant: the operand copy of x1 is E4M3 instead of bf16, in the same buffer)
    L.check(launch_layernorm(lg, n, M, rm.n_rows, H, m->cfg.ln_eps, sp_o, (int64_t)m->Mmax * H, L.st, f8 ? 1 : 0));
    L.end();

    // FFN1 + bias + GELU -> u
    for (int i = 0; i < n; ++i) {
        g.A[i] = bf ? (const void*)(ws + io[i].scr->x1b) : (const void*)(ws + io[i].scr->x1f);
        g.W[i] = W + (f8 ? io[i].w->W1q : io[i].w->W1);
        g.bias[i] = (const float*)(W + io[i].w->b1);
        g.residual[i] = nullptr;
        g.C[i] = ws + io[i].scr->u;
        g.N[i] = F;
        g.scale[i] = io[i].w->inv_s1;
    }
    s = GemmShape{n, M, F, H, H, F, 0, gelu_act, bf ? 0 : 1, rm.n_rows, 1, 0};
    if (f8) {                                                        // E4M3 in, E4M3 out (FFN2's operand), unit activation scale
        s.out_f32 = 2;
        s.out_scale = 1.0f;
        L.begin(MT_K_GEMM_FFN1);
        L.check(launch_gemm_fp8(g, s, L.st));
        L.end();
    } else {
        L.gemm(MT_K_GEMM_FFN1, g, s, false);
    }

    // FFN2 -> y (fp32 partial products), then LayerNorm(y + bias + residual) -> layer output
    const int sp_f = pick_splits(F, H, MT_MAX_SPLITS_FFN2, MT_FEW_SPLITS_FFN2);
    for (int i = 0; i < n; ++i) {
        g.A[i] = ws + io[i].scr->u;
        g.W[i] = W + (f8 ? io[i].w->W2q : io[i].w->W2);
        g.bias[i] = (fuse_res && sp_f == 1) ? (const float*)(W + io[i].w->b2) : nullptr;
        g.residual[i] = (fuse_res && sp_f == 1) ? (const float*)(ws + io[i].scr->x1f) : nullptr;
        g.C[i] = ws + io[i].scr->y;
        g.N[i] = H;
        g.scale[i] = io[i].w->inv_s2;
    }
    s = GemmShape{n, M, H, F, F, H, H, ACT_NONE, 1, rm.n_rows, sp_f, (int64_t)m->Mmax * H};
    if (f8) {
        L.begin(MT_K_GEMM_FFN2);
        L.check(launch_gemm_fp8(g, s, L.st));
        L.end();
    } else {
        L.gemm(MT_K_GEMM_FFN2, g, s, false);
    }

    for (int i = 0; i < n; ++i) {
        lg.x[i] = (const float*)(ws + io[i].scr->y);
        lg.bias[i] = (fuse_res && sp_f == 1) ? nullptr : (const float*)(W + io[i].w->b2);
        lg.residual[i] = (fuse_res && sp_f == 1) ? nullptr : (const float*)(ws + io[i].scr->x1f);
        lg.gamma[i] = (const float*)(W + io[i].w->ln2g);
        lg.beta[i] = (const float*)(W + io[i].w->ln2b);
        lg.out_f32[i] = io[i].out_f;
        lg.out_bf16[i] = bf ? (bf16_t*)io[i].out_b : nullptr;
    }
    L.begin(MT_K_LN);
    L.check(launch_layernorm(lg, n, M, rm.n_rows, H, m->cfg.ln_eps, sp_f, (int64_t)m->Mmax * H, L.st));
    L.end();
}

// The last own layer of n tasks (n <= kMaxGroup), restricted to what the pooler needs.
struct LastIO {
    const float* in_f;     // [rows][H] layer input, float32
    const void* in_a;      // same, activation type (bf16 / fp32)
    const LayerW* w;
    const Scratch* scr;    // qkv buffer receives K | V of all rows
    const ClsScratch* cls;
};

void run_last_layer_group(Launcher& L, const std::vector<LastIO>& io, const RowMap& rm, int B, int S)
{
    mt_model* m = L.m;
    const int H = m->cfg.hidden, F = m->cfg.ffn, A = m->cfg.heads, M = B * S;
    const int n = (int)io.size();
    unsigned char* W = m->d_w;
    unsigned char* ws = m->ws_act;
    const bool bf = m->bf16;
    const size_t esz = m->esz;
    const int gelu_act = m->cfg.gelu == MT_GELU_TANH ? ACT_GELU_TANH : ACT_GELU_ERF;
    const int64_t MBH = (int64_t)m->cfg.max_batch * H;

    GemmGroup g;
    memset(&g, 0, sizeof g);
    GemmShape s;
    // keys and values are not projected at all when the first-token attention kernels cover the shape
    const bool kvfree = bf && A <= 16 && (size_t)S * ((A + 3) / 4 * 4) * 4 <= 64 * 1024;

    if (!kvfree) {
        // K | V projection for every row: rows H..3H-1 of Wqkv, written to columns H..3H-1 of the qkv buffer
        for (int i = 0; i < n; ++i) {
            g.A[i] = io[i].in_a;
            g.W[i] = W + io[i].w->Wqkv + (size_t)H * H * esz;
            g.bias[i] = (const float*)(W + io[i].w->bqkv) + H;
            g.residual[i] = nullptr;
            g.C[i] = ws + io[i].scr->qkv + (size_t)H * esz;
            g.N[i] = 2 * H;
        }
        s = GemmShape{n, M, 2 * H, H, H, 3 * H, 0, ACT_NONE, bf ? 0 : 1, rm.n_rows, 1, 0};
        L.gemm(MT_K_GEMM_QKV, g, s, false);

    }

    // first-token rows of the input (residual and operand copies), then their queries
    FirstRowsGroup fg;
    memset(&fg, 0, sizeof fg);
    for (int i = 0; i < n; ++i) {
        fg.xf[i] = io[i].in_f;
        fg.out_f[i] = (float*)(ws + io[i].cls->in_f);
        fg.xa[i] = bf ? io[i].in_a : nullptr;
        fg.out_a[i] = bf ? (void*)(ws + io[i].cls->in_a) : nullptr;
    }
    L.begin(MT_K_ATTN);
    L.check(launch_gather_first_rows(fg, n, B, H, (int)esz, rm.seq_start, M, L.st));
    L.end();
    for (int i = 0; i < n; ++i) {
        g.A[i] = ws + io[i].cls->in_a;
        g.W[i] = W + io[i].w->Wqkv;
        g.bias[i] = (const float*)(W + io[i].w->bqkv);
        g.C[i] = ws + io[i].cls->q;
        g.N[i] = H;
    }
    s = GemmShape{n, B, H, H, H, H, 0, ACT_NONE, bf ? 0 : 1, nullptr, 1, 0};
    L.gemm(MT_K_GEMM_FIRST, g, s, false);

    if (!kvfree) {
        AttnClsGroup ag;
        memset(&ag, 0, sizeof ag);
        for (int i = 0; i < n; ++i) {
            ag.q[i] = ws + io[i].cls->q;
            ag.kv[i] = ws + io[i].scr->qkv;
            ag.ctx[i] = ws + io[i].cls->ctx;
        }
        L.begin(MT_K_ATTN);
        L.check(launch_attention_cls(ag, n, bf ? 1 : 0, rm.seq_start, rm.seq_len, B, S, H, A, L.st));
        L.end();

    } else {
        // First-token attention without projecting keys and values.  With q~[b][a] = Wk_a^T q[b][a], the score of
        // key j is q~[b][a] . x_j plus a per-row constant (q . bk) that the softmax drops, and the head's context is
        // Wv_a (sum_j p_j x_j) + bv_a.  Four small launches replace the K|V projection over all rows:
        //   q~  : per head, [B x d] . WkT_a            (few-row kernel, one sub-problem per head)
        //   s   : per sequence, x rows . q~[b]^T        (few-row kernel, ragged batch over sequences)
        //   xbar: softmax over the sequence, weighted sum of its x rows per head
        //   ctx : per head, xbar[b][a] . Wv_a^T + bv_a  (few-row kernel, one sub-problem per head)
        const int d = H / A, A_pad = (A + 3) / 4 * 4;
        for (int i = 0; i < n; ++i) {
            g.A[i] = ws + io[i].cls->q;
            g.W[i] = W + io[i].w->WkT;
            g.bias[i] = nullptr;
            g.C[i] = ws + io[i].cls->qt;
            g.N[i] = H;
        }
        s = GemmShape{n, B, H, d, H, (int64_t)A_pad * H, 0, ACT_NONE, 0, nullptr, 1, 0, H};
        s.n_sub = A;
        s.sub_a = d;
        s.sub_w = d;
        s.sub_c = H;
        L.gemm(MT_K_GEMM_FIRST, g, s, false);

        for (int i = 0; i < n; ++i) {
            g.A[i] = io[i].in_a;
            g.W[i] = ws + io[i].cls->qt;
            g.C[i] = ws + io[i].cls->scores;
            g.N[i] = A_pad;
        }
        s = GemmShape{n, S, A_pad, H, H, A_pad, 0, ACT_NONE, 1, nullptr, 1, 0, 0};
        s.n_sub = B;
        s.sub_w = (int64_t)A_pad * H;
        s.d_sub_row0 = rm.seq_start;
        s.d_sub_rows = rm.seq_len;
        L.gemm(MT_K_GEMM_FIRST, g, s, false);

        PoolGroup pg;
        memset(&pg, 0, sizeof pg);
        for (int i = 0; i < n; ++i) {
            pg.scores[i] = (const float*)(ws + io[i].cls->scores);
            pg.x[i] = io[i].in_a;
            pg.xbar[i] = ws + io[i].cls->xbar;
        }
        L.begin(MT_K_ATTN);
        L.check(launch_first_token_pool(pg, n, rm.seq_start, rm.seq_len, B, S, H, A, A_pad, L.st));
        L.end();

        for (int i = 0; i < n; ++i) {
            g.A[i] = ws + io[i].cls->xbar;
            g.W[i] = W + io[i].w->Wqkv + (size_t)2 * H * H * esz;
            g.bias[i] = (const float*)(W + io[i].w->bqkv) + 2 * H;
            g.C[i] = ws + io[i].cls->ctx;
            g.N[i] = d;
        }
        s = GemmShape{n, B, d, H, (int64_t)A_pad * H, H, 0, ACT_NONE, 0, nullptr, 1, 0, 0};
        s.n_sub = A;
        s.sub_a = H;
        s.sub_w = (int64_t)d * H;
        s.sub_c = d;
        s.sub_bias = d;
        L.gemm(MT_K_GEMM_FIRST, g, s, false);
    }

    // projection (split along K: only B rows, so the weight stream is what has to be spread), LayerNorm
    auto splits_for = [&](int K, int want) {
        if (!bf) return 1;
        if (B >= 128) return 1;          // enough rows for the tiled kernel, which takes such launches unsplit (25 vs 87 us at 256 rows)
        int sp = want;
        while (sp > 1 && K % (64 * sp) != 0) sp >>= 1;
        return sp;
    };
    const int sp_o = splits_for(H, 2);
    for (int i = 0; i < n; ++i) {
        g.A[i] = ws + io[i].cls->ctx;
        g.W[i] = W + io[i].w->Wo;
        g.bias[i] = nullptr;
        g.C[i] = ws + io[i].cls->y;
        g.N[i] = H;
    }
    s = GemmShape{n, B, H, H, H, H, 0, ACT_NONE, 1, nullptr, sp_o, MBH};
    L.gemm(MT_K_GEMM_FIRST, g, s, false);

    LnGroup lg;
    memset(&lg, 0, sizeof lg);
    for (int i = 0; i < n; ++i) {
        lg.x[i] = (const float*)(ws + io[i].cls->y);
        lg.bias[i] = (const float*)(W + io[i].w->bo);
        lg.residual[i] = (const float*)(ws + io[i].cls->in_f);
        lg.gamma[i] = (const float*)(W + io[i].w->ln1g);
        lg.beta[i] = (const float*)(W + io[i].w->ln1b);
        lg.out_f32[i] = (float*)(ws + io[i].cls->x1f);
        lg.out_bf16[i] = bf ? (bf16_t*)(ws + io[i].cls->x1a) : nullptr;
    }
    L.begin(MT_K_LN);
    L.check(launch_layernorm(lg, n, B, nullptr, H, m->cfg.ln_eps, sp_o, MBH, L.st));
    L.end();

    for (int i = 0; i < n; ++i) {
        g.A[i] = ws + io[i].cls->x1a;
        g.W[i] = W + io[i].w->W1;
        g.bias[i] = (const float*)(W + io[i].w->b1);
        g.C[i] = ws + io[i].cls->u;
        g.N[i] = F;
    }
    s = GemmShape{n, B, F, H, H, F, 0, gelu_act, bf ? 0 : 1, nullptr, 1, 0};
    L.gemm(MT_K_GEMM_FIRST, g, s, false);

    const int sp_f = splits_for(F, 4);
    for (int i = 0; i < n; ++i) {
        g.A[i] = ws + io[i].cls->u;
        g.W[i] = W + io[i].w->W2;
        g.bias[i] = nullptr;
        g.C[i] = ws + io[i].cls->y;
        g.N[i] = H;
    }
    s = GemmShape{n, B, H, F, F, H, 0, ACT_NONE, 1, nullptr, sp_f, MBH};
    L.gemm(MT_K_GEMM_FIRST, g, s, false);

    for (int i = 0; i < n; ++i) {
        lg.x[i] = (const float*)(ws + io[i].cls->y);
        lg.bias[i] = (const float*)(W + io[i].w->b2);
        lg.residual[i] = (const float*)(ws + io[i].cls->x1f);
        lg.gamma[i] = (const float*)(W + io[i].w->ln2g);
        lg.beta[i] = (const float*)(W + io[i].w->ln2b);
        lg.out_f32[i] = (float*)(ws + io[i].cls->out_f);
        lg.out_bf16[i] = nullptr;
    }
    L.begin(MT_K_LN);
    L.check(launch_layernorm(lg, n, B, nullptr, H, m->cfg.ln_eps, sp_f, MBH, L.st));
    L.end();
}

}  // namespace

extern "C" {

const char* mt_error_name(int code)
{
    switch (code) {
        case MT_OK: return "MT_OK";
        case MT_ERR_NULL: return "MT_ERR_NULL";
        case MT_ERR_CONFIG: return "MT_ERR_CONFIG";
        case MT_ERR_SHAPE: return "MT_ERR_SHAPE";
        case MT_ERR_STATE: return "MT_ERR_STATE";
        case MT_ERR_BLOB: return "MT_ERR_BLOB";
        case MT_ERR_HIP: return "MT_ERR_HIP";
        default: return "MT_ERR_UNKNOWN";
    }
}

int mt_create(const mt_config* cfg, mt_model** out)
{
    if (!cfg || !out) return MT_ERR_NULL;
    *out = nullptr;
    if (cfg->struct_size != sizeof(mt_config) || cfg->version != MT_ABI_VERSION) return MT_ERR_CONFIG;
    if (cfg->n_tasks < 1 || !cfg->tasks) return cfg->tasks ? MT_ERR_CONFIG : MT_ERR_NULL;
    if (cfg->vocab < 1 || cfg->hidden < 1 || cfg->heads < 1 || cfg->ffn < 1 || cfg->max_pos < 1 || cfg->type_vocab < 1 ||
        cfg->n_trunk_layers < 0 || cfg->max_batch < 1 || cfg->max_seq < 1)
        return MT_ERR_CONFIG;
    if (cfg->hidden % cfg->heads != 0 || cfg->max_seq > cfg->max_pos) return MT_ERR_CONFIG;
    if (cfg->precision != MT_BF16 && cfg->precision != MT_FP32_CHECK && cfg->precision != MT_FP8_FFN && cfg->precision != MT_FP8_LAYER)
        return MT_ERR_CONFIG;
    if (cfg->gelu != MT_GELU_ERF && cfg->gelu != MT_GELU_TANH) return MT_ERR_CONFIG;
    if (!(cfg->ln_eps >= 0.0f)) return MT_ERR_CONFIG;
    // (the FP8 contraction walks K in slices of 64 through a 3-stage ring: K >= 192 for both feed-forward matrices)
    if ((cfg->precision == MT_FP8_FFN || cfg->precision == MT_FP8_LAYER) && (cfg->hidden < 192 || cfg->ffn < 192)) return MT_ERR_CONFIG;
    if (cfg->precision != MT_FP32_CHECK &&
        (cfg->hidden != cfg->heads * 64 || cfg->hidden % 64 != 0 || cfg->ffn % 64 != 0 || cfg->max_seq > kAttnBf16MaxSeq))
        return MT_ERR_CONFIG;
    if (cfg->precision == MT_FP32_CHECK && cfg->max_seq > 4096) return MT_ERR_CONFIG;
    int deepest = 0;
    for (int t = 0; t < cfg->n_tasks; ++t) {
        const mt_task_desc& d = cfg->tasks[t];
        if (d.fork_layer < 0 || d.fork_layer > cfg->n_trunk_layers || d.n_layers < 0 || d.n_classes < 1) return MT_ERR_CONFIG;
        if (d.head != MT_HEAD_SEQUENCE && d.head != MT_HEAD_TOKEN) return MT_ERR_CONFIG;
        deepest = std::max(deepest, d.fork_layer);
    }
    if (deepest != cfg->n_trunk_layers) return MT_ERR_CONFIG;   // the trunk is exactly as deep as the deepest fork

    mt_model* m = new (std::nothrow) mt_model();
    if (!m) return MT_ERR_CONFIG;
    m->cfg = *cfg;
    m->tasks.assign(cfg->tasks, cfg->tasks + cfg->n_tasks);
    m->cfg.tasks = m->tasks.data();
    m->bf16 = cfg->precision != MT_FP32_CHECK;
    m->fp8 = cfg->precision == MT_FP8_FFN || cfg->precision == MT_FP8_LAYER;
    m->fp8_attn = cfg->precision == MT_FP8_LAYER;
    m->esz = m->bf16 ? 2 : 4;
    const size_t H = cfg->hidden, F = cfg->ffn, T = cfg->n_tasks, D = cfg->n_trunk_layers;
    for (const auto& d : m->tasks) {
        int& width = d.head == MT_HEAD_TOKEN ? m->C_tok : m->C_tot;
        m->logit_off.push_back(width);
        width += d.n_classes;
    }

    // ---- weight arena: trunk region, then one private region per task
    Bump wb;
    m->w_word = wb.take((size_t)cfg->vocab * H * m->esz);
    m->w_pos = wb.take((size_t)cfg->max_pos * H * m->esz);
    m->w_type = wb.take((size_t)cfg->type_vocab * H * m->esz);
    m->w_embg = wb.take(H * 4);
    m->w_embb = wb.take(H * 4);
    for (size_t l = 0; l < D; ++l) m->trunk.push_back(layout_layer(wb, H, F, m->esz, m->fp8, m->fp8_attn));
    m->w_trunk_end = wb.off;
    m->taskw.resize(T);
    for (size_t t = 0; t < T; ++t) {
        TaskW& tw = m->taskw[t];
        tw.begin = wb.off;
        for (int l = 0; l < m->tasks[t].n_layers; ++l) tw.layers.push_back(layout_layer(wb, H, F, m->esz, m->fp8, m->fp8_attn));
        const bool seq_head = m->tasks[t].head == MT_HEAD_SEQUENCE;
        if (m->bf16 && seq_head && !tw.layers.empty()) tw.layers.back().WkT = wb.take(H * H * 2);
        tw.Wp = seq_head ? wb.take(H * H * m->esz * (m->bf16 ? 2 : 1)) : 0;
        tw.bp = seq_head ? wb.take(H * 4) : 0;
        tw.Wc = wb.take((size_t)m->tasks[t].n_classes * H * m->esz);
        tw.bc = wb.take((size_t)m->tasks[t].n_classes * 4);
        tw.end = wb.off;
    }
    m->weight_bytes = wb.off;

    // ---- workspace
    m->Mmax = (size_t)cfg->max_batch * cfg->max_seq;
    const size_t M = m->Mmax;
    Bump sb;
    m->tap_of_layer.assign(D + 1, -1);
    for (const auto& d : m->tasks) {
        if (m->tap_of_layer[d.fork_layer] < 0) {
            m->tap_of_layer[d.fork_layer] = (int)m->tap_f.size();
            m->tap_f.push_back(sb.take(M * H * 4));
            m->tap_b.push_back(m->bf16 ? sb.take(M * H * 2) : 0);
        }
    }
    for (int i = 0; i < 2; ++i) {
        m->pp_f[i] = sb.take(M * H * 4);
        m->pp_b[i] = m->bf16 ? sb.take(M * H * 2) : 0;
    }
    m->trunk_scr = layout_scratch(sb, M, H, F, m->esz, m->bf16, m->bf16 ? 4 : 1);
    const size_t MB = (size_t)cfg->max_batch;
    for (size_t t = 0; t < T; ++t) {
        if (m->tasks[t].n_layers > 0 && m->tasks[t].head == MT_HEAD_TOKEN) {   // every layer runs on all rows
            m->task_scr.push_back(layout_scratch(sb, M, H, F, m->esz, m->bf16, 1));
            m->task_xf.push_back(sb.take(M * H * 4));
            m->task_xb.push_back(m->bf16 ? sb.take(M * H * 2) : 0);
            m->task_cls.push_back(ClsScratch{});
        } else if (m->tasks[t].n_layers > 0) {
            m->task_scr.push_back(layout_scratch(sb, M, H, F, m->esz, m->bf16, 1));
            m->task_xf.push_back(sb.take(M * H * 4));
            m->task_xb.push_back(m->bf16 ? sb.take(M * H * 2) : 0);
            ClsScratch c;
            c.in_f = sb.take(MB * H * 4);
            c.in_a = m->bf16 ? sb.take(MB * H * 2) : c.in_f;
            c.q = sb.take(MB * H * m->esz);
            c.ctx = sb.take(MB * H * m->esz);
            c.y = sb.take(4 * MB * H * 4);
            c.x1f = sb.take(MB * H * 4);
            c.x1a = m->bf16 ? sb.take(MB * H * 2) : c.x1f;
            c.u = sb.take(MB * F * m->esz);
            c.out_f = sb.take(MB * H * 4);
            if (m->bf16) {
                const size_t A_pad = ((size_t)cfg->heads + 3) / 4 * 4;
                c.qt = sb.take(MB * A_pad * H * 2);
                c.scores = sb.take(M * A_pad * 4);
                c.xbar = sb.take(MB * A_pad * H * 2);
            }
            m->task_cls.push_back(c);
        } else {
            m->task_scr.push_back(Scratch{});
            m->task_xf.push_back(sb.take(M * H * 4));          // only per-sequence routing uses it: the sub-batch's tap rows
            m->task_xb.push_back(m->bf16 ? sb.take(M * H * 2) : 0);
            m->task_cls.push_back(ClsScratch{});
        }
    }
    for (size_t t = 0; t < T; ++t) {
        RouteMapOff r;
        r.n = sb.take(4);
        r.src = sb.take(M * 4);
        r.start = sb.take(MB * 4);
        r.len = sb.take(MB * 4);
        r.seq = sb.take(MB * 4);
        r.rowof = sb.take(M * 4);
        m->route.push_back(r);
    }
    m->rm_n = sb.take(4);
    m->rm_src = sb.take(M * 4);
    m->rm_rowof = sb.take(M * 4);
    m->rm_start = sb.take((size_t)cfg->max_batch * 4);
    m->rm_len = sb.take((size_t)cfg->max_batch * 4);
    m->pooled = sb.take(T * (size_t)cfg->max_batch * H * 4);
    m->cls_split = sb.take(T * (size_t)cfg->max_batch * H * 4);   // [hi | lo] bf16 halves, or float32 rows in the validation mode
    m->chk_count = sb.take(4);
    m->mr_ids = sb.take(M * 4);
    m->mr_mask = sb.take(M * 4);
    m->mr_logits = sb.take((size_t)cfg->max_batch * std::max(m->C_tot, 1) * 4);
    m->workspace_bytes = sb.off;
    m->task_loaded.assign(T, 0);
    m->last_enabled.assign(T, 0);
    *out = m;
    return MT_OK;
}

void mt_destroy(mt_model* m)
{
    if (!m) return;
    for (auto& r : m->prof) {
        if (r.owns_t0) (void)hipEventDestroy(r.t0);
        (void)hipEventDestroy(r.t1);
    }
    for (auto e : m->event_pool) (void)hipEventDestroy(e);
    for (auto st : m->aux_streams) (void)hipStreamDestroy(st);
    for (auto e : m->aux_join) (void)hipEventDestroy(e);
    if (m->aux_fork) (void)hipEventDestroy(m->aux_fork);
    delete m;
}

size_t mt_weight_bytes(const mt_model* m) { return m ? m->weight_bytes : 0; }
size_t mt_workspace_bytes(const mt_model* m) { return m ? m->workspace_bytes : 0; }
int mt_logit_offset(const mt_model* m, int32_t task)
{
    if (!m) return MT_ERR_NULL;
    if (task < 0 || task >= (int)m->tasks.size()) return MT_ERR_SHAPE;
    if (m->tasks[task].head != MT_HEAD_SEQUENCE) return MT_ERR_CONFIG;
    return m->logit_off[task];
}
int mt_n_logits(const mt_model* m) { return m ? m->C_tot : MT_ERR_NULL; }
int mt_token_logit_offset(const mt_model* m, int32_t task)
{
    if (!m) return MT_ERR_NULL;
    if (task < 0 || task >= (int)m->tasks.size()) return MT_ERR_SHAPE;
    if (m->tasks[task].head != MT_HEAD_TOKEN) return MT_ERR_CONFIG;
    return m->logit_off[task];
}
int mt_n_token_logits(const mt_model* m) { return m ? m->C_tok : MT_ERR_NULL; }
int mt_layer_count(const mt_model* m)
{
    if (!m) return MT_ERR_NULL;
    int n = m->cfg.n_trunk_layers;
    for (const auto& d : m->tasks) n += d.n_layers;
    return n;
}
int mt_schedule_steps(const mt_model* m, const uint8_t* h_task_mask)
{
    if (!m) return MT_ERR_NULL;
    int steps = 0;
    for (size_t t = 0; t < m->tasks.size(); ++t) {
        if (h_task_mask && !h_task_mask[t]) continue;
        steps = std::max(steps, m->tasks[t].fork_layer + m->tasks[t].n_layers);
    }
    return steps;
}

const char* mt_last_error(const mt_model* m) { return m ? m->err.c_str() : "null model"; }

int mt_bind(mt_model* m, void* d_weights, size_t weight_bytes, void* d_workspace, size_t workspace_bytes)
{
    if (!m) return MT_ERR_NULL;
    if (!d_weights || !d_workspace) return fail(m, MT_ERR_NULL, "mt_bind: null arena");
    if (weight_bytes < m->weight_bytes || workspace_bytes < m->workspace_bytes)
        return fail(m, MT_ERR_SHAPE, "mt_bind: arenas too small (need %zu weight bytes, %zu workspace bytes)", m->weight_bytes,
                    m->workspace_bytes);
    if (((uintptr_t)d_weights | (uintptr_t)d_workspace) % kAlign)
        return fail(m, MT_ERR_SHAPE, "mt_bind: arenas must be %zu-byte aligned", kAlign);
    m->d_w = static_cast<unsigned char*>(d_weights);
    m->d_ws = static_cast<unsigned char*>(d_workspace);
    m->trunk_loaded = false;
    std::fill(m->task_loaded.begin(), m->task_loaded.end(), 0);
    return MT_OK;
}

int mt_share_weights(mt_model* m, const mt_model* owner)
{
    if (!m || !owner) return MT_ERR_NULL;
    const mt_config &a = m->cfg, &b = owner->cfg;
    bool same = a.vocab == b.vocab && a.hidden == b.hidden && a.heads == b.heads && a.ffn == b.ffn && a.max_pos == b.max_pos &&
                a.type_vocab == b.type_vocab && a.n_trunk_layers == b.n_trunk_layers && a.n_tasks == b.n_tasks &&
                a.precision == b.precision && a.gelu == b.gelu && a.ln_eps == b.ln_eps && m->weight_bytes == owner->weight_bytes &&
                m->tasks.size() == owner->tasks.size();
    for (size_t t = 0; same && t < m->tasks.size(); ++t)
        same = m->tasks[t].fork_layer == owner->tasks[t].fork_layer && m->tasks[t].n_layers == owner->tasks[t].n_layers &&
               m->tasks[t].n_classes == owner->tasks[t].n_classes && m->tasks[t].head == owner->tasks[t].head;
    if (!same) return fail(m, MT_ERR_CONFIG, "mt_share_weights: the two models were created from different configurations");
    if (!m->d_w || m->d_w != owner->d_w) return fail(m, MT_ERR_STATE, "mt_share_weights: not bound to the owner's weight arena");
    if (m->d_ws == owner->d_ws) return fail(m, MT_ERR_STATE, "mt_share_weights: the replica needs a workspace of its own");
    bool any = owner->trunk_loaded;
    for (char c : owner->task_loaded) any = any || c;
    if (!any) return fail(m, MT_ERR_STATE, "mt_share_weights: owner has no weights loaded");
    m->trunk_loaded = owner->trunk_loaded;
    m->task_loaded = owner->task_loaded;
    for (size_t l = 0; l < m->trunk.size(); ++l) {                 // the storage scales live beside the layout
        m->trunk[l].inv_s1 = owner->trunk[l].inv_s1;
        m->trunk[l].inv_s2 = owner->trunk[l].inv_s2;
        m->trunk[l].inv_sqkv = owner->trunk[l].inv_sqkv;
        m->trunk[l].inv_so = owner->trunk[l].inv_so;
    }
    for (size_t t = 0; t < m->taskw.size(); ++t)
        for (size_t l = 0; l < m->taskw[t].layers.size(); ++l) {
            m->taskw[t].layers[l].inv_s1 = owner->taskw[t].layers[l].inv_s1;
            m->taskw[t].layers[l].inv_s2 = owner->taskw[t].layers[l].inv_s2;
            m->taskw[t].layers[l].inv_sqkv = owner->taskw[t].layers[l].inv_sqkv;
            m->taskw[t].layers[l].inv_so = owner->taskw[t].layers[l].inv_so;
        }
    return MT_OK;
}

int mt_load_weights(mt_model* m, int32_t scope, const void* h_blob, size_t nbytes, void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (!h_blob) return fail(m, MT_ERR_NULL, "mt_load_weights: null blob");
    if (!m->d_w) return fail(m, MT_ERR_STATE, "mt_load_weights: call mt_bind first");
    const int T = (int)m->tasks.size();
    if (scope < -1 || scope >= T) return fail(m, MT_ERR_BLOB, "mt_load_weights: scope %d out of range", scope);
    if (nbytes < 16) return fail(m, MT_ERR_BLOB, "mt_load_weights: blob shorter than its header");
    const unsigned char* hb = static_cast<const unsigned char*>(h_blob);
    int32_t hdr[3];
    memcpy(hdr, hb + 4, 12);
    if (memcmp(hb, "MTW1", 4) != 0) return fail(m, MT_ERR_BLOB, "mt_load_weights: bad magic");
    if (hdr[0] != scope) return fail(m, MT_ERR_BLOB, "mt_load_weights: blob is for scope %d, not %d", hdr[0], scope);
    const size_t H = m->cfg.hidden, F = m->cfg.ffn;
    const size_t lf = layer_floats(H, F);
    size_t want_floats, want_tensors;
    if (scope < 0) {
        want_floats = ((size_t)m->cfg.vocab + m->cfg.max_pos + m->cfg.type_vocab) * H + 2 * H + (size_t)m->cfg.n_trunk_layers * lf;
        want_tensors = 5 + 16 * (size_t)m->cfg.n_trunk_layers;
    } else {
        const mt_task_desc& d = m->tasks[scope];
        const bool seq_head = d.head == MT_HEAD_SEQUENCE;
        want_floats = (size_t)d.n_layers * lf + (seq_head ? H * H + H : 0) + (size_t)d.n_classes * H + d.n_classes;
        want_tensors = 16 * (size_t)d.n_layers + (seq_head ? 4 : 2);
    }
    if ((size_t)hdr[1] != want_tensors) return fail(m, MT_ERR_BLOB, "mt_load_weights: %d tensors, expected %zu", hdr[1], want_tensors);
    if (nbytes != 16 + want_floats * 4)
        return fail(m, MT_ERR_BLOB, "mt_load_weights: %zu bytes, expected %zu", nbytes, 16 + want_floats * 4);

    // the blob's float data may be unaligned in principle; copy through memcpy-safe access by aligning once
    std::vector<float> aligned;
    const float* p = reinterpret_cast<const float*>(hb + 16);
    if ((uintptr_t)p % 4) {
        aligned.resize(want_floats);
        memcpy(aligned.data(), hb + 16, want_floats * 4);
        p = aligned.data();
    }

    const size_t begin = scope < 0 ? 0 : m->taskw[scope].begin;
    const size_t end = scope < 0 ? m->w_trunk_end : m->taskw[scope].end;
    void* img_v = nullptr;
    if (hipHostMalloc(&img_v, end - begin, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        return fail(m, MT_ERR_HIP, "mt_load_weights: cannot allocate %zu bytes of pinned staging", end - begin);
    }
    unsigned char* img = static_cast<unsigned char*>(img_v);
    memset(img, 0, end - begin);
    auto at = [&](size_t off) { return img + (off - begin); };
    if (scope < 0) {
        put_matrix(at(m->w_word), p, (size_t)m->cfg.vocab * H, m->bf16); p += (size_t)m->cfg.vocab * H;
        put_matrix(at(m->w_pos), p, (size_t)m->cfg.max_pos * H, m->bf16); p += (size_t)m->cfg.max_pos * H;
        put_matrix(at(m->w_type), p, (size_t)m->cfg.type_vocab * H, m->bf16); p += (size_t)m->cfg.type_vocab * H;
        memcpy(at(m->w_embg), p, H * 4); p += H;
        memcpy(at(m->w_embb), p, H * 4); p += H;
        for (LayerW& L : m->trunk) p += stage_layer(m, L, p, img, begin);
    } else {
        TaskW& tw = m->taskw[scope];
        const size_t C = m->tasks[scope].n_classes;
        for (LayerW& L : tw.layers) p += stage_layer(m, L, p, img, begin);
        const bool seq_head = m->tasks[scope].head == MT_HEAD_SEQUENCE;
        if (!seq_head) {
            // a token-level scope carries no pooler
        } else if (m->bf16) {   // rows of [W | W]
            std::vector<uint16_t> row(H);
            for (size_t r = 0; r < H; ++r) {
                put_matrix(reinterpret_cast<unsigned char*>(row.data()), p + r * H, H, true);
                memcpy(at(tw.Wp) + r * 2 * H * 2, row.data(), H * 2);
                memcpy(at(tw.Wp) + r * 2 * H * 2 + H * 2, row.data(), H * 2);
            }
        } else {
            put_matrix(at(tw.Wp), p, H * H, false);
        }
        if (seq_head) {
            p += H * H;
            memcpy(at(tw.bp), p, H * 4); p += H;
        }
        put_matrix(at(tw.Wc), p, C * H, m->bf16); p += C * H;
        memcpy(at(tw.bc), p, C * 4); p += C;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    hipError_t e = hipMemcpyAsync(m->d_w + begin, img, end - begin, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipHostFree(img);
    if (e != hipSuccess) return fail(m, MT_ERR_HIP, "mt_load_weights: copy failed: %s", hipGetErrorString(e));
    if (scope < 0) m->trunk_loaded = true;
    else m->task_loaded[scope] = 1;
    return MT_OK;
}

// The forward pass.  h_route == NULL: every enabled task (h_task_mask) runs on every sequence, branches interleaved
// with the trunk.  h_route [batch][n_tasks]: per-sequence routing, a task runs on the sequences that ask for it.
// Streams and events for running routed groups side by side; false (and nothing kept) if the runtime refuses.
static bool ensure_aux_streams(mt_model* m)
{
    constexpr int kAux = 4;
    if (!m->aux_streams.empty()) return true;
    std::vector<hipStream_t> st;
    std::vector<hipEvent_t> ev;
    hipEvent_t fork = nullptr;
    bool ok = hipEventCreateWithFlags(&fork, hipEventDisableTiming) == hipSuccess;
    for (int j = 0; ok && j < kAux; ++j) {
        hipStream_t s = nullptr;
        hipEvent_t e = nullptr;
        ok = hipStreamCreateWithFlags(&s, hipStreamNonBlocking) == hipSuccess;      // default priority
        if (ok) st.push_back(s);
        ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
        if (ok) ev.push_back(e);
    }
    if (!ok) {
        (void)hipGetLastError();
        for (auto s : st) (void)hipStreamDestroy(s);
        for (auto e : ev) (void)hipEventDestroy(e);
        if (fork) (void)hipEventDestroy(fork);
        return false;
    }
    m->aux_streams = st;
    m->aux_join = ev;
    m->aux_fork = fork;
    return true;
}

static int forward_impl(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask,
                        int32_t batch, int32_t seq, const uint8_t* h_task_mask, const uint8_t* h_route, float* d_out_logits,
                        float* d_out_token_logits, void* hip_stream, unsigned char* ws_other = nullptr)
{
    if (!m) return MT_ERR_NULL;
    if (!d_input_ids || !d_attn_mask) return fail(m, MT_ERR_NULL, "mt_forward: null device pointer");
    if (!m->d_w || !m->d_ws) return fail(m, MT_ERR_STATE, "mt_forward: call mt_bind first");
    if (batch < 1 || seq < 1 || batch > m->cfg.max_batch || seq > m->cfg.max_seq)
        return fail(m, MT_ERR_SHAPE, "mt_forward: batch %d x seq %d outside 1..%d x 1..%d", batch, seq, m->cfg.max_batch, m->cfg.max_seq);
    const int T = (int)m->tasks.size();
    if (h_route && batch > kMaxRouted) return fail(m, MT_ERR_SHAPE, "mt_forward_routed: at most %d sequences per call", kMaxRouted);
    std::vector<uint8_t> route_any;                     // routed mode: does any sequence ask for task t
    if (h_route) {
        route_any.assign(T, 0);
        for (int b = 0; b < batch; ++b)
            for (int t = 0; t < T; ++t) route_any[t] |= h_route[(size_t)b * T + t] ? 1 : 0;
        h_task_mask = route_any.data();
    }
    std::vector<int> enabled;
    int depth = 0, max_y = 0;
    for (int t = 0; t < T; ++t) {
        if (h_task_mask && !h_task_mask[t]) continue;
        if (!m->task_loaded[t]) return fail(m, MT_ERR_STATE, "mt_forward: task %d has no weights loaded", t);
        if (m->tasks[t].head == MT_HEAD_TOKEN) {
            if (!d_out_token_logits)
                return fail(m, MT_ERR_NULL, "mt_forward: task %d has a token-level head: pass a token logits buffer (mt_forward_tokens)", t);
        } else if (!d_out_logits) {
            return fail(m, MT_ERR_NULL, "mt_forward: null logits buffer");
        }
        enabled.push_back(t);
        depth = std::max(depth, m->tasks[t].fork_layer);
        max_y = std::max(max_y, m->tasks[t].n_layers);
    }
    if (!m->trunk_loaded) return fail(m, MT_ERR_STATE, "mt_forward: trunk has no weights loaded");
    std::fill(m->last_enabled.begin(), m->last_enabled.end(), 0);
    m->last_B = batch;
    m->last_S = seq;
    m->last_depth = -1;                 // no trunk state of this call exists (yet)
    m->ws_act = ws_other ? ws_other : m->d_ws;
    if (enabled.empty()) return MT_OK;
    m->last_depth = depth;

    const int B = batch, S = seq, H = m->cfg.hidden;
    unsigned char* W = m->d_w;
    unsigned char* ws = m->ws_act;
    const bool bf = m->bf16;
    Launcher L{m, static_cast<hipStream_t>(hip_stream)};

    // ---- embeddings -> X^(0)
    auto trunk_out = [&](int layer, int pp, float*& of, void*& ob) {
        const int tap = m->tap_of_layer[layer];
        if (tap >= 0) {
            of = (float*)(ws + m->tap_f[tap]);
            ob = bf ? (void*)(ws + m->tap_b[tap]) : nullptr;
        } else {
            of = (float*)(ws + m->pp_f[pp]);
            ob = bf ? (void*)(ws + m->pp_b[pp]) : nullptr;
        }
    };
    RowMap rm{(int32_t*)(ws + m->rm_n), (int32_t*)(ws + m->rm_src), (int32_t*)(ws + m->rm_rowof), (int32_t*)(ws + m->rm_start),
              (int32_t*)(ws + m->rm_len)};
    float* cur_f;
    void* cur_b;
    trunk_out(0, 0, cur_f, cur_b);
    L.begin(MT_K_EMBED);
    L.check(launch_build_row_map(d_attn_mask, B, S, rm, L.st));
    L.check(launch_embed_ln(d_input_ids, d_token_type_ids, m->cfg.type_vocab, rm.src, rm.n_rows, B, S, H, m->cfg.vocab, W + m->w_word, W + m->w_pos, W + m->w_type, bf ? 1 : 0,
                            (const float*)(W + m->w_embg), (const float*)(W + m->w_embb), m->cfg.ln_eps, cur_f,
                            (bf16_t*)cur_b, L.st));
    L.end();

    // ---- trunk and branches as one wavefront (Fig. 1(c)): step k evaluates trunk layer k+1 together with, for
    //      every task that forked at or before k, its own layer k - fork (if it has one), as ONE grouped launch
    //      sequence: a branch starts as soon as its tap exists instead of waiting for the whole trunk, so the
    //      number of sequential layer steps is max(D, max_t(fork_t + layers_t)) instead of D + max_t layers_t.
    //      A task's last own layer takes the first-token-only path.
    // routed mode: the trunk alone here, the branches follow per group of sequences
    const int n_steps = h_route ? depth : mt_schedule_steps(m, h_task_mask);      // >= depth: every fork is a fork + 0 layers bound
    (void)max_y;
    for (int step = 0; step < n_steps; ++step) {
        std::vector<LayerIO> full;
        std::vector<LastIO> last;
        float* nf = nullptr;
        void* nb = nullptr;
        if (step < depth) {
            trunk_out(step + 1, (step + 1) & 1, nf, nb);
            full.push_back(LayerIO{cur_f, cur_b, &m->trunk[step], &m->trunk_scr, nf, nb});
        }
        for (int t : enabled) {
            if (h_route) break;
            const mt_task_desc& d = m->tasks[t];
            const int stage = step - d.fork_layer;
            if (stage < 0 || stage >= d.n_layers) continue;
            const float* in_f;
            const void* in_b;
            if (stage == 0) {
                const int tap = m->tap_of_layer[d.fork_layer];
                in_f = (const float*)(ws + m->tap_f[tap]);
                in_b = bf ? (const void*)(ws + m->tap_b[tap]) : nullptr;
            } else {
                in_f = (const float*)(ws + m->task_xf[t]);
                in_b = bf ? (const void*)(ws + m->task_xb[t]) : nullptr;
            }
            if (stage == d.n_layers - 1 && d.head == MT_HEAD_SEQUENCE) {
                last.push_back(LastIO{in_f, bf ? in_b : (const void*)in_f, &m->taskw[t].layers[stage], &m->task_scr[t], &m->task_cls[t]});
            } else {
                full.push_back(LayerIO{in_f, in_b, &m->taskw[t].layers[stage], &m->task_scr[t], (float*)(ws + m->task_xf[t]),
                                       bf ? (void*)(ws + m->task_xb[t]) : nullptr});
            }
        }
        for (size_t lo = 0; lo < full.size(); lo += kMaxGroup) {
            std::vector<LayerIO> part(full.begin() + lo, full.begin() + std::min(full.size(), lo + (size_t)kMaxGroup));
            run_layer_group(L, part, rm, B, S);
        }
        for (size_t lo = 0; lo < last.size(); lo += kMaxGroup) {
            std::vector<LastIO> part(last.begin() + lo, last.begin() + std::min(last.size(), lo + (size_t)kMaxGroup));
            run_last_layer_group(L, part, rm, B, S);
        }
        if (step < depth) {
            cur_f = nf;
            cur_b = nb;
        }
    }

    // ---- poolers and classifiers.  The pooler input stays float32-accurate in both modes: the bf16
    // path feeds the matrix cores with the [hi | lo] split of the first-token rows against [W | W].
    auto run_heads = [&](Launcher& L, const std::vector<int>& all, const RowMap& hrm, int HB, bool gathered, const int32_t* out_row) {
    std::vector<int> list;
    for (int t : all)
        if (m->tasks[t].head == MT_HEAD_SEQUENCE) list.push_back(t);
    for (size_t lo = 0; lo < list.size(); lo += kMaxGroup) {
        const int n = (int)std::min(list.size() - lo, (size_t)kMaxGroup);
        GemmGroup g;
        memset(&g, 0, sizeof g);
        SplitGroup sg;
        memset(&sg, 0, sizeof sg);
        ClsGroup cg;
        memset(&cg, 0, sizeof cg);
        int maxC = 0;
        for (int i = 0; i < n; ++i) {
            const int t = list[lo + i];
            const mt_task_desc& d = m->tasks[t];
            const float* z = d.n_layers > 0 ? (const float*)(ws + m->task_cls[t].out_f)     // one row per sequence already
                             : gathered     ? (const float*)(ws + m->task_xf[t])          // the sub-batch's copy of the tap
                                            : (const float*)(ws + m->tap_f[m->tap_of_layer[d.fork_layer]]);
            float* pooled = (float*)(ws + m->pooled + (size_t)t * m->cfg.max_batch * H * 4);
            sg.x[i] = z;
            sg.compact[i] = d.n_layers > 0 ? 1 : 0;
            sg.out[i] = bf ? (bf16_t*)(ws + m->cls_split + (size_t)t * m->cfg.max_batch * 2 * H * 2)
                           : (bf16_t*)(ws + m->cls_split + (size_t)t * m->cfg.max_batch * H * 4);   // fp32 mode: float32 rows
            g.A[i] = bf ? (const void*)sg.out[i] : (const void*)(ws + m->cls_split + (size_t)t * m->cfg.max_batch * H * 4);
            g.W[i] = W + m->taskw[t].Wp;
            g.bias[i] = (const float*)(W + m->taskw[t].bp);
            g.C[i] = pooled;
            g.N[i] = H;
            cg.pooled[i] = pooled;
            cg.Wc[i] = W + m->taskw[t].Wc;
            cg.bc[i] = (const float*)(W + m->taskw[t].bc);
            cg.out[i] = d_out_logits + m->logit_off[t];
            cg.C[i] = d.n_classes;
            maxC = std::max(maxC, d.n_classes);
        }
        L.begin(MT_K_POOL);
        if (bf) {
            L.check(launch_cls_split(sg, n, HB, H, hrm.seq_start, S, HB * S, L.st));
            GemmShape s{n, HB, H, 2 * H, 2 * H, H, 0, ACT_TANH, 1, nullptr, 1, 0};
            L.check(launch_gemm_bf16(g, s, L.st));
        } else {
            L.check(launch_gather_rows(sg, n, HB, H, hrm.seq_start, S, HB * S, L.st));
            GemmShape s{n, HB, H, H, H, H, 0, ACT_TANH, 1, nullptr, 1, 0};
            L.check(launch_gemm_f32(g, s, 0, L.st));
        }
        L.check(launch_classifier(cg, n, HB, H, maxC, bf ? 1 : 0, m->C_tot, out_row, L.st));
        L.end();
    }
    };

    // ---- token-level heads: one linear layer on every kept row of the task's final state, scattered to [B][S][C_tok]
    auto run_token_heads = [&](Launcher& L, const std::vector<int>& all, bool gathered, const int32_t* pos_row, const int32_t* n_rows) {
        std::vector<int> list;
        for (int t : all)
            if (m->tasks[t].head == MT_HEAD_TOKEN) list.push_back(t);
        for (size_t lo = 0; lo < list.size(); lo += kMaxGroup) {
            const int n = (int)std::min(list.size() - lo, (size_t)kMaxGroup);
            TokGroup tg;
            memset(&tg, 0, sizeof tg);
            for (int i = 0; i < n; ++i) {
                const int t = list[lo + i];
                const mt_task_desc& d = m->tasks[t];
                tg.x[i] = (d.n_layers > 0 || gathered) ? (const float*)(ws + m->task_xf[t])
                                                       : (const float*)(ws + m->tap_f[m->tap_of_layer[d.fork_layer]]);
                tg.Wc[i] = W + m->taskw[t].Wc;
                tg.bc[i] = (const float*)(W + m->taskw[t].bc);
                tg.out[i] = d_out_token_logits + m->logit_off[t];
                tg.C[i] = d.n_classes;
            }
            L.begin(MT_K_POOL);
            L.check(launch_token_classifier(tg, n, B * S, H, bf ? 1 : 0, m->C_tok, pos_row, n_rows, L.st));
            L.end();
        }
    };

    if (!h_route) {
        run_heads(L, enabled, rm, B, false, nullptr);
        run_token_heads(L, enabled, false, rm.row_of, rm.n_rows);
    } else {
        // ---- per-sequence routing: tasks wanted by the same set of sequences form a group; the group's sequences are
        // gathered from each task's tap into a padding-free row order of their own, on which the task's layers,
        // pooler and classifier run exactly as on a whole batch; logits land in the rows of the chosen sequences.
        struct Group {
            std::vector<int> tasks;
            int t0;
        };
        std::vector<Group> groups;
        std::vector<char> done(T, 0);
        for (int t0 : enabled) {
            if (done[t0]) continue;
            Group grp;
            grp.t0 = t0;
            for (int t : enabled) {
                if (done[t]) continue;
                bool same = true;
                for (int b = 0; b < B && same; ++b) same = (h_route[(size_t)b * T + t] != 0) == (h_route[(size_t)b * T + t0] != 0);
                if (same) {
                    grp.tasks.push_back(t);
                    done[t] = 1;
                }
            }
            groups.push_back(std::move(grp));
        }
        // Groups touch disjoint scratch (per task) and disjoint logits, and only read the trunk's taps and the batch's
        // row map: with more than one group they are issued round-robin to the model's own streams, which wait for
        // the trunk through one event and are joined back into the caller's stream at the end.  Per-launch timing
        // (mt_profile_enable) keeps everything on the caller's stream.
        const bool side = groups.size() > 1 && !m->profiling && ensure_aux_streams(m);
        const int n_side = side ? (int)std::min(groups.size(), m->aux_streams.size()) : 0;
        if (side) {
            L.check(hipEventRecord(m->aux_fork, L.st));
            for (int j = 0; j < n_side; ++j) L.check(hipStreamWaitEvent(m->aux_streams[j], m->aux_fork, 0));
        }
        for (size_t gi = 0; gi < groups.size(); ++gi) {
            const std::vector<int>& grp_tasks = groups[gi].tasks;
            const int t0 = groups[gi].t0;
            Launcher LS{m, side ? m->aux_streams[gi % n_side] : L.st};
            Launcher& GL = side ? LS : L;
            RouteIdx idx;
            int nb = 0;
            for (int b = 0; b < B; ++b)
                if (h_route[(size_t)b * T + t0]) idx.seq[nb++] = (uint16_t)b;
            const RouteMapOff& ro = m->route[t0];
            RowMap crm{(int32_t*)(ws + ro.n), (int32_t*)(ws + ro.src), nullptr, (int32_t*)(ws + ro.start), (int32_t*)(ws + ro.len)};
            int32_t* c_seq = (int32_t*)(ws + ro.seq);
            GL.begin(MT_K_EMBED);
            GL.check(launch_route_map(idx, nb, rm.seq_start, rm.seq_len, crm.seq_start, crm.seq_len, crm.src, c_seq, crm.n_rows, GL.st));
            for (int t : grp_tasks) {
                const int tap = m->tap_of_layer[m->tasks[t].fork_layer];
                GL.check(launch_route_gather((const float*)(ws + m->tap_f[tap]), bf ? (const void*)(ws + m->tap_b[tap]) : nullptr,
                                             (float*)(ws + m->task_xf[t]), bf ? (void*)(ws + m->task_xb[t]) : nullptr, crm.src, crm.n_rows,
                                             nb * S, H, 2, GL.st));
            }
            GL.end();
            int gy = 0;
            for (int t : grp_tasks) gy = std::max(gy, m->tasks[t].n_layers);
            for (int stage = 0; stage < gy; ++stage) {
                std::vector<LayerIO> full;
                std::vector<LastIO> last;
                for (int t : grp_tasks) {
                    const mt_task_desc& d = m->tasks[t];
                    if (stage >= d.n_layers) continue;
                    const float* in_f = (const float*)(ws + m->task_xf[t]);
                    const void* in_b = bf ? (const void*)(ws + m->task_xb[t]) : nullptr;
                    if (stage == d.n_layers - 1 && d.head == MT_HEAD_SEQUENCE)
                        last.push_back(LastIO{in_f, bf ? in_b : (const void*)in_f, &m->taskw[t].layers[stage], &m->task_scr[t], &m->task_cls[t]});
                    else
                        full.push_back(LayerIO{in_f, in_b, &m->taskw[t].layers[stage], &m->task_scr[t], (float*)(ws + m->task_xf[t]),
                                               bf ? (void*)(ws + m->task_xb[t]) : nullptr});
                }
                for (size_t lo = 0; lo < full.size(); lo += kMaxGroup) {
                    std::vector<LayerIO> part(full.begin() + lo, full.begin() + std::min(full.size(), lo + (size_t)kMaxGroup));
                    run_layer_group(GL, part, crm, nb, S);
                }
                for (size_t lo = 0; lo < last.size(); lo += kMaxGroup) {
                    std::vector<LastIO> part(last.begin() + lo, last.begin() + std::min(last.size(), lo + (size_t)kMaxGroup));
                    run_last_layer_group(GL, part, crm, nb, S);
                }
            }
            run_heads(GL, grp_tasks, crm, nb, true, c_seq);
            bool any_token = false;
            for (int t : grp_tasks) any_token = any_token || m->tasks[t].head == MT_HEAD_TOKEN;
            if (any_token) {
                // token-level heads: logits of the group's real tokens go to their own positions of [B][S][C_tok], zeros to
                // the padded positions of its sequences, nothing to the other sequences
                int32_t* c_rowof = (int32_t*)(ws + ro.rowof);
                GL.begin(MT_K_POOL);
                GL.check(launch_route_rowof(idx, nb, B, S, rm.row_of, rm.seq_start, crm.seq_start, c_rowof, GL.st));
                GL.end();
                run_token_heads(GL, grp_tasks, true, c_rowof, crm.n_rows);
            }
            if (side) L.check(LS.first_err);
        }
        if (side) {
            for (int j = 0; j < n_side; ++j) {
                L.check(hipEventRecord(m->aux_join[j], m->aux_streams[j]));
                L.check(hipStreamWaitEvent(L.st, m->aux_join[j], 0));
            }
        }
    }

    if (L.first_err != hipSuccess) return fail(m, MT_ERR_HIP, "mt_forward: launch failed: %s", hipGetErrorString(L.first_err));
    if (!h_route)            // after a routed forward a task's state covers its own sub-batch only: not readable
        for (int t : enabled) m->last_enabled[t] = 1;
    return MT_OK;
}

int mt_forward_typed(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask, int32_t batch,
                     int32_t seq, const uint8_t* h_task_mask, float* d_out_logits, void* hip_stream)
{
    return forward_impl(m, d_input_ids, d_token_type_ids, d_attn_mask, batch, seq, h_task_mask, nullptr, d_out_logits, nullptr,
                        hip_stream);
}

int mt_forward_tokens(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask,
                      int32_t batch, int32_t seq, const uint8_t* h_task_mask, float* d_out_logits, float* d_out_token_logits,
                      void* hip_stream)
{
    return forward_impl(m, d_input_ids, d_token_type_ids, d_attn_mask, batch, seq, h_task_mask, nullptr, d_out_logits,
                        d_out_token_logits, hip_stream);
}

int mt_forward(mt_model* m, const int32_t* d_input_ids, const int32_t* d_attn_mask, int32_t batch, int32_t seq,
               const uint8_t* h_task_mask, float* d_out_logits, void* hip_stream)
{
    return forward_impl(m, d_input_ids, nullptr, d_attn_mask, batch, seq, h_task_mask, nullptr, d_out_logits, nullptr, hip_stream);
}

int mt_forward_requests(mt_model* m, int32_t n_requests, const int32_t* const* h_d_input_ids, const int32_t* const* h_d_attn_mask,
                        const int32_t* h_batch, int32_t seq, const uint8_t* h_task_mask, float* const* h_d_out_logits, void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (!h_d_input_ids || !h_d_attn_mask || !h_d_out_logits || !h_batch) return fail(m, MT_ERR_NULL, "mt_forward_requests: null table");
    if (n_requests < 1 || n_requests > kMaxRequests)
        return fail(m, MT_ERR_SHAPE, "mt_forward_requests: %d requests, at most %d per call", n_requests, kMaxRequests);
    RequestPtrs rq;
    memset(&rq, 0, sizeof rq);
    int64_t total = 0;
    int largest = 0;
    for (int r = 0; r < n_requests; ++r) {
        if (h_batch[r] < 1) return fail(m, MT_ERR_SHAPE, "mt_forward_requests: request %d has batch %d", r, h_batch[r]);
        rq.first[r] = (int32_t)total;
        total += h_batch[r];
        largest = std::max(largest, (int)h_batch[r]);
        if (total > m->cfg.max_batch) break;
    }
    if (seq < 1 || total > m->cfg.max_batch || seq > m->cfg.max_seq)
        return fail(m, MT_ERR_SHAPE, "mt_forward_requests: %d requests with %lld sequences in all x seq %d outside max_batch %d x max_seq %d",
                    n_requests, (long long)total, seq, m->cfg.max_batch, m->cfg.max_seq);
    rq.first[n_requests] = (int32_t)total;
    if (m->C_tot > kMaxLogitCols) return fail(m, MT_ERR_CONFIG, "mt_forward_requests: more than %d logit columns", kMaxLogitCols);
    if (!m->d_w || !m->d_ws) return fail(m, MT_ERR_STATE, "mt_forward_requests: call mt_bind first");
    for (int r = 0; r < n_requests; ++r) {
        if (!h_d_input_ids[r] || !h_d_attn_mask[r] || !h_d_out_logits[r])
            return fail(m, MT_ERR_NULL, "mt_forward_requests: request %d has a null device pointer", r);
        rq.ids[r] = h_d_input_ids[r];
        rq.mask[r] = h_d_attn_mask[r];
        rq.out[r] = h_d_out_logits[r];
    }
    for (size_t t = 0; t < m->tasks.size(); ++t) {
        if (h_task_mask && !h_task_mask[t]) continue;
        if (m->tasks[t].head == MT_HEAD_TOKEN)
            return fail(m, MT_ERR_CONFIG, "mt_forward_requests: task %zu has a token-level head (use mt_forward_tokens per request)", t);
        for (int c = m->logit_off[t]; c < m->logit_off[t] + m->tasks[t].n_classes; ++c) rq.col_on[c >> 5] |= 1u << (c & 31);
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int32_t* ids_all = (int32_t*)(m->d_ws + m->mr_ids);
    int32_t* mask_all = (int32_t*)(m->d_ws + m->mr_mask);
    float* logits_all = (float*)(m->d_ws + m->mr_logits);
    hipError_t e = launch_gather_requests(rq, n_requests, largest, seq, ids_all, mask_all, st);
    if (e != hipSuccess) return fail(m, MT_ERR_HIP, "mt_forward_requests: %s", hipGetErrorString(e));
    const int rc = forward_impl(m, ids_all, nullptr, mask_all, (int)total, seq, h_task_mask, nullptr, logits_all, nullptr, hip_stream);
    if (rc != MT_OK) return rc;
    e = launch_scatter_logits(rq, n_requests, largest, m->C_tot, logits_all, st);
    if (e != hipSuccess) return fail(m, MT_ERR_HIP, "mt_forward_requests: %s", hipGetErrorString(e));
    return MT_OK;
}

int mt_forward_multi(mt_model* m, int32_t n_requests, const int32_t* const* h_d_input_ids, const int32_t* const* h_d_attn_mask,
                     int32_t batch, int32_t seq, const uint8_t* h_task_mask, float* const* h_d_out_logits, void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (n_requests < 1 || n_requests > kMaxRequests)
        return fail(m, MT_ERR_SHAPE, "mt_forward_multi: %d requests, at most %d per call", n_requests, kMaxRequests);
    if (batch < 1) return fail(m, MT_ERR_SHAPE, "mt_forward_multi: batch %d", batch);
    int32_t sizes[kMaxRequests];
    for (int r = 0; r < n_requests; ++r) sizes[r] = batch;
    return mt_forward_requests(m, n_requests, h_d_input_ids, h_d_attn_mask, sizes, seq, h_task_mask, h_d_out_logits, hip_stream);
}

// ---- the forward pass for callers that must not allocate: its workspace is a fixed array in device memory that is
// part of the loaded code object (every GPU the library runs on holds its own copy until the process ends).
// MT_STATIC_SCRATCH_BYTES is declared in mt.h.  Host code never uses the array's name as an address: the name is a
// host-side stand-in, and the per-device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char mt_static_scratch[MT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of the array, or nullptr with *err set.
unsigned char* static_scratch_of_current_device(hipError_t* err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(mt_static_scratch));
        if (*err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int mt_forward_static(mt_model* m, const int32_t* d_input_ids, const int32_t* d_attn_mask, int32_t batch, int32_t seq,
                      const uint8_t* h_task_mask, float* d_out_logits, void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (m->workspace_bytes > (size_t)MT_STATIC_SCRATCH_BYTES)
        return fail(m, MT_ERR_SHAPE,
                    "mt_forward_static: this model's workspace (max_batch %d x max_seq %d: %zu bytes) exceeds the static scratch of %zu "
                    "bytes; create the model with smaller bounds or use mt_forward",
                    m->cfg.max_batch, m->cfg.max_seq, m->workspace_bytes, (size_t)MT_STATIC_SCRATCH_BYTES);
    if (m->profiling) return fail(m, MT_ERR_STATE, "mt_forward_static: per-launch timing creates events; switch mt_profile_enable off");
    hipError_t e = hipSuccess;
    unsigned char* scratch = static_scratch_of_current_device(&e);
    if (!scratch) return fail(m, MT_ERR_HIP, "mt_forward_static: static scratch address: %s", hipGetErrorString(e));
    return forward_impl(m, d_input_ids, nullptr, d_attn_mask, batch, seq, h_task_mask, nullptr, d_out_logits, nullptr, hip_stream, scratch);
}

int mt_forward_routed(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask, int32_t batch,
                      int32_t seq, const uint8_t* h_route, float* d_out_logits, void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (!h_route) return fail(m, MT_ERR_NULL, "mt_forward_routed: null routing table");
    return forward_impl(m, d_input_ids, d_token_type_ids, d_attn_mask, batch, seq, nullptr, h_route, d_out_logits, nullptr, hip_stream);
}

int mt_forward_routed_tokens(mt_model* m, const int32_t* d_input_ids, const int32_t* d_token_type_ids, const int32_t* d_attn_mask,
                             int32_t batch, int32_t seq, const uint8_t* h_route, float* d_out_logits, float* d_out_token_logits,
                             void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (!h_route) return fail(m, MT_ERR_NULL, "mt_forward_routed_tokens: null routing table");
    return forward_impl(m, d_input_ids, d_token_type_ids, d_attn_mask, batch, seq, nullptr, h_route, d_out_logits, d_out_token_logits,
                        hip_stream);
}

int mt_check_mask(mt_model* m, const int32_t* d_attn_mask, int32_t batch, int32_t seq, int32_t* h_bad_sequences, void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (!d_attn_mask || !h_bad_sequences) return fail(m, MT_ERR_NULL, "mt_check_mask: null pointer");
    if (!m->d_ws) return fail(m, MT_ERR_STATE, "mt_check_mask: call mt_bind first");
    if (batch < 1 || seq < 1) return fail(m, MT_ERR_SHAPE, "mt_check_mask: batch %d x seq %d", batch, seq);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int32_t* d_count = (int32_t*)(m->d_ws + m->chk_count);
    hipError_t e = launch_count_bad_first_tokens(d_attn_mask, batch, seq, d_count, st);
    if (e == hipSuccess) e = hipMemcpyAsync(h_bad_sequences, d_count, 4, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(m, MT_ERR_HIP, "mt_check_mask: %s", hipGetErrorString(e));
    if (*h_bad_sequences != 0)
        return fail(m, MT_ERR_SHAPE, "mt_check_mask: %d of %d sequences have no real token at position 0 (the task heads read it)",
                    *h_bad_sequences, batch);
    return MT_OK;
}

int mt_read_hidden(mt_model* m, int32_t task, int32_t layer, float* d_out, size_t out_bytes, void* hip_stream)
{
    if (!m) return MT_ERR_NULL;
    if (!d_out) return fail(m, MT_ERR_NULL, "mt_read_hidden: null output");
    if (!m->ws_act || m->last_B == 0) return fail(m, MT_ERR_STATE, "mt_read_hidden: no forward pass has run");
    const size_t bytes = (size_t)m->last_B * m->last_S * m->cfg.hidden * 4;
    if (out_bytes < bytes) return fail(m, MT_ERR_SHAPE, "mt_read_hidden: need %zu bytes", bytes);
    const unsigned char* src;
    if (task < 0) {
        if (layer < 0 || layer > m->cfg.n_trunk_layers || m->tap_of_layer[layer] < 0)
            return fail(m, MT_ERR_SHAPE, "mt_read_hidden: no task forks at trunk layer %d", layer);
        if (layer > m->last_depth)
            return fail(m, MT_ERR_STATE, "mt_read_hidden: the last forward pass ran the trunk to layer %d only, not to layer %d",
                        m->last_depth, layer);
        src = m->ws_act + m->tap_f[m->tap_of_layer[layer]];
    } else {
        if (task >= (int)m->tasks.size()) return fail(m, MT_ERR_SHAPE, "mt_read_hidden: task %d out of range", task);
        if (!m->last_enabled[task]) return fail(m, MT_ERR_STATE, "mt_read_hidden: task %d was not computed", task);
        const mt_task_desc& d = m->tasks[task];
        if (d.n_layers > 0 && d.head == MT_HEAD_TOKEN) {
            src = m->ws_act + m->task_xf[task];
        } else if (d.n_layers > 0) {   // only the first-token rows of a branch's final state exist
            hipError_t e = launch_place_first_rows((const float*)(m->ws_act + m->task_cls[task].out_f), m->last_B, m->last_S,
                                                   m->cfg.hidden, d_out, static_cast<hipStream_t>(hip_stream));
            if (e != hipSuccess) return fail(m, MT_ERR_HIP, "mt_read_hidden: %s", hipGetErrorString(e));
            return MT_OK;
        } else {
            src = m->ws_act + m->tap_f[m->tap_of_layer[d.fork_layer]];
        }
    }
    hipError_t e = launch_unpack_rows((const float*)src, (const int32_t*)(m->ws_act + m->rm_rowof), m->last_B * m->last_S, m->cfg.hidden,
                                      d_out, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(m, MT_ERR_HIP, "mt_read_hidden: %s", hipGetErrorString(e));
    return MT_OK;
}

int mt_profile_enable(mt_model* m, int32_t on)
{
    if (!m) return MT_ERR_NULL;
    m->profiling = on != 0;
    return MT_OK;
}

int mt_profile_read(mt_model* m, float* h_ms, int32_t* h_launches)
{
    if (!m) return MT_ERR_NULL;
    if (!h_ms || !h_launches) return fail(m, MT_ERR_NULL, "mt_profile_read: null output");
    for (int k = 0; k < MT_K_COUNT; ++k) {
        h_ms[k] = 0.f;
        h_launches[k] = 0;
    }
    int rc = MT_OK;
    for (auto& r : m->prof) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.t1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.t0, r.t1);
        if (e != hipSuccess) rc = fail(m, MT_ERR_HIP, "mt_profile_read: %s", hipGetErrorString(e));
        else {
            h_ms[r.klass] += ms;
            h_launches[r.klass] += 1;
        }
    }
    for (auto& r : m->prof) {
        if (r.owns_t0) m->event_pool.push_back(r.t0);
        m->event_pool.push_back(r.t1);
    }
    m->prof.clear();
    return rc;
}

int mt_debug_mfma_peak(int32_t iters, void* d_scratch, size_t scratch_bytes, float* h_tflops, void* hip_stream)
{
    if (!d_scratch || !h_tflops) return MT_ERR_NULL;
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
        return MT_ERR_HIP;
    if (iters < 1 || scratch_bytes < (size_t)mfma_rate_out_floats(n_cu) * 4) return MT_ERR_SHAPE;
    return run_mfma_rate(iters, n_cu, static_cast<float*>(d_scratch), static_cast<hipStream_t>(hip_stream), h_tflops) == hipSuccess ? MT_OK
                                                                                                                       : MT_ERR_HIP;
}

int mt_debug_set_gemm_tile(int32_t sel)
{
    const int prev = mt::g_gemm_bf16_tile_override;
    mt::g_gemm_bf16_tile_override = (sel >= 0 && sel <= 27) ? sel : 0;
    return prev;
}

int mt_op_linear(int32_t precision, const void* d_A, int64_t lda, const void* d_W, const float* d_bias,
                 const float* d_residual, void* d_C, int64_t ldc, int32_t M, int32_t N, int32_t K, int32_t act_kind,
                 int32_t out_f32, void* hip_stream)
{
    if (!d_A || !d_W || !d_C) return MT_ERR_NULL;
    if (M < 1 || N < 1 || K < 1 || act_kind < 0 || act_kind > 3) return MT_ERR_SHAPE;
    GemmGroup g;
    memset(&g, 0, sizeof g);
    g.A[0] = d_A;
    g.W[0] = d_W;
    g.C[0] = d_C;
    g.bias[0] = d_bias;
    g.residual[0] = d_residual;
    g.N[0] = N;
    GemmShape s{1, M, N, K, lda, ldc, ldc, act_kind, (precision == MT_BF16) ? (out_f32 ? 1 : 0) : 1, nullptr, 1, 0};
    hipError_t e = precision == MT_BF16 ? launch_gemm_bf16(g, s, static_cast<hipStream_t>(hip_stream))
                                        : launch_gemm_f32(g, s, 0, static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidValue) return MT_ERR_SHAPE;
    return e == hipSuccess ? MT_OK : MT_ERR_HIP;
}

int mt_op_linear_fp8(const void* d_A, int64_t lda, const void* d_W, float scale, const float* d_bias, const float* d_residual,
                     void* d_C, int64_t ldc, int32_t M, int32_t N, int32_t K, int32_t act_kind, int32_t out_kind, float out_scale,
                     void* hip_stream)
{
    if (!d_A || !d_W || !d_C) return MT_ERR_NULL;
    if (M < 1 || N < 1 || K < 1 || act_kind < 0 || act_kind > 2 || out_kind < 0 || out_kind > 2) return MT_ERR_SHAPE;
    GemmGroup g;
    memset(&g, 0, sizeof g);
    g.A[0] = d_A;
    g.W[0] = d_W;
    g.C[0] = d_C;
    g.bias[0] = d_bias;
    g.residual[0] = d_residual;
    g.N[0] = N;
    g.scale[0] = scale;
    GemmShape s{1, M, N, K, lda, ldc, ldc, act_kind, out_kind, nullptr, 1, 0};
    s.out_scale = out_scale;
    hipError_t e = launch_gemm_fp8(g, s, static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidValue) return MT_ERR_SHAPE;
    return e == hipSuccess ? MT_OK : MT_ERR_HIP;
}

float mt_debug_e4m3_quantize(const float* h_w, size_t n, uint8_t* h_out)
{
    if (!h_w) return 0.f;
    const float sc = e4m3_scale_for(h_w, n);
    if (h_out)
        for (size_t i = 0; i < n; ++i) h_out[i] = f32_to_e4m3_rne(h_w[i] * sc);
    return sc;
}

int mt_op_linear_sub(const void* d_A, int64_t lda, const void* d_W, int64_t ldw, const float* d_bias, void* d_C, int64_t ldc,
                     int32_t M, int32_t N, int32_t K, int32_t n_sub, int64_t sub_a, int64_t sub_w, int64_t sub_c,
                     int64_t sub_bias, const int32_t* d_sub_row0, const int32_t* d_sub_rows, int32_t out_f32,
                     void* hip_stream)
{
    if (!d_A || !d_W || !d_C) return MT_ERR_NULL;
    if (M < 1 || N < 1 || K < 1 || n_sub < 1 || (d_sub_row0 == nullptr) != (d_sub_rows == nullptr)) return MT_ERR_SHAPE;
    GemmGroup g;
    memset(&g, 0, sizeof g);
    g.A[0] = d_A;
    g.W[0] = d_W;
    g.C[0] = d_C;
    g.bias[0] = d_bias;
    g.N[0] = N;
    GemmShape s{1, M, N, K, lda, ldc, 0, ACT_NONE, out_f32 ? 1 : 0, nullptr, 1, 0, ldw};
    s.n_sub = n_sub;
    s.sub_a = sub_a;
    s.sub_w = sub_w;
    s.sub_c = sub_c;
    s.sub_bias = sub_bias;
    s.d_sub_row0 = d_sub_row0;
    s.d_sub_rows = d_sub_rows;
    hipError_t e = launch_gemm_skinny_bf16(g, s, static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidValue) return MT_ERR_SHAPE;
    return e == hipSuccess ? MT_OK : MT_ERR_HIP;
}

int mt_op_first_token_pool(const float* d_scores, const void* d_x, void* d_xbar, const int32_t* d_seq_start,
                           const int32_t* d_seq_len, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                           int32_t heads_pad, void* hip_stream)
{
    if (!d_scores || !d_x || !d_xbar || !d_seq_start || !d_seq_len) return MT_ERR_NULL;
    if (batch < 1 || seq < 1 || hidden < 2 || heads < 1 || hidden % heads != 0) return MT_ERR_SHAPE;
    PoolGroup pg;
    memset(&pg, 0, sizeof pg);
    pg.scores[0] = d_scores;
    pg.x[0] = d_x;
    pg.xbar[0] = d_xbar;
    hipError_t e = launch_first_token_pool(pg, 1, d_seq_start, d_seq_len, batch, seq, hidden, heads, heads_pad,
                                           static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidValue) return MT_ERR_SHAPE;
    return e == hipSuccess ? MT_OK : MT_ERR_HIP;
}

int mt_op_linear_batched(int32_t precision, int32_t G, const void* d_A, int64_t strideA, int64_t lda, const void* d_W,
                         int64_t strideW, const float* d_bias, int64_t strideBias, const float* d_residual,
                         int64_t strideRes, void* d_C, int64_t strideC, int64_t ldc, int32_t M, int32_t N, int32_t K,
                         int32_t act_kind, int32_t out_f32, void* hip_stream)
{
    if (!d_A || !d_W || !d_C) return MT_ERR_NULL;
    if (G < 1 || G > kMaxGroup || M < 1 || N < 1 || K < 1 || act_kind < 0 || act_kind > 3) return MT_ERR_SHAPE;
    const bool bf = precision == MT_BF16;
    const size_t esz = bf ? 2 : 4;
    const int of32 = bf ? (out_f32 ? 1 : 0) : 1;
    GemmGroup g;
    memset(&g, 0, sizeof g);
    for (int i = 0; i < G; ++i) {
        g.A[i] = static_cast<const unsigned char*>(d_A) + (size_t)i * strideA * esz;
        g.W[i] = static_cast<const unsigned char*>(d_W) + (size_t)i * strideW * esz;
        g.C[i] = static_cast<unsigned char*>(d_C) + (size_t)i * strideC * (of32 ? 4 : 2);
        g.bias[i] = d_bias ? d_bias + (size_t)i * strideBias : nullptr;
        g.residual[i] = d_residual ? d_residual + (size_t)i * strideRes : nullptr;
        g.N[i] = N;
    }
    GemmShape s{G, M, N, K, lda, ldc, ldc, act_kind, of32, nullptr, 1, 0};
    hipError_t e = bf ? launch_gemm_bf16(g, s, static_cast<hipStream_t>(hip_stream))
                      : launch_gemm_f32(g, s, 0, static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidValue) return MT_ERR_SHAPE;
    return e == hipSuccess ? MT_OK : MT_ERR_HIP;
}

int mt_op_attention(int32_t precision, const void* d_qkv, const int32_t* d_mask, void* d_ctx, int32_t batch, int32_t seq,
                    int32_t hidden, int32_t heads, void* hip_stream)
{
    if (!d_qkv || !d_mask || !d_ctx) return MT_ERR_NULL;
    if (batch < 1 || seq < 1 || heads < 1 || hidden % heads) return MT_ERR_SHAPE;
    AttnGroup g;
    memset(&g, 0, sizeof g);
    g.qkv[0] = d_qkv;
    g.ctx[0] = d_ctx;
    hipError_t e = precision == MT_BF16
                       ? launch_attention_bf16(g, 1, d_mask, nullptr, nullptr, batch, seq, hidden, heads, static_cast<hipStream_t>(hip_stream))
                       : launch_attention_f32(g, 1, d_mask, nullptr, nullptr, batch, seq, hidden, heads, static_cast<hipStream_t>(hip_stream));
    if (e == hipErrorInvalidValue) return MT_ERR_SHAPE;
    return e == hipSuccess ? MT_OK : MT_ERR_HIP;
}

int mt_op_layernorm(const float* d_x, const float* d_gamma, const float* d_beta, float eps, float* d_out_f32, void* d_out_bf16,
                    int32_t M, int32_t H, void* hip_stream)
{
    if (!d_x || !d_gamma || !d_beta) return MT_ERR_NULL;
    if (M < 1 || H < 1) return MT_ERR_SHAPE;
    LnGroup g;
    memset(&g, 0, sizeof g);
    g.x[0] = d_x;
    g.gamma[0] = d_gamma;
    g.beta[0] = d_beta;
    g.out_f32[0] = d_out_f32;
    g.out_bf16[0] = static_cast<bf16_t*>(d_out_bf16);
    hipError_t e = launch_layernorm(g, 1, M, nullptr, H, eps, 1, 0, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MT_OK : MT_ERR_HIP;
}

}  // extern "C"
