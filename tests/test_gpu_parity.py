"""Parity of the HIP library against the CPU oracle, through the C ABI, on a real MI355X.

Tolerances.  float32 validation mode: per task max|g-o| <= 1e-4 * max(max|o|, 1e-3).  bf16 mode:
max |delta logit| <= 2e-2; every (sequence, task) pair whose oracle top-2 margin exceeds 4e-2 must
have the same argmax (a consequence of the 2e-2 bound); ties break to the lowest index on both sides.
Single operations: float32 outputs of the bf16 GEMM carry only accumulation-order error (inputs are
bf16-representable on both sides), bf16 outputs add one rounding of relative size 2^-8.
"""
import ctypes
import dataclasses
import sys

import numpy as np
import pytest

import mt_synth as ms
import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2107_05377_amd as mt  # noqa: E402


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mt.lib()    # fails loudly if the HIP library is missing


def dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return t if dtype is None else t.to(dtype)


def bf16_grid(x):
    return ms.round_to_bf16_grid(np.ascontiguousarray(x, dtype=np.float32).copy())


MINI = ms.MTSpec("mini", vocab=50, hidden=32, heads=4, ffn=64, max_pos=24, n_trunk_layers=3,
                 tasks=(ms.TaskSpec(1, 2, 2), ms.TaskSpec(3, 1, 3), ms.TaskSpec(2, 0, 1), ms.TaskSpec(0, 1, 2)),
                 precision="fp32", batch=3, seq=12, len_lo=3, len_hi=12, input_seed=77, weights_seed=4242)

# bf16-mode model small enough for the oracle to run whole batches: hetero forks, a task with no own
# layer, a fork at the embeddings, ragged sequence length (not a multiple of 32), 3 row tiles.
SMALL = ms.MTSpec("small", vocab=500, hidden=128, heads=2, ffn=256, max_pos=64, n_trunk_layers=3,
                  tasks=(ms.TaskSpec(3, 2, 2), ms.TaskSpec(1, 1, 3), ms.TaskSpec(2, 0, 1), ms.TaskSpec(0, 1, 2),
                         ms.TaskSpec(3, 2, 2)),
                  precision="bf16", batch=7, seq=44, len_lo=5, len_hi=44, input_seed=5, weights_seed=99)


# ------------------------------------------------------------------ single operations

@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18, 19, 20, 21, 22, 23, 24, 25, 26])
def test_gemm_bf16_vs_oracle(tile):
    say(f"gemm_bf16 tile={tile}")
    rng = np.random.default_rng(10 + tile)
    M, N, K = 300, 392, 192            # several tiles in M and N with ragged tails in both
    A = bf16_grid(rng.standard_normal((M, K)))
    W = bf16_grid(rng.standard_normal((N, K)) * 0.1)
    bias = rng.standard_normal(N).astype(np.float32)
    res = rng.standard_normal((M, N)).astype(np.float32)
    prev = mt.set_gemm_tile(tile)
    try:
        dA, dW, db, dr = dev(A, torch.bfloat16), dev(W, torch.bfloat16), dev(bias), dev(res)
        ref = oracle.linear(A, W, bias)
        out = mt.op_linear(mt.MT_BF16, dA, dW, db, out_f32=True).cpu().numpy()
        assert np.abs(out - ref).max() <= 2e-4 * max(1.0, np.abs(ref).max())
        out = mt.op_linear(mt.MT_BF16, dA, dW, db, residual=dr, out_f32=True).cpu().numpy()
        assert np.abs(out - (ref.astype(np.float64) + res)).max() <= 2e-4 * max(1.0, np.abs(ref).max())
        out = mt.op_linear(mt.MT_BF16, dA, dW, db, act=1).float().cpu().numpy()
        g = oracle.gelu(ref)
        assert np.abs(out - g).max() <= 2 ** -8 * np.abs(g).max() + 1e-3
        out = mt.op_linear(mt.MT_BF16, dA, dW, None).float().cpu().numpy()
        ref0 = oracle.linear(A, W, None)
        assert np.abs(out - ref0).max() <= 2 ** -8 * np.abs(ref0).max() + 1e-3
    finally:
        mt.set_gemm_tile(prev)
    torch.cuda.synchronize()


def test_gemm_bf16_persistent_vs_oracle(tile=27):
    """The persistent contraction (one workgroup per compute unit walking a tile list):
    8 problems of ragged M and N (more 256x256 tiles than compute units, so that workgroups really walk from tile to tile and
    from problem to problem), every epilogue the model uses."""
    say(f"gemm_bf16 persistent, selector {tile}")
    rng = np.random.default_rng(40 + tile)
    G, M, N, K = 8, 1560, 1300, 320          # 8 x 7 x 6 = 336 tiles for 256 workgroups
    A = bf16_grid(rng.standard_normal((G, M, K)))
    W = bf16_grid(rng.standard_normal((G, N, K)) * 0.1)
    bias = rng.standard_normal((G, N)).astype(np.float32)
    res = rng.standard_normal((G, M, N)).astype(np.float32)
    ref = np.stack([oracle.linear(A[g], W[g], bias[g]) for g in range(G)])
    scale = max(1.0, float(np.abs(ref).max()))
    prev = mt.set_gemm_tile(tile)
    try:
        dA, dW, db, dr = dev(A, torch.bfloat16), dev(W, torch.bfloat16), dev(bias), dev(res)
        out = mt.op_linear_batched(mt.MT_BF16, dA, dW, db, None, 0, True).cpu().numpy()
        assert np.abs(out - ref).max() <= 2e-4 * scale
        out = mt.op_linear_batched(mt.MT_BF16, dA, dW, db, dr, 0, True).cpu().numpy()
        assert np.abs(out - (ref.astype(np.float64) + res)).max() <= 2e-4 * scale
        out = mt.op_linear_batched(mt.MT_BF16, dA, dW, db, None, 1, False).float().cpu().numpy()
        g = np.stack([oracle.gelu(ref[i]) for i in range(G)])
        assert np.abs(out - g).max() <= 2 ** -8 * np.abs(g).max() + 1e-3
        out = mt.op_linear_batched(mt.MT_BF16, dA[0], dW, None, None, 0, False).float().cpu().numpy()      # shared A
        ref0 = np.stack([oracle.linear(A[0], W[i], None) for i in range(G)])
        assert np.abs(out - ref0).max() <= 2 ** -8 * np.abs(ref0).max() + 1e-3
        # untouched beyond the ragged edges: a canary row and column around a [M][N] window of a larger buffer
        big = torch.full((G, M + 1, N + 8), 7.0, dtype=torch.float32, device="cuda")
        rc = mt.lib().mt_op_linear_batched(mt.MT_BF16, G, dA.data_ptr(), M * K, K, dW.data_ptr(), N * K, db.data_ptr(), N, None, 0,
                                           big.data_ptr(), (M + 1) * (N + 8), N + 8, M, N, K, 0, 1, None)
        assert rc == mt.MT_OK
        o = big.cpu().numpy()
        assert np.abs(o[:, :M, :N] - ref).max() <= 2e-4 * scale
        assert (o[:, M, :] == 7.0).all() and (o[:, :, N:] == 7.0).all()
    finally:
        mt.set_gemm_tile(prev)
    torch.cuda.synchronize()


def test_gemm_bf16_bert_shapes_sampled():
    """BERT-base shapes in the default (shape-chosen) tile configuration, checked on sampled rows."""
    rng = np.random.default_rng(3)
    for (M, N, K) in ((4096, 2304, 768), (4096, 768, 3072), (4096, 3072, 768)):
        say(f"gemm_bf16 {M}x{N}x{K}")
        A = bf16_grid(rng.standard_normal((M, K)))
        W = bf16_grid(rng.standard_normal((N, K)) * 0.02)
        out = mt.op_linear(mt.MT_BF16, dev(A, torch.bfloat16), dev(W, torch.bfloat16), None, out_f32=True).cpu().numpy()
        rows = np.concatenate([[0, 1, M - 1], rng.integers(0, M, 29)])
        ref = oracle.linear(A[rows], W, None)
        assert np.abs(out[rows] - ref).max() <= 2e-4 * np.abs(ref).max()


def test_gemm_bf16_grouped_and_split_vs_oracle():
    """The grouped launch (one problem per task): own and shared activations, per-problem weights and bias."""
    rng = np.random.default_rng(21)
    G, M, N, K = 3, 200, 264, 128
    A = bf16_grid(rng.standard_normal((G, M, K)))
    W = bf16_grid(rng.standard_normal((G, N, K)) * 0.1)
    bias = rng.standard_normal((G, N)).astype(np.float32)
    res = rng.standard_normal((G, M, N)).astype(np.float32)
    for tile in (0, 1, 9, 11, 13):
        prev = mt.set_gemm_tile(tile)
        try:
            out = mt.op_linear_batched(mt.MT_BF16, dev(A, torch.bfloat16), dev(W, torch.bfloat16), dev(bias), dev(res),
                                       out_f32=True).cpu().numpy()
            shared = mt.op_linear_batched(mt.MT_BF16, dev(A[1], torch.bfloat16), dev(W, torch.bfloat16), dev(bias),
                                          act=1).float().cpu().numpy()
        finally:
            mt.set_gemm_tile(prev)
        for g in range(G):
            ref = oracle.linear(A[g], W[g], bias[g]).astype(np.float64) + res[g]
            assert np.abs(out[g] - ref).max() <= 2e-4 * np.abs(ref).max()
            refs = oracle.gelu(oracle.linear(A[1], W[g], bias[g]))
            assert np.abs(shared[g] - refs).max() <= 2 ** -8 * np.abs(refs).max() + 1e-3


def test_gemm_sub_problems_and_ragged_batches_vs_oracle():
    """The few-row kernel's sub-problem forms, as the first-token attention uses them: per-head problems carved out
    of wider matrices by offsets and strides, and a ragged batch whose row ranges are read on the device."""
    rng = np.random.default_rng(77)
    B, A, d = 37, 3, 64                      # rows not a multiple of 32; 3 heads of width 64
    H = A * d
    # (1) per head: C[:, a, :] = Q[:, a*d:(a+1)*d] . WkT[:, a*d:(a+1)*d]^T   (K = d, strided operands, bf16 out)
    Q = bf16_grid(rng.standard_normal((B, H)))
    WkT = bf16_grid(rng.standard_normal((H, H)) * 0.1)
    C1 = torch.full((B, A + 1, H), 7.0, dtype=torch.bfloat16, device="cuda")
    mt.op_linear_sub(dev(Q, torch.bfloat16), H, dev(WkT, torch.bfloat16), H, None, C1, (A + 1) * H, B, H, d, A, d, d, H)
    got = C1.float().cpu().numpy()
    for a in range(A):
        ref = oracle.linear(Q[:, a * d:(a + 1) * d].copy(), WkT[:, a * d:(a + 1) * d].copy(), None)
        assert np.abs(got[:, a, :] - ref).max() <= 2 ** -8 * np.abs(ref).max() + 1e-3
    assert (got[:, A, :] == 7.0).all()                                   # the pad slot is untouched
    # (2) per head with bias, N = d: C[:, a*d:(a+1)*d] = X[:, a, :] . Wv[a*d:(a+1)*d, :]^T + bv[a*d:(a+1)*d]
    X = bf16_grid(rng.standard_normal((B, A, H)))
    Wv = bf16_grid(rng.standard_normal((H, H)) * 0.1)
    bv = rng.standard_normal(H).astype(np.float32)
    C2 = torch.zeros((B, H), dtype=torch.float32, device="cuda")
    mt.op_linear_sub(dev(X, torch.bfloat16), A * H, dev(Wv, torch.bfloat16), 0, dev(bv), C2, H, B, d, H, A, H, d * H, d, d, out_f32=True)
    got = C2.cpu().numpy()
    for a in range(A):
        ref = oracle.linear(X[:, a, :].copy(), Wv[a * d:(a + 1) * d].copy(), bv[a * d:(a + 1) * d].copy())
        assert np.abs(got[:, a * d:(a + 1) * d] - ref).max() <= 2e-4 * max(1.0, np.abs(ref).max())
    # (3) ragged batch: sequence u owns rows row0[u] .. row0[u]+rows[u]-1 of a packed row order (lengths 0..70,
    #     crossing 32-row blocks) and has its own small W (12 rows, like one row per head)
    lens = np.array([5, 33, 1, 64, 0, 70, 32, 17], dtype=np.int32)
    row0 = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int32)
    R, Np, K = int(lens.sum()), 12, 192
    Xr = bf16_grid(rng.standard_normal((R, K)))
    Wq = bf16_grid(rng.standard_normal((len(lens), Np, K)) * 0.1)
    C3 = torch.full((R + 3, Np), -5.0, dtype=torch.float32, device="cuda")
    mt.op_linear_sub(dev(Xr, torch.bfloat16), K, dev(Wq, torch.bfloat16), 0, None, C3, Np, 80, Np, K, len(lens), 0, Np * K, 0,
                     row0=dev(row0), rows=dev(lens), out_f32=True)
    got = C3.cpu().numpy()
    for u in range(len(lens)):
        if lens[u] == 0:
            continue
        ref = oracle.linear(Xr[row0[u]:row0[u] + lens[u]].copy(), Wq[u].copy(), None)
        assert np.abs(got[row0[u]:row0[u] + lens[u]] - ref).max() <= 2e-4 * max(1.0, np.abs(ref).max())
    assert (got[R:] == -5.0).all()
    torch.cuda.synchronize()


@pytest.mark.parametrize("H,A,A_pad", [(768, 12, 12), (128, 2, 4), (1024, 16, 16), (320, 5, 8)])
def test_first_token_pool_vs_oracle(H, A, A_pad):
    """Softmax over each sequence's rows of given raw scores and the weighted sum of its input rows, per head."""
    rng = np.random.default_rng(5 + H)
    lens = np.array([1, 9, 64, 8, 0, 128, 65, 7, 100], dtype=np.int32)
    row0 = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int32)
    R, B, S = int(lens.sum()), len(lens), 128
    scores = (rng.standard_normal((R, A_pad)) * 20.0).astype(np.float32)
    X = bf16_grid(rng.standard_normal((R, H)))
    got = mt.op_first_token_pool(dev(scores), dev(X, torch.bfloat16), dev(row0), dev(lens), B, S, H, A, A_pad).float().cpu().numpy()
    scale = np.float32(1.0 / np.sqrt(np.float32(H // A)))
    for b in range(B):
        if lens[b] == 0:
            continue
        rows = slice(row0[b], row0[b] + lens[b])
        for a in range(A):
            p = oracle.softmax_row((scores[rows, a] * scale).astype(np.float32))
            ref = p.astype(np.float64) @ X[rows].astype(np.float64)
            assert np.abs(got[b, a] - ref).max() <= 2 ** -8 * max(np.abs(ref).max(), 1e-3) + 1e-4, (b, a)
    assert (got[:, A:, :] == 0).all()
    torch.cuda.synchronize()


def test_gemm_f32_vs_oracle():
    rng = np.random.default_rng(4)
    for (M, N, K) in ((70, 67, 33), (5, 3, 64), (130, 129, 100)):
        A = rng.standard_normal((M, K)).astype(np.float32)
        W = rng.standard_normal((N, K)).astype(np.float32)
        b = rng.standard_normal(N).astype(np.float32)
        r = rng.standard_normal((M, N)).astype(np.float32)
        out = mt.op_linear(mt.MT_FP32_CHECK, dev(A), dev(W), dev(b), residual=dev(r), act=3).cpu().numpy()
        ref = np.tanh(oracle.linear(A, W, b).astype(np.float64)) + r
        assert np.abs(out - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("B,S,heads", [(3, 128, 2), (2, 40, 1), (2, 200, 2), (1, 512, 1), (4, 64, 3)])
def test_attention_bf16_vs_oracle(B, S, heads):
    say(f"attention_bf16 B={B} S={S} heads={heads}")
    rng = np.random.default_rng(S)
    H = heads * 64
    q = bf16_grid(rng.standard_normal((B, S, H)))
    k = bf16_grid(rng.standard_normal((B, S, H)))
    v = bf16_grid(rng.standard_normal((B, S, H)))
    lengths = rng.integers(1, S + 1, B)
    lengths[0] = S
    mask = (np.arange(S)[None, :] < lengths[:, None]).astype(np.int32)
    if B > 1 and lengths[1] > 3:
        mask[1, 2] = 0          # a hole inside a sequence
    qkv = np.concatenate([q, k, v], axis=2).reshape(B * S, 3 * H)
    dqkv = dev(qkv, torch.bfloat16)
    ctx = mt.op_attention(mt.MT_BF16, dqkv, dev(mask), B, S, H, heads).float().cpu().numpy().reshape(B, S, H)
    ref = oracle.attention(q, k, v, mask, heads)
    real = mask.astype(bool)
    err = np.abs(ctx[real] - ref[real]).max()
    say(f"  max err {err:.4g}")
    assert err <= 2e-2


def test_attention_f32_vs_oracle():
    rng = np.random.default_rng(8)
    for (B, S, H, A) in ((2, 16, 64, 2), (3, 21, 60, 3), (1, 130, 32, 1)):
        q, k, v = (rng.standard_normal((B, S, H)).astype(np.float32) for _ in range(3))
        lengths = rng.integers(1, S + 1, B)
        mask = (np.arange(S)[None, :] < lengths[:, None]).astype(np.int32)
        qkv = np.concatenate([q, k, v], axis=2).reshape(B * S, 3 * H)
        ctx = mt.op_attention(mt.MT_FP32_CHECK, dev(qkv), dev(mask), B, S, H, A).cpu().numpy().reshape(B, S, H)
        ref = oracle.attention(q, k, v, mask, A)
        assert np.abs(ctx - ref).max() <= 2e-5


@pytest.mark.parametrize("H", [768, 1024, 64, 100])
def test_layernorm_vs_oracle(H):
    rng = np.random.default_rng(H)
    M = 37
    x = (rng.standard_normal((M, H)) * 2 + 0.5).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    b = (0.1 * rng.standard_normal(H)).astype(np.float32)
    of, ob = mt.op_layernorm(dev(x), dev(g), dev(b), 1e-12, want_bf16=True)
    ref = oracle.layernorm(x, g, b, 1e-12)
    assert np.abs(of.cpu().numpy() - ref).max() <= 1e-5
    assert np.abs(ob.float().cpu().numpy() - ref).max() <= 2 ** -8 * np.abs(ref).max()


# ------------------------------------------------------------------ whole model, float32 validation mode

def _params(spec, stress, std=0.02):
    tr, tri = ms.make_trunk_params(spec, stress=stress, std=std)
    tps = [ms.make_task_params(spec, t, stress=stress, std=std) for t in range(spec.n_tasks)]
    return tr, tri, tps


def _load(spec, tr, tri, tps, **kw):
    model = mt.Model(mt.make_config(spec, **kw))
    model.load_params(-1, tr, len(tri))
    for t, (tp, tpi) in enumerate(tps):
        model.load_params(t, tp, len(tpi))
    return model


def rel_err_per_task(spec, got, ref):
    out, col = [], 0
    for t in spec.tasks:
        g, o = got[:, col:col + t.n_classes], ref[:, col:col + t.n_classes]
        out.append(np.abs(g - o).max() / max(np.abs(o).max(), 1e-3))
        col += t.n_classes
    return out


@pytest.mark.parametrize("spec,stress,std", [(ms.get_config("tiny"), False, 0.02), (ms.get_config("tiny"), True, 0.02),
                                             (MINI, True, 0.1)])
def test_fp32_mode_matches_oracle(spec, stress, std):
    say(f"fp32 mode {spec.name} stress={stress}")
    tr, tri, tps = _params(spec, stress, std)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec)
    ref, hidden = orc.mt_forward(ids, mask, want_hidden=True)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    errs = rel_err_per_task(spec, got, ref)
    say("  rel err per task", errs)
    assert max(errs) <= 1e-4
    assert np.all(np.abs(got - ref) <= 1e-4 * np.abs(ref) + 1e-6)
    # the kept trunk states (taps) agree with the oracle's on real tokens
    real = mask.astype(bool)
    for layer in sorted({t.fork_layer for t in spec.tasks}):
        h = model.read_hidden(-1, layer, *ids.shape).cpu().numpy()
        assert np.abs(h[real] - hidden[layer][real]).max() <= 2e-5
    model.close()


def test_fp32_mode_base_shapes_one_sequence():
    """float32 validation mode at BERT-base width (H=768, 12 heads, F=3072), shallow, 2 sequences."""
    spec = dataclasses.replace(ms.get_config("base"), precision="fp32", n_trunk_layers=1,
                               tasks=(ms.TaskSpec(1, 1, 2), ms.TaskSpec(1, 0, 3)), batch=2, seq=24, len_lo=5, len_hi=24,
                               vocab=2000)
    tr, tri, tps = _params(spec, True)
    ids, mask, _ = ms.make_inputs(spec)
    ref = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask)
    model = _load(spec, tr, tri, tps)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    assert max(rel_err_per_task(spec, got, ref)) <= 1e-4
    model.close()


# ------------------------------------------------------------------ whole model, bf16 mode

def argmax_stats(spec, got, ref):
    """(#pairs, #agree, #pairs with margin > 4e-2, #agree among those) over classification tasks."""
    n = agree = n_safe = agree_safe = 0
    col = 0
    for t in spec.tasks:
        if t.n_classes >= 2:
            g, o = got[:, col:col + t.n_classes], ref[:, col:col + t.n_classes]
            ga, oa = g.argmax(1), o.argmax(1)          # numpy argmax returns the lowest index among ties
            srt = np.sort(o, axis=1)
            margin = srt[:, -1] - srt[:, -2]
            n += len(ga)
            agree += int((ga == oa).sum())
            safe = margin > 4e-2
            n_safe += int(safe.sum())
            agree_safe += int((ga == oa)[safe].sum())
        col += t.n_classes
    return n, agree, n_safe, agree_safe


@pytest.mark.parametrize("stress", [False, True])
def test_bf16_mode_small_model_matches_oracle(stress):
    spec = SMALL
    say(f"bf16 small model stress={stress}")
    tr, tri, tps = _params(spec, stress, 0.05)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    model = _load(spec, tr, tri, tps)
    for bi in range(2):
        ids, mask, _ = ms.make_inputs(spec, batch_index=bi)
        ref = orc.mt_forward(ids, mask)
        got = model.forward(dev(ids), dev(mask)).cpu().numpy()
        err = np.abs(got - ref).max()
        say(f"  batch {bi}: max |dlogit| {err:.4g}")
        assert err <= 2e-2
        n, agree, n_safe, agree_safe = argmax_stats(spec, got, ref)
        assert agree_safe == n_safe
    # smaller batch and sequence than the maximum, on the same model
    ids, mask, _ = ms.make_inputs(spec, batch=2, seq=33, batch_index=5)
    assert np.abs(model.forward(dev(ids), dev(mask)).cpu().numpy() - orc.mt_forward(ids, mask)).max() <= 2e-2
    model.close()


def test_bf16_mode_many_heads_takes_the_projected_key_value_form():
    """More than 16 heads: the last layer of a branch projects keys and values for every row and attends with
    one wavefront per (task, sequence, head) instead of the key/value-free form; same logits contract."""
    spec = ms.MTSpec("wide", vocab=300, hidden=1280, heads=20, ffn=256, max_pos=48, n_trunk_layers=1,
                     tasks=(ms.TaskSpec(1, 2, 3), ms.TaskSpec(0, 1, 2)), precision="bf16",
                     batch=5, seq=40, len_lo=3, len_hi=40, input_seed=123)
    tr, tri, tps = _params(spec, True, 0.03)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec)
    err = np.abs(model.forward(dev(ids), dev(mask)).cpu().numpy() - orc.mt_forward(ids, mask)).max()
    say(f"  20 heads: max |dlogit| {err:.4g}")
    assert err <= 2e-2
    model.close()


def test_bf16_mode_masks_with_holes_and_extreme_lengths():
    """Padding-free row order: masks that are not prefixes, a sequence of one token, full sequences."""
    spec = SMALL
    tr, tri, tps = _params(spec, True, 0.05)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec, batch_index=3)
    mask = mask.copy()
    mask[0, :] = 1                       # a full sequence
    mask[1, 1:] = 0                      # a single token
    mask[2, :] = 1
    mask[2, [3, 4, 17, 40]] = 0          # holes inside a sequence
    mask[3, :] = 0
    mask[3, [0, 5, 43]] = 1              # scattered real tokens, the last position among them
    ref = orc.mt_forward(ids, mask)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    err = np.abs(got - ref).max()
    say(f"  holes: max |dlogit| {err:.4g}")
    assert err <= 2e-2
    # the kept trunk state, put back in [batch, seq] order, matches on every real token and is zero elsewhere
    _, hidden = orc.mt_forward(ids, mask, want_hidden=True)
    h = model.read_hidden(-1, 3, *ids.shape).cpu().numpy()
    real = mask.astype(bool)
    assert np.abs(h[real] - hidden[3][real]).max() <= 5e-2
    assert (h[~real] == 0).all()
    model.close()


@pytest.mark.parametrize("name,batch,rows", [("hetero", 64, [0, 33]), ("latency", 8, list(range(8))), ("latency", 1, [0]),
                                             ("large", 128, [0, 77]), ("industrial", 16, [0, 5, 11]),
                                             ("wo_kd", 8, [0, 5]), ("mixed", 8, [1, 6])])
def test_bf16_other_workloads_sampled(name, batch, rows):
    """Forks at different trunk layers (a trunk tap per fork, branch stages of shrinking groups) and the
    small-batch serving shape, in the launch configuration the benchmark uses."""
    spec = ms.get_config(name)
    say(f"workload {name}: building weights")
    tr, tri, tps = _params(spec, False)
    model = _load(spec, tr, tri, tps, max_batch=batch)
    assert model.layer_count() == spec.n_trunk_layers + sum(t.n_layers for t in spec.tasks)
    ids, mask, lengths = ms.make_inputs(spec, batch=batch)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    assert np.isfinite(got).all()
    say("  oracle on rows", rows)
    ref = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids[rows], mask[rows])
    err = np.abs(got[rows] - ref).max()
    n, agree, n_safe, agree_safe = argmax_stats(spec, got[rows], ref)
    say(f"  max |dlogit| {err:.4g}; argmax agree {agree}/{n}; margin>4e-2: {agree_safe}/{n_safe}")
    assert err <= 2e-2 and agree_safe == n_safe
    model.close()


@pytest.fixture(scope="module")
def base_model():
    spec = ms.get_config("base")
    say("building base model (synthetic BERT-base shapes, 8 tasks)")
    tr, tri, tps = _params(spec, False)
    model = _load(spec, tr, tri, tps)
    yield spec, model, tr, [p for p, _ in tps]
    model.close()


def test_bf16_base_full_batch_sampled_sequences(base_model):
    """The benchmark's launch configuration (B=32, S=128, all 8 tasks); the oracle evaluates sampled
    sequences one batch-row at a time (sequences are independent, so rows of a sub-batch are exact)."""
    spec, model, tr, tps = base_model
    orc = oracle.Oracle(spec, tr, tps)
    ids, mask, lengths = ms.make_inputs(spec)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    assert np.isfinite(got).all()
    rows = [0, int(np.argmin(lengths)), int(np.argmax(lengths)), 17]
    say("  oracle on rows", rows, "lengths", lengths[rows])
    ref = orc.mt_forward(ids[rows], mask[rows])
    err = np.abs(got[rows] - ref).max()
    n, agree, n_safe, agree_safe = argmax_stats(spec, got[rows], ref)
    say(f"  max |dlogit| {err:.4g}; argmax agree {agree}/{n}; with margin>4e-2: {agree_safe}/{n_safe}")
    assert err <= 2e-2
    assert agree_safe == n_safe


def test_bf16_base_invariants_at_full_size(base_model):
    spec, model, _, _ = base_model
    ids, mask, lengths = ms.make_inputs(spec, batch_index=1)
    d_ids, d_mask = dev(ids), dev(mask)
    base = model.forward(d_ids, d_mask).cpu().numpy()
    # determinism
    assert np.array_equal(model.forward(d_ids, d_mask).cpu().numpy(), base)
    # token ids under the mask are irrelevant
    ids2 = ids.copy()
    ids2[mask == 0] = (ids2[mask == 0] * 7 + 3) % spec.vocab
    assert np.array_equal(model.forward(dev(ids2), d_mask).cpu().numpy(), base)
    # each sequence alone gives its row of the batched run.  Not bit for bit: a problem of few rows runs in the
    # few-row contraction kernel, which adds the K range up in four quarters, so some bf16 roundings of the
    # activations fall the other way; the bound is a quarter of the logit tolerance.
    for b in (0, 5):
        one = model.forward(dev(ids[b:b + 1]), dev(mask[b:b + 1])).cpu().numpy()
        assert np.abs(one[0] - base[b]).max() <= 5e-3
    # truncating the padding away changes nothing
    L = int(lengths[:4].max())
    L = (L + 7) // 8 * 8
    cut = model.forward(dev(ids[:4, :L]), dev(mask[:4, :L])).cpu().numpy()
    assert np.abs(cut - base[:4]).max() <= 5e-3        # four sequences can also fall under the few-row limit
    # task mask: disabled tasks' columns stay untouched, enabled ones are unchanged
    out = torch.full((ids.shape[0], model.n_logits), 7.0, device="cuda")
    tm = [1, 0, 1, 1, 0, 0, 1, 0]
    model.forward(d_ids, d_mask, out=out, task_mask=tm)
    o = out.cpu().numpy()
    col = 0
    for t, task in enumerate(spec.tasks):
        sl = slice(col, col + task.n_classes)
        if tm[t]:
            assert np.array_equal(o[:, sl], base[:, sl])
        else:
            assert (o[:, sl] == 7.0).all()
        col += task.n_classes


def test_bf16_base_task_isolation(base_model):
    """Reloading one task's checkpoint leaves every other task's logits bit-identical (Section 5.1)."""
    spec, model, _, tps = base_model
    ids, mask, _ = ms.make_inputs(spec, batch=4, batch_index=2)
    d_ids, d_mask = dev(ids), dev(mask)
    before = model.forward(d_ids, d_mask).cpu().numpy()
    new, newi = ms.make_task_params(spec, 3, seed=777)
    model.load_params(3, new, len(newi))
    after = model.forward(d_ids, d_mask).cpu().numpy()
    lo, hi = model.logit_offset(3), model.logit_offset(3) + 3
    assert np.array_equal(after[:, :lo], before[:, :lo]) and np.array_equal(after[:, hi:], before[:, hi:])
    assert np.abs(after[:, lo:hi] - before[:, lo:hi]).max() > 1e-3
    old, oldi = ms.make_task_params(spec, 3)
    model.load_params(3, old, len(oldi))
    assert np.array_equal(model.forward(d_ids, d_mask).cpu().numpy(), before)


def test_bf16_vs_fp32_mode_argmax_over_many_sequences(base_model):
    """Argmax agreement over 1024 sequences x 7 classification tasks between the bf16 path and the
    float32 validation path of the same library (itself held to 1e-4 of the oracle above)."""
    spec, model, tr, tps = base_model
    f32 = mt.Model(mt.make_config(spec, precision=mt.MT_FP32_CHECK))
    f32.load_params(-1, tr, len(ms.trunk_tensors(spec)))
    for t, p in enumerate(tps):
        f32.load_params(t, p, len(ms.task_tensors(spec, t)))
    n = agree = n_safe = agree_safe = 0
    worst = 0.0
    for bi in range(32):
        ids, mask, _ = ms.make_inputs(spec, batch_index=100 + bi)
        d_ids, d_mask = dev(ids), dev(mask)
        a = model.forward(d_ids, d_mask).cpu().numpy()
        b = f32.forward(d_ids, d_mask).cpu().numpy()
        worst = max(worst, float(np.abs(a - b).max()))
        s = argmax_stats(spec, a, b)
        n, agree, n_safe, agree_safe = n + s[0], agree + s[1], n_safe + s[2], agree_safe + s[3]
    say(f"  bf16 vs fp32 mode: max |dlogit| {worst:.4g}; argmax agree {agree}/{n} = {agree / n:.5f}; "
        f"margin>4e-2: {agree_safe}/{n_safe}")
    f32.close()
    assert worst <= 2e-2
    assert agree_safe == n_safe
    assert agree / n >= 0.999


def test_replicas_in_flight_match_serial(base_model):
    """Forwards of two replicas (shared weights, own workspaces) overlapping on two streams give, batch by batch,
    exactly what one model gives running them one after another."""
    spec, model, _, _ = base_model
    batches = []
    for i in range(4):
        ids, mask, _ = ms.make_inputs(spec, batch_index=10 + i)
        batches.append((dev(ids), dev(mask)))
    serial = [model.forward(*b).clone() for b in batches]
    torch.cuda.synchronize()
    reps = [model, model.replica()]
    streams = [torch.cuda.Stream() for _ in reps]
    outs = [torch.zeros_like(serial[0]) for _ in batches]
    for rounds in range(3):
        for i, b in enumerate(batches):
            j = i % 2
            with torch.cuda.stream(streams[j]):
                reps[j].forward(*b, out=outs[i])
        torch.cuda.synchronize()
        for i in range(len(batches)):
            assert torch.equal(outs[i], serial[i]), f"round {rounds}, batch {i}"
    reps[1].close()


def test_segment_ids_match_oracle():
    """Sentence-pair inputs: the typed forward adds the segment's row of the type table (fp32 mode to 1e-4,
    bf16 mode to the logit tolerance); all-zero ids and NULL give the plain forward bit for bit."""
    mini = ms.MTSpec("mini", vocab=50, hidden=32, heads=4, ffn=64, max_pos=24, n_trunk_layers=3,
                     tasks=(ms.TaskSpec(1, 2, 2), ms.TaskSpec(3, 1, 3), ms.TaskSpec(2, 0, 1), ms.TaskSpec(0, 1, 2)),
                     precision="fp32", batch=3, seq=12, len_lo=3, len_hi=12, input_seed=77, weights_seed=4242)
    small = ms.MTSpec("pair_bf16", vocab=500, hidden=128, heads=2, ffn=256, max_pos=64, n_trunk_layers=2,
                      tasks=(ms.TaskSpec(2, 2, 3), ms.TaskSpec(1, 1, 2), ms.TaskSpec(0, 1, 2)), precision="bf16",
                      batch=6, seq=48, len_lo=5, len_hi=48, input_seed=91)
    for spec, stress in ((mini, True), (small, True)):
        tr, tri, tps = _params(spec, stress, std=0.1 if spec.precision == "fp32" else 0.02)
        model = _load(spec, tr, tri, tps)
        ids, mask, lengths = ms.make_inputs(spec)
        tt = np.zeros_like(ids)
        for b in range(ids.shape[0]):
            tt[b, max(1, int(lengths[b]) // 2):] = 1
        plain = model.forward(dev(ids), dev(mask)).cpu().numpy()
        assert np.array_equal(model.forward(dev(ids), dev(mask), type_ids=dev(np.zeros_like(ids))).cpu().numpy(), plain)
        got = model.forward(dev(ids), dev(mask), type_ids=dev(tt)).cpu().numpy()
        ref = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask, type_ids=tt)
        assert np.abs(got - plain).max() > 1e-5
        if spec.precision == "fp32":
            assert max(rel_err_per_task(spec, got, ref)) <= 1e-4
        else:
            assert np.abs(got - ref).max() <= 2e-2
        model.close()


@pytest.mark.parametrize("kind", ["fp32", "bf16"])
def test_per_sequence_routing_matches_oracle(kind):
    """Each sequence asks for its own subset of tasks: wanted logits equal the oracle's (sequences are independent,
    so the oracle's full forward is the reference), everything else is left untouched."""
    if kind == "fp32":
        spec, std = MINI, 0.1
    else:
        spec, std = SMALL, 0.05
    tr, tri, tps = _params(spec, True, std)
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec, batch_index=3)
    B, T = ids.shape[0], spec.n_tasks
    rng = np.random.default_rng(11)
    route = (rng.random((B, T)) < 0.5).astype(np.uint8)
    route[0, :] = 1                      # one sequence wants everything
    route[1, :] = 0                      # one wants nothing
    if T >= 3:
        route[:, 2] = route[:, 1]        # two tasks with the same sequence set share a group
    ref = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask)
    out = torch.full((B, model.n_logits), 9.0, device="cuda")
    model.forward_routed(dev(ids), dev(mask), route, out)
    got = out.cpu().numpy()
    col = 0
    for t, task in enumerate(spec.tasks):
        sl = slice(col, col + task.n_classes)
        for b in range(B):
            if route[b, t]:
                if kind == "fp32":
                    assert np.abs(got[b, sl] - ref[b, sl]).max() <= 1e-4 * max(np.abs(ref[:, sl]).max(), 1e-3), (b, t)
                else:
                    assert np.abs(got[b, sl] - ref[b, sl]).max() <= 2e-2, (b, t)
            else:
                assert (got[b, sl] == 9.0).all(), (b, t)
        col += task.n_classes
    # all-ones routing equals the plain forward up to the rounding differences of a different launch grouping
    out2 = torch.zeros((B, model.n_logits), device="cuda")
    model.forward_routed(dev(ids), dev(mask), np.ones((B, T)), out2)
    plain = model.forward(dev(ids), dev(mask)).cpu().numpy()
    assert np.abs(out2.cpu().numpy() - plain).max() <= (1e-5 if kind == "fp32" else 5e-3)
    model.close()


def test_per_sequence_routing_at_full_size(base_model):
    """base workload, every sequence wanting a random half of the 8 tasks: wanted logits agree with the plain
    forward (same model, other launch grouping: rounding-level differences), the rest is untouched."""
    spec, model, _, _ = base_model
    ids, mask, _ = ms.make_inputs(spec, batch_index=4)
    B, T = ids.shape[0], spec.n_tasks
    route = (np.random.default_rng(3).random((B, T)) < 0.5).astype(np.uint8)
    plain = model.forward(dev(ids), dev(mask)).cpu().numpy()
    out = torch.full((B, model.n_logits), -3.0, device="cuda")
    model.forward_routed(dev(ids), dev(mask), route, out)
    got = out.cpu().numpy()
    col = 0
    for t, task in enumerate(spec.tasks):
        sl = slice(col, col + task.n_classes)
        want = route[:, t] != 0
        assert np.abs(got[want][:, sl] - plain[want][:, sl]).max() <= 5e-3
        assert (got[~want][:, sl] == -3.0).all()
        col += task.n_classes


def _random_spec(rng, bf16):
    """A small random merged model: random widths, forks anywhere in the trunk (including the embeddings), branches
    of 0..3 own layers, 1..6 classes, ragged batch and sequence sizes."""
    if bf16:
        heads = int(rng.integers(1, 4))
        hidden = 64 * heads
        ffn = 64 * int(rng.integers(1, 5))
    else:
        heads = int(rng.choice([1, 2, 3, 4]))
        hidden = heads * int(rng.choice([4, 8, 12, 20]))
        ffn = int(rng.choice([8, 24, 40, 100]))
    depth = int(rng.integers(0, 4))
    n_tasks = int(rng.integers(1, 6))
    tasks = []
    for _ in range(n_tasks):
        tasks.append(ms.TaskSpec(int(rng.integers(0, depth + 1)), int(rng.integers(0, 4)), int(rng.integers(1, 7))))
    tasks[int(rng.integers(0, n_tasks))] = ms.TaskSpec(depth, int(rng.integers(0, 4)), int(rng.integers(1, 7)))   # someone forks at D
    seq = int(rng.integers(2, 71))
    return ms.MTSpec("rand", vocab=int(rng.integers(20, 400)), hidden=hidden, heads=heads, ffn=ffn, max_pos=seq + 3,
                     n_trunk_layers=depth, tasks=tuple(tasks), precision="bf16" if bf16 else "fp32",
                     batch=int(rng.integers(1, 8)), seq=seq, len_lo=1, len_hi=seq, input_seed=int(rng.integers(1, 10 ** 6)),
                     weights_seed=int(rng.integers(1, 10 ** 6)))


@pytest.mark.parametrize("seed,bf16", [(s, False) for s in range(10)] + [(100 + s, True) for s in range(8)])
def test_random_small_models_match_oracle(seed, bf16):
    rng = np.random.default_rng(seed)
    spec = _random_spec(rng, bf16)
    say(f"random model seed={seed}: H={spec.hidden} A={spec.heads} F={spec.ffn} D={spec.n_trunk_layers} "
        f"tasks={[(t.fork_layer, t.n_layers, t.n_classes) for t in spec.tasks]} B={spec.batch} S={spec.seq}")
    tr, tri, tps = _params(spec, True, 0.05 if bf16 else 0.1)
    model = _load(spec, tr, tri, tps)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    ids, mask, lengths = ms.make_inputs(spec)
    if spec.seq >= 6 and spec.batch >= 2:                   # a hole in one mask (never at position 0)
        j = 1 + int(rng.integers(0, max(1, int(lengths[1]) - 1)))
        mask[1, j] = 0
    ref = orc.mt_forward(ids, mask)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    if bf16:
        assert np.abs(got - ref).max() <= 2e-2
    else:
        assert max(rel_err_per_task(spec, got, ref)) <= 1e-4
    # a task mask and a routing table on the same model
    tm = [int(rng.integers(0, 2)) for _ in spec.tasks]
    tm[int(rng.integers(0, spec.n_tasks))] = 1
    out = torch.full((spec.batch, model.n_logits), 5.0, device="cuda")
    model.forward(dev(ids), dev(mask), out=out, task_mask=tm)
    route = (rng.random((spec.batch, spec.n_tasks)) < 0.6).astype(np.uint8)
    out_r = torch.full((spec.batch, model.n_logits), 5.0, device="cuda")
    model.forward_routed(dev(ids), dev(mask), route, out_r)
    o, o_r = out.cpu().numpy(), out_r.cpu().numpy()
    tol = 2e-2 if bf16 else 1e-4 * max(np.abs(ref).max(), 1e-3)
    col = 0
    for t, task in enumerate(spec.tasks):
        sl = slice(col, col + task.n_classes)
        if tm[t]:
            assert np.abs(o[:, sl] - ref[:, sl]).max() <= tol
        else:
            assert (o[:, sl] == 5.0).all()
        for b in range(spec.batch):
            if route[b, t]:
                assert np.abs(o_r[b, sl] - ref[b, sl]).max() <= tol
            else:
                assert (o_r[b, sl] == 5.0).all()
        col += task.n_classes
    model.close()


# ------------------------------------------------------------------ token-level heads (tagging tasks, Appendix E)

TOKF = ms.MTSpec("tokf", vocab=50, hidden=32, heads=4, ffn=64, max_pos=24, n_trunk_layers=2,
                 tasks=(ms.TaskSpec(1, 1, 2), ms.TaskSpec(2, 1, 5, token_level=True), ms.TaskSpec(2, 0, 3),
                        ms.TaskSpec(0, 2, 4, token_level=True), ms.TaskSpec(1, 0, 32, token_level=True)),
                 precision="fp32", batch=3, seq=10, len_lo=2, len_hi=10, input_seed=78, weights_seed=4243)
TOKB = ms.MTSpec("tokb", vocab=500, hidden=128, heads=2, ffn=256, max_pos=80, n_trunk_layers=3,
                 tasks=(ms.TaskSpec(3, 2, 2), ms.TaskSpec(1, 1, 7, token_level=True), ms.TaskSpec(2, 0, 1),
                        ms.TaskSpec(3, 0, 3, token_level=True), ms.TaskSpec(0, 3, 12, token_level=True), ms.TaskSpec(3, 1, 4)),
                 precision="bf16", batch=9, seq=71, len_lo=1, len_hi=71, input_seed=79, weights_seed=4244)


def _token_case(spec, stress, std, mask_edit=None, batch_index=0):
    tr, tri, tps = _params(spec, stress, std)
    model = _load(spec, tr, tri, tps)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    ids, mask, lengths = ms.make_inputs(spec, batch_index=batch_index)
    if mask_edit is not None:
        mask = mask.copy()
        mask_edit(mask)
    ref, ref_tok = orc.mt_forward(ids, mask, want_tokens=True)
    return model, orc, ids, mask, ref, ref_tok


@pytest.mark.parametrize("stress", [False, True])
def test_token_heads_fp32_mode_match_oracle(stress):
    spec = TOKF
    say(f"token-level heads, fp32 mode, stress={stress}")
    model, orc, ids, mask, ref, ref_tok = _token_case(spec, stress, 0.1)
    assert model.n_logits == 5 and model.n_token_logits == 41
    assert [model.token_logit_offset(t) for t in (1, 3, 4)] == [0, 5, 9]
    got, tok = model.forward_tokens(dev(ids), dev(mask))
    got, tok = got.cpu().numpy(), tok.cpu().numpy()
    real = mask.astype(bool)
    assert np.abs(got - ref).max() <= 1e-4 * max(np.abs(ref).max(), 1e-3)
    for t in (1, 3, 4):
        c0, c1 = spec.logit_offset(t), spec.logit_offset(t) + spec.tasks[t].n_classes
        scale = max(np.abs(ref_tok[:, :, c0:c1][real]).max(), 1e-3)
        assert np.abs(tok[:, :, c0:c1][real] - ref_tok[:, :, c0:c1][real]).max() <= 1e-4 * scale, t
    assert (tok[~real] == 0).all() and (~real).any()
    # the whole final state of a token-level branch is kept and readable
    h = model.read_hidden(3, 0, *ids.shape).cpu().numpy()
    assert (h[~real] == 0).all() and np.abs(h[real]).max() > 0.1
    # the plain entry point refuses a token-level task instead of dropping its output, and serves the others
    with pytest.raises(mt.MTError):
        model.forward(dev(ids), dev(mask))
    seq_only = [0 if t.token_level else 1 for t in spec.tasks]
    assert np.array_equal(model.forward(dev(ids), dev(mask), task_mask=seq_only).cpu().numpy(), got)
    with pytest.raises(mt.MTError):
        model.forward_routed(dev(ids), dev(mask), np.ones((spec.batch, spec.n_tasks)), torch.zeros((spec.batch, 5), device="cuda"))
    # disabled token-level tasks leave their columns alone
    o = torch.full((spec.batch, 5), 3.0, device="cuda")
    ot = torch.full((spec.batch, spec.seq, 41), 3.0, device="cuda")
    model.forward_tokens(dev(ids), dev(mask), out=o, out_tokens=ot, task_mask=[0, 1, 0, 0, 1])
    assert (o == 3.0).all() and (ot[:, :, 5:9] == 3.0).all()
    assert torch.equal(ot[:, :, :5].cpu(), torch.from_numpy(tok[:, :, :5])) and torch.equal(ot[:, :, 9:].cpu(), torch.from_numpy(tok[:, :, 9:]))
    model.close()


def test_token_heads_bf16_mode_match_oracle():
    spec = TOKB
    say("token-level heads, bf16 mode, ragged lengths, a mask with holes")

    def edit(mask):
        mask[0, :] = 1
        mask[1, 1:] = 0
        mask[2, :] = 1
        mask[2, [3, 4, 17, 40, 70]] = 0
    for bi, ed in ((0, None), (1, edit)):
        model, orc, ids, mask, ref, ref_tok = _token_case(spec, True, 0.05, ed, batch_index=bi)
        got, tok = model.forward_tokens(dev(ids), dev(mask))
        got, tok = got.cpu().numpy(), tok.cpu().numpy()
        real = mask.astype(bool)
        e_seq, e_tok = np.abs(got - ref).max(), np.abs(tok[real] - ref_tok[real]).max()
        say(f"  batch {bi}: max |dlogit| per sequence {e_seq:.4g}, per token {e_tok:.4g} over {int(real.sum())} tokens")
        assert e_seq <= 2e-2 and e_tok <= 2e-2
        assert (tok[~real] == 0).all()
        # tag decisions: wherever the oracle's margin exceeds twice the tolerance the chosen label agrees
        for t in (1, 3, 4):
            c0, c1 = spec.logit_offset(t), spec.logit_offset(t) + spec.tasks[t].n_classes
            g, o = tok[:, :, c0:c1][real], ref_tok[:, :, c0:c1][real]
            srt = np.sort(o, axis=1)
            safe = (srt[:, -1] - srt[:, -2]) > 4e-2
            assert (g.argmax(1) == o.argmax(1))[safe].all()
        # smaller batch and sequence than the maximum on the same model
        ids2, mask2, _ = ms.make_inputs(spec, batch=2, seq=33, batch_index=7)
        r2, rt2 = orc.mt_forward(ids2, mask2, want_tokens=True)
        g2, t2 = model.forward_tokens(dev(ids2), dev(mask2))
        assert np.abs(g2.cpu().numpy() - r2).max() <= 2e-2
        assert np.abs(t2.cpu().numpy()[mask2.astype(bool)] - rt2[mask2.astype(bool)]).max() <= 2e-2
        model.close()


def test_token_heads_assistant_workload_sampled():
    """21 tasks on 8 shared layers, three of them tagging every token, at the serving shape of the benchmark."""
    spec = ms.get_config("assistant")
    say("workload assistant: building weights")
    tr, tri, tps = _params(spec, False)
    model = _load(spec, tr, tri, tps)
    ids, mask, lengths = ms.make_inputs(spec)
    got, tok = model.forward_tokens(dev(ids), dev(mask))
    got, tok = got.cpu().numpy(), tok.cpu().numpy()
    rows = [0, 7, 13]
    say("  oracle on rows", rows)
    ref, ref_tok = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids[rows], mask[rows], want_tokens=True)
    real = mask[rows].astype(bool)
    e_seq, e_tok = np.abs(got[rows] - ref).max(), np.abs(tok[rows][real] - ref_tok[real]).max()
    say(f"  max |dlogit| per sequence {e_seq:.4g}, per token {e_tok:.4g}")
    assert e_seq <= 2e-2 and e_tok <= 2e-2
    assert (tok[~mask.astype(bool)] == 0).all() and np.isfinite(tok).all()
    model.close()


@pytest.mark.parametrize("precision,hidden,heads", [("fp32", 256, 4), ("bf16", 256, 4), ("fp32", 512, 2), ("bf16", 1280, 20)])
def test_token_heads_wide_rows(precision, hidden, heads):
    """Hidden sizes that are multiples of 256 take the token classifier that keeps a row in registers; class counts
    that are not multiples of four, a task without own layers, one sequence of a single token."""
    spec = ms.MTSpec("tokw", vocab=300, hidden=hidden, heads=heads, ffn=256, max_pos=40, n_trunk_layers=1,
                     tasks=(ms.TaskSpec(1, 1, 6, token_level=True), ms.TaskSpec(1, 0, 1, token_level=True),
                            ms.TaskSpec(0, 1, 3), ms.TaskSpec(0, 1, 67, token_level=True)),
                     precision=precision, batch=5, seq=37, len_lo=1, len_hi=37, input_seed=80, weights_seed=4245)

    def edit(mask):
        mask[0, 1:] = 0
        mask[1, :] = 1
    # weight scale: 0.1 in float32 mode; in bf16 mode 0.05, and 0.03 at H = 1280 as in the many-heads case above (the
    # absolute logit tolerance is meant for logits of order one, which a wider model reaches with smaller weights)
    std = 0.1 if precision == "fp32" else (0.03 if hidden > 1024 else 0.05)
    model, orc, ids, mask, ref, ref_tok = _token_case(spec, True, std, edit)
    got, tok = model.forward_tokens(dev(ids), dev(mask))
    got, tok = got.cpu().numpy(), tok.cpu().numpy()
    real = mask.astype(bool)
    e_seq, e_tok = np.abs(got - ref).max(), np.abs(tok[real] - ref_tok[real]).max()
    say(f"  logit scale: per sequence {np.abs(ref).max():.3g}, per token {np.abs(ref_tok[real]).max():.3g}")
    say(f"  {precision} H={hidden}: max |dlogit| per sequence {e_seq:.4g}, per token {e_tok:.4g}")
    if precision == "bf16":
        assert e_seq <= 2e-2 and e_tok <= 2e-2
    else:
        assert e_seq <= 1e-4 * max(np.abs(ref).max(), 1e-3) and e_tok <= 1e-4 * max(np.abs(ref_tok[real]).max(), 1e-3)
    assert (tok[~real] == 0).all()
    model.close()


# ------------------------------------------------------------------ the largest sizes the library accepts

def test_bf16_longest_sequence():
    """max_seq = 608 (the bf16 path's limit): one full-length sequence, one of a single token, one in between, with a
    token-level task so that every row of the last layer is checked too."""
    spec = ms.MTSpec("long", vocab=400, hidden=128, heads=2, ffn=256, max_pos=1024, n_trunk_layers=2,
                     tasks=(ms.TaskSpec(2, 2, 3), ms.TaskSpec(1, 1, 2), ms.TaskSpec(2, 1, 5, token_level=True), ms.TaskSpec(0, 0, 2)),
                     precision="bf16", batch=3, seq=608, len_lo=300, len_hi=600, input_seed=81, weights_seed=4246)

    def edit(mask):
        mask[0, :] = 1
        mask[1, 1:] = 0
    model, orc, ids, mask, ref, ref_tok = _token_case(spec, True, 0.05, edit)
    got, tok = model.forward_tokens(dev(ids), dev(mask))
    got, tok = got.cpu().numpy(), tok.cpu().numpy()
    real = mask.astype(bool)
    e_seq, e_tok = np.abs(got - ref).max(), np.abs(tok[real] - ref_tok[real]).max()
    say(f"  S=608: max |dlogit| per sequence {e_seq:.4g}, per token {e_tok:.4g} over {int(real.sum())} tokens")
    assert e_seq <= 2e-2 and e_tok <= 2e-2 and (tok[~real] == 0).all()
    # one more sequence or one more position than the model was created for is refused on the host
    with pytest.raises(mt.MTError):
        model.forward(dev(np.zeros((4, 608), np.int32)), dev(np.ones((4, 608), np.int32)), task_mask=[1, 1, 0, 1])
    with pytest.raises(mt.MTError):
        model.forward(dev(np.zeros((3, 609), np.int32)), dev(np.ones((3, 609), np.int32)), task_mask=[1, 1, 0, 1])
    model.close()
    cfg = mt.make_config(dataclasses.replace(spec, seq=609))
    h = ctypes.c_void_p()
    assert mt.lib().mt_create(ctypes.byref(cfg), ctypes.byref(h)) == mt.MT_ERR_CONFIG


def test_routing_at_the_largest_batch():
    """1024 sequences (the routed call's limit), every sequence with its own random task set."""
    spec = ms.MTSpec("wide_batch", vocab=300, hidden=128, heads=2, ffn=256, max_pos=8, n_trunk_layers=1,
                     tasks=(ms.TaskSpec(1, 1, 2), ms.TaskSpec(0, 2, 3), ms.TaskSpec(1, 0, 4)),
                     precision="bf16", batch=1024, seq=6, len_lo=1, len_hi=6, input_seed=82, weights_seed=4247)
    tr, tri, tps = _params(spec, True, 0.05)
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec)
    ref = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    assert np.abs(got - ref).max() <= 2e-2
    rng = np.random.default_rng(3)
    route = (rng.random((1024, 3)) < 0.5).astype(np.uint8)
    out = torch.full((1024, model.n_logits), -7.0, device="cuda")
    model.forward_routed(dev(ids), dev(mask), route, out)
    o = out.cpu().numpy()
    for t in range(3):
        sl = slice(model.logit_offset(t), model.logit_offset(t) + spec.tasks[t].n_classes)
        want = route[:, t].astype(bool)
        assert np.abs(o[want, sl] - ref[want, sl]).max() <= 2e-2
        assert (o[~want, sl] == -7.0).all()
    model.close()


def test_tasks_are_added_while_serving():
    """Section 5.1's modular update: a graph declared with room for five tasks serves with two of them loaded (the
    others masked off), a third is loaded later without touching the first two, and an unloaded task is refused."""
    spec = SMALL
    tr, tri, tps = _params(spec, True, 0.05)
    model = mt.Model(mt.make_config(spec))
    model.load_params(-1, tr, len(tri))
    for t in (0, 3):
        model.load_params(t, tps[t][0], len(tps[t][1]))
    ids, mask, _ = ms.make_inputs(spec)
    ref = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask)
    d_ids, d_mask = dev(ids), dev(mask)
    with pytest.raises(mt.MTError):
        model.forward(d_ids, d_mask)                                   # tasks 1, 2, 4 have no weights yet
    first = torch.full((spec.batch, model.n_logits), 4.0, device="cuda")
    model.forward(d_ids, d_mask, out=first, task_mask=[1, 0, 0, 1, 0])
    first = first.cpu().numpy()
    cols = lambda t: slice(model.logit_offset(t), model.logit_offset(t) + spec.tasks[t].n_classes)
    for t in (0, 3):
        assert np.abs(first[:, cols(t)] - ref[:, cols(t)]).max() <= 2e-2
    for t in (1, 2, 4):
        assert (first[:, cols(t)] == 4.0).all()
    model.load_params(4, tps[4][0], len(tps[4][1]))                    # a new task arrives
    second = torch.full((spec.batch, model.n_logits), 4.0, device="cuda")
    model.forward(d_ids, d_mask, out=second, task_mask=[1, 0, 0, 1, 1])
    second = second.cpu().numpy()
    for t in (0, 3):
        assert np.array_equal(second[:, cols(t)], first[:, cols(t)])   # bit for bit
    assert np.abs(second[:, cols(4)] - ref[:, cols(4)]).max() <= 2e-2
    model.close()


@pytest.mark.parametrize("which", ["fp32", "bf16"])
def test_a_sequence_without_real_tokens_disturbs_nothing(which):
    """A sequence whose mask is all zero breaks the precondition (its own outputs are unspecified), but it has no rows
    in the padding-free order and must leave every other sequence's logits as they are; a batch of such sequences
    only has to come back."""
    spec = TOKF if which == "fp32" else TOKB
    tr, tri, tps = _params(spec, True, 0.1 if which == "fp32" else 0.05)
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec)
    ref, ref_tok = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask, want_tokens=True)
    dead = mask.copy()
    dead[1, :] = 0
    got, tok = model.forward_tokens(dev(ids), dev(dead))
    got, tok = got.cpu().numpy(), tok.cpu().numpy()
    keep = [b for b in range(spec.batch) if b != 1]
    tol = 1e-4 * max(np.abs(ref).max(), np.abs(ref_tok).max()) if which == "fp32" else 2e-2
    real = mask[keep].astype(bool)
    assert np.abs(got[keep] - ref[keep]).max() <= tol
    assert np.abs(tok[keep][real] - ref_tok[keep][real]).max() <= tol
    assert (tok[1] == 0).all()                                # no kept row: the token head writes zeros there
    model.forward_tokens(dev(ids), dev(np.zeros_like(mask)))   # no row at all
    torch.cuda.synchronize()
    again, _ = model.forward_tokens(dev(ids), dev(mask))       # and the model still serves
    assert np.abs(again.cpu().numpy() - ref).max() <= tol
    model.close()


@pytest.mark.parametrize("which", ["fp32", "bf16"])
def test_several_requests_in_one_forward_match_oracle(which):
    """mt_forward_multi: request batches arriving in separate device arrays run as one combined batch; every request
    gets the oracle's logits for its own sequences, columns of masked-off tasks stay untouched, and pointer tables
    are read before the call returns (they are rebuilt for every call here)."""
    spec = MINI if which == "fp32" else SMALL
    tr, tri, tps = _params(spec, True, 0.1 if which == "fp32" else 0.05)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    n_req = 5
    model = _load(spec, tr, tri, tps, max_batch=n_req * spec.batch)
    one = _load(spec, tr, tri, tps)
    reqs, refs = [], []
    for r in range(n_req):
        ids, mask, _ = ms.make_inputs(spec, batch_index=20 + r)
        reqs.append((dev(ids), dev(mask)))
        refs.append(orc.mt_forward(ids, mask))
    outs = model.forward_multi(reqs)
    for r in range(n_req):
        got = outs[r].cpu().numpy()
        if which == "fp32":
            assert max(rel_err_per_task(spec, got, refs[r])) <= 1e-4
        else:
            assert np.abs(got - refs[r]).max() <= 2e-2
        alone = one.forward(*reqs[r]).cpu().numpy()
        assert np.abs(got - alone).max() <= (1e-5 if which == "fp32" else 5e-3)
    # fewer requests than the model was created for, and a task mask
    tm = [1] + [0] * (spec.n_tasks - 2) + [1]
    outs2 = [torch.full((spec.batch, model.n_logits), 7.0, device="cuda") for _ in range(2)]
    model.forward_multi(reqs[3:5], outs=outs2, task_mask=tm)
    for k, r in enumerate((3, 4)):
        o = outs2[k].cpu().numpy()
        want = outs[r].cpu().numpy()
        for t in range(spec.n_tasks):
            lo = spec.logit_offset(t)
            sl = slice(lo, lo + spec.tasks[t].n_classes)
            if tm[t]:
                assert np.abs(o[:, sl] - want[:, sl]).max() <= (1e-5 if which == "fp32" else 5e-3)
            else:
                assert (o[:, sl] == 7.0).all()
    with pytest.raises(mt.MTError) as ei:                       # more sequences than the model was created for
        one.forward_multi(reqs[:2])
    assert ei.value.code == mt.MT_ERR_SHAPE
    model.close()
    one.close()


@pytest.mark.parametrize("which", ["fp32", "bf16"])
def test_token_heads_under_per_sequence_routing(which):
    """Routing with tagging tasks: a wanted (sequence, task) pair gets the oracle's token logits on its real tokens and
    zeros on its padding; unwanted pairs and other tasks' columns are left untouched; sequence-level tasks of the
    same call behave as in mt_forward_routed."""
    spec = TOKF if which == "fp32" else TOKB
    tr, tri, tps = _params(spec, True, 0.1 if which == "fp32" else 0.05)
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec, batch_index=1)
    ref, ref_tok = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask, want_tokens=True)
    B, S, T = ids.shape[0], ids.shape[1], spec.n_tasks
    rng = np.random.default_rng(5)
    route = (rng.random((B, T)) < 0.6).astype(np.uint8)
    route[0, :] = 1
    route[1, :] = 0
    tok_tasks = [t for t in range(T) if spec.tasks[t].token_level]
    route[:, tok_tasks[1]] = route[:, tok_tasks[0]]                 # two tagging tasks share a group
    out = torch.full((B, model.n_logits), 9.0, device="cuda")
    tok = torch.full((B, S, model.n_token_logits), 9.0, device="cuda")
    model.forward_routed_tokens(dev(ids), dev(mask), route, out, tok)
    got, got_tok = out.cpu().numpy(), tok.cpu().numpy()
    tol_seq = 1e-4 * max(np.abs(ref).max(), 1e-3) if which == "fp32" else 2e-2
    tol_tok = 1e-4 * max(np.abs(ref_tok).max(), 1e-3) if which == "fp32" else 2e-2
    for t, task in enumerate(spec.tasks):
        lo = spec.logit_offset(t)
        sl = slice(lo, lo + task.n_classes)
        for b in range(B):
            real = mask[b].astype(bool)
            if task.token_level:
                if route[b, t]:
                    assert np.abs(got_tok[b, real, sl] - ref_tok[b, real, sl]).max() <= tol_tok, (b, t)
                    assert (got_tok[b, ~real, sl] == 0.0).all(), (b, t)
                else:
                    assert (got_tok[b, :, sl] == 9.0).all(), (b, t)
            elif route[b, t]:
                assert np.abs(got[b, sl] - ref[b, sl]).max() <= tol_seq, (b, t)
            else:
                assert (got[b, sl] == 9.0).all(), (b, t)
    # the plain routed entry point has nowhere to put token logits
    with pytest.raises(mt.MTError) as ei:
        model.forward_routed(dev(ids), dev(mask), route, out)
    assert ei.value.code == mt.MT_ERR_NULL
    model.close()


def test_mask_precondition_is_checkable():
    """Position 0 of every sequence must be real: mt_check_mask counts the sequences that break it; a sequence that
    does is served from its first real token (pinned here against the oracle run on the shifted sequence)."""
    spec = MINI
    tr, tri, tps = _params(spec, True, 0.1)
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec)
    assert model.check_mask(dev(mask)) == 0
    bad = mask.copy()
    bad[1, 0] = 0
    bad[2, :] = 0
    with pytest.raises(mt.MTError) as ei:
        model.check_mask(dev(bad))
    assert ei.value.code == mt.MT_ERR_SHAPE and "2 of 3" in str(ei.value)
    # sequence 0 is untouched by its neighbours' bad masks
    ref = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask)
    got = model.forward(dev(ids), dev(bad)).cpu().numpy()
    assert max(rel_err_per_task(spec, got[:1], ref[:1])) <= 1e-4
    model.close()


def test_read_hidden_refuses_states_the_last_forward_did_not_write():
    """A trunk tap is readable only if the last forward pass ran the trunk that deep: with the deeper tasks masked
    off the trunk stops at the deepest enabled fork, and with no task enabled nothing runs at all."""
    spec = MINI                                         # forks at layers 1, 3, 2, 0
    tr, tri, tps = _params(spec, True, 0.1)
    model = _load(spec, tr, tri, tps)
    ids, mask, _ = ms.make_inputs(spec)
    _, hidden = oracle.Oracle(spec, tr, [p for p, _ in tps]).mt_forward(ids, mask, want_hidden=True)
    real = mask.astype(bool)
    model.forward(dev(ids), dev(mask))
    for layer in (0, 1, 2, 3):
        h = model.read_hidden(-1, layer, *ids.shape).cpu().numpy()
        assert np.abs(h[real] - hidden[layer][real]).max() <= 2e-5
    model.forward(dev(ids), dev(mask), task_mask=[1, 0, 0, 1])       # deepest enabled fork: layer 1
    h = model.read_hidden(-1, 1, *ids.shape).cpu().numpy()
    assert np.abs(h[real] - hidden[1][real]).max() <= 2e-5
    for layer in (2, 3):
        with pytest.raises(mt.MTError) as ei:
            model.read_hidden(-1, layer, *ids.shape)
        assert ei.value.code == mt.MT_ERR_STATE
    with pytest.raises(mt.MTError) as ei:
        model.read_hidden(1, 0, *ids.shape)                           # task 1 was masked off
    assert ei.value.code == mt.MT_ERR_STATE
    model.forward(dev(ids), dev(mask), task_mask=[0, 0, 0, 0])       # nothing enabled: nothing was computed
    with pytest.raises(mt.MTError) as ei:
        model.read_hidden(-1, 0, *ids.shape)
    assert ei.value.code == mt.MT_ERR_STATE
    model.close()


def test_forward_is_capture_safe_and_replays_bit_identically():
    """mt_forward only enqueues kernels (no allocation, copy, memset or wait inside), so a caller may capture it in a HIP
    graph.  Each of several replays, with launched work and synchronisations between them, must equal the launched
    result bit for bit, also after the captured input buffers have been refilled."""
    spec = ms.get_config("latency")
    model, _ = mt.load_synthetic(spec)
    for b in (1, 8):
        ids_h, mask_h, _ = ms.make_inputs(spec, batch=b)
        ids, mask = dev(ids_h), dev(mask_h)
        launched = model.forward(ids, mask).clone()
        torch.cuda.synchronize()
        out_g = torch.zeros_like(launched)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            model.forward(ids, mask, out=out_g)
        other_h = ms.make_inputs(spec, batch=b, batch_index=5)
        for rep in range(3):
            out_g.zero_()
            model.forward(dev(other_h[0]), dev(other_h[1]))          # launched work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out_g, launched), f"replay {rep} at batch {b} differs from the launched forward"
        ids.copy_(dev(other_h[0]))
        mask.copy_(dev(other_h[1]))
        graph.replay()
        torch.cuda.synchronize()
        want = model.forward(dev(other_h[0]), dev(other_h[1]))
        torch.cuda.synchronize()
        assert torch.equal(out_g, want)
        del graph
    model.close()


def test_sixty_four_requests_in_one_forward_and_one_too_many():
    """The largest request count of mt_forward_multi (64): single-sequence requests of a small bf16 model, each against
    the oracle; 65 requests are refused."""
    spec = dataclasses.replace(SMALL, batch=1)
    tr, tri, tps = _params(spec, True, 0.05)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    model = _load(spec, tr, tri, tps, max_batch=65)
    reqs, refs = [], []
    for r in range(65):
        ids, mask, _ = ms.make_inputs(spec, batch=1, batch_index=100 + r)
        reqs.append((dev(ids), dev(mask)))
        if r < 64:
            refs.append(orc.mt_forward(ids, mask))
    outs = model.forward_multi(reqs[:64])
    worst = max(float(np.abs(outs[r].cpu().numpy() - refs[r]).max()) for r in range(64))
    say(f"  64 single-sequence requests in one forward: max |dlogit| {worst:.4g}")
    assert worst <= 2e-2
    with pytest.raises(mt.MTError) as ei:
        model.forward_multi(reqs)
    assert ei.value.code == mt.MT_ERR_SHAPE and "at most 64" in str(ei.value)
    model.close()


@pytest.mark.parametrize("which", ["fp32", "bf16"])
def test_requests_of_different_sizes_in_one_forward(which):
    """mt_forward_requests: requests bring their own sequence counts (1, 3, 2, 7, 1, 4 here); every request gets the
    oracle's logits for its own sequences, a masked-off task's columns stay untouched, totals beyond max_batch and
    empty requests are refused."""
    spec = MINI if which == "fp32" else SMALL
    tr, tri, tps = _params(spec, True, 0.1 if which == "fp32" else 0.05)
    orc = oracle.Oracle(spec, tr, [p for p, _ in tps])
    sizes = [1, 3, 2, 7, 1, 4]
    model = _load(spec, tr, tri, tps, max_batch=sum(sizes))
    reqs, refs = [], []
    for r, b in enumerate(sizes):
        ids, mask, _ = ms.make_inputs(spec, batch=b, batch_index=40 + r)
        reqs.append((dev(ids), dev(mask)))
        refs.append(orc.mt_forward(ids, mask))
    tm = [1] * spec.n_tasks
    tm[1] = 0
    outs = [torch.full((b, model.n_logits), 7.0, device="cuda") for b in sizes]
    model.forward_requests(reqs, outs=outs, task_mask=tm)
    off = spec.logit_offset(1)
    dead = slice(off, off + spec.tasks[1].n_classes)
    for r in range(len(sizes)):
        got = outs[r].cpu().numpy()
        assert (got[:, dead] == 7.0).all()
        live = np.ones(got.shape[1], dtype=bool)
        live[dead] = False
        if which == "fp32":
            assert np.abs(got[:, live] - refs[r][:, live]).max() <= 1e-4 * max(np.abs(refs[r]).max(), 1e-3)
        else:
            assert np.abs(got[:, live] - refs[r][:, live]).max() <= 2e-2
    extra = ms.make_inputs(spec, batch=1, batch_index=77)
    with pytest.raises(mt.MTError) as ei:
        model.forward_requests(reqs + [(dev(extra[0]), dev(extra[1]))])
    assert ei.value.code == mt.MT_ERR_SHAPE
    model.close()
