"""The FP8 variants (MT_FP8_FFN: the two feed-forward contractions of every all-rows layer in OCP E4M3; MT_FP8_LAYER: the
query/key/value and attention output projections too) against the oracle.

What each side consumes: the generator snaps the feed-forward matrices to the E4M3 grid under their power-of-two
storage scale (and everything else to the bfloat16 grid), so the float32 oracle and the library hold identical
weights; what the tolerance has to cover is the rounding of the two feed-forward OPERANDS (LayerNorm output, GELU
output) to E4M3, relative step 2^-4 against bfloat16's 2^-9 on the other operands.

Tolerance.  The bf16 path's measured error is about 2e-3 for a bar of 2e-2.  Two of a layer's four contraction
operands are now 32 times coarser, and they belong to the block whose output is a fraction (about a third at these
weights) of the residual stream it is added to: expected error about 32 * 0.5 * 2e-3 = 3e-2.  Bar: max |delta logit|
<= 8e-2 (four times the bf16 bar), and identical argmax on every (sequence, task) pair whose oracle margin exceeds
twice that.  MT_FP8_LAYER rounds all four contraction operands of a layer to E4M3 (the layer input, the attention
context, the LayerNorm output, the GELU output).  Independent roundings add in quadrature, so twice as many coarse
operands raise the expectation by sqrt(2), to about 4.2e-2: the same bar of 8e-2 is kept for both (relative to the
largest logit when that exceeds 1).
"""
import dataclasses
import sys

import numpy as np
import pytest

import mt_synth as ms
import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2107_05377_amd as mt  # noqa: E402

TOL = {"fp8": 8e-2, "fp8_all": 8e-2}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def e4m3_values(codes):
    return torch.from_numpy(np.ascontiguousarray(codes)).view(torch.float8_e4m3fn).float().numpy()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mt.lib()


@pytest.mark.parametrize("M,N,K", [(300, 392, 192), (2318, 768, 3072), (1560, 1300, 320)])
def test_fp8_contraction_vs_oracle(M, N, K):
    """Operands exactly representable in E4M3, so the oracle's float64 dot products are the exact result and only the
    float32 accumulation order differs; all three output kinds, ragged edges, a canary beyond them."""
    if K % 64:
        K = K // 64 * 64
    say(f"fp8 contraction {M}x{N}x{K}")
    rng = np.random.default_rng(M + N)
    a_codes = mt.e4m3_quantize(rng.standard_normal((M, K)).astype(np.float32) * 100)[1]          # scale 1 or 2: any codes do
    w_scale, w_codes = mt.e4m3_quantize((rng.standard_normal((N, K)) * 0.02).astype(np.float32))
    A, W = e4m3_values(a_codes), e4m3_values(w_codes) / np.float32(w_scale)
    bias = rng.standard_normal(N).astype(np.float32)
    res = rng.standard_normal((M, N)).astype(np.float32)
    ref = oracle.linear(A, W, bias)
    scale = max(1.0, float(np.abs(ref).max()))
    dA, dW, db, dr = dev(a_codes), dev(w_codes), dev(bias), dev(res)
    out = mt.op_linear_fp8(dA, dW, 1.0 / w_scale, db, None, 0, 1).cpu().numpy()
    assert np.abs(out - ref).max() <= 2e-4 * scale
    out = mt.op_linear_fp8(dA, dW, 1.0 / w_scale, db, dr, 0, 1).cpu().numpy()
    assert np.abs(out - (ref.astype(np.float64) + res)).max() <= 2e-4 * scale
    out = mt.op_linear_fp8(dA, dW, 1.0 / w_scale, db, None, 1, 0).float().cpu().numpy()
    g = oracle.gelu(ref)
    assert np.abs(out - g).max() <= 2 ** -8 * np.abs(g).max() + 1e-3
    # E4M3 output: the nearest code of the exact value, or a neighbour where the float32 value sits at a rounding boundary
    out8 = e4m3_values(mt.op_linear_fp8(dA, dW, 1.0 / w_scale, db, None, 1, 2, 0.5).cpu().numpy())
    want = np.clip(g * 0.5, -448, 448)
    assert np.all(np.abs(out8 - want) <= 2.0 ** -4 * np.abs(want) + 2.0 ** -9 + 1e-3)
    assert np.abs(out8 - want).mean() <= 2.0 ** -5 * np.abs(want).mean() + 2.0 ** -10
    big = torch.full((M + 1, N + 8), 7.0, dtype=torch.float32, device="cuda")
    rc = mt.lib().mt_op_linear_fp8(dA.data_ptr(), K, dW.data_ptr(), 1.0 / w_scale, db.data_ptr(), None, big.data_ptr(), N + 8, M, N, K, 0, 1, 1.0, None)
    assert rc == mt.MT_OK
    o = big.cpu().numpy()
    assert np.abs(o[:M, :N] - ref).max() <= 2e-4 * scale and (o[M] == 7.0).all() and (o[:, N:] == 7.0).all()


SMALL8 = ms.MTSpec("small_fp8", vocab=500, hidden=256, heads=4, ffn=512, max_pos=64, n_trunk_layers=3,
                   tasks=(ms.TaskSpec(3, 2, 2), ms.TaskSpec(1, 1, 3), ms.TaskSpec(2, 0, 1), ms.TaskSpec(0, 2, 4, token_level=True),
                          ms.TaskSpec(3, 2, 2)),
                   precision="fp8", batch=7, seq=44, len_lo=5, len_hi=44, input_seed=5, weights_seed=99)


def _model(spec, stress=False, std=0.02, **kw):
    tr, tri = ms.make_trunk_params(spec, stress=stress, std=std)
    tps = [ms.make_task_params(spec, t, stress=stress, std=std) for t in range(spec.n_tasks)]
    model = mt.Model(mt.make_config(spec, **kw))
    model.load_params(-1, tr, len(tri))
    for t, (tp, tpi) in enumerate(tps):
        model.load_params(t, tp, len(tpi))
    return model, oracle.Oracle(spec, tr, [p for p, _ in tps])


def _safe_agreement(spec, got, ref, margin):
    col, n, agree = 0, 0, 0
    for t in spec.tasks:
        if t.token_level:
            continue
        if t.n_classes >= 2:
            g, o = got[:, col:col + t.n_classes], ref[:, col:col + t.n_classes]
            srt = np.sort(o, axis=1)
            safe = (srt[:, -1] - srt[:, -2]) > margin
            n += int(safe.sum())
            agree += int((g.argmax(1) == o.argmax(1))[safe].sum())
        col += t.n_classes
    return n, agree


@pytest.mark.parametrize("precision", ["fp8", "fp8_all"])
@pytest.mark.parametrize("stress", [False, True])
def test_fp8_small_model_whole_batches(stress, precision):
    """Heterogeneous forks, a task without own layers, a tagging task (all its layers on all rows, so its last layer is
    FP8 too), sequence tasks (last layer first-token-only, bf16), whole batches against the oracle."""
    spec = dataclasses.replace(SMALL8, precision=precision)
    model, orc = _model(spec, stress, 0.05)
    for bi in range(3):
        ids, mask, _ = ms.make_inputs(spec, batch_index=bi)
        ref, ref_tok = orc.mt_forward(ids, mask, want_tokens=True)
        got, tok = model.forward_tokens(dev(ids), dev(mask))
        got, tok = got.cpu().numpy(), tok.cpu().numpy()
        real = mask.astype(bool)
        err = max(float(np.abs(got - ref).max()), float(np.abs(tok[real] - ref_tok[real]).max()))
        bar = TOL[precision] * max(1.0, float(np.abs(ref).max()), float(np.abs(ref_tok[real]).max()))
        say(f"  {precision} small model stress={stress} batch {bi}: max |dlogit| {err:.4g} (bar {bar:.3g})")
        assert err <= bar
        n, agree = _safe_agreement(spec, got, ref, 2 * bar)
        assert agree == n
        assert (tok[~real] == 0).all()
    # the same checkpoints in the bf16 mode of the library are closer to the oracle: the FP8 path really ran
    spec_b = dataclasses.replace(spec, precision="bf16")
    mb = mt.Model(mt.make_config(spec_b))
    tr, tri = ms.make_trunk_params(spec, stress=stress, std=0.05)
    mb.load_params(-1, tr, len(tri))
    for t in range(spec.n_tasks):
        tp, tpi = ms.make_task_params(spec, t, stress=stress, std=0.05)
        mb.load_params(t, tp, len(tpi))
    ids, mask, _ = ms.make_inputs(spec)
    ref = orc.mt_forward(ids, mask)
    e_b = float(np.abs(mb.forward_tokens(dev(ids), dev(mask))[0].cpu().numpy() - ref).max())
    e_8 = float(np.abs(model.forward_tokens(dev(ids), dev(mask))[0].cpu().numpy() - ref).max())
    say(f"  same checkpoints: bf16 mode {e_b:.4g}, {precision} mode {e_8:.4g}")
    assert e_b <= 2e-2 and e_8 > e_b
    mb.close()
    model.close()


@pytest.mark.parametrize("precision", ["fp8", "fp8_all"])
def test_fp8_base_workload_sampled_and_served(precision):
    """`base` shapes (B = 32, S = 128, 8 tasks) with E4M3 feed-forward matrices: sampled sequences against the oracle
    through mt_forward and through mt_forward_multi (8 request batches per call, the benchmark's configuration),
    replicas share the storage scales."""
    spec = dataclasses.replace(ms.get_config("base"), name="base_" + precision, precision=precision)
    model, orc = _model(spec, max_batch=8 * 32)
    ids, mask, lengths = ms.make_inputs(spec)
    rows = [0, int(np.argmin(lengths)), int(np.argmax(lengths)), 17]
    say("  oracle on rows", rows)
    ref = orc.mt_forward(ids[rows], mask[rows])
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    assert np.isfinite(got).all()
    err = float(np.abs(got[rows] - ref).max())
    reqs = [(dev(ids), dev(mask))]
    for r in range(1, 8):
        i2, m2, _ = ms.make_inputs(spec, batch_index=r)
        reqs.append((dev(i2), dev(m2)))
    multi = model.forward_multi(reqs)[0].cpu().numpy()
    err_m = float(np.abs(multi[rows] - ref).max())
    rep = model.replica()
    again = rep.forward(dev(ids), dev(mask)).cpu().numpy()
    say(f"  {precision} base: max |dlogit| {err:.4g} (one request), {err_m:.4g} (eight per call); bar {TOL[precision]}")
    assert err <= TOL[precision] and err_m <= TOL[precision]
    assert np.array_equal(again, got)
    n, agree = _safe_agreement(spec, got[rows], ref, 2 * TOL[precision])
    assert agree == n
    rep.close()
    model.close()
