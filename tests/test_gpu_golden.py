"""Full-size parity against STORED oracle logits (tests/golden/oracle_logits_*.npy, written by
tests/golden/make_logits.py from oracle/ and mt_synth/ alone: the oracle needs minutes to hours at these sizes).

Whole batches are compared, in the launch configurations the benchmark times: `base` request batches of 32
sequences served 8 per call (mt_forward_multi) and one per call (mt_forward), `hetero`, `latency` and `large`
through mt_forward at their own batch sizes.

Bars.  bf16 mode: max |delta logit| <= 2e-2; argmax identical on >= 99.9 % of the (sequence, task) pairs of the
classification tasks (ties to the lowest index on both sides) and on every pair whose oracle top-2 margin exceeds
4e-2 (which the first bound implies).  float32 validation mode: per task max|g-o| <= 1e-4 * max(max|o|, 1e-3).
"""
import os
import sys

import numpy as np
import pytest

import mt_synth as ms

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
import paper_2107_05377_amd as mt  # noqa: E402

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def stored(name):
    path = os.path.join(GOLDEN, f"oracle_logits_{name}.npy")
    assert os.path.exists(path), f"{path} is missing: run python tests/golden/make_logits.py {name}"
    ref = np.load(path)
    assert ref.dtype == np.float32 and np.isfinite(ref).all()
    return ref


def argmax_stats(spec, got, ref):
    """(#pairs, #agree, #pairs with margin > 4e-2, #agree among those) over the classification tasks."""
    n = agree = n_safe = agree_safe = 0
    col = 0
    for t in spec.tasks:
        if t.n_classes >= 2:
            g, o = got[:, col:col + t.n_classes], ref[:, col:col + t.n_classes]
            ga, oa = g.argmax(1), o.argmax(1)          # numpy argmax returns the lowest index among ties
            srt = np.sort(o, axis=1)
            safe = (srt[:, -1] - srt[:, -2]) > 4e-2
            n += len(ga)
            agree += int((ga == oa).sum())
            n_safe += int(safe.sum())
            agree_safe += int((ga == oa)[safe].sum())
        col += t.n_classes
    return n, agree, n_safe, agree_safe


def rel_err_per_task(spec, got, ref):
    out, col = [], 0
    for t in spec.tasks:
        g, o = got[:, col:col + t.n_classes], ref[:, col:col + t.n_classes]
        out.append(float(np.abs(g - o).max() / max(np.abs(o).max(), 1e-3)))
        col += t.n_classes
    return out


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mt.lib()


@pytest.fixture(scope="module")
def base_served():
    spec = ms.get_config("base")
    say("loading base (8 requests of 32 sequences per call)")
    model, _ = mt.load_synthetic(spec, max_batch=8 * spec.batch)
    yield spec, model
    model.close()


def test_bf16_base_4096_sequences_eight_requests_per_call(base_served):
    """The benchmark's launch configuration: 16 calls of 8 request batches; every logit of all 4096 sequences."""
    spec, model = base_served
    ref = stored("base")                                 # [128][32][16]
    assert ref.shape == (128, spec.batch, spec.n_logits)
    worst, tot = 0.0, np.zeros(4, dtype=np.int64)
    for c in range(16):
        reqs = []
        for r in range(8):
            ids, mask, _ = ms.make_inputs(spec, batch_index=8 * c + r)
            reqs.append((dev(ids), dev(mask)))
        outs = model.forward_multi(reqs)
        for r in range(8):
            got = outs[r].cpu().numpy()
            assert np.isfinite(got).all()
            worst = max(worst, float(np.abs(got - ref[8 * c + r]).max()))
            tot += np.array(argmax_stats(spec, got, ref[8 * c + r]))
    n, agree, n_safe, agree_safe = (int(v) for v in tot)
    say(f"  base, 4096 sequences, 8 requests per call: max |dlogit| {worst:.4g}; argmax agree {agree}/{n} = {agree / n:.5f}; "
        f"margin > 4e-2: {agree_safe}/{n_safe}")
    assert worst <= 2e-2
    assert agree_safe == n_safe
    assert agree / n >= 0.999


def test_bf16_base_one_request_per_call(base_served):
    """The same model one request batch at a time (mt_forward, B = 32: the single-problem launch shapes)."""
    spec, model = base_served
    ref = stored("base")
    worst, tot = 0.0, np.zeros(4, dtype=np.int64)
    for bi in range(100, 128):
        ids, mask, _ = ms.make_inputs(spec, batch_index=bi)
        got = model.forward(dev(ids), dev(mask)).cpu().numpy()
        worst = max(worst, float(np.abs(got - ref[bi]).max()))
        tot += np.array(argmax_stats(spec, got, ref[bi]))
    n, agree, n_safe, agree_safe = (int(v) for v in tot)
    say(f"  base, 896 sequences, one request per call: max |dlogit| {worst:.4g}; argmax agree {agree}/{n}; margin > 4e-2: {agree_safe}/{n_safe}")
    assert worst <= 2e-2
    assert agree_safe == n_safe
    assert agree / n >= 0.999


def test_fp32_mode_base_full_depth_two_whole_batches():
    """The float32 validation mode at the full depth of `base` (8 trunk layers, two layers per task), whole batches."""
    spec = ms.get_config("base")
    ref = stored("base")
    model, _ = mt.load_synthetic(spec, precision=mt.MT_FP32_CHECK)
    for bi in (0, 1):
        ids, mask, _ = ms.make_inputs(spec, batch_index=bi)
        got = model.forward(dev(ids), dev(mask)).cpu().numpy()
        errs = rel_err_per_task(spec, got, ref[bi])
        say(f"  fp32 mode, base batch {bi}: rel err per task {['%.2e' % e for e in errs]}")
        assert max(errs) <= 1e-4
        assert np.all(np.abs(got - ref[bi]) <= 1e-4 * np.abs(ref[bi]) + 1e-6)
    model.close()


@pytest.mark.parametrize("name", ["hetero", "latency", "large"])
def test_bf16_other_workloads_whole_batches(name):
    spec = ms.get_config(name)
    ref = stored(name)[0]
    assert ref.shape == (spec.batch, spec.n_logits)
    model, _ = mt.load_synthetic(spec)
    ids, mask, _ = ms.make_inputs(spec)
    got = model.forward(dev(ids), dev(mask)).cpu().numpy()
    err = float(np.abs(got - ref).max())
    n, agree, n_safe, agree_safe = argmax_stats(spec, got, ref)
    say(f"  {name}, whole batch of {spec.batch}: max |dlogit| {err:.4g}; argmax agree {agree}/{n}; margin > 4e-2: {agree_safe}/{n_safe}")
    assert err <= 2e-2 and agree_safe == n_safe
    if name == "latency":                                # smaller request sizes are prefixes of the same batch
        for b in (1, 2, 4):
            ids_b, mask_b, _ = ms.make_inputs(spec, batch=b)
            assert np.array_equal(ids_b, ids[:b]) and np.array_equal(mask_b, mask[:b])
            got_b = model.forward(dev(ids_b), dev(mask_b)).cpu().numpy()
            assert np.abs(got_b - ref[:b]).max() <= 2e-2
    if name == "hetero":                                 # and four request batches in one call
        model.close()
        model, _ = mt.load_synthetic(spec, max_batch=4 * spec.batch)
        reqs = [(dev(ids), dev(mask))]
        for r in range(1, 4):
            i2, m2, _ = ms.make_inputs(spec, batch_index=r)
            reqs.append((dev(i2), dev(m2)))
        outs = model.forward_multi(reqs)
        assert np.abs(outs[0].cpu().numpy() - ref).max() <= 2e-2
    model.close()
