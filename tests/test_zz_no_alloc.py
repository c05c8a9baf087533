"""mt_forward_static (the forward pass that allocates nothing: its workspace is a fixed device array inside the
library) against mt_forward on the same model and inputs, through the C ABI.

Both run the same kernels on the same values, so the logits must be bit-identical; each is also held to the
oracle.  Two calls in a row share the array: the second, on a smaller input, must not be disturbed by what the
first left behind."""
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


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


BF = ms.MTSpec("static_bf16", vocab=500, hidden=128, heads=2, ffn=256, max_pos=64, n_trunk_layers=3,
               tasks=(ms.TaskSpec(3, 2, 2), ms.TaskSpec(1, 1, 3), ms.TaskSpec(2, 0, 1), ms.TaskSpec(0, 1, 2)),
               precision="bf16", batch=7, seq=44, len_lo=5, len_hi=44, input_seed=31, weights_seed=99)
F32 = dataclasses.replace(BF, name="static_fp32", precision="fp32", hidden=64, ffn=128)


def _model(spec, **kw):
    tr, tri = ms.make_trunk_params(spec, stress=True, std=0.05)
    tps = [ms.make_task_params(spec, t, stress=True, std=0.05) for t in range(spec.n_tasks)]
    model = mt.Model(mt.make_config(spec, **kw))
    model.load_params(-1, tr, len(tri))
    for t, (tp, tpi) in enumerate(tps):
        model.load_params(t, tp, len(tpi))
    return model, oracle.Oracle(spec, tr, [p for p, _ in tps])


@pytest.mark.parametrize("spec", [BF, F32], ids=["bf16", "fp32"])
def test_static_scratch_forward_equals_forward_twice_in_a_row(spec):
    assert torch.cuda.is_available()
    mt.lib()
    model, orc = _model(spec)
    assert model.workspace_bytes() <= mt.MT_STATIC_SCRATCH_BYTES
    tol = 2e-2 if spec.precision == "bf16" else None
    # first call: the whole batch; second call: fewer and shorter sequences, then the first again
    ids, mask, _ = ms.make_inputs(spec)
    ids2, mask2, _ = ms.make_inputs(spec, batch=3, seq=24, batch_index=1, len_hi=24)
    for (i, k) in ((ids, mask), (ids2, mask2), (ids, mask)):
        say(f"{spec.name}: batch {i.shape}")
        d_i, d_k = dev(i), dev(k)
        want = model.forward(d_i, d_k).cpu().numpy()
        out = torch.full((i.shape[0], model.n_logits), 7.0, dtype=torch.float32, device="cuda")
        got = model.forward_static(d_i, d_k, out).cpu().numpy()
        assert np.array_equal(got, want)
        ref = orc.mt_forward(i, k)
        bound = tol if tol is not None else 1e-4 * max(float(np.abs(ref).max()), 1e-3)
        assert np.abs(got - ref).max() <= bound
    # a task mask leaves the other columns untouched here too
    out = torch.full((ids.shape[0], model.n_logits), 7.0, dtype=torch.float32, device="cuda")
    model.forward_static(dev(ids), dev(mask), out, task_mask=[1, 0, 1, 0])
    o = out.cpu().numpy()
    full = model.forward(dev(ids), dev(mask)).cpu().numpy()
    assert np.array_equal(o[:, 0:2], full[:, 0:2]) and (o[:, 2:5] == 7.0).all()
    assert np.array_equal(o[:, 5:6], full[:, 5:6]) and (o[:, 6:8] == 7.0).all()
    model.close()


def test_static_scratch_forward_refuses_a_model_that_does_not_fit():
    spec = dataclasses.replace(ms.get_config("base"), n_trunk_layers=1, tasks=(ms.TaskSpec(1, 1, 2),), vocab=1000)
    model = mt.Model(mt.make_config(spec))            # 32 x 128 rows at BERT-base width: far beyond the array
    assert model.workspace_bytes() > mt.MT_STATIC_SCRATCH_BYTES
    ids, mask, _ = ms.make_inputs(spec, batch=1, seq=16, len_hi=16)
    out = torch.zeros((1, model.n_logits), dtype=torch.float32, device="cuda")
    with pytest.raises(mt.MTError) as ei:
        model.forward_static(dev(ids), dev(mask), out)
    assert ei.value.code == mt.MT_ERR_SHAPE and "static scratch" in str(ei.value)
    model.close()
