"""Pins for the CPU oracle: values the paper prints, closed forms, invariants, library routines and a
brute-force second implementation.  None of these tests touches the GPU library."""
import math
import os
import re

import numpy as np
import pytest

import mt_synth as ms
import oracle
from oracle import brute_tiny

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_layer_counts.txt")

MINI = ms.MTSpec("mini", vocab=50, hidden=32, heads=4, ffn=64, max_pos=24, n_trunk_layers=3,
                 tasks=(ms.TaskSpec(1, 2, 2), ms.TaskSpec(3, 1, 3), ms.TaskSpec(2, 0, 1), ms.TaskSpec(0, 1, 2)),
                 precision="fp32", batch=3, seq=12, len_lo=3, len_hi=12, input_seed=77, weights_seed=4242)


def build(spec, stress=False, std=0.02):
    tr, tri = ms.make_trunk_params(spec, stress=stress, std=std)
    tp, tpi = zip(*[ms.make_task_params(spec, t, stress=stress, std=std) for t in range(spec.n_tasks)])
    return tr, tri, list(tp), list(tpi)


def layer_slice(spec, flat, index, l):
    off = {n: o for n, _, o in index}[f"L{l}.Wq"]
    return flat[off:off + oracle.layer_param_count(spec.hidden, spec.ffn)]


# ------------------------------------------------------------------ P1: the paper's printed layer counts

def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        label, _src, tuples, shared, own, total = [c.strip() for c in line.split("|")]
        tl = [(int(a), int(b)) for a, b in re.findall(r"\((\d+),(\d+)\)", tuples)]
        rows.append((label, tl, int(shared), int(own), int(total)))
    return rows


@pytest.mark.parametrize("label,tuples,shared,own,total", _golden_rows())
def test_overhead_matches_paper(label, tuples, shared, own, total):
    assert shared + own == total
    if tuples:
        assert max(x for x, _ in tuples) == shared and sum(y for _, y in tuples) == own
        assert oracle.overhead(tuples) == total


def test_overhead_kd_n_rows():
    # Table 2 "Ours (KD-n)": every student keeps its teacher's frozen layers (Section 3.2) and gets n own layers.
    frozen = [2, 7, 2, 4, 6, 7, 4, 4]
    for n, total in ((1, 15), (2, 23), (3, 31)):
        assert oracle.overhead([(x, n) for x in frozen]) == total
    # Appendix E: 21 tasks on 8 shared layers with 32 task layers in total.
    ys = [2] * 11 + [1] * 10
    assert oracle.overhead([(8, y) for y in ys]) == 40 and abs(sum(ys) / 21 - 1.5) < 0.03


# ------------------------------------------------------------------ P10: single operations vs library routines

def test_linear_vs_numpy_fp64():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 45)).astype(np.float32)
    w = rng.standard_normal((11, 45)).astype(np.float32)
    b = rng.standard_normal(11).astype(np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b
    np.testing.assert_allclose(oracle.linear(x, w, b), ref, rtol=0, atol=2e-6)
    # a transposed operand or a dropped bias must fail
    assert np.abs(oracle.linear(x, w, None) - ref).max() > 1e-2
    np.testing.assert_allclose(oracle.linear(x, w, None), ref - b, rtol=0, atol=2e-6)


def test_gelu_vs_libm_and_torch():
    import torch
    x = np.linspace(-6, 6, 1001).astype(np.float32)
    ref = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x.astype(np.float64)])
    np.testing.assert_allclose(oracle.gelu(x), ref, rtol=1e-7, atol=1e-9)
    t = torch.from_numpy(x).double()
    np.testing.assert_allclose(oracle.gelu(x), torch.nn.functional.gelu(t).numpy(), rtol=1e-7, atol=1e-9)
    np.testing.assert_allclose(oracle.gelu(x, tanh_form=True),
                               torch.nn.functional.gelu(t, approximate="tanh").numpy(), rtol=1e-7, atol=1e-9)
    assert np.abs(oracle.gelu(x) - oracle.gelu(x, tanh_form=True)).max() > 1e-4   # the two forms differ


def test_softmax_vs_scipy():
    from scipy.special import softmax
    rng = np.random.default_rng(1)
    s = (rng.standard_normal(37) * 5).astype(np.float32)
    s[[3, 9]] += -10000.0
    p = oracle.softmax_row(s)
    np.testing.assert_allclose(p, softmax(s.astype(np.float64)), rtol=0, atol=1e-7)
    assert p[3] == 0.0 and p[9] == 0.0 and abs(p.sum() - 1) < 1e-6 and (p >= 0).all()


def test_layernorm_vs_numpy_and_properties():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((5, 64)) * 3 + 1.5).astype(np.float32)
    r = rng.standard_normal((5, 64)).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(64)).astype(np.float32)
    b = (0.1 * rng.standard_normal(64)).astype(np.float32)
    v = x.astype(np.float64) + r
    ref = g * (v - v.mean(1, keepdims=True)) / np.sqrt(v.var(1, keepdims=True) + 1e-12) + b
    np.testing.assert_allclose(oracle.layernorm(x, g, b, 1e-12, residual=r), ref, rtol=0, atol=1e-6)
    import torch
    tref = torch.nn.functional.layer_norm(torch.from_numpy(v), (64,), torch.from_numpy(g).double(),
                                          torch.from_numpy(b).double(), 1e-12).numpy()
    np.testing.assert_allclose(oracle.layernorm(x, g, b, 1e-12, residual=r), tref, rtol=0, atol=1e-6)
    # P6: gamma=1, beta=0 -> zero mean, unit (biased) variance, idempotent
    one, zero = np.ones(64, np.float32), np.zeros(64, np.float32)
    y = oracle.layernorm(x, one, zero)
    assert np.abs(y.mean(1)).max() <= 1e-6
    assert np.abs(y.astype(np.float64).var(1) - 1).max() <= 1e-5
    np.testing.assert_allclose(oracle.layernorm(y, one, zero), y, rtol=0, atol=1e-6)
    # eps sits inside the square root: a constant row maps to beta, not NaN
    c = np.full((1, 64), 2.5, np.float32)
    np.testing.assert_array_equal(oracle.layernorm(c, g, b, 1e-12), b[None, :])


def test_encoder_layer_vs_torch_transformer_layer():
    """The layer arithmetic is the post-LN Transformer encoder layer; torch's float64 implementation
    of that textbook block is an independent writing of it."""
    import torch
    spec = MINI
    tr, tri, tp, tpi = build(spec, stress=True, std=0.15)
    lp = layer_slice(spec, tr, tri, 1)
    P = {n.split(".")[1]: tr[o:o + int(np.prod(s))].reshape(s).astype(np.float64)
         for n, s, o in tri if n.startswith("L1.")}
    H, F, A = spec.hidden, spec.ffn, spec.heads
    layer = torch.nn.TransformerEncoderLayer(H, A, F, dropout=0.0, activation="gelu", layer_norm_eps=1e-12,
                                             batch_first=True, norm_first=False, dtype=torch.float64)
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(torch.from_numpy(np.concatenate([P["Wq"], P["Wk"], P["Wv"]])))
        layer.self_attn.in_proj_bias.copy_(torch.from_numpy(np.concatenate([P["bq"], P["bk"], P["bv"]])))
        layer.self_attn.out_proj.weight.copy_(torch.from_numpy(P["Wo"]))
        layer.self_attn.out_proj.bias.copy_(torch.from_numpy(P["bo"]))
        layer.linear1.weight.copy_(torch.from_numpy(P["W1"])); layer.linear1.bias.copy_(torch.from_numpy(P["b1"]))
        layer.linear2.weight.copy_(torch.from_numpy(P["W2"])); layer.linear2.bias.copy_(torch.from_numpy(P["b2"]))
        layer.norm1.weight.copy_(torch.from_numpy(P["ln1_g"])); layer.norm1.bias.copy_(torch.from_numpy(P["ln1_b"]))
        layer.norm2.weight.copy_(torch.from_numpy(P["ln2_g"])); layer.norm2.bias.copy_(torch.from_numpy(P["ln2_b"]))
    layer.train()   # keeps torch on its plain (non-fused) path; dropout is 0
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 12, H)).astype(np.float32)
    lengths = np.array([12, 5, 1])
    mask = (np.arange(12)[None, :] < lengths[:, None]).astype(np.int32)
    with torch.no_grad():
        ref = layer(torch.from_numpy(x).double(), src_key_padding_mask=torch.from_numpy(mask == 0)).numpy()
    got = oracle.encoder_layer(spec, lp, x, mask)
    valid = mask.astype(bool)
    assert np.abs(got[valid] - ref[valid]).max() <= 5e-6


# ------------------------------------------------------------------ P5 / P8: attention

def test_attention_probabilities_and_uniform_case():
    rng = np.random.default_rng(4)
    B, S, H, A = 2, 9, 24, 3
    q = rng.standard_normal((B, S, H)).astype(np.float32)
    k = rng.standard_normal((B, S, H)).astype(np.float32)
    v = rng.standard_normal((B, S, H)).astype(np.float32)
    mask = np.array([[1, 1, 1, 1, 1, 0, 0, 0, 0], [1, 0, 1, 1, 0, 1, 1, 1, 0]], np.int32)
    ctx, p = oracle.attention(q, k, v, mask, A, want_probs=True)
    assert np.abs(p.sum(-1) - 1).max() <= 1e-6 and (p >= 0).all()
    assert (p[0][:, :, 5:] == 0).all() and (p[1][:, :, [1, 4, 8]] == 0).all()
    # reference by definition, per head, float64
    d = H // A
    for b in range(B):
        for a in range(A):
            sl = slice(a * d, (a + 1) * d)
            s = q[b, :, sl].astype(np.float64) @ k[b, :, sl].astype(np.float64).T / math.sqrt(d)
            s = s + np.where(mask[b] == 1, 0.0, -10000.0)[None, :]
            e = np.exp(s - s.max(1, keepdims=True))
            pr = e / e.sum(1, keepdims=True)
            np.testing.assert_allclose(p[b, a], pr, rtol=0, atol=1e-6)
            np.testing.assert_allclose(ctx[b, :, sl], pr @ v[b, :, sl].astype(np.float64), rtol=0, atol=2e-6)
    # P8: zero queries -> uniform weights over valid keys -> context is the masked mean of V
    ctx0 = oracle.attention(np.zeros_like(q), k, v, mask, A)
    for b in range(B):
        mean_v = v[b][mask[b] == 1].astype(np.float64).mean(0)
        np.testing.assert_allclose(ctx0[b], np.broadcast_to(mean_v, (S, H)), rtol=0, atol=1e-6)


# ------------------------------------------------------------------ P7: brute force on tiny shapes

@pytest.mark.parametrize("spec,stress", [(ms.get_config("tiny"), False), (ms.get_config("tiny"), True),
                                          (MINI, True)])
def test_oracle_vs_brute_force(spec, stress):
    std = 0.02 if spec.name == "tiny" else 0.1
    tr, tri, tp, tpi = build(spec, stress=stress, std=std)
    ids, mask, _ = ms.make_inputs(spec)
    lg = oracle.Oracle(spec, tr, tp).mt_forward(ids, mask)
    T = brute_tiny.unpack(tr, tri)
    col = 0
    for t, task in enumerate(spec.tasks):
        K = brute_tiny.unpack(tp[t], tpi[t])
        for b in range(ids.shape[0]):
            ref = brute_tiny.student_logits(T, K, ids[b].tolist(), mask[b].tolist(), fork_layer=task.fork_layer,
                                            n_layers=task.n_layers, heads=spec.heads, eps=spec.ln_eps)
            assert np.abs(lg[b, col:col + task.n_classes] - np.array(ref)).max() <= (1e-6 if std == 0.02 else 5e-6)
        col += task.n_classes


def test_tanh_gelu_switch_reaches_the_model():
    import dataclasses
    spec = dataclasses.replace(MINI, gelu="tanh")
    tr, tri, tp, tpi = build(spec, stress=True, std=0.1)
    ids, mask, _ = ms.make_inputs(spec)
    lg_t = oracle.Oracle(spec, tr, tp).mt_forward(ids, mask)
    lg_e = oracle.Oracle(MINI, tr, tp).mt_forward(ids, mask)
    assert np.abs(lg_t - lg_e).max() > 1e-6
    T, K = brute_tiny.unpack(tr, tri), brute_tiny.unpack(tp[0], tpi[0])
    ref = brute_tiny.student_logits(T, K, ids[0].tolist(), mask[0].tolist(), fork_layer=1, n_layers=2,
                                    heads=spec.heads, eps=spec.ln_eps, tanh_form=True)
    assert np.abs(lg_t[0, :2] - np.array(ref)).max() <= 5e-6


# ------------------------------------------------------------------ segment (token type) ids for sentence-pair inputs

def _segments(mask, rng):
    """Sentence-pair style ids: 0 up to a split point inside the sequence, 1 after it."""
    tt = np.zeros_like(mask)
    for b in range(mask.shape[0]):
        n = int(mask[b].sum())
        cut = int(rng.integers(1, max(2, n)))
        tt[b, cut:] = 1
    return tt


def test_segment_ids_zero_is_the_default_and_brute_force_agrees():
    spec = MINI
    tr, tri, tp, tpi = build(spec, stress=True, std=0.1)
    ids, mask, _ = ms.make_inputs(spec)
    orc = oracle.Oracle(spec, tr, tp)
    base = orc.mt_forward(ids, mask)
    np.testing.assert_array_equal(orc.mt_forward(ids, mask, type_ids=np.zeros_like(ids)), base)
    tt = _segments(mask, np.random.default_rng(5))
    lg = orc.mt_forward(ids, mask, type_ids=tt)
    assert np.abs(lg - base).max() > 1e-6                         # the second table row is really used
    T = brute_tiny.unpack(tr, tri)
    col = 0
    for t, task in enumerate(spec.tasks):
        K = brute_tiny.unpack(tp[t], tpi[t])
        np.testing.assert_array_equal(orc.st_forward(t, ids, mask, type_ids=tt), lg[:, col:col + task.n_classes])
        for b in range(ids.shape[0]):
            ref = brute_tiny.student_logits(T, K, ids[b].tolist(), mask[b].tolist(), fork_layer=task.fork_layer, n_layers=task.n_layers,
                                            heads=spec.heads, eps=spec.ln_eps, type_ids=tt[b].tolist())
            assert np.abs(lg[b, col:col + task.n_classes] - np.array(ref)).max() <= 5e-6
        col += task.n_classes


def test_segment_ids_relabelling_invariance():
    """Swapping the two rows of the type table and flipping every id is the same model: identical logits."""
    spec = MINI
    tr, tri, tp, _ = build(spec, stress=True, std=0.1)
    ids, mask, _ = ms.make_inputs(spec)
    tt = _segments(mask, np.random.default_rng(6))
    lg = oracle.Oracle(spec, tr, tp).mt_forward(ids, mask, type_ids=tt)
    off = {n: o for n, _, o in tri}["type_emb"]
    H = spec.hidden
    tr2 = tr.copy()
    tr2[off:off + H], tr2[off + H:off + 2 * H] = tr[off + H:off + 2 * H], tr[off:off + H]
    np.testing.assert_array_equal(oracle.Oracle(spec, tr2, tp).mt_forward(ids, mask, type_ids=1 - tt), lg)


# ------------------------------------------------------------------ token-level heads (tagging / slot-filling tasks, Appendix E)

TOK = ms.MTSpec("tok", vocab=50, hidden=32, heads=4, ffn=64, max_pos=24, n_trunk_layers=2,
                tasks=(ms.TaskSpec(1, 1, 2), ms.TaskSpec(2, 1, 5, token_level=True), ms.TaskSpec(2, 0, 3),
                       ms.TaskSpec(0, 2, 4, token_level=True), ms.TaskSpec(1, 0, 32, token_level=True)),
                precision="fp32", batch=3, seq=10, len_lo=2, len_hi=10, input_seed=78, weights_seed=4243)


def test_token_head_layout_and_brute_force():
    spec = TOK
    assert spec.n_logits == 5 and spec.n_token_logits == 41
    assert [spec.logit_offset(t) for t in range(5)] == [0, 0, 2, 5, 9]
    tr, tri, tp, tpi = build(spec, stress=True, std=0.1)
    assert tp[1].size == oracle.layer_param_count(32, 64) + 5 * 32 + 5          # no pooler in a token-level scope
    ids, mask, _ = ms.make_inputs(spec)
    orc = oracle.Oracle(spec, tr, tp)
    lg, tok = orc.mt_forward(ids, mask, want_tokens=True)
    assert lg.shape == (3, 5) and tok.shape == (3, 10, 41)
    T = brute_tiny.unpack(tr, tri)
    for t, task in enumerate(spec.tasks):
        K = brute_tiny.unpack(tp[t], tpi[t])
        c0 = spec.logit_offset(t)
        for b in range(ids.shape[0]):
            ref = np.array(brute_tiny.student_logits(T, K, ids[b].tolist(), mask[b].tolist(), fork_layer=task.fork_layer,
                                                     n_layers=task.n_layers, heads=spec.heads, eps=spec.ln_eps,
                                                     token_level=task.token_level))
            got = tok[b, :, c0:c0 + task.n_classes] if task.token_level else lg[b, c0:c0 + task.n_classes]
            assert got.shape == ref.shape and np.abs(got - ref).max() <= 5e-6
        # the merged model's columns are the student's own outputs
        alone = orc.st_forward(t, ids, mask)
        np.testing.assert_array_equal(alone, tok[:, :, c0:c0 + task.n_classes] if task.token_level else lg[:, c0:c0 + task.n_classes])


def test_token_head_with_unit_rows_reads_the_hidden_state():
    """A token-level task without own layers whose head is [I | 0] with zero bias returns the trunk's hidden state at
    its fork, position by position: the head is a plain per-token linear map and nothing else."""
    spec = TOK
    tr, tri, tp, tpi = build(spec, stress=True, std=0.1)
    H = spec.hidden
    off = {n: o for n, _, o in tpi[4]}
    tp[4][off["Wc"]:off["Wc"] + 32 * H] = np.eye(32, H, dtype=np.float32).ravel()
    tp[4][off["bc"]:off["bc"] + 32] = 0.0
    ids, mask, _ = ms.make_inputs(spec)
    lg, tok, hidden = oracle.Oracle(spec, tr, tp).mt_forward(ids, mask, want_tokens=True, want_hidden=True)
    np.testing.assert_array_equal(tok[:, :, 9:41], hidden[1][:, :, :32])
    # ... and a bias shifts every position by the same vector
    tp[4][off["bc"]:off["bc"] + 32] = np.arange(32, dtype=np.float32)
    _, tok2 = oracle.Oracle(spec, tr, tp).mt_forward(ids, mask, want_tokens=True)
    np.testing.assert_allclose(tok2[:, :, 9:41] - tok[:, :, 9:41], np.broadcast_to(np.arange(32, dtype=np.float32), (3, 10, 32)),
                               rtol=0, atol=1e-5)


def test_token_logits_ignore_padding_and_other_sequences():
    spec = TOK
    tr, _, tp, _ = build(spec, stress=True, std=0.1)
    ids, mask, lens = ms.make_inputs(spec)
    orc = oracle.Oracle(spec, tr, tp)
    _, tok = orc.mt_forward(ids, mask, want_tokens=True)
    ids2 = ids.copy()
    ids2[mask == 0] = (ids2[mask == 0] + 7) % spec.vocab              # other tokens under the padding
    _, tok2 = orc.mt_forward(ids2, mask, want_tokens=True)
    assert int((mask == 0).sum()) > 0
    np.testing.assert_allclose(tok2[mask == 1], tok[mask == 1], rtol=0, atol=1e-6)
    for b in range(ids.shape[0]):                                      # each sequence on its own, cut to its length
        n = int(lens[b])
        _, one = orc.mt_forward(ids[b:b + 1, :n], mask[b:b + 1, :n], want_tokens=True)
        np.testing.assert_allclose(one[0], tok[b, :n], rtol=0, atol=2e-6)


def test_token_tasks_need_their_output_buffer():
    spec = TOK
    tr, _, tp, _ = build(spec)
    ids, mask, _ = ms.make_inputs(spec)
    orc = oracle.Oracle(spec, tr, tp)
    import ctypes as C
    from oracle import binding as ob
    lg = np.empty((3, 5), dtype=np.float32)
    ptrs = (C.POINTER(C.c_float) * 5)(*[ob._fp(p) for p in orc.task_params])
    rc = ob.lib().orc_mt_forward_typed(C.byref(orc.cfg), orc.tasks, ob._fp(orc.trunk), ptrs, ob._ip(ids), None, ob._ip(mask),
                                       C.c_int64(3), C.c_int64(10), ob._fp(lg), None)
    assert rc == -1


# ------------------------------------------------------------------ P2 / P3: merging is exact, tasks are isolated

@pytest.mark.parametrize("spec", [ms.get_config("tiny"), MINI])
def test_merged_equals_each_student_alone(spec):
    tr, _, tp, _ = build(spec, stress=True, std=0.1)
    ids, mask, _ = ms.make_inputs(spec)
    orc = oracle.Oracle(spec, tr, tp)
    lg = orc.mt_forward(ids, mask)
    col = 0
    for t, task in enumerate(spec.tasks):
        np.testing.assert_array_equal(lg[:, col:col + task.n_classes], orc.st_forward(t, ids, mask))
        col += task.n_classes


def test_task_isolation():
    spec = MINI
    tr, _, tp, _ = build(spec, stress=True, std=0.1)
    ids, mask, _ = ms.make_inputs(spec)
    base = oracle.Oracle(spec, tr, tp).mt_forward(ids, mask)
    tp2 = list(tp)
    tp2[1] = ms.make_task_params(spec, 1, stress=True, std=0.1, seed=999)[0]
    other = oracle.Oracle(spec, tr, tp2).mt_forward(ids, mask)
    np.testing.assert_array_equal(other[:, :2], base[:, :2])
    np.testing.assert_array_equal(other[:, 5:], base[:, 5:])
    assert np.abs(other[:, 2:5] - base[:, 2:5]).max() > 1e-4


# ------------------------------------------------------------------ P4 / P11: padding invariance, batch equivariance

def test_padding_invariance():
    spec = MINI
    tr, _, tp, _ = build(spec, stress=True, std=0.1)
    orc = oracle.Oracle(spec, tr, tp)
    ids, mask, lengths = ms.make_inputs(spec, len_hi=9)
    base = orc.mt_forward(ids, mask)
    # (a) token ids under the mask do not matter
    ids2 = ids.copy()
    ids2[mask == 0] = (ids2[mask == 0] * 7 + 3) % spec.vocab
    assert (ids2 != ids).any()
    np.testing.assert_array_equal(orc.mt_forward(ids2, mask), base)
    # (b) truncating to the longest sequence, (c) padding further
    L = int(lengths.max())
    np.testing.assert_allclose(orc.mt_forward(ids[:, :L], mask[:, :L]), base, rtol=0, atol=1e-6)
    idp = np.concatenate([ids, np.full((ids.shape[0], 5), 11, np.int32)], 1)
    mkp = np.concatenate([mask, np.zeros((ids.shape[0], 5), np.int32)], 1)
    np.testing.assert_allclose(orc.mt_forward(idp, mkp), base, rtol=0, atol=1e-6)
    # a masked key in the middle of a sequence is ignored as well
    m3 = mask.copy(); m3[:, 2] = 0
    i3 = ids.copy(); i3[:, 2] = (i3[:, 2] + 1) % spec.vocab
    np.testing.assert_array_equal(orc.mt_forward(i3, m3), orc.mt_forward(ids, m3))
    assert np.abs(orc.mt_forward(ids, m3) - base).max() > 1e-5      # but masking a real token does change the result


def test_batch_equivariance():
    spec = MINI
    tr, _, tp, _ = build(spec, stress=True, std=0.1)
    orc = oracle.Oracle(spec, tr, tp)
    ids, mask, _ = ms.make_inputs(spec, batch=4)
    base = orc.mt_forward(ids, mask)
    perm = np.array([2, 0, 3, 1])
    np.testing.assert_array_equal(orc.mt_forward(ids[perm], mask[perm]), base[perm])
    for b in range(4):
        np.testing.assert_array_equal(orc.mt_forward(ids[b:b + 1], mask[b:b + 1])[0], base[b])


# ------------------------------------------------------------------ P9: a layer whose output projections vanish is the identity

def test_identity_layer_special_case():
    spec = MINI
    tr, tri, tp, tpi = build(spec, stress=False, std=0.1)       # gamma=1, beta=0, biases 0
    lp = layer_slice(spec, tr, tri, 0).copy()
    names = ms.layer_tensors(spec.hidden, spec.ffn)
    off = 0
    for n, s in names:
        size = int(np.prod(s))
        if n in ("Wo", "bo", "W2", "b2"):
            lp[off:off + size] = 0
        off += size
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 6, spec.hidden)).astype(np.float32)
    one, zero = np.ones(spec.hidden, np.float32), np.zeros(spec.hidden, np.float32)
    xn = oracle.layernorm(x.reshape(-1, spec.hidden), one, zero).reshape(x.shape)
    out = oracle.encoder_layer(spec, lp, xn, np.ones((2, 6), np.int32))
    np.testing.assert_allclose(out, xn, rtol=0, atol=2e-6)
    # a model with one more such layer in a branch gives the same logits and costs exactly one more layer
    assert oracle.overhead([(3, 2), (3, 1)]) == oracle.overhead([(3, 1), (3, 1)]) + 1


def test_all_keys_masked_row_stays_finite():
    q = np.ones((1, 3, 8), np.float32)
    ctx, p = oracle.attention(q, q, q, np.zeros((1, 3), np.int32), 2, want_probs=True)
    assert np.isfinite(ctx).all() and np.allclose(p, 1 / 3)
