"""Brute-force float64 evaluation of one student model, one output element at a time.

TEST INFRASTRUCTURE ONLY.  A second, independent writing of the definition used to pin
mt_oracle.c on tiny shapes: pure Python loops over scalars, float64 throughout, no intermediate
rounding, no code shared with the C oracle or the GPU library.  It evaluates the single-task
student of paper Section 3.2/3.3 (x shared layers, y own layers, pooler, head) for ONE sequence;
the merged model must reproduce it for every task.

Parameters arrive as {name: float64 ndarray} dictionaries built from the canonical (name, shape,
offset) index of the flat parameter vectors.
"""
from __future__ import annotations

import math

import numpy as np


def unpack(flat, index):
    return {name: np.asarray(flat[off:off + int(np.prod(shape))], dtype=np.float64).reshape(shape)
            for name, shape, off in index}


def _layernorm(vec, gamma, beta, eps):
    n = len(vec)
    mu = sum(vec) / n
    var = sum((v - mu) ** 2 for v in vec) / n
    return [gamma[i] * (vec[i] - mu) / math.sqrt(var + eps) + beta[i] for i in range(n)]


def _affine(W, b, x):
    return [sum(W[o][i] * x[i] for i in range(len(x))) + b[o] for o in range(len(b))]


def _gelu(v, tanh_form):
    if tanh_form:
        return 0.5 * v * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))
    return 0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0)))


def _layer(P, pre, X, mask, heads, eps, tanh_form):
    S = len(X)
    H = len(X[0])
    d = H // heads
    g = lambda n: P[pre + n].tolist()
    Wq, bq, Wk, bk, Wv, bv, Wo, bo = g("Wq"), g("bq"), g("Wk"), g("bk"), g("Wv"), g("bv"), g("Wo"), g("bo")
    Q = [_affine(Wq, bq, x) for x in X]
    K = [_affine(Wk, bk, x) for x in X]
    V = [_affine(Wv, bv, x) for x in X]
    ctx = [[0.0] * H for _ in range(S)]
    for a in range(heads):
        cols = range(a * d, (a + 1) * d)
        for i in range(S):
            sc = []
            for j in range(S):
                dot = sum(Q[i][c] * K[j][c] for c in cols) / math.sqrt(d)
                sc.append(dot + (0.0 if mask[j] else -10000.0))
            mx = max(sc)
            ex = [math.exp(v - mx) for v in sc]
            tot = sum(ex)
            for c in cols:
                ctx[i][c] = sum(ex[j] / tot * V[j][c] for j in range(S))
    X1 = []
    for i in range(S):
        ao = _affine(Wo, bo, ctx[i])
        X1.append(_layernorm([X[i][c] + ao[c] for c in range(H)], g("ln1_g"), g("ln1_b"), eps))
    W1, b1, W2, b2 = g("W1"), g("b1"), g("W2"), g("b2")
    out = []
    for i in range(S):
        u = [_gelu(v, tanh_form) for v in _affine(W1, b1, X1[i])]
        fo = _affine(W2, b2, u)
        out.append(_layernorm([X1[i][c] + fo[c] for c in range(H)], g("ln2_g"), g("ln2_b"), eps))
    return out


def student_logits(trunk, task, ids, mask, *, fork_layer, n_layers, heads, eps=1e-12, tanh_form=False, type_ids=None,
                   token_level=False):
    """Logits of one student for ONE sequence.  trunk/task: dicts from unpack(); ids, mask: length-S lists.
    token_level: the student labels every token: a list of S rows of C logits, no pooler."""
    S = len(ids)
    word, pos, typ = trunk["word_emb"], trunk["pos_emb"], trunk["type_emb"]
    H = word.shape[1]
    X = []
    for s in range(S):
        seg = type_ids[s] if type_ids is not None else 0
        e = [float(word[ids[s]][c] + pos[s][c] + typ[seg][c]) for c in range(H)]
        X.append(_layernorm(e, trunk["emb_ln_g"].tolist(), trunk["emb_ln_b"].tolist(), eps))
    for l in range(fork_layer):
        X = _layer(trunk, f"L{l}.", X, mask, heads, eps, tanh_form)
    for l in range(n_layers):
        X = _layer(task, f"L{l}.", X, mask, heads, eps, tanh_form)
    if token_level:
        return [_affine(task["Wc"].tolist(), task["bc"].tolist(), X[s]) for s in range(S)]
    pooled = [math.tanh(v) for v in _affine(task["Wp"].tolist(), task["bp"].tolist(), X[0])]
    return _affine(task["Wc"].tolist(), task["bc"].tolist(), pooled)
