"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what include/mt.h
declares, validates configurations, counts layers like the paper, and reports call-order errors."""
import ctypes as C
import dataclasses
import os
import re

import numpy as np
import pytest

import mt_synth as ms
import paper_2107_05377_amd as mt
from paper_2107_05377_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(mt.LIB_PATH):
        from paper_2107_05377_amd.build import build
        build()


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mt.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(mt_[a-z0-9_]+)\s*\(", header)))
    assert "mt_create" in declared and "mt_forward" in declared and "mt_load_weights" in declared
    L = C.CDLL(mt.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), f"{name} declared in mt.h but not exported"
    assert sorted(binding.EXPORTS) == declared


def _create(spec, **kw):
    cfg = mt.make_config(spec, **kw)
    h = C.c_void_p()
    rc = mt.lib().mt_create(C.byref(cfg), C.byref(h))
    return rc, h, cfg


def test_create_and_sizes():
    spec = ms.get_config("base")
    rc, h, _ = _create(spec)
    assert rc == mt.MT_OK
    L = mt.lib()
    assert L.mt_layer_count(h) == 8 + 16            # 8 shared + 2 x 8 task layers
    assert L.mt_n_logits(h) == 16
    assert [L.mt_logit_offset(h, t) for t in range(8)] == [0, 2, 4, 6, 9, 11, 13, 15]
    assert L.mt_logit_offset(h, 8) == mt.MT_ERR_SHAPE
    wb = L.mt_weight_bytes(h)
    # embeddings, 24 layers of 12 H^2, per task the pooler stored as [W | W] (2 H^2) and the transposed key
    # matrix of its last layer (H^2), 16 classifier rows
    n_mat = (30522 + 512 + 2) * 768 + 24 * 12 * 768 * 768 + 8 * 3 * (768 * 768) + 16 * 768
    assert 2 * n_mat <= wb <= 2 * n_mat * 1.02           # bf16 matrices dominate the arena
    assert L.mt_workspace_bytes(h) > 8 * 4096 * 3072 * 2
    L.mt_destroy(h)


GOLD = [
    ("wo_kd", [(2, 10), (7, 5), (2, 10), (4, 8), (6, 6), (7, 5), (4, 8), (4, 8)], 67),
    ("mixed", [(2, 3), (7, 5), (2, 1), (4, 3), (6, 2), (7, 3), (4, 8), (4, 1)], 33),
    ("c2", [(2, 2), (7, 1), (2, 1), (4, 2), (6, 2), (7, 1), (4, 3), (4, 1)], 20),
    ("c3", [(2, 1), (7, 1), (2, 1), (4, 2), (6, 1), (7, 1), (4, 3), (4, 1)], 18),
    ("fig1c", [(4, 3), (8, 2)], 13),
]


@pytest.mark.parametrize("label,tuples,total", GOLD)
def test_layer_count_matches_paper_tables(label, tuples, total):
    """Table 2 / Table 5 (x, y) tuples and Fig. 1(c): shared depth + sum of task layers."""
    import dataclasses
    base = ms.get_config("base")
    spec = dataclasses.replace(base, n_trunk_layers=max(x for x, _ in tuples),
                               tasks=tuple(ms.TaskSpec(x, y, 2) for x, y in tuples))
    rc, h, _ = _create(spec)
    assert rc == mt.MT_OK
    assert mt.lib().mt_layer_count(h) == total
    mt.lib().mt_destroy(h)


def test_config_validation():
    import dataclasses
    base = ms.get_config("base")
    bad = [
        dataclasses.replace(base, n_trunk_layers=9),                                 # trunk deeper than any fork
        dataclasses.replace(base, tasks=(ms.TaskSpec(9, 1, 2),)),                     # fork beyond the trunk
        dataclasses.replace(base, tasks=(ms.TaskSpec(8, -1, 2),)),
        dataclasses.replace(base, tasks=(ms.TaskSpec(8, 1, 0),)),
        dataclasses.replace(base, heads=16),                                          # bf16 path needs head width 64
        dataclasses.replace(base, hidden=770, heads=11),
        dataclasses.replace(base, seq=1024, max_pos=512),                             # max_seq > max_pos
        dataclasses.replace(base, tasks=()),
        dataclasses.replace(base, seq=609, max_pos=1024),                             # bf16 attention keeps a sequence's keys in LDS
    ]
    for spec in bad:
        rc, h, _ = _create(spec)
        assert rc in (mt.MT_ERR_CONFIG, mt.MT_ERR_NULL), spec
        assert not h
    # fp32 validation mode takes any head width
    rc, h, _ = _create(ms.get_config("tiny"))
    assert rc == mt.MT_OK
    mt.lib().mt_destroy(h)
    # struct size / version guard
    cfg = mt.make_config(base)
    cfg.version = 99
    h = C.c_void_p()
    assert mt.lib().mt_create(C.byref(cfg), C.byref(h)) == mt.MT_ERR_CONFIG
    assert mt.lib().mt_create(None, C.byref(h)) == mt.MT_ERR_NULL


def test_call_order_and_blob_errors():
    spec = ms.get_config("tiny")
    rc, h, _ = _create(spec)
    assert rc == mt.MT_OK
    L = mt.lib()
    fake = C.c_void_p(0x10000)     # never dereferenced: every call below fails its host-side checks first
    assert L.mt_forward(h, fake, fake, 2, 16, None, fake, None) == mt.MT_ERR_STATE
    assert b"mt_bind" in L.mt_last_error(h)
    assert L.mt_load_weights(h, -1, fake, 100, None) == mt.MT_ERR_STATE
    assert L.mt_bind(h, None, 0, None, 0) == mt.MT_ERR_NULL
    assert L.mt_bind(h, fake, 16, fake, 16) == mt.MT_ERR_SHAPE
    assert L.mt_bind(h, C.c_void_p(0x10004), 1 << 40, fake, 1 << 40) == mt.MT_ERR_SHAPE      # alignment
    assert L.mt_bind(h, fake, 1 << 40, fake, 1 << 40) == mt.MT_OK
    assert L.mt_forward(h, fake, fake, 2, 16, None, fake, None) == mt.MT_ERR_STATE            # nothing loaded
    assert L.mt_forward(h, fake, fake, 3, 16, None, fake, None) == mt.MT_ERR_SHAPE            # batch > max_batch
    assert L.mt_forward(h, fake, fake, 2, 17, None, fake, None) == mt.MT_ERR_SHAPE
    assert L.mt_forward(h, None, fake, 2, 16, None, fake, None) == mt.MT_ERR_NULL
    trunk, tri = ms.make_trunk_params(spec)
    good = mt.pack_blob(-1, len(tri), trunk)
    for blob in (b"XXXX" + good[4:], good[:-4], good + b"\0\0\0\0", mt.pack_blob(0, len(tri), trunk),
                 mt.pack_blob(-1, len(tri) + 1, trunk), good[:10]):
        buf = C.create_string_buffer(blob, len(blob))
        assert L.mt_load_weights(h, -1, C.cast(buf, C.c_void_p), len(blob), None) == mt.MT_ERR_BLOB
    assert L.mt_load_weights(h, 5, C.cast(C.create_string_buffer(good, len(good)), C.c_void_p), len(good), None) == mt.MT_ERR_BLOB
    assert L.mt_read_hidden(h, -1, 2, fake, 1 << 30, None) == mt.MT_ERR_STATE
    assert L.mt_error_name(mt.MT_ERR_BLOB) == b"MT_ERR_BLOB"
    L.mt_destroy(h)


def test_industrial_workload_layer_count():
    """Appendix E: 21 tasks served by 40 transformer layers, 8 of them shared."""
    spec = ms.get_config("industrial")
    assert spec.n_tasks == 21 and spec.n_trunk_layers == 8 and sum(t.n_layers for t in spec.tasks) == 32
    rc, h, _ = _create(spec)
    assert rc == mt.MT_OK
    assert mt.lib().mt_layer_count(h) == 40
    assert mt.lib().mt_n_logits(h) == sum(t.n_classes for t in spec.tasks)
    mt.lib().mt_destroy(h)


def test_token_level_heads_layout_and_checks():
    """Tagging tasks (Appendix E) sit in a per-token logit row of their own; their scope has no pooler."""
    spec = ms.get_config("assistant")
    assert spec.n_tasks == 21 and [t for t, k in enumerate(spec.tasks) if k.token_level] == [7, 12, 15]
    rc, h, _ = _create(spec)
    assert rc == mt.MT_OK
    L = mt.lib()
    assert L.mt_layer_count(h) == 40
    assert L.mt_n_token_logits(h) == 30 + 16 + 9 == spec.n_token_logits
    assert L.mt_n_logits(h) == spec.n_logits == sum(t.n_classes for t in spec.tasks) - 55
    assert [L.mt_token_logit_offset(h, t) for t in (7, 12, 15)] == [0, 30, 46]
    assert L.mt_token_logit_offset(h, 0) == mt.MT_ERR_CONFIG and L.mt_logit_offset(h, 7) == mt.MT_ERR_CONFIG
    assert L.mt_token_logit_offset(h, 21) == mt.MT_ERR_SHAPE
    assert [L.mt_logit_offset(h, t) for t in (0, 6, 8)] == [spec.logit_offset(t) for t in (0, 6, 8)]
    # the same table with sequence heads only stores, for each of the three tasks, a pooler as [W | W] (2 H^2) and the
    # transposed key matrix of its last layer (H^2): 3 * 3 H^2 bf16 values more
    rc2, h2, _ = _create(ms.get_config("industrial"))
    assert rc2 == mt.MT_OK
    diff = L.mt_weight_bytes(h2) - L.mt_weight_bytes(h)
    assert 2 * 9 * 768 * 768 <= diff <= 2 * 9 * 768 * 768 + 3 * 768 * 4 + 4096
    L.mt_destroy(h2)
    # a token-level task needs the token buffer
    fake = C.c_void_p(0x10000)     # never dereferenced: the calls below fail their host-side checks first
    assert L.mt_bind(h, fake, 1 << 40, fake, 1 << 40) == mt.MT_OK
    cfg = mt.make_config(spec)
    cfg.tasks[3].head = 2
    hb = C.c_void_p()
    assert L.mt_create(C.byref(cfg), C.byref(hb)) == mt.MT_ERR_CONFIG
    # blob size of a token-level scope: layers + Wc + bc, two tensors after the layers
    flat, idx = ms.make_task_params(spec, 7)
    assert len(idx) == 16 * spec.tasks[7].n_layers + 2
    blob = mt.pack_blob(7, len(idx) + 2, flat)
    buf = C.create_string_buffer(blob, len(blob))
    assert L.mt_load_weights(h, 7, C.cast(buf, C.c_void_p), len(blob), None) == mt.MT_ERR_BLOB
    L.mt_destroy(h)


def test_wavefront_schedule_step_counts():
    """A branch starts as soon as its tap exists: steps = max over tasks of fork + own layers (Fig. 1(c))."""
    L = mt.lib()
    _, h, _ = _create(ms.get_config("base"))
    assert L.mt_schedule_steps(h, None) == 8 + 2
    L.mt_destroy(h)
    spec = ms.get_config("hetero")                      # forks 11,10,9,8,7,6,6,8 with 1,1,2,2,3,3,3,2 own layers
    _, h, _ = _create(spec)
    assert L.mt_schedule_steps(h, None) == 12           # a trunk-first schedule would take 11 + 3 = 14
    only = (C.c_uint8 * 8)(0, 0, 0, 0, 0, 1, 0, 0)      # task 5 alone: fork 6 + 3 layers
    assert L.mt_schedule_steps(h, only) == 9
    L.mt_destroy(h)
    fig = ms.MTSpec("fig1c", vocab=100, hidden=64, heads=1, ffn=64, max_pos=16, n_trunk_layers=8,
                    tasks=(ms.TaskSpec(4, 3, 2), ms.TaskSpec(8, 2, 2)), precision="fp32", batch=1, seq=8, len_lo=1, len_hi=8,
                    input_seed=1)
    _, h, _ = _create(fig)
    assert L.mt_layer_count(h) == 13 and L.mt_schedule_steps(h, None) == 10
    L.mt_destroy(h)


def test_paper_task_tables_as_workloads():
    """Table 2: the undistilled table needs 7 + 60 = 67 layers, the mixed one 7 + 26 = 33; in the wavefront schedule
    the deepest chain decides the step count (fork 2 + 10 own layers, fork 4 + 8 own layers = 12)."""
    L = mt.lib()
    for name, total, steps in (("wo_kd", 67, 12), ("mixed", 33, 12)):
        rc, h, _ = _create(ms.get_config(name))
        assert rc == mt.MT_OK
        assert L.mt_layer_count(h) == total
        assert L.mt_schedule_steps(h, None) == steps
        L.mt_destroy(h)


def test_share_weights_checks():
    """A replica must match the owner's configuration, share its weight arena, bring a workspace of its own,
    and the owner must have something loaded."""
    L = mt.lib()
    spec = ms.get_config("tiny")
    _, a, _ = _create(spec)
    _, b, _ = _create(spec)
    _, c, _ = _create(ms.get_config("hetero"))
    w, ws1, ws2 = C.c_void_p(0x10000), C.c_void_p(0x20000), C.c_void_p(0x30000)
    assert L.mt_share_weights(None, a) == mt.MT_ERR_NULL
    assert L.mt_bind(a, w, 1 << 40, ws1, 1 << 40) == mt.MT_OK
    assert L.mt_share_weights(c, a) == mt.MT_ERR_CONFIG
    assert L.mt_share_weights(b, a) == mt.MT_ERR_STATE                  # b not bound
    assert L.mt_bind(b, ws2, 1 << 40, ws2, 1 << 40) == mt.MT_OK
    assert L.mt_share_weights(b, a) == mt.MT_ERR_STATE                  # other weight arena
    assert L.mt_bind(b, w, 1 << 40, ws1, 1 << 40) == mt.MT_OK
    assert L.mt_share_weights(b, a) == mt.MT_ERR_STATE                  # same workspace
    assert L.mt_bind(b, w, 1 << 40, ws2, 1 << 40) == mt.MT_OK
    assert L.mt_share_weights(b, a) == mt.MT_ERR_STATE                  # owner has nothing loaded
    assert b"nothing loaded" in L.mt_last_error(b) or b"no weights" in L.mt_last_error(b)
    for h in (a, b, c):
        L.mt_destroy(h)


def test_op_entry_points_reject_bad_arguments():
    L = mt.lib()
    fake = C.c_void_p(0x10000)
    assert L.mt_op_linear(mt.MT_BF16, None, 8, fake, None, None, fake, 8, 4, 8, 64, 0, 0, None) == mt.MT_ERR_NULL
    assert L.mt_op_linear(mt.MT_BF16, fake, 8, fake, None, None, fake, 8, 0, 8, 64, 0, 0, None) == mt.MT_ERR_SHAPE
    assert L.mt_op_linear(mt.MT_BF16, fake, 72, fake, None, None, fake, 8, 4, 8, 72, 0, 0, None) == mt.MT_ERR_SHAPE   # K % 64
    assert L.mt_op_attention(mt.MT_BF16, fake, fake, fake, 1, 16, 96, 2, None) == mt.MT_ERR_SHAPE                   # head width 48
    assert L.mt_op_layernorm(None, fake, fake, 1e-12, fake, None, 4, 64, None) == mt.MT_ERR_NULL


def test_pack_blob_layout():
    flat = np.arange(5, dtype=np.float32)
    blob = mt.pack_blob(3, 7, flat)
    assert blob[:4] == b"MTW1" and len(blob) == 16 + 20
    assert np.frombuffer(blob[4:16], dtype="<i4").tolist() == [3, 7, 0]
    assert np.frombuffer(blob[16:], dtype="<f4").tolist() == [0, 1, 2, 3, 4]


def test_random_task_tables_host_bookkeeping():
    """Random task tables (forks, depths, class counts, head kinds): the library's layer count equals the oracle's
    overhead formula (Section 4.1), the wavefront step count is max over tasks of fork + own layers, logit offsets
    follow the order of the tasks inside each kind of row, and a checkpoint blob of the canonical size is what the
    loader asks for (checked through its size error, no device needed)."""
    import oracle
    rng = np.random.default_rng(2107)
    L = mt.lib()
    for _ in range(40):
        depth = int(rng.integers(0, 7))
        n_tasks = int(rng.integers(1, 9))
        tasks = [ms.TaskSpec(int(rng.integers(0, depth + 1)), int(rng.integers(0, 4)), int(rng.integers(1, 9)),
                             token_level=bool(rng.integers(0, 2))) for _ in range(n_tasks)]
        k = int(rng.integers(0, n_tasks))
        tasks[k] = ms.TaskSpec(depth, tasks[k].n_layers, tasks[k].n_classes, token_level=tasks[k].token_level)
        spec = ms.MTSpec("rnd", vocab=64, hidden=64, heads=2, ffn=128, max_pos=16, n_trunk_layers=depth, tasks=tuple(tasks),
                         precision="fp32", batch=2, seq=8, len_lo=1, len_hi=8)
        rc, h, _ = _create(spec)
        assert rc == mt.MT_OK, tasks
        assert L.mt_layer_count(h) == oracle.overhead([(t.fork_layer, t.n_layers) for t in tasks])
        assert L.mt_schedule_steps(h, None) == max(t.fork_layer + t.n_layers for t in tasks)
        mask = (C.c_uint8 * n_tasks)(*[int(rng.integers(0, 2)) for _ in range(n_tasks)])
        on = [t for t, m in zip(tasks, mask) if m]
        assert L.mt_schedule_steps(h, mask) == (max(t.fork_layer + t.n_layers for t in on) if on else 0)
        assert L.mt_n_logits(h) == spec.n_logits and L.mt_n_token_logits(h) == spec.n_token_logits
        for t, task in enumerate(tasks):
            good, bad = (L.mt_token_logit_offset, L.mt_logit_offset) if task.token_level else (L.mt_logit_offset, L.mt_token_logit_offset)
            assert good(h, t) == spec.logit_offset(t) and bad(h, t) == mt.MT_ERR_CONFIG
        # blob sizes: one float too many is refused, and the message names the canonical size
        fake = C.c_void_p(0x10000)
        assert L.mt_bind(h, fake, 1 << 40, fake, 1 << 40) == mt.MT_OK
        t = int(rng.integers(0, n_tasks))
        flat, idx = ms.make_task_params(spec, t)
        blob = mt.pack_blob(t, len(idx), np.concatenate([flat, np.zeros(1, np.float32)]))
        buf = C.create_string_buffer(blob, len(blob))
        assert L.mt_load_weights(h, t, C.cast(buf, C.c_void_p), len(blob), None) == mt.MT_ERR_BLOB
        assert str(16 + 4 * flat.size).encode() in L.mt_last_error(h)
        L.mt_destroy(h)


def test_fp8_weight_storage_rule_host_side():
    """The FP8 variant's weight conversion (host side of mt_load_weights) against two independent writings: torch's
    float8_e4m3fn cast of the scaled values, and the generator's snap-to-grid (which must be a fixed point of it)."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    w = (rng.standard_normal(50000) * 0.02).astype(np.float32)
    w[:8] = [0.0, -0.0, 1e-9, -3e-5, 0.09, -0.11, 2.0 ** -12, 0.0123]
    s, codes = mt.e4m3_quantize(w)
    assert s == ms.e4m3_scale(w) and s == 2.0 ** np.floor(np.log2(448.0 / np.abs(w).max()))
    assert s * np.abs(w).max() <= 448.0 < 2 * s * np.abs(w).max()
    ref = torch.from_numpy(w * np.float32(s)).to(torch.float8_e4m3fn)
    assert np.array_equal(codes & 0x7F, ref.view(torch.uint8).numpy() & 0x7F)          # magnitudes (the sign of a zero aside)
    nz = ref.float().numpy() != 0
    assert np.array_equal(codes[nz], ref.view(torch.uint8).numpy()[nz])
    # saturation, ties to even, the sub-normal range, on hand-picked values at unit scale
    # (the largest entry, 256, gives scale 1)
    s1, c1 = mt.e4m3_quantize(np.array([17.0, 19.0, 2.0 ** -6, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 0.0, 256.0], dtype=np.float32))
    got = torch.from_numpy(c1).view(torch.float8_e4m3fn).float().numpy()
    assert s1 == 1.0
    assert np.array_equal(got, np.array([16.0, 20.0, 2.0 ** -6, 2.0 ** -9, 0.0, 2.0 ** -8, 0.0, 256.0], dtype=np.float32))
    # values already on the grid come back unchanged, with the same scale: what lets the oracle use the same numbers
    # (here the largest entry, 0.11, rounds down onto 224 / 2048, which admits the scale 4096: the generator then snaps
    #  with 4096, and the result is a fixed point of the library's rule)
    g = ms.round_to_e4m3_grid(w.copy())
    s2, codes2 = mt.e4m3_quantize(g)
    assert s2 == ms.e4m3_scale(g) == 4096.0
    back = torch.from_numpy(codes2).view(torch.float8_e4m3fn).float().numpy() / np.float32(s2)
    assert np.array_equal(back, g)
    assert np.abs(g - w).max() <= 2.0 ** -4 * np.abs(w).max()
    for seed in range(20):                              # and for matrices like the generator's
        w2 = (np.random.default_rng(100 + seed).standard_normal(4096) * 0.02).astype(np.float32)
        g2 = ms.round_to_e4m3_grid(w2.copy())
        s3, c3 = mt.e4m3_quantize(g2)
        assert np.array_equal(torch.from_numpy(c3).view(torch.float8_e4m3fn).float().numpy() / np.float32(s3), g2)


def test_fp8_variant_configuration_rules():
    spec = dataclasses.replace(ms.get_config("base"), precision="fp8")
    rc, h, _ = _create(spec)
    assert rc == mt.MT_OK
    L = mt.lib()
    rc2, h2, _ = _create(ms.get_config("base"))
    # two E4M3 copies (F*H bytes each) per layer on top of the bf16 arena
    n_layers = spec.n_trunk_layers + sum(t.n_layers for t in spec.tasks)
    diff = L.mt_weight_bytes(h) - L.mt_weight_bytes(h2)
    assert 2 * n_layers * 768 * 3072 <= diff <= 2 * n_layers * (768 * 3072 + 256)
    L.mt_destroy(h)
    L.mt_destroy(h2)
    small = dataclasses.replace(spec, hidden=128, heads=2, ffn=256)          # K of the first contraction below the 3-slice ring
    assert _create(small)[0] == mt.MT_ERR_CONFIG


def test_fp8_layer_precision_generator_and_configuration():
    """MT_FP8_LAYER: the generator puts Wq, Wk, Wv of a layer on the E4M3 grid of ONE storage scale (that of the three
    together, as the library stores them in one matrix) and Wo, W1, W2 on their own; the library's rule applied to the
    stacked matrix reproduces the values exactly; the arena grows by the four E4M3 copies per layer."""
    torch = pytest.importorskip("torch")
    small = ms.MTSpec("fp8_all_host", vocab=100, hidden=256, heads=4, ffn=512, max_pos=32, n_trunk_layers=2,
                      tasks=(ms.TaskSpec(2, 1, 2),), precision="fp8_all", batch=2, seq=16, len_lo=4, len_hi=16)
    flat, index = ms.make_trunk_params(small)
    named = {n: flat[o:o + int(np.prod(sh))] for n, sh, o in index}
    for layer in range(small.n_trunk_layers):
        names = [n for n in named if n.endswith(".Wq") or n == "Wq"]
        pre = sorted({n.rsplit("Wq", 1)[0] for n in names})[layer]
        qkv = np.concatenate([named[pre + "Wq"], named[pre + "Wk"], named[pre + "Wv"]])
        s, codes = mt.e4m3_quantize(qkv)
        assert s == ms.e4m3_scale(qkv)
        assert np.array_equal(torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy() / np.float32(s), qkv)
        for one in ("Wo", "W1", "W2"):
            w = named[pre + one]
            s1, c1 = mt.e4m3_quantize(w)
            assert np.array_equal(torch.from_numpy(c1).view(torch.float8_e4m3fn).float().numpy() / np.float32(s1), w)
    # the bf16 and fp8 precisions draw the same numbers before snapping, and "fp8" leaves the attention matrices on the bf16 grid
    flat_b, _ = ms.make_trunk_params(dataclasses.replace(small, precision="bf16"))
    flat_f, _ = ms.make_trunk_params(dataclasses.replace(small, precision="fp8"))
    n0, sh0, o0 = next((n, sh, o) for n, sh, o in index if n.endswith("Wq"))
    sl = slice(o0, o0 + int(np.prod(sh0)))
    assert np.array_equal(flat_b[sl], flat_f[sl]) and not np.array_equal(flat_b[sl], flat[sl])
    assert np.abs(flat[sl] - flat_b[sl]).max() <= 2.0 ** -4 * np.abs(flat_b[sl]).max()
    # configuration: accepted, and the arena holds 3HH + HH + 2FH more bytes per layer than the bf16 one
    base = ms.get_config("base")
    L = mt.lib()
    rc, h, _ = _create(dataclasses.replace(base, precision="fp8_all"))
    rc2, h2, _ = _create(base)
    assert rc == mt.MT_OK and rc2 == mt.MT_OK
    n_layers = base.n_trunk_layers + sum(t.n_layers for t in base.tasks)
    per_layer = 4 * 768 * 768 + 2 * 768 * 3072
    diff = L.mt_weight_bytes(h) - L.mt_weight_bytes(h2)
    assert n_layers * per_layer <= diff <= n_layers * (per_layer + 4 * 256)
    L.mt_destroy(h)
    L.mt_destroy(h2)
