"""Counter-based seeded generators for weights and inputs.

splitmix64 (Steele, Lea, Flood 2014; the public-domain finaliser used to seed xoshiro) is applied
to `key + (counter+1)*golden`, so element i of a tensor depends only on (key, i).  Uniforms take the
top 53 bits; normals are Box-Muller pairs (cosine, sine) on the counter pair (2j, 2j+1).

Weight recipe: every matrix and embedding table ~ N(0, std 0.02); biases 0, LayerNorm gamma 1 and
beta 0.  `stress=True` instead draws biases and beta ~ N(0, 0.02) and gamma ~ 1 + N(0, 0.02) so that
bias/gamma/beta code paths carry signal.  `bf16_grid=True` snaps matrices and embedding tables to
values representable in bfloat16 (round to nearest even), so a consumer that stores them as
bfloat16 and one that keeps float32 see identical numbers.  A spec of precision "fp8" additionally snaps the
two feed-forward matrices of every layer to the FP8 E4M3 grid under their power-of-two storage scale; precision
"fp8_all" snaps the attention output matrix Wo likewise, and Wq, Wk, Wv of a layer under ONE scale taken over the three
(a consumer may store them as one [3H, H] matrix).

Input recipe: sequence lengths uniform on the inclusive range [len_lo, len_hi]; the attention mask
is a prefix of ones; token ids are uniform in [0, vocab) at every position, padded ones included.
"""
from __future__ import annotations

import numpy as np

from .spec import MTSpec, trunk_tensors, task_tensors

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def splitmix64(key: int, counters: np.ndarray) -> np.ndarray:
    """Output of splitmix64 for state `key + (counter+1)*golden`, vectorised over uint64 counters."""
    with np.errstate(over="ignore"):
        z = np.uint64(key & 0xFFFFFFFFFFFFFFFF) + (counters.astype(np.uint64) + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _subkey(seed: int, *ids: int) -> int:
    k = seed & 0xFFFFFFFFFFFFFFFF
    for i in ids:
        k = int(splitmix64(k, np.array([i & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))[0])
    return k


def uniform01(key: int, start: int, n: int) -> np.ndarray:
    """n doubles in [0,1) for counters start..start+n-1."""
    c = np.arange(start, start + n, dtype=np.uint64)
    return (splitmix64(key, c) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal(key: int, n: int, out: np.ndarray | None = None) -> np.ndarray:
    """n standard normals (float32); elements 2j and 2j+1 are the cosine and sine Box-Muller
    outputs of the uniforms drawn at counters 2j and 2j+1."""
    res = np.empty(n, dtype=np.float32) if out is None else out
    for lo in range(0, n, _CHUNK):            # _CHUNK is even, so pairs never straddle chunks
        m = min(_CHUNK, n - lo)
        mp = (m + 1) // 2
        c = np.arange(lo, lo + 2 * mp, dtype=np.uint64)
        r = splitmix64(key, c) >> np.uint64(11)
        u1 = (r[0::2].astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)   # (0,1]
        u2 = r[1::2].astype(np.float64) * (1.0 / 9007199254740992.0)           # [0,1)
        rad = np.sqrt(-2.0 * np.log(u1))
        ang = 2.0 * np.pi * u2
        pair = np.empty(2 * mp, dtype=np.float32)
        pair[0::2] = rad * np.cos(ang)
        pair[1::2] = rad * np.sin(ang)
        res[lo:lo + m] = pair[:m]
    return res


def round_to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Snap float32 values to the nearest bfloat16-representable value (ties to even), in place."""
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += np.uint32(0x7FFF) + lsb
    u &= np.uint32(0xFFFF0000)
    return x


def e4m3_scale(x: np.ndarray) -> float:
    """Storage scale of an FP8 (OCP E4M3, largest finite value 448) matrix: the largest power of two s with
    s * max|x| <= 448; 1 for an all-zero matrix."""
    mx = float(np.abs(x).max()) if x.size else 0.0
    if not (mx > 0.0) or not np.isfinite(mx):
        return 1.0
    s = 2.0 ** np.floor(np.log2(448.0 / mx))
    while s * mx > 448.0:
        s *= 0.5
    while 2.0 * s * mx <= 448.0:
        s *= 2.0
    return float(s)


def _snap_e4m3(x: np.ndarray, s: float) -> np.ndarray:
    """The values an OCP FP8 E4M3 store of s * x holds, divided by s again (a new array)."""
    s = np.float32(s)
    y = (x * s).astype(np.float32)
    a = np.abs(y)
    small = a < np.float32(2.0 ** -6)
    u = a.view(np.uint32).copy()
    u += np.uint32(0x7FFFF) + ((u >> np.uint32(20)) & np.uint32(1))
    u &= np.uint32(0xFFF00000)
    big = np.minimum(u.view(np.float32), np.float32(448.0))
    sub = (np.rint(a.astype(np.float64) * 512.0) / 512.0).astype(np.float32)
    q = np.where(small, sub, big).astype(np.float32)
    return (np.copysign(q, y) / s).astype(np.float32)


def round_to_e4m3_grid(x: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Snap float32 values, in place, to the values an OCP FP8 E4M3 store of scale * x holds (3 mantissa bits, round to
    nearest even; multiples of 2^-9 below 2^-6; saturating at 448), divided by the scale again.
    scale None: the storage scale e4m3_scale, chosen so that the RESULT has that same storage scale (a largest entry that
    rounds down onto 224 / scale would otherwise admit twice the scale: then the snap is redone with the doubled one)."""
    if scale is not None:
        x[...] = _snap_e4m3(x, scale)
        return x
    s = e4m3_scale(x)
    for _ in range(4):
        y = _snap_e4m3(x, s)
        s2 = e4m3_scale(y)
        if s2 == s:
            break
        s = s2
    assert e4m3_scale(y) == s
    x[...] = y
    return x


def round_group_to_e4m3_grid(views) -> float:
    """Snap several float32 arrays, in place, to the E4M3 grid under ONE storage scale: that of their union, chosen so
    that the snapped union has the same storage scale again (see round_to_e4m3_grid).  Returns the scale."""
    def joint(arrs):
        return min(e4m3_scale(a) for a in arrs)      # the union's largest entry decides
    s = joint(views)
    snapped = [_snap_e4m3(v, s) for v in views]
    for _ in range(4):
        s2 = joint(snapped)
        if s2 == s:
            break
        s = s2
        snapped = [_snap_e4m3(v, s) for v in views]
    assert joint(snapped) == s
    for v, y in zip(views, snapped):
        v[...] = y
    return s


def _fp8_flags(precision: str):
    """(feed-forward matrices on the E4M3 grid, attention matrices on the E4M3 grid) for a spec's precision."""
    return precision in ("fp8", "fp8_all"), precision == "fp8_all"


def _fill(flat: np.ndarray, tensors, seed: int, scope_id: int, std: float, stress: bool, bf16_grid: bool, fp8_ffn: bool = False,
          fp8_attn: bool = False):
    off = 0
    index = []
    held = {}                                     # Wq, Wk of the layer being filled, until its Wv arrives
    for ti, (name, shape) in enumerate(tensors):
        n = int(np.prod(shape))
        view = flat[off:off + n]
        base = name.split(".")[-1]
        key = _subkey(seed, scope_id, ti)
        if len(shape) == 2:                       # matrices and embedding tables
            normal(key, n, out=view)
            view *= np.float32(std)
            if (fp8_ffn and base in ("W1", "W2")) or (fp8_attn and base == "Wo"):
                round_to_e4m3_grid(view)          # E4M3 values (times a power of two) are bfloat16 values too
            elif fp8_attn and base in ("Wq", "Wk"):
                held[base] = view
            elif fp8_attn and base == "Wv":
                round_group_to_e4m3_grid([held.pop("Wq"), held.pop("Wk"), view])
            elif bf16_grid:
                round_to_bf16_grid(view)
        elif base.endswith("_g"):                 # LayerNorm gamma
            view[:] = 1.0
            if stress:
                view += normal(key, n) * np.float32(std)
        else:                                     # biases and LayerNorm beta
            view[:] = 0.0
            if stress:
                view += normal(key, n) * np.float32(std)
        index.append((name, tuple(shape), off))
        off += n
    assert off == flat.size
    return index


def _count(tensors) -> int:
    return int(sum(int(np.prod(s)) for _, s in tensors))


def make_trunk_params(spec: MTSpec, *, stress: bool = False, bf16_grid: bool | None = None,
                      seed: int | None = None, std: float = 0.02):
    """Flat float32 parameter vector of the trunk scope (canonical order) and its (name, shape, offset) index."""
    bf16_grid = (spec.precision in ("bf16", "fp8", "fp8_all")) if bf16_grid is None else bf16_grid
    tensors = trunk_tensors(spec)
    flat = np.empty(_count(tensors), dtype=np.float32)
    index = _fill(flat, tensors, spec.weights_seed if seed is None else seed, 0, std, stress, bf16_grid, *_fp8_flags(spec.precision))
    return flat, index


def make_task_params(spec: MTSpec, t: int, *, stress: bool = False, bf16_grid: bool | None = None,
                     seed: int | None = None, std: float = 0.02):
    """Flat float32 parameter vector of task t's scope (canonical order) and its index."""
    bf16_grid = (spec.precision in ("bf16", "fp8", "fp8_all")) if bf16_grid is None else bf16_grid
    tensors = task_tensors(spec, t)
    flat = np.empty(_count(tensors), dtype=np.float32)
    index = _fill(flat, tensors, spec.weights_seed if seed is None else seed, 1 + t, std, stress, bf16_grid, *_fp8_flags(spec.precision))
    return flat, index


def make_inputs(spec: MTSpec, *, batch: int | None = None, seq: int | None = None, batch_index: int = 0,
                len_lo: int | None = None, len_hi: int | None = None, seed: int | None = None):
    """(input_ids[B,S] int32, attn_mask[B,S] int32, lengths[B] int32) for one synthetic batch."""
    b = spec.batch if batch is None else batch
    s = spec.seq if seq is None else seq
    lo = spec.len_lo if len_lo is None else len_lo
    hi = spec.len_hi if len_hi is None else len_hi
    hi = min(hi, s)
    lo = min(lo, hi)
    sd = spec.input_seed if seed is None else seed
    k_len = _subkey(sd, 1, batch_index)
    k_ids = _subkey(sd, 2, batch_index)
    lengths = (lo + np.floor(uniform01(k_len, 0, b) * (hi - lo + 1))).astype(np.int32)
    lengths = np.minimum(lengths, hi).astype(np.int32)
    ids = np.floor(uniform01(k_ids, 0, b * s) * spec.vocab).astype(np.int32).reshape(b, s)
    ids = np.minimum(ids, spec.vocab - 1).astype(np.int32)
    mask = (np.arange(s, dtype=np.int32)[None, :] < lengths[:, None]).astype(np.int32)
    return ids, mask, lengths
