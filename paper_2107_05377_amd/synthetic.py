"""Fill a Model with the seeded synthetic checkpoints of mt_synth (one blob per scope)."""
from __future__ import annotations

from .binding import Model, make_config


def load_synthetic(spec, *, max_batch=None, max_seq=None, precision=None, stress=False, std=0.02,
                   device="cuda:0", keep_params=False):
    """Create + bind a Model for `spec` and load trunk and task checkpoints drawn by mt_synth.

    Returns (model, params) where params is (trunk_flat, [task_flat...]) if keep_params else None.
    """
    import mt_synth as ms
    model = Model(make_config(spec, max_batch=max_batch, max_seq=max_seq, precision=precision), device=device)
    trunk, tri = ms.make_trunk_params(spec, stress=stress, std=std)
    model.load_params(-1, trunk, len(tri))
    tasks = []
    for t in range(spec.n_tasks):
        tp, tpi = ms.make_task_params(spec, t, stress=stress, std=std)
        model.load_params(t, tp, len(tpi))
        tasks.append(tp if keep_params else None)
    return model, ((trunk, tasks) if keep_params else None)
