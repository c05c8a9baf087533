"""Shape descriptions of merged multi-task models and the canonical parameter order.

A merged model (paper Section 3.3, Fig. 1(c)) is a linear trunk of shared frozen encoder layers
plus one branch per task.  Task t reads the trunk after `fork_layer` layers (the x of the paper's
(x, y) tuples under Table 2) and owns `n_layers` task-specific layers (the y), a pooler and a
linear head with `n_classes` outputs.

Parameter order (every linear is W[out][in] row-major, y = W x + b):
  trunk scope : word_emb[V,H] pos_emb[P,H] type_emb[2,H] emb_ln_g[H] emb_ln_b[H], then per layer
                Wq[H,H] bq[H] Wk bk Wv bv Wo[H,H] bo ln1_g ln1_b W1[F,H] b1[F] W2[H,F] b2[H] ln2_g ln2_b
  task scope  : n_layers layers in the same order, then Wp[H,H] bp[H] Wc[C,H] bc[C]
                (a token-level task has no pooler: its layers are followed by Wc[C,H] bc[C] only)
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple


@dataclass(frozen=True)
class TaskSpec:
    fork_layer: int   # x_t: number of shared frozen layers this task reads through
    n_layers: int     # y_t: task-specific layers
    n_classes: int    # C_t (1 = regression)
    token_level: bool = False   # True: one label per token (tagging, slot filling), a linear head on every position


@dataclass(frozen=True)
class MTSpec:
    name: str
    vocab: int
    hidden: int
    heads: int
    ffn: int
    max_pos: int
    n_trunk_layers: int
    tasks: Tuple[TaskSpec, ...]
    precision: str            # "bf16" or "fp32"
    batch: int
    seq: int
    len_lo: int
    len_hi: int
    type_vocab: int = 2
    ln_eps: float = 1e-12
    gelu: str = "erf"
    input_seed: int = 1000
    weights_seed: int = 20210705

    @property
    def n_tasks(self) -> int:
        return len(self.tasks)

    @property
    def n_logits(self) -> int:
        """Width of the per-sequence logit row: the sequence-level tasks' classes side by side."""
        return sum(t.n_classes for t in self.tasks if not t.token_level)

    @property
    def n_token_logits(self) -> int:
        """Width of the per-token logit row: the token-level tasks' classes side by side."""
        return sum(t.n_classes for t in self.tasks if t.token_level)

    def logit_offset(self, t: int) -> int:
        """First column of task t inside the row of its own kind (per-sequence or per-token)."""
        kind = self.tasks[t].token_level
        return sum(u.n_classes for u in self.tasks[:t] if u.token_level == kind)


def layer_tensors(h: int, f: int) -> List[Tuple[str, Tuple[int, ...]]]:
    return [("Wq", (h, h)), ("bq", (h,)), ("Wk", (h, h)), ("bk", (h,)), ("Wv", (h, h)), ("bv", (h,)),
            ("Wo", (h, h)), ("bo", (h,)), ("ln1_g", (h,)), ("ln1_b", (h,)),
            ("W1", (f, h)), ("b1", (f,)), ("W2", (h, f)), ("b2", (h,)), ("ln2_g", (h,)), ("ln2_b", (h,))]


def trunk_tensors(spec: MTSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    h = spec.hidden
    out = [("word_emb", (spec.vocab, h)), ("pos_emb", (spec.max_pos, h)), ("type_emb", (spec.type_vocab, h)),
           ("emb_ln_g", (h,)), ("emb_ln_b", (h,))]
    for l in range(spec.n_trunk_layers):
        out += [(f"L{l}.{n}", s) for n, s in layer_tensors(h, spec.ffn)]
    return out


def task_tensors(spec: MTSpec, t: int) -> List[Tuple[str, Tuple[int, ...]]]:
    h = spec.hidden
    task = spec.tasks[t]
    out = []
    for l in range(task.n_layers):
        out += [(f"L{l}.{n}", s) for n, s in layer_tensors(h, spec.ffn)]
    if not task.token_level:
        out += [("Wp", (h, h)), ("bp", (h,))]
    out += [("Wc", (task.n_classes, h)), ("bc", (task.n_classes,))]
    return out


_GLUE_CLASSES = (2, 2, 2, 3, 2, 2, 2, 1)   # QNLI RTE QQP MNLI SST-2 MRPC CoLA STS-B (Table 1 column order)


def _uniform_tasks(x: int, y: int, classes=_GLUE_CLASSES) -> Tuple[TaskSpec, ...]:
    return tuple(TaskSpec(x, y, c) for c in classes)


def _hetero_tasks() -> Tuple[TaskSpec, ...]:
    ks = (1, 2, 3, 4, 5, 6, 6, 4)     # fine-tuned depth k of the teacher; student keeps 12-k frozen, ceil(k/2) distilled
    return tuple(TaskSpec(12 - k, (k + 1) // 2, c) for k, c in zip(ks, _GLUE_CLASSES))


def _industrial_tasks() -> Tuple[TaskSpec, ...]:
    # Appendix E: 21 tasks on 8 shared layers, 32 task layers in all (1.5 per task on average): 11 tasks keep two
    # distilled layers, 10 keep one.  Class counts are stand-ins for intent / domain / emotion style label sets.
    classes = (2, 3, 5, 8, 12, 2, 4, 30, 2, 6, 3, 2, 16, 4, 2, 9, 3, 2, 50, 7, 2)
    return tuple(TaskSpec(8, 2 if t % 2 == 0 else 1, c) for t, c in enumerate(classes))


def _assistant_tasks() -> Tuple[TaskSpec, ...]:
    # Appendix E names tagging-style tasks (named entities, slot filling) next to the classifiers: the same
    # 21-task table with three of the tasks labelling every token instead of the sequence.
    token = {7: 30, 12: 16, 15: 9}       # slot labels, entity labels (BIO over 4 types), a small tag set
    return tuple(TaskSpec(t.fork_layer, t.n_layers, t.n_classes, token_level=(i in token))
                 for i, t in enumerate(_industrial_tasks()))


def _table_tasks(tuples) -> Tuple[TaskSpec, ...]:
    return tuple(TaskSpec(x, y, c) for (x, y), c in zip(tuples, _GLUE_CLASSES))


# Table 2's task tables (fork x, own layers y) in the order QNLI RTE QQP MNLI SST-2 MRPC CoLA STS-B
_WO_KD = ((2, 10), (7, 5), (2, 10), (4, 8), (6, 6), (7, 5), (4, 8), (4, 8))        # "Ours (w/o KD)": 7 + 60 layers
_MIXED = ((2, 3), (7, 5), (2, 1), (4, 3), (6, 2), (7, 3), (4, 8), (4, 1))          # "Ours (mixed)":  7 + 26 layers


CONFIGS = {
    "tiny": MTSpec("tiny", vocab=1000, hidden=64, heads=2, ffn=256, max_pos=32, n_trunk_layers=2,
                   tasks=(TaskSpec(2, 1, 2), TaskSpec(2, 1, 3)), precision="fp32",
                   batch=2, seq=16, len_lo=4, len_hi=16, input_seed=1000),
    "base": MTSpec("base", vocab=30522, hidden=768, heads=12, ffn=3072, max_pos=512, n_trunk_layers=8,
                   tasks=_uniform_tasks(8, 2), precision="bf16",
                   batch=32, seq=128, len_lo=16, len_hi=128, input_seed=1001),
    "hetero": MTSpec("hetero", vocab=30522, hidden=768, heads=12, ffn=3072, max_pos=512, n_trunk_layers=11,
                     tasks=_hetero_tasks(), precision="bf16",
                     batch=64, seq=128, len_lo=16, len_hi=128, input_seed=1002),
    "latency": MTSpec("latency", vocab=30522, hidden=768, heads=12, ffn=3072, max_pos=512, n_trunk_layers=6,
                      tasks=_uniform_tasks(6, 2), precision="bf16",
                      batch=8, seq=64, len_lo=8, len_hi=64, input_seed=1003),
    "large": MTSpec("large", vocab=30522, hidden=1024, heads=16, ffn=4096, max_pos=512, n_trunk_layers=18,
                    tasks=_uniform_tasks(18, 2), precision="bf16",
                    batch=128, seq=256, len_lo=64, len_hi=256, input_seed=1004),
    # second workload (Appendix E): many small tasks over short utterances
    "industrial": MTSpec("industrial", vocab=21128, hidden=768, heads=12, ffn=3072, max_pos=512, n_trunk_layers=8,
                         tasks=_industrial_tasks(), precision="bf16",
                         batch=16, seq=32, len_lo=4, len_hi=32, input_seed=1005),
    "assistant": MTSpec("assistant", vocab=21128, hidden=768, heads=12, ffn=3072, max_pos=512, n_trunk_layers=8,
                        tasks=_assistant_tasks(), precision="bf16",
                        batch=16, seq=32, len_lo=4, len_hi=32, input_seed=1008),
    # stress shapes for the schedule: the paper's undistilled and mixed task tables (Table 2), deep uneven branches
    "wo_kd": MTSpec("wo_kd", vocab=30522, hidden=768, heads=12, ffn=3072, max_pos=512, n_trunk_layers=7,
                    tasks=_table_tasks(_WO_KD), precision="bf16",
                    batch=32, seq=128, len_lo=16, len_hi=128, input_seed=1006),
    "mixed": MTSpec("mixed", vocab=30522, hidden=768, heads=12, ffn=3072, max_pos=512, n_trunk_layers=7,
                    tasks=_table_tasks(_MIXED), precision="bf16",
                    batch=32, seq=128, len_lo=16, len_hi=128, input_seed=1007),
}
_ORDER = ["tiny", "base", "hetero", "latency", "large", "industrial", "wo_kd", "mixed", "assistant"]


def get_config(key) -> MTSpec:
    """Look a workload up by name or by index 0..8 (tiny, base, hetero, latency, large, industrial, wo_kd, mixed, assistant)."""
    if isinstance(key, int):
        key = _ORDER[key]
    return CONFIGS[key]
