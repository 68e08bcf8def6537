"""The five synthetic LLaMA-shaped shard workloads.

Each names a model shape, the sharding factor and rank of the rank whose share of the
model states (Section IV-B: P, G and OS sharded over ``s`` GPUs; factor 1 = Full-Replica)
is processed, the number ``k`` of partial bf16 gradient buffers that stand in for the
peers of a reduce-scatter, and the seeded input distributions.  Only integers and
distribution parameters live here: no arithmetic of the step.
"""
from __future__ import annotations

import dataclasses

from . import synth


def llama_param_count(layers: int, hidden: int, ffn: int, vocab: int) -> int:
    """Phi of a LLaMA-style decoder: untied embedding and head, four attention
    matrices, three MLP matrices and two norm gains per layer, one final norm gain."""
    per_layer = 4 * hidden * hidden + 3 * hidden * ffn + 2 * hidden
    return 2 * vocab * hidden + layers * per_layer + hidden


def llama_tensor_sizes(layers: int, hidden: int, ffn: int, vocab: int):
    """Element counts of the model's tensors in flat (model) order: embedding; per layer the
    attention norm gain, four attention matrices, the MLP norm gain and three MLP matrices; the
    final norm gain; the output head.  Their sum is llama_param_count."""
    sizes = [vocab * hidden]
    for _ in range(layers):
        sizes += [hidden, hidden * hidden, hidden * hidden, hidden * hidden, hidden * hidden,
                  hidden, hidden * ffn, hidden * ffn, ffn * hidden]
    sizes += [hidden, vocab * hidden]
    return sizes


@dataclasses.dataclass(frozen=True)
class Workload:
    config_id: int
    name: str
    layers: int
    hidden: int
    ffn: int
    vocab: int
    shard_factor: int
    rank: int
    k: int
    sigma_grad: float
    step: int
    bucket_elems: int = 0      # 0 = the whole shard in one launch
    drop_tail: int = 0         # elements cut from the end of the shard (ragged length)
    inter_tensor: bool = False  # shard = whole tensors chosen greedily (Section IV-C.2), not a flat range
    sigma_param: float = 0.02
    sigma_m: float = 1e-4
    scale_v: float = 1e-6
    lr: float = 3e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    max_norm: float = 1.0
    clip_eps: float = 1e-6

    @property
    def seed(self) -> int:
        return 20231100 + self.config_id

    @property
    def total_elems(self) -> int:
        return llama_param_count(self.layers, self.hidden, self.ffn, self.vocab)

    @property
    def tensor_sizes(self):
        return llama_tensor_sizes(self.layers, self.hidden, self.ffn, self.vocab)

    def key(self, tensor_id: int) -> int:
        return synth.stream_key(self.seed, tensor_id)

    def bytes_per_elem_fused(self) -> int:
        """Algorithmic HBM bytes per element of the fused pass: 2k read for the bf16
        partials, 12 read + 12 written for fp32 master/m/v (the 12-byte OS of Section
        II-C), 2 written for the bf16 parameter."""
        return 2 * self.k + 26

    def bytes_per_elem_norm(self) -> int:
        return 2 * self.k


WORKLOADS = (
    Workload(0, "tiny-llama/s1/k2", 2, 256, 688, 1000, 1, 0, 2, 1e-3, 10),
    Workload(1, "llama-7b/s8r3/k8", 32, 4096, 11008, 32000, 8, 3, 8, 1e-3, 10),
    Workload(2, "llama-7b/full-replica/k1", 32, 4096, 11008, 32000, 1, 0, 1, 1e-3, 1000),
    Workload(3, "llama-13b/s16r7/k16", 40, 5120, 13824, 32000, 16, 7, 16, 1e-2, 10),
    Workload(4, "llama-30b/s8r5/k8/bucketed", 60, 6656, 17920, 32000, 8, 5, 8, 1e-3, 10,
             bucket_elems=25_000_001, drop_tail=3),
    # beyond the five listed workloads: the inter-tensor scheme the paper adopts.  One all-reduced flat
    # bf16 gradient buffer of the whole model (k = 1), the rank's whole tensors selected from it.
    Workload(5, "llama-7b/inter-tensor/s8r3/k1", 32, 4096, 11008, 32000, 8, 3, 1, 1e-3, 10, inter_tensor=True),
)


def get(config_id: int) -> Workload:
    return WORKLOADS[config_id]
