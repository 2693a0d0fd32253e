"""Seeded synthetic workloads for the mixed-precision stacked-LSTM training step.

This module only names the benchmark configurations and draws their random
inputs (weights, input sequences, token ids, targets).  It holds none of the
method's arithmetic: no LSTM, no loss, no optimiser.  Both the CPU oracle's
tests and the HIP path's tests/bench draw their inputs from here so that the
two sides see bit-identical, already-rounded numbers.

The five configurations stand in for the paper's workloads (Section "Neural
Network architecture", Fig. 2; Appendix "Datasets"): the JET multimodal time
series and the Large Movie Review text set are not available, so inputs of the
same shape and value distribution are synthesised.  No item of either data set
is reproduced.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Tuple

import numpy as np

# head kinds (shared vocabulary with the C ABI and, independently, the oracle)
HEAD_STEP_BCE = 1   # per-timestep sigmoid + binary cross-entropy
HEAD_LAST_BCE = 2   # last-timestep sigmoid + binary cross-entropy
HEAD_STEP_MSE = 3   # per-timestep linear + mean squared error
HEAD_FC_HINGE = 4   # the paper's head: fully connected ReLU layer per time slice, one output, hinge loss, labels +-1

DTYPE_CODE = {"fp32": 0, "fp16": 1, "bf16": 2}


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    num_layers: int
    input_dim: int          # feature dim of x (ignored when vocab > 0)
    hidden: int
    seq_len: int
    batch: int
    dtype: str              # "fp32" | "fp16" | "bf16"
    head: int
    vocab: int = 0
    embed_dim: int = 0
    n_workers: int = 1
    loss_scale: float = 1.0
    dynamic_scale: bool = False
    momentum: float = 0.9
    lr0: float = 1e-3
    # worker-count schedule (Section "Learning rate schedule")
    n_half: float = 1e12            # single-worker configs: Eq. 4 leaves lr0 unchanged
    warmup_steps: int = 0
    gamma: float = 1.0
    fc_units: int = 0               # units of the fully connected head layer (HEAD_FC_HINGE)
    target_kind: str = "bernoulli"   # "bernoulli" | "normal" | "sign" (+1 with probability target_p, else -1)
    target_p: float = 0.1
    data_seed: int = 0
    weight_seed: int = 7

    @property
    def layer_input_dims(self) -> List[int]:
        first = self.embed_dim if self.vocab > 0 else self.input_dim
        return [first] + [self.hidden] * (self.num_layers - 1)

    def with_(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, Workload] = {
    # config 1: one forward + BPTT + plain SGD step, all fp32
    "tiny": Workload("tiny", 1, 14, 32, 16, 4, "fp32", HEAD_STEP_BCE,
                     loss_scale=1.0, momentum=0.0, lr0=1e-3, data_seed=0, weight_seed=8),
    # config 2: stand-in for the JET multimodal time-series model (2 x 200 units)
    "jet": Workload("jet", 2, 64, 200, 128, 128, "fp16", HEAD_STEP_BCE,
                    loss_scale=1024.0, data_seed=2, weight_seed=9),
    # config 3: stand-in for the movie-review text classifier
    "text": Workload("text", 1, 0, 256, 400, 128, "fp16", HEAD_LAST_BCE,
                     vocab=20000, embed_dim=128, loss_scale=1024.0,
                     target_p=0.5, data_seed=3, weight_seed=10),
    # config 4: ~88 M parameter model, dynamic loss scaling from 2^15
    "large": Workload("large", 3, 512, 2048, 128, 256, "fp16", HEAD_STEP_MSE,
                      loss_scale=32768.0, dynamic_scale=True, target_kind="normal",
                      data_seed=4, weight_seed=11),
    # config 5: 64 simulated workers on the config-2 model
    "workers64": Workload("workers64", 2, 64, 200, 128, 128, "fp16", HEAD_STEP_BCE,
                          n_workers=64, loss_scale=32768.0, dynamic_scale=True,
                          n_half=64.0, warmup_steps=5, gamma=0.97,
                          data_seed=1000, weight_seed=12),
}


# Not one of the five benchmark configurations: the paper's own network (Fig. 2: 9 signals, two LSTM
# layers of 200 units, a fully connected ReLU layer of 200 units on every temporal slice, one output,
# hinge loss) at its batch size 256, sequence length 128 and static loss multiplier 10, on synthetic
# signals.  `bench.py --workload fig2` reports it.
EXTRA: Dict[str, Workload] = {
    "fig2": Workload("fig2", 2, 9, 200, 128, 256, "fp16", HEAD_FC_HINGE, fc_units=200, target_kind="sign",
                     target_p=0.1, loss_scale=10.0, data_seed=43, weight_seed=44),
}


def param_segments(w: Workload) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of the parameter tensors in flat-buffer order.

    Order: [embedding] {W_l[4H,I_l], U_l[4H,H], b_l[4H]} for each layer,
    then head weight [H] and head bias [1] (with a fully connected head layer:
    W_fc[F,H], b_fc[F], head weight [F], head bias [1]).  Pure bookkeeping.
    """
    segs: List[Tuple[str, Tuple[int, ...]]] = []
    if w.vocab > 0:
        segs.append(("E", (w.vocab, w.embed_dim)))
    G = 4 * w.hidden
    for l, i_l in enumerate(w.layer_input_dims):
        segs.append((f"W{l}", (G, i_l)))
        segs.append((f"U{l}", (G, w.hidden)))
        segs.append((f"b{l}", (G,)))
    if w.fc_units > 0:
        segs.append(("W_fc", (w.fc_units, w.hidden)))
        segs.append(("b_fc", (w.fc_units,)))
        segs.append(("w_head", (w.fc_units,)))
    else:
        segs.append(("w_head", (w.hidden,)))
    segs.append(("b_head", (1,)))
    return segs


def param_count(w: Workload) -> int:
    return int(sum(int(np.prod(s)) for _, s in param_segments(w)))


def make_params(w: Workload, seed: Optional[int] = None) -> np.ndarray:
    """Flat fp32 initial parameters: U(-1/sqrt(H), 1/sqrt(H)) for the LSTM and
    head tensors, 0.1*N(0,1) for the embedding table."""
    rng = np.random.default_rng(w.weight_seed if seed is None else seed)
    bound = 1.0 / np.sqrt(float(w.hidden))
    parts = []
    for name, shape in param_segments(w):
        n = int(np.prod(shape))
        if name == "E":
            parts.append((0.1 * rng.standard_normal(n)).astype(np.float32))
        else:
            parts.append(rng.uniform(-bound, bound, n).astype(np.float32))
    return np.concatenate(parts)


def _bounded_zipf(rng: np.random.Generator, n: int, vocab: int, s: float) -> np.ndarray:
    ranks = np.arange(1, vocab + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-s))
    cdf /= cdf[-1]
    u = rng.random(n)
    return np.minimum(np.searchsorted(cdf, u, side="left"), vocab - 1).astype(np.int32)


def make_batch(w: Workload, worker: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """(x, targets) for one worker's micro-batch.

    x is fp32 [T,B,I] drawn N(0,1), or int32 token ids [T,B] from a bounded
    Zipf(s=1.1) law when the workload has an embedding front-end.  targets is
    fp32 [T,B,1] (per-step heads) or [B,1] (last-step head).
    """
    rng = np.random.default_rng(w.data_seed + worker)
    T, B = w.seq_len, w.batch
    if w.vocab > 0:
        x = _bounded_zipf(rng, T * B, w.vocab, 1.1).reshape(T, B)
    else:
        x = rng.standard_normal((T, B, w.input_dim)).astype(np.float32)
    tshape = (B, 1) if w.head == HEAD_LAST_BCE else (T, B, 1)
    if w.target_kind == "normal":
        y = rng.standard_normal(tshape).astype(np.float32)
    elif w.target_kind == "sign":
        y = np.where(rng.random(tshape) < w.target_p, 1.0, -1.0).astype(np.float32)
    else:
        y = (rng.random(tshape) < w.target_p).astype(np.float32)
    return x, y


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32 array once to the storage type and return it as fp32
    (exactly representable), so both sides start from identical numbers."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "fp16":
        t = t.to(torch.float16).to(torch.float32)
    elif dtype == "bf16":
        t = t.to(torch.bfloat16).to(torch.float32)
    elif dtype != "fp32":
        raise ValueError(dtype)
    return t.numpy()
