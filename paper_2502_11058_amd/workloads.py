"""Synthetic workloads: tensor shapes of the benchmark configurations and seeded input generators.

This module is harness only.  It describes *what the inputs look like* (tensor list per layer, replica count
N, period H, optimizer hyper-parameters, value distributions, per-layer profiled times) and produces seeded
random inputs.  It contains none of the method's arithmetic: no packing, averaging, optimizer or scheduling
code lives here, so both the HIP path and the CPU oracle can be fed from it without sharing implementation.

Layer convention (Sec. 3.3 of the paper orders layers 1..L from input to output and runs BP from L down to 1):
layer ids are 0-based here, 0 = input side.  A schedulable layer is one transformer block (all its tensors);
token embedding, position embedding and final-norm + LM head are layers of their own.
"""
from __future__ import annotations

import hashlib
import json
import os
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class TensorSpec:
    name: str
    layer: int
    numel: int


@dataclass
class Workload:
    name: str
    tensors: List[TensorSpec]
    n_replicas: int                 # N (the paper's K): local worker + N-1 peers
    period: int                     # H
    optimizer: str                  # "sgdm" | "adamw"
    param_dtype: str                # "f32": fp32 params; "bf16": bf16 model copy + fp32 master, bf16 grads
    lr: float
    momentum: float = 0.9
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    sigma_param: float = 0.02
    sigma_drift: float = 1e-3
    sigma_grad: float = 1e-2
    iterations: int = 16
    policy: str = "enp"             # default schedule policy for the configuration
    time_noise: bool = False        # per-layer U(0.8,1.2) factor on fwd/bwd times
    base_seed: int = 1234
    extra: Dict[str, object] = field(default_factory=dict)

    @property
    def n_layers(self) -> int:
        return self.tensors[-1].layer + 1

    @property
    def n_params(self) -> int:
        return sum(t.numel for t in self.tensors)

    def layer_numel(self) -> List[int]:
        out = [0] * self.n_layers
        for t in self.tensors:
            out[t.layer] += t.numel
        return out


# ----------------------------------------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------------------------------------

CONFIG_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "configs")


def load_config(name: str) -> Dict[str, object]:
    """The benchmark configurations are data: configs/<name>.json holds the model dimensions, N, H, the optimizer and
    its hyper-parameters, the value distributions and the default schedule policy."""
    with open(os.path.join(CONFIG_DIR, name + ".json")) as f:
        return json.load(f)


def _common(c: Dict[str, object]) -> Dict[str, object]:
    keys = ("n_replicas", "period", "optimizer", "param_dtype", "lr", "momentum", "beta1", "beta2", "eps", "weight_decay",
            "sigma_param", "sigma_drift", "sigma_grad", "iterations", "policy", "time_noise")
    return {k: c[k] for k in keys if k in c}


def _mlp_tensors(c) -> List[TensorSpec]:
    ts: List[TensorSpec] = []
    n = int(c["width"])
    for l in range(int(c["n_layers"])):
        ts.append(TensorSpec(f"mlp.{l}.weight", l, n * n))
        ts.append(TensorSpec(f"mlp.{l}.bias", l, n))
    return ts


def _gpt2_tensors(c, with_biases: bool) -> List[TensorSpec]:
    d, ff, vocab, ctx, nb = (int(c[k]) for k in ("d", "ffn", "vocab", "context", "n_blocks"))
    ts = [TensorSpec("wte", 0, vocab * d), TensorSpec("wpe", 1, ctx * d)]
    for b in range(nb):
        l = 2 + b
        ts.append(TensorSpec(f"h.{b}.ln_1.weight", l, d))
        ts.append(TensorSpec(f"h.{b}.ln_1.bias", l, d))
        ts.append(TensorSpec(f"h.{b}.attn.c_attn.weight", l, d * 3 * d))
        if with_biases:
            ts.append(TensorSpec(f"h.{b}.attn.c_attn.bias", l, 3 * d))
        ts.append(TensorSpec(f"h.{b}.attn.c_proj.weight", l, d * d))
        if with_biases:
            ts.append(TensorSpec(f"h.{b}.attn.c_proj.bias", l, d))
        ts.append(TensorSpec(f"h.{b}.ln_2.weight", l, d))
        ts.append(TensorSpec(f"h.{b}.ln_2.bias", l, d))
        ts.append(TensorSpec(f"h.{b}.mlp.c_fc.weight", l, d * ff))
        if with_biases:
            ts.append(TensorSpec(f"h.{b}.mlp.c_fc.bias", l, ff))
        ts.append(TensorSpec(f"h.{b}.mlp.c_proj.weight", l, ff * d))
        if with_biases:
            ts.append(TensorSpec(f"h.{b}.mlp.c_proj.bias", l, d))
    if with_biases:
        ts.append(TensorSpec("ln_f.weight", 2 + nb, d))
        ts.append(TensorSpec("ln_f.bias", 2 + nb, d))
    return ts


def _llama_tensors(c) -> List[TensorSpec]:
    nb, d, ffn, nh, nkv, vocab = (int(c[k]) for k in ("n_blocks", "d", "ffn", "n_heads", "n_kv", "vocab"))
    kv = nkv * (d // nh)
    ts = [TensorSpec("embed_tokens", 0, vocab * d)]
    for b in range(nb):
        l = 1 + b
        ts += [
            TensorSpec(f"layers.{b}.input_layernorm", l, d),
            TensorSpec(f"layers.{b}.q_proj", l, d * d),
            TensorSpec(f"layers.{b}.k_proj", l, d * kv),
            TensorSpec(f"layers.{b}.v_proj", l, d * kv),
            TensorSpec(f"layers.{b}.o_proj", l, d * d),
            TensorSpec(f"layers.{b}.post_attention_layernorm", l, d),
            TensorSpec(f"layers.{b}.gate_proj", l, d * ffn),
            TensorSpec(f"layers.{b}.up_proj", l, d * ffn),
            TensorSpec(f"layers.{b}.down_proj", l, ffn * d),
        ]
    ts += [TensorSpec("norm", 1 + nb, d), TensorSpec("lm_head", 1 + nb, vocab * d)]
    return ts


def from_config(name: str, cfg: Dict[str, object] = None, **variant) -> Workload:
    c = dict(cfg if cfg is not None else load_config(name))
    fam = c["family"]
    if fam == "mlp":
        ts = _mlp_tensors(c)
    elif fam == "gpt2":
        ts = _gpt2_tensors(c, bool(variant.get("with_biases", False)))
    elif fam == "llama":
        ts = _llama_tensors(c)
    else:
        raise ValueError(f"unknown model family {fam!r} in configuration {name}")
    return Workload(name, ts, **_common(c))


def tiny() -> Workload:
    """8-layer MLP, each layer a 256x256 weight and a bias of 256; N=4, H=4, SGD-momentum."""
    return from_config("tiny")


def gpt2_small(with_biases: bool = False) -> Workload:
    """12 blocks at d=768 plus token and position embeddings; fp32, N=8, H=4, SGD-momentum."""
    return from_config("gpt2_small", with_biases=with_biases)


def _llama(name: str, n_blocks: int, d: int, ffn: int, n_heads: int, n_kv: int, vocab: int, *, n_replicas: int,
           period: int, iterations: int, policy: str, time_noise: bool) -> Workload:
    """A Llama-shaped workload from explicit dimensions (the hyper-parameters and distributions of the Llama configurations)."""
    cfg = dict(load_config("llama2_7b"), n_blocks=n_blocks, d=d, ffn=ffn, n_heads=n_heads, n_kv=n_kv, vocab=vocab,
               n_replicas=n_replicas, period=period, iterations=iterations, policy=policy, time_noise=time_noise)
    return from_config(name, cfg)


def tinyllama_1b() -> Workload:
    return from_config("tinyllama_1b")


def llama2_7b() -> Workload:
    return from_config("llama2_7b")


def llama3_8b() -> Workload:
    return from_config("llama3_8b")


def odd(optimizer: str = "adamw", param_dtype: str = "bf16", n_replicas: int = 3, period: int = 2) -> Workload:
    """Unit-test shape: awkward tensor sizes so that every head/tail/misalignment branch is exercised."""
    sizes = [[1, 3], [5, 257], [65537], [1000003, 2], [4096], [7, 8, 9]]
    ts = []
    for l, grp in enumerate(sizes):
        for j, n in enumerate(grp):
            ts.append(TensorSpec(f"odd.{l}.{j}", l, n))
    return Workload(f"odd_{optimizer}_{param_dtype}", ts, n_replicas=n_replicas, period=period,
                    optimizer=optimizer, param_dtype=param_dtype, lr=3e-4 if optimizer == "adamw" else 0.01,
                    sigma_drift=1e-4, sigma_grad=1e-3, iterations=6, policy="round_robin")


def small_llama(n_blocks: int = 4, d: int = 256, ffn: int = 688, vocab: int = 1000, n_replicas: int = 8,
                period: int = 4) -> Workload:
    """A Llama-shaped model small enough for the CPU oracle to run whole trajectories in a second."""
    w = _llama("small_llama", n_blocks, d, ffn, 8, 2, vocab, n_replicas=n_replicas, period=period,
               iterations=16, policy="opt", time_noise=True)
    return w


WORKLOADS = {
    "tiny": tiny,
    "gpt2_small": gpt2_small,
    "tinyllama_1b": tinyllama_1b,
    "llama2_7b": llama2_7b,
    "llama3_8b": llama3_8b,
    "odd": odd,
    "small_llama": small_llama,
}


def get(name: str) -> Workload:
    return WORKLOADS[name]()


# ----------------------------------------------------------------------------------------------------------
# seeded inputs
# ----------------------------------------------------------------------------------------------------------

def seed_for(base_seed: int, config: str, kind: str, iteration: int = 0, peer: int = 0, tensor: int = 0) -> int:
    """Stable 63-bit stream id from (config, kind, iteration, peer, tensor)."""
    key = f"{base_seed}/{config}/{kind}/{iteration}/{peer}/{tensor}".encode()
    return int.from_bytes(hashlib.blake2b(key, digest_size=8).digest(), "little") & ((1 << 63) - 1)


def normal_(out: torch.Tensor, sigma: float, seed: int) -> torch.Tensor:
    """Fill `out` (any device, fp32 or bf16) with N(0, sigma^2) draws from a generator seeded with `seed`.

    Draws are made in fp32 and rounded once to the tensor's dtype.  CPU and GPU generators give different
    streams; a test always generates once and hands the same bytes to both implementations."""
    g = torch.Generator(device=out.device)
    g.manual_seed(seed)
    if out.dtype == torch.float32:
        out.normal_(0.0, sigma, generator=g)
    else:
        tmp = torch.empty(out.shape, dtype=torch.float32, device=out.device)
        tmp.normal_(0.0, sigma, generator=g)
        out.copy_(tmp)
    return out


def synthetic_times(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-layer profiled times in integer nanoseconds: (t_fp, t_bp, t_comm).

    Recipe: wire bytes of a layer = 4 * numel (fp32 on the wire).  t_comm = bytes / 1 Gbps = 8 ns per byte,
    t_bp = 2 ns per byte, t_fp = 1 ns per byte; with `time_noise` each fwd/bwd time is scaled by an
    independent U(0.8, 1.2) factor drawn from a numpy generator seeded from the workload.
    `w.extra["comm_ns_per_byte"]` overrides the 8 ns per byte (a faster network leaves bubbles to fill)."""
    numel = np.asarray(w.layer_numel(), dtype=np.float64)
    nbytes = 4.0 * numel
    L = len(numel)
    if w.time_noise:
        rng = np.random.default_rng(seed_for(w.base_seed, w.name, "times"))
        uf = rng.uniform(0.8, 1.2, size=L)
        ub = rng.uniform(0.8, 1.2, size=L)
    else:
        uf = np.ones(L)
        ub = np.ones(L)
    t_fp = np.rint(1.0 * nbytes * uf).astype(np.int64)
    t_bp = np.rint(2.0 * nbytes * ub).astype(np.int64)
    t_comm = np.rint(float(w.extra.get("comm_ns_per_byte", 8.0)) * nbytes).astype(np.int64)
    return t_fp, t_bp, t_comm
