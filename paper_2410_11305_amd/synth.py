"""Seeded synthetic inputs for the QSpec linear-layer workloads.

This module holds no arithmetic of the method itself: it only draws the
random tensors (weight codes, weight scales, activations) that both the HIP
path and the test oracle consume, and lists the layer shapes of the five
benchmark configurations.  The shapes are the linear layers of Llama-class
decoder blocks (the models of paper Sec. 4.1 / Table 4), batch sizes 4..128
and draft lengths gamma = 3 or 5 (Sec. 4.1; Fig. 5 ablation); they stand in
for the paper's checkpoints and prompt sets, which are not available offline.

Recipe (NumPy PCG64, seed = 10000*config + 100*layer + stream):
  stream 0  weight codes   integers in [-8, 7], int8 [N, K]
  stream 1  weight scales  uniform [0.002, 0.01) -> fp16 [N, K/128]
  stream 2  draft x        N(0,1) fp32 [M_draft, K], outlier channels x20, -> fp16
  stream 3  verify x       same, [M_verify, K]
  stream 4  outlier channel indices (without replacement), shared by 2 and 3
Inputs of the steps after the verify pass (accept_case): stream 5 of a config,
  logits   N(0, 2) fp32 [B, gamma+1, V] -> fp16, with one planted token per row
           raised to (row maximum + 4), so the greedy token is known by construction
  drafts   the planted token of their row with probability p_accept, else another id
  V is the Llama vocabulary size of the config's model class (32000; 128256 exists
  in the Llama-3 checkpoints the paper also serves and is covered by the tests).
Inputs of the fused producers (producer_case): the residual stream x as above
  (N(0,1), outlier channels x20), an RMSNorm weight 1 + 0.1 N(0,1) -> fp16, and a merged
  gate/up tensor N(0, 1.5) -> fp16 [M, 2I]; eps = 1e-5 (the Llama-2 value).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

import numpy as np

GROUP = 128


@dataclass(frozen=True)
class Layer:
    name: str
    K: int
    N: int


@dataclass(frozen=True)
class Config:
    index: int
    label: str
    layers: tuple
    batch: int
    gamma: int
    n_outliers_exact: int = -1      # >= 0: that many outlier channels, else 1 % of K

    @property
    def draft_M(self) -> int:       # one token per sequence per draft step (Sec. 3.1)
        return self.batch

    @property
    def verify_M(self) -> int:      # gamma drafts + 1 per sequence in one pass (Sec. 3.1)
        return self.batch * (self.gamma + 1)


_L7B = (Layer("qkv", 4096, 12288), Layer("o", 4096, 4096),
        Layer("gate_up", 4096, 22016), Layer("down", 11008, 4096))
_L13B = (Layer("qkv", 5120, 15360), Layer("o", 5120, 5120),
         Layer("gate_up", 5120, 27648), Layer("down", 13824, 5120))
_L70B = (Layer("qkv", 8192, 10240), Layer("o", 8192, 8192),
         Layer("gate_up", 8192, 57344), Layer("down", 28672, 8192))

CONFIGS: Dict[int, Config] = {
    1: Config(1, "single-1024", (Layer("lin", 1024, 1024),), 4, 3, n_outliers_exact=4),
    2: Config(2, "llama7b-b8-g3", _L7B, 8, 3),
    3: Config(3, "llama7b-b32-g3", _L7B, 32, 3),
    4: Config(4, "llama13b-b64-g5", _L13B, 64, 5),
    5: Config(5, "llama70b-b128-g3", _L70B, 128, 3),
}


def _seed(config: int, layer_index: int, stream: int) -> int:
    return 10000 * config + 100 * layer_index + stream


def n_outliers(cfg: Config, K: int) -> int:
    if cfg.n_outliers_exact >= 0:
        return cfg.n_outliers_exact
    return int(round(0.01 * K))


def weight_codes(config: int, layer_index: int, N: int, K: int) -> np.ndarray:
    rng = np.random.default_rng(_seed(config, layer_index, 0))
    return rng.integers(-8, 8, size=(N, K), dtype=np.int8)


def weight_scales(config: int, layer_index: int, N: int, K: int) -> np.ndarray:
    rng = np.random.default_rng(_seed(config, layer_index, 1))
    return rng.uniform(0.002, 0.01, size=(N, K // GROUP)).astype(np.float16)


def outlier_channels(config: int, layer_index: int, K: int) -> np.ndarray:
    cfg = CONFIGS[config]
    rng = np.random.default_rng(_seed(config, layer_index, 4))
    return np.sort(rng.choice(K, size=n_outliers(cfg, K), replace=False))


def activations(config: int, layer_index: int, M: int, K: int, verify: bool) -> np.ndarray:
    rng = np.random.default_rng(_seed(config, layer_index, 3 if verify else 2))
    x = rng.standard_normal((M, K), dtype=np.float32)
    x[:, outlier_channels(config, layer_index, K)] *= np.float32(20.0)
    return x.astype(np.float16)


def generic_case(seed: int, M: int, N: int, K: int, outlier_frac: float = 0.01):
    """Same recipe for an arbitrary (M, N, K): returns codes, scales, x."""
    rng = np.random.default_rng(seed)
    codes = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    scales = rng.uniform(0.002, 0.01, size=(N, K // GROUP)).astype(np.float16)
    x = rng.standard_normal((M, K), dtype=np.float32)
    n_out = max(1, int(round(outlier_frac * K)))
    x[:, rng.choice(K, size=n_out, replace=False)] *= np.float32(20.0)
    return codes, scales, x.astype(np.float16)


def layer_table(config: int) -> List[dict]:
    cfg = CONFIGS[config]
    return [dict(config=config, layer_index=i, name=l.name, K=l.K, N=l.N,
                 draft_M=cfg.draft_M, verify_M=cfg.verify_M)
            for i, l in enumerate(cfg.layers)]


VOCAB = {1: 1024, 2: 32000, 3: 32000, 4: 32000, 5: 32000}     # Llama-2 class vocabulary; config 1 is a toy size


def accept_case(seed: int, B: int, gamma: int, V: int, p_accept: float = 0.8):
    """Logits of a verify pass and drafted tokens: returns (logits fp16 [B, gamma+1, V],
    draft int32 [B, gamma], planted int32 [B, gamma+1])."""
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((B, gamma + 1, V), dtype=np.float32) * np.float32(2.0))
    planted = rng.integers(0, V, size=(B, gamma + 1)).astype(np.int32)
    top = logits.max(axis=2)
    for b in range(B):
        for j in range(gamma + 1):
            logits[b, j, planted[b, j]] = top[b, j] + np.float32(4.0)
    draft = planted[:, :gamma].copy()
    miss = rng.random((B, gamma)) >= p_accept
    other = rng.integers(1, max(V, 2), size=(B, gamma)).astype(np.int32)
    draft[miss] = (draft[miss] + other[miss]) % V if V > 1 else draft[miss]
    return logits.astype(np.float16), draft.astype(np.int32), planted


def accept_inputs(config: int):
    cfg = CONFIGS[config]
    return accept_case(_seed(config, 0, 5), cfg.batch, cfg.gamma, VOCAB[config])


RMS_EPS = 1e-5


def producer_case(seed: int, M: int, K: int, I: int, outlier_frac: float = 0.01):
    """Inputs of the fused producers: returns (x fp16 [M, K], norm weight fp16 [K],
    gate_up fp16 [M, 2I])."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K), dtype=np.float32)
    n_out = max(1, int(round(outlier_frac * K)))
    x[:, rng.choice(K, size=n_out, replace=False)] *= np.float32(20.0)
    w = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    gate_up = (rng.standard_normal((M, 2 * I), dtype=np.float32) * np.float32(1.5)).astype(np.float16)
    return x.astype(np.float16), w, gate_up


def producer_inputs(config: int):
    """Draft-pass producer inputs of a configuration: hidden size = K of its first layer,
    intermediate size = K of its last layer (the down projection)."""
    cfg = CONFIGS[config]
    K, I = cfg.layers[0].K, cfg.layers[-1].K
    return producer_case(_seed(config, 0, 6), cfg.draft_M, K, I)
