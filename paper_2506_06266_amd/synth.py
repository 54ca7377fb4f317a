"""Seeded synthetic inputs shaped like the Cartridge / Self-Study workloads.

This module only draws random numbers and shapes them; it contains none of
the method's arithmetic (no attention, no loss).  Both the CPU oracle's tests
and the HIP path's tests consume what it returns, so both sides always see the
same bits: a tensor is generated once, on one device, and copied to the other.

The paper's training workload is batches of synthetic conversations (at most
1024 tokens each, global batch 64) run through Llama-3B / Llama-8B with a
trainable prefix of p in {128 ... 8192} KV slots (Fig. "scaling-indexing"
caption), distilled against the teacher's recorded top output probabilities
(App. A.2 "Training Objective").  The real conversations, corpora, model
weights and teacher log-probs are not available; the tensors below stand in
for the per-layer Q/K/V, the prefix Z, the student logits and the teacher
top-k records at those shapes.

In every "N(0, s)" below s is a standard deviation.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class AttnConfig:
    name: str
    seed: int
    B: int
    S: int
    Hq: int
    Hkv: int
    D: int
    P: int
    dtype: str          # "f32" | "bf16"
    qkv_std: float      # std of Q, K_own, V_own
    do_std: float       # std of dO
    z_std: float        # std of Z_k, Z_v
    q_std: Optional[float] = None   # overrides qkv_std for Q and K when set ("sharp" input)


@dataclass(frozen=True)
class KLConfig:
    name: str
    seed: int
    N: int
    V: int
    K: int
    dtype: str
    logit_std: float
    teacher_std: float
    mass: float

    @property
    def scale(self) -> float:
        return 1.0 / self.N


@dataclass(frozen=True)
class DecodeConfig:
    name: str
    seed: int
    B: int
    Hq: int
    Hkv: int
    D: int
    P: int
    min_len: int
    max_len: int
    dtype: str
    qkv_std: float
    z_std: float


_R128 = 1.0 / math.sqrt(128.0)

ATTN_CONFIGS: Dict[str, AttnConfig] = {
    # tiny fp32 case for the oracle, gradient checks and full element-wise parity
    "cfg1_attn": AttnConfig("cfg1_attn", 1001, 2, 64, 2, 1, 64, 32, "f32", 1.0, 1.0, 1.0 / 8.0),
    # Llama-3B-shaped layer
    "cfg2": AttnConfig("cfg2", 2001, 32, 1024, 24, 8, 128, 2048, "bf16", _R128, _R128, 0.02),
    # Llama-8B-shaped layer: the headline attention config
    "cfg3": AttnConfig("cfg3", 3001, 16, 2048, 32, 8, 128, 4096, "bf16", _R128, _R128, 0.02),
    # shrunken bf16 case with unit-variance Q,K so that the softmax is far from uniform
    "sharp": AttnConfig("sharp", 6001, 2, 256, 8, 2, 128, 512, "bf16", 1.0, 1.0, 1.0, q_std=1.0),
    # shrunken bf16 case at cfg2/cfg3's value distributions with ragged tile tails
    "ragged": AttnConfig("ragged", 6002, 3, 200, 8, 2, 128, 333, "bf16", _R128, _R128, 0.02),
}

KL_CONFIGS: Dict[str, KLConfig] = {
    "cfg1_loss": KLConfig("cfg1_loss", 1002, 128, 1000, 20, "f32", 2.0, 2.0, 0.9),
    "cfg4": KLConfig("cfg4", 4001, 16384, 128256, 20, "bf16", 3.0, 3.0, 0.95),
    # shrunken bf16 cases: full vocabulary / few rows, and a vocabulary with a ragged vector tail
    "kl_small": KLConfig("kl_small", 4002, 48, 128256, 20, "bf16", 3.0, 3.0, 0.95),
    "kl_ragged": KLConfig("kl_ragged", 4003, 37, 50257, 20, "bf16", 3.0, 3.0, 0.95),
    # more rows than the loss kernel has workgroups (each walks several rows), small vocabulary
    "kl_many_rows": KLConfig("kl_many_rows", 4004, 700, 4096, 20, "bf16", 3.0, 3.0, 0.95),
}

DECODE_CONFIGS: Dict[str, DecodeConfig] = {
    "cfg5": DecodeConfig("cfg5", 5001, 128, 32, 8, 128, 8192, 1, 1024, "bf16", _R128, 0.02),
    # the comparison run: no cartridge, every request carries a full 131072-token KV cache
    "cfg5_long": DecodeConfig("cfg5_long", 5002, 8, 32, 8, 128, 0, 131072, 131072, "bf16", _R128, 0.02),
    "decode_small": DecodeConfig("decode_small", 5003, 9, 8, 2, 128, 300, 1, 150, "bf16", _R128, 0.02),
    "decode_f32": DecodeConfig("decode_f32", 5004, 5, 4, 2, 64, 40, 1, 50, "f32", 1.0, 1.0 / 8.0),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _normal(shape, std: float, dtype: torch.dtype, gen: torch.Generator, device) -> torch.Tensor:
    """N(0, std) drawn in fp32, rounded once (nearest-even) to the storage dtype."""
    numel = 1
    for s in shape:
        numel *= s
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    chunk = 1 << 26                      # bound the fp32 staging buffer
    for lo in range(0, numel, chunk):
        hi = min(numel, lo + chunk)
        x = torch.randn(hi - lo, dtype=torch.float32, device=device, generator=gen)
        flat[lo:hi] = (x * std).to(dtype)
    return out


def attn_inputs(cfg: AttnConfig, device="cpu") -> Dict[str, torch.Tensor]:
    """Q [B,S,Hq,D], K_own/V_own [B,S,Hkv,D], Z_k/Z_v [Hkv,P,D], dO [B,S,Hq,D]."""
    g = _gen(cfg.seed, device)
    dt = torch_dtype(cfg.dtype)
    qk_std = cfg.q_std if cfg.q_std is not None else cfg.qkv_std
    return {
        "q": _normal((cfg.B, cfg.S, cfg.Hq, cfg.D), qk_std, dt, g, device),
        "k_own": _normal((cfg.B, cfg.S, cfg.Hkv, cfg.D), qk_std, dt, g, device),
        "v_own": _normal((cfg.B, cfg.S, cfg.Hkv, cfg.D), cfg.qkv_std, dt, g, device),
        "z_k": _normal((cfg.Hkv, cfg.P, cfg.D), cfg.z_std, dt, g, device),
        "z_v": _normal((cfg.Hkv, cfg.P, cfg.D), cfg.z_std, dt, g, device),
        "d_o": _normal((cfg.B, cfg.S, cfg.Hq, cfg.D), cfg.do_std, dt, g, device),
    }


@dataclass(frozen=True)
class PackedConfig:
    """A packed batch of conversations of different lengths at the layer shape of `base`
    (whose B and S are not used): n_seq lengths drawn uniformly from [min_len, max_len]."""
    name: str
    seed: int
    base: str
    n_seq: int
    min_len: int
    max_len: int


PACKED_CONFIGS: Dict[str, PackedConfig] = {
    # one global batch of the paper's training runs: 64 conversations of at most 1024 tokens,
    # Llama-8B layer shape, p = 4096
    "cfg3_packed": PackedConfig("cfg3_packed", 3101, "cfg3", 64, 64, 1024),
    "ragged_packed": PackedConfig("ragged_packed", 6102, "ragged", 7, 1, 300),
}


def packed_lengths(cfg: PackedConfig) -> torch.Tensor:
    """The n_seq sequence lengths (int64, host)."""
    g = _gen(cfg.seed, "cpu")
    return torch.randint(cfg.min_len, cfg.max_len + 1, (cfg.n_seq,), generator=g)


def attn_packed_inputs(cfg: PackedConfig, device="cpu") -> Dict[str, torch.Tensor]:
    """Q [T,Hq,D], K_own/V_own [T,Hkv,D], Z_k/Z_v [Hkv,P,D], dO [T,Hq,D], cu_seqlens [n_seq+1]
    int32 (on `device`), T = the sum of packed_lengths(cfg)."""
    a = ATTN_CONFIGS[cfg.base]
    lens = packed_lengths(cfg)
    T = int(lens.sum())
    g = _gen(cfg.seed + 1, device)
    dt = torch_dtype(a.dtype)
    qk_std = a.q_std if a.q_std is not None else a.qkv_std
    cu = torch.zeros(cfg.n_seq + 1, dtype=torch.int32)
    cu[1:] = torch.cumsum(lens, 0).to(torch.int32)
    return {
        "q": _normal((T, a.Hq, a.D), qk_std, dt, g, device),
        "k_own": _normal((T, a.Hkv, a.D), qk_std, dt, g, device),
        "v_own": _normal((T, a.Hkv, a.D), a.qkv_std, dt, g, device),
        "z_k": _normal((a.Hkv, a.P, a.D), a.z_std, dt, g, device),
        "z_v": _normal((a.Hkv, a.P, a.D), a.z_std, dt, g, device),
        "d_o": _normal((T, a.Hq, a.D), a.do_std, dt, g, device),
        "cu_seqlens": cu.to(device),
    }


def _distinct_indices(n: int, v: int, k: int, gen: torch.Generator, device) -> torch.Tensor:
    """[n,k] int32, each row k distinct values uniform in [0,v): rows with a repeat are redrawn."""
    idx = torch.randint(0, v, (n, k), generator=gen, device=device, dtype=torch.int64)
    while True:
        s, _ = torch.sort(idx, dim=1)
        bad = (s[:, 1:] == s[:, :-1]).any(dim=1)
        nbad = int(bad.sum().item())
        if nbad == 0:
            break
        idx[bad] = torch.randint(0, v, (nbad, k), generator=gen, device=device, dtype=torch.int64)
    return idx.to(torch.int32)


def kl_inputs(cfg: KLConfig, device="cpu") -> Dict[str, torch.Tensor]:
    """Student logits [N,V]; teacher records: idx [N,K] int32 (distinct per row) and
    logp [N,K] fp32 with sum_j exp(logp) == cfg.mass, stored by descending probability."""
    g = _gen(cfg.seed, device)
    logits = _normal((cfg.N, cfg.V), cfg.logit_std, torch_dtype(cfg.dtype), g, device)
    idx = _distinct_indices(cfg.N, cfg.V, cfg.K, g, device)
    raw = torch.randn(cfg.N, cfg.K, dtype=torch.float64, device=device, generator=g) * cfg.teacher_std
    raw, _ = torch.sort(raw, dim=1, descending=True)
    raw = raw - raw.max(dim=1, keepdim=True).values
    w = torch.exp(raw)
    prob = w / w.sum(dim=1, keepdim=True) * cfg.mass
    logp = torch.log(prob).to(torch.float32)
    return {"logits": logits, "teacher_idx": idx, "teacher_logp": logp}


def decode_inputs(cfg: DecodeConfig, device="cpu") -> Dict[str, torch.Tensor]:
    """q [B,Hq,D]; Z_k/Z_v [Hkv,P,D]; ragged own K/V [T,Hkv,D] with cu_lens [B+1] int32."""
    g = _gen(cfg.seed, device)
    dt = torch_dtype(cfg.dtype)
    lens = torch.randint(cfg.min_len, cfg.max_len + 1, (cfg.B,), generator=g, device=device,
                         dtype=torch.int64)
    cu = torch.zeros(cfg.B + 1, dtype=torch.int64, device=device)
    cu[1:] = torch.cumsum(lens, 0)
    total = int(cu[-1].item())
    return {
        "q": _normal((cfg.B, cfg.Hq, cfg.D), cfg.qkv_std, dt, g, device),
        "z_k": _normal((cfg.Hkv, cfg.P, cfg.D), cfg.z_std, dt, g, device),
        "z_v": _normal((cfg.Hkv, cfg.P, cfg.D), cfg.z_std, dt, g, device),
        "k_own": _normal((total, cfg.Hkv, cfg.D), cfg.qkv_std, dt, g, device),
        "v_own": _normal((total, cfg.Hkv, cfg.D), cfg.qkv_std, dt, g, device),
        "cu_lens": cu.to(torch.int32),
    }
