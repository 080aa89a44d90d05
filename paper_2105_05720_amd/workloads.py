"""Seeded synthetic workloads: parameter lists, initial state and fp16 gradient slices.

This module holds no optimizer arithmetic.  It serves the GPU tests, the benchmark and the CPU oracle
tests alike: both sides of every comparison read the same generated bits.

The paper's data-parallel experiments update BERT and GPT-2 parameter lists in mixed precision
(Section 6.1; Table 2 for the scattered-tensor BERT case; Table 4 for the model sizes).  The real
models and their training data are not available here; the update depends only on tensor shapes and
value ranges, so the published architecture shapes with seeded Gaussian values stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import torch


@dataclass(frozen=True)
class ParamSpec:
    name: str
    numel: int
    kind: str          # "matrix" (N(0, 0.02)), "ln_gamma" (ones), "bias" (zeros; also LayerNorm beta)

    @property
    def decays(self) -> bool:
        return self.kind == "matrix"


def flat_list(n: int) -> List[ParamSpec]:
    return [ParamSpec("flat", n, "matrix")]


def _linear(prefix: str, fan_in: int, fan_out: int) -> List[ParamSpec]:
    return [ParamSpec(prefix + ".weight", fan_in * fan_out, "matrix"), ParamSpec(prefix + ".bias", fan_out, "bias")]


def _layernorm(prefix: str, h: int) -> List[ParamSpec]:
    return [ParamSpec(prefix + ".gamma", h, "ln_gamma"), ParamSpec(prefix + ".beta", h, "bias")]


def bert_large_list(layers: int = 24, hidden: int = 1024, ffn: int = 4096, vocab: int = 30522,
                    positions: int = 512, types: int = 2) -> List[ParamSpec]:
    """BERT-Large pre-training parameter list: embeddings, encoder, pooler, MLM and NSP heads."""
    p: List[ParamSpec] = [
        ParamSpec("emb.word", vocab * hidden, "matrix"),
        ParamSpec("emb.position", positions * hidden, "matrix"),
        ParamSpec("emb.type", types * hidden, "matrix"),
    ] + _layernorm("emb.ln", hidden)
    for l in range(layers):
        pre = "layer%d." % l
        for nm in ("q", "k", "v", "attn_out"):
            p += _linear(pre + nm, hidden, hidden)
        p += _layernorm(pre + "attn_ln", hidden)
        p += _linear(pre + "ffn_in", hidden, ffn)
        p += _linear(pre + "ffn_out", ffn, hidden)
        p += _layernorm(pre + "ffn_ln", hidden)
    p += _linear("pooler", hidden, hidden)
    p += _linear("mlm.transform", hidden, hidden)
    p += _layernorm("mlm.ln", hidden)
    p += [ParamSpec("mlm.decoder_bias", vocab, "bias")]
    p += _linear("nsp", hidden, 2)
    return p


def gpt2_xl_list(layers: int = 48, hidden: int = 1600, vocab: int = 50257, positions: int = 1024) -> List[ParamSpec]:
    """GPT-2 1.5B parameter list (tied output embedding)."""
    p: List[ParamSpec] = [ParamSpec("wte", vocab * hidden, "matrix"), ParamSpec("wpe", positions * hidden, "matrix")]
    for l in range(layers):
        pre = "h%d." % l
        p += _layernorm(pre + "ln_1", hidden)
        p += _linear(pre + "attn.qkv", hidden, 3 * hidden)
        p += _linear(pre + "attn.proj", hidden, hidden)
        p += _layernorm(pre + "ln_2", hidden)
        p += _linear(pre + "mlp.fc", hidden, 4 * hidden)
        p += _linear(pre + "mlp.proj", 4 * hidden, hidden)
    p += _layernorm("ln_f", hidden)
    return p


def megatron_8p3b_shard_list(layers: int = 72, hidden: int = 3072, vocab: int = 51200, positions: int = 1024,
                             shards: int = 8) -> List[ParamSpec]:
    """One rank's 1/shards slice of an 8.3B transformer: one slice per layer plus one embedding slice.

    A layer holds 12 h^2 + 13 h parameters; each per-layer slice is one trust-ratio unit.
    """
    per_layer = 12 * hidden * hidden + 13 * hidden
    assert per_layer % shards == 0 and ((vocab + positions) * hidden) % shards == 0
    p = [ParamSpec("layer%d.slice" % l, per_layer // shards, "matrix") for l in range(layers)]
    p.append(ParamSpec("emb.slice", (vocab + positions) * hidden // shards, "matrix"))
    return p


@dataclass(frozen=True)
class Config:
    """One of the five benchmark configurations."""
    index: int
    optimizer: str                 # "adam" | "lamb"
    params: Tuple[ParamSpec, ...]
    R: int
    grad_std: float                # std of the fp16 gradient values as stored (already loss-scaled)
    loss_scale: float
    steps: int
    seed: int
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-6
    weight_decay: float = 0.01
    decay_all: bool = False        # config 1's single flat tensor decays; elsewhere bias/LayerNorm do not

    @property
    def numel(self) -> int:
        return sum(s.numel for s in self.params)

    def wd_of(self, spec: ParamSpec) -> float:
        return self.weight_decay if (self.decay_all or spec.decays) else 0.0


def config(index: int) -> Config:
    if index == 1:
        return Config(1, "adam", tuple(flat_list(1 << 20)), R=4, grad_std=1e-2, loss_scale=1.0, steps=3, seed=0,
                      decay_all=True)
    if index == 2:
        return Config(2, "adam", tuple(bert_large_list()), R=8, grad_std=1e-3, loss_scale=1.0, steps=1, seed=2)
    if index == 3:
        return Config(3, "lamb", tuple(bert_large_list()), R=8, grad_std=1e-3, loss_scale=1.0, steps=2, seed=3)
    if index == 4:
        return Config(4, "adam", tuple(gpt2_xl_list()), R=8, grad_std=1024 * 1e-3, loss_scale=1024.0, steps=3, seed=4)
    if index == 5:
        return Config(5, "lamb", tuple(megatron_8p3b_shard_list()), R=8, grad_std=1e-3, loss_scale=1.0, steps=2,
                      seed=5)
    raise ValueError("config index must be 1..5")


# Config 4 plants one +inf in its second step: rank 3, layer 24's 1600x6400 matrix, element 12345.
CFG4_INF_STEP = 2
CFG4_INF_RANK = 3
CFG4_INF_TENSOR = "h24.mlp.fc.weight"
CFG4_INF_INDEX = 12345
HALF_POS_INF = 0x7C00


def seed_key(cfg_seed: int, step: int, rank: int, tensor_index: int) -> int:
    """One generator seed per (config, step, rank, tensor); rank 99 is reserved for the initial weights."""
    return ((cfg_seed * 1000 + step) * 100 + rank) * 10000 + tensor_index


def _gen(device, key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(key)
    return g


def init_weight(spec: ParamSpec, cfg_seed: int, tensor_index: int, device, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """fp32 initial master weights of one tensor: N(0, 0.02), ones (LayerNorm gain) or zeros (bias)."""
    if out is None:
        out = torch.empty(spec.numel, dtype=torch.float32, device=device)
    if spec.numel == 0:
        return out
    if spec.kind == "matrix":
        out.normal_(0.0, 0.02, generator=_gen(out.device, seed_key(cfg_seed, 0, 99, tensor_index)))
    elif spec.kind == "ln_gamma":
        out.fill_(1.0)
    else:
        out.zero_()
    return out


def grad_slice(numel: int, std: float, cfg_seed: int, step: int, rank: int, tensor_index: int, device,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One rank's fp16 gradient slice for one tensor: fp16(N(0, std)) drawn in fp32 then rounded."""
    if out is None:
        out = torch.empty(numel, dtype=torch.float16, device=device)
    if numel == 0:
        return out
    # (an fp32 `out` keeps the drawn values unrounded: the Float 32 variant of the workload)
    g32 = torch.empty(numel, dtype=torch.float32, device=out.device)
    g32.normal_(0.0, std, generator=_gen(out.device, seed_key(cfg_seed, step, rank, tensor_index)))
    out.copy_(g32)          # round to nearest even, subnormals kept
    return out


def aligned_offsets(numels, align_elems: int) -> Tuple[List[int], int]:
    """Element offsets that place tensors back to back in one arena, each start a multiple of align_elems."""
    offs, cur = [], 0
    for n in numels:
        offs.append(cur)
        cur += -(-n // align_elems) * align_elems
    return offs, max(cur, align_elems)


def table_bytes_paper(n: int) -> int:
    """Memory of the paper's bucket table for one tensor of n elements (Section 5.4): 12 B per 2^10 elements."""
    return 12 * (-(-n // 1024))


# ---- filling a device shard (any object with w_of/m_of/v_of/w16_of/grad_of(k) views) with a config's bits ----

def fill_state(shard, cfg: Config) -> None:
    """Initial committed state of a config: seeded weights, m = v = 0, fp16 copy of the weights."""
    for k, spec in enumerate(cfg.params):
        init_weight(spec, cfg.seed, k, shard.device, out=shard.w_of(k))
        shard.m_of(k).zero_()
        shard.v_of(k).zero_()
        shard.w16_of(k).copy_(shard.w_of(k))


def fill_grads(shard, cfg: Config, call_index: int) -> None:
    """The R gradient slices of one optimizer call.  call_index counts calls from 1 (a skipped step consumes
    an index too, so a repeated step draws fresh gradients).  Config 4 plants its +inf in call 2."""
    for k, spec in enumerate(cfg.params):
        for r in range(cfg.R):
            grad_slice(spec.numel, cfg.grad_std, cfg.seed, call_index, r, k, shard.device, out=shard.grad_of(r, k))
    if cfg.index == 4 and call_index == CFG4_INF_STEP:
        k = [s.name for s in cfg.params].index(CFG4_INF_TENSOR)
        # 0x7C00 as a signed 16-bit pattern
        shard.grad_of(CFG4_INF_RANK, k).view(torch.int16)[CFG4_INF_INDEX] = HALF_POS_INF
