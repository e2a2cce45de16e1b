"""Seeded synthetic inputs for the attention hot path.

Holds no attention arithmetic: only shapes, seeds and random draws, so that the CPU
oracle (tests) and the HIP path consume the same bytes.  The five configurations are
the per-GPU shapes that hybrid sequence parallelism (Sec. 2.4 "SP-2", Sec. 3.2.2
"Sequence Parallelism") gives one GPU: all S tokens of heads/s_sp heads, head
dimension 128 as in every model of Table 2.  The paper evaluates throughput only and
names no dataset, so N(0,1) activations stand in for real ones.
"""
from dataclasses import dataclass
import math

import numpy as np
import torch


@dataclass(frozen=True)
class AttnConfig:
    name: str
    index: int
    B: int
    S: int
    Hq: int
    Hkv: int
    D: int
    causal: bool = True
    packed: bool = False          # documents given by cu_seqlens (block-diagonal mask)
    doc_len_min: int = 512
    doc_len_max: int = 65536

    @property
    def seed(self):
        return 1000 + self.index

    @property
    def scale(self):
        return 1.0 / math.sqrt(self.D)


CONFIGS = [
    AttnConfig("tiny_s512_h2_d64", 0, B=1, S=512, Hq=2, Hkv=2, D=64),
    AttnConfig("7b_s32k_h32_d128", 1, B=1, S=32768, Hq=32, Hkv=32, D=128),
    AttnConfig("7b_s128k_h8_d128", 2, B=1, S=131072, Hq=8, Hkv=8, D=128),
    AttnConfig("gqa_s64k_hq8_hkv1_d128", 3, B=1, S=65536, Hq=8, Hkv=1, D=128),
    AttnConfig("packed_256k_h4_d128", 4, B=1, S=262144, Hq=4, Hkv=4, D=128, packed=True),
]


def doc_lengths(total, lo, hi, seed):
    """Document lengths drawn log-uniformly in [lo, hi], one after another, the last one cut to fill
    exactly `total` tokens (so the tail may be shorter than lo)."""
    rng = np.random.default_rng(seed)
    out, used = [], 0
    while used < total:
        L = int(round(math.exp(rng.uniform(math.log(lo), math.log(hi)))))
        L = min(L, total - used)
        out.append(L)
        used += L
    return out


def cu_seqlens_of(lengths):
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return cu


def make_cu_seqlens(cfg):
    """int32 numpy prefix sums for a packed configuration, None for a dense one."""
    if not cfg.packed:
        return None
    return cu_seqlens_of(doc_lengths(cfg.S, cfg.doc_len_min, cfg.doc_len_max, cfg.seed))


def make_inputs(cfg, device="cpu", with_dout=True):
    """q, k, v, dO ~ N(0,1) rounded to bf16 (round to nearest even), drawn on the CPU from
    torch.manual_seed(cfg.seed) in that order, then moved to `device`."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(cfg.seed)
    shapes = [(cfg.B, cfg.S, cfg.Hq, cfg.D), (cfg.B, cfg.S, cfg.Hkv, cfg.D), (cfg.B, cfg.S, cfg.Hkv, cfg.D)]
    if with_dout:
        shapes.append((cfg.B, cfg.S, cfg.Hq, cfg.D))
    out = []
    for shp in shapes:
        x = torch.randn(shp, generator=gen, dtype=torch.float32).to(torch.bfloat16)
        out.append(x.to(device) if device != "cpu" else x)
    return tuple(out)


def fwd_flops(cfg, cu_seqlens=None):
    """Forward FLOP with causal halving: 2 * D * Hq * sum over documents of L^2 (x B)."""
    if cu_seqlens is None:
        sq = float(cfg.S) ** 2
    else:
        L = np.diff(np.asarray(cu_seqlens, dtype=np.int64)).astype(np.float64)
        sq = float((L * L).sum())
    f = 4.0 * sq * cfg.D * cfg.Hq * cfg.B
    return f / 2.0 if cfg.causal else f


def bwd_flops(cfg, cu_seqlens=None):
    return 2.5 * fwd_flops(cfg, cu_seqlens)


# -- the re-layouts either side of the sequence-parallel all-to-alls -----------------------------------

@dataclass(frozen=True)
class SpConfig:
    """One GPU's buffers around the two all-to-alls of a layer (Sec. 2.4 "SP-2", Sec. 3.2.2): micro-batch B,
    Sl = S/P tokens per sequence slice, Hq / Hkv heads of the whole layer, P = s_sp peers."""
    name: str
    index: int
    B: int
    Sl: int
    Hq: int
    Hkv: int
    D: int
    P: int

    @property
    def seed(self):
        return 2000 + self.index

    @property
    def n_qkv(self):
        return self.B * self.Sl * (self.Hq + 2 * self.Hkv) * self.D

    @property
    def n_o(self):
        return self.B * self.Sl * self.Hq * self.D


# The paper's own plans (Appendix Tables 4-7, "Our Work" rows) for 7B at 32K (s_sp = 4: 8 heads per GPU),
# 7B at 256K (s_sp = 32: one head per GPU, the shortest runs) and 65B at 64K (s_sp = 8), plus a small case.
SP_CONFIGS = [
    SpConfig("tiny_b2_sl96_h8_kv4_d64_p4", 0, B=2, Sl=96, Hq=8, Hkv=4, D=64, P=4),
    SpConfig("7b_s32k_sp4", 1, B=1, Sl=8192, Hq=32, Hkv=32, D=128, P=4),
    SpConfig("7b_s256k_sp32", 2, B=1, Sl=8192, Hq=32, Hkv=32, D=128, P=32),
    SpConfig("65b_s64k_sp8", 3, B=1, Sl=8192, Hq=64, Hkv=64, D=128, P=8),
]


def make_bit_patterns(n, seed, device="cpu"):
    """n random 16-bit patterns (int16), drawn on the CPU: the permutations move bf16 values as bits, and
    arbitrary patterns include NaNs, infinities and denormals."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    x = torch.randint(-32768, 32768, (n,), generator=gen, dtype=torch.int16)
    return x.to(device) if device != "cpu" else x
