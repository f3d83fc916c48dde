"""Seeded synthetic inputs shaped like the paper's three models (Sec. 3.6, Sec. 4 set-up).

This module only draws numbers and lays out block tables.  It holds none of the
method's arithmetic (no quantizer, no attention), so both the GPU library's tests
and the CPU oracle's tests may take their inputs from it.

Values come from a counter-based generator built from integer tensor operations
only, so the same (seed, tensor, layer, agent, token, head, dim) coordinate gives
the same binary16 bit pattern on the CPU and on the GPU, and any slice of a large
cache can be regenerated alone:

    u16   = top 16 bits of mix64(key(seed, tensor, layer, agent) + GAMMA * counter)
    value = N(0,1) quantile table[u16]            (65,536 mid-point quantiles, float32)
    K only: 4 outlier channels per (layer, kv head) are multiplied by 8
    stored as binary16 (round to nearest even)

The paper's K/V came from trained models run over text; those are not available, so
these caches take only their shapes (layers, heads, head_dim, context lengths).
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

MASK64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15
TENSOR_Q, TENSOR_K, TENSOR_V = 1, 2, 3
BLOCK_TOKENS = 256


def _signed(x: int) -> int:
    x &= MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix64_int(x: int) -> int:
    x &= MASK64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & MASK64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & MASK64
    x ^= x >> 31
    return x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """logical shift right of int64 lanes"""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finalizer on int64 tensors (wrapping multiplies)."""
    x = x ^ _lsr(x, 30)
    x = x * _signed(0xBF58476D1CE4E5B9)
    x = x ^ _lsr(x, 27)
    x = x * _signed(0x94D049BB133111EB)
    x = x ^ _lsr(x, 31)
    return x


_TABLE = None


def normal_table() -> torch.Tensor:
    """65,536 mid-point quantiles of N(0,1) as float32, computed once on the CPU."""
    global _TABLE
    if _TABLE is None:
        u = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
        _TABLE = torch.special.ndtri(u).to(torch.float32)
    return _TABLE


_TABLE_DEV = {}


def _table_on(device) -> torch.Tensor:
    device = torch.device(device)
    if device.type == "cpu":
        return normal_table()
    key = str(device)
    if key not in _TABLE_DEV:
        _TABLE_DEV[key] = normal_table().to(device)
    return _TABLE_DEV[key]


def stream_key(seed: int, tensor: int, layer: int, agent: int) -> int:
    k = _mix64_int(seed * GAMMA + 0x1234567)
    k = _mix64_int(k ^ (tensor * 0xD6E8FEB86659FD93))
    k = _mix64_int(k + layer * GAMMA)
    k = _mix64_int(k ^ (agent * 0xCA5A826395121157))
    return k


def draw(seed: int, tensor: int, layer: int, agent: int, t0: int, t1: int, heads: int, dim: int,
         device="cpu", scale_channels: Optional[np.ndarray] = None, h0: int = 0, h1: Optional[int] = None,
         mult: float = 8.0) -> torch.Tensor:
    """binary16 values [t1-t0][h1-h0][dim] of the logical tensor (tensor, layer, agent) whose full
    shape is [tokens][heads][dim]; counter = (t*heads + h)*dim + d.
    scale_channels: int array [heads][n] of channel indices multiplied by `mult` (8 for the K outliers)."""
    h1 = heads if h1 is None else h1
    dev = torch.device(device)
    t = torch.arange(t0, t1, dtype=torch.int64, device=dev).view(-1, 1, 1)
    h = torch.arange(h0, h1, dtype=torch.int64, device=dev).view(1, -1, 1)
    d = torch.arange(dim, dtype=torch.int64, device=dev).view(1, 1, -1)
    counter = (t * heads + h) * dim + d
    key = _signed(stream_key(seed, tensor, layer, agent))
    bits = _mix64(counter * _signed(GAMMA) + key)
    idx = _lsr(bits, 48)
    x = _table_on(dev)[idx]
    if scale_channels is not None:
        mult_t = torch.ones(heads, dim, dtype=torch.float32)
        for hh in range(heads):
            mult_t[hh, torch.as_tensor(np.asarray(scale_channels[hh]), dtype=torch.int64)] = mult
        x = x * mult_t[h0:h1].to(dev).unsqueeze(0)
    return x.to(torch.float16)


def outlier_channels(seed: int, layers: int, kv_heads: int, dim: int, n: int = 4, tag: int = 0xC0FFEE) -> np.ndarray:
    """4 distinct channels per (layer, kv head), fixed across tokens and agents: int64 [layers][kv_heads][n]."""
    rng = np.random.default_rng([seed, tag])
    out = np.empty((layers, kv_heads, n), np.int64)
    for l in range(layers):
        for h in range(kv_heads):
            out[l, h] = np.sort(rng.choice(dim, size=n, replace=False))
    return out


@dataclass
class Workload:
    """One of the benchmark configurations: shapes of the paper's models, synthetic contents."""
    name: str
    seed: int
    num_layers: int
    num_q_heads: int
    num_kv_heads: int
    k_dim: int
    v_dim: int
    v_aliases_k: bool
    seq_lens: List[int]          # cached tokens per agent BEFORE any appended chunk
    q_len: int = 1               # 1 = decode, >1 = appended chunk length
    block_tokens: int = BLOCK_TOKENS
    outliers: np.ndarray = field(default=None, repr=False)
    wide_v: bool = False         # test shapes only: a quarter of the V channels is multiplied by 8 (group ranges of 20 to 45)
    v_outliers: np.ndarray = field(default=None, repr=False)
    v_mult: float = 8.0          # with wide_v: the factor, and the share of the V channels that gets it (1 / v_every)
    v_every: int = 4

    def __post_init__(self):
        if self.outliers is None:
            self.outliers = outlier_channels(self.seed, self.num_layers, self.num_kv_heads, self.k_dim)
        if self.wide_v and self.v_outliers is None:
            self.v_outliers = outlier_channels(self.seed, self.num_layers, self.num_kv_heads, self.v_dim,
                                               n=self.v_dim // self.v_every, tag=0xFACADE)

    @property
    def num_agents(self):
        return len(self.seq_lens)

    @property
    def sm_scale(self):
        return float(1.0 / np.sqrt(self.k_dim))

    @property
    def n_rep(self):
        return self.num_q_heads // self.num_kv_heads

    def final_lens(self):
        """keys visible to the last query row: cache plus appended chunk (decode: cache only)."""
        extra = self.q_len if self.q_len > 1 else 0
        return [n + extra for n in self.seq_lens]

    def k_rows(self, layer, agent, t0, t1, device="cpu", h0=0, h1=None):
        return draw(self.seed, TENSOR_K, layer, agent, t0, t1, self.num_kv_heads, self.k_dim, device,
                    self.outliers[layer], h0, h1)

    def v_rows(self, layer, agent, t0, t1, device="cpu", h0=0, h1=None):
        return draw(self.seed, TENSOR_V, layer, agent, t0, t1, self.num_kv_heads, self.v_dim, device,
                    self.v_outliers[layer] if self.wide_v else None, h0, h1, mult=self.v_mult)

    def q_rows(self, layer, agent, device="cpu"):
        """[q_len][q_heads][k_dim]"""
        return draw(self.seed, TENSOR_Q, layer, agent, 0, self.q_len, self.num_q_heads, self.k_dim, device)

    def q_all(self, device="cpu", layer_begin=0, layer_end=None):
        """[layers][A][q_len][q_heads][k_dim]"""
        layer_end = self.num_layers if layer_end is None else layer_end
        return torch.stack([torch.stack([self.q_rows(l, a, device) for a in range(self.num_agents)])
                            for l in range(layer_begin, layer_end)])

    def block_table(self):
        """Physical block ids shuffled over the whole pool: (int32 [A][max_blocks], num_blocks).
        Unused table entries hold -1."""
        bt = self.block_tokens
        need = [(n + bt - 1) // bt for n in self.final_lens()]
        total = max(1, sum(need))
        rng = np.random.default_rng([self.seed, 0xB10C])
        perm = rng.permutation(total).astype(np.int32)
        max_blocks = max(1, max(need) if need else 1)
        table = np.full((self.num_agents, max_blocks), -1, np.int32)
        pos = 0
        for a, nb in enumerate(need):
            table[a, :nb] = perm[pos:pos + nb]
            pos += nb
        return table, total

    def q4_bytes_per_token_layer(self):
        """algorithmic Q4 bytes read per cached token per layer: codes + scale + bias of the K and V rows."""
        if self.v_aliases_k:
            return self.num_kv_heads * (self.k_dim // 2 + 4 * (self.k_dim // 64))
        return self.num_kv_heads * ((self.k_dim + self.v_dim) // 2 + 4 * ((self.k_dim + self.v_dim) // 64))


def ragged_lengths(seed: int, agents: int, lo: int, hi: int) -> List[int]:
    rng = np.random.default_rng([seed, 0x1E46])
    return [int(x) for x in rng.integers(lo, hi + 1, size=agents)]


def config(i: int) -> Workload:
    """The five benchmark configurations (Llama-3.1-8B-, Gemma-3-12B-, DeepSeek-V2-Lite-shaped caches)."""
    if i == 0:
        return Workload("llama8b_1agent_1layer_1k_decode", 0, 1, 32, 8, 128, 128, False, [1024])
    if i == 1:
        return Workload("llama8b_5agents_32layers_4k_decode", 1, 32, 32, 8, 128, 128, False, [4096] * 5)
    if i == 2:
        return Workload("gemma12b_10agents_48layers_ragged_1k_8k_decode", 2, 48, 16, 8, 256, 256, False,
                        ragged_lengths(2, 10, 1024, 8192))
    if i == 3:
        return Workload("dsv2lite_mla_latent_5agents_27layers_32k_decode", 3, 27, 16, 1, 576, 512, True,
                        [32768] * 5)
    if i == 4:
        return Workload("gemma12b_10agents_48layers_ragged_4k_32k_append512", 4, 48, 16, 8, 256, 256, False,
                        ragged_lengths(4, 10, 4096, 32768), q_len=512)
    raise ValueError(i)


def per_head_mla_config() -> Workload:
    """The decompressed per-head form of the MLA cache (keys 192 = 128 + 64 rotary, values 128, one KV head per
    query head): 5 agents x 8,192 tokens x 27 layers, 3.2 GB of Q4."""
    return Workload("dsv2lite_mla_per_head_5agents_27layers_8k_decode", 5, 27, 16, 16, 192, 128, False, [8192] * 5)


def small(seed, num_layers, num_q_heads, num_kv_heads, k_dim, v_dim=None, v_aliases_k=False, seq_lens=(300,),
          q_len=1, name="small", wide_v=False, v_mult=8.0, v_every=4) -> Workload:
    return Workload(name, seed, num_layers, num_q_heads, num_kv_heads, k_dim, k_dim if v_dim is None else v_dim,
                    v_aliases_k, list(seq_lens), q_len, wide_v=wide_v, v_mult=v_mult, v_every=v_every)
