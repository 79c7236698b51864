"""Seeded synthetic inputs for the QTALE inference hot path.

This module only draws random numbers and lays them out; it contains none of
the method's arithmetic (no quantizer, no router, no layer math).  Both the
CPU oracle's tests and the GPU harness take their inputs from here so that the
two sides see identical bits.

Every tensor is drawn from its own generator seeded by (seed, layer, slot), so
any single tensor can be regenerated without generating the ones before it.

Recipe (LLaMA-shaped stand-ins for the paper's fine-tuned checkpoints, which
are not available): linear weights ~ N(0, 0.02) fp32, router weight
~ N(0, 0.02) fp32 with zero bias, hidden states ~ N(0, 1) rounded to the
activation dtype, RMSNorm gains 1 (benchmarks) or 1 + N(0, 0.02) (tests),
K/V cache entries ~ N(0, 1) rounded to fp16.
"""
from dataclasses import dataclass, asdict

import torch


@dataclass(frozen=True)
class LayerShape:
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    inter: int
    bits: int = 4
    group: int = 128
    act_dtype: str = "bf16"          # "fp16" or "bf16": dtype of the residual stream
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    def linear_shapes(self):
        """(name, N, K) of the seven linears of one decoder layer, in slot order."""
        H, d = self.hidden, self.head_dim
        return [("q", self.n_heads * d, H), ("k", self.n_kv_heads * d, H),
                ("v", self.n_kv_heads * d, H), ("o", H, self.n_heads * d),
                ("gate", self.inter, H), ("up", self.inter, H),
                ("down", H, self.inter)]

    def params_per_layer(self):
        return sum(n * k for _, n, k in self.linear_shapes())

    def asdict(self):
        return asdict(self)


# The shapes of the five workload configurations.
C1 = LayerShape(256, 4, 4, 64, 688, 4, 32, "fp16")
C2 = LayerShape(4096, 32, 32, 128, 11008, 4, 128, "bf16")      # LLaMA-7B-shaped
C4 = LayerShape(4096, 32, 8, 128, 14336, 4, 128, "bf16")       # LLaMA-3-8B-shaped (GQA)
C5 = LayerShape(5120, 40, 40, 128, 13824, 4, 128, "bf16")      # LLaMA-13B-shaped

_SLOTS = {"q": 0, "k": 1, "v": 2, "o": 3, "gate": 4, "up": 5, "down": 6,
          "router_w": 7, "g1": 8, "g2": 9, "x": 10, "k_cache": 11, "v_cache": 12,
          "x_step": 13, "misc": 14, "router_w1": 15, "router_b1": 16, "router_w2": 17, "router_b2": 18}


def _gen(seed, layer, slot, extra=0, device="cpu"):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(layer) * 1009 + _SLOTS[slot] * 17 + int(extra) * 7919) % (2 ** 62))
    return g


def torch_dtype(name):
    return {"fp16": torch.float16, "bf16": torch.bfloat16}[name]


def linear_weight(shape: LayerShape, name, layer, seed, std=0.02, device="cpu"):
    """fp32 [N, K] weight of one linear, N(0, std).  device="cuda" draws on the GPU (same
    distribution, different bits than the CPU generator); parity tests always use the CPU."""
    for nm, n, k in shape.linear_shapes():
        if nm == name:
            return torch.randn(n, k, generator=_gen(seed, layer, name, device=device), dtype=torch.float32,
                               device=device) * std
    raise KeyError(name)


def router_weight(shape: LayerShape, layer, seed, std=0.02, device="cpu"):
    return torch.randn(shape.hidden, generator=_gen(seed, layer, "router_w", device=device), dtype=torch.float32,
                       device=device) * std


def router_mlp(shape: LayerShape, layer, seed, R=16, std1=0.02, std2=0.25, device="cpu"):
    """Parameters (W1 [R,H], b1 [R], W2 [2,R], b2 [2]) of a two-output MLP router, all fp32 random draws.  With the
    default spreads and N(0,1) inputs the execute-minus-bypass logit is of order 1 at H=4096."""
    g = lambda slot: _gen(seed, layer, slot, device=device)
    W1 = torch.randn(R, shape.hidden, generator=g("router_w1"), dtype=torch.float32, device=device) * std1
    b1 = torch.randn(R, generator=g("router_b1"), dtype=torch.float32, device=device) * std1
    W2 = torch.randn(2, R, generator=g("router_w2"), dtype=torch.float32, device=device) * std2
    b2 = torch.randn(2, generator=g("router_b2"), dtype=torch.float32, device=device) * std1
    return W1, b1, W2, b2


def norm_gains(shape: LayerShape, layer, seed, unit=True):
    """RMSNorm gains in the activation dtype: all ones, or 1 + N(0, 0.02) when unit=False."""
    dt = torch_dtype(shape.act_dtype)
    if unit:
        return torch.ones(shape.hidden, dtype=dt), torch.ones(shape.hidden, dtype=dt)
    g1 = 1.0 + 0.02 * torch.randn(shape.hidden, generator=_gen(seed, layer, "g1"))
    g2 = 1.0 + 0.02 * torch.randn(shape.hidden, generator=_gen(seed, layer, "g2"))
    return g1.to(dt), g2.to(dt)


def layer_tensors(shape: LayerShape, layer, seed, unit_gains=True, std=0.02, device="cpu"):
    """All fp32 weights of one layer plus router and gains, as a dict."""
    out = {nm: linear_weight(shape, nm, layer, seed, std, device) for nm, _, _ in shape.linear_shapes()}
    out["router_w"] = router_weight(shape, layer, seed, std, device)
    out["router_b"] = 0.0
    out["g1"], out["g2"] = norm_gains(shape, layer, seed, unit_gains)
    return out


def hidden_states(shape: LayerShape, T, seed, slot="x", extra=0, device="cpu"):
    """[T, hidden] ~ N(0,1) rounded to the activation dtype."""
    x = torch.randn(T, shape.hidden, generator=_gen(seed, 0, slot, extra, device), dtype=torch.float32, device=device)
    return x.to(torch_dtype(shape.act_dtype))


def kv_cache(shape: LayerShape, B, cap, layer, seed):
    """Two fp16 tensors [B, cap, n_kv*head_dim] ~ N(0,1)."""
    w = shape.n_kv_heads * shape.head_dim
    k = torch.randn(B, cap, w, generator=_gen(seed, layer, "k_cache"), dtype=torch.float32).to(torch.float16)
    v = torch.randn(B, cap, w, generator=_gen(seed, layer, "v_cache"), dtype=torch.float32).to(torch.float16)
    return k, v


def equal_sequences(B, S):
    """seq_offsets [B+1] and positions [B*S] for B sequences of S tokens starting at position 0."""
    offs = torch.arange(0, (B + 1) * S, S, dtype=torch.int32)
    pos = torch.arange(S, dtype=torch.int32).repeat(B)
    return offs, pos


def ragged_sequences(lengths, starts=None):
    """seq_offsets and positions for sequences of the given lengths; starts[b] is the
    absolute position of the first token of sequence b (default 0)."""
    offs = [0]
    pos = []
    for b, n in enumerate(lengths):
        offs.append(offs[-1] + int(n))
        s0 = 0 if starts is None else int(starts[b])
        pos.extend(range(s0, s0 + int(n)))
    return torch.tensor(offs, dtype=torch.int32), torch.tensor(pos, dtype=torch.int32)
