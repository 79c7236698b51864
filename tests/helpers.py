"""Test-side glue: builds oracle inputs from the seeded generators.  Holds no kernel or oracle arithmetic."""
import numpy as np
import torch

import synth_inputs as si
from oracle import qtale_oracle as orc


def to_f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def cfg_dict(shape):
    return dict(n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                rms_eps=shape.rms_eps, rope_base=shape.rope_base)


def oracle_layer(shape, layer, seed, unit_gains=False, router_b=0.0, tensors=None):
    """Quantize the seeded fp32 weights with the oracle's quantizer and return
    (LayerParams with dequantized fp64 weights, dict name -> (codes, scales, zeros))."""
    t = tensors if tensors is not None else si.layer_tensors(shape, layer, seed, unit_gains)
    deq, q = {}, {}
    for name, _, _ in shape.linear_shapes():
        codes, s, z = orc.quantize_rtn(t[name].numpy(), shape.bits, shape.group)
        q[name] = (codes, s, z)
        deq[name] = orc.dequantize(codes, s, z, shape.group)
    p = orc.LayerParams(deq["q"], deq["k"], deq["v"], deq["o"], deq["gate"], deq["up"], deq["down"],
                        to_f64(t["g1"]), to_f64(t["g2"]), t["router_w"].numpy(), router_b)
    return p, q


def round_like(x64, dtype_name):
    """Round fp64 values to the 16-bit activation dtype and back."""
    return torch.from_numpy(np.asarray(x64)).to(si.torch_dtype(dtype_name)).to(torch.float64).numpy()


TINY = si.LayerShape(hidden=16, n_heads=2, n_kv_heads=2, head_dim=8, inter=24, bits=4, group=8, act_dtype="fp16")
TINY_GQA = si.LayerShape(hidden=16, n_heads=4, n_kv_heads=2, head_dim=4, inter=20, bits=4, group=8, act_dtype="bf16")
