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


# ---- parity bar ----------------------------------------------------------------------------------------------
# Contract (hidden states, GEMM outputs): max |gpu - oracle| / max(|oracle|, rms(oracle row)) <= 2e-2.
# What the kernels deliver is below that: the final rounding to the output dtype alone gives up to 2^-8 (bf16) or
# 2^-11 (fp16), and the fp16 operands of the four GEMMs and of attention add their share (the maximum is taken over
# 1e5 to 1e8 elements).  A second, tighter bar at 1.5 to 2 times the largest error measured on the GPU (a full
# `pytest -m gpu` run with QTALE_PARITY_REPORT=<file> writes every measured error there) catches regressions the contract
# would let through.  Largest errors measured: single GEMM, fp16 out 3.9e-3; layers with hidden >= 1024: bf16 7.8e-3,
# fp16 3.7e-3; small layers (hidden 128-512, where one fp16 rounding is a larger share of a short dot product):
# bf16 1.04e-2, fp16 7.6e-3.
TOL = 2e-2
GUARD = {("bf16", "large"): 1.2e-2, ("fp16", "large"): 7e-3, ("bf16", "small"): 2e-2, ("fp16", "small"): 1.5e-2,
         ("fp16", "gemm"): 8e-3}
OBSERVED = []


def check_parity(err, out_dtype, what="", hidden=None):
    """err: orc.parity_error(...) of a GPU result; out_dtype: "fp16" | "bf16", the dtype the result was rounded to;
    hidden: the layer's hidden size (None for a single GEMM output or cache entries)."""
    size = "gemm" if hidden is None else ("large" if hidden >= 1024 else "small")
    OBSERVED.append((what, out_dtype, float(err)))
    assert err <= TOL, (what, err)
    assert err <= GUARD[(out_dtype, size)], ("regression guard (contract is %g)" % TOL, what, out_dtype, size, err)
