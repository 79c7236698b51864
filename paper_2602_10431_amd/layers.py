"""Device-memory helpers: move one layer's fp32 weights to the GPU and quantize them with the library."""
import torch

from . import binding as B

_NAMES = ["q", "k", "v", "o", "gate", "up", "down"]


def cfg_from_shape(shape):
    """shape: any object with hidden, n_heads, n_kv_heads, head_dim, inter, bits, group, act_dtype, rms_eps, rope_base."""
    return B.make_cfg(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.inter, shape.bits,
                      shape.group, shape.act_dtype, shape.rms_eps, shape.rope_base)


def quantize_layer(tensors, bits=4, group=128, device="cuda", keep_canonical=True):
    """tensors: dict with fp32 CPU (or CUDA) weights 'q','k','v','o','gate','up','down' [N,K], 'router_w' [H]
    fp32, 'router_b' float, 'g1','g2' [H] in the activation dtype; optional 'router_mlp' = (W1, b1, W2, b2) fp32
    for the two-output MLP router.  Each weight is uploaded, quantized by qtale_quantize on the GPU and its fp32
    copy released."""
    lin = {}
    for name in _NAMES:
        W = tensors[name].to(device=device, dtype=torch.float32).contiguous()
        lin[name] = B.qtale_quantize(W, bits, group, keep_canonical)
        torch.cuda.current_stream().synchronize()
        del W
    return B.LayerWeights(lin["q"], lin["k"], lin["v"], lin["o"], lin["gate"], lin["up"], lin["down"],
                          tensors["g1"].to(device).contiguous(), tensors["g2"].to(device).contiguous(),
                          tensors["router_w"].to(device=device, dtype=torch.float32).contiguous(),
                          float(tensors.get("router_b", 0.0)),
                          None if tensors.get("router_mlp") is None else
                          tuple(t.to(device=device, dtype=torch.float32).contiguous() for t in tensors["router_mlp"]))
