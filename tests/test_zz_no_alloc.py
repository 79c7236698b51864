"""qtale_layer_forward_static (the entry point that allocates nothing: its workspace is an array inside the
library) against qtale_layer_forward, through the C ABI: same kernels, so outputs, indices, counts, scores and
cache contents must be bit-identical.  Two calls in a row, the second with a smaller input, then a decode step
on a cache; the size limit is checked on the way."""
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qt():
    import paper_2602_10431_amd as pkg
    pkg.load_library()
    return pkg


def _both(qt, cfg, lw, ctx, x, offs, pos, make_kv=None):
    outs = []
    for static in (False, True):
        T = x.shape[0]
        xg = x.cuda()
        idx = torch.full((T,), -1, dtype=torch.int32, device="cuda")
        cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        sc = torch.zeros(T, dtype=torch.float32, device="cuda")
        kv = make_kv() if make_kv else None
        if static:
            before = torch.cuda.memory_allocated()
            qt.qtale_layer_forward_static(ctx, cfg, lw, xg, offs, pos, kv=kv, sel_idx=idx, sel_count=cnt, scores=sc)
            assert torch.cuda.memory_allocated() == before
        else:
            qt.qtale_layer_forward(ctx, cfg, lw, xg, offs, pos, kv=kv, sel_idx=idx, sel_count=cnt, scores=sc)
        torch.cuda.synchronize()
        outs.append((xg.cpu(), idx.cpu(), cnt.cpu(), sc.cpu(),
                     None if kv is None else (kv.k.cpu(), kv.v.cpu(), kv.kv_len.cpu())))
    a, b = outs
    k = int(a[2].item())
    assert k == int(b[2].item()) and k > 0
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16))
    assert torch.equal(a[1][:k], b[1][:k])
    assert torch.equal(a[3].view(torch.int32), b[3].view(torch.int32))
    if a[4] is not None:
        for u, v in zip(a[4], b[4]):
            assert torch.equal(u, v)
    return k


def test_static_scratch_layer_matches_workspace_layer(qt):
    shape = si.LayerShape(512, 4, 2, 128, 1376, 4, 128, "bf16")
    cfg = qt.cfg_from_shape(shape)
    lw = qt.quantize_layer(si.layer_tensors(shape, 0, 5, unit_gains=False, std=0.057), shape.bits, shape.group)
    ctx = qt.Context()
    assert qt.qtale_static_scratch_bytes() == 40 << 20
    # first call: 333 tokens in four ragged sequences, ratio mode
    qt.qtale_set_exec_ratio(ctx, 0.6)
    offs, pos = si.ragged_sequences([100, 1, 200, 32], [0, 5, 17, 1000])
    k1 = _both(qt, cfg, lw, ctx, si.hidden_states(shape, 333, 5), offs.cuda(), pos.cuda())
    assert k1 == 200
    # second call, smaller input, threshold mode: whatever the first call left in the array must not matter
    qt.qtale_set_threshold(ctx, 0.45)
    offs, pos = si.ragged_sequences([40, 30], [3, 0])
    _both(qt, cfg, lw, ctx, si.hidden_states(shape, 70, 6), offs.cuda(), pos.cuda())
    # third call: a decode step of 6 one-token sequences on a cache (split-key attention partials live in the array)
    qt.qtale_set_exec_ratio(ctx, 0.67)
    B, cap, ctx_len = 6, 1100, 1030
    g = torch.Generator().manual_seed(11)
    k0 = torch.randn(B, shape.n_kv_heads, cap, shape.head_dim, generator=g).to(torch.float16)
    v0 = torch.randn(B, shape.n_kv_heads, cap, shape.head_dim, generator=g).to(torch.float16)

    def make_kv():
        return qt.KVCache(k0.cuda(), v0.cuda(), torch.full((B,), ctx_len, dtype=torch.int32, device="cuda"))

    offs = torch.arange(B + 1, dtype=torch.int32)
    pos = torch.full((B,), ctx_len, dtype=torch.int32)
    assert _both(qt, cfg, lw, ctx, si.hidden_states(shape, B, 7), offs.cuda(), pos.cuda(), make_kv) == 4


def test_static_scratch_rejects_calls_beyond_its_size(qt):
    shape = si.C2
    cfg = qt.cfg_from_shape(shape)
    T = 4096
    assert qt.qtale_workspace_bytes(cfg, T, 1) > qt.qtale_static_scratch_bytes()
    lib = qt.load_library()
    ctx = qt.Context()
    x = torch.zeros(8, dtype=torch.int32, device="cuda")      # never touched: the size check comes first
    code = lib.qtale_layer_forward_static(ctx._h, qt.C.byref(cfg), None, x.data_ptr(), T, x.data_ptr(), 1, x.data_ptr(),
                                          None, None, None, None, None)
    assert code == -4
