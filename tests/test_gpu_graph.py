"""HIP graph of a stack forward (run with -m gpu): replays must reproduce the eager calls bit for bit,
step after step of a decode loop, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qt():
    import paper_2602_10431_amd as pkg
    pkg.load_library()
    return pkg


def _decode_setup(qt, shape, L, B, cap, seed, old_lens):
    tensors = [si.layer_tensors(shape, l, seed, unit_gains=False, std=1.28 / shape.hidden ** 0.5) for l in range(L)]
    layers = [qt.quantize_layer(t, shape.bits, shape.group) for t in tensors]
    caches = [si.kv_cache(shape, B, cap, l, seed) for l in range(L)]

    def fresh_stack():
        kvs = [qt.KVCache.from_token_major(k.cuda(), v.cuda(), torch.tensor(old_lens, dtype=torch.int32).cuda(), shape.n_kv_heads)
               for k, v in caches]
        return qt.Stack(qt.cfg_from_shape(shape), layers, kvs), kvs

    return fresh_stack


@pytest.mark.parametrize("mode,val", [("ratio", 0.6), ("threshold", 0.45)])
def test_graph_replays_match_eager_decode_steps(qt, mode, val):
    shape = si.LayerShape(256, 4, 2, 64, 688, 4, 32, "fp16")
    L, B, cap, seed, steps = 3, 6, 64, 41, 4
    old = [37, 5, 20, 48, 1, 30]
    fresh_stack = _decode_setup(qt, shape, L, B, cap, seed, old)
    offs = torch.arange(0, B + 1, dtype=torch.int32).cuda()
    xs = [si.hidden_states(shape, B, seed, slot="x_step", extra=i) for i in range(steps)]
    ctx = qt.Context()
    (qt.qtale_set_exec_ratio if mode == "ratio" else qt.qtale_set_threshold)(ctx, val)

    # eager reference
    stack, kvs = fresh_stack()
    want, want_cnt = [], []
    for i in range(steps):
        x = xs[i].cuda()
        pos = (torch.tensor(old, dtype=torch.int32) + i).cuda()
        cnt = torch.zeros(L, dtype=torch.int32, device="cuda")
        qt.qtale_stack_forward(ctx, stack, x, offs, pos, sel_count=cnt)
        torch.cuda.synchronize()
        want.append(x.cpu())
        want_cnt.append(cnt.cpu())
    want_len = [kv.kv_len.cpu() for kv in kvs]
    want_k = [kv.k.cpu() for kv in kvs]

    # graph: fixed buffers, rewritten in place between replays
    stack2, kvs2 = fresh_stack()
    x_buf = torch.zeros_like(xs[0]).cuda()
    pos_buf = torch.zeros(B, dtype=torch.int32, device="cuda")
    cnt_buf = torch.zeros(L, dtype=torch.int32, device="cuda")
    graph = qt.StackGraph(ctx, stack2, x_buf, offs, pos_buf, sel_count=cnt_buf)
    torch.cuda.synchronize()
    assert torch.equal(x_buf.cpu(), torch.zeros_like(xs[0]))      # capture executes nothing
    assert all(torch.equal(kv.kv_len.cpu(), torch.tensor(old, dtype=torch.int32)) for kv in kvs2)
    for i in range(steps):
        x_buf.copy_(xs[i])
        pos_buf.copy_(torch.tensor(old, dtype=torch.int32) + i)
        graph.launch()
        noise = float(torch.randn(4096, device="cuda").square().sum().item())   # eager work + sync between replays
        assert noise > 0
        assert torch.equal(x_buf.cpu(), want[i]), i
        assert torch.equal(cnt_buf.cpu(), want_cnt[i]), i
    for l in range(L):
        assert torch.equal(kvs2[l].kv_len.cpu(), want_len[l])
        assert torch.equal(kvs2[l].k.cpu(), want_k[l])


def test_graph_prefill_replay_and_rejections(qt):
    shape = si.C1
    L, T = 2, 160
    layers = [qt.quantize_layer(si.layer_tensors(shape, l, 42), shape.bits, shape.group) for l in range(L)]
    stack = qt.Stack(qt.cfg_from_shape(shape), layers)
    offs, pos = si.ragged_sequences([100, 60])
    offs, pos = offs.cuda(), pos.cuda()
    ctx = qt.Context()
    qt.qtale_set_exec_ratio(ctx, 0.5)
    x = si.hidden_states(shape, T, 42)
    ref = x.cuda()
    qt.qtale_stack_forward(ctx, stack, ref, offs, pos)
    buf = torch.empty_like(ref)
    graph = qt.StackGraph(ctx, stack, buf, offs, pos)
    for _ in range(3):
        buf.copy_(x)
        graph.launch()
        torch.cuda.synchronize()
        assert torch.equal(buf, ref)
    qt.qtale_profile_enable(ctx, True)                            # event spans cannot go into a graph
    with pytest.raises(qt.QtaleError):
        qt.StackGraph(ctx, stack, buf, offs, pos)
    qt.qtale_profile_enable(ctx, False)
