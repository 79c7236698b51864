"""Edge and degenerate cases of the layer on the GPU (run with -m gpu): empty calls, empty sequences, nobody
or everybody executing (by ratio and by threshold, i.e. with the count known on the host or only on the
device), single tokens, many one-token sequences, first decode step on empty caches."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import qtale_oracle as orc
from tests.helpers import cfg_dict, check_parity, oracle_layer, to_f64

pytestmark = pytest.mark.gpu
SHAPE = si.LayerShape(256, 4, 2, 64, 688, 4, 32, "fp16")


@pytest.fixture(scope="module")
def qt():
    import paper_2602_10431_amd as pkg
    pkg.load_library()
    return pkg


@pytest.fixture(scope="module")
def layer(qt):
    tensors = si.layer_tensors(SHAPE, 0, 50, unit_gains=False, std=0.08)
    return tensors, qt.quantize_layer(tensors, SHAPE.bits, SHAPE.group), oracle_layer(SHAPE, 0, 50, tensors=tensors)[0]


def _run(qt, lw, x, offs, pos, mode, val, kv=None):
    ctx = qt.Context()
    (qt.qtale_set_exec_ratio if mode == "ratio" else qt.qtale_set_threshold)(ctx, val)
    T = x.shape[0]
    xg = x.cuda()
    idx = torch.full((max(T, 1),), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    qt.qtale_layer_forward(ctx, qt.cfg_from_shape(SHAPE), lw, xg, offs.cuda(), pos.cuda(), kv=kv, sel_idx=idx, sel_count=cnt)
    torch.cuda.synchronize()
    return xg.cpu(), idx.cpu().numpy(), int(cnt.item())


def _check(qt, layer, T, lens, mode, val, starts=None, seed=51):
    tensors, lw, p = layer
    x = si.hidden_states(SHAPE, T, seed)
    offs, pos = si.ragged_sequences(lens, starts)
    got, idx, k = _run(qt, lw, x, offs, pos, mode, val)
    want, widx, _ = orc.layer_forward(to_f64(x), p, cfg_dict(SHAPE), offs.numpy(), pos.numpy(), mode, val)
    assert k == len(widx) and np.array_equal(idx[:k], widx)
    skipped = np.setdiff1d(np.arange(T), widx)
    assert torch.equal(got[skipped], x[skipped])
    if k:
        check_parity(orc.parity_error(to_f64(got)[widx], want[widx]), SHAPE.act_dtype, "edge layer", hidden=SHAPE.hidden)
    return k


def test_empty_call_is_a_no_op(qt, layer):
    _, lw, _ = layer
    ctx = qt.Context()
    x = torch.empty((0, SHAPE.hidden), dtype=torch.float16, device="cuda")
    offs = torch.zeros(1, dtype=torch.int32, device="cuda")
    pos = torch.empty(0, dtype=torch.int32, device="cuda")
    qt.qtale_layer_forward(ctx, qt.cfg_from_shape(SHAPE), lw, x, offs, pos)
    torch.cuda.synchronize()


@pytest.mark.parametrize("mode,val,expect", [("ratio", 0.0, 0), ("threshold", 1.0, 0), ("threshold", 0.999999, None),
                                             ("ratio", 1.0, 90), ("threshold", 0.0, 90), ("threshold", 1e-6, None)])
def test_nobody_and_everybody(qt, layer, mode, val, expect):
    # threshold mode decides on the device: an executed count of 0 must flow through every kernel
    k = _check(qt, layer, 90, [50, 40], mode, val)
    if expect is not None:
        assert k == expect


def test_single_token_call(qt, layer):
    assert _check(qt, layer, 1, [1], "ratio", 1.0, starts=[17]) == 1
    assert _check(qt, layer, 1, [1], "ratio", 0.4) == 0


def test_empty_sequences_between_real_ones(qt, layer):
    _check(qt, layer, 70, [0, 30, 0, 0, 40, 0], "ratio", 0.5, starts=[0, 3, 9, 0, 100, 5])


def test_many_one_token_sequences_without_cache(qt, layer):
    # every executed token attends to itself only
    _check(qt, layer, 150, [1] * 150, "ratio", 0.7, starts=list(range(150)))


def test_one_executed_token_per_sequence_by_threshold(qt, layer):
    _check(qt, layer, 257, [129, 128], "threshold", 0.5)


def test_sizes_around_tile_boundaries(qt, layer):
    for T in (63, 64, 65, 127, 128, 129, 255, 257):
        _check(qt, layer, T, [T], "ratio", 1.0, seed=60 + T)


def test_first_decode_step_on_empty_caches(qt, layer):
    tensors, lw, p = layer
    B, cap = 5, 8
    x = si.hidden_states(SHAPE, B, 52)
    offs, pos = si.ragged_sequences([1] * B, starts=[0] * B)
    kc, vc = si.kv_cache(SHAPE, B, cap, 0, 52)
    kv = qt.KVCache.from_token_major(kc.cuda(), vc.cuda(), torch.zeros(B, dtype=torch.int32).cuda(), SHAPE.n_kv_heads)
    got, idx, k = _run(qt, lw, x, offs, pos, "ratio", 0.6, kv=kv)
    okv = orc.KVCache(to_f64(kc), to_f64(vc), [0] * B)
    want, widx, _ = orc.layer_forward(to_f64(x), p, cfg_dict(SHAPE), offs.numpy(), pos.numpy(), "ratio", 0.6, okv)
    assert k == 3 and np.array_equal(idx[:k], widx)
    check_parity(orc.parity_error(to_f64(got)[widx], want[widx]), SHAPE.act_dtype, "first decode step", hidden=SHAPE.hidden)
    assert np.array_equal(kv.kv_len.cpu().numpy(), okv.kv_len)
    assert sorted(kv.kv_len.cpu().tolist()) == [0, 0, 1, 1, 1]


def test_cache_exactly_full_after_the_call(qt, layer):
    tensors, lw, p = layer
    lens, old, cap = [4, 2], [4, 6], 8                            # both sequences end at kv_len == cap if all execute
    x = si.hidden_states(SHAPE, 6, 53)
    offs, pos = si.ragged_sequences(lens, starts=old)
    kc, vc = si.kv_cache(SHAPE, 2, cap, 0, 53)
    kv = qt.KVCache.from_token_major(kc.cuda(), vc.cuda(), torch.tensor(old, dtype=torch.int32).cuda(), SHAPE.n_kv_heads)
    got, idx, k = _run(qt, lw, x, offs, pos, "ratio", 1.0, kv=kv)
    okv = orc.KVCache(to_f64(kc), to_f64(vc), old)
    want, widx, _ = orc.layer_forward(to_f64(x), p, cfg_dict(SHAPE), offs.numpy(), pos.numpy(), "ratio", 1.0, okv)
    assert k == 6 and kv.kv_len.cpu().tolist() == [8, 8]
    check_parity(orc.parity_error(to_f64(got), want), SHAPE.act_dtype, "cache exactly full", hidden=SHAPE.hidden)
