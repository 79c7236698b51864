"""Pins for the oracle's token-adaptive layer (CPU only).

Eq. 1 (residual layer), Eq. 3 (bypassed tokens keep x), Eq. 9 (decision), App. B.2 (gather), and the
appendix FLOPs table.  The layer math is pinned by an independent per-token brute-force loop, by a
separately written dense layer, by torch's fp64 library attention, and by closed-form special cases."""
import math
import os

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import qtale_oracle as orc
from tests.helpers import TINY, TINY_GQA, cfg_dict, oracle_layer, to_f64

STD = 0.25          # tiny shapes need large weights for f(x) to be comparable with x


def _tiny(shape, T, seed, std=STD):
    t = si.layer_tensors(shape, 0, seed, unit_gains=False, std=std)
    p, _ = oracle_layer(shape, 0, seed, tensors=t)
    x = to_f64(si.hidden_states(shape, T, seed))
    return p, x


def test_ratio_one_equals_dense_layer_and_ratio_zero_is_identity():
    shape = TINY_GQA
    p, x = _tiny(shape, 11, 1)
    offs, pos = si.ragged_sequences([4, 7])
    out1, idx1, _ = orc.layer_forward(x, p, cfg_dict(shape), offs.numpy(), pos.numpy(), "ratio", 1.0)
    dense = orc.dense_layer_forward(x, p, cfg_dict(shape), offs.numpy(), pos.numpy())
    assert list(idx1) == list(range(11))
    np.testing.assert_allclose(out1, dense, rtol=1e-11, atol=1e-12)
    assert np.abs(dense - x).max() > 0.05                        # the layer really does something
    out0, idx0, _ = orc.layer_forward(x, p, cfg_dict(shape), offs.numpy(), pos.numpy(), "ratio", 0.0)
    assert len(idx0) == 0 and np.array_equal(out0, x)


def test_dense_layer_against_torch_library_ops():
    shape = TINY_GQA
    p, x = _tiny(shape, 9, 2)
    offs, pos = si.ragged_sequences([9], starts=[3])
    dense = orc.dense_layer_forward(x, p, cfg_dict(shape), offs.numpy(), pos.numpy())
    # third opinion: torch fp64, library attention
    nh, nkv, d = shape.n_heads, shape.n_kv_heads, shape.head_dim
    X = torch.from_numpy(x)
    T = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    n1 = X * torch.rsqrt(X.pow(2).mean(-1, keepdim=True) + shape.rms_eps) * T(p.g1)
    q = (n1 @ T(p.Wq).T).view(9, nh, d)
    k = (n1 @ T(p.Wk).T).view(9, nkv, d)
    v = (n1 @ T(p.Wv).T).view(9, nkv, d)
    inv = shape.rope_base ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.from_numpy(pos.numpy().astype(np.float64))[:, None] * inv[None]
    cos, sin = torch.cos(ang)[:, None], torch.sin(ang)[:, None]

    def rot(m):
        a, b = m[..., : d // 2], m[..., d // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], -1)

    q, k = rot(q), rot(k)
    k = k.repeat_interleave(nh // nkv, dim=1)
    v = v.repeat_interleave(nh // nkv, dim=1)
    att = torch.nn.functional.scaled_dot_product_attention(
        q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None], is_causal=True)[0]
    h1 = X + att.transpose(0, 1).reshape(9, nh * d) @ T(p.Wo).T
    n2 = h1 * torch.rsqrt(h1.pow(2).mean(-1, keepdim=True) + shape.rms_eps) * T(p.g2)
    y = h1 + (torch.nn.functional.silu(n2 @ T(p.Wg).T) * (n2 @ T(p.Wu).T)) @ T(p.Wd).T
    np.testing.assert_allclose(dense, y.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("shape", [TINY, TINY_GQA])
@pytest.mark.parametrize("mode,control", [("ratio", 0.5), ("ratio", 0.75), ("threshold", 0.4)])
def test_gather_form_equals_per_token_bruteforce(shape, mode, control):
    p, x = _tiny(shape, 12, 3)
    offs, pos = si.ragged_sequences([5, 3, 4], starts=[0, 2, 7])
    a, idx_a, _ = orc.layer_forward(x, p, cfg_dict(shape), offs.numpy(), pos.numpy(), mode, control)
    b, idx_b, _ = orc.layer_forward_bruteforce(x, p, cfg_dict(shape), offs.numpy(), pos.numpy(), mode, control)
    assert np.array_equal(idx_a, idx_b) and 0 < len(idx_a) < 12
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)
    skipped = np.setdiff1d(np.arange(12), idx_a)
    assert np.array_equal(a[skipped], x[skipped])                # Eq. 3: bit-identical bypass


def test_gather_form_equals_bruteforce_with_cache():
    shape = TINY_GQA
    p, x = _tiny(shape, 6, 4)
    offs, pos = si.ragged_sequences([2, 1, 3], starts=[3, 5, 1])
    kc, vc = si.kv_cache(shape, 3, 8, 0, 4)
    kv = orc.KVCache(to_f64(kc), to_f64(vc), [3, 5, 1])
    kv_b = orc.KVCache(to_f64(kc), to_f64(vc), [3, 5, 1])
    a, idx, _ = orc.layer_forward(x, p, cfg_dict(shape), offs.numpy(), pos.numpy(), "ratio", 0.67, kv)
    b, idx_b, app = orc.layer_forward_bruteforce(x, p, cfg_dict(shape), offs.numpy(), pos.numpy(), "ratio", 0.67, kv_b)
    assert np.array_equal(idx, idx_b) and len(idx) == 4
    np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12)
    for bb in range(3):                                          # appended rows, executed tokens only
        n_new = len(app[bb])
        assert kv.kv_len[bb] == [3, 5, 1][bb] + n_new
        for j, (kk, vv) in enumerate(app[bb]):
            np.testing.assert_allclose(kv.k[bb, [3, 5, 1][bb] + j], kk, rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(kv.v[bb, [3, 5, 1][bb] + j], vv, rtol=1e-11, atol=1e-13)
    assert sum(len(a_) for a_ in app) == 4


def test_prefill_then_decode_with_cache_equals_one_call():
    # sequence of 5 tokens at once  ==  4 tokens (filling the cache) then the 5th with the cache
    shape = TINY
    p, x = _tiny(shape, 5, 5)
    cfg = cfg_dict(shape)
    offs5, pos5 = si.ragged_sequences([5])
    forced = [0, 2, 3, 4]
    full, _, _ = orc.layer_forward(x, p, cfg, offs5.numpy(), pos5.numpy(), "forced", forced)
    w = shape.n_kv_heads * shape.head_dim
    kv = orc.KVCache(np.zeros((1, 8, w)), np.zeros((1, 8, w)), [0])
    offs4, pos4 = si.ragged_sequences([4])
    first, _, _ = orc.layer_forward(x[:4], p, cfg, offs4.numpy(), pos4.numpy(), "forced", [0, 2, 3], kv)
    assert kv.kv_len[0] == 3                                     # the skipped token appended nothing
    offs1, pos1 = si.ragged_sequences([1], starts=[4])
    last, _, _ = orc.layer_forward(x[4:], p, cfg, offs1.numpy(), pos1.numpy(), "forced", [0], kv)
    assert kv.kv_len[0] == 4
    np.testing.assert_allclose(np.concatenate([first, last]), full, rtol=1e-10, atol=1e-12)


def test_skipped_token_is_invisible_and_rope_uses_original_positions():
    shape = TINY
    p, x = _tiny(shape, 3, 6)
    cfg = cfg_dict(shape)
    e0, s, e1 = x[0], x[1], x[2]
    offsA, posA = si.ragged_sequences([2])
    offsB, posB = si.ragged_sequences([3])
    outA, _, _ = orc.layer_forward(np.stack([e0, e1]), p, cfg, offsA.numpy(), posA.numpy(), "forced", [0, 1])
    outB, _, _ = orc.layer_forward(np.stack([e0, s, e1]), p, cfg, offsB.numpy(), posB.numpy(), "forced", [0, 2])
    np.testing.assert_allclose(outA[0], outB[0], rtol=1e-12)     # first token sees only itself
    assert np.abs(outA[1] - outB[2]).max() > 1e-4                # distance 1 vs 2: rotary is relative
    outB2, _, _ = orc.layer_forward(np.stack([e0, 5 * s + 1, e1]), p, cfg, offsB.numpy(), posB.numpy(), "forced", [0, 2])
    assert np.array_equal(outB[[0, 2]], outB2[[0, 2]])           # the skipped token's content is invisible
    # shifting every position by the same amount changes nothing (relative encoding)
    outC, _, _ = orc.layer_forward(np.stack([e0, s, e1]), p, cfg, offsB.numpy(), posB.numpy() + 11, "forced", [0, 2])
    np.testing.assert_allclose(outB, outC, rtol=1e-9, atol=1e-11)


def test_single_executed_token_attends_to_itself_only():
    shape = TINY_GQA
    p, x = _tiny(shape, 4, 7)
    cfg = cfg_dict(shape)
    offs, pos = si.ragged_sequences([4])
    out, idx, _ = orc.layer_forward(x, p, cfg, offs.numpy(), pos.numpy(), "forced", [2])
    n1 = orc.rmsnorm(x[2], p.g1, shape.rms_eps)
    v = p.Wv @ n1
    rep = shape.n_heads // shape.n_kv_heads
    attn = np.concatenate([v[(h // rep) * shape.head_dim:(h // rep + 1) * shape.head_dim] for h in range(shape.n_heads)])
    h1 = x[2] + p.Wo @ attn
    n2 = orc.rmsnorm(h1, p.g2, shape.rms_eps)
    g = p.Wg @ n2
    y = h1 + p.Wd @ (g / (1 + np.exp(-g)) * (p.Wu @ n2))
    np.testing.assert_allclose(out[2], y, rtol=1e-11)
    assert np.array_equal(out[[0, 1, 3]], x[[0, 1, 3]])


def test_rope_properties():
    rng = np.random.default_rng(0)
    d = 8
    a, b = rng.standard_normal(2 * d), rng.standard_normal(2 * d)
    assert np.array_equal(orc.rope(a, 0, d, 10000.0), a)
    np.testing.assert_allclose(np.linalg.norm(orc.rope(a, 17, d, 10000.0)), np.linalg.norm(a))
    dots = [float(orc.rope(a, m + 5, d, 10000.0) @ orc.rope(b, m, d, 10000.0)) for m in (0, 3, 40)]
    np.testing.assert_allclose(dots, dots[0], rtol=1e-10)
    # element 0 pairs with element d/2, first frequency is 1 rad per position
    e = np.zeros(d)
    e[0] = 1.0
    r = orc.rope(e, 1, d, 10000.0)
    np.testing.assert_allclose([r[0], r[d // 2]], [math.cos(1.0), math.sin(1.0)])
    r = orc.rope(np.eye(d)[1], 1, d, 10000.0)
    np.testing.assert_allclose([r[1], r[1 + d // 2]], [math.cos(10000.0 ** (-2 / d)), math.sin(10000.0 ** (-2 / d))])


def test_rmsnorm_and_silu_closed_forms():
    g = np.array([1.0, 2.0, 0.5, 1.0])
    np.testing.assert_allclose(orc.rmsnorm(np.full(4, 3.0), g, 1e-5), 3.0 / math.sqrt(9.0 + 1e-5) * g)
    a = np.linspace(-4, 4, 9)
    np.testing.assert_allclose(orc.silu(a) - orc.silu(-a), a, atol=1e-14)
    assert orc.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(orc.silu(np.array([1.0]))[0], 1 / (1 + math.exp(-1)))


def test_stack_uses_one_control_for_all_layers_and_counts_match():
    shape = TINY
    layers = [oracle_layer(shape, l, 8, tensors=si.layer_tensors(shape, l, 8, False, STD))[0] for l in range(3)]
    x = to_f64(si.hidden_states(shape, 10, 8))
    offs, pos = si.ragged_sequences([6, 4])
    y, sel, inputs = orc.stack_forward(x, layers, cfg_dict(shape), offs.numpy(), pos.numpy(), "ratio", 0.4)
    assert [len(s) for s in sel] == [4, 4, 4]
    # layer by layer replay
    cur = x
    for l in range(3):
        assert np.array_equal(inputs[l], cur)
        cur, idx, _ = orc.layer_forward(cur, layers[l], cfg_dict(shape), offs.numpy(), pos.numpy(), "ratio", 0.4)
        assert np.array_equal(idx, sel[l])
    assert np.array_equal(cur, y)


def test_flops_per_token_matches_the_papers_table():
    path = os.path.join(os.path.dirname(__file__), "golden", "flops_per_token.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for name, H, nh, nkv, d, I, L, gflop in rows:
        got = orc.flops_per_token(int(H), int(nh), int(nkv), int(d), int(I), int(L)) / 1e9
        assert round(got, 1) == float(gflop), (name, got)


def test_parity_metric():
    want = np.array([[1.0, 0.0, -1.0, 0.0]])
    got = want + np.array([[0.01, 0.01, 0.0, 0.0]])
    rms = math.sqrt(0.5)
    np.testing.assert_allclose(orc.parity_error(got, want), 0.01 / rms)
