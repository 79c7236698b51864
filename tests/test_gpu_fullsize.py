"""Full-size parity (run with -m gpu): the LLaMA-shaped workloads in the launch configuration bench.py times.

* one layer of every prefill workload: router scores and the executed set over ALL tokens of the call bit-exact,
  EVERY executed row of every sequence against the oracle (contract 2e-2, plus the regression guard of
  tests/helpers.py), bypassed rows bit-identical to the input, packed codes of one full-size matrix bit-exact;
* the 32-layer 7B stack call that bench.py times, teacher-forced: scores and selections of all 32 layers bit-exact
  on the GPU's own layer inputs, three layers through the oracle on all their executed rows;
* decode steps at full size: selections, cache lengths, sampled sequences through the oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import qtale_oracle as orc
from tests.helpers import cfg_dict, check_parity, oracle_layer, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qt():
    import paper_2602_10431_amd as pkg
    pkg.load_library()
    return pkg


def _prefill_case(qt, shape, B, S, ratio, seed, threshold=None):
    T = B * S
    tensors = si.layer_tensors(shape, 0, seed, unit_gains=True)
    x = si.hidden_states(shape, T, seed)
    offs, pos = si.equal_sequences(B, S)
    cfg = qt.cfg_from_shape(shape)
    lw = qt.quantize_layer(tensors, shape.bits, shape.group)
    ctx = qt.Context()
    if threshold is None:
        qt.qtale_set_exec_ratio(ctx, ratio)
    else:
        qt.qtale_set_threshold(ctx, threshold)                   # count known on the device only
    xg = x.cuda()
    idx = torch.full((T,), -1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    z = torch.empty(T, dtype=torch.float32, device="cuda")
    qt.qtale_layer_forward(ctx, cfg, lw, xg, offs.cuda(), pos.cuda(), sel_idx=idx, sel_count=cnt, scores=z)
    torch.cuda.synchronize()
    # selection over the whole call
    z_ref = orc.router_scores(to_f64(x), tensors["router_w"].numpy(), 0.0)
    assert np.array_equal(z.cpu().numpy().view(np.uint32), z_ref.view(np.uint32))
    want_idx = orc.select_ratio(z_ref, ratio) if threshold is None else orc.select_threshold(z_ref, threshold)
    k = int(cnt.item())
    assert k == len(want_idx)
    if threshold is None:
        assert k == orc.executed_count(ratio, T)
    got_idx = idx[:k].cpu().numpy()
    assert np.array_equal(got_idx, want_idx)
    # bypassed rows untouched everywhere
    got = xg.cpu()
    skipped = np.setdiff1d(np.arange(T), want_idx)
    assert torch.equal(got[skipped], x[skipped])
    # every executed row of every sequence through the oracle (the executed set is the one just checked)
    p, q = oracle_layer(shape, 0, seed, tensors=tensors)
    want, _, _ = orc.layer_forward(to_f64(x), p, cfg_dict(shape), offs.numpy(), pos.numpy(), "forced", want_idx)
    err = orc.parity_error(to_f64(got)[want_idx], want[want_idx])
    check_parity(err, shape.act_dtype, ("full-size prefill layer", shape.hidden, shape.bits, B, S, ratio, threshold), hidden=shape.hidden)
    # codes of the largest matrix
    codes = q["down"][0]
    assert np.array_equal(lw.lin["down"].codes.cpu().numpy().view(np.uint32), orc.pack_codes(codes, shape.bits))
    return err


def test_llama7b_shaped_prefill_layer_8x1024_bf16_ratio_half(qt):
    _prefill_case(qt, si.C2, 8, 1024, 0.5, seed=11)


def test_llama7b_shaped_prefill_layer_threshold_mode(qt):
    # Eq. 9 verbatim at full size: about 62 % of the 8192 tokens execute at theta = 0.4 with these scores; the
    # GEMM grids cover all 8192 rows and the workgroups beyond the live tiles leave at once
    _prefill_case(qt, si.C2, 8, 1024, None, seed=14, threshold=0.4)


@pytest.mark.parametrize("rows", [4115, 4196])
def test_llama7b_shaped_prefill_layer_rows_beyond_the_last_full_tile(qt, rows):
    # 4115 executed rows = 32 full 128-row tiles + 19 rows, 4196 = 32 tiles + 100 rows: the linears whose 33rd row of
    # tiles would start another round of workgroups on a 256-CU chip (q|k|v, o-proj with its residual, down-proj with
    # residual + scatter) hand those rows to the small-row kernels, as one chunk or as two 64-row chunks; gate/up keeps
    # its 33rd tile row
    ratio = rows / 8192
    assert orc.executed_count(ratio, 8192) == rows
    _prefill_case(qt, si.C2, 8, 1024, ratio, seed=18)


def test_llama7b_shaped_prefill_layer_threshold_mode_split_decided_on_device(qt):
    # threshold mode with a count that leaves 1..64 rows beyond the last full 128-row tile: the count exists on the
    # device only, so both the tiled launch and the small-row launch take the split decision from it
    shape, T, seed = si.C2, 8192, 19
    x = si.hidden_states(shape, T, seed)
    z = orc.router_scores(to_f64(x), si.layer_tensors(shape, 0, seed, unit_gains=True)["router_w"].numpy(), 0.0)
    theta = next(th for th in (0.40 + 0.0005 * i for i in range(400))
                 if 1 <= len(orc.select_threshold(z, th)) % 128 <= 64 and len(orc.select_threshold(z, th)) > 2000)
    _prefill_case(qt, shape, 8, 1024, None, seed=seed, threshold=theta)


def test_llama7b_shaped_prefill_layer_three_bit(qt):
    import dataclasses
    _prefill_case(qt, dataclasses.replace(si.C2, bits=3), 8, 1024, 0.5, seed=15)


def test_llama7b_shaped_stack_32_layers_8x1024_teacher_forced(qt):
    # the call bench.py times: qtale_stack_forward over 32 layers, prefill 8 x 1024, bf16, ratio 0.5.  Every layer is
    # judged on the GPU's own input to it (dbg_hidden): scores and selections of all 32 layers bit-exact, bypassed rows
    # bit-identical across every layer, and layers 0, 13 and 31 through the oracle on all their executed rows.
    shape, L, B, S, ratio, seed = si.C2, 32, 8, 1024, 0.5, 21
    T = B * S
    checked = (0, 13, 31)
    layers, router_w, kept = [], [], {}
    for l in range(L):
        t = si.layer_tensors(shape, l, seed, device="cuda")      # drawn on the GPU (fast); the oracle gets the same bits
        layers.append(qt.quantize_layer(t, shape.bits, shape.group, keep_canonical=False))
        router_w.append(t["router_w"].cpu().numpy())
        if l in checked:
            kept[l] = {k: (v.cpu() if torch.is_tensor(v) else v) for k, v in t.items()}
        del t
    x = si.hidden_states(shape, T, seed)
    offs, pos = si.equal_sequences(B, S)
    stack = qt.Stack(qt.cfg_from_shape(shape), layers)
    ctx = qt.Context()
    qt.qtale_set_exec_ratio(ctx, ratio)
    xg = x.cuda()
    idx = torch.full((L, T), -1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(L, dtype=torch.int32, device="cuda")
    z = torch.empty((L, T), dtype=torch.float32, device="cuda")
    dbg = torch.empty((L, T, shape.hidden), dtype=x.dtype, device="cuda")
    qt.qtale_stack_forward(ctx, stack, xg, offs.cuda(), pos.cuda(), sel_idx=idx, sel_count=cnt, scores=z, dbg_hidden=dbg)
    torch.cuda.synchronize()
    assert torch.equal(dbg[0].cpu(), x)
    k_want = orc.executed_count(ratio, T)
    counts = cnt.cpu().numpy()
    for l in range(L):
        xin = dbg[l].cpu()
        xout = (dbg[l + 1] if l + 1 < L else xg).cpu()
        z_ref = orc.router_scores(to_f64(xin), router_w[l], 0.0)
        assert np.array_equal(z[l].cpu().numpy().view(np.uint32), z_ref.view(np.uint32)), l
        widx = orc.select_ratio(z_ref, ratio)
        assert counts[l] == k_want == len(widx), l
        assert np.array_equal(idx[l, :k_want].cpu().numpy(), widx), l
        skipped = np.setdiff1d(np.arange(T), widx)
        assert torch.equal(xout[skipped], xin[skipped]), l
        if l in checked:
            p, _ = oracle_layer(shape, l, seed, tensors=kept[l])
            want, _, _ = orc.layer_forward(to_f64(xin), p, cfg_dict(shape), offs.numpy(), pos.numpy(), "forced", widx)
            check_parity(orc.parity_error(to_f64(xout)[widx], want[widx]), shape.act_dtype, ("7B stack, layer", l), hidden=shape.hidden)


@pytest.mark.parametrize("ratio,threshold", [(0.5, None), (None, 0.4)])
def test_llama7b_shaped_single_prompt_1x1024(qt, ratio, threshold):
    # one 1024-token prompt: 512 (ratio) or about 640 (threshold) executed rows, the row counts at which the
    # 4096-column linears run on 64-row tiles
    _prefill_case(qt, si.C2, 1, 1024, ratio, seed=16, threshold=threshold)


def test_llama3_8b_shaped_gqa_prefill_layer_4x4096_ratio_06(qt):
    _prefill_case(qt, si.C4, 4, 4096, 0.6, seed=12)


@pytest.mark.parametrize("B,ratios", [(64, [(1.0, 64), (0.8, 51), (0.6, 38), (0.4, 26)]),
                                      (8, [(1.0, 8), (0.5, 4)])])     # 8 rows: decode attention splits the keys
def test_llama7b_shaped_decode_step_ctx2048(qt, B, ratios):
    shape = si.LayerShape(4096, 32, 32, 128, 11008, 4, 128, "fp16")
    ctx_len, cap, seed = 2048, 2048 + 8, 13
    tensors = si.layer_tensors(shape, 0, seed, unit_gains=True)
    x = si.hidden_states(shape, B, seed)
    offs, pos = si.ragged_sequences([1] * B, starts=[ctx_len] * B)
    kc, vc = si.kv_cache(shape, B, cap, 0, seed)
    cfg = qt.cfg_from_shape(shape)
    lw = qt.quantize_layer(tensors, shape.bits, shape.group)
    p, _ = oracle_layer(shape, 0, seed, tensors=tensors)
    z_ref = orc.router_scores(to_f64(x), tensors["router_w"].numpy(), 0.0)
    ctx = qt.Context()
    check = [0, 17, 40, 63] if B == 64 else [0, 3, 7]
    for ratio, k_want in ratios:
        qt.qtale_set_exec_ratio(ctx, ratio)                      # runtime change, weights untouched
        kv = qt.KVCache.from_token_major(kc.cuda(), vc.cuda(), torch.full((B,), ctx_len, dtype=torch.int32).cuda(), shape.n_kv_heads)
        xg = x.cuda()
        idx = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        qt.qtale_layer_forward(ctx, cfg, lw, xg, offs.cuda(), pos.cuda(), kv=kv, sel_idx=idx, sel_count=cnt)
        torch.cuda.synchronize()
        want_idx = orc.select_ratio(z_ref, ratio)
        k = int(cnt.item())
        assert k == k_want == len(want_idx)
        assert np.array_equal(idx[:k].cpu().numpy(), want_idx)
        got = xg.cpu()
        skipped = np.setdiff1d(np.arange(B), want_idx)
        assert torch.equal(got[skipped], x[skipped])
        lens = kv.kv_len.cpu().numpy()
        executed = np.isin(np.arange(B), want_idx)
        assert np.array_equal(lens, ctx_len + executed.astype(np.int32))   # bypassed tokens append nothing
        # a few sequences through the oracle (each decode token only sees its own sequence's cache)
        sub = [b for b in check if executed[b]] or [int(want_idx[0])]
        okv = orc.KVCache(to_f64(kc[sub]), to_f64(vc[sub]), [ctx_len] * len(sub))
        o_s, p_s = si.ragged_sequences([1] * len(sub), starts=[ctx_len] * len(sub))
        want, _, _ = orc.layer_forward(to_f64(x[sub]), p, cfg_dict(shape), o_s.numpy(), p_s.numpy(), "forced",
                                       list(range(len(sub))), okv)
        check_parity(orc.parity_error(to_f64(got[sub]), want), shape.act_dtype, ("7B decode step", B, ratio), hidden=shape.hidden)
        gk = to_f64(kv.k[sub, :, ctx_len].reshape(len(sub), -1).cpu())
        gv = to_f64(kv.v[sub, :, ctx_len].reshape(len(sub), -1).cpu())
        check_parity(orc.parity_error(gk, okv.k[:, ctx_len]), "fp16", "7B decode appended keys")
        check_parity(orc.parity_error(gv, okv.v[:, ctx_len]), "fp16", "7B decode appended values")


C5 = si.LayerShape(5120, 40, 40, 128, 13824, 4, 128, "bf16")     # LLaMA-13B-shaped layer


@pytest.mark.parametrize("bits,ratio", [(4, 0.3), (3, 1.0)])
def test_llama13b_shaped_prefill_layer_16x512(qt, bits, ratio):
    import dataclasses
    _prefill_case(qt, dataclasses.replace(C5, bits=bits), 16, 512, ratio, seed=16 + bits)


def test_llama13b_shaped_decode_step_batch128_ctx4096(qt):
    # decode after the prefill: 128 one-token sequences against 4096 cached entries each; ratio 1.0 runs the
    # matrix-core GEMM with a single 128-row tile, ratio 0.3 (38 rows) the skinny kernel
    shape = si.LayerShape(5120, 40, 40, 128, 13824, 4, 128, "fp16")
    B, ctx_len, cap, seed = 128, 4096, 4096 + 8, 18
    tensors = si.layer_tensors(shape, 0, seed, unit_gains=True)
    x = si.hidden_states(shape, B, seed)
    offs, pos = si.ragged_sequences([1] * B, starts=[ctx_len] * B)
    g = torch.Generator(device="cuda").manual_seed(seed)
    kc = torch.randn(B, shape.n_kv_heads, cap, shape.head_dim, device="cuda", dtype=torch.float16, generator=g)   # 5.4 GB each,
    vc = torch.randn(B, shape.n_kv_heads, cap, shape.head_dim, device="cuda", dtype=torch.float16, generator=g)   # library layout
    cfg = qt.cfg_from_shape(shape)
    lw = qt.quantize_layer(tensors, shape.bits, shape.group)
    p, _ = oracle_layer(shape, 0, seed, tensors=tensors)
    z_ref = orc.router_scores(to_f64(x), tensors["router_w"].numpy(), 0.0)
    ctx = qt.Context()
    for ratio in (1.0, 0.3):
        qt.qtale_set_exec_ratio(ctx, ratio)
        kv = qt.KVCache(kc, vc, torch.full((B,), ctx_len, dtype=torch.int32).cuda())
        xg = x.cuda()
        idx = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        qt.qtale_layer_forward(ctx, cfg, lw, xg, offs.cuda(), pos.cuda(), kv=kv, sel_idx=idx, sel_count=cnt)
        torch.cuda.synchronize()
        want_idx = orc.select_ratio(z_ref, ratio)
        k = int(cnt.item())
        assert k == len(want_idx) == orc.executed_count(ratio, B)
        assert np.array_equal(idx[:k].cpu().numpy(), want_idx)
        got = xg.cpu()
        skipped = np.setdiff1d(np.arange(B), want_idx)
        assert torch.equal(got[skipped], x[skipped])
        executed = np.isin(np.arange(B), want_idx)
        assert np.array_equal(kv.kv_len.cpu().numpy(), ctx_len + executed.astype(np.int32))
        sub = [int(t) for t in want_idx[[0, len(want_idx) // 2, -1]]]
        tok = lambda t: t[sub, :, :ctx_len + 1].permute(0, 2, 1, 3).reshape(len(sub), ctx_len + 1, -1).cpu()   # one row per token
        kc_sub, vc_sub = tok(kc), tok(vc)
        okv = orc.KVCache(to_f64(kc_sub), to_f64(vc_sub), [ctx_len] * len(sub))
        o_s, p_s = si.ragged_sequences([1] * len(sub), starts=[ctx_len] * len(sub))
        want, _, _ = orc.layer_forward(to_f64(x[sub]), p, cfg_dict(shape), o_s.numpy(), p_s.numpy(), "forced",
                                       list(range(len(sub))), okv)
        check_parity(orc.parity_error(to_f64(got[sub]), want), shape.act_dtype, ("13B decode step", ratio), hidden=shape.hidden)
        check_parity(orc.parity_error(to_f64(kv.k[sub, :, ctx_len].reshape(len(sub), -1).cpu()), okv.k[:, ctx_len]), "fp16", "13B decode appended keys")
        # the rows appended at index ctx_len lie beyond the length the next ratio starts from: no restore needed

