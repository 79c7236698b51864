"""GPU parity of the individual steps against the CPU oracle, through the C ABI (run with -m gpu).

Bit-exact: packed int4 codes, fp16 scales/zero-points, router scores, selected indices and counts.
Floating point (W4A16 GEMMs): |gpu - oracle| <= 2e-2 * max(|oracle|, rms(oracle row))."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import qtale_oracle as orc
from tests.helpers import check_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qt():
    import paper_2602_10431_amd as pkg
    pkg.load_library()
    return pkg


def _w(N, K, seed, std=0.02):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(N, K, generator=g) * std


@pytest.mark.parametrize("bits", [4, 3, 2])
@pytest.mark.parametrize("N,K,G", [(256, 256, 32), (256, 688, 32), (688, 256, 32), (100, 136, 64),
                                   (512, 1024, 128), (33, 4096, 128), (4096, 264, 128)])
def test_quantize_is_bit_exact(qt, N, K, G, bits):
    W = _w(N, K, N * 7 + K)
    W[0, : min(K, G)] = 0.0                                     # a constant-zero group
    W[1, : min(K, G)] = W[1, : min(K, G)].abs() + 1e-3          # an all-positive group
    ql = qt.qtale_quantize(W.cuda(), bits, G)
    torch.cuda.synchronize()
    codes, s, z = orc.quantize_rtn(W.numpy(), bits, G)
    assert np.array_equal(ql.codes.cpu().numpy().view(np.uint32), orc.pack_codes(codes, bits))
    assert np.array_equal(ql.scales.cpu().numpy().view(np.uint16), s.view(np.uint16))
    assert np.array_equal(ql.zeros.cpu().numpy().view(np.uint16), z.view(np.uint16))


def test_quantize_rejects_bad_parameters(qt):
    W = _w(8, 64, 0).cuda()
    for bits, group in [(1, 128), (5, 128), (4, 48), (8, 128)]:
        with pytest.raises(qt.QtaleError):
            qt.qtale_quantize(W, bits, group)
    with pytest.raises(qt.QtaleError):
        qt.qtale_quantize(_w(8, 60, 0).cuda(), 4, 32)           # K % 8 != 0


@pytest.mark.parametrize("M,N,K,G", [(64, 256, 256, 32), (32, 256, 688, 32), (7, 688, 256, 32), (300, 416, 512, 128),
                                     (257, 1024, 1024, 128), (1, 96, 64, 64), (513, 4096, 264, 128),
                                     (65, 4096, 1024, 128), (130, 416, 688, 32), (256, 1024, 512, 64),
                                     (700, 416, 688, 32), (1000, 96, 1096, 64), (1500, 200, 320, 128)])
@pytest.mark.parametrize("bits", [4, 3, 2])
def test_linear_w4a16_matches_oracle(qt, M, N, K, G, bits):
    W = _w(N, K, M + N + K)
    A = torch.randn(M, K, generator=torch.Generator().manual_seed(M)).to(torch.float16)
    ql = qt.qtale_quantize(W.cuda(), bits, G)
    out = qt.qtale_linear_w4a16(ql, A.cuda())
    torch.cuda.synchronize()
    codes, s, z = orc.quantize_rtn(W.numpy(), bits, G)
    want = A.to(torch.float64).numpy() @ orc.dequantize(codes, s, z, G).T
    check_parity(orc.parity_error(out.cpu().to(torch.float64).numpy(), want), "fp16", "w4a16 gemm")


@pytest.mark.parametrize("bits", [4, 3, 2])
@pytest.mark.parametrize("M,K,N,G", [(256, 256, 96, 32), (64, 64, 512, 64), (512, 512, 40, 128)])
def test_identity_activations_return_the_dequantized_weights_exactly(qt, M, K, N, G, bits):
    # A = I: out[m][n] is the single product 1 * W'[n][m], so the kernel's in-register dequantisation
    # must equal fp16((code - zero) * scale) bit for bit (prefill kernel for M > 64, skinny kernel else)
    W = _w(N, K, 5 * N + K + bits)
    ql = qt.qtale_quantize(W.cuda(), bits, G)
    out = qt.qtale_linear_w4a16(ql, torch.eye(K, dtype=torch.float16).cuda())
    torch.cuda.synchronize()
    codes, s, z = orc.quantize_rtn(W.numpy(), bits, G)
    want = torch.from_numpy(orc.dequantize(codes, s, z, G).T.copy()).to(torch.float16)
    assert torch.equal(out.cpu(), want)


def test_prepack_from_canonical_three_bit_codes(qt):
    # weights quantized elsewhere (here: by the oracle) and handed over in the canonical 3-bit layout
    N, K, G = 64, 688, 32
    W = _w(N, K, 77)
    codes, s, z = orc.quantize_rtn(W.numpy(), 3, G)
    words = torch.from_numpy(orc.pack_codes(codes, 3).view(np.int32)).cuda()
    ql = qt.qtale_prepack(words, torch.from_numpy(s).cuda(), torch.from_numpy(z).cuda(), N, K, 3, G)
    A = torch.randn(16, K, generator=torch.Generator().manual_seed(4)).to(torch.float16)
    out = qt.qtale_linear_w4a16(ql, A.cuda())
    torch.cuda.synchronize()
    want = A.to(torch.float64).numpy() @ orc.dequantize(codes, s, z, G).T
    check_parity(orc.parity_error(out.cpu().to(torch.float64).numpy(), want), "fp16", "w4a16 gemm")


@pytest.mark.parametrize("M,I,K,G", [(64, 688, 256, 32), (200, 352, 512, 128), (5, 64, 128, 64),
                                     (600, 352, 688, 32), (300, 1000, 136, 64), (1100, 96, 448, 128)])
@pytest.mark.parametrize("bits", [4, 3, 2])
def test_swiglu_w4a16_matches_oracle(qt, M, I, K, G, bits):
    Wg, Wu = _w(I, K, 1, 0.05), _w(I, K, 2, 0.05)
    A = torch.randn(M, K, generator=torch.Generator().manual_seed(3)).to(torch.float16)
    qg, qu = qt.qtale_quantize(Wg.cuda(), bits, G), qt.qtale_quantize(Wu.cuda(), bits, G)
    out = qt.qtale_swiglu_w4a16(qg, qu, A.cuda())
    torch.cuda.synchronize()
    A64 = A.to(torch.float64).numpy()
    dg = orc.dequantize(*orc.quantize_rtn(Wg.numpy(), bits, G), G)
    du = orc.dequantize(*orc.quantize_rtn(Wu.numpy(), bits, G), G)
    want = orc.silu(A64 @ dg.T) * (A64 @ du.T)
    check_parity(orc.parity_error(out.cpu().to(torch.float64).numpy(), want), "fp16", "w4a16 gemm")


@pytest.mark.parametrize("T,H,dtype", [(64, 256, "fp16"), (1000, 512, "bf16"), (1, 64, "fp16"), (5000, 256, "bf16"),
                                       (1025, 4096, "bf16")])
def test_router_and_selection_are_bit_exact(qt, T, H, dtype):
    shape = si.LayerShape(H, 4, 4, 64, 256, 4, 32, dtype)
    x = si.hidden_states(shape, T, T)
    w = si.router_weight(shape, 0, T)
    z_ref = orc.router_scores(x.to(torch.float64).numpy(), w.numpy(), 0.125)
    ctx = qt.Context()
    lens = [T // 3, T - T // 3 - T // 5, T // 5] if T >= 5 else [T]
    offs, _ = si.ragged_sequences(lens)
    for mode, val in [("ratio", 0.0), ("ratio", 0.3), ("ratio", 0.5), ("ratio", 1.0), ("threshold", 0.5),
                      ("threshold", 0.2), ("threshold", 0.0), ("threshold", 1.0)]:
        if mode == "ratio":
            qt.qtale_set_exec_ratio(ctx, val)
            want = orc.select_ratio(z_ref, val)
        else:
            qt.qtale_set_threshold(ctx, val)
            want = orc.select_threshold(z_ref, val)
        z, idx, cnt, cu = qt.qtale_router_select(ctx, x.cuda(), w.cuda(), 0.125, offs.cuda())
        torch.cuda.synchronize()
        assert np.array_equal(z.cpu().numpy().view(np.uint32), z_ref.view(np.uint32))
        k = int(cnt.item())
        assert k == len(want), (mode, val)
        assert np.array_equal(idx[:k].cpu().numpy(), want)
        cu_ref = np.searchsorted(want, offs.numpy(), side="left")
        assert np.array_equal(cu.cpu().numpy(), cu_ref)


def test_selection_beyond_the_on_chip_caches(qt):
    # 40000 tokens in 3000 sequences: more keys and more sequence offsets than the selection kernel keeps in LDS
    T, H, B = 40000, 64, 3000
    shape = si.LayerShape(H, 1, 1, 64, 64, 4, 32, "bf16")
    x = si.hidden_states(shape, T, 5)
    w = si.router_weight(shape, 0, 5)
    z_ref = orc.router_scores(x.to(torch.float64).numpy(), w.numpy(), -0.05)
    rng = np.random.default_rng(5)
    cuts = np.sort(rng.integers(0, T + 1, size=B - 1))
    offs = torch.from_numpy(np.concatenate([[0], cuts, [T]]).astype(np.int32))
    ctx = qt.Context()
    for mode, val in [("ratio", 0.37), ("ratio", 1.0), ("threshold", 0.5), ("threshold", 0.31)]:
        if mode == "ratio":
            qt.qtale_set_exec_ratio(ctx, val)
            want = orc.select_ratio(z_ref, val)
        else:
            qt.qtale_set_threshold(ctx, val)
            want = orc.select_threshold(z_ref, val)
        z, idx, cnt, cu = qt.qtale_router_select(ctx, x.cuda(), w.cuda(), -0.05, offs.cuda())
        torch.cuda.synchronize()
        assert np.array_equal(z.cpu().numpy().view(np.uint32), z_ref.view(np.uint32))
        k = int(cnt.item())
        assert k == len(want), (mode, val)
        assert np.array_equal(idx[:k].cpu().numpy(), want)
        assert np.array_equal(cu.cpu().numpy(), np.searchsorted(want, offs.numpy(), side="left"))


def test_selection_ties_go_to_lower_index(qt):
    # identical rows give identical scores: ties must be resolved by token index
    shape = si.LayerShape(64, 1, 1, 64, 64, 4, 32, "fp16")
    base = si.hidden_states(shape, 4, 1)
    x = base[[0, 1, 0, 0, 2, 0, 3, 0, 0]].contiguous()           # five copies of row 0
    w = si.router_weight(shape, 0, 2)
    z_ref = orc.router_scores(x.to(torch.float64).numpy(), w.numpy(), 0.0)
    ctx = qt.Context()
    for r in [0.2, 0.34, 0.5, 0.67, 0.9]:
        qt.qtale_set_exec_ratio(ctx, r)
        z, idx, cnt, _ = qt.qtale_router_select(ctx, x.cuda(), w.cuda(), 0.0)
        torch.cuda.synchronize()
        want = orc.select_ratio(z_ref, r)
        assert int(cnt.item()) == len(want) and np.array_equal(idx[: len(want)].cpu().numpy(), want)


def test_selection_is_deterministic(qt):
    shape = si.LayerShape(256, 4, 4, 64, 256, 4, 32, "bf16")
    x = si.hidden_states(shape, 3000, 9).cuda()
    w = si.router_weight(shape, 0, 9).cuda()
    ctx = qt.Context()
    qt.qtale_set_exec_ratio(ctx, 0.37)
    a = qt.qtale_router_select(ctx, x, w)
    b = qt.qtale_router_select(ctx, x, w)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


def _mlp_router(H, R, seed):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(R, H, generator=g) * 0.05, torch.randn(R, generator=g) * 0.1,
            torch.randn(2, R, generator=g) * 0.5, torch.randn(2, generator=g) * 0.1)


@pytest.mark.parametrize("T,H,R,dtype", [(64, 256, 16, "fp16"), (1000, 512, 8, "bf16"), (5, 64, 1, "fp16"),
                                         (300, 4096, 32, "bf16"), (17, 1024, 40, "fp16"), (2048, 4096, 16, "bf16")])
def test_mlp_router_scores_are_bit_exact(qt, T, H, R, dtype):
    # hidden widths below, at and above one 16-unit pass; H below and above one 512-column chunk; ragged token tail
    shape = si.LayerShape(H, 1, 1, 64, 64, 4, 32, dtype)
    x = si.hidden_states(shape, T, 70 + R)
    W1, b1, W2, b2 = _mlp_router(H, R, T + R)
    z = qt.qtale_router_mlp_scores(x.cuda(), W1.cuda(), b1.cuda(), W2.cuda(), b2.cuda())
    torch.cuda.synchronize()
    want = orc.router_scores_mlp(x.to(torch.float64).numpy(), W1.numpy(), b1.numpy(), W2.numpy(), b2.numpy())
    assert np.array_equal(z.cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("K,G,bits", [(40, 32, 4), (72, 64, 3), (264, 128, 2), (320, 32, 3), (384, 128, 4), (456, 64, 2)])
def test_large_tile_gemm_short_and_ragged_k(qt, K, G, bits):
    # 2600 rows x 2048 columns is past the 64-row-tile regime, so these run the 128 x 256 tiles: one to eight
    # k-tiles (every remainder of the three-slot weight ring), K not a multiple of 64, every code width
    M, N = 2600, 2048
    W = _w(N, K, K)
    A = torch.randn(M, K, generator=torch.Generator().manual_seed(K)).to(torch.float16)
    ql = qt.qtale_quantize(W.cuda(), bits, G)
    out = qt.qtale_linear_w4a16(ql, A.cuda())
    torch.cuda.synchronize()
    codes, s, z = orc.quantize_rtn(W.numpy(), bits, G)
    want = A.to(torch.float64).numpy() @ orc.dequantize(codes, s, z, G).T
    check_parity(orc.parity_error(out.cpu().to(torch.float64).numpy(), want), "fp16", "w4a16 gemm")


@pytest.mark.parametrize("K,G,bits", [(136, 64, 4), (320, 32, 3)])
def test_large_tile_swiglu_short_and_ragged_k(qt, K, G, bits):
    M, I = 2600, 2048
    g = torch.Generator().manual_seed(K)
    Wg, Wu = torch.randn(I, K, generator=g) * 0.05, torch.randn(I, K, generator=g) * 0.05
    A = torch.randn(M, K, generator=g).to(torch.float16)
    qg, qu = qt.qtale_quantize(Wg.cuda(), bits, G), qt.qtale_quantize(Wu.cuda(), bits, G)
    out = qt.qtale_swiglu_w4a16(qg, qu, A.cuda())
    torch.cuda.synchronize()
    A64 = A.to(torch.float64).numpy()
    dg = orc.dequantize(*orc.quantize_rtn(Wg.numpy(), bits, G), G)
    du = orc.dequantize(*orc.quantize_rtn(Wu.numpy(), bits, G), G)
    want = orc.silu(A64 @ dg.T) * (A64 @ du.T)
    check_parity(orc.parity_error(out.cpu().to(torch.float64).numpy(), want), "fp16", "w4a16 gemm")


@pytest.mark.parametrize("M,K,G", [(2088, 256, 128), (2148, 256, 128), (2088, 456, 64)])
@pytest.mark.parametrize("bits", [4, 3])
def test_large_tile_gemm_rows_beyond_the_last_full_tile(qt, M, K, G, bits):
    # 16 full 128-row tiles + 40 (or 100) rows on outputs of 32 column tiles: the 17th row of tiles would be tiles
    # 513..544 on a chip that holds 512 workgroups, so those rows run on the small-row kernels instead (one chunk, two
    # 64-row chunks); plain store and SwiGLU epilogues; K = 456 is not a multiple of the 64-wide k-tile in either launch
    g = torch.Generator().manual_seed(M + bits)
    A = torch.randn(M, K, generator=g).to(torch.float16)
    A64 = A.to(torch.float64).numpy()
    W = torch.randn(8192, K, generator=g) * 0.05
    out = qt.qtale_linear_w4a16(qt.qtale_quantize(W.cuda(), bits, G), A.cuda())
    torch.cuda.synchronize()
    want = A64 @ orc.dequantize(*orc.quantize_rtn(W.numpy(), bits, G), G).T
    check_parity(orc.parity_error(out.cpu().to(torch.float64).numpy(), want), "fp16", ("w4a16 gemm", M, bits))
    assert orc.parity_error(out[-(M % 128):].cpu().to(torch.float64).numpy(), want[-(M % 128):]) < 2e-2
    Wg, Wu = torch.randn(4096, K, generator=g) * 0.05, torch.randn(4096, K, generator=g) * 0.05
    out = qt.qtale_swiglu_w4a16(qt.qtale_quantize(Wg.cuda(), bits, G), qt.qtale_quantize(Wu.cuda(), bits, G), A.cuda())
    torch.cuda.synchronize()
    dg = orc.dequantize(*orc.quantize_rtn(Wg.numpy(), bits, G), G)
    du = orc.dequantize(*orc.quantize_rtn(Wu.numpy(), bits, G), G)
    want = orc.silu(A64 @ dg.T) * (A64 @ du.T)
    check_parity(orc.parity_error(out.cpu().to(torch.float64).numpy(), want), "fp16", ("w4a16 gemm", M, bits))
    assert orc.parity_error(out[-(M % 128):].cpu().to(torch.float64).numpy(), want[-(M % 128):]) < 2e-2


def test_linear_random_shape_sweep(qt):
    # 40 seeded shapes across the dispatch regimes (few rows / 64-row chunks / 64-row tiles / 128-row tiles), ragged K, output
    # widths that are not multiples of the 32-column fragment, all code widths and group sizes
    rng = np.random.default_rng(2024)
    for case in range(40):
        bits = int(rng.choice([4, 3, 2]))
        G = int(rng.choice([32, 64, 128]))
        M = int(rng.choice([1, 3, 17, 31, 33, 64, 65, 100, 129, 200, 256, 257, 300, 520, 777, 1290]))
        N = 8 * int(rng.integers(1, 90))
        K = 8 * int(rng.integers(2, 140))
        g = torch.Generator().manual_seed(1000 + case)
        W = torch.randn(N, K, generator=g) * 0.05
        A = torch.randn(M, K, generator=g).to(torch.float16)
        ql = qt.qtale_quantize(W.cuda(), bits, G)
        out = qt.qtale_linear_w4a16(ql, A.cuda())
        torch.cuda.synchronize()
        codes, s, z = orc.quantize_rtn(W.numpy(), bits, G)
        assert np.array_equal(ql.codes.cpu().numpy().view(np.uint32), orc.pack_codes(codes, bits)), (case, bits, G, N, K)
        want = A.to(torch.float64).numpy() @ orc.dequantize(codes, s, z, G).T
        err = orc.parity_error(out.cpu().to(torch.float64).numpy(), want)
        check_parity(err, "fp16", ("linear sweep", case, bits, G, M, N, K))


def test_swiglu_random_shape_sweep(qt):
    rng = np.random.default_rng(77)
    for case in range(16):
        bits = int(rng.choice([4, 3, 2]))
        G = int(rng.choice([32, 64, 128]))
        M = int(rng.choice([1, 30, 64, 70, 190, 256, 300, 650, 1300]))
        I = 8 * int(rng.integers(1, 120))
        K = 8 * int(rng.integers(2, 100))
        g = torch.Generator().manual_seed(2000 + case)
        Wg, Wu = torch.randn(I, K, generator=g) * 0.05, torch.randn(I, K, generator=g) * 0.05
        A = torch.randn(M, K, generator=g).to(torch.float16)
        qg, qu = qt.qtale_quantize(Wg.cuda(), bits, G), qt.qtale_quantize(Wu.cuda(), bits, G)
        out = qt.qtale_swiglu_w4a16(qg, qu, A.cuda())
        torch.cuda.synchronize()
        A64 = A.to(torch.float64).numpy()
        dg = orc.dequantize(*orc.quantize_rtn(Wg.numpy(), bits, G), G)
        du = orc.dequantize(*orc.quantize_rtn(Wu.numpy(), bits, G), G)
        want = orc.silu(A64 @ dg.T) * (A64 @ du.T)
        err = orc.parity_error(out.cpu().to(torch.float64).numpy(), want)
        check_parity(err, "fp16", ("swiglu sweep", case, bits, G, M, I, K))

