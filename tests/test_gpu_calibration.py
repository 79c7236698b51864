"""GPU parity of the threshold calibration (two-phase grid search of Sec. 3.4) against the CPU oracle
(run with -m gpu).  With fixed scores every count is an integer, so theta, the ratio table and the set of
evaluated candidates must agree exactly; with the stack in the loop the realised ratios may differ by the
few (layer, token) pairs whose score sits within rounding of the threshold."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import qtale_oracle as orc
from tests.helpers import cfg_dict, oracle_layer, round_like, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qt():
    import paper_2602_10431_amd as pkg
    pkg.load_library()
    return pkg


@pytest.mark.parametrize("target", [1.0, 0.9, 0.7, 0.5, 0.33, 0.0])
def test_calibration_from_fixed_scores_is_exact(qt, target):
    g = torch.Generator().manual_seed(int(target * 100))
    z = torch.randn(4, 5000, generator=g) * 1.28
    z[0, 0], z[1, 7], z[2, 9] = float("nan"), float("inf"), float("-inf")
    z[3, :50] = float(orc.theta_to_logit(np.float32(0.25)))      # ties exactly at a grid threshold execute
    ctx = qt.Context()
    theta, r, seen = qt.qtale_calibrate_threshold_from_scores(ctx, z.cuda(), target)
    wtheta, wr, wseen = orc.calibrate_theta_from_scores(z.numpy(), target)
    assert np.float32(theta) == wtheta
    assert sorted(seen) == sorted(wseen)                          # same candidates evaluated
    for n in seen:
        assert np.float32(seen[n]) == np.float32(wseen[n]), n
    assert np.float32(r) == np.float32(wr)
    mode, value = qt.qtale_get_control(ctx)
    assert mode == qt.QTALE_MODE_THRESHOLD and np.float32(value) == wtheta


def test_uniform_execute_probabilities_calibrate_to_one_minus_ratio(qt):
    N = 1 << 20                                                   # several blocks per counter
    u = (np.arange(N) + 0.5) / N
    z = torch.from_numpy(np.log(u / (1.0 - u)).astype(np.float32))
    ctx = qt.Context()
    for target, want in [(0.7, 0.30), (0.55, 0.45), (0.93, 0.07)]:
        theta, r, _ = qt.qtale_calibrate_threshold_from_scores(ctx, z.cuda(), target)
        assert np.float32(theta) == np.float32(want)
        assert abs(r - target) <= 2.0 / N


def test_stack_calibration_against_oracle_and_against_its_own_runs(qt):
    shape = si.C1
    L, T, seed, target = 3, 96, 31, 0.6
    tensors = [si.layer_tensors(shape, l, seed, unit_gains=False, std=0.06) for l in range(L)]
    for t in tensors:
        t["router_w"] = t["router_w"] * 4.0                       # spread the scores over several grid steps
    x = si.hidden_states(shape, T, seed)
    offs, pos = si.ragged_sequences([64, 32])
    cfg = qt.cfg_from_shape(shape)
    stack = qt.Stack(cfg, [qt.quantize_layer(t, shape.bits, shape.group) for t in tensors])
    ctx = qt.Context()
    xg = x.cuda()
    theta, r, seen = qt.qtale_calibrate_threshold(ctx, stack, xg, offs.cuda(), pos.cuda(), target)
    assert torch.equal(xg.cpu(), x)                               # the calibration batch is only read
    mode, value = qt.qtale_get_control(ctx)
    assert mode == qt.QTALE_MODE_THRESHOLD and np.float32(value) == np.float32(theta)
    assert list(range(5, 51, 5)) == [n for n in sorted(seen) if n % 5 == 0 and n in range(5, 51, 5)]
    assert abs(r - target) == min(abs(v - target) for v in seen.values())
    # every table entry is the realised ratio of a threshold-mode run of the same library
    for n in (min(seen), int(round(theta * 100)), max(seen)):
        qt.qtale_set_threshold(ctx, n / 100.0)
        cnt = torch.zeros(L, dtype=torch.int32, device="cuda")
        qt.qtale_stack_forward(ctx, stack, x.cuda(), offs.cuda(), pos.cuda(), sel_count=cnt)
        assert np.float32(seen[n]) == np.float32(int(cnt.sum().item()) / (L * T))
    # oracle: same search, hidden states rounded to the activation dtype between layers like the GPU's
    layers = [oracle_layer(shape, l, seed, tensors=tensors[l])[0] for l in range(L)]
    wtheta, wr, wseen = orc.calibrate_theta(to_f64(x), layers, cfg_dict(shape), offs.numpy(), pos.numpy(), target,
                                            round_to=lambda a: round_like(a, shape.act_dtype))
    slack = 3.0 / (L * T)                                         # (layer, token) pairs that may flip at the threshold
    for n in set(seen) & set(wseen):
        assert abs(seen[n] - wseen[n]) <= slack, (n, seen[n], wseen[n])
    assert abs(r - target) <= abs(wr - target) + slack
    assert abs(theta - float(wtheta)) <= 0.0101                   # same grid point or its neighbour
