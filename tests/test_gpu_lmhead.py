"""GPU parity: hb_lmhead_argmax against the float64 oracle.

Margin rule: where the oracle's top-1 logit leads the runner-up by more than EPS, the GPU id
must be the oracle's; elsewhere (a near tie that fp32 accumulation order may flip) it must be
one of the two.  EPS = 1e-4 * |h| * |w|_typ bounds the fp32 accumulation error of a K-term dot
product (K * 2^-24 * sum|h_k w_k| is a few 1e-6 of that product for K = 3584)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import lmhead_logits_ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def step():
    import paper_2509_18824_amd.step as s
    return s


def _check(hidden, weight, ids, mx, rows=None, block=192):
    rows = np.arange(hidden.shape[0]) if rows is None else np.asarray(rows)
    w = W.widen(weight)
    w_rms = np.sqrt((w * w).sum(1).mean())
    got_all = ids.cpu().numpy()
    mx_all = mx.cpu().numpy() if mx is not None else None
    n_clear = 0
    for i0 in range(0, len(rows), block):  # blocks of rows bound the float64 logits in memory
        rb = rows[i0:i0 + block]
        h = W.widen(hidden)[rb]
        logits = lmhead_logits_ref(h, w)
        r = np.arange(len(rb))
        top1 = np.argmax(logits, axis=1)  # first maximum = lowest id
        best = logits[r, top1]
        if logits.shape[1] > 1:
            rest = logits.copy()
            rest[r, top1] = -np.inf
            top2 = np.argmax(rest, axis=1)
        else:
            top2 = top1
        margin = best - logits[r, top2]
        eps = 1e-4 * np.linalg.norm(h, axis=1) * w_rms
        got = got_all[rb]
        clear = margin > eps
        assert (got[clear] == top1[clear]).all(), "argmax differs where the margin is clear"
        assert np.logical_or(got == top1, got == top2)[~clear].all()
        if mx_all is not None:
            assert np.abs(mx_all[rb] - logits[r, got]).max() <= 1e-2
        n_clear += int(clear.sum())
    return n_clear


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
# K % 64 == 0 takes the matrix-core kernel: the shapes below cover its four hidden-tile heights
# (64 .. 256 rows), one and several hidden tiles, odd and even numbers of K steps, and
# vocabularies below, at and above one 256-row tile
@pytest.mark.parametrize("M,K,V", [(1, 8, 1), (5, 64, 1000), (60, 136, 777), (128, 512, 4099), (300, 264, 513),
                                   (250, 192, 1500), (300, 256, 777), (1000, 128, 3000), (380, 64, 600),
                                   (64, 320, 256), (193, 448, 255)])
def test_small_shapes(step, dtype, M, K, V):
    hidden, weight = W.make_lmhead_inputs(M * 7 + V, M, K, V, dtype=dtype, w_std=0.05)
    ids, mx = step.lmhead_argmax(hidden.cuda(), weight.cuda())
    torch.cuda.synchronize()
    _check(hidden, weight, ids, mx)


def test_work_units_of_the_left_over_cus(step):
    """960 rows are five 192-row hidden tiles: six lockstep groups occupy 30 of an XCD's 32 CUs.
    With 152 vocabulary tiles (19 per XCD) the other two CUs take the XCD's first tile as five
    (vocabulary tile, hidden tile) units, which saves the groups their fourth round.  Every row
    is checked against the oracle over the whole vocabulary, and winners are planted in the tiles
    that travel that way (vocabulary ids below 8 * 256) and in the ragged last tile."""
    M, K, V = 960, 192, 152 * 256 - 100
    hidden, weight = W.make_lmhead_inputs(4242, M, K, V, dtype="bf16", w_std=0.05)
    rng = np.random.default_rng(7)
    planted = {}
    for m in rng.choice(M, size=120, replace=False):
        v = int(rng.integers(0, 2048)) if m % 3 else int(rng.integers(V - 156, V))
        weight[v] = (hidden[m].float() * 0.5).to(weight.dtype)
        planted[int(m)] = v
    ids, mx = step.lmhead_argmax(hidden.cuda(), weight.cuda())
    torch.cuda.synchronize()
    _check(hidden, weight, ids, mx)
    got = ids.cpu().numpy()
    hit = sum(int(got[m]) == v for m, v in planted.items())
    assert hit >= 100  # a later planted row can only lose to another planted row of the same kind


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_planted_winner_ties_and_nan(step, dtype):
    M, K, V = 70, 256, 3000
    hidden, weight = W.make_lmhead_inputs(5, M, K, V, dtype=dtype, w_std=0.02)
    rng = np.random.default_rng(0)
    plant = rng.choice(V, size=M, replace=False)
    for m in range(0, M, 2):
        weight[plant[m]] = hidden[m] * 0.5  # logit = |h|^2 / 2, far above the N(0, 0.02) rows
    # exact ties: three identical rows, the lowest id must win
    tie = sorted(rng.choice(V, size=3, replace=False).tolist())
    while set(tie) & set(plant.tolist()):
        tie = sorted(rng.choice(V, size=3, replace=False).tolist())
    for v in tie:
        weight[v] = hidden[1] * 0.75
    ids, mx = step.lmhead_argmax(hidden.cuda(), weight.cuda())
    ids = ids.cpu().numpy()
    assert (ids[0::2] == plant[0::2]).all()
    assert ids[1] == tie[0]
    # a NaN logit never wins
    weight[7] = float("nan")
    ids2, _ = step.lmhead_argmax(hidden.cuda(), weight.cuda())
    ids2 = ids2.cpu().numpy()
    assert (ids2 != 7).all() and (ids2[0::2] == plant[0::2]).all()


def test_deterministic(step):
    hidden, weight = W.make_lmhead_inputs(9, 200, 512, 20000, w_std=0.02)
    h, w = hidden.cuda(), weight.cuda()
    a, am = step.lmhead_argmax(h, w)
    b, bm = step.lmhead_argmax(h, w)
    assert torch.equal(a, b) and torch.equal(am, bm)


@pytest.fixture(scope="module")
def full_weight():
    return W.make_lmhead_inputs(4000, 960, 3584, 152064, dtype="bf16")


@pytest.mark.parametrize("M", [960, 128])
def test_full_vocabulary_every_row(step, full_weight, M):
    """hidden 3584 x vocab 152064 (the full-step workload; M = 960 tree nodes, or 128 for the
    8-node-chain run); the oracle recomputes every row over the whole vocabulary."""
    hidden, weight = full_weight
    hidden = hidden[:M].contiguous()
    ids, mx = step.lmhead_argmax(hidden.cuda(), weight.cuda())
    torch.cuda.synchronize()
    n_clear = _check(hidden, weight, ids, mx)
    assert n_clear >= 0.9 * M
    assert (ids >= 0).all() and (ids < 152064).all()
