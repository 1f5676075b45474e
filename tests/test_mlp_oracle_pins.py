"""Pins for the dense-tower oracle (oracle/mlp_oracle.py), all on the CPU."""
import numpy as np
import pytest
import torch

from oracle import ctr_oracle as O
from oracle import mlp_oracle as M

F32 = np.float32


def test_bf16_rounding_is_nearest_even_and_matches_a_library():
    assert M.bf16_round(F32(1.0)) == 1.0
    assert M.bf16_round(F32(1.0 + 2.0 ** -8)) == 1.0                    # tie -> even mantissa
    assert M.bf16_round(F32(1.0 + 3 * 2.0 ** -8)) == F32(1.0 + 2.0 ** -6)
    assert M.bf16_round(F32(1.0 + 2.0 ** -8 + 2.0 ** -20)) == F32(1.0 + 2.0 ** -7)
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(F32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(M.bf16_round(a), ref)


def test_parameter_layout_and_init_statistics():
    in_dim, hidden = 64, [32, 16]
    p = M.init_params(in_dim, hidden, 7)
    assert p.size == M.n_params(in_dim, hidden) == 64 * 32 + 32 + 32 * 16 + 16 + 16 + 1
    W1 = p[:64 * 32]
    assert abs(W1.std() - np.sqrt(2 / 64)) < 0.02 * np.sqrt(2 / 64) * 3 and abs(W1.mean()) < 0.02
    assert not p[64 * 32:64 * 32 + 32].any()                              # biases start at zero
    assert np.array_equal(p, M.init_params(in_dim, hidden, 7))
    assert not np.array_equal(p, M.init_params(in_dim, hidden, 8))
    big = M.init_params(4096, [64], 1)[:4096 * 64]
    assert abs(big.std() / np.sqrt(2 / 4096) - 1) < 0.01


def _torch_reference(o, pooled, labels):
    """The same network in float64 torch with autograd (no bf16 rounding)."""
    flat = torch.tensor(o.params[0].astype(np.float64), requires_grad=True)
    x = torch.tensor(np.asarray(pooled, np.float64), requires_grad=True)
    h, off = x, 0
    for li, (i, k) in enumerate(o.shapes):
        W = flat[off:off + i * k].reshape(i, k)
        off += i * k
        b = flat[off:off + k]
        off += k
        h = h @ W + b
        if li < len(o.shapes) - 1:
            h = torch.relu(h)
    loss = torch.nn.functional.binary_cross_entropy_with_logits(h[:, 0], torch.tensor(np.asarray(labels, np.float64)))
    loss.backward()
    return loss.item(), flat.grad.numpy(), x.grad.numpy()


@pytest.mark.parametrize("in_dim,hidden,B", [(8, [8], 5), (24, [16, 8, 8], 9), (16, [8, 8], 1)])
def test_gradients_match_autograd_and_finite_differences(in_dim, hidden, B):
    rng = np.random.default_rng(1)
    o = M.MlpOracle(in_dim, hidden, init_seed=3, exact=True)
    o.params[0][:] += (0.1 * rng.standard_normal(o.n)).astype(F32)       # non-zero biases too
    pooled = rng.standard_normal((B, in_dim)).astype(F32)
    labels = (rng.random(B) < 0.4).astype(F32)
    loss, g, dp = o.loss_and_grads(0, pooled, labels)
    tl, tg, tdp = _torch_reference(o, pooled, labels)
    assert abs(loss - tl) < 1e-12
    np.testing.assert_allclose(g, tg, rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(dp, tdp, rtol=1e-9, atol=1e-13)
    # central differences on a few coordinates of the parameters
    for i in rng.integers(0, o.n, 6):
        h = 1e-3
        save = o.params[0][i]
        o.params[0][i] = save + F32(h)
        lp = o.loss_and_grads(0, pooled, labels)[0]
        up = float(o.params[0][i])
        o.params[0][i] = save - F32(h)
        lm = o.loss_and_grads(0, pooled, labels)[0]
        dn = float(o.params[0][i])
        o.params[0][i] = save
        assert abs((lp - lm) / (up - dn) - g[i]) < 1e-5 * max(1.0, abs(g[i]))


def test_loss_closed_forms_at_zero_parameters():
    """All parameters zero: every logit is 0, the loss is ln 2, d loss / d logit = (1/2 - y) / B, so the
    output bias gets sum(1/2 - y) / B and everything else zero."""
    o = M.MlpOracle(8, [8], exact=True)
    o.params[0][:] = 0
    y = np.array([1, 0, 0, 1, 0], F32)
    loss, g, dp = o.loss_and_grads(0, np.ones((5, 8), F32), y)
    assert abs(loss - np.log(2)) < 1e-15
    assert abs(g[-1] - np.sum(0.5 - y.astype(np.float64)) / 5) < 1e-15 and not g[:-1].any() and not dp.any()


def test_one_unit_network_by_hand():
    """in = 1... (padded to the smallest legal widths): logit = u * relu(w x) + c; d loss/d w =
    (sigmoid(logit) - y) u x for w x > 0 and 0 otherwise."""
    o = M.MlpOracle(8, [8], exact=True)
    o.params[0][:] = 0
    w, u, c = 0.7, -1.3, 0.2
    o.params[0][0] = w                       # W1[0, 0]
    o.params[0][8 * 8 + 8] = u               # w_out[0]
    o.params[0][-1] = c
    x = np.zeros((2, 8), F32)
    x[0, 0], x[1, 0] = 2.0, -1.0             # second sample is cut by the ReLU
    y = np.array([1.0, 0.0], F32)
    loss, g, dp = o.loss_and_grads(0, x, y)
    w, u, c = float(F32(w)), float(F32(u)), float(F32(c))
    z = np.array([u * w * 2.0 + c, c])
    sig = 1 / (1 + np.exp(-z))
    assert abs(loss - np.mean(np.log1p(np.exp(z)) - y * z)) < 1e-12
    assert abs(g[0] - (sig[0] - 1.0) / 2 * u * 2.0) < 1e-12
    assert abs(dp[0, 0] - (sig[0] - 1.0) / 2 * u * w) < 1e-12 and dp[1, 0] == 0
    assert abs(g[8 * 8 + 8] - (sig[0] - 1.0) / 2 * w * 2.0) < 1e-12


def test_backward_goes_through_the_rounded_weights():
    """The products of the backward pass take the same bf16 weight copies as the forward pass.  All-positive
    network whose inputs and activations are exactly representable, weights 1 + 2^-9 (bf16: 1.0): the gradient of
    the pooled input is then sum_j bf16(dlogit * u_j) * 1.0, not * (1 + 2^-9)."""
    o = M.MlpOracle(8, [8])
    p = o.params[0]
    p[:] = 0
    p[:64] = F32(1 + 2.0 ** -9)              # W1
    u = F32(0.25)
    p[64 + 8:64 + 16] = u                    # w_out
    x = np.full((2, 8), F32(1 + 2.0 ** -9))  # the input is rounded too: bf16 1.0 and 2.0
    x[1] = F32(2 + 2.0 ** -8)
    y = np.array([1.0, 0.0], F32)
    loss, g, dp = o.loss_and_grads(0, x, y)
    x = np.round(x)
    z = np.array([8.0, 16.0]) * 8 * 0.25     # hidden = 8 x (resp. 16), logit = sum of 8 hidden * 0.25
    dlogit = (1 / (1 + np.exp(-z)) - y) / 2
    assert abs(loss - np.mean(np.log1p(np.exp(z)) - y * z)) < 1e-12
    dz = M.bf16_round((dlogit * 0.25).astype(F32)).astype(np.float64)   # per hidden unit, equal for all 8
    assert np.allclose(dp, (8 * dz)[:, None] * np.ones((1, 8)), rtol=1e-12, atol=0)
    # weight gradient of the first layer: x^T dz, exactly
    assert np.allclose(g[:64].reshape(8, 8), np.outer(np.ones(8), np.ones(8)) * (x[0, 0] * dz[0] + x[1, 0] * dz[1]),
                       rtol=1e-12, atol=0)


def _replay_on_sparse_oracle(o_kwargs, grads_per_step, n, W, kstep, k):
    """Feeds recorded dense gradients to the C++ table oracle with every row touched every step."""
    D = 4
    rows = n // D
    t = O.OracleTable(rows, D, n_replicas=W, kstep=kstep, **o_kwargs)
    keys = np.arange(1, rows + 1, dtype=np.uint64)
    off = np.arange(0, rows + 1, dtype=np.uint32)
    return t, keys, off


@pytest.mark.parametrize("W,k,mixed", [(1, 0, False), (1, 1, False), (3, 2, False), (3, 2, True)])
def test_dense_optimizer_equals_the_table_oracle_with_every_row_touched(W, k, mixed):
    """Two independent implementations of Algorithm 2 (numpy here, C++ in the table oracle) must agree
    bit for bit when the table's every row is touched at every step.  `mixed`: replica 0 takes its k-th step
    as a local one, so the merge must add the pending step for the other replicas only."""
    rng = np.random.default_rng(5)
    in_dim, hidden, B = 8, [8], 6                         # 8*8+8+8+1 = 81 parameters -> use the first 80
    kstep = k > 0
    hp = dict(lr=2e-3, beta1=0.9, beta2=0.999, eps=1e-8)
    o = M.MlpOracle(in_dim, hidden, n_replicas=W, kstep=kstep, init_seed=2, **hp)
    n4 = (o.n // 4) * 4
    t, keys, off = _replay_on_sparse_oracle(dict(init_seed=0, **hp), None, n4, W, kstep, k)
    x0 = o.params[0][:n4].reshape(-1, 4)
    assert t.table_load(keys, x0, np.zeros_like(x0), np.full_like(x0, F32(1e-8))) == O.OK
    for s in range(1, 7):
        mode = M.STEP_MERGE_PENDING if (kstep and s % k == 0) else M.STEP_LOCAL
        for j in range(W):
            mode_j = M.STEP_LOCAL if (mixed and j == 0) else mode
            pooled = rng.standard_normal((B, in_dim)).astype(F32)
            labels = (rng.random(B) < 0.5).astype(F32)
            g = o.loss_and_grads(j, pooled, labels)[1].astype(F32)
            o.step(j, pooled, labels, mode_j)
            st, _ = t.pull_pool(j, keys, off)
            assert st == O.OK and t.push_adam(j, g[:n4].reshape(-1, 4), mode_j) == O.OK
        if mode == M.STEP_MERGE_PENDING:
            o.kstep_merge()
            assert t.kstep_merge() == O.OK
        for j in range(W):
            e = t.table_export(j)
            assert np.array_equal(e["x"].reshape(-1), o.params[j][:n4]), (s, j)
            assert np.array_equal(e["m"].reshape(-1), o.m[j][:n4]) and np.array_equal(e["v"].reshape(-1), o.v[j][:n4])
            if kstep:
                assert np.array_equal(e["vhat"].reshape(-1), o.vhat[:n4])


def test_bf16_rounding_points_change_the_result_only_slightly():
    rng = np.random.default_rng(2)
    a = M.MlpOracle(64, [32, 16], init_seed=1, exact=True)
    b = M.MlpOracle(64, [32, 16], init_seed=1, exact=False)
    pooled = rng.standard_normal((32, 64)).astype(F32)
    labels = (rng.random(32) < 0.3).astype(F32)
    la, ga, da = a.loss_and_grads(0, pooled, labels)
    lb, gb, db = b.loss_and_grads(0, pooled, labels)
    assert 0 < abs(la - lb) < 2e-2
    assert np.linalg.norm(ga - gb) / np.linalg.norm(ga) < 3e-2
    assert np.linalg.norm(da - db) / np.linalg.norm(da) < 3e-2


def test_bf16_gradient_option_rounds_the_returned_gradient_only():
    """step(grad_bf16=True): the returned input gradient is the plain one rounded once to bf16 (checked against
    a library's conversion); loss, parameters and moments are those of the plain step."""
    import torch
    rng = np.random.default_rng(5)
    a = M.MlpOracle(48, [24, 8], init_seed=2)
    b = M.MlpOracle(48, [24, 8], init_seed=2)
    for _ in range(2):
        pooled = (0.1 * rng.standard_normal((16, 48))).astype(F32)
        labels = (rng.random(16) < 0.3).astype(F32)
        la, ga = a.step(0, pooled, labels)
        lb, gb = b.step(0, pooled, labels, grad_bf16=True)
        assert la == lb
        assert np.array_equal(gb, torch.from_numpy(ga).to(torch.bfloat16).to(torch.float32).numpy())
        assert (gb != ga).any()
        assert np.array_equal(a.params[0], b.params[0]) and np.array_equal(a.m[0], b.m[0])
        assert np.array_equal(a.v[0], b.v[0])
