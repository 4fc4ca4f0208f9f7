"""Pins for the floating-point part of the CPU oracle: MLP, TD target, loss, backward, optimizers.

The paper prints no worked numeric train step, so these pins are a hand-worked
example in exact dyadic arithmetic, closed forms, finite differences, special
cases that reduce to library routines, and the paper's update equation itself.
"""
import numpy as np
import pytest
import scipy.special
import torch

import oracle
from paper_1801_03138_amd import synth


def _flat(*parts):
    return np.concatenate([np.asarray(p, np.float64).ravel() for p in parts])


# A 2-2-2-2 network worked by hand.  Every value is a dyadic rational, so all
# arithmetic below is exact in binary floating point.  Matrices are [in x out].
W1 = [[1, -1], [2, 1]];      B1 = [0, -1]
W2 = [[1, -2], [5, 5]];      B2 = [-1, 1]
W3 = [[0.5, -1], [7, 7]];    B3 = [0.25, 0.5]
HAND = _flat(W1, B1, W2, B2, W3, B3)
S_HAND, SN_HAND = [[1.0, 1.0]], [[2.0, 0.0]]
# s  = (1,1): z1 = (3,-1) h1 = (3,0); z2 = (2,-5) h2 = (2,0); Q  = (1.25,-1.5)
# s' = (2,0): z1 = (2,-3) h1 = (2,0); z2 = (1,-3) h2 = (1,0); Q' = (0.75,-0.5)


def _hand_cfg(loss, opt=oracle.SGD, lr=1.0, bf16=0):
    return oracle.make_cfg(2, 2, 2, 1, loss=loss, opt=opt, lr=lr, gamma=0.5, bf16=bf16)


def test_forward_hand_worked():
    cfg = _hand_cfg(oracle.MSE)
    Q, h1, h2 = oracle.mlp_forward(cfg, HAND, S_HAND + SN_HAND, want_hidden=True)
    assert Q.tolist() == [[1.25, -1.5], [0.75, -0.5]]
    assert h1.tolist() == [[3, 0], [2, 0]] and h2.tolist() == [[2, 0], [1, 0]]


@pytest.mark.parametrize("bf16", [0, 1])
def test_step_hand_worked_small_error(bf16):
    # a=0: q=1.25, y = 1 + 0.5*0.75 = 1.375, delta = 0.125, loss = 0.0078125 for both losses
    for loss in (oracle.MSE, oracle.HUBER):
        out = oracle.train_step(_hand_cfg(loss, bf16=bf16), HAND, None, None, 0, S_HAND, SN_HAND,
                                [0], [1.0], [0])
        assert out.y.tolist() == [1.375] and out.delta.tolist() == [0.125]
        assert out.loss == 0.0078125
        g = _flat([[-0.0625, 0], [-0.0625, 0]], [-0.0625, 0], [[-0.1875, 0], [0, 0]],
                  [-0.0625, 0], [[-0.25, 0], [0, 0]], [-0.125, 0])
        assert out.grads.tolist() == g.tolist()
        assert out.params.tolist() == (HAND - g).tolist()


def test_step_hand_worked_large_error_and_terminal():
    # a=1: q=-1.5, delta = 2.875.  MSE: loss 4.1328125, slope 2.875.  Huber: loss 2.375, slope 1.
    mse = oracle.train_step(_hand_cfg(oracle.MSE), HAND, None, None, 0, S_HAND, SN_HAND, [1],
                            [1.0], [0])
    hub = oracle.train_step(_hand_cfg(oracle.HUBER), HAND, None, None, 0, S_HAND, SN_HAND, [1],
                            [1.0], [0])
    assert mse.delta.tolist() == [2.875] and mse.loss == 4.1328125 and hub.loss == 2.375
    # dQ = -slope at action 1: dW3[:,1] = h2 * dQ, dz2 = dQ*W3[:,1] masked = (-(-1)*slope, 0)
    g_hub = _flat([[1, 0], [1, 0]], [1, 0], [[3, 0], [0, 0]], [1, 0], [[0, -2], [0, 0]], [0, -1])
    assert hub.grads.tolist() == g_hub.tolist()
    assert mse.grads.tolist() == (2.875 * g_hub).tolist()
    # terminal: the target is the reward alone, whatever s' is
    term = oracle.train_step(_hand_cfg(oracle.MSE), HAND, None, None, 0, S_HAND, [[1e6, -1e6]],
                             [0], [1.0], [1])
    assert term.y.tolist() == [1.0] and term.delta.tolist() == [-0.25]


def test_forward_reduces_to_affine_product_when_relu_is_identity():
    """All-positive inputs, weights and biases: the net is three affine maps (library matmul)."""
    D, H, A, n = 27, 64, 8, 50
    g = np.random.default_rng(0)
    p = g.uniform(0.01, 1.0, oracle.param_count(D, H, A))
    X = g.uniform(0.01, 2.0, (n, D))
    w1, b1, w2, b2, w3, b3 = synth.split_params(p, D, H, A)
    want = ((X @ w1 + b1) @ w2 + b2) @ w3 + b3
    got = oracle.mlp_forward(oracle.make_cfg(D, H, A, n), p, X)
    np.testing.assert_allclose(got, want, rtol=1e-13)


def test_forward_against_library_network():
    """Signed weights: compare with torch.nn.functional on float64 (library routine)."""
    D, H, A, n = 27, 64, 8, 40
    p = synth.init_params(D, H, A, seed=3).astype(np.float64)
    X = np.random.default_rng(1).standard_normal((n, D))
    w1, b1, w2, b2, w3, b3 = [torch.from_numpy(np.array(x)) for x in synth.split_params(p, D, H, A)]
    F = torch.nn.functional
    x = torch.from_numpy(X)
    want = F.linear(F.relu(F.linear(F.relu(F.linear(x, w1.T, b1)), w2.T, b2)), w3.T, b3).numpy()
    got, h1, h2 = oracle.mlp_forward(oracle.make_cfg(D, H, A, n), p, X, want_hidden=True)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    assert (h1 >= 0).all() and (h2 >= 0).all() and (h1 == 0).any() and (h1 > 0).any()


def _random_problem(D, H, A, B, seed, reward_scale=1.0):
    p = synth.init_params(D, H, A, seed=seed).astype(np.float64)
    rows = synth.experiences(B, D, A, 0.25, seed=seed)
    return p, rows["s"].astype(np.float64), rows["s_next"].astype(np.float64), rows["a"], \
        rows["r"].astype(np.float64) * reward_scale, rows["term"]


def test_target_selection_and_loss_definitions():
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 0)
    cfg = oracle.make_cfg(D, H, A, B, loss=oracle.HUBER, lr=0.0, gamma=0.99)
    out = oracle.train_step(cfg, p, None, None, 0, S, Sn, a, r, term)
    assert term.any() and not term.all()
    # Q and Q' are the forward pass on s and s'
    assert np.array_equal(out.Q, oracle.mlp_forward(cfg, p, S))
    assert np.array_equal(out.Qn, oracle.mlp_forward(cfg, p, Sn))
    # y = r + gamma (1 - terminal) max_a Q'
    np.testing.assert_allclose(out.y, r + 0.99 * (1 - term) * out.Qn.max(axis=1), rtol=1e-15)
    # Q(s,a) by two-dimensional indexing equals entry i*A + a_i of the flattened output
    np.testing.assert_allclose(out.y - out.delta, out.Q[np.arange(B), a], rtol=0, atol=1e-15)
    assert np.array_equal(out.Q.ravel()[np.arange(0, B * A, A) + a], out.Q[np.arange(B), a])
    # mean Huber loss (library routine); some errors beyond the threshold are present
    assert (np.abs(out.delta) > 1).any() and (np.abs(out.delta) < 1).any()
    np.testing.assert_allclose(out.loss, scipy.special.huber(1.0, out.delta).mean(), rtol=1e-14)
    # lr = 0 leaves the parameters untouched while loss and gradients are still reported
    assert np.array_equal(out.params, p) and np.abs(out.grads).max() > 0
    # the loss with frozen targets is the same number
    np.testing.assert_allclose(oracle.loss_fixed_targets(cfg, p, S, a, out.y), out.loss, rtol=1e-14)
    mse = oracle.train_step(oracle.make_cfg(D, H, A, B, loss=oracle.MSE, lr=0.0), p, None, None,
                            0, S, Sn, a, r, term)
    np.testing.assert_allclose(mse.loss, (0.5 * mse.delta ** 2).mean(), rtol=1e-14)


def test_huber_equals_mse_for_small_errors():
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 1, reward_scale=0.01)
    hub = oracle.train_step(oracle.make_cfg(D, H, A, B, loss=oracle.HUBER), p, None, None, 0, S,
                            Sn, a, r, term)
    mse = oracle.train_step(oracle.make_cfg(D, H, A, B, loss=oracle.MSE), p, None, None, 0, S,
                            Sn, a, r, term)
    assert np.abs(hub.delta).max() < 1
    assert np.array_equal(hub.grads, mse.grads) and hub.loss == mse.loss
    assert np.array_equal(hub.params, mse.params)


def test_terminal_rows_ignore_next_state():
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 2)
    cfg = oracle.make_cfg(D, H, A, B)
    ref = oracle.train_step(cfg, p, None, None, 0, S, Sn, a, r, term)
    poisoned = Sn.copy()
    poisoned[term == 1] = 1e4
    out = oracle.train_step(cfg, p, None, None, 0, S, poisoned, a, r, term)
    assert np.array_equal(out.y, ref.y) and np.array_equal(out.params, ref.params)
    assert np.array_equal(out.y[term == 1], r[term == 1])


def _preactivation_margin(p, X, D, H, A):
    w1, b1, w2, b2, _, _ = synth.split_params(p, D, H, A)
    z1 = X @ w1 + b1
    z2 = np.maximum(z1, 0) @ w2 + b2
    return min(np.abs(z1).min(), np.abs(z2).min())


def test_gradients_match_finite_differences():
    """Central differences of the frozen-target loss on 300 random parameters (Tiny-sized net)."""
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 4)
    assert _preactivation_margin(p, S, D, H, A) > 2e-5
    for loss in (oracle.HUBER, oracle.MSE):
        cfg = oracle.make_cfg(D, H, A, B, loss=loss, lr=0.0)
        out = oracle.train_step(cfg, p, None, None, 0, S, Sn, a, r, term)
        assert np.abs(np.abs(out.delta) - 1).min() > 1e-3
        g = np.random.default_rng(5)
        # every layer is covered: pick from each parameter block
        sizes = [D * H, H, H * H, H, H * A, A]
        offs = np.concatenate([[0], np.cumsum(sizes)])
        picks = np.concatenate([offs[b] + g.choice(sizes[b], min(sizes[b], 50), replace=False)
                                for b in range(6)])
        h = 1e-6
        scale = np.abs(out.grads).max()
        for k in picks:
            pp, pm = p.copy(), p.copy()
            pp[k] += h
            pm[k] -= h
            fd = (oracle.loss_fixed_targets(cfg, pp, S, a, out.y)
                  - oracle.loss_fixed_targets(cfg, pm, S, a, out.y)) / (2 * h)
            assert abs(fd - out.grads[k]) <= 1e-6 * scale + 1e-6 * abs(fd), (k, fd, out.grads[k])


def test_one_sample_step_is_the_papers_update_equation():
    """B=1, half-squared error, SGD, non-terminal: w += alpha * delta * grad_w Q_w(s,a)."""
    D, H, A = 27, 64, 8
    p, S, Sn, a, r, term = _random_problem(D, H, A, 1, 6)
    term[:] = 0
    alpha = 0.05
    cfg = oracle.make_cfg(D, H, A, 1, loss=oracle.MSE, opt=oracle.SGD, lr=alpha, gamma=0.9)
    assert _preactivation_margin(p, S, D, H, A) > 2e-5
    out = oracle.train_step(cfg, p, None, None, 0, S, Sn, a, r, term)
    qn = oracle.mlp_forward(cfg, p, Sn)
    delta = r[0] + 0.9 * qn.max() - oracle.mlp_forward(cfg, p, S)[0, a[0]]
    np.testing.assert_allclose(out.delta[0], delta, rtol=1e-14)
    # grad_w Q_w(s,a) by central differences of the forward pass alone
    g = np.random.default_rng(7)
    h = 1e-6
    step = out.params - p
    for k in g.choice(p.size, 300, replace=False):
        pp, pm = p.copy(), p.copy()
        pp[k] += h
        pm[k] -= h
        dq = (oracle.mlp_forward(cfg, pp, S)[0, a[0]] - oracle.mlp_forward(cfg, pm, S)[0, a[0]]) / (2 * h)
        assert abs(step[k] - alpha * delta * dq) <= 1e-8 * np.abs(step).max(), k
    assert np.abs(step).max() > 0


def test_untaken_actions_get_no_output_gradient():
    D, H, A, B = 5, 4, 6, 3
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 8)
    a[:] = [1, 4, 1]
    out = oracle.train_step(oracle.make_cfg(D, H, A, B), p, None, None, 0, S, Sn, a, r, term)
    gW3 = synth.split_params(out.grads, D, H, A)[4]
    gb3 = synth.split_params(out.grads, D, H, A)[5]
    assert not gW3[:, [0, 2, 3, 5]].any() and not gb3[[0, 2, 3, 5]].any()
    assert gb3[1] != 0 and gb3[4] != 0


def test_sgd_step_is_minus_lr_times_gradient():
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 9)
    out = oracle.train_step(oracle.make_cfg(D, H, A, B, lr=1e-3), p, None, None, 0, S, Sn, a, r, term)
    np.testing.assert_allclose(out.params, p - 1e-3 * out.grads, rtol=1e-15)


def test_adam_first_step_closed_form():
    """From zero moments the first Adam step is -lr * g / (|g| + eps), and t becomes 1."""
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 10)
    lr, eps = 1e-4, 1e-8
    out = oracle.train_step(oracle.make_cfg(D, H, A, B, opt=oracle.ADAM, lr=lr, eps=eps), p, None,
                            None, 0, S, Sn, a, r, term)
    g = out.grads
    assert out.t == 1
    np.testing.assert_allclose(out.params - p, -lr * g / (np.abs(g) + eps), rtol=1e-9, atol=1e-20)
    np.testing.assert_allclose(out.m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(out.v, 0.001 * g * g, rtol=1e-9)


def test_adam_bias_correction_with_constant_gradient_history():
    """If the moments are those of t-1 steps of a constant gradient g, step t again moves by -lr g/(|g|+eps)."""
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 11)
    lr, eps, b1, b2, t_prev = 1e-4, 1e-8, 0.9, 0.999, 5
    g = oracle.train_step(oracle.make_cfg(D, H, A, B, lr=0.0), p, None, None, 0, S, Sn, a, r,
                          term).grads
    m0 = g * (1 - b1 ** t_prev)
    v0 = g * g * (1 - b2 ** t_prev)
    out = oracle.train_step(oracle.make_cfg(D, H, A, B, opt=oracle.ADAM, lr=lr, eps=eps, beta1=b1,
                                            beta2=b2), p, m0, v0, t_prev, S, Sn, a, r, term)
    assert out.t == t_prev + 1
    np.testing.assert_allclose(out.params - p, -lr * g / (np.abs(g) + eps), rtol=1e-8, atol=1e-20)


def test_update_rule_alone_hand_worked():
    """oracle.opt_apply on given gradients, every number worked by hand in dyadic arithmetic.
    SGD: w - lr g.  Adam with beta1 = 1/2, beta2 = 3/4, eps = 0, lr = 1, second step (t: 1 -> 2)
    from m = 2, v = 4 with g = 4:  m' = 1 + 2 = 3,  v' = 3 + 4 = 7,  1 - beta1^2 = 3/4,
    1 - beta2^2 = 7/16,  m^ = 4,  v^ = 16,  step = 4 / sqrt(16) = 1."""
    sgd = oracle.make_cfg(2, 2, 2, 1, opt=oracle.SGD, lr=0.25)
    p, m, v, t = oracle.opt_apply(sgd, [1.0, -2.0, 0.5], None, None, 7, [4.0, -8.0, 0.0])
    assert p.tolist() == [0.0, 0.0, 0.5] and m is None and v is None and t == 7
    adam = oracle.make_cfg(2, 2, 2, 1, opt=oracle.ADAM, lr=1.0, beta1=0.5, beta2=0.75, eps=0.0)
    p, m, v, t = oracle.opt_apply(adam, [10.0, 10.0], [2.0, -2.0], [4.0, 4.0], 1, [4.0, -4.0])
    assert t == 2 and m.tolist() == [3.0, -3.0] and v.tolist() == [7.0, 7.0]
    assert p.tolist() == [9.0, 11.0]
    # eps sits outside the root: with eps = 4 the same step is 4 / (4 + 4) = 1/2
    adam_eps = oracle.make_cfg(2, 2, 2, 1, opt=oracle.ADAM, lr=1.0, beta1=0.5, beta2=0.75, eps=4.0)
    p, _, _, _ = oracle.opt_apply(adam_eps, [10.0, 10.0], [2.0, -2.0], [4.0, 4.0], 1, [4.0, -4.0])
    assert p.tolist() == [9.5, 10.5]
    # a zero gradient from zero moments does not move the weight (0 / (0 + eps))
    p, m, v, t = oracle.opt_apply(oracle.make_cfg(2, 2, 2, 1, opt=oracle.ADAM), [3.0], [0.0], [0.0], 0, [0.0])
    assert p.tolist() == [3.0] and m.tolist() == [0.0] and v.tolist() == [0.0] and t == 1


def test_train_step_applies_the_update_rule_to_its_gradient():
    D, H, A, B = 27, 64, 8, 32
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 13)
    g0 = np.random.default_rng(3)
    m0, v0 = g0.standard_normal(p.size) * 1e-3, g0.random(p.size) * 1e-5
    for opt in (oracle.SGD, oracle.ADAM):
        cfg = oracle.make_cfg(D, H, A, B, opt=opt, lr=1e-3)
        out = oracle.train_step(cfg, p, m0, v0, 4, S, Sn, a, r, term)
        q, m, v, t = oracle.opt_apply(cfg, p, m0, v0, 4, out.grads)
        assert np.array_equal(q, out.params)
        if opt == oracle.ADAM:
            assert t == out.t == 5 and np.array_equal(m, out.m) and np.array_equal(v, out.v)


# ----------------------------------------------------------------------------- bf16
def test_bf16_rounding_against_library_and_ties():
    x = np.random.default_rng(0).standard_normal(20000).astype(np.float32)
    x = np.concatenate([x, x * 1e-30, x * 1e30, [0.0, -0.0, np.inf, -np.inf]]).astype(np.float32)
    want = synth.f32_to_bf16_bits(x)
    got = np.array([oracle.bf16_bits(float(v)) for v in x], np.uint16)
    assert np.array_equal(got, want)
    # ties go to the even neighbour: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.round_bf16(1 + 2.0 ** -8) == 1.0
    assert oracle.round_bf16(1 + 3 * 2.0 ** -8) == 1 + 2.0 ** -6
    assert oracle.round_bf16(1 + 2.0 ** -8 + 2.0 ** -20) == 1 + 2.0 ** -7
    assert np.isnan(oracle.round_bf16(float("nan")))


def test_bf16_mode_rounds_weights_but_not_master_copy():
    """A weight of 1 + 2^-10 acts as 1.0 in the products, yet the update starts from the unrounded value."""
    p = HAND.copy()
    p[0] = 1 + 2.0 ** -10
    out = oracle.train_step(_hand_cfg(oracle.MSE, bf16=1), p, None, None, 0, S_HAND, SN_HAND, [0],
                            [1.0], [0])
    ref = oracle.train_step(_hand_cfg(oracle.MSE, bf16=0), HAND, None, None, 0, S_HAND, SN_HAND,
                            [0], [1.0], [0])
    assert np.array_equal(out.Q, ref.Q) and np.array_equal(out.grads, ref.grads)
    assert out.params[0] == p[0] - ref.grads[0]
    exact = oracle.train_step(_hand_cfg(oracle.MSE, bf16=0), p, None, None, 0, S_HAND, SN_HAND,
                              [0], [1.0], [0])
    assert not np.array_equal(exact.Q, ref.Q)


def test_bf16_mode_rounds_the_pre_activation_gradients():
    """Hand-worked backward pass whose pre-activation gradients are not bf16 numbers (bf16 keeps
    8 significant bits, round to nearest even).  Network HAND, s = (1,3), s' = (2,0), action 0:
      z1 = (7,1) h1 = (7,1); z2 = (11,-8) h2 = (11,0); Q = (5.75,-10.5); max Q' = 0.75
      r = 5.5 + 3*2^-12: y = r + 0.5*0.75, delta = y - 5.75 = 2^-3 + 3*2^-12 =: e (|e| < 1)
      dQ = (-e, 0);  gW3 = h2^T dQ = [[-11 e, 0], [0, 0]], gb3 = (-e, 0)      (not rounded)
      dZ2 = (-e * 0.5, 0) = (-(2^-4)(1 + 3*2^-9), 0) -> bf16 -(2^-4)(1 + 2^-7) =: -p  (rounds up)
      gW2 = h1^T dZ2 = [[-7 p, 0], [-p, 0]], gb2 = (-p, 0)
      dZ1 = (-p * 1, -p * 5); 5 p = 2^-2 (1 + 2^-2 + 2^-7 + 2^-9) -> bf16 2^-2 (1 + 2^-2 + 2^-7) =: q
      gW1 = s^T dZ1 = [[-p, -q], [-3 p, -3 q]], gb1 = (-p, -q)."""
    e = 2.0 ** -3 + 3 * 2.0 ** -12
    pp = 2.0 ** -4 * (1 + 2.0 ** -7)
    qq = 2.0 ** -2 * (1 + 2.0 ** -2 + 2.0 ** -7)
    r = 5.5 + 3 * 2.0 ** -12
    for loss in (oracle.MSE, oracle.HUBER):
        out = oracle.train_step(_hand_cfg(loss, bf16=1), HAND, None, None, 0, [[1.0, 3.0]], SN_HAND,
                                [0], [r], [0])
        assert out.Q.tolist() == [[5.75, -10.5]] and out.delta.tolist() == [e]
        g = _flat([[-pp, -qq], [-3 * pp, -3 * qq]], [-pp, -qq], [[-7 * pp, 0], [-pp, 0]], [-pp, 0],
                  [[-11 * e, 0], [0, 0]], [-e, 0])
        assert out.grads.tolist() == g.tolist()
        assert out.params.tolist() == (HAND - g).tolist()
    # without mixed precision nothing is rounded: dZ2 = -e/2, dZ1 = (-e/2, -5e/2)
    exact = oracle.train_step(_hand_cfg(oracle.MSE, bf16=0), HAND, None, None, 0, [[1.0, 3.0]],
                              SN_HAND, [0], [r], [0])
    g = _flat([[-e / 2, -5 * e / 2], [-3 * e / 2, -15 * e / 2]], [-e / 2, -5 * e / 2],
              [[-7 * e / 2, 0], [-e / 2, 0]], [-e / 2, 0], [[-11 * e, 0], [0, 0]], [-e, 0])
    assert exact.grads.tolist() == g.tolist()


def test_bf16_mode_rounds_hidden_activations():
    D, H, A, B = 27, 64, 8, 16
    p, S, Sn, a, r, term = _random_problem(D, H, A, B, 12)
    S = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(S)).astype(np.float64)
    cfg = oracle.make_cfg(D, H, A, B, bf16=1)
    Q, h1, h2 = oracle.mlp_forward(cfg, p, S, want_hidden=True)
    for h in (h1, h2):
        f = h.astype(np.float32)
        assert np.array_equal(f.astype(np.float64), h)
        assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(f)), f)
    # mixed precision stays close to the exact network
    exact = oracle.mlp_forward(oracle.make_cfg(D, H, A, B), p, S)
    assert 0 < np.abs(Q - exact).max() < 2e-2 * np.abs(exact).max()


# ---------------------------------------------------------------- frozen target network
# A second 2-2-2-2 network as the target; s' = (2,0):
#   z1 = (2*2, 2*(-2)) + (1, 0) = (5,-4) h1 = (5,0); z2 = (5*1 - 1, 5*0 + 0.5) = (4, 0.5) h2 = (4, 0.5)
#   Q' = (4*0.25 + 0.5*2 + 0, 4*1 + 0.5*(-2) - 0.5) = (2, 2.5)  ->  max = 2.5
TW1 = [[2, -2], [3, 3]];     TB1 = [1, 0]
TW2 = [[1, 0], [9, 9]];      TB2 = [-1, 0.5]
TW3 = [[0.25, 1], [2, -2]];  TB3 = [0, -0.5]
TARGET = _flat(TW1, TB1, TW2, TB2, TW3, TB3)


def test_target_network_hand_worked():
    """Q(s', .) comes from the target network, everything else from the trained one."""
    cfg = _hand_cfg(oracle.MSE)
    Qt = oracle.mlp_forward(cfg, TARGET, SN_HAND)
    assert Qt.tolist() == [[2.0, 2.5]]
    out = oracle.train_step(cfg, HAND, None, None, 0, S_HAND, SN_HAND, [0], [1.0], [0], target=TARGET)
    # y = 1 + 0.5 * 2.5 = 2.25, q = Q(s,0) = 1.25 from the trained network, delta = 1
    assert out.Qn.tolist() == [[2.0, 2.5]] and out.Q.tolist() == [[1.25, -1.5]]
    assert out.y.tolist() == [2.25] and out.delta.tolist() == [1.0] and out.loss == 0.5
    # gradient = -delta * dQ(s,0)/dw of the trained network: 8x the small-error case (delta 0.125)
    g = 8 * _flat([[-0.0625, 0], [-0.0625, 0]], [-0.0625, 0], [[-0.1875, 0], [0, 0]], [-0.0625, 0],
                  [[-0.25, 0], [0, 0]], [-0.125, 0])
    assert out.grads.tolist() == g.tolist()
    assert out.params.tolist() == (HAND - g).tolist()


def test_target_equal_to_trained_network_changes_nothing():
    D, H, A, n = 9, 16, 5, 12
    rows = synth.experiences(n, D, A, 0.2, seed=3)
    p = synth.init_params(D, H, A, 2).astype(np.float64)
    cfg = oracle.make_cfg(D, H, A, n, loss=oracle.HUBER, opt=oracle.ADAM, lr=1e-3)
    args = (rows["s"], rows["s_next"], rows["a"], rows["r"], rows["term"])
    a = oracle.train_step(cfg, p, None, None, 0, *args)
    b = oracle.train_step(cfg, p, None, None, 0, *args, target=p)
    for f in ("params", "Q", "Qn", "y", "delta", "grads", "m", "v"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f


def test_targets_depend_on_the_target_network_only():
    """y = r + gamma (1 - terminal) max_a Q_target(s', a): moving the trained weights leaves y
    alone, moving the target weights leaves Q(s, .) alone; no gradient reaches the target."""
    D, H, A, n = 9, 16, 5, 12
    rows = synth.experiences(n, D, A, 0.2, seed=4)
    p = synth.init_params(D, H, A, 2).astype(np.float64)
    q = synth.init_params(D, H, A, 7).astype(np.float64)
    tgt = synth.init_params(D, H, A, 9).astype(np.float64)
    cfg = oracle.make_cfg(D, H, A, n, loss=oracle.MSE, opt=oracle.SGD, lr=1e-2)
    args = (rows["s"], rows["s_next"], rows["a"], rows["r"], rows["term"])
    a = oracle.train_step(cfg, p, None, None, 0, *args, target=tgt)
    b = oracle.train_step(cfg, q, None, None, 0, *args, target=tgt)
    c = oracle.train_step(cfg, p, None, None, 0, *args, target=q)
    assert np.array_equal(a.y, b.y) and np.array_equal(a.Qn, b.Qn)
    assert np.array_equal(a.Q, c.Q) and not np.array_equal(a.y, c.y)
    want_y = rows["r"] + cfg.gamma * (1 - rows["term"]) * oracle.mlp_forward(cfg, tgt, rows["s_next"]).max(1)
    assert np.allclose(a.y, want_y, rtol=1e-14, atol=0)
    # the step is plain SGD on L(w) with y held constant: finite differences of that loss
    rng = np.random.default_rng(0)
    for k in rng.choice(len(p), 40, replace=False):
        e = np.zeros_like(p); e[k] = 1e-5
        fd = (oracle.loss_fixed_targets(cfg, p + e, rows["s"], rows["a"], a.y) -
              oracle.loss_fixed_targets(cfg, p - e, rows["s"], rows["a"], a.y)) / 2e-5
        assert abs(fd - a.grads[k]) <= 1e-7 * max(1.0, abs(fd))


def test_target_sync_schedule():
    new, old = np.arange(4.0), np.zeros(4)
    assert oracle.target_after_step(old, new, 10, 5).tolist() == new.tolist()
    assert oracle.target_after_step(old, new, 11, 5).tolist() == old.tolist()
    assert oracle.target_after_step(old, new, 7, 0).tolist() == old.tolist()


# ---------------------------------------------------------------- dueling head
def _dueling_numpy(p, X, D, H, A):
    """The dueling network written with library matmuls: shared layer, then a value stream and
    an advantage stream of H/2 units each, Q = V + A - mean A (Deep Q-Network Model)."""
    p = np.asarray(p, np.float64)
    o = 0
    W1 = p[o:o + D * H].reshape(D, H); o += D * H
    b1 = p[o:o + H]; o += H
    W2 = p[o:o + H * H].reshape(H, H); o += H * H
    b2 = p[o:o + H]; o += H
    W3 = p[o:o + H * (A + 1)].reshape(H, A + 1); o += H * (A + 1)
    b3 = p[o:o + A + 1]
    h1 = np.maximum(np.asarray(X, np.float64) @ W1 + b1, 0)
    hv = np.maximum(h1 @ W2[:, :H // 2] + b2[:H // 2], 0)       # value stream
    ha = np.maximum(h1 @ W2[:, H // 2:] + b2[H // 2:], 0)       # advantage stream
    V = hv @ W3[:H // 2, 0] + b3[0]
    Adv = ha @ W3[H // 2:, 1:] + b3[1:]
    return V[:, None] + Adv - Adv.mean(1, keepdims=True), V


def test_dueling_forward_hand_worked():
    # first two layers of the second hand-worked network: s = (1,1) gives h2 = (14, 9.5),
    # s' = (2,0) gives h2 = (4, 0.5); unit 0 is the value stream, unit 1 the advantage stream.
    # V = 0.5 h2[0] + 0.25; A = (h2[1] + 0.5, -0.5 h2[1] - 1).  The 99s are the structural zeros.
    p = _flat(TW1, TB1, TW2, TB2, [[0.5, 99, 99], [99, 1, -0.5]], [0.25, 0.5, -1])
    cfg = oracle.make_cfg(2, 2, 2, 1, loss=oracle.MSE, opt=oracle.SGD, lr=1.0, gamma=0.5, dueling=1)
    Q, h1, h2 = oracle.mlp_forward(cfg, p, S_HAND + SN_HAND, want_hidden=True)
    assert h2.tolist() == [[14, 9.5], [4, 0.5]]
    # s: V = 7.25, A = (10, -5.75), mean 2.125; s': V = 2.25, A = (1, -1.25), mean -0.125
    assert Q.tolist() == [[15.125, -0.625], [3.375, 1.125]]


def test_dueling_head_identities():
    D, H, A, n = 9, 16, 5, 40
    rows = synth.experiences(n, D, A, 0.2, seed=11)
    p = synth.init_params(D, H, A + 1, 3).astype(np.float64)
    cfg = oracle.make_cfg(D, H, A, n, loss=oracle.HUBER, opt=oracle.SGD, lr=1e-2, dueling=1)
    Q = oracle.mlp_forward(cfg, p, rows["s"])
    want, V = _dueling_numpy(p, rows["s"], D, H, A)
    assert np.allclose(Q, want, rtol=1e-13, atol=1e-13)
    assert np.allclose(Q.mean(1), V, rtol=1e-13, atol=1e-13)          # mean_a Q(s, a) = V(s)
    # weights between the streams do not exist: changing them changes nothing
    q = p.copy()
    oW3 = D * H + H + H * H + H
    W3 = q[oW3:oW3 + H * (A + 1)].reshape(H, A + 1)
    W3[H // 2:, 0] += 5.0
    W3[:H // 2, 1:] -= 3.0
    assert np.array_equal(oracle.mlp_forward(cfg, q, rows["s"]), Q)
    a = oracle.train_step(cfg, p, None, None, 0, rows["s"], rows["s_next"], rows["a"], rows["r"], rows["term"])
    g3 = a.grads[oW3:oW3 + H * (A + 1)].reshape(H, A + 1)
    assert not g3[H // 2:, 0].any() and not g3[:H // 2, 1:].any()
    assert g3[:H // 2, 0].any() and g3[H // 2:, 1:].any()
    # the advantage gradients of a sample sum to zero over the actions, the value gradient is dQ
    gb3 = a.grads[oW3 + H * (A + 1):]
    assert abs(gb3[1:].sum()) < 1e-15 and abs(gb3[0] - (-np.clip(a.delta, -1, 1) / n).sum()) < 1e-15


def test_dueling_gradients_match_finite_differences():
    D, H, A, n = 7, 8, 4, 30
    rows = synth.experiences(n, D, A, 0.2, seed=12)
    p = synth.init_params(D, H, A + 1, 4).astype(np.float64)
    cfg = oracle.make_cfg(D, H, A, n, loss=oracle.HUBER, opt=oracle.SGD, lr=1e-2, dueling=1)
    out = oracle.train_step(cfg, p, None, None, 0, rows["s"], rows["s_next"], rows["a"], rows["r"], rows["term"])
    assert np.allclose(out.params, p - 1e-2 * out.grads, rtol=0, atol=1e-18)
    h = 1e-5
    for k in range(len(p)):
        e = np.zeros_like(p); e[k] = h
        fd = (oracle.loss_fixed_targets(cfg, p + e, rows["s"], rows["a"], out.y) -
              oracle.loss_fixed_targets(cfg, p - e, rows["s"], rows["a"], out.y)) / (2 * h)
        assert abs(fd - out.grads[k]) <= 2e-7 * max(1.0, abs(fd)), k


def test_dueling_with_one_action_is_the_value_stream_alone():
    """A = 1: the advantage cancels, Q = V, and the step is that of a plain D-H-H-1 network whose
    last layer sees the value stream only."""
    D, H, n = 6, 8, 20
    rows = synth.experiences(n, D, 1, 0.2, seed=13)
    p = synth.init_params(D, H, 2, 5).astype(np.float64)
    cfg = oracle.make_cfg(D, H, 1, n, loss=oracle.MSE, opt=oracle.SGD, lr=1e-2, dueling=1)
    plain = oracle.make_cfg(D, H, 1, n, loss=oracle.MSE, opt=oracle.SGD, lr=1e-2)
    oW3 = D * H + H + H * H + H
    W3 = p[oW3:oW3 + 2 * H].reshape(H, 2)
    w_plain = W3[:, 0].copy(); w_plain[H // 2:] = 0
    q = np.concatenate([p[:oW3], w_plain, p[oW3 + 2 * H:oW3 + 2 * H + 1]])
    assert np.allclose(oracle.mlp_forward(cfg, p, rows["s"]), oracle.mlp_forward(plain, q, rows["s"]),
                       rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- two hidden widths
def _two_width_problem(D, H, G, A, n, seed, dueling):
    rows = synth.experiences(n, D, A, 0.2, seed=seed)
    p = synth.init_params(D, H, A + (1 if dueling else 0), seed, hidden2=G).astype(np.float64)
    return p, rows


def test_two_widths_forward_against_library_network():
    """D -> H -> G -> A with H != G: torch.nn.functional in float64 (library routine), and the
    hidden activations have the two different widths."""
    D, H, G, A, n = 7, 8, 12, 3, 25
    p, rows = _two_width_problem(D, H, G, A, n, 3, False)
    w1, b1, w2, b2, w3, b3 = [torch.from_numpy(np.array(x)) for x in synth.split_params(p, D, H, A, hidden2=G)]
    F = torch.nn.functional
    x = torch.from_numpy(rows["s"].astype(np.float64))
    want = F.linear(F.relu(F.linear(F.relu(F.linear(x, w1.T, b1)), w2.T, b2)), w3.T, b3).numpy()
    cfg = oracle.make_cfg(D, H, A, n, hidden2=G)
    got, h1, h2 = oracle.mlp_forward(cfg, p, rows["s"], want_hidden=True)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    assert h1.shape == (n, H) and h2.shape == (n, G)
    assert oracle.cfg_param_count(cfg) == D * H + H + H * G + G + G * A + A == p.size
    # hidden2 equal to hidden is the same network as hidden2 = 0
    q = synth.init_params(D, H, A, 5).astype(np.float64)
    a = oracle.mlp_forward(oracle.make_cfg(D, H, A, n), q, rows["s"])
    b = oracle.mlp_forward(oracle.make_cfg(D, H, A, n, hidden2=H), q, rows["s"])
    assert np.array_equal(a, b)


@pytest.mark.parametrize("dueling", [0, 1])
def test_two_widths_gradients_match_finite_differences(dueling):
    """Every parameter of a D-H-G-A network with H != G (plain and dueling head) against central
    differences of the frozen-target loss; then the SGD step is -lr times that gradient."""
    D, H, G, A, n = 5, 4, 6, 3, 20
    p, rows = _two_width_problem(D, H, G, A, n, 21, dueling)
    cfg = oracle.make_cfg(D, H, A, n, loss=oracle.HUBER, opt=oracle.SGD, lr=1e-2, dueling=dueling, hidden2=G)
    out = oracle.train_step(cfg, p, None, None, 0, rows["s"], rows["s_next"], rows["a"], rows["r"], rows["term"])
    assert np.allclose(out.params, p - 1e-2 * out.grads, rtol=0, atol=1e-18)
    assert np.abs(np.abs(out.delta) - 1).min() > 1e-4
    w1, b1, w2, b2, _, _ = synth.split_params(p, D, H, A + dueling, hidden2=G)
    z1 = rows["s"] @ w1 + b1
    assert min(np.abs(z1).min(), np.abs(np.maximum(z1, 0) @ w2 + b2).min()) > 1e-4
    h = 1e-6
    for k in range(len(p)):
        e = np.zeros_like(p); e[k] = h
        fd = (oracle.loss_fixed_targets(cfg, p + e, rows["s"], rows["a"], out.y) -
              oracle.loss_fixed_targets(cfg, p - e, rows["s"], rows["a"], out.y)) / (2 * h)
        assert abs(fd - out.grads[k]) <= 2e-7 * max(1.0, abs(fd)), k


def test_two_widths_dueling_streams_split_the_second_layer():
    """The paper's shape in small: shared layer H, then a value stream and an advantage stream of
    G/2 units each (Deep Q-Network Model).  Library matmuls stream by stream; mean_a Q = V."""
    D, H, G, A, n = 6, 4, 10, 5, 30
    p, rows = _two_width_problem(D, H, G, A, n, 8, True)
    W1, b1, W2, b2, W3, b3 = synth.split_params(p, D, H, A + 1, hidden2=G)
    h1 = np.maximum(rows["s"].astype(np.float64) @ W1 + b1, 0)
    hv = np.maximum(h1 @ W2[:, :G // 2] + b2[:G // 2], 0)
    ha = np.maximum(h1 @ W2[:, G // 2:] + b2[G // 2:], 0)
    V = hv @ W3[:G // 2, 0] + b3[0]
    Adv = ha @ W3[G // 2:, 1:] + b3[1:]
    want = V[:, None] + Adv - Adv.mean(1, keepdims=True)
    cfg = oracle.make_cfg(D, H, A, n, dueling=1, hidden2=G)
    Q = oracle.mlp_forward(cfg, p, rows["s"])
    assert np.allclose(Q, want, rtol=1e-13, atol=1e-13) and np.allclose(Q.mean(1), V, rtol=1e-13, atol=1e-13)
    out = oracle.train_step(cfg, p, None, None, 0, rows["s"], rows["s_next"], rows["a"], rows["r"], rows["term"])
    g3 = synth.split_params(out.grads, D, H, A + 1, hidden2=G)[4]
    assert not g3[G // 2:, 0].any() and not g3[:G // 2, 1:].any()
    assert g3[:G // 2, 0].any() and g3[G // 2:, 1:].any()
