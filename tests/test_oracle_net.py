"""Pins for the oracle's network arithmetic: forward, backward, TD loss (Eq. 1), RMSProp (Appendix B).

None of these compares the oracle with itself: they use closed forms, finite differences, brute
force, invariants, and PyTorch's CPU library routines as a third opinion.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from datagen import synth
from oracle import dqn as odqn

TINY = odqn.make_desc((2, 12, 12), [(3, 4, 2), (4, 3, 1)], [8, 3])   # 12->5->3 ; 4*3*3=36 -> 8 -> 3


def split_params(desc, theta):
    """Blob -> list of (w, b) tensors in layer order, shaped like the library's layout."""
    out, off = [], 0
    c, h, w = desc.in_c, desc.in_h, desc.in_w
    for i in range(desc.n_conv):
        o, k, s = desc.conv_out[i], desc.conv_k[i], desc.conv_s[i]
        n = o * c * k * k
        out.append((theta[off:off + n].reshape(o, c, k, k), theta[off + n:off + n + o]))
        off += n + o
        c, h, w = o, (h - k) // s + 1, (w - k) // s + 1
    feat = c * h * w
    for i in range(desc.n_fc):
        o = desc.fc_out[i]
        n = o * feat
        out.append((theta[off:off + n].reshape(o, feat), theta[off + n:off + n + o]))
        off += n + o
        feat = o
    assert off == theta.numel() if hasattr(theta, "numel") else off == theta.size
    return out


def torch_forward(desc, theta_t, x_t):
    layers = split_params(desc, theta_t)
    h = x_t
    for i in range(desc.n_conv):
        w, b = layers[i]
        h = F.relu(F.conv2d(h, w, b, stride=desc.conv_s[i]))
    h = h.flatten(1)
    for i in range(desc.n_fc):
        w, b = layers[desc.n_conv + i]
        h = F.linear(h, w, b)
        if i != desc.n_fc - 1:
            h = F.relu(h)
    return h


def rand_theta(desc, seed, scale=0.3):
    rng = np.random.default_rng(seed)
    return rng.uniform(-scale, scale, size=odqn.num_params(desc))


# ---------------------------------------------------------------------------------- forward
def test_param_count_matches_layer_table():
    for A in (4, 6, 18):
        assert odqn.num_params(odqn.nature_desc(A)) == synth.num_params(A)
    assert synth.num_params(18) == 1693362 and synth.num_params(4) == 1686180


def test_forward_matches_torch_tiny_and_nature():
    for desc, shape, seed in ((TINY, (3, 2, 12, 12), 0), (odqn.nature_desc(6), (2, 4, 84, 84), 1)):
        theta = rand_theta(desc, seed, 0.05)
        x = np.random.default_rng(seed + 10).uniform(0, 1, size=shape)
        q, _ = odqn.forward(desc, theta, x)
        qt = torch_forward(desc, torch.tensor(theta), torch.tensor(x)).numpy()
        assert np.allclose(q, qt, rtol=1e-11, atol=1e-12)


def test_zero_weights_give_last_bias_exactly():
    desc = odqn.nature_desc(4)
    theta = np.zeros(odqn.num_params(desc))
    theta[-4:] = [0.5, -1.25, 3.0, 0.125]
    x = np.random.default_rng(2).uniform(0, 1, size=(2, 4, 84, 84))
    q, _ = odqn.forward(desc, theta, x)
    assert np.array_equal(q, np.tile(theta[-4:], (2, 1)))


def test_delta_kernel_is_a_strided_window():
    # one conv layer, weight = 1 at (o=0, c=1, p=2, q=3): output[i,j] = x[1, 2i+2, 2j+3]
    desc = odqn.make_desc((2, 12, 12), [(1, 4, 2)], [1])
    n = odqn.num_params(desc)
    theta = np.zeros(n)
    theta[(0 * 2 + 1) * 16 + 2 * 4 + 3] = 1.0
    x = np.random.default_rng(3).uniform(0.1, 1, size=(1, 2, 12, 12))
    _, acts = odqn.forward(desc, theta, x)
    conv_out = acts[0, :25].reshape(5, 5)
    assert np.array_equal(conv_out, x[0, 1, 2:12:2, 3:12:2][:5, :5])


def test_batched_forward_equals_single_calls():
    desc = odqn.nature_desc(6)
    theta = rand_theta(desc, 4, 0.05)
    x = np.random.default_rng(5).uniform(0, 1, size=(3, 4, 84, 84))
    q, _ = odqn.forward(desc, theta, x)
    for b in range(3):
        qb, _ = odqn.forward(desc, theta, x[b:b + 1])
        assert np.array_equal(q[b:b + 1], qb)      # one minibatch of W states == W single calls


# --------------------------------------------------------------------------------- backward
def _loss_for(desc, theta, x, a, y, huber=1.0):
    q, _ = odqn.forward(desc, theta, x)
    d = q[np.arange(len(a)), a] - y
    ad = np.abs(d)
    return np.where(ad <= huber, 0.5 * d * d, huber * (ad - 0.5 * huber)).mean()


def test_backward_matches_central_differences_tiny_net():
    desc = TINY
    rng = np.random.default_rng(6)
    theta = rand_theta(desc, 7, 0.4)
    B = 3
    x = rng.uniform(0, 1, size=(B, 2, 12, 12))
    a = np.array([0, 2, 1], dtype=np.int32)
    y = np.array([0.3, -2.5, 0.1])          # sample 1 lands in the linear (clipped) part
    q, acts = odqn.forward(desc, theta, x)
    d = q[np.arange(B), a] - y
    assert abs(d[1]) > 1.0 and abs(d[0]) < 1.0
    dq = np.zeros_like(q)
    dq[np.arange(B), a] = np.clip(d, -1, 1) / B
    g = odqn.backward(desc, theta, x, acts, dq)
    h = 1e-6
    num = np.zeros_like(theta)
    for i in range(theta.size):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        num[i] = (_loss_for(desc, tp, x, a, y) - _loss_for(desc, tm, x, a, y)) / (2 * h)
    assert np.abs(g).max() > 1e-3
    assert np.abs(g - num).max() <= 1e-6 * max(1.0, np.abs(num).max())
    assert np.abs(g - num).max() / np.abs(num).max() <= 1e-6


def test_backward_matches_torch_autograd_nature_net():
    desc = odqn.nature_desc(6)
    theta = rand_theta(desc, 8, 0.05)
    rng = np.random.default_rng(9)
    B = 2
    x = rng.uniform(0, 1, size=(B, 4, 84, 84))
    a = np.array([5, 1], dtype=np.int32)
    y = np.array([0.2, 3.0])
    q, acts = odqn.forward(desc, theta, x)
    d = q[np.arange(B), a] - y
    dq = np.zeros_like(q)
    dq[np.arange(B), a] = np.clip(d, -1, 1) / B
    g = odqn.backward(desc, theta, x, acts, dq)
    tt = torch.tensor(theta, requires_grad=True)
    qt = torch_forward(desc, tt, torch.tensor(x))
    sel = qt[torch.arange(B), torch.tensor(a.astype(np.int64))]
    F.huber_loss(sel, torch.tensor(y), delta=1.0, reduction="mean").backward()
    gt = tt.grad.numpy()
    assert np.abs(g - gt).max() <= 1e-10 * max(1.0, np.abs(gt).max())
    assert np.abs(gt).max() > 0


# ----------------------------------------------------------------------------------- TD loss
def test_td_target_bruteforce_and_terminal_mask():
    rng = np.random.default_rng(10)
    B, A = 64, 18
    q_sa, q_nt, q_no = rng.normal(size=(3, B, A))
    a = rng.integers(0, A, size=B).astype(np.int32)
    r = rng.choice([-1.0, 0.0, 1.0], size=B)
    done = (rng.uniform(size=B) < 0.3).astype(np.float64)
    gamma = 0.99
    loss, y, td, dq = odqn.td_loss(q_sa, q_nt, None, a, r, done, gamma, 1.0)
    for b in range(B):
        want = r[b] + (0.0 if done[b] else gamma * max(q_nt[b]))
        assert y[b] == want
        if done[b]:
            assert y[b] == r[b]                       # terminal: no bootstrap, bitwise
    # Double-DQN: online argmax, target evaluation
    _, y2, _, _ = odqn.td_loss(q_sa, q_nt, q_no, a, r, done, gamma, 1.0)
    for b in range(B):
        astar = int(np.argmax(q_no[b]))
        assert y2[b] == r[b] + gamma * (1 - done[b]) * q_nt[b, astar]
    # gamma = 0: y = r whatever the next state holds
    _, y0, _, _ = odqn.td_loss(q_sa, q_nt, None, a, r, np.zeros(B), 0.0, 1.0)
    assert np.array_equal(y0, r)


def test_terminal_sample_ignores_next_state_values():
    rng = np.random.default_rng(11)
    B, A = 8, 4
    q_sa, q_nt = rng.normal(size=(2, B, A))
    a = rng.integers(0, A, size=B).astype(np.int32)
    r = rng.normal(size=B)
    done = np.ones(B)
    l1, _, _, dq1 = odqn.td_loss(q_sa, q_nt, None, a, r, done, 0.99, 1.0)
    l2, _, _, dq2 = odqn.td_loss(q_sa, q_nt * 7 + 3, None, a, r, done, 0.99, 1.0)
    assert l1 == l2 and np.array_equal(dq1, dq2)


def test_small_errors_reduce_to_eq1():
    # |delta| <= 1: the clipped loss is Eq. 1's half squared error and its gradient is delta / B.
    B, A = 16, 6
    rng = np.random.default_rng(12)
    q_nt = rng.uniform(-0.2, 0.2, size=(B, A))
    q_sa = rng.uniform(-0.2, 0.2, size=(B, A))
    a = rng.integers(0, A, size=B).astype(np.int32)
    r = np.zeros(B)
    loss, y, td, dq = odqn.td_loss(q_sa, q_nt, None, a, r, np.zeros(B), 0.99, 1.0)
    eq1 = 0.5 * (r + 0.99 * q_nt.max(1) - q_sa[np.arange(B), a]) ** 2
    assert np.isclose(loss, eq1.mean(), rtol=1e-14)
    want = np.zeros((B, A))
    want[np.arange(B), a] = -(r + 0.99 * q_nt.max(1) - q_sa[np.arange(B), a]) / B
    assert np.allclose(dq, want, rtol=1e-14, atol=0)


def test_huber_matches_torch_and_clips():
    rng = np.random.default_rng(13)
    B, A = 32, 4
    q_sa = rng.normal(scale=3, size=(B, A))
    q_nt = rng.normal(scale=3, size=(B, A))
    a = rng.integers(0, A, size=B).astype(np.int32)
    r = rng.normal(size=B)
    done = np.zeros(B)
    loss, y, td, dq = odqn.td_loss(q_sa, q_nt, None, a, r, done, 0.99, 1.0)
    lt = F.huber_loss(torch.tensor(q_sa[np.arange(B), a]), torch.tensor(y), delta=1.0)
    assert np.isclose(loss, float(lt), rtol=1e-13)
    assert np.abs(dq).max() <= 1.0 / B + 1e-18 and (np.abs(td) > 1).any()
    assert (dq != 0).sum() <= B


# ----------------------------------------------------------------------------------- RMSProp
def test_rmsprop_first_step_closed_form():
    lr, alpha, eps = 2.5e-4, 0.95, 0.01
    g = np.array([0.0, 1e-3, -0.5, 2.0, -1e4, 1e8])
    for centered, c in ((True, math.sqrt(alpha * (1 - alpha))), (False, math.sqrt(1 - alpha))):
        theta = np.zeros_like(g)
        v = np.zeros_like(g)
        m = np.zeros_like(g)
        odqn.rmsprop_step(theta, g, v, m, lr, alpha, eps, centered)
        want = -lr * g / (c * np.abs(g) + eps)
        assert np.allclose(theta, want, rtol=1e-12, atol=0)
        assert theta[0] == 0.0
    # limits quoted from the constants of Appendix B: lr / sqrt(alpha (1 - alpha)), lr / sqrt(1 - alpha)
    assert math.isclose(lr / math.sqrt(alpha * (1 - alpha)), 1.1471e-3, rel_tol=1e-4)
    assert math.isclose(lr / math.sqrt(1 - alpha), 1.1180e-3, rel_tol=1e-4)


@pytest.mark.parametrize("centered", [True, False])
def test_rmsprop_matches_torch_optimizer(centered):
    rng = np.random.default_rng(14)
    n = 257
    theta = rng.normal(size=n)
    v = np.zeros(n)
    m = np.zeros(n)
    p = torch.tensor(theta.copy(), requires_grad=True)
    opt = torch.optim.RMSprop([p], lr=2.5e-4, alpha=0.95, eps=0.01, centered=centered)
    for _ in range(6):
        g = rng.normal(scale=rng.uniform(0.001, 2.0), size=n)
        odqn.rmsprop_step(theta, g, v, m, 2.5e-4, 0.95, 0.01, centered)
        p.grad = torch.tensor(g)
        opt.step()
    assert np.allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------------- whole train step
def test_train_step_invariants_and_torch_cross_check():
    A, B = 4, 3
    params = synth.init_params(21, A)
    agent = odqn.OracleDQN(A, params, seed=1)
    rng = np.random.default_rng(15)
    s = rng.integers(0, 256, size=(B, 4, 84, 84), dtype=np.uint8)
    s2 = rng.integers(0, 256, size=(B, 4, 84, 84), dtype=np.uint8)
    a = np.array([1, 3, 0], dtype=np.int32)
    r = np.array([1.0, -1.0, 0.0], dtype=np.float32)
    done = np.array([0.0, 1.0, 0.0], dtype=np.float32)

    # torch replica of one step (fp64): conv2d/linear/huber_loss/RMSprop(centered)
    desc = agent.desc
    p = torch.tensor(agent.theta.copy(), requires_grad=True)
    pt = torch.tensor(agent.theta_target.copy())
    opt = torch.optim.RMSprop([p], lr=2.5e-4, alpha=0.95, eps=0.01, centered=True)
    xs, xs2 = torch.tensor(s, dtype=torch.float64) / 255, torch.tensor(s2, dtype=torch.float64) / 255
    for _ in range(2):
        target_before = agent.theta_target.copy()
        loss, q_sa, y = agent.train_step(s, a, r, s2, done)
        assert np.array_equal(agent.theta_target, target_before)     # theta^- frozen between syncs
        with torch.no_grad():
            yt = torch.tensor(r, dtype=torch.float64) + 0.99 * (1 - torch.tensor(done, dtype=torch.float64)) * \
                torch_forward(desc, pt, xs2).max(1).values
        opt.zero_grad()
        sel = torch_forward(desc, p, xs)[torch.arange(B), torch.tensor(a.astype(np.int64))]
        lt = F.huber_loss(sel, yt, delta=1.0)
        lt.backward()
        opt.step()
        assert np.isclose(loss, float(lt.detach()), rtol=1e-10)
        assert np.allclose(agent.theta, p.detach().numpy(), rtol=1e-9, atol=1e-12)
    assert not np.array_equal(agent.theta, agent.theta_target)
    # terminal sample: its loss term does not depend on s'
    agent2 = odqn.OracleDQN(A, params, seed=1)
    s2b = s2.copy()
    s2b[1] = 255 - s2b[1]
    l_a, _, y_a = odqn.OracleDQN(A, params).train_step(s, a, r, s2, done)
    l_b, _, y_b = agent2.train_step(s, a, r, s2b, done)
    assert l_a == l_b and y_a[1] == r[1] == y_b[1]
    agent.sync_target()
    assert np.array_equal(agent.theta, agent.theta_target)           # bitwise copy at sync


def test_act_uses_target_parameters():
    A = 4
    params = synth.init_params(22, A)
    agent = odqn.OracleDQN(A, params, seed=3)
    rng = np.random.default_rng(16)
    s = rng.integers(0, 256, size=(2, 4, 84, 84), dtype=np.uint8)
    q_before = agent.q_values(s, use_target=True)
    agent.train_step(s, np.array([0, 1], dtype=np.int32), np.ones(2, np.float32), s,
                     np.zeros(2, np.float32))
    assert np.array_equal(agent.q_values(s, use_target=True), q_before)
    assert not np.array_equal(agent.q_values(s, use_target=False), q_before)
