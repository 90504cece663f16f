"""GPU parity of the act step and the train step against the CPU oracle (fp32 and bf16 modes).

Tolerances: Q-values relative error <= 1e-4 (fp32 mode) and <= 2e-2 (bf16 mode); parameters after
the update <= 1e-3 (fp32 mode); relative error is max|gpu - ref| / max|ref| per tensor.  Actions are
compared exactly wherever the oracle's top-two gap exceeds the Q tolerance; exploration draws and
random actions are integer-determined and must match everywhere.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2111_01264_amd as P
from datagen import synth
from oracle import dqn as odqn
from oracle import philox
from oracle.replay import OracleReplay
from tests.gpu_util import blob_slices, dev, fill_replay_from_host, make_cfg, rel_err

Q_TOL = {P.DQN_PRECISION_FP32: 1e-4, P.DQN_PRECISION_BF16: 2e-2}


def gpu_act(ctx, states, eps, step, use_target, A):
    W = states.shape[0]
    acts = torch.empty(W, dtype=torch.int32, device="cuda")
    q = torch.empty((W, A), dtype=torch.float32, device="cuda")
    d_states = dev(states)
    torch.cuda.synchronize()
    P.dqn_act(ctx, d_states, W, eps, step, use_target, acts, q)
    torch.cuda.synchronize()
    return acts.cpu().numpy(), q.cpu().numpy()


def check_actions(acts, q_ref, eps, seed, step, tol):
    W, A = q_ref.shape
    want = odqn.epsilon_greedy(q_ref, eps, seed, step)
    for j in range(W):
        x0, x1, _, _ = philox.draw(seed, philox.TAG_ACT, step, j)
        explored = np.float32(x0 >> 8) * np.float32(2.0 ** -24) < np.float32(eps)
        top = np.sort(q_ref[j])[::-1]
        gap = top[0] - top[1] if A > 1 else np.inf
        if explored or gap > tol * max(np.abs(q_ref).max(), 1e-6):
            assert acts[j] == want[j], (j, acts[j], want[j])
        else:
            assert q_ref[j, acts[j]] >= top[0] - 2 * tol * max(np.abs(q_ref).max(), 1e-6)


@pytest.mark.parametrize("precision", [P.DQN_PRECISION_FP32, P.DQN_PRECISION_BF16])
# W = 32 is the largest round the small-batch fc1 kernel takes, 33 the smallest for the large-batch one, 64 a whole
# number of its 32-row tiles (the W of the batch-256 sweep point), 37 a ragged one
@pytest.mark.parametrize("A,W", [(4, 1), (6, 8), (18, 32), (18, 33), (18, 37), (18, 64)])
def test_act_parity(precision, A, W):
    seed = 211101264
    cfg = make_cfg(A, max_envs=64, precision=precision, seed=seed)
    sa, stt = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = P.dqn_create(cfg, sa, stt)
    try:
        theta = synth.init_params(seed, A)
        theta_t = synth.init_params(seed + 1, A)
        P.dqn_set_params(ctx, P.DQN_PARAMS_ONLINE, theta)
        P.dqn_set_params(ctx, P.DQN_PARAMS_TARGET, theta_t)
        assert np.array_equal(P.dqn_get_params(ctx, P.DQN_PARAMS_ONLINE), theta)     # layout round trip
        assert np.array_equal(P.dqn_get_params(ctx, P.DQN_PARAMS_TARGET), theta_t)
        orc = odqn.OracleDQN(A, theta, seed=seed)
        orc.theta_target = theta_t.astype(np.float64)
        for step, eps in ((0, 0.1), (5, 1.0), (2 ** 33 + 1, 0.0)):
            states = synth.act_states(seed, step % 1000, W)
            for use_target in (1, 0):
                acts, q = gpu_act(ctx, states, eps, step, use_target, A)
                q_ref = orc.q_values(states, use_target=bool(use_target))
                err = rel_err(q, q_ref)
                assert err <= Q_TOL[precision], (err, use_target)
                check_actions(acts, q_ref, eps, seed, step, Q_TOL[precision])
        # one minibatch of W states == W single calls (Section 4)
        states = synth.act_states(seed, 3, W)
        _, q_all = gpu_act(ctx, states, 0.0, 9, 1, A)
        for j in range(min(W, 3)):
            _, q_one = gpu_act(ctx, states[j:j + 1], 0.0, 9, 1, A)
            assert rel_err(q_one, q_all[j:j + 1]) <= 1e-5
        with pytest.raises(P.DqnError):
            P.dqn_act(ctx, dev(states), 65, 0.1, 0, 1, torch.empty(65, dtype=torch.int32, device="cuda"), None)
    finally:
        P.dqn_destroy(ctx)


def run_train_parity(A, B, steps, precision, double_dqn, N, lanes, p_term, seed, check_params, p_reward=0.05):
    cfg = make_cfg(A, max_batch=B, max_envs=8, precision=precision, double_dqn=double_dqn, seed=seed)
    sa, stt = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = P.dqn_create(cfg, sa, stt)
    rb = P.replay_create(N, lanes, min(500, N // lanes), seed, sa, stt)
    orep = OracleReplay(N, lanes, seed)
    try:
        theta = synth.init_params(seed, A)
        P.dqn_set_params(ctx, P.DQN_PARAMS_ONLINE, theta)
        P.dqn_set_params(ctx, P.DQN_PARAMS_TARGET, theta)
        orc = odqn.OracleDQN(A, theta, double_dqn=bool(double_dqn), seed=seed)
        fill_replay_from_host(rb, seed, lanes, N // lanes, A, p_neg=p_reward, p_pos=p_reward, p_term=p_term, oracle=orep)
        s = torch.empty((B, 4, 84, 84), dtype=torch.uint8, device="cuda")
        s2 = torch.empty_like(s)
        a = torch.empty(B, dtype=torch.int32, device="cuda")
        r = torch.empty(B, dtype=torch.float32, device="cuda")
        d = torch.empty(B, dtype=torch.float32, device="cuda")
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        sl = blob_slices(A)
        qtol = Q_TOL[precision]
        for step in range(steps):
            P.replay_sample_gather(rb, B, step, None, s, s2, a, r, d, None)
            P.dqn_train_step(ctx, s, a, r, s2, d, B, loss)
            torch.cuda.synchronize()
            idx = orep.sample_indices(B, step)
            ws, ws2, wa, wr, wd = orep.gather(idx)
            assert np.array_equal(s.cpu().numpy(), ws) and np.array_equal(s2.cpu().numpy(), ws2)
            assert np.array_equal(a.cpu().numpy(), wa) and np.array_equal(r.cpu().numpy(), wr)
            assert np.array_equal(d.cpu().numpy(), wd)
            target_before = orc.theta_target.copy()
            theta_before = orc.theta.copy()
            wloss, q_sa, y = orc.train_step(ws, wa, wr, ws2, wd)
            q_on, q_nt, q_no = P.dqn_get_train_q(ctx, B, A, bool(double_dqn))
            assert rel_err(q_on, q_sa) <= qtol, ("q_online", step, rel_err(q_on, q_sa))
            q_nt_ref = odqn.forward(orc.desc, target_before, odqn.scale_states(ws2))[0]
            assert rel_err(q_nt, q_nt_ref) <= qtol, ("q_next_target", step)
            if double_dqn:
                q_no_ref = odqn.forward(orc.desc, theta_before, odqn.scale_states(ws2))[0]
                assert rel_err(q_no, q_no_ref) <= qtol, ("q_next_online", step)
            g = P.dqn_get_params(ctx, P.DQN_PARAMS_GRAD)
            th = P.dqn_get_params(ctx, P.DQN_PARAMS_ONLINE)
            if check_params:
                assert abs(float(loss.item()) - wloss) <= 1e-4 * max(abs(wloss), 1e-3), (step, loss.item(), wloss)
                for name, slc in sl.items():
                    eg = rel_err(g[slc], orc.last_grad[slc])
                    assert eg <= 2e-3, ("grad", name, step, eg)
                    et = rel_err(th[slc], orc.theta[slc])
                    assert et <= 1e-3, ("theta", name, step, et)
            else:
                assert abs(float(loss.item()) - wloss) <= 0.1 * max(abs(wloss), 1e-2), (step, loss.item(), wloss)
                for name, slc in sl.items():
                    # l2-relative: a ReLU whose pre-activation sits within bf16 rounding of zero flips
                    # for single samples, which dominates a max-norm but not the l2 norm
                    ref = orc.last_grad[slc]
                    eg = float(np.linalg.norm(g[slc] - ref) / max(np.linalg.norm(ref), 1e-12))
                    print("bf16 grad l2 rel err", name, step, "%.4f" % eg)
                    assert eg <= 0.2, ("grad", name, step, eg)
            # theta^- is unchanged between syncs (bitwise)
            assert np.array_equal(P.dqn_get_params(ctx, P.DQN_PARAMS_TARGET), theta)
        P.dqn_sync_target(ctx, rb, 1)
        orc.sync_target()
        th = P.dqn_get_params(ctx, P.DQN_PARAMS_ONLINE)
        assert np.array_equal(P.dqn_get_params(ctx, P.DQN_PARAMS_TARGET), th)      # bitwise copy
        # acting after the sync uses the new target parameters
        states = synth.act_states(seed, 0, 4)
        acts = torch.empty(4, dtype=torch.int32, device="cuda")
        q = torch.empty((4, A), dtype=torch.float32, device="cuda")
        P.dqn_act(ctx, dev(states), 4, 0.0, 0, 1, acts, q)
        torch.cuda.synchronize()
        assert rel_err(q.cpu().numpy(), orc.q_values(states, True)) <= max(qtol, 2e-3 if check_params else qtol) * 5
    finally:
        P.replay_destroy(rb)
        P.dqn_destroy(ctx)


def test_train_parity_fp32_tiny_config():
    # A=4, 10,000-frame replay, 10 train steps at batch 32 (fp32 mode)
    run_train_parity(A=4, B=32, steps=10, precision=P.DQN_PRECISION_FP32, double_dqn=0, N=10000, lanes=1,
                     p_term=0.001, seed=211101264, check_params=True)


def test_train_parity_fp32_ragged_batch_double_dqn():
    run_train_parity(A=18, B=27, steps=3, precision=P.DQN_PRECISION_FP32, double_dqn=1, N=2000, lanes=4,
                     p_term=0.05, seed=5, check_params=True)


# bf16 mode: the stated bound is on Q (2e-2).  Gradients are also compared, on a reward mix that keeps
# most TD errors of order one (with sparse rewards delta is a difference of nearly equal Q-values and
# inherits their relative error many times over, which says nothing about the backward kernels).
def test_train_parity_bf16():
    run_train_parity(A=6, B=32, steps=3, precision=P.DQN_PRECISION_BF16, double_dqn=0, N=2000, lanes=8,
                     p_term=0.01, seed=6, check_params=False, p_reward=0.4)


def test_train_parity_bf16_double_dqn():
    run_train_parity(A=18, B=40, steps=2, precision=P.DQN_PRECISION_BF16, double_dqn=1, N=2000, lanes=8,
                     p_term=0.01, seed=8, check_params=False, p_reward=0.4)


def test_train_parity_bf16_several_samples_per_workgroup():
    # batch 300 > the number of compute units: the fused conv kernels (forward and data-gradient) walk more than
    # one sample per persistent workgroup, with a ragged last range
    run_train_parity(A=6, B=300, steps=1, precision=P.DQN_PRECISION_BF16, double_dqn=0, N=4000, lanes=8,
                     p_term=0.01, seed=9, check_params=False, p_reward=0.4)

