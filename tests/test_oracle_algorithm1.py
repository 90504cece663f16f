"""Pins of the Algorithm 1 oracle (oracle/algorithm1.py) against what the paper fixes: the schedule counts of the
listing, the determinism claim of Section 3 (any interleaving of sampler and trainer inside a block gives the same
result, because actions come from theta^- and D is frozen until the flush), and the consistency of the states an
environment acts from with the states the replay gather rebuilds (Section 2.1: stacks of the four latest frames)."""
import numpy as np
import pytest

from datagen import synth
from oracle import dqn as odqn
from oracle.algorithm1 import Algorithm1, SyntheticEnvs
from oracle.replay import OracleReplay

A = 5
TINY = odqn.make_desc((4, 84, 84), [(4, 8, 4), (6, 4, 2)], [16, A])     # small net on real-size frames


def tiny_params(seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(-0.2, 0.2, size=odqn.num_params(TINY)).astype(np.float32)


def make(seed, W, C, F, B, epsilon, p_term=0.1, capacity_per_lane=64):
    dqn = odqn.OracleDQN(A, tiny_params(seed), seed=seed, desc=TINY, lr=1e-2)
    rep = OracleReplay(W * capacity_per_lane, W, seed)
    envs = SyntheticEnvs(synth, seed, W, A, 0.3, 0.3, p_term)
    return Algorithm1(dqn, rep, envs, C, F, B, epsilon)


def test_env_outcome_definition_scalar():
    # re-derive rewards / terminals with Python integers from the documented definition
    seed, W, n = 77, 3, 5
    t_neg, t_pos, t_term = synth.thresholds(0.3, 0.3, 0.1)
    key = synth.stream_key(seed, synth.STREAM_ENV_META)
    for acts in ([0, 1, 2], [4, 4, 4], [3, 0, 1]):
        r, d = synth.env_outcomes(seed, W, n, acts, A, 0.3, 0.3, 0.1)
        for j in range(W):
            w = synth._mix64_int(synth._mix64_int(key + n * W + j) + synth.GAMMA)
            rb, tb, ab = w & 0xFFFFFF, (w >> 24) & 0xFFFFFF, (w >> 48) & 0xFFFF
            good = (ab * A) >> 16
            want = (-1.0 if rb < t_neg else (1.0 if rb >= (1 << 24) - t_pos else 0.0)) if acts[j] == good else 0.0
            assert r[j] == want and d[j] == (1 if tb < t_term else 0)
    # observations: o_n of environment j is frame n*W + j of its stream
    assert np.array_equal(synth.env_frames(seed, W, n)[1], synth.frames(seed, synth.STREAM_ENV, [n * W + 1])[0])


def test_schedule_counts_of_the_listing():
    W, C, F, B = 2, 8, 4, 4
    alg = make(3, W, C, F, B, 0.25)
    alg.prepopulate(16)
    assert alg.act_steps == 16 // W and alg.train_steps == 0
    assert alg.replay.count == [8, 8] and all(len(s) == 0 for s in alg.replay.staged)
    theta0 = alg.dqn.theta.copy()
    alg.run(3 * C)
    assert alg.t == 3 * C
    assert alg.train_steps == 3 * C // F                       # C / F minibatches per block
    assert alg.act_steps == (16 + 3 * C) // W                  # one act step per W timesteps
    # the last block's experiences are still in the temporary buffers; everything before is in D
    assert alg.replay.count == [8 + 2 * C // W] * W and [len(s) for s in alg.replay.staged] == [C // W] * W
    # theta^- is theta as of the last synchronisation point: different from theta0 and from the current theta
    assert not np.array_equal(alg.dqn.theta_target, theta0) and not np.array_equal(alg.dqn.theta_target, alg.dqn.theta)
    assert len(alg.losses) == alg.train_steps and all(np.isfinite(alg.losses))


@pytest.mark.parametrize("epsilon", [0.0, 0.3])
def test_sampler_and_trainer_commute_inside_a_block(epsilon):
    W, C, F, B = 2, 8, 2, 4
    runs = []
    for trainer_first in (True, False):
        alg = make(11, W, C, F, B, epsilon)
        alg.prepopulate(24)
        alg.run(3 * C, trainer_first=trainer_first)
        runs.append(alg)
    a, b = runs
    assert np.array_equal(a.dqn.theta, b.dqn.theta) and np.array_equal(a.dqn.theta_target, b.dqn.theta_target)
    assert np.array_equal(a.replay.frames, b.replay.frames) and np.array_equal(a.replay.actions, b.replay.actions)
    assert np.array_equal(a.replay.rewards, b.replay.rewards) and np.array_equal(a.replay.terminals, b.replay.terminals)
    assert a.envs.reward_sum == b.envs.reward_sum and a.envs.episodes == b.envs.episodes
    assert a.losses == b.losses


def test_acting_from_online_parameters_would_break_the_commutation():
    # the same comparison with actions taken from theta instead of theta^- (standard DQN): the two orders now differ,
    # which is why Section 3 moves the policy to theta^-
    W, C, F, B = 2, 8, 2, 4
    thetas = []
    for trainer_first in (True, False):
        alg = make(11, W, C, F, B, 0.0)
        alg.dqn_act = alg.dqn.act
        alg.dqn.act = lambda s, e, n, use_target=True, _f=alg.dqn_act: _f(s, e, n, use_target=False)
        alg.prepopulate(24)
        alg.run(3 * C, trainer_first=trainer_first)
        thetas.append((alg.replay.actions.copy(), alg.dqn.theta.copy()))
    assert not (np.array_equal(thetas[0][0], thetas[1][0]) and np.array_equal(thetas[0][1], thetas[1][1]))


def test_states_acted_from_equal_states_rebuilt_from_the_replay():
    W, C, F, B = 3, 6, 3, 4
    alg = make(5, W, C, F, B, 0.5, p_term=0.25)
    history = []                                               # states every environment acted from, per act step
    step0 = alg.envs.step
    def recording_step(actions):
        history.append(alg.envs.states.copy())
        return step0(actions)
    alg.envs.step = recording_step
    alg.prepopulate(30)
    alg.run(2 * C)
    alg.replay.flush()
    assert alg.envs.episodes > 3                               # resets did occur
    M = alg.replay.M
    for lane in range(W):
        for j in range(3, alg.replay.count[lane] - 1):
            s, s2, a, r, d = alg.replay.gather([lane * M + j])
            # age j of the lane is the environment's j-th step (nothing has been overwritten)
            assert np.array_equal(s[0], history[j][lane])
            if not d[0]:
                assert np.array_equal(s2[0], history[j + 1][lane])
            else:                                              # the gather still shows the successor frame; the target ignores it
                assert np.array_equal(s2[0][3], history[j + 1][lane][3])


# ---- the ablation variants (Section 5.1): Concurrent Training / Synchronized Execution switched off ----------------

from oracle.algorithm1 import Ablation  # noqa: E402


def make_variant(seed, W, C, F, B, epsilon, concurrent, synchronized, lr=1e-2, p_term=0.1):
    dqn = odqn.OracleDQN(A, tiny_params(seed), seed=seed, desc=TINY, lr=lr)
    rep = OracleReplay(W * 64, W, seed)
    envs = SyntheticEnvs(synth, seed, W, A, 0.3, 0.3, p_term)
    return Ablation(dqn, rep, envs, C, F, B, epsilon, concurrent, synchronized)


def snapshot(alg):
    alg.replay.flush()
    r = alg.replay
    return (r.frames.copy(), r.actions.copy(), r.rewards.copy(), r.terminals.copy(), list(r.count),
            alg.envs.reward_sum, alg.envs.episodes)


def same_snapshot(x, y):
    return all(np.array_equal(p, q) if isinstance(p, np.ndarray) else p == q for p, q in zip(x, y))


@pytest.mark.parametrize("concurrent", [True, False])
def test_one_query_per_sampler_equals_the_shared_minibatch_when_greedy(concurrent):
    # Section 4: Synchronized Execution changes how Q is computed (one minibatch of W instead of W queries), not
    # what; with epsilon = 0 no random number enters, so both must act, store and learn identically
    W, C, F, B = 4, 8, 4, 4
    out = []
    for synchronized in (True, False):
        alg = make_variant(21, W, C, F, B, 0.0, concurrent, synchronized)
        alg.synchronized = True                    # the random prepopulation draws depend on the query shape:
        alg.prepopulate(24)                        # give both runs the same one
        alg.synchronized = synchronized
        alg.run(3 * C)
        out.append((alg.dqn.theta.copy(), alg.dqn.theta_target.copy(), snapshot(alg), alg.train_steps, alg.act_steps))
    assert np.array_equal(out[0][0], out[1][0]) and np.array_equal(out[0][1], out[1][1])
    assert same_snapshot(out[0][2], out[1][2]) and out[0][3:] == out[1][3:]


def test_unsynchronized_samplers_draw_from_their_own_counters():
    # with exploration the W single queries use counters n*W + j (index 0), the shared minibatch counter n (index j)
    W = 4
    alg = make_variant(22, W, 8, 4, 4, 1.0, True, False)
    seen = []
    act0 = alg.dqn.act
    def recording(states, eps, step, use_target=True):
        seen.append((states.shape[0], step))
        return act0(states, eps, step, use_target=use_target)
    alg.dqn.act = recording
    alg.prepopulate(3 * W)
    assert seen == [(1, n * W + j) for n in range(3) for j in range(W)]


def test_with_a_zero_step_size_all_four_variants_collect_the_same_experiences():
    # lr = 0 keeps theta = theta^- forever, so where the parameters are read from and when training happens cannot
    # matter: the four variants differ only in scheduling
    W, C, F, B = 2, 8, 2, 4
    snaps = []
    for concurrent in (True, False):
        for synchronized in (True, False):
            alg = make_variant(23, W, C, F, B, 0.0, concurrent, synchronized, lr=0.0)
            alg.synchronized = True                # same random prepopulation for all four
            alg.prepopulate(24)
            alg.synchronized = synchronized
            alg.run(2 * C)
            assert alg.train_steps == 2 * C // F
            snaps.append(snapshot(alg))
    assert all(same_snapshot(snaps[0], s) for s in snaps[1:])


def test_standard_dqn_schedule():
    # without Concurrent Training: acts from theta, which changes between rounds; t // F train steps after a round
    # ending at t; every experience is visible to the very next minibatch
    W, C, F, B, prepop = 2, 8, 4, 4, 24
    alg = make_variant(24, W, C, F, B, 0.25, False, True)
    acts, trains = [], []
    act0, sample0 = alg.dqn.act, alg.replay.sample_indices
    def act(states, eps, step, use_target=True):
        acts.append((use_target, alg.train_steps, alg.dqn.theta.copy()))
        return act0(states, eps, step, use_target=use_target)
    def sample(Bn, step):
        trains.append((step, alg.t, alg.replay.num_valid(), [len(x) for x in alg.replay.staged]))
        return sample0(Bn, step)
    alg.dqn.act, alg.replay.sample_indices = act, sample
    alg.prepopulate(prepop)
    n_pre = len(acts)
    alg.run(2 * C)
    run_acts = acts[n_pre:]
    assert all(not use_target for use_target, _, _ in run_acts)
    assert [k for _, k, _ in run_acts] == [(n * W) // F for n in range(2 * C // W)]      # train steps made before round n
    changed = [not np.array_equal(run_acts[i][2], run_acts[i + 1][2]) for i in range(len(run_acts) - 1)]
    assert changed == [run_acts[i][1] != run_acts[i + 1][1] for i in range(len(run_acts) - 1)] and any(changed)
    assert [k for k, _, _, _ in trains] == list(range(2 * C // F))
    for k, t, valid, staged in trains:
        assert t == -(-(k + 1) * F // W) * W                    # the first round end with t // F > k
        assert valid == W * ((prepop + t) // W - 4) and staged == [0] * W
    # theta^- is theta as of the last multiple of C
    assert alg.train_steps == 2 * C // F and alg.t == 2 * C


def test_concurrent_training_freezes_what_the_minibatches_see():
    # the counterpart: with Concurrent Training the number of visible transitions changes only at synchronisation points
    W, C, F, B, prepop = 2, 8, 2, 4, 24
    alg = make_variant(25, W, C, F, B, 0.25, True, False)
    seen = []
    sample0 = alg.replay.sample_indices
    alg.replay.sample_indices = lambda Bn, step: (seen.append((step, alg.replay.num_valid())), sample0(Bn, step))[1]
    alg.prepopulate(prepop)
    alg.run(3 * C)
    per_block = C // F
    assert [v for _, v in seen] == [W * ((prepop + (k // per_block) * C) // W - 4) for k in range(3 * per_block)]
