"""CPU oracle of Algorithm 1 (DQN with Concurrent Training and Synchronized Execution, main thread), run as ONE
sequential program.  TEST INFRASTRUCTURE ONLY.

The paper's threads only change *when* things run, not *what* is computed: within a block of C timesteps the
sampler side reads theta^- and appends to temporary buffers, the trainer side reads D (constant until the next
flush) and theta^- and writes theta (Section 3), so any interleaving of the two gives the same result.  This oracle
takes the simplest one: at every synchronisation point flush, copy theta^- <- theta, run the block's C / F train
steps, then the block's C / W act steps.  `trainer_first=False` runs the act steps first; the two orders must agree
(a pin of the determinism claim of Section 3).

Readings (the paper leaves these open): timesteps are counted from 0 and the synchronisation happens when
t mod C == 0 (the listing counts from 1 and tests t mod C == 1 -- the same instants); one act step serves all W
environments and advances t by W (Section 4), so C must be a multiple of W and of F; epsilon is a constant of the
run; D is prepopulated by the same loop with epsilon = 1 and no training ("collected randomly"); environment j
writes lane j of D; the state of an environment is the stack of its four latest observations with those from
before the latest episode start replaced by zeros -- the same rule the replay gather applies (oracle/replay.py).

The ablation of Section 5.1 switches the two techniques off independently (`Ablation` below):
  * without Synchronized Execution every sampler queries the network by itself: W evaluations of one state instead
    of one evaluation of W states per round of W timesteps (Section 4's "asynchronous" samplers).  Reading: the
    samplers still advance in rounds of W timesteps (the schedule below needs a common clock), and the evaluation of
    environment j at its n-th step draws its epsilon-greedy numbers at counter n * W + j, index 0;
  * without Concurrent Training the agent is standard DQN (Section 2.1): it acts from theta, every experience
    enters D at once (no temporary buffers: a flush after every round), and a train step is due at every F-th
    timestep -- after a round that ends at t, t // F train steps have been made, each sampling from D as it is
    after that round; theta^- <- theta every C timesteps.  Sampling cannot run while training does.
"""
from __future__ import annotations

import numpy as np


class SyntheticEnvs:
    """W synthetic environments advanced in lock-step; holds their observation stacks (uint8 [W,4,84,84])."""

    def __init__(self, synth, seed, W, num_actions, p_neg, p_pos, p_term):
        self.synth, self.seed, self.W, self.A = synth, seed, W, num_actions
        self.p = (p_neg, p_pos, p_term)
        self.n = 0                                              # steps taken by every environment
        self.frame = synth.env_frames(seed, W, 0)               # o_n of every environment
        self.states = np.zeros((W, 4, 84, 84), dtype=np.uint8)
        self.states[:, 3] = self.frame
        self.reward_sum = 0.0
        self.episodes = 0

    def step(self, actions):
        """Returns the experiences (o_n, a, r, d) of this step and advances to o_{n+1}."""
        r, d = self.synth.env_outcomes(self.seed, self.W, self.n, actions, self.A, *self.p)
        exp = (self.frame.copy(), np.asarray(actions, dtype=np.int32).copy(), r, d)
        self.n += 1
        self.frame = self.synth.env_frames(self.seed, self.W, self.n)
        for j in range(self.W):
            if d[j]:
                self.states[j, :3] = 0                          # earlier frames belong to the finished episode
            else:
                self.states[j, :3] = self.states[j, 1:].copy()
            self.states[j, 3] = self.frame[j]
        self.reward_sum += float(r.sum())
        self.episodes += int(d.sum())
        return exp


class Algorithm1:
    def __init__(self, dqn, replay, envs, C, F, B, epsilon):
        W = envs.W
        assert C % W == 0 and C % F == 0 and replay.L == W
        self.dqn, self.replay, self.envs = dqn, replay, envs
        self.C, self.F, self.B, self.W, self.epsilon = C, F, B, W, epsilon
        self.t = 0
        self.act_steps = 0
        self.train_steps = 0
        self.losses = []

    def _act_block(self, timesteps, epsilon):
        for _ in range(timesteps // self.W):
            actions, _ = self.dqn.act(self.envs.states, epsilon, self.act_steps, use_target=True)
            self.act_steps += 1
            frames, a, r, d = self.envs.step(actions)
            for j in range(self.W):
                self.replay.push(j, frames[j:j + 1], a[j:j + 1], r[j:j + 1], d[j:j + 1])

    def _train_block(self):
        for _ in range(self.C // self.F):
            idx = self.replay.sample_indices(self.B, self.train_steps)
            s, s2, a, r, done = self.replay.gather(idx)
            loss, _, _ = self.dqn.train_step(s, a, r, s2, done)
            self.losses.append(loss)
            self.train_steps += 1

    def prepopulate(self, timesteps):
        """Random experiences into D: the act loop with epsilon = 1, no training, then a flush."""
        assert timesteps % self.W == 0
        self._act_block(timesteps, 1.0)
        self.replay.flush()

    def run(self, timesteps, trainer_first=True):
        assert timesteps % self.C == 0
        for _ in range(timesteps // self.C):
            # t mod C == 0: both sides are idle; flush the temporary buffers, theta^- <- theta, dispatch the trainer
            self.replay.flush()
            self.dqn.sync_target()
            if trainer_first:
                self._train_block()
                self._act_block(self.C, self.epsilon)
            else:
                frozen = _FrozenView(self.replay)
                self._act_block(self.C, self.epsilon)       # appends go to the temporary buffers only
                frozen.check_unchanged()
                self._train_block()
            self.t += self.C


class Ablation(Algorithm1):
    """Algorithm 1 with Concurrent Training and / or Synchronized Execution switched off (Section 5.1)."""

    def __init__(self, dqn, replay, envs, C, F, B, epsilon, concurrent, synchronized):
        super().__init__(dqn, replay, envs, C, F, B, epsilon)
        self.concurrent, self.synchronized = concurrent, synchronized

    def _actions(self, epsilon, use_target):
        if self.synchronized:
            actions, _ = self.dqn.act(self.envs.states, epsilon, self.act_steps, use_target=use_target)
            return actions
        out = np.empty(self.W, dtype=np.int32)
        for j in range(self.W):                                  # one query per sampler
            a, _ = self.dqn.act(self.envs.states[j:j + 1], epsilon, self.act_steps * self.W + j, use_target=use_target)
            out[j] = a[0]
        return out

    def _round(self, epsilon, use_target):
        actions = self._actions(epsilon, use_target)
        self.act_steps += 1                                      # rounds of W timesteps
        frames, a, r, d = self.envs.step(actions)
        for j in range(self.W):
            self.replay.push(j, frames[j:j + 1], a[j:j + 1], r[j:j + 1], d[j:j + 1])

    def _act_block(self, timesteps, epsilon):
        for _ in range(timesteps // self.W):
            self._round(epsilon, use_target=True)

    def run(self, timesteps, trainer_first=True):
        if self.concurrent:
            return super().run(timesteps, trainer_first)
        assert timesteps % self.C == 0
        for _ in range(timesteps // self.C):
            self.replay.flush()
            self.dqn.sync_target()                               # t mod C == 0
            for _ in range(self.C // self.W):
                self._round(self.epsilon, use_target=False)      # standard DQN acts from theta
                self.replay.flush()                              # experiences enter D at once
                self.t += self.W
                while self.train_steps < self.t // self.F:
                    idx = self.replay.sample_indices(self.B, self.train_steps)
                    s, s2, a, r, done = self.replay.gather(idx)
                    loss, _, _ = self.dqn.train_step(s, a, r, s2, done)
                    self.losses.append(loss)
                    self.train_steps += 1


class _FrozenView:
    """Remembers what is visible in D; used to assert that a block of act steps leaves it untouched."""

    def __init__(self, replay):
        self.replay = replay
        self.head, self.count = list(replay.head), list(replay.count)
        self.digest = (replay.frames.sum(dtype=np.int64), replay.actions.sum(dtype=np.int64), float(replay.rewards.sum()))

    def check_unchanged(self):
        r = self.replay
        assert self.head == list(r.head) and self.count == list(r.count)
        assert self.digest == (r.frames.sum(dtype=np.int64), r.actions.sum(dtype=np.int64), float(r.rewards.sum()))
