#!/usr/bin/env python3
"""Throughput of the DQN hot path on one MI355X: train steps/sec (batch 32) with the act steps
that belong to them running concurrently on a second stream, on seeded synthetic data shaped like
the paper's workload (Table 5: replay of 1,000,000 frames, minibatch 32, C = 10,000; Section 5.1:
W = 8 samplers, epsilon = 0.1).

One "step" = 4 act steps (W states each: Q evaluation, epsilon-greedy, push of W experiences) on the
act stream + one replay sample/gather and one train step on the train stream; every `sync_every`
train steps the synchronisation point of Algorithm 1 (flush, theta^- <- theta).  As in the paper, a
trainer thread drives the train stream while the sampler side drives the act stream.

Prints ONE JSON line.  `--sweep` instead prints one JSON line per point of the batch/W sweep (bf16 MFMA
utilisation per kernel and gather bandwidth; a readable table goes to stderr).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm": (8000.0, "GB/s"), "bf16": (2500.0, "TFLOP/s"), "f32": (157.3, "TFLOP/s")}
N_PARAMS_BASE = 1684128


def kernel_work(name, B, A, groups, precision):
    """Algorithmic (flops, bytes) of one launch of a train-step kernel.  GEMM flops are
    2*M*N*K of the layer; bytes are what the method must move for that layer (operands once)."""
    e = 2 if precision == "bf16" else 4
    n_par = N_PARAMS_BASE + 513 * A
    G = groups
    t = {
        "conv1_fwd": (2.0 * G * B * 400 * 32 * 256, G * B * (28224 + 12800 * e)),
        "conv2_fwd": (2.0 * G * B * 81 * 64 * 512, G * B * (12800 + 5184) * e),
        "conv3_fwd": (2.0 * G * B * 49 * 64 * 576, G * B * (5184 + 3136) * e),
        "fc1_fwd": (2.0 * G * B * 512 * 3136, G * (B * (3136 + 512) * e) + min(G, 2) * 512 * 3136 * e),
        "head_td": (2.0 * G * B * A * 512, G * B * 512 * e),
        "(unused)": (1.0, 1.0),
        "fc1_wgrad": (2.0 * 512 * 3136 * B, 512 * 3136 * 4 + B * (3136 + 512) * e),
        "fc1_dgrad": (2.0 * B * 3136 * 512, 512 * 3136 * e + B * (3136 * 2 + 512) * e),
        "conv3_wgrad": (2.0 * 64 * 576 * B * 49, B * (5184 + 3136) * e + 64 * 576 * 4),
        "conv3_dgrad": (2.0 * B * 49 * 64 * 576, B * (3136 + 2 * 5184) * e),      # the method's MACs (= the forward layer's), not the zero-padded gather form
        "conv2_wgrad": (2.0 * 64 * 512 * B * 81, B * (12800 + 5184) * e + 64 * 512 * 4),
        "conv2_dgrad": (2.0 * B * 81 * 64 * 512, B * (5184 + 2 * 12800) * e),
        "conv1_wgrad": (2.0 * 32 * 256 * B * 400, B * (28224 + 12800 * e) + 32 * 256 * 4),
        "small_grads": (1.0 * B * (12800 + 5184 + 3136 + 512), B * (12800 + 5184 + 3136 + 512 + 512) * e),
        "rmsprop": (10.0 * n_par, n_par * (28 + (2 if precision == "bf16" else 0))),
    }
    parts = ("fc1_wgrad", "conv3_wgrad", "conv2_wgrad", "conv1_wgrad", "small_grads")
    t["conv_tower"] = (sum(t[k][0] for k in ("conv1_fwd", "conv2_fwd", "conv3_fwd")), G * B * (28224 + 3136 * e) + B * (12800 + 5184) * e)
    t["conv_tower_bwd"] = (t["conv3_dgrad"][0] + t["conv2_dgrad"][0], B * (3136 + 2 * 5184 + 2 * 12800) * e)   # dz2 stays in LDS
    t["wgrad_all"] = (sum(t[k][0] for k in parts), sum(t[k][1] for k in parts))   # bf16: one fused launch
    return t[name]


# HBM traffic per launch measured with rocprofv3 (FETCH_SIZE and WRITE_SIZE in separate runs, scaled by what the
# same counters read for the target copy of known size; summaries under profiles/hbm_traffic_*.txt):
# {(kernel, batch, precision): (bytes, source files of the kernel, sha1 over their concatenation when the counters
# were taken)}.  Reported only while the kernel's sources still hash to that value.
_C = "paper_2111_01264_amd/csrc/"
_RMS_SRC = (_C + "head_kernels.h", _C + "net.hip")
_WG_SRC = (_C + "wgrad_all.h", _C + "wgrad_conv.h", _C + "wgrad_fc1.h", _C + "gemm_tn_tr.h", _C + "gemm_mfma.h", _C + "head_kernels.h", _C + "common.h", _C + "net.hip")
_TOWER_SRC = (_C + "conv_tower.h", _C + "conv_ws.h", _C + "gemm_mfma.h", _C + "common.h", _C + "net.hip")
_TOWER_BWD_SRC = (_C + "conv_tower_bwd.h", _C + "conv_tower.h", _C + "conv_ws.h", _C + "gemm_mfma.h", _C + "net.hip")
TRAFFIC = {
    ("rmsprop", 32, "bf16"): (66.16e6, _RMS_SRC, "04b098e8e5afd762a19a4e8bad05d9ea95f77a45", "profiles/hbm_traffic_b32.txt"),
    ("wgrad_all", 32, "bf16"): (25.63e6, _WG_SRC, "0a99a0aeb00340b719a0eaf1e2dca707da54d3b6", "profiles/hbm_traffic_b32.txt"),
    ("conv_tower", 32, "bf16"): (10.26e6, _TOWER_SRC, "b0874bb25d0a1959b7edaf5b96e267f8279aa4cd", "profiles/hbm_traffic_b32.txt"),
    ("conv_tower_bwd", 32, "bf16"): (4.78e6, _TOWER_BWD_SRC, "bb4819da911de89f68019999026c0078f3c48051", "profiles/hbm_traffic_b32.txt"),
    ("rmsprop", 256, "bf16"): (71.34e6, _RMS_SRC, "04b098e8e5afd762a19a4e8bad05d9ea95f77a45", "profiles/hbm_traffic_b256.txt"),
    ("wgrad_all", 256, "bf16"): (85.73e6, _WG_SRC, "0a99a0aeb00340b719a0eaf1e2dca707da54d3b6", "profiles/hbm_traffic_b256.txt"),
    ("conv_tower", 256, "bf16"): (24.22e6, _TOWER_SRC, "b0874bb25d0a1959b7edaf5b96e267f8279aa4cd", "profiles/hbm_traffic_b256.txt"),
    ("conv_tower_bwd", 256, "bf16"): (21.25e6, _TOWER_BWD_SRC, "bb4819da911de89f68019999026c0078f3c48051", "profiles/hbm_traffic_b256.txt"),
}


def measured_traffic(name, B, precision):
    import hashlib
    ent = TRAFFIC.get((name, B, precision))
    if not ent:
        return None, None
    nbytes, srcs, sha, where = ent
    h = hashlib.sha1()
    try:
        for src in srcs:
            with open(os.path.join(ROOT, src), "rb") as f:
                h.update(f.read())
    except OSError:
        return None, None
    return (nbytes, where) if h.hexdigest() == sha else (None, None)


def roofline_for(name, avg_ms, B, A, groups, precision):
    flops, nbytes = kernel_work(name, B, A, groups, precision)
    peak_f = PEAK["bf16" if precision == "bf16" else "f32"][0]
    ridge = peak_f * 1e12 / (PEAK["hbm"][0] * 1e9)
    sec = avg_ms * 1e-3
    if flops / max(nbytes, 1) >= ridge * 0.25 and name not in ("rmsprop", "small_grads", "(unused)", "head_td"):
        ach = flops / sec / 1e12
        return {"kernel": name, "bound": "mfma", "achieved": ach, "peak": peak_f, "unit": "TFLOP/s",
                "frac": ach / peak_f, "traffic": None, "avg_launch_us": avg_ms * 1e3}
    ach = nbytes / sec / 1e9
    return {"kernel": name, "bound": "hbm", "achieved": ach, "peak": PEAK["hbm"][0], "unit": "GB/s",
            "frac": ach / PEAK["hbm"][0], "traffic": None, "avg_launch_us": avg_ms * 1e3}


class Workload:
    """Device-resident state of one benchmark configuration."""

    def __init__(self, args):
        import torch
        import paper_2111_01264_amd as P
        from datagen import synth
        self.torch, self.P, self.synth = torch, P, synth
        self.A, self.B, self.W = args.actions, args.batch, args.envs
        self.lanes = args.lanes
        self.seed = args.seed
        self.precision = args.precision
        self.acts_per_train = args.acts_per_train
        self.fused_push = not args.separate_push
        self.fused_gather = not args.separate_gather
        self.sync_every = args.sync_every
        self.double = int(args.double_dqn)
        torch.cuda.set_device(0)
        self.act_stream, self.train_stream = torch.cuda.Stream(), torch.cuda.Stream()
        cfg = P.dqn_config()
        cfg.num_actions, cfg.max_batch, cfg.max_envs = self.A, self.B, self.W
        cfg.precision = P.DQN_PRECISION_BF16 if args.precision == "bf16" else P.DQN_PRECISION_FP32
        cfg.double_dqn, cfg.centered = self.double, 1
        cfg.gamma, cfg.huber_delta, cfg.lr, cfg.rms_alpha, cfg.rms_eps = 0.99, 1.0, 2.5e-4, 0.95, 0.01
        cfg.seed = self.seed
        self.ctx = P.dqn_create(cfg, self.act_stream, self.train_stream)
        theta = synth.init_params(self.seed, self.A)
        P.dqn_set_params(self.ctx, P.DQN_PARAMS_ONLINE, theta)
        P.dqn_set_params(self.ctx, P.DQN_PARAMS_TARGET, theta)
        per_lane = args.frames // self.lanes
        staging = min(per_lane, max(self.acts_per_train * self.sync_every, 5000))
        self.rb = P.replay_create(args.frames, self.lanes, staging, self.seed, self.act_stream, self.train_stream)
        self._fill(per_lane, args)
        # pools of act-step inputs: states, the new frame each sampler produced, reward, terminal
        pool = 16
        self.pool = pool
        dev = "cuda"
        self.states = torch.empty((pool, self.W, 4, 84, 84), dtype=torch.uint8, device=dev)
        P.synth_frames(self.states, pool * self.W * 4, 0, 1, self.seed, synth.STREAM_ACT, synth.PIX_T,
                       synth.BACKGROUND, None)
        self.new_frames = torch.empty((pool, self.lanes, 84, 84), dtype=torch.uint8, device=dev)
        P.synth_frames(self.new_frames, pool * self.lanes, 1 << 40, 1, self.seed, synth.STREAM_ACT, synth.PIX_T,
                       synth.BACKGROUND, None)
        self.rew = torch.empty((pool, self.lanes), dtype=torch.float32, device=dev)
        self.term = torch.empty((pool, self.lanes), dtype=torch.uint8, device=dev)
        scratch_a = torch.empty((pool, self.lanes), dtype=torch.int32, device=dev)
        tn, tp, tt = synth.thresholds(args.p_reward, args.p_reward, args.p_term)
        P.synth_transitions(scratch_a, self.rew, self.term, pool * self.lanes, 1 << 41, 1, self.seed, self.A, tn, tp,
                            tt, None)
        self.actions = torch.zeros(max(self.W, self.lanes), dtype=torch.int32, device=dev)
        self.s = torch.empty((self.B, 4, 84, 84), dtype=torch.uint8, device=dev)
        self.s2 = torch.empty_like(self.s)
        self.a = torch.empty(self.B, dtype=torch.int32, device=dev)
        self.r = torch.empty(self.B, dtype=torch.float32, device=dev)
        self.d = torch.empty(self.B, dtype=torch.float32, device=dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        self.train_steps = 0
        self.act_steps = 0
        self.prepare_raw()

    def _fill(self, per_lane, args):
        torch, P, synth = self.torch, self.P, self.synth
        chunk = min(5000, per_lane)
        buf = torch.empty((chunk, 84, 84), dtype=torch.uint8, device="cuda")
        a = torch.empty(chunk, dtype=torch.int32, device="cuda")
        r = torch.empty(chunk, dtype=torch.float32, device="cuda")
        t = torch.empty(chunk, dtype=torch.uint8, device="cuda")
        tn, tp, tt = synth.thresholds(args.p_reward, args.p_reward, args.p_term)
        with torch.cuda.stream(self.act_stream):
            for lo in range(0, per_lane, chunk):
                n = min(chunk, per_lane - lo)
                for lane in range(self.lanes):
                    # frame id of (lane, time) = time * lanes + lane
                    P.synth_frames(buf, n, lo * self.lanes + lane, self.lanes, self.seed, synth.STREAM_REPLAY,
                                   synth.PIX_T, synth.BACKGROUND, self.act_stream)
                    P.synth_transitions(a, r, t, n, lo * self.lanes + lane, self.lanes, self.seed, self.A, tn, tp, tt,
                                        self.act_stream)
                    P.replay_push(self.rb, lane, buf, a, r, t, n)
                P.replay_flush(self.rb, 1)
        torch.cuda.synchronize()

    def prepare_raw(self):
        """Pre-marshalled arguments for the hot loops (pointers as plain ints)."""
        lib = self.P.binding._lib
        self._lib = lib
        self._p_states = [self.states[k].data_ptr() for k in range(self.pool)]
        self._p_frames = [self.new_frames[k].data_ptr() for k in range(self.pool)]
        self._p_rew = [self.rew[k].data_ptr() for k in range(self.pool)]
        self._p_term = [self.term[k].data_ptr() for k in range(self.pool)]
        self._p_actions = self.actions.data_ptr()
        self._p_train = (self.s.data_ptr(), self.s2.data_ptr(), self.a.data_ptr(), self.r.data_ptr(),
                         self.d.data_ptr(), self.loss.data_ptr())

    def _fail(self, what, rc):
        raise RuntimeError("%s failed (%d): %s" % (what, rc, self.P.dqn_last_error()))

    def sync_point(self):
        """Algorithm 1: both workers are idle; flush the temporary buffers, theta^- <- theta."""
        self.P.dqn_sync_target(self.ctx, self.rb, 0)

    def act_part(self, n_train_steps):
        """Sampler side of n train steps: acts_per_train act steps each (Q evaluation, epsilon-greedy, push of the
        experiences the step produced).  From the second step on, the push of step t-1 and the Q evaluation of
        step t are one call (dqn_act_push_step); the last push of the part is issued by itself."""
        lib, ctx, rb, W, pool = self._lib, self.ctx, self.rb, self.W, self.pool
        push = self.W == self.lanes
        pa = self._p_actions
        pending = -1
        for _ in range(n_train_steps * self.acts_per_train):
            k = self.act_steps % pool
            if push and pending >= 0 and self.fused_push:
                rc = lib.dqn_act_push_step(ctx, rb, self._p_frames[pending], pa, self._p_rew[pending], self._p_term[pending],
                                           self._p_states[k], W, 0.1, self.act_steps, 1, pa, None)
                if rc:
                    self._fail("dqn_act_push_step", rc)
            else:
                rc = lib.dqn_act(ctx, self._p_states[k], W, 0.1, self.act_steps, 1, pa, None)
                if rc:
                    self._fail("dqn_act", rc)
                if push and not self.fused_push:
                    rc = lib.replay_push_step(rb, self._p_frames[k], pa, self._p_rew[k], self._p_term[k])
                    if rc:
                        self._fail("replay_push_step", rc)
            pending = k
            self.act_steps += 1
        if push and self.fused_push and pending >= 0:
            rc = lib.replay_push_step(rb, self._p_frames[pending], pa, self._p_rew[pending], self._p_term[pending])
            if rc:
                self._fail("replay_push_step", rc)

    def train_part(self, n_train_steps):
        """Trainer side: sample + gather + train step, n times."""
        lib, ctx, rb, B = self._lib, self.ctx, self.rb, self.B
        ps, ps2, pa, pr, pd, pl = self._p_train
        if self.fused_gather:
            # one call per step; the gather of the next minibatch rides in this step's launches (not for the last
            # step of the part: a synchronisation point may follow, and the replay memory changes there)
            for i in range(n_train_steps):
                rc = lib.dqn_train_step_sampled(ctx, rb, B, self.train_steps, 1 if i + 1 < n_train_steps else 0, pl)
                if rc:
                    self._fail("dqn_train_step_sampled", rc)
                self.train_steps += 1
            return
        for _ in range(n_train_steps):
            rc = lib.replay_sample_gather(rb, B, self.train_steps, None, ps, ps2, pa, pr, pd, None)
            if rc:
                self._fail("replay_sample_gather", rc)
            rc = lib.dqn_train_step(ctx, ps, pa, pr, ps2, pd, B, pl)
            if rc:
                self._fail("dqn_train_step", rc)
            self.train_steps += 1

    def run(self, steps, part="both"):
        """`steps` benchmark steps: the trainer thread and the sampler (this) thread run concurrently
        between synchronisation points, as in Algorithm 1 (no host synchronisation with the GPU).
        part = "train" / "act" runs only that side (same sync schedule), for the alone-vs-overlapped figures."""
        done = 0
        while done < steps:
            if part != "both":
                self.sync_point()
                n = min(steps - done, self.sync_every)
                if part == "train":
                    self.train_part(n)
                else:
                    self.act_part(n)
                done += n
                continue
            if self.train_steps % self.sync_every == 0:
                self.sync_point()
            n = min(steps - done, self.sync_every - self.train_steps % self.sync_every)
            self._trainer_submit(n)
            self.act_part(n)
            self._trainer_wait()
            done += n

    # The trainer thread lives as long as the workload (as Algorithm 1's trainer thread does): starting a thread per
    # call would put its start-up inside every timed region, which shows in short runs.
    def _trainer_loop(self):
        while True:
            n = self._trainer_tasks.get()
            if n is None:
                return
            try:
                self.train_part(n)
            except Exception as e:      # noqa: BLE001
                self._trainer_err.append(e)
            self._trainer_done.set()

    def _trainer_submit(self, n):
        import queue
        import threading
        if getattr(self, "_trainer_thread", None) is None:
            self._trainer_tasks, self._trainer_done, self._trainer_err = queue.SimpleQueue(), threading.Event(), []
            self._trainer_thread = threading.Thread(target=self._trainer_loop, daemon=True)
            self._trainer_thread.start()
        self._trainer_done.clear()
        self._trainer_tasks.put(n)

    def _trainer_wait(self):
        self._trainer_done.wait()
        if self._trainer_err:
            raise self._trainer_err.pop()

    def close(self):
        if getattr(self, "_trainer_thread", None) is not None:
            self._trainer_tasks.put(None)
            self._trainer_thread.join()
            self._trainer_thread = None
        self.torch.cuda.synchronize()
        self.P.replay_destroy(self.rb)
        self.P.dqn_destroy(self.ctx)


def time_steps(wl, steps, part="both"):
    torch = wl.torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    wl.run(steps, part)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def kernel_breakdown(wl, steps_each):
    """Average launch duration (ms) of every train-step kernel, one kernel at a time."""
    P = wl.P
    out = {}
    for kid in range(1, P.dqn_profile_kernel_count() + 1):
        if P.dqn_profile_kernel_name(kid).startswith("("):
            continue
        P.dqn_profile_select(wl.ctx, kid)
        wl.run(steps_each)
        ms, n = P.dqn_profile_read(wl.ctx)
        if n > 0:
            out[P.dqn_profile_kernel_name(kid)] = ms / n
    P.dqn_profile_select(wl.ctx, 0)
    return out


def cpu_baseline(args):
    """The oracle, as it stands, on the host cores: same step composition, bounded sample."""
    from datagen import synth
    from oracle import dqn as odqn
    from oracle.replay import OracleReplay
    A, B, W, lanes, seed = args.actions, args.batch, args.envs, args.lanes, args.seed
    n_frames = 64 * lanes                       # a small ring is enough for a timing sample
    rep = OracleReplay(n_frames, lanes, seed)
    for lane in range(lanes):
        ids = np.arange(64, dtype=np.uint64) * np.uint64(lanes) + np.uint64(lane)
        a, r, d = synth.transitions(seed, ids, A)
        rep.push(lane, synth.frames(seed, synth.STREAM_REPLAY, ids), a, r, d)
    rep.flush()
    agent = odqn.OracleDQN(A, synth.init_params(seed, A), seed=seed, double_dqn=bool(args.double_dqn))
    states = synth.act_states(seed, 0, W)
    def timed(budget, step0):
        done, t0 = 0, time.perf_counter()
        while True:
            for k in range(args.acts_per_train):
                agent.act(states, 0.1, (step0 + done) * args.acts_per_train + k, use_target=True)
            s, s2, a, r, d = rep.gather(rep.sample_indices(B, step0 + done))
            agent.train_step(s, a, r, s2, d)
            done += 1
            el = time.perf_counter() - t0
            if el >= budget or done >= 1000:
                return done, el

    n_all, el_all = timed(args.cpu_seconds, 0)
    # the same loop on one thread (results are bitwise those of any thread count)
    cores = odqn.set_threads(1)
    n_one, el_one = timed(args.cpu_seconds * 0.6, n_all)
    odqn.set_threads(cores)
    what = "each: %d act steps of W=%d + gather + train step at batch %d" % (args.acts_per_train, W, B)
    return {"value": n_all / el_all, "unit": "train steps/s", "cores": cores, "kind": "oracle",
            "sample": "%d steps (%s) in %.1f s on %d threads; single thread: %d steps in %.1f s"
                      % (n_all, what, el_all, cores, n_one, el_one),
            "single_thread": {"value": n_one / el_one, "unit": "train steps/s", "cores": 1}}


def run_alg1(args, W, concurrent, synchronized, blocks, warmup_blocks, prepopulate, frames):
    """One timed run of the orchestrator; returns rates and totals."""
    import torch
    import paper_2111_01264_amd as P
    from datagen import synth
    C, F, B, A = args.alg1_c, args.alg1_f, args.batch, args.actions
    torch.cuda.set_device(0)
    sa, stt = torch.cuda.Stream(), torch.cuda.Stream()
    cfg = P.dqn_config()
    cfg.num_actions, cfg.max_batch, cfg.max_envs = A, B, W
    cfg.precision = P.DQN_PRECISION_BF16 if args.precision == "bf16" else P.DQN_PRECISION_FP32
    cfg.double_dqn, cfg.centered = int(args.double_dqn), 1
    cfg.gamma, cfg.huber_delta, cfg.lr, cfg.rms_alpha, cfg.rms_eps = 0.99, 1.0, 2.5e-4, 0.95, 0.01
    cfg.seed = args.seed
    ctx = P.dqn_create(cfg, sa, stt)
    theta = synth.init_params(args.seed, A)
    P.dqn_set_params(ctx, P.DQN_PARAMS_ONLINE, theta)
    P.dqn_set_params(ctx, P.DQN_PARAMS_TARGET, theta)
    frames -= frames % W
    rb = P.replay_create(frames, W, C // W, args.seed, sa, stt)
    ac = P.dqn_alg1_config()
    ac.W, ac.C, ac.F, ac.B, ac.epsilon = W, C, F, B, 0.1
    ac.t_reward_neg, ac.t_reward_pos, ac.t_term = synth.thresholds(args.p_reward, args.p_reward, args.p_term)
    ac.concurrent, ac.synchronized, ac.env_step_ns = concurrent, synchronized, args.alg1_env_ns
    ac.env_seed = args.seed
    h = P.dqn_alg1_create(ctx, rb, ac)
    try:
        # prepopulation (Table 5: N = 50000), in pieces the temporary buffers can hold; also the sampler side's rate alone
        n_pre = prepopulate - prepopulate % C
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_pre // C):
            P.dqn_alg1_prepopulate(h, C)
        torch.cuda.synchronize()
        pre_s = time.perf_counter() - t0
        if warmup_blocks:
            P.dqn_alg1_run(h, C * warmup_blocks)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        P.dqn_alg1_run(h, C * blocks)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        stats = P.dqn_alg1_stats(h)
    finally:
        torch.cuda.synchronize()
        P.dqn_alg1_destroy(h)
        P.replay_destroy(rb)
        P.dqn_destroy(ctx)
    return {"elapsed": el, "timesteps_per_sec": C * blocks / el, "train_steps_per_sec": C // F * blocks / el,
            "act_rounds_per_sec": C // W * blocks / el, "samplers_alone_timesteps_per_sec": n_pre / pre_s if n_pre else None,
            "prepopulated": n_pre, "frames": frames, "totals": stats}


ALG1_CONTEXT = ("paper: 200M frames = 50M timesteps in 9 h on one GTX 1080 with the real emulator (about 1,500 "
                "timesteps/s); here the environment is a seeded frame generator, so this rate bounds the loop "
                "around the emulator, not the emulator")


def algorithm1(args):
    """Algorithm 1 end to end (dqn_alg1_*): W sampler threads on synthetic host environments, the trainer thread,
    synchronisation every C timesteps.  Prints one JSON line of its own; not the headline metric."""
    W, C, F, B, A = args.envs, args.alg1_c, args.alg1_f, args.batch, args.actions
    blocks, warm = args.alg1_blocks, max(args.alg1_warmup_blocks, 1)
    r = run_alg1(args, W, 1, 1, blocks, warm, args.alg1_prepopulate, args.frames)
    out = {
        "metric": "Algorithm 1 timesteps/sec (W=%d synthetic host environments, batch %d)" % (W, B),
        "value": r["timesteps_per_sec"], "unit": "timesteps/s",
        "train_steps_per_sec": r["train_steps_per_sec"], "act_steps_per_sec": r["act_rounds_per_sec"],
        "samplers_alone_timesteps_per_sec": r["samplers_alone_timesteps_per_sec"],
        "n_gpus": 1, "steps": blocks, "warmup": warm, "ms_per_step": 1e3 * r["elapsed"] / blocks,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if args.precision == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "Algorithm 1, Table 5 schedule: A=%d, W=%d, C=%d, F=%d, batch %d, replay %d frames, "
                               "prepopulation %d, %d ns of stand-in emulator time per environment step; a step is one "
                               "block of C timesteps" % (A, W, C, F, B, r["frames"], r["prepopulated"], args.alg1_env_ns),
                   "seed": args.seed},
        "totals": r["totals"], "context": ALG1_CONTEXT,
    }
    print(json.dumps(out))
    return 0


def ablation(args):
    """The shape of Tables 1-3 (Section 5.1) on synthetic environments: {standard, concurrent, synchronized, both} x
    W in {1, 2, 4, 8} (synchronization needs W > 1: 14 variants), timesteps/s each and the speed-up over standard
    DQN with one sampler.  Prints a table, then one JSON line."""
    C = args.alg1_c
    rows = []
    for name, conc, sync in (("standard", 0, 0), ("concurrent", 1, 0), ("synchronized", 0, 1), ("both", 1, 1)):
        for W in (1, 2, 4, 8):
            if sync and W == 1:
                continue
            r = run_alg1(args, W, conc, sync, args.alg1_blocks, 1, C, min(args.frames, 200000))
            rows.append({"variant": name, "W": W, "timesteps_per_sec": r["timesteps_per_sec"],
                         "hours_per_50M_timesteps": 50e6 / r["timesteps_per_sec"] / 3600})
    base = rows[0]["timesteps_per_sec"]
    for r in rows:
        r["speedup"] = r["timesteps_per_sec"] / base
        print("%-13s W=%d  %9.0f timesteps/s  %6.2f h per 50M timesteps  x%.2f" %
              (r["variant"], r["W"], r["timesteps_per_sec"], r["hours_per_50M_timesteps"], r["speedup"]), file=sys.stderr)
    print(json.dumps({"metric": "ablation of Section 5.1 on synthetic environments, timesteps/sec", "unit": "timesteps/s",
                      "rows": rows, "n_gpus": 1, "data": "synthetic", "dtype": "bf16" if args.precision == "bf16" else "f32",
                      "config": {"workload": "A=%d, C=%d, F=%d, batch %d, %d timed blocks of C timesteps per variant, %d ns of "
                                             "stand-in emulator time per environment step"
                                             % (args.actions, C, args.alg1_f, args.batch, args.alg1_blocks, args.alg1_env_ns)},
                      "context": ALG1_CONTEXT}))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--precision", choices=["bf16", "fp32"], default="bf16")
    ap.add_argument("--actions", type=int, default=18)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--envs", type=int, default=8)
    ap.add_argument("--lanes", type=int, default=8)
    ap.add_argument("--frames", type=int, default=1000000)
    ap.add_argument("--acts-per-train", type=int, default=4)
    ap.add_argument("--sync-every", type=int, default=10000)
    ap.add_argument("--double-dqn", action="store_true")
    ap.add_argument("--p-reward", type=float, default=0.05)
    ap.add_argument("--p-term", type=float, default=0.001)
    ap.add_argument("--seed", type=int, default=211101264 + 2)
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-push", action="store_true",
                    help="replay_push_step and dqn_act as two calls per act step instead of dqn_act_push_step")
    ap.add_argument("--separate-gather", action="store_true",
                    help="replay_sample_gather and dqn_train_step as two calls instead of dqn_train_step_sampled")
    ap.add_argument("--sweep", action="store_true", help="the batch/W roofline sweep: one JSON line per point")
    ap.add_argument("--algorithm1", action="store_true",
                    help="time the Algorithm 1 orchestrator (dqn_alg1_*) instead: one JSON line of its own")
    ap.add_argument("--ablation", action="store_true",
                    help="the 14 variants of the Section 5.1 ablation on synthetic environments (table + one JSON line)")
    ap.add_argument("--alg1-c", type=int, default=10000, help="target update period C in timesteps (Table 5)")
    ap.add_argument("--alg1-f", type=int, default=4, help="training period F in timesteps (Table 5)")
    ap.add_argument("--alg1-prepopulate", type=int, default=50000, help="prepopulation N (Table 5), rounded down to C")
    ap.add_argument("--alg1-blocks", type=int, default=20, help="timed blocks of C timesteps")
    ap.add_argument("--alg1-warmup-blocks", type=int, default=2)
    ap.add_argument("--alg1-env-ns", type=int, default=0,
                    help="busy time per environment step standing in for an emulator's own cost (default: none)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one MI355X: this library runs on one GPU, run with --gpus 1", file=sys.stderr)
        return 2

    if args.sweep:
        return sweep(args)
    if args.algorithm1:
        return algorithm1(args)
    if args.ablation:
        return ablation(args)

    wl = Workload(args)
    groups = 3 if args.double_dqn else 2
    time_steps(wl, max(args.warmup // 2, 1))
    # find the dominant train-step kernel before the timed region, then time it inside the region
    breakdown = kernel_breakdown(wl, max(min(args.warmup // 30, 50), 5))
    breakdown.pop("event_pair", None)
    dominant = max(breakdown, key=breakdown.get)
    time_steps(wl, max(args.warmup // 2, 1))
    kid = [wl.P.dqn_profile_kernel_name(i) for i in range(wl.P.dqn_profile_kernel_count() + 1)].index(dominant)
    # a sample of the dominant kernel's launches spread over the whole timed region (at most 4096 are kept); the
    # timing events are bound to the kernel's own dispatch, so the average is the kernel's begin-to-end time on the
    # GPU -- the duration rocprofv3's kernel trace reports for it
    every = max(1, -(-args.steps // 2048))
    wl.P.dqn_profile_select_every(wl.ctx, kid, every)
    elapsed = time_steps(wl, args.steps)
    ms, n = wl.P.dqn_profile_read(wl.ctx)
    wl.P.dqn_profile_select(wl.ctx, 0)
    roof = roofline_for(dominant, max(ms / max(n, 1), 1e-6), args.batch, args.actions, groups, args.precision)
    roof["traffic"], roof["traffic_source"] = measured_traffic(dominant, args.batch, args.precision)
    roof["timed_launches"] = n
    roof["timed_every"] = every
    roof["timing"] = "HIP events bound to the kernel's dispatch on the train stream (hipExtLaunchKernel), live in the timed region"
    # each side alone (what the overlap hides): short runs outside the timed region
    alone_steps = max(min(args.steps // 5, 2000), 200)
    train_alone = alone_steps / time_steps(wl, alone_steps, "train")
    act_alone = (alone_steps * args.acts_per_train * args.envs / time_steps(wl, alone_steps, "act")) if args.acts_per_train else 0.0
    wl.close()

    out = {
        "metric": "train steps/sec (batch %d) + act states/sec" % args.batch,
        "value": args.steps / elapsed,
        "unit": "train steps/s",
        "act_states_per_sec": args.steps * args.acts_per_train * args.envs / elapsed,
        "alone": {"train_steps_per_sec": train_alone, "act_states_per_sec": act_alone,
                  "note": "each side run by itself over %d steps; `value` is with both overlapped" % alone_steps},
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if args.precision == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": "paper-shaped slice: A=%d, W=%d envs, replay %d frames in %d lanes, batch %d, "
                               "%d act steps per train step on a concurrent stream, target sync every %d train steps"
                               % (args.actions, args.envs, args.frames, args.lanes, args.batch, args.acts_per_train,
                                  args.sync_every),
                   "double_dqn": bool(args.double_dqn), "seed": args.seed},
        "kernel_avg_us": {k: round(v * 1e3, 2) for k, v in breakdown.items()},
        "roofline": roof,
        "context": "paper: 25 h -> 9 h for 200M frames on one GTX 1080 (end to end, emulator included)",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args)
    print(json.dumps(out))
    return 0


def sweep(args):
    """Batch in {128,256,512} x W in {32,64,128}, bf16: one JSON line per point with the per-kernel durations (events
    bound to each kernel's dispatch), their roofline fractions on algorithmic FLOPs / bytes, the gather's bandwidth
    and a `roofline` object for the point's longest train-step kernel; a readable table goes to stderr."""
    import copy
    for B, W in ((128, 32), (256, 64), (512, 128)):
        a = copy.copy(args)
        a.batch, a.envs, a.acts_per_train = B, W, 1
        a.frames = min(args.frames, 200000)
        wl = Workload(a)
        groups = 3 if a.double_dqn else 2
        time_steps(wl, 60)
        br = kernel_breakdown(wl, 100)
        br.pop("event_pair", None)
        steps = 300
        el = time_steps(wl, steps)
        torch = wl.torch
        # the stand-alone gather kernel, timed with events on the train stream over 50 back-to-back launches
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(wl.train_stream)
        for i in range(50):
            wl.P.replay_sample_gather(wl.rb, B, i, None, wl.s, wl.s2, wl.a, wl.r, wl.d, None)
        e1.record(wl.train_stream)
        torch.cuda.synchronize()
        g_ms = e0.elapsed_time(e1) / 50
        wl.close()
        kernels = {name: roofline_for(name, ms, B, a.actions, groups, a.precision) for name, ms in br.items()}
        longest = max(br, key=br.get)
        roof = dict(kernels[longest])
        roof["traffic"], roof["traffic_source"] = measured_traffic(longest, B, a.precision)
        print("B=%d W=%d  %.1f train steps/s  %.1f us/step  gather %.1f us = %.0f GB/s" %
              (B, W, steps / el, 1e6 * el / steps, g_ms * 1e3, 91728 * B / (g_ms * 1e-3) / 1e9), file=sys.stderr)
        for name, r in kernels.items():
            print("   %-14s %8.1f us  %-4s %9.1f %-7s  %5.1f %%" % (name, r["avg_launch_us"], r["bound"], r["achieved"],
                                                                     r["unit"], 100 * r["frac"]), file=sys.stderr)
        print(json.dumps({
            "metric": "train steps/sec (batch %d) + act states/sec" % B, "value": steps / el, "unit": "train steps/s",
            "act_states_per_sec": steps * W / el, "n_gpus": 1, "steps": steps, "warmup": 60, "ms_per_step": 1e3 * el / steps,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if a.precision == "bf16" else "f32",
            "data": "synthetic",
            "config": {"workload": "roofline scaling point: A=%d, batch %d, W=%d, 1 act step per train step on a concurrent "
                                   "stream, replay %d frames" % (a.actions, B, W, a.frames), "double_dqn": bool(a.double_dqn),
                       "seed": a.seed},
            "roofline": roof,
            "kernels": {k: {"avg_launch_us": round(v["avg_launch_us"], 2), "bound": v["bound"], "frac": round(v["frac"], 4)}
                        for k, v in kernels.items()},
            "gather": {"avg_launch_us": g_ms * 1e3, "achieved": 91728 * B / (g_ms * 1e-3) / 1e9, "unit": "GB/s",
                       "frac": 91728 * B / (g_ms * 1e-3) / 1e9 / PEAK["hbm"][0],
                       "note": "stand-alone replay_sample_gather, 50 back-to-back launches between two event records"},
        }))
    return 0


if __name__ == "__main__":
    sys.exit(main())
