"""Tight parity of the bf16 backward / optimiser kernels with the fp64 oracle, on inputs where no ReLU can flip.

The bf16 train step runs its own kernels for the data gradients, the weight gradients and the 16-bit branch of the
optimiser.  On realistic data a ReLU whose pre-activation lies within operand rounding of zero switches state for single
samples, which moves whole rows of a gradient and leaves only norm-wise bounds meaningful.  Here the parameters come
from datagen.synth.margin_params: every hidden channel's weighted sum of non-negative inputs has the sign of its bias
(|bias| = 0.5), so every hidden unit is on -- or, in the split variant, odd channels are off -- for ANY input, with a
margin three orders of magnitude above bf16 rounding.  What is left between the two sides is operand rounding:

  * every bf16 operand carries a relative rounding error uniform in +-2^-9 (standard deviation 1.1e-3), a product
    of two of them 1.6e-3; a gradient element is a sum of such products with independent errors, so its error has
    a standard deviation of about 1.6e-3 of the root-sum-square of its terms -- at most of the element's own typical
    size -- and the factors handed down the backward chain (dz of up to four layers, each stored as bf16) add in
    quadrature: about 3.5e-3 of a typical element.  The largest of ~10^6 such errors is about five standard deviations,
    1.7e-2 of a TYPICAL element, while the tensor's largest element is several times a typical one: <= ~0.5 % of
    max|ref|;
  * the TD error delta = Q(s,a) - y is formed from Q values with relative error <= 2e-2 * max|Q|; the rewards used
    here (+-2 and +-30 against |Q| < 0.4, clipping threshold 10) keep |delta| >= 1.2 or clipped, so dL/dQ carries
    <= 2e-2 * 0.4 / 1.2 = 0.7 % from that.

Bound asserted: every gradient tensor max|gpu - ref| <= 2e-2 * max|ref| (the bound the library states for Q; the model above
leaves it a factor of about two to four); first-step optimiser state v, m and the update theta_1 - theta_0 to what that gradient
bound implies (d(update)/dg <= lr / eps for the first step from zero state).  A dropped k-tile, a wrong split-K slice
count, a shifted filter tap or a mis-masked border pixel changes elements by far more than that.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2111_01264_amd as P
from datagen import synth
from oracle import dqn as odqn
from oracle.replay import OracleReplay
from tests.gpu_util import blob_slices, dev, make_cfg, rel_err

GRAD_TOL = 2e-2
Q_TOL = 2e-2
REWARDS = np.array([-30.0, -2.0, 2.0, 30.0], dtype=np.float32)
HUBER = 10.0     # errors of +-2 stay in the quadratic zone, those of +-30 are clipped
LR = 2.5e-5      # RMSProp's first step moves every parameter by up to lr / 0.218 whatever its gradient; fc2 adds 512 of
                 # them times h ~ 3, so the default 2.5e-4 would lift |Q| to ~1.7 in one step and the second step's TD
                 # errors would inherit the Q tolerance many times over; with 2.5e-5 |Q| stays below 0.4
Q_MAX = 0.4


def check_margin_by_construction(theta, A, split):
    """Every hidden weight has the sign of its channel's bias, |bias| = MARGIN_BIAS."""
    sl = blob_slices(A)
    for name, shape, _ in synth.layer_shapes(A):
        if name == "fc2":
            continue
        w = theta[sl[name + ".w"]].reshape(shape[0], -1)
        b = theta[sl[name + ".b"]]
        assert np.all(np.abs(b) == np.float32(synth.MARGIN_BIAS))
        assert np.all(np.sign(w) * np.sign(b)[:, None] >= 0)
        assert np.all(b[0::2] > 0) and np.all((b[1::2] < 0) if split else (b[1::2] > 0))


def compare_step(ctx, orc, A, B, double_dqn, loss_dev, wloss, q_sa, first_step, theta0, lr, eps, alpha):
    """Asserts Q, loss, every gradient tensor and (first step) v, m, update against the oracle's step."""
    sl = blob_slices(A)
    assert np.abs(q_sa).max() < Q_MAX      # the premise of the dL/dQ bound in the module docstring
    q_on, _, _ = P.dqn_get_train_q(ctx, B, A, bool(double_dqn))
    assert rel_err(q_on, q_sa) <= Q_TOL, ("q_online", rel_err(q_on, q_sa))
    assert abs(float(loss_dev.item()) - wloss) <= 1e-2 * abs(wloss), (loss_dev.item(), wloss)
    g = P.dqn_get_params(ctx, P.DQN_PARAMS_GRAD)
    errs = {name: rel_err(g[slc], orc.last_grad[slc]) for name, slc in sl.items()}
    print("bf16 flip-free: B=%d per-tensor max-norm gradient errors: %s" % (B, " ".join("%s %.1e" % kv for kv in errs.items())))
    for name, e in errs.items():
        assert e <= GRAD_TOL, ("grad", name, e)
    if not first_step:
        return
    th = P.dqn_get_params(ctx, P.DQN_PARAMS_ONLINE)
    v = P.dqn_get_params(ctx, P.DQN_PARAMS_RMS_V)
    m = P.dqn_get_params(ctx, P.DQN_PARAMS_RMS_M)
    for name, slc in sl.items():
        gmax = np.abs(orc.last_grad[slc]).max()
        assert np.abs(m[slc] - orc.m[slc]).max() <= (1 - alpha) * GRAD_TOL * gmax + 1e-12, ("m", name)
        assert np.abs(v[slc] - orc.v[slc]).max() <= (1 - alpha) * 2.1 * GRAD_TOL * gmax * gmax + 1e-12, ("v", name)
        # first step from zero state: |d(update)/dg| <= lr / eps; plus half an ulp of theta in fp32
        bound = lr / eps * GRAD_TOL * gmax + 2.0 ** -24 * np.abs(theta0[slc]).max()
        d_gpu = th[slc].astype(np.float64) - theta0[slc].astype(np.float64)
        d_ref = orc.theta[slc] - theta0[slc].astype(np.float64)
        assert np.abs(d_gpu - d_ref).max() <= bound, ("update", name, np.abs(d_gpu - d_ref).max(), bound)


# 45 and 97: the conv weight-gradient workgroups walk two / four samples each and the last one gets a single sample (the
# padding item of an odd range); 32: one sample per workgroup; 300, 256: many per workgroup, ragged and even
@pytest.mark.parametrize("B,split,double_dqn", [(32, False, 0), (32, True, 1), (45, False, 0), (97, True, 1), (300, True, 0),
                                                (256, False, 1)])
def test_bf16_train_step_max_norm_no_relu_flips(B, split, double_dqn):
    A, seed = 18, 4100 + B
    cfg = make_cfg(A, max_batch=B, max_envs=8, precision=P.DQN_PRECISION_BF16, double_dqn=double_dqn, seed=seed)
    cfg.lr, cfg.huber_delta = LR, HUBER
    sa, stt = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = P.dqn_create(cfg, sa, stt)
    try:
        theta0 = synth.margin_params(seed, A, split)
        theta_t = synth.margin_params(seed + 1, A, split)
        check_margin_by_construction(theta0, A, split)
        check_margin_by_construction(theta_t, A, split)
        P.dqn_set_params(ctx, P.DQN_PARAMS_ONLINE, theta0)
        P.dqn_set_params(ctx, P.DQN_PARAMS_TARGET, theta_t)
        orc = odqn.OracleDQN(A, theta0, double_dqn=bool(double_dqn), seed=seed, lr=LR, huber=HUBER)
        orc.theta_target = theta_t.astype(np.float64)
        rng = np.random.default_rng(seed)
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        for step in range(2):
            s = synth.block_frames(seed + 10 + step, B * 4).reshape(B, 4, 84, 84)
            s2 = synth.block_frames(seed + 20 + step, B * 4).reshape(B, 4, 84, 84)
            a = rng.integers(0, A, size=B).astype(np.int32)
            r = REWARDS[rng.integers(0, 4, size=B)]
            d = (rng.random(B) < 0.2).astype(np.float32)
            P.dqn_train_step(ctx, dev(s), dev(a), dev(r), dev(s2), dev(d), B, loss)
            torch.cuda.synchronize()
            wloss, q_sa, _ = orc.train_step(s, a, r, s2, d)
            compare_step(ctx, orc, A, B, double_dqn, loss, wloss, q_sa, step == 0, theta0, cfg.lr, cfg.rms_eps,
                         cfg.rms_alpha)
    finally:
        P.dqn_destroy(ctx)


@pytest.mark.parametrize("B", [512, 101])
def test_bf16_sampled_train_step_max_norm_no_relu_flips(B):
    # through the replay memory and dqn_train_step_sampled (at these sizes the minibatch exists only as replay slots: the
    # conv kernels read the frames from the replay memory), two steps in a row so that the second one uses what the
    # first one prepared; 101 leaves the last conv workgroups a single sample
    A, lanes, per_lane, seed = 18, 8, 160, 777 + B
    N = lanes * per_lane
    cfg = make_cfg(A, max_batch=B, max_envs=8, precision=P.DQN_PRECISION_BF16, double_dqn=0, seed=seed)
    cfg.lr, cfg.huber_delta = LR, HUBER
    sa, stt = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = P.dqn_create(cfg, sa, stt)
    rb = P.replay_create(N, lanes, per_lane, seed, sa, stt)
    orep = OracleReplay(N, lanes, seed)
    try:
        theta0 = synth.margin_params(seed, A, True)
        check_margin_by_construction(theta0, A, True)
        P.dqn_set_params(ctx, P.DQN_PARAMS_ONLINE, theta0)
        P.dqn_set_params(ctx, P.DQN_PARAMS_TARGET, theta0)
        orc = odqn.OracleDQN(A, theta0, seed=seed, lr=LR, huber=HUBER)
        rng = np.random.default_rng(seed)
        for lane in range(lanes):
            f = synth.block_frames(seed + 1 + lane, per_lane)
            a = rng.integers(0, A, size=per_lane).astype(np.int32)
            r = REWARDS[rng.integers(0, 4, size=per_lane)]
            d = (rng.random(per_lane) < 0.03).astype(np.uint8)
            P.replay_push(rb, lane, dev(f), dev(a), dev(r), dev(d), per_lane)
            orep.push(lane, f, a, r, d)
        P.replay_flush(rb, 1)
        orep.flush()
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        for step in range(2):
            P.dqn_train_step_sampled(ctx, rb, B, step, 1, loss)
            torch.cuda.synchronize()
            ws, ws2, wa, wr, wd = orep.gather(orep.sample_indices(B, step))
            wloss, q_sa, _ = orc.train_step(ws, wa, wr, ws2, wd)
            compare_step(ctx, orc, A, B, 0, loss, wloss, q_sa, step == 0, theta0, cfg.lr, cfg.rms_eps, cfg.rms_alpha)
    finally:
        P.replay_destroy(rb)
        P.dqn_destroy(ctx)
