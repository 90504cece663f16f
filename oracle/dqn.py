"""CPU oracle of the DQN act step and minibatch train step.  TEST INFRASTRUCTURE ONLY.

Thin ctypes layer over `dqn_oracle.c` (double precision, direct loops) plus the few steps that are
easier to read in Python: input scaling, epsilon-greedy selection, the order of the train step.

Paper passages followed: Section 2.1 (Q-network, greedy policy, Eq. 1, target network, epsilon-greedy),
Section 3 (actions computed from the target parameters under Concurrent Training), Section 4 (one
minibatch of W states per act step), Appendix B (RMSProp constants), Table 5 (gamma, minibatch 32).
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build
from . import philox

MAX_LAYERS = 4


class NetDesc(C.Structure):
    _fields_ = [
        ("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
        ("n_conv", C.c_int32),
        ("conv_out", C.c_int32 * MAX_LAYERS), ("conv_k", C.c_int32 * MAX_LAYERS),
        ("conv_s", C.c_int32 * MAX_LAYERS),
        ("n_fc", C.c_int32),
        ("fc_out", C.c_int32 * MAX_LAYERS),
    ]


def make_desc(in_shape, convs, fcs) -> NetDesc:
    """in_shape = (C, H, W); convs = [(out, k, stride), ...]; fcs = [out, ...]."""
    d = NetDesc()
    d.in_c, d.in_h, d.in_w = in_shape
    d.n_conv = len(convs)
    for i, (o, k, s) in enumerate(convs):
        d.conv_out[i], d.conv_k[i], d.conv_s[i] = o, k, s
    d.n_fc = len(fcs)
    for i, o in enumerate(fcs):
        d.fc_out[i] = o
    return d


def nature_desc(num_actions: int) -> NetDesc:
    """[4,84,84] -> conv 32@8x8 s4 -> conv 64@4x4 s2 -> conv 64@3x3 s1 -> fc 512 -> fc A."""
    return make_desc((4, 84, 84), [(32, 8, 4), (64, 4, 2), (64, 3, 1)], [512, num_actions])


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        dp = C.POINTER(C.c_double)
        ip = C.POINTER(C.c_int32)
        L.onet_num_params.restype = C.c_size_t
        L.onet_num_params.argtypes = [C.POINTER(NetDesc)]
        L.onet_acts_per_sample.restype = C.c_size_t
        L.onet_acts_per_sample.argtypes = [C.POINTER(NetDesc)]
        L.onet_forward.restype = None
        L.onet_forward.argtypes = [C.POINTER(NetDesc), dp, dp, C.c_int, dp, dp]
        L.onet_backward.restype = None
        L.onet_backward.argtypes = [C.POINTER(NetDesc), dp, dp, C.c_int, dp, dp, dp, dp]
        L.greedy_actions.restype = None
        L.greedy_actions.argtypes = [dp, C.c_int, C.c_int, ip]
        L.td_loss.restype = C.c_double
        L.td_loss.argtypes = [dp, dp, dp, ip, dp, dp, C.c_double, C.c_double, C.c_int, C.c_int,
                              dp, dp, dp]
        L.rmsprop_step.restype = None
        L.rmsprop_step.argtypes = [dp, dp, dp, dp, C.c_size_t, C.c_double, C.c_double, C.c_double,
                                   C.c_int]
        L.oracle_max_threads.restype = C.c_int
        L.oracle_max_threads.argtypes = []
        L.oracle_set_threads.restype = C.c_int
        L.oracle_set_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def set_threads(n: int) -> int:
    """Thread count of the C loops from now on (timing only: results are independent of it); returns the previous one."""
    return int(lib().oracle_set_threads(int(n)))


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_params(desc: NetDesc) -> int:
    return int(lib().onet_num_params(C.byref(desc)))


def forward(desc: NetDesc, theta, x):
    """x: [B, C, H, W] float64 (already scaled).  Returns (q [B,A], acts workspace)."""
    theta, x = _f64(theta), _f64(x)
    B = x.shape[0]
    A = desc.fc_out[desc.n_fc - 1]
    acts = np.zeros((B, int(lib().onet_acts_per_sample(C.byref(desc)))), dtype=np.float64)
    q = np.zeros((B, A), dtype=np.float64)
    lib().onet_forward(C.byref(desc), _dp(theta), _dp(x), B, _dp(acts), _dp(q))
    return q, acts


def backward(desc: NetDesc, theta, x, acts, dq):
    theta, x, acts, dq = _f64(theta), _f64(x), _f64(acts), _f64(dq)
    grad = np.zeros(theta.size, dtype=np.float64)
    dz = np.zeros_like(acts)
    lib().onet_backward(C.byref(desc), _dp(theta), _dp(x), x.shape[0], _dp(acts), _dp(dq), _dp(dz),
                        _dp(grad))
    return grad


def greedy_actions(q):
    q = _f64(q)
    out = np.zeros(q.shape[0], dtype=np.int32)
    lib().greedy_actions(_dp(q), q.shape[0], q.shape[1], _ip(out))
    return out


def td_loss(q_sa, q_next_t, q_next_o, a, r, done, gamma, huber):
    """Returns (loss, y[B], td[B], dq[B,A]).  q_next_o=None -> Eq. 1's max over theta^-."""
    q_sa, q_next_t = _f64(q_sa), _f64(q_next_t)
    B, A = q_sa.shape
    a = np.ascontiguousarray(a, dtype=np.int32)
    r, done = _f64(r), _f64(done)
    y = np.zeros(B)
    td = np.zeros(B)
    dq = np.zeros((B, A))
    qo = None
    if q_next_o is not None:
        q_next_o = _f64(q_next_o)
        qo = _dp(q_next_o)
    loss = lib().td_loss(_dp(q_sa), _dp(q_next_t), qo, _ip(a), _dp(r), _dp(done), gamma, huber,
                         B, A, _dp(y), _dp(td), _dp(dq))
    return float(loss), y, td, dq


def rmsprop_step(theta, g, v, m, lr, alpha, eps, centered=True):
    """In-place on float64 arrays theta, v, m."""
    g = _f64(g)
    assert theta.dtype == np.float64 and v.dtype == np.float64 and m.dtype == np.float64
    lib().rmsprop_step(_dp(theta), _dp(g), _dp(v), _dp(m), theta.size, lr, alpha, eps,
                       int(bool(centered)))


def scale_states(states_u8):
    """uint8 [.., 4, 84, 84] -> float64 in [0, 1]."""
    return np.asarray(states_u8, dtype=np.float64) / 255.0


def epsilon_greedy(q, epsilon, seed, act_step):
    """Random action with probability epsilon, greedy (lowest-index argmax) otherwise; the
    inverted wording of Section 2.1 is read the way Sections 2.1's schedule remark and 5.1 need it.
    Environment j at act step n uses the generator outputs (x0, x1, ..) for (seed, ACT, n, j):
    u = (x0 >> 8) * 2**-24 compared with epsilon in float32; random action = (x1 * A) >> 32."""
    q = _f64(q)
    W, A = q.shape
    greedy = greedy_actions(q)
    out = np.empty(W, dtype=np.int32)
    eps32 = np.float32(epsilon)
    for j in range(W):
        x0, x1, _, _ = philox.draw(seed, philox.TAG_ACT, act_step, j)
        u = np.float32(x0 >> 8) * np.float32(2.0 ** -24)
        out[j] = (x1 * A) >> 32 if u < eps32 else greedy[j]
    return out


class OracleDQN:
    """theta, theta^-, RMSProp state in float64; the calls mirror the library's."""

    def __init__(self, num_actions, params_f32, gamma=0.99, huber=1.0, lr=2.5e-4, alpha=0.95,
                 eps=0.01, centered=True, double_dqn=False, seed=0, desc=None):
        self.desc = desc if desc is not None else nature_desc(num_actions)
        self.A = num_actions
        self.theta = np.array(params_f32, dtype=np.float64)
        assert self.theta.size == num_params(self.desc)
        self.theta_target = self.theta.copy()
        self.v = np.zeros_like(self.theta)
        self.m = np.zeros_like(self.theta)
        self.gamma, self.huber, self.lr, self.alpha, self.eps = gamma, huber, lr, alpha, eps
        self.centered, self.double_dqn, self.seed = centered, double_dqn, seed
        self.last_grad = None

    def q_values(self, states_u8, use_target=True):
        th = self.theta_target if use_target else self.theta
        return forward(self.desc, th, scale_states(states_u8))[0]

    def act(self, states_u8, epsilon, act_step, use_target=True):
        q = self.q_values(states_u8, use_target)
        return epsilon_greedy(q, epsilon, self.seed, act_step), q

    def train_step(self, s, a, r, s2, done):
        x, x2 = scale_states(s), scale_states(s2)
        q_sa, acts = forward(self.desc, self.theta, x)
        q_next_t, _ = forward(self.desc, self.theta_target, x2)
        q_next_o = forward(self.desc, self.theta, x2)[0] if self.double_dqn else None
        loss, y, td, dq = td_loss(q_sa, q_next_t, q_next_o, a, r, done, self.gamma, self.huber)
        g = backward(self.desc, self.theta, x, acts, dq)
        rmsprop_step(self.theta, g, self.v, self.m, self.lr, self.alpha, self.eps, self.centered)
        self.last_grad = g
        return loss, q_sa, y

    def sync_target(self):
        self.theta_target = self.theta.copy()
