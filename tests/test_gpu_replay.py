"""GPU parity: replay ring, staging/flush, sampling, frame-stack gather -- bit-exact vs the oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2111_01264_amd as P
from datagen import synth
from oracle.replay import OracleReplay
from tests.gpu_util import dev, fill_replay_from_host


def gather_gpu(rb, B, step, idx_in=None):
    s = torch.empty((B, 4, 84, 84), dtype=torch.uint8, device="cuda")
    s2 = torch.empty_like(s)
    a = torch.empty(B, dtype=torch.int32, device="cuda")
    r = torch.empty(B, dtype=torch.float32, device="cuda")
    d = torch.empty(B, dtype=torch.float32, device="cuda")
    idx = torch.empty(B, dtype=torch.int64, device="cuda")
    P.replay_sample_gather(rb, B, step, idx_in, s, s2, a, r, d, idx)
    torch.cuda.synchronize()
    return s.cpu().numpy(), s2.cpu().numpy(), a.cpu().numpy(), r.cpu().numpy(), d.cpu().numpy(), idx.cpu().numpy()


def check_equal(got, want_idx, orc):
    s, s2, a, r, d, idx = got
    assert np.array_equal(idx, want_idx)
    ws, ws2, wa, wr, wd = orc.gather(want_idx)
    assert np.array_equal(s, ws) and np.array_equal(s2, ws2)
    assert np.array_equal(a, wa) and np.array_equal(r, wr) and np.array_equal(d, wd)


def test_synth_kernels_match_generator():
    n, seed = 37, 99
    dst = torch.empty((n, 84, 84), dtype=torch.uint8, device="cuda")
    P.synth_frames(dst, n, 1000, 3, seed, synth.STREAM_REPLAY, synth.PIX_T, synth.BACKGROUND, None)
    ids = 1000 + 3 * np.arange(n)
    assert np.array_equal(dst.cpu().numpy(), synth.frames(seed, synth.STREAM_REPLAY, ids))
    m = 5000
    a = torch.empty(m, dtype=torch.int32, device="cuda")
    r = torch.empty(m, dtype=torch.float32, device="cuda")
    t = torch.empty(m, dtype=torch.uint8, device="cuda")
    tn, tp, tt = synth.thresholds(0.1, 0.1, 0.01)
    P.synth_transitions(a, r, t, m, 7, 2, seed, 18, tn, tp, tt, None)
    wa, wr, wt = synth.transitions(seed, 7 + 2 * np.arange(m), 18, 0.1, 0.1, 0.01)
    assert np.array_equal(a.cpu().numpy(), wa) and np.array_equal(r.cpu().numpy(), wr)
    assert np.array_equal(t.cpu().numpy(), wt)


@pytest.mark.parametrize("lanes", [1, 4])
def test_push_flush_sample_gather_bit_exact(lanes):
    N, seed = 400 * lanes, 31 + lanes
    st = torch.cuda.Stream()
    rb = P.replay_create(N, lanes, 150, seed, st, st)
    orc = OracleReplay(N, lanes, seed)
    rng = np.random.default_rng(lanes)
    tcount = [0] * lanes
    try:
        for rnd in range(7):         # ragged pushes, wrap-around after a few rounds, frequent terminals
            for lane in range(lanes):
                n = int(rng.integers(0, 150))
                ids = (np.arange(tcount[lane], tcount[lane] + n, dtype=np.uint64) * np.uint64(lanes) + np.uint64(lane))
                tcount[lane] += n
                f = synth.frames(seed, synth.STREAM_REPLAY, ids)
                a, r, d = synth.transitions(seed, ids, 6, 0.05, 0.05, 0.2)
                if n:
                    # staged in two calls to exercise appends
                    h = n // 2
                    P.replay_push(rb, lane, dev(f[:h]), dev(a[:h]), dev(r[:h]), dev(d[:h]), h)
                    P.replay_push(rb, lane, dev(f[h:]), dev(a[h:]), dev(r[h:]), dev(d[h:]), n - h)
                    orc.push(lane, f, a, r, d)
            if rnd == 0:
                assert P.replay_num_valid(rb) == 0            # staged pushes are invisible
            before = None
            if P.replay_num_valid(rb) > 0:
                before = gather_gpu(rb, 16, 1000 + rnd)
                check_equal(before, orc.sample_indices(16, 1000 + rnd), orc)   # D unchanged while staging fills
            P.replay_flush(rb, 1)
            orc.flush()
            assert P.replay_num_valid(rb) == orc.num_valid()
            if orc.num_valid() > 0:
                for step in (rnd, rnd + 100):
                    check_equal(gather_gpu(rb, 37, step), orc.sample_indices(37, step), orc)
        # every valid transition through idx_in, in ragged batches
        allidx = np.array([l * orc.M + j for l in range(lanes) for j in range(3, orc.count[l] - 1)], dtype=np.int64)
        for lo in range(0, allidx.size, 301):
            part = allidx[lo:lo + 301]
            check_equal(gather_gpu(rb, part.size, 0, dev(part)), part, orc)
        # invalid indices are reported, not read
        bad = np.array([0, orc.M * lanes + 5, -3, orc.count[0] - 1], dtype=np.int64)
        s, s2, a, r, d, idx = gather_gpu(rb, 4, 0, dev(bad))
        assert (a == -1).all() and not s.any() and not s2.any()
    finally:
        P.replay_destroy(rb)


def test_error_paths():
    st = torch.cuda.Stream()
    rb = P.replay_create(64, 2, 8, 1, st, st)
    try:
        z = torch.zeros((9, 84, 84), dtype=torch.uint8, device="cuda")
        ai = torch.zeros(9, dtype=torch.int32, device="cuda")
        rf = torch.zeros(9, dtype=torch.float32, device="cuda")
        tu = torch.zeros(9, dtype=torch.uint8, device="cuda")
        with pytest.raises(P.DqnError) as e:
            P.replay_push(rb, 2, z, ai, rf, tu, 1)
        assert e.value.code == P.DQN_EINVAL
        with pytest.raises(P.DqnError) as e:
            P.replay_push(rb, 0, z, ai, rf, tu, 9)      # staging holds 8
        assert e.value.code == P.DQN_ESTATE
        s = torch.empty((2, 4, 84, 84), dtype=torch.uint8, device="cuda")
        with pytest.raises(P.DqnError) as e:
            P.replay_sample_gather(rb, 2, 0, None, s, s, ai, rf, rf, None)
        assert e.value.code == P.DQN_ESTATE              # nothing flushed yet
        P.replay_push(rb, 0, z, ai, rf, tu, 4)
        P.replay_flush(rb, 1)
        assert P.replay_num_valid(rb) == 0                # 4 frames: no complete transition
    finally:
        P.replay_destroy(rb)
