"""Pins for the oracle's wider rows: the server->worker bit-planes, per-worker coefficients
(and sign-momentum as beta1 == beta2), and the Global Lion comparison scheme."""
import numpy as np

import oracle
from test_oracle_pins import F32, bf16_bits, lion_single_worker, load_hand


# ----------------------------------------------------------------------------- down-link planes
def check_down_link(orc):
    h = load_hand()
    for key, N in (("N3", 3), ("N4", 4)):
        counts = np.array(h[key]["counts"], np.uint16)
        assert orc.encode_delta(counts, N, oracle.VOTE)[:, 0].tolist() == h["down_link"][key]["vote_planes"]
        assert orc.encode_delta(counts, N, oracle.AVG)[:, 0].tolist() == h["down_link"][key]["avg_planes"]
    rng = np.random.default_rng(3)
    for N in list(range(1, 41)) + [255, 256, 257, 1000, 65535]:
        # message sizes of Table 1: d bits for the vote (odd N; even N pays a tie plane), and
        # ceil(log2(N+1)) d bits for the average
        assert orc.delta_planes(N, oracle.VOTE) == (1 if N % 2 else 2)
        assert orc.delta_planes(N, oracle.AVG) == int(N).bit_length()
        d = N + 1 if N < 300 else 700
        counts = (np.arange(d) % (N + 1)).astype(np.uint16)
        rng.shuffle(counts)
        W = (d + 63) // 64
        for mode in (oracle.VOTE, oracle.AVG):
            planes = orc.encode_delta(counts, N, mode)
            assert planes.shape == (orc.delta_planes(N, mode), W)
            bits = np.unpackbits(planes.view(np.uint8), axis=1, bitorder="little")[:, : W * 64]
            assert not bits[:, d:].any()                      # bits past d are zero
            p = counts.astype(np.int64)
            if mode == oracle.AVG:
                rebuilt = sum(bits[b, :d].astype(np.int64) << b for b in range(planes.shape[0]))
                assert np.array_equal(rebuilt, p)
            else:
                assert np.array_equal(bits[0, :d].astype(bool), 2 * p > N)
                if N % 2 == 0:
                    assert np.array_equal(bits[1, :d].astype(bool), 2 * p == N)
            # a worker that decodes the message takes exactly the step the server-side apply takes
            x0 = rng.normal(0, 1, d).astype(F32)
            xa, xb = x0.copy(), x0.copy()
            Da = orc.apply(xa, counts, N, mode, 0.125, 0.25, want_delta=True)
            Db = orc.apply_encoded(xb, planes, N, mode, 0.125, 0.25, want_delta=True)
            assert np.array_equal(Da, Db) and np.array_equal(xa.view(np.uint32), xb.view(np.uint32))


def test_down_link_planes():
    check_down_link(oracle.default())


# ----------------------------------------------------------------------------- per-worker betas
def check_per_worker_betas(orc):
    h = load_hand()["per_worker_beta"]
    m = np.array(h["m"], F32)
    packed = orc.worker_step_pw(m, np.array(h["g"], F32), h["beta1"], h["beta2"])
    assert packed[:, 0].tolist() == h["words"] and m.tolist() == h["m1"]
    rng = np.random.default_rng(21)
    N, d = 6, 333
    b1 = np.array([0.9, 0.5, 0.95, 0.0, 1.0, 0.8], F32)
    b2 = np.array([0.99, 0.75, 0.98, 0.5, 0.25, 0.8], F32)
    m0 = rng.normal(0, 1, (N, d)).astype(F32)
    for use_bf16 in (False, True):
        g = rng.normal(0, 1, (N, d)).astype(F32)
        g_in = bf16_bits(g) if use_bf16 else g
        g_val = (g_in.astype(np.uint32) << 16).view(F32) if use_bf16 else g
        m = m0.copy()
        packed = orc.worker_step_pw(m, g_in, b1, b2)
        for i in range(N):
            # each worker is a single-worker Lion with its own coefficients (Eq. (1))
            _, m_ref, delta = lion_single_worker(np.zeros(d, F32), m0[i], g_val[i], b1[i], b2[i], 0.0, 0.0)
            assert np.array_equal(m[i].view(np.uint32), m_ref.view(np.uint32))
            row = np.unpackbits(packed[i].view(np.uint8), bitorder="little")[:d]
            assert np.array_equal(row.astype(bool), delta > 0)
        # equal coefficients for everyone: same as the shared-scalar worker step
        m_a, m_b = m0.copy(), m0.copy()
        pa = orc.worker_step_pw(m_a, g_in, np.full(N, 0.9, F32), np.full(N, 0.99, F32))
        pb = orc.worker_step(m_b, g_in, 0.9, 0.99)
        assert np.array_equal(pa, pb) and np.array_equal(m_a, m_b)
        # sign-momentum (beta1 == beta2): the bit is the sign of the new momentum, 0 -> +1
        m_s = m0.copy()
        ps = orc.worker_step_pw(m_s, g_in, np.full(N, 0.99, F32), np.full(N, 0.99, F32))
        bits = np.unpackbits(ps.view(np.uint8), axis=1, bitorder="little")[:, :d]
        assert np.array_equal(bits.astype(bool), ~(m_s < 0))


def test_per_worker_betas_and_signum():
    check_per_worker_betas(oracle.default())


# ----------------------------------------------------------------------------- Global Lion
def check_global_lion(orc):
    h = load_hand()
    gl = h["global_lion"]
    g = np.array([h["grads"][w] for w in gl["workers"]], F32)
    x = np.array(h["x0"], F32)
    m = np.zeros((3, 4), F32)
    bits = orc.global_lion_step(x, m, g, h["beta1"], h["beta2"], h["lr"], h["lambda"])
    assert int(bits[0]) == gl["sign_word"] and x.tolist() == gl["x1"]
    assert m.tolist() == [h["m1"][w] for w in gl["workers"]]
    rng = np.random.default_rng(31)
    d = 500
    # N = 1 is standard Lion (Eq. (1)), bit for bit
    x = rng.normal(0, 0.02, d).astype(F32)
    m = np.zeros((1, d), F32)
    xr, mr = x.copy(), m[0].copy()
    for _ in range(60):
        g = (rng.standard_t(3, d) * 1e-3).astype(F32)
        orc.global_lion_step(x, m, g[None, :].copy(), 0.9, 0.99, 3e-4, 0.1)
        xr, mr, _ = lion_single_worker(xr, mr, g, 0.9, 0.99, 3e-4, 0.1)
        assert np.array_equal(x.view(np.uint32), xr.view(np.uint32))
        assert np.array_equal(m[0].view(np.uint32), mr.view(np.uint32))
    # N identical workers, N a power of two: the mean blend is exactly one worker's blend
    for N in (2, 4, 8):
        x = rng.normal(0, 0.02, d).astype(F32)
        m1 = rng.normal(0, 1e-3, d).astype(F32)
        g1 = rng.normal(0, 1e-3, d).astype(F32)
        xr, mr, _ = lion_single_worker(x.copy(), m1, g1, 0.9, 0.99, 3e-4, 0.1)
        m = np.tile(m1, (N, 1))
        orc.global_lion_step(x, m, np.tile(g1, (N, 1)), 0.9, 0.99, 3e-4, 0.1)
        assert np.array_equal(x.view(np.uint32), xr.view(np.uint32))
        assert all(np.array_equal(m[i].view(np.uint32), mr.view(np.uint32)) for i in range(N))
    # where the workers are unanimous, averaging their blends cannot change the sign: Global
    # Lion and the majority vote of Distributed Lion take the same step there; and worker
    # momenta are the same in both schemes
    N = 5
    x0 = rng.normal(0, 0.02, d).astype(F32)
    m0 = rng.normal(0, 1, (N, d)).astype(F32)
    g = rng.normal(0, 1, (N, d)).astype(F32)
    xg, mg = x0.copy(), m0.copy()
    bits = orc.global_lion_step(xg, mg, g, 0.9, 0.99, 0.01, 0.1)
    xd, md = x0.copy(), m0.copy()
    _, counts = orc.step(xd, md, g, oracle.VOTE, 0.9, 0.99, 0.01, 0.1)
    assert np.array_equal(mg, md)
    unanimous = (counts == 0) | (counts == N)
    assert unanimous.sum() > 10
    assert np.array_equal(xg[unanimous].view(np.uint32), xd[unanimous].view(np.uint32))
    # the sign bits against a float64 mean of separately computed blends
    c = (F32(0.9) * m0 + (F32(1) - F32(0.9)) * g).astype(np.float64).mean(axis=0)
    got = np.unpackbits(bits.view(np.uint8), bitorder="little")[:d].astype(bool)
    safe = np.abs(c) > 1e-5
    assert np.array_equal(got[safe], c[safe] > 0)


def test_global_lion():
    check_global_lion(oracle.default())


NEXT_CHECKS = (check_down_link, check_per_worker_betas, check_global_lion)
