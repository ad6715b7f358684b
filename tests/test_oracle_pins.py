"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle.

Each check lives in a function taking the oracle object, so that the same
checks can be run against deliberately broken copies of the oracle
(see test_oracle_mutants.py) to show that a plausible mistake fails a pin.
"""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

F32 = np.float32


def bf16_bits(a):
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16); test-side helper."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------- P1
def lion_single_worker(x, m, g, beta1, beta2, lr, lam):
    """Standard Lion, Eq. (1), written on its own with numpy fp32 arrays (one rounding per op)."""
    b1, b2 = F32(beta1), F32(beta2)
    c = b1 * m + (F32(1) - b1) * g
    delta = np.where(c < 0, F32(-1), F32(1)).astype(F32)
    m_new = b2 * m + (F32(1) - b2) * g
    x_new = x - F32(lr) * (delta + F32(lam) * x)
    return x_new.astype(F32), m_new.astype(F32), delta


def check_n1_is_lion(orc, steps=120, d=777):
    rng = np.random.default_rng(101)
    for mode, use_bf16 in itertools.product((oracle.VOTE, oracle.AVG), (False, True)):
        x = rng.normal(0, 0.02, d).astype(F32)
        m = np.zeros((1, d), F32)
        xr, mr = x.copy(), m[0].copy()
        for _ in range(steps):
            g = (rng.standard_t(3, d) * 1e-3).astype(F32)
            if use_bf16:
                gb = bf16_bits(g)
                g_in, g_ref = gb[None, :], bf16_to_f32(gb)
            else:
                g_in, g_ref = g[None, :], g
            packed, counts = orc.step(x, m, np.ascontiguousarray(g_in), mode, 0.9, 0.99, 3e-4, 0.1)
            xr, mr, delta = lion_single_worker(xr, mr, g_ref, 0.9, 0.99, 3e-4, 0.1)
            assert np.array_equal(x.view(np.uint32), xr.view(np.uint32))
            assert np.array_equal(m[0].view(np.uint32), mr.view(np.uint32))
            assert np.array_equal(counts, (delta > 0).astype(np.uint16))


def test_p1_single_worker_is_standard_lion():
    check_n1_is_lion(oracle.default())


# ----------------------------------------------------------------------------- P2
def load_hand(golden_dir=None):
    here = golden_dir or os.path.join(os.path.dirname(__file__), "golden")
    with open(os.path.join(here, "hand_worked.json")) as f:
        return json.load(f)


def check_hand_worked(orc):
    h = load_hand()
    b1, b2, lr, lam = h["beta1"], h["beta2"], h["lr"], h["lambda"]
    for key in ("N3", "N4"):
        case = h[key]
        names = case["workers"]
        N = len(names)
        g = np.array([h["grads"][w] for w in names], F32)
        # majority vote
        x = np.array(h["x0"], F32)
        m = np.zeros((N, 4), F32)
        packed, counts = orc.step(x, m, g, oracle.VOTE, b1, b2, lr, lam)
        assert packed[:, 0].tolist() == [h["words"][w] for w in names]
        assert counts.tolist() == case["counts"]
        assert (2 * counts.astype(int) - N).tolist() == case["S"]
        assert x.tolist() == case["vote"]["x1"]
        assert m.tolist() == [h["m1"][w] for w in names]
        # the Delta itself
        x_chk = np.array(h["x0"], F32)
        Delta = orc.apply(x_chk, counts, N, oracle.VOTE, lr, lam, want_delta=True)
        assert Delta.tolist() == case["vote"]["Delta"]
        if "second_step_zero_grads" in case["vote"]:
            s2 = case["vote"]["second_step_zero_grads"]
            m_before = m.copy()
            packed2, _ = orc.step(x, m, np.zeros_like(g), oracle.VOTE, b1, b2, lr, lam)
            assert packed2[:, 0].tolist() == [s2["words"][w] for w in names]
            assert x.tolist() == s2["x2"]
            assert np.array_equal(m, F32(s2["m2_scale"]) * m_before)
        # averaging
        x = np.array(h["x0"], F32)
        m = np.zeros((N, 4), F32)
        orc.step(x, m, g, oracle.AVG, b1, b2, lr, lam)
        if "x1" in case["avg"]:
            assert x.tolist() == case["avg"]["x1"]
            x_chk = np.array(h["x0"], F32)
            Delta = orc.apply(x_chk, counts, N, oracle.AVG, lr, lam, want_delta=True)
            assert Delta.tolist() == case["avg"]["Delta"]
        else:
            want = [Fraction(a, b) for a, b in case["avg"]["x1_rational"]]
            for got, w in zip(x.tolist(), want):
                # three roundings (divide, add, multiply/subtract) of values below 2
                assert abs(Fraction(got) - w) <= 4 * Fraction(1, 2 ** 24) * 2
            x_chk = np.array(h["x0"], F32)
            Delta = orc.apply(x_chk, counts, N, oracle.AVG, lr, lam, want_delta=True)
            for got, (a, b) in zip(Delta.tolist(), case["avg"]["Delta_rational"]):
                assert abs(Fraction(got) - Fraction(a, b)) <= Fraction(1, 2 ** 25)


def test_p2_hand_worked_vectors():
    check_hand_worked(oracle.default())


# ----------------------------------------------------------------------------- P3
def check_closed_forms(orc):
    lr, lam = 1e-2, 0.5
    T = 200
    # (i) zero gradients, zero momentum: c = 0 everywhere, every worker votes +1, Delta = +1 in
    # both modes, so x_t = (1 - lr*lam)^t (x_0 + 1/lam) - 1/lam; momentum stays 0; words all ones.
    for mode, N, d in ((oracle.VOTE, 4, 130), (oracle.AVG, 3, 130), (oracle.AVG, 8, 67)):
        rng = np.random.default_rng(7)
        x0 = rng.normal(0, 1.0, d).astype(F32)
        x = x0.copy()
        m = np.zeros((N, d), F32)
        g = np.zeros((N, d), F32)
        for t in range(1, T + 1):
            packed, counts = orc.step(x, m, g, mode, 0.9, 0.99, lr, lam)
            assert np.all(counts == N)
            W = packed.shape[1]
            full = np.uint64(0xFFFFFFFFFFFFFFFF)
            assert np.all(packed[:, : W - 1] == full)
            tail = d - 64 * (W - 1)
            assert np.all(packed[:, W - 1] == (full if tail == 64 else np.uint64((1 << tail) - 1)))
            assert not m.any()
            closed = (1 - float(F32(lr)) * float(F32(lam))) ** t * (x0.astype(np.float64) + 1 / lam) - 1 / lam
            bound = 4 * t * 2.0 ** -24 * max(np.abs(x0).max(), 1 / lam)
            assert np.max(np.abs(x.astype(np.float64) - closed)) <= bound
    # (ii) pure weight decay: two workers with opposite gradients tie, the vote is 0,
    # x_t = (1 - lr*lam)^t x_0; with averaging the mean of (+1, -1) is 0 too.
    for mode in (oracle.VOTE, oracle.AVG):
        rng = np.random.default_rng(8)
        d = 200
        x0 = rng.normal(0, 1.0, d).astype(F32)
        v = (np.abs(rng.normal(0, 1.0, d)) + 0.1).astype(F32)
        x = x0.copy()
        m = np.zeros((2, d), F32)
        for t in range(1, T + 1):
            g = np.stack([v, -v])
            _, counts = orc.step(x, m, g, mode, 0.9, 0.99, lr, lam)
            assert np.all(counts == 1)
            closed = (1 - float(F32(lr)) * float(F32(lam))) ** t * x0.astype(np.float64)
            bound = 4 * t * 2.0 ** -24 * np.abs(x0).max()
            assert np.max(np.abs(x.astype(np.float64) - closed)) <= bound
        # momentum: m_t = (1 - beta2^t) v exactly in real arithmetic
        b2 = float(F32(0.99))
        want = (1 - b2 ** T) * v.astype(np.float64)
        assert np.allclose(m[0], want, rtol=1e-4) and np.allclose(m[1], -want, rtol=1e-4)


def test_p3_closed_forms():
    check_closed_forms(oracle.default())


# ----------------------------------------------------------------------------- P4
def check_invariants(orc):
    rng = np.random.default_rng(11)
    lr, lam = 0.05, 0.5          # box F = [-2, 2]; x0 spread well outside it
    for N in (1, 2, 3, 4, 7, 8):
        d = 64 * 3 + 17
        x_v = (rng.normal(0, 4.0, d)).astype(F32)
        x_a = x_v.copy()
        m = rng.normal(0, 1, (N, d)).astype(F32)
        for t in range(30):
            g = rng.normal(0, 1, (N, d)).astype(F32)
            m_v, m_a = m.copy(), m.copy()
            xv_prev, xa_prev = x_v.copy(), x_a.copy()
            # worker permutation must not change anything the server produces
            perm = rng.permutation(N)
            x_p, m_p = x_v.copy(), m[perm].copy()
            packed, counts = orc.step(x_v, m_v, g, oracle.VOTE, 0.9, 0.99, lr, lam)
            _, counts_a = orc.step(x_a, m_a, g, oracle.AVG, 0.9, 0.99, lr, lam)
            packed_p, counts_p = orc.step(x_p, m_p, g[perm].copy(), oracle.VOTE, 0.9, 0.99, lr, lam)
            assert np.array_equal(counts, counts_p) and np.array_equal(x_v.view(np.uint32), x_p.view(np.uint32))
            assert np.array_equal(packed[perm], packed_p) and np.array_equal(m_v[perm], m_p)
            assert np.array_equal(counts, counts_a) and np.array_equal(m_v, m_a)
            # ranges
            assert counts.max() <= N
            W = packed.shape[1]
            assert np.all(packed[:, W - 1] >> np.uint64(d - 64 * (W - 1)) == 0)
            assert int(sum(bin(int(w)).count("1") for w in packed.ravel())) == int(counts.sum())
            Dv = orc.apply(xv_prev.copy(), counts, N, oracle.VOTE, lr, lam, want_delta=True)
            Da = orc.apply(xa_prev.copy(), counts, N, oracle.AVG, lr, lam, want_delta=True)
            assert set(np.unique(Dv).tolist()) <= {-1.0, 0.0, 1.0}
            ties = Dv == 0
            assert np.all(2 * counts[ties].astype(int) == N) and (N % 2 == 0 or not ties.any())
            assert np.array_equal(np.sign(Da), Dv)
            assert np.all(np.abs(Da) <= 1)
            # Phase I (Theorem 4.1): distance to F = {|lam x| <= 1} contracts by (1 - lr*lam)
            # per step in every coordinate, and a point inside F stays inside.
            for prev, cur in ((xv_prev, x_v), (xa_prev, x_a)):
                dist_prev = np.maximum(np.abs(prev.astype(np.float64)) - 1 / lam, 0)
                dist_cur = np.maximum(np.abs(cur.astype(np.float64)) - 1 / lam, 0)
                slack = 4 * 2.0 ** -24 * np.maximum(np.abs(prev), 1)
                assert np.all(dist_cur <= (1 - lr * lam) * dist_prev + slack)
            m = m_v


def test_p4_invariants():
    check_invariants(oracle.default())


# ----------------------------------------------------------------------------- P5
def check_brute_force(orc):
    lr, lam = 0.125, 0.25
    for N in (1, 2, 3, 4, 5):
        for extra in (0, 61, 64, 67):
            d = 2 ** N + extra
            k = np.arange(d) % (2 ** N)
            # worker i votes +1 on coordinate j iff bit i of (j mod 2^N) is set
            signs = np.array([[1 if (kk >> i) & 1 else -1 for kk in k] for i in range(N)], np.int64)
            g = signs.astype(F32)
            for mode in (oracle.VOTE, oracle.AVG):
                x0 = (((np.arange(d) % 17) - 8) / 8).astype(F32)      # few-bit dyadic values
                x = x0.copy()
                m = np.zeros((N, d), F32)
                packed, counts = orc.step(x, m, g, mode, 0.5, 0.5, lr, lam)
                pop = np.array([bin(int(kk)).count("1") for kk in k])
                assert np.array_equal(counts, pop)
                S = signs.sum(axis=0)               # direct integer sum of the +-1 votes
                for j in range(d):
                    for i in range(N):
                        bit = (int(packed[i, j // 64]) >> (j % 64)) & 1
                        assert bit == (1 if signs[i, j] > 0 else 0)
                    if mode == oracle.VOTE:
                        Delta = Fraction(int(np.sign(S[j])))
                    else:
                        Delta = Fraction(int(S[j]), N)
                    want = Fraction(float(x0[j])) - Fraction(lr) * (Delta + Fraction(lam) * Fraction(float(x0[j])))
                    assert abs(Fraction(float(x[j])) - want) <= Fraction(1, 2 ** 22)
                    if mode == oracle.VOTE or N in (1, 2, 4):
                        # all quantities dyadic with few bits: the fp32 result is exact
                        assert Fraction(float(x[j])) == want


def test_p5_brute_force_all_sign_patterns():
    check_brute_force(oracle.default())


# ----------------------------------------------------------------------------- P6
def check_packing_cross(orc):
    rng = np.random.default_rng(13)
    for N, d in ((1, 1), (3, 63), (4, 64), (5, 65), (9, 1000), (16, 64 * 5 + 3)):
        m = rng.normal(0, 1, (N, d)).astype(F32)
        g = rng.normal(0, 1, (N, d)).astype(F32)
        # exact zeros and negative zeros must vote +1
        g[:, ::7] = 0
        m[:, ::7] = 0
        if d > 14:
            g[0, 14] = -0.0
        m_in = m.copy()
        packed, delta = orc.worker_step(m, g, 0.9, 0.99, want_delta=True)
        assert np.all(delta[:, ::7] == 1)
        c_packed = orc.aggregate_packed(packed, d)
        c_signs = orc.aggregate_signs(delta)
        assert np.array_equal(c_packed, c_signs)
        assert np.array_equal(c_signs, (delta > 0).sum(axis=0))
        # packing against numpy's own bit packer (little-endian bit order)
        bits = (delta > 0).astype(np.uint8)
        pad = (-d) % 64
        bits = np.pad(bits, ((0, 0), (0, pad)))
        ref = np.packbits(bits, axis=1, bitorder="little").view("<u8")
        assert np.array_equal(packed, ref)
        # momentum moved toward g, old momentum was used for the sign
        c = F32(0.9) * m_in + (F32(1) - F32(0.9)) * g
        assert np.array_equal(delta > 0, ~(c < 0))


def test_p6_packing_cross_check():
    check_packing_cross(oracle.default())


# ----------------------------------------------------------------------------- misc
def check_no_fma(orc):
    """Cases where a fused multiply-add would flip the vote: both products round, the sum is 0."""
    # beta1*m rounds to exactly -(1-beta1)*g after individual rounding; with an FMA the
    # unrounded product leaves a tiny negative residue.
    b1 = F32(0.9)
    omb1 = F32(1) - b1
    found = 0
    rng = np.random.default_rng(5)
    for _ in range(20000):
        g = F32(rng.normal())
        b = omb1 * g
        m_try = F32(-b / b1)
        for mm in (m_try, np.nextafter(m_try, F32(10)), np.nextafter(m_try, F32(-10))):
            a = b1 * mm
            if F32(a + b) == 0 and (float(b1) * float(mm) + float(b)) < 0:
                m = np.array([[mm]], F32)
                packed = orc.worker_step(m, np.array([[g]], F32), 0.9, 0.99)
                assert int(packed[0, 0]) == 1    # fp32-rounded sum is 0 -> +1; an FMA would say -1
                found += 1
    assert found > 10


def test_sign_decided_in_fp32_without_fma():
    check_no_fma(oracle.default())


ALL_CHECKS = (check_hand_worked, check_brute_force, check_packing_cross, check_closed_forms,
              check_invariants, check_no_fma, check_n1_is_lion)


def test_threads_and_strides_do_not_change_results():
    rng = np.random.default_rng(17)
    orc = oracle.default()
    N, d = 5, 64 * 37 + 11
    x0 = rng.normal(0, 0.02, d).astype(F32)
    m0 = rng.normal(0, 1e-3, (N, d)).astype(F32)
    g = bf16_bits(rng.normal(0, 1e-3, (N, d)))
    ref = None
    for threads in (1, 2, 3, 8, 64):
        x = x0.copy()
        big = np.zeros((N, d + 29), F32)
        m = big[:, :d]
        m[...] = m0
        packed, counts = orc.step(x, m, g, oracle.AVG, 0.9, 0.99, 3e-4, 0.1, threads=threads)
        assert not big[:, d:].any()
        cur = (x.copy(), m.copy(), packed, counts)
        if ref is None:
            ref = cur
        else:
            for a, b in zip(ref, cur):
                assert np.array_equal(a, b)


def test_multi_tensor_is_per_tensor_flat():
    rng = np.random.default_rng(19)
    orc = oracle.default()
    N = 3
    sizes = [64, 1000, 5, 128]
    xs = [rng.normal(0, 0.02, n).astype(F32) for n in sizes]
    ms = [rng.normal(0, 1e-3, (N, n)).astype(F32) for n in sizes]
    gs = [rng.normal(0, 1e-3, (N, n)).astype(F32) for n in sizes]
    xs2 = [a.copy() for a in xs]
    ms2 = [a.copy() for a in ms]
    packed, counts = orc.step_mt(xs, ms, gs, oracle.VOTE, 0.9, 0.99, 1e-4, 10.0)
    assert packed.shape == (N, sum((n + 63) // 64 for n in sizes))
    assert counts.shape == (sum(sizes),)
    off_w = 0
    off = 0
    for k, n in enumerate(sizes):
        pk, ck = orc.step(xs2[k], ms2[k], gs[k], oracle.VOTE, 0.9, 0.99, 1e-4, 10.0)
        W = (n + 63) // 64
        assert np.array_equal(packed[:, off_w:off_w + W], pk)
        assert np.array_equal(counts[off:off + n], ck)
        assert np.array_equal(xs[k], xs2[k])
        off_w += W
        off += n
