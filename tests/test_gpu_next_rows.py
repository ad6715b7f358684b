"""GPU parity for the rows around the hot path: down-link bit-planes, per-worker coefficients
(and sign-momentum), Global Lion -- each against the CPU oracle through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_00438_amd as dl
from helpers import assert_f32_equal, strided_rows, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def announce(*what):
    print("[case]", *what, flush=True)


def random_words(rng, N, d, p_one):
    W = dl.words_for(d)
    bits = rng.random((N, W * 64)) < p_one
    bits[:, d:] = False
    return np.packbits(bits, axis=1, bitorder="little").view("<u8")


@pytest.mark.parametrize("waves", [1, 8, 16])
def test_down_link_planes_match_oracle(waves, tune):
    tune(sliced_waves=waves, group_max_workers=0)              # the bit-sliced encoder, its workgroup size forced
    rng = np.random.default_rng(77)
    cases = [(1, 1), (2, 63), (3, 64), (4, 65), (5, 4096), (7, 8191), (8, 8193), (9, 300), (16, 10_000),
             (31, 5000), (32, 4097), (33, 129), (64, 20_000), (100, 9000), (255, 1000), (256, 70_001),
             (257, 4096), (1000, 3000), (4096, 200), (65535, 130)]
    for N, d in cases:
        W = dl.words_for(d)
        for p_one in (0.5, 0.1):
            words = random_words(rng, N, d, p_one)
            if N % 2 == 0:                       # force some exact ties
                words[N // 2:, :] = ~words[: N // 2, :]
                tail = d - 64 * (W - 1)
                if tail < 64:
                    words[:, W - 1] &= np.uint64((1 << tail) - 1)
            counts = oracle.aggregate_packed(np.ascontiguousarray(words), d)
            packed = strided_rows(N, W, W + (N % 3), torch.int64, DEV)
            packed.copy_(torch.from_numpy(words.view(np.int64)))
            for mode in (dl.VOTE, dl.AVG):
                announce("down-link", "N", N, "d", d, "p", p_one, "mode", mode)
                P = dl.dlion_delta_planes(N, mode)
                assert P == oracle.delta_planes(N, mode)
                want = oracle.encode_delta(counts, N, mode)
                delta = strided_rows(P, W, W + 1, torch.int64, DEV)
                dl.dlion_aggregate_encode(packed, d, mode, delta)
                torch.cuda.synchronize()
                assert np.array_equal(to_np(delta), want), f"N={N} d={d} mode={mode}: planes"
                assert (delta._base[:, W:] == -1).all()
                xv = rng.normal(0, 0.02, d).astype(np.float32)
                off = (N + d) % 2                # x not 16-byte aligned on every other case
                xbuf = torch.zeros(d + 1, dtype=torch.float32, device=DEV)
                x = xbuf[off:off + d]
                x.copy_(torch.from_numpy(xv))
                xn = xv.copy()
                oracle.apply_encoded(xn, want, N, mode, 0.25, 0.5)
                dl.dlion_apply_encoded(x, delta, N, mode, 0.25, 0.5)
                torch.cuda.synchronize()
                assert_f32_equal(to_np(x), xn, f"N={N} d={d} mode={mode}: x")
                # and the message is equivalent to applying the counts directly
                xc = xv.copy()
                oracle.apply(xc, counts, N, mode, 0.25, 0.5)
                assert np.array_equal(xc.view(np.uint32), xn.view(np.uint32))


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_per_worker_coefficients_match_oracle(g_dtype):
    rng = np.random.default_rng(78)
    # N past 64 and 128: the vector path fetches the coefficients 64 workers at a time
    for N, d in ((1, 100), (2, 257), (5, 4096 + 3), (8, 70_001), (33, 1000), (64, 300), (65, 513), (130, 700)):
        for kind in ("mixed", "signum"):
            b1 = rng.choice(np.array([0.0, 0.5, 0.8, 0.9, 0.95, 1.0], np.float32), N)
            b2 = rng.choice(np.array([0.25, 0.9, 0.98, 0.99, 0.999], np.float32), N) if kind == "mixed" else b1.copy()
            for mode in (dl.VOTE, dl.AVG):
                announce("per-worker", g_dtype, "N", N, "d", d, kind, "mode", mode)
                stride = ((d + 63) // 64) * 64
                x = torch.from_numpy(rng.normal(0, 0.02, d).astype(np.float32)).to(DEV)
                m = strided_rows(N, d, stride, torch.float32, DEV)
                m.copy_(torch.from_numpy(rng.normal(0, 1e-3, (N, d)).astype(np.float32)))
                g = strided_rows(N, d, stride, g_dtype, DEV)
                g.copy_(torch.from_numpy(rng.normal(0, 1e-3, (N, d)).astype(np.float32)).to(g_dtype))
                t1, t2 = torch.from_numpy(b1).to(DEV), torch.from_numpy(b2).to(DEV)
                W = dl.words_for(d)
                for step in range(2):
                    xn, mn, gn = to_np(x), to_np(m), to_np(g)
                    pn = oracle.worker_step_pw(mn, gn, b1, b2)
                    cn = oracle.aggregate_packed(pn, d)
                    oracle.apply(xn, cn, N, mode, 3e-4, 0.1)
                    # unfused worker step on a copy, fused step in place
                    m_u = m.clone()
                    packed_u = torch.zeros((N, W), dtype=torch.int64, device=DEV)
                    dl.dlion_worker_step_pw(m_u, g, packed_u, t1, t2)
                    packed = torch.zeros((N, W), dtype=torch.int64, device=DEV)
                    counts = torch.zeros(d, dtype=torch.int16, device=DEV)
                    dl.dlion_step_pw(x, m, g, mode, t1, t2, 3e-4, 0.1, packed=packed, counts=counts)
                    torch.cuda.synchronize()
                    assert np.array_equal(to_np(packed_u), pn) and np.array_equal(to_np(packed), pn)
                    assert np.array_equal(to_np(counts), cn)
                    assert_f32_equal(to_np(m_u), mn, "worker_step_pw: m")
                    assert_f32_equal(to_np(m), mn, "step_pw: m")
                    assert_f32_equal(to_np(x), xn, "step_pw: x")
                if kind == "signum":
                    bits = np.unpackbits(to_np(packed).view(np.uint8), axis=1, bitorder="little")[:, :d]
                    assert np.array_equal(bits.astype(bool), ~(to_np(m) < 0))


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_global_lion_matches_oracle(g_dtype):
    rng = np.random.default_rng(79)
    for N, d in ((1, 1), (1, 1000), (2, 255), (3, 256), (4, 257), (7, 4096 + 3), (8, 70_001), (16, 5000),
                 (33, 3000)):
        for aligned in (True, False):
            stride = ((d + 63) // 64) * 64 if aligned else d + (1 if d % 2 == 0 else 2)
            announce("global lion", g_dtype, "N", N, "d", d, "stride", stride)
            x = torch.from_numpy(rng.normal(0, 0.02, d).astype(np.float32)).to(DEV)
            m = strided_rows(N, d, stride, torch.float32, DEV)
            m.copy_(torch.from_numpy(rng.normal(0, 1e-3, (N, d)).astype(np.float32)))
            g = strided_rows(N, d, stride, g_dtype, DEV)
            gv = rng.normal(0, 1e-3, (N, d)).astype(np.float32)
            if N > 1:
                gv[1, ::5] = -gv[0, ::5]         # exact cancellations: mean 0 must vote +1
                gv[2:, ::5] = 0
            g.copy_(torch.from_numpy(gv).to(g_dtype))
            if N > 1:
                m[:, ::5] = 0
            bits = torch.full((dl.words_for(d),), -1, dtype=torch.int64, device=DEV)
            for step in range(3):
                xn, mn = to_np(x), to_np(m)
                bn = oracle.global_lion_step(xn, mn, to_np(g), 0.9, 0.99, 3e-4, 0.1)
                dl.dlion_global_lion_step(x, m, g, 0.9, 0.99, 3e-4, 0.1, sign_bits=bits if step else None)
                torch.cuda.synchronize()
                if step:
                    assert np.array_equal(to_np(bits), bn), f"N={N} d={d}: sign bits"
                assert_f32_equal(to_np(m), mn, "global lion: m")
                assert_f32_equal(to_np(x), xn, "global lion: x")
