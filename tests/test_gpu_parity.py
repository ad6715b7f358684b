"""GPU parity: the HIP path against the CPU oracle, element by element, through the C ABI.

Packed words and vote counts must be bit-exact; fp32 momentum and weights must
agree within max relative error 1e-6 (they are expected to be bit-identical,
which is reported but the stated bar is what is asserted).
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_2404_00438_amd as dl
from paper_2404_00438_amd import workloads as wl
from helpers import assert_f32_equal, strided_rows, to_np

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
HYP = dict(beta1=0.9, beta2=0.99, lr=3e-4, lam=0.1)


def announce(*what):
    print("[case]", *what, flush=True)


def draw_state(rng, N, d, g_dtype, m_stride=None, g_stride=None, scale=1e-3):
    """Random x, m, g on the device, rows optionally padded to a given stride."""
    m_stride = d if m_stride is None else m_stride
    g_stride = d if g_stride is None else g_stride
    x = torch.from_numpy(rng.normal(0, 0.02, d).astype(np.float32)).to(DEV)
    m = strided_rows(N, d, m_stride, torch.float32, DEV)
    m.copy_(torch.from_numpy(rng.normal(0, scale, (N, d)).astype(np.float32)))
    g = strided_rows(N, d, g_stride, g_dtype, DEV)
    g.copy_(torch.from_numpy(rng.standard_t(3, (N, d)).astype(np.float32) * scale).to(g_dtype))
    return x, m, g


def oracle_step(x, m, g, mode, hyp):
    xn, mn, gn = to_np(x), to_np(m), to_np(g)
    packed, counts = oracle.step(xn, mn, gn, mode, hyp["beta1"], hyp["beta2"], hyp["lr"], hyp["lam"])
    return xn, mn, packed, counts


def compare_all(tag, x, m, packed, counts, xn, mn, pn, cn):
    if packed is not None:
        assert np.array_equal(to_np(packed), pn), f"{tag}: packed words differ"
    if counts is not None:
        assert np.array_equal(to_np(counts)[: cn.shape[0]], cn), f"{tag}: counts differ"
    assert_f32_equal(to_np(m), mn, f"{tag}: m")
    assert_f32_equal(to_np(x), xn, f"{tag}: x")


SIZES = [1, 63, 64, 65, 255, 256, 257, 1000, 4096 + 3, 70_001]
WORKERS = [1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 33]


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("mode", [dl.VOTE, dl.AVG], ids=["vote", "avg"])
def test_fused_step_matches_oracle(g_dtype, mode):
    rng = np.random.default_rng(1234)
    for d, N in itertools.product(SIZES, WORKERS):
        if d > 5000 and N not in (4, 8, 17):
            continue
        for aligned in (True, False):
            # aligned rows: stride rounded up to 64 elements; unaligned: odd stride (dword path)
            stride = ((d + 63) // 64) * 64 if aligned else d + (1 if d % 2 == 0 else 2)
            announce("fused", g_dtype, mode, "d", d, "N", N, "stride", stride)
            x, m, g = draw_state(rng, N, d, g_dtype, stride, stride)
            W = dl.words_for(d)
            packed = strided_rows(N, W, W + 3, torch.int64, DEV)
            counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            for step in range(3):
                xn, mn, pn, cn = oracle_step(x, m, g, mode, HYP)
                dl.dlion_step(x, m, g, mode, HYP["beta1"], HYP["beta2"], HYP["lr"], HYP["lam"],
                              packed=packed, counts=counts)
                torch.cuda.synchronize()
                compare_all(f"d={d} N={N} step={step}", x, m, packed, counts, xn, mn, pn, cn)
            # padding of strided buffers untouched
            assert torch.isnan(m._base[:, d:]).all() if stride > d else True
            assert (packed._base[:, W:] == -1).all()


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_output_flags_do_not_change_state(g_dtype):
    """The bench configuration (no packed, no counts) gives the same x, m as the instrumented one."""
    rng = np.random.default_rng(99)
    for d, N, mode in ((70_001, 8, dl.AVG), (4096, 5, dl.VOTE), (300, 2, dl.AVG)):
        announce("flags", g_dtype, d, N, mode)
        stride = ((d + 63) // 64) * 64
        x0, m0, g = draw_state(rng, N, d, g_dtype, stride, stride)
        xn, mn, pn, cn = oracle_step(x0, m0, g, mode, HYP)
        for want_p, want_c in itertools.product((False, True), repeat=2):
            x, m = x0.clone(), m0.clone()
            packed = torch.zeros((N, dl.words_for(d)), dtype=torch.int64, device=DEV) if want_p else None
            counts = torch.zeros(d, dtype=torch.int16, device=DEV) if want_c else None
            dl.dlion_step(x, m, g, mode, HYP["beta1"], HYP["beta2"], HYP["lr"], HYP["lam"],
                          packed=packed, counts=counts)
            torch.cuda.synchronize()
            compare_all(f"flags p={want_p} c={want_c}", x, m, packed, counts, xn, mn, pn, cn)


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_unfused_pipeline_matches_oracle(g_dtype):
    """worker_step -> aggregate -> apply, and worker_step -> aggregate_apply."""
    rng = np.random.default_rng(4321)
    for (d, N), mode in itertools.product(((1, 1), (65, 3), (256, 4), (1000, 8), (70_001, 5), (8192, 16),
                                           (5000, 300)), (dl.VOTE, dl.AVG)):
        for aligned in (True, False):
            stride = ((d + 63) // 64) * 64 if aligned else d + (1 if d % 2 == 0 else 2)
            announce("unfused", g_dtype, d, N, mode, stride)
            x, m, g = draw_state(rng, N, d, g_dtype, stride, stride)
            x2 = x.clone()
            W = dl.words_for(d)
            xn, mn, pn, cn = oracle_step(x, m, g, mode, HYP)
            packed = torch.full((N, W), -1, dtype=torch.int64, device=DEV)
            counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_worker_step(m, g, packed, HYP["beta1"], HYP["beta2"])
            dl.dlion_aggregate(packed, d, counts)
            dl.dlion_apply(x, counts, N, mode, HYP["lr"], HYP["lam"])
            counts2 = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_aggregate_apply(x2, packed, mode, HYP["lr"], HYP["lam"], counts=counts2)
            x3 = x2.clone()
            torch.cuda.synchronize()
            compare_all("unfused", x, m, packed, counts, xn, mn, pn, cn)
            compare_all("aggregate_apply", x2, m, packed, counts2, xn, mn, pn, cn)
            # and without the optional counts output (applied a second time, on x3 = x after 1 step)
            xn2 = xn.copy()
            oracle.apply(xn2, cn, N, mode, HYP["lr"], HYP["lam"])
            dl.dlion_aggregate_apply(x3, packed, mode, HYP["lr"], HYP["lam"])
            torch.cuda.synchronize()
            assert_f32_equal(to_np(x3), xn2, "aggregate_apply (no counts): x")


def test_special_values():
    """Zeros, negative zeros, subnormals, infinities and NaNs: sign(0)=+1, subnormals kept."""
    N, d = 4, 512
    tiny = np.float32(1e-45)             # smallest subnormal
    vals = np.array([0.0, -0.0, tiny, -tiny, 1e-39, -1e-39, 1.1754944e-38, -1.1754944e-38, 1.0, -1.0,
                     np.inf, -np.inf, np.nan, 3.4e38, -3.4e38, 1e-30], dtype=np.float32)
    rng = np.random.default_rng(5)
    for g_dtype in (torch.float32, torch.bfloat16):
        for mode in (dl.VOTE, dl.AVG):
            announce("special", g_dtype, mode)
            mv = rng.choice(vals, size=(N, d)).astype(np.float32)
            gv = rng.choice(vals, size=(N, d)).astype(np.float32)
            xv = rng.choice(vals, size=d).astype(np.float32)
            x = torch.from_numpy(xv).to(DEV)
            m = torch.from_numpy(mv).to(DEV)
            g = torch.from_numpy(gv).to(DEV).to(g_dtype)
            packed = torch.zeros((N, dl.words_for(d)), dtype=torch.int64, device=DEV)
            counts = torch.zeros(d, dtype=torch.int16, device=DEV)
            xn, mn, pn, cn = oracle_step(x, m, g, mode, dict(beta1=0.9, beta2=0.99, lr=0.5, lam=0.5))
            dl.dlion_step(x, m, g, mode, 0.9, 0.99, 0.5, 0.5, packed=packed, counts=counts)
            torch.cuda.synchronize()
            compare_all("special", x, m, packed, counts, xn, mn, pn, cn)
            # subnormal momentum must survive: 0.99 * 1e-39 is subnormal and must not flush to 0
            sub = (np.abs(mn) > 0) & (np.abs(mn) < 1.1754944e-38)
            assert sub.any()
            assert np.array_equal(to_np(m)[sub].view(np.uint32), mn[sub].view(np.uint32))


def test_average_division_every_count():
    """Averaging must be one correctly rounded fp32 division for every N, every count p."""
    for N in (1, 2, 3, 5, 6, 7, 9, 10, 11, 13, 24, 31, 33, 100, 255, 256, 257, 1000, 4097, 65535):
        announce("avg division N", N)
        d = N + 1
        counts_np = np.arange(d, dtype=np.uint16)
        xv = np.linspace(-1, 1, d).astype(np.float32)
        x = torch.from_numpy(xv.copy()).to(DEV)
        counts = torch.from_numpy(counts_np.view(np.int16).copy()).to(DEV)
        for mode in (dl.VOTE, dl.AVG):
            xn = to_np(x)
            oracle.apply(xn, counts_np, N, mode, 0.25, 0.5)
            dl.dlion_apply(x, counts, N, mode, 0.25, 0.5)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(x).view(np.uint32), xn.view(np.uint32)), f"N={N} mode={mode}"


def test_sign_without_fma_on_device():
    """Pairs (m, g) where the individually rounded sum is exactly 0 but a fused multiply-add
    would give a negative number: the device must vote +1 like the oracle."""
    b1 = np.float32(0.9)
    omb1 = np.float32(1) - b1
    rng = np.random.default_rng(5)
    ms, gs = [], []
    while len(ms) < 4096:
        g = np.float32(rng.normal())
        b = omb1 * g
        mm = np.float32(-b / b1)
        for cand in (mm, np.nextafter(mm, np.float32(10)), np.nextafter(mm, np.float32(-10))):
            if np.float32(b1 * cand + b) == 0 and (float(b1) * float(cand) + float(b)) != 0:
                ms.append(cand)
                gs.append(g)
    d = len(ms)
    m = torch.tensor(np.array(ms, np.float32)[None, :]).to(DEV)
    g = torch.tensor(np.array(gs, np.float32)[None, :]).to(DEV)
    mn, gn = to_np(m), to_np(g)
    want = oracle.worker_step(mn, gn, 0.9, 0.99)
    packed = torch.zeros((1, dl.words_for(d)), dtype=torch.int64, device=DEV)
    dl.dlion_worker_step(m, g, packed, 0.9, 0.99)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(packed), want)
    assert (want == np.uint64(0xFFFFFFFFFFFFFFFF)).all()


def make_list(rng, numels, N, g_dtype):
    xs = [torch.from_numpy(rng.normal(0, 0.02, n).astype(np.float32)).to(DEV) for n in numels]
    ms = [torch.from_numpy(rng.normal(0, 1e-3, (N, n)).astype(np.float32)).to(DEV) for n in numels]
    gs = [torch.from_numpy(rng.normal(0, 1e-3, (N, n)).astype(np.float32)).to(DEV).to(g_dtype) for n in numels]
    return xs, ms, gs


def unpad_counts(counts, table):
    c = to_np(counts)
    return np.concatenate([c[64 * wb: 64 * wb + n] for wb, n in zip(table.word_begin, table.numels)])


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("mode", [dl.VOTE, dl.AVG], ids=["vote", "avg"])
def test_tensor_list_matches_oracle(g_dtype, mode):
    rng = np.random.default_rng(777)
    numels = [1000, 5, 64, 256, 768, 257, 1, 2304 * 8, 4097, 63]
    hyp = dict(beta1=0.9, beta2=0.99, lr=1e-4, lam=10.0)
    for N in (1, 4, 16, 5, 130):              # 130: beyond the few-worker kernel, the per-nibble one takes the list
        announce("tensor list", g_dtype, mode, "N", N)
        xs, ms, gs = make_list(rng, numels, N, g_dtype)
        table = dl.SegTable(xs, ms, gs)
        Wt = table.total_words
        assert Wt == sum((n + 63) // 64 for n in numels)
        packed = torch.full((N, Wt), -1, dtype=torch.int64, device=DEV)
        counts = torch.full((64 * Wt,), -1, dtype=torch.int16, device=DEV)
        for step in range(2):
            xn = [to_np(t) for t in xs]
            mn = [to_np(t) for t in ms]
            gn = [to_np(t) for t in gs]
            pn, cn = oracle.step_mt(xn, mn, gn, mode, hyp["beta1"], hyp["beta2"], hyp["lr"], hyp["lam"])
            # unfused on copies first
            xs_u = [t.clone() for t in xs]
            ms_u = [t.clone() for t in ms]
            tab_u = dl.SegTable(xs_u, ms_u, gs)
            packed_u = torch.full((N, Wt), -1, dtype=torch.int64, device=DEV)
            counts_u = torch.full((64 * Wt,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_worker_step_mt(tab_u, packed_u, hyp["beta1"], hyp["beta2"])
            dl.dlion_aggregate_mt(tab_u, packed_u, counts_u)
            dl.dlion_apply_mt(tab_u, counts_u, N, mode, hyp["lr"], hyp["lam"])
            xs_a = [t.clone() for t in xs]
            tab_a = dl.SegTable(xs_a, None, None)
            dl.dlion_aggregate_apply_mt(tab_a, packed_u, mode, hyp["lr"], hyp["lam"])
            xs_b = [t.clone() for t in xs]
            counts_b = torch.full((64 * Wt,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_aggregate_apply_mt(dl.SegTable(xs_b, None, None), packed_u, mode, hyp["lr"], hyp["lam"], counts=counts_b)
            # fused in place
            dl.dlion_step_mt(table, N, mode, hyp["beta1"], hyp["beta2"], hyp["lr"], hyp["lam"],
                             packed=packed, counts=counts)
            torch.cuda.synchronize()
            for tag, P, C, X, M in (("fused", packed, counts, xs, ms), ("unfused", packed_u, counts_u, xs_u, ms_u)):
                assert np.array_equal(to_np(P), pn), f"{tag}: packed"
                assert np.array_equal(unpad_counts(C, table), cn), f"{tag}: counts"
                # padding between tensors is written as 0
                cfull = to_np(C)
                for wb, n in zip(table.word_begin, table.numels):
                    assert not cfull[64 * wb + n: 64 * (wb + (n + 63) // 64)].any()
                for k in range(len(numels)):
                    assert_f32_equal(to_np(X[k]), xn[k], f"{tag}: x[{k}]")
                    assert_f32_equal(to_np(M[k]), mn[k], f"{tag}: m[{k}]")
            for k in range(len(numels)):
                assert_f32_equal(to_np(xs_a[k]), xn[k], f"aggregate_apply_mt: x[{k}]")
                assert_f32_equal(to_np(xs_b[k]), xn[k], f"aggregate_apply_mt with counts: x[{k}]")
            assert np.array_equal(to_np(counts_b), to_np(counts_u)), "aggregate_apply_mt: counts (padding included)"


def test_tiny_config_full_run():
    """Config 'tiny' exactly as stated: d = 1,000,003, N = 4, vote, fp32 N(0,1) gradients, 10 steps."""
    w = wl.CONFIGS["tiny"]
    x = wl.init_x(w, DEV)
    for stride in (w.d, ((w.d + 63) // 64) * 64):
        announce("tiny", "stride", stride)
        x = wl.init_x(w, DEV)
        m = wl.init_m(w, DEV, row_stride=stride)
        xn, mn = to_np(x), to_np(m)
        packed = torch.zeros((w.N, dl.words_for(w.d)), dtype=torch.int64, device=DEV)
        counts = torch.zeros(w.d, dtype=torch.int16, device=DEV)
        exact = True
        for t in range(w.steps):
            g = wl.make_grads(w, t, DEV)
            pn, cn = oracle.step(xn, mn, to_np(g), w.mode, w.beta1, w.beta2, w.lr, w.lam, threads=8)
            dl.dlion_step(x, m, g, w.mode, w.beta1, w.beta2, w.lr, w.lam, packed=packed, counts=counts)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(packed), pn), f"step {t}: packed"
            assert np.array_equal(to_np(counts), cn), f"step {t}: counts"
            exact &= assert_f32_equal(to_np(m), mn, f"step {t}: m")
            exact &= assert_f32_equal(to_np(x), xn, f"step {t}: x")
        # last word: only 3 valid bits
        assert (to_np(packed)[:, -1] >> np.uint64(3) == 0).all()
        print("tiny: bit-identical fp32 state:", exact, flush=True)


@pytest.mark.parametrize("waves", [1, 8, 16])
def test_many_worker_aggregate_matches_oracle(waves, tune):
    """The bit-sliced server-side kernel: counts bit-exact, apply within the bar.  The library would give
    the smaller N to the few-worker kernel and pick the workgroup size from N and d, so the bit-sliced
    kernel and each of its workgroup sizes are forced."""
    tune(sliced_min_workers=1, sliced_waves=waves, group_max_workers=0)
    rng = np.random.default_rng(2024)
    cases = [(1, 300), (2, 8192), (3, 8193), (7, 70_001), (8, 129), (15, 5000),
             (16, 4096), (17, 4097), (31, 1), (32, 63), (33, 10_000), (64, 8192 + 5), (127, 4095),
             (128, 70_001), (255, 5000), (256, 12_345), (257, 4096 * 3), (511, 300), (512, 4096),
             (1000, 9000), (4095, 700), (4096, 130), (5000, 4100), (65535, 130)]
    for N, d in cases:
        W = dl.words_for(d)
        for p_one, pad in ((0.5, 0), (0.9, 3), (1.0, 1)):
            announce("sliced", "N", N, "d", d, "p", p_one, "row pad", pad)
            if p_one == 1.0:
                words = np.full((N, W), np.uint64(0xFFFFFFFFFFFFFFFF))
            else:
                bits = rng.random((N, W * 64)) < p_one
                words = np.packbits(bits, axis=1, bitorder="little").view("<u8")
            tail = d - 64 * (W - 1)
            if tail < 64:
                words[:, W - 1] &= np.uint64((1 << tail) - 1)
            packed = strided_rows(N, W, W + pad, torch.int64, DEV)
            packed.copy_(torch.from_numpy(words.view(np.int64)))
            want = oracle.aggregate_packed(np.ascontiguousarray(words), d)
            counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_aggregate(packed, d, counts)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(counts), want), f"N={N} d={d}: counts"
            for mode in (dl.VOTE, dl.AVG):
                xv = rng.normal(0, 0.02, d).astype(np.float32)
                # odd offset into a larger buffer: x not 16-byte aligned on every other case
                off = 1 if (N + d) % 2 else 0
                xbuf = torch.zeros(d + 1, dtype=torch.float32, device=DEV)
                x = xbuf[off:off + d]
                x.copy_(torch.from_numpy(xv))
                xn = xv.copy()
                oracle.apply(xn, want, N, mode, 0.25, 0.5)
                counts2 = torch.full((d,), -1, dtype=torch.int16, device=DEV)
                dl.dlion_aggregate_apply(x, packed, mode, 0.25, 0.5, counts=counts2 if mode == dl.AVG else None)
                torch.cuda.synchronize()
                assert_f32_equal(to_np(x), xn, f"N={N} d={d} mode={mode}: x")
                if mode == dl.AVG:
                    assert np.array_equal(to_np(counts2), want)


def test_few_worker_kernel_matches_oracle(tune):
    """Server side for few workers (eight waves share 8192 coordinates): counts, planes and x against
    the oracle for every N the kernel takes a different path for (1 to 4 planes per wave, odd and even,
    waves with no row or with a partly empty batch of rows), on sizes with whole spans, a ragged last span,
    a ragged last line of 1024 coordinates and a ragged last word."""
    tune(group_max_workers=120)
    rng = np.random.default_rng(31337)
    sizes = [1, 63, 1024, 1025, 8192, 8192 + 64, 3 * 8192 + 1000, 70_001]
    workers = [1, 2, 3, 4, 7, 8, 9, 15, 16, 17, 24, 25, 31, 32, 33, 48, 56, 57, 63, 64, 65, 100, 119, 120]
    for N in workers:
        for d in sizes if N in (1, 2, 16, 31, 32, 64, 120) else (8192 + 64, 70_001):
            W = dl.words_for(d)
            for p_one in (0.5, 1.0):
                announce("few workers", "N", N, "d", d, "p", p_one)
                if p_one == 1.0:
                    words = np.full((N, W), np.uint64(0xFFFFFFFFFFFFFFFF))
                else:
                    words = np.packbits(rng.random((N, W * 64)) < p_one, axis=1, bitorder="little").view("<u8")
                    if N % 2 == 0:                       # exact ties on every coordinate of the first words
                        words[N // 2:, : (W + 1) // 2] = ~words[: N // 2, : (W + 1) // 2]
                tail = d - 64 * (W - 1)
                if tail < 64:
                    words[:, W - 1] &= np.uint64((1 << tail) - 1)
                packed = strided_rows(N, W, W + (N + d) % 3, torch.int64, DEV)
                packed.copy_(torch.from_numpy(words.view(np.int64)))
                want = oracle.aggregate_packed(np.ascontiguousarray(words), d)
                counts = torch.full((d + 5,), -1, dtype=torch.int16, device=DEV)
                dl.dlion_aggregate(packed, d, counts[:d])
                torch.cuda.synchronize()
                assert np.array_equal(to_np(counts[:d]), want), f"N={N} d={d}: counts"
                assert (counts[d:] == -1).all()
                for mode in (dl.VOTE, dl.AVG):
                    P = dl.dlion_delta_planes(N, mode)
                    delta = strided_rows(P, W, W + 1, torch.int64, DEV)
                    dl.dlion_aggregate_encode(packed, d, mode, delta)
                    torch.cuda.synchronize()
                    assert np.array_equal(to_np(delta), oracle.encode_delta(want, N, mode)), f"N={N} d={d} mode={mode}: planes"
                    assert (delta._base[:, W:] == -1).all()
                    xv = rng.normal(0, 0.02, d).astype(np.float32)
                    xn = xv.copy()
                    oracle.apply(xn, want, N, mode, 0.25, 0.5)
                    for with_counts in (False, True):
                        off = (N + d) % 2                # x not 16-byte aligned on every other case
                        xbuf = torch.full((d + 2,), 7.0, dtype=torch.float32, device=DEV)
                        x = xbuf[off:off + d]
                        x.copy_(torch.from_numpy(xv))
                        counts2 = torch.full((d + 5,), -1, dtype=torch.int16, device=DEV)
                        dl.dlion_aggregate_apply(x, packed, mode, 0.25, 0.5, counts=counts2[:d] if with_counts else None)
                        torch.cuda.synchronize()
                        assert_f32_equal(to_np(x), xn, f"N={N} d={d} mode={mode} counts={with_counts}: x")
                        assert (xbuf[off + d:] == 7.0).all()
                        if with_counts:
                            assert np.array_equal(to_np(counts2[:d]), want)
                            assert (counts2[d:] == -1).all()


def test_server_side_kernel_choice_at_its_boundaries():
    """The library's own choice between the few-worker, bit-sliced and per-nibble kernels (no override), on
    both sides of every N at which it changes: counts, planes and x against the oracle."""
    rng = np.random.default_rng(4242)
    for N in (8, 9, 11, 12, 24, 25, 56, 57, 64, 65, 100, 101, 120, 121):
        for d in (9000, 70_001):
            announce("kernel choice", "N", N, "d", d)
            W = dl.words_for(d)
            bits = rng.random((N, W * 64)) < 0.5
            bits[:, d:] = False
            words = np.packbits(bits, axis=1, bitorder="little").view("<u8")
            want = oracle.aggregate_packed(np.ascontiguousarray(words), d)
            packed = strided_rows(N, W, W + 2, torch.int64, DEV)
            packed.copy_(torch.from_numpy(words.view(np.int64)))
            counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_aggregate(packed, d, counts)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(counts), want), f"N={N} d={d}: counts"
            for mode in (dl.VOTE, dl.AVG):
                xv = rng.normal(0, 0.02, d).astype(np.float32)
                xn = xv.copy()
                oracle.apply(xn, want, N, mode, 0.25, 0.5)
                x = torch.from_numpy(xv).to(DEV)
                dl.dlion_aggregate_apply(x, packed, mode, 0.25, 0.5)
                delta = torch.full((dl.dlion_delta_planes(N, mode), W), -1, dtype=torch.int64, device=DEV)
                dl.dlion_aggregate_encode(packed, d, mode, delta)
                torch.cuda.synchronize()
                assert_f32_equal(to_np(x), xn, f"N={N} d={d} mode={mode}: x")
                assert np.array_equal(to_np(delta), oracle.encode_delta(want, N, mode)), f"N={N} d={d} mode={mode}: planes"


def offset_view(shape, dtype, skip):
    """Tensor of the given shape that starts `skip` elements into its allocation (allocations are
    256-byte aligned, so skip = 1 leaves only the element's own alignment)."""
    n = int(np.prod(shape))
    buf = torch.empty(n + skip + 1, dtype=dtype, device=DEV)
    if dtype in (torch.float32, torch.bfloat16):
        buf.fill_(float("nan"))
    else:
        buf.fill_(-1)
    return buf, buf[skip:skip + n].view(*shape)


@pytest.mark.parametrize("g_dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_arrays_with_only_their_element_alignment(g_dtype):
    """Every array starts one element past an aligned address and rows follow each other without
    padding: full tiles still take the 128-bit accesses, so those must work at any alignment."""
    rng = np.random.default_rng(808)
    for (d, N), mode in itertools.product(((256, 1), (1027, 3), (4099, 8), (70_001, 5), (8193, 20)),
                                          (dl.VOTE, dl.AVG)):
        announce("element-aligned", g_dtype, "d", d, "N", N, "mode", mode)
        W = dl.words_for(d)
        xb, x = offset_view((d,), torch.float32, 1)
        mb, m = offset_view((N, d), torch.float32, 1)
        gb, g = offset_view((N, d), g_dtype, 1)
        pb, packed = offset_view((N, W), torch.int64, 1)
        cb, counts = offset_view((d,), torch.int16, 1)
        x.copy_(torch.from_numpy(rng.normal(0, 0.02, d).astype(np.float32)))
        m.copy_(torch.from_numpy(rng.normal(0, 1e-3, (N, d)).astype(np.float32)))
        g.copy_(torch.from_numpy(rng.standard_t(3, (N, d)).astype(np.float32) * 1e-3).to(g_dtype))
        assert x.data_ptr() % 16 == 4 and m.data_ptr() % 16 == 4 and counts.data_ptr() % 8 == 2
        for step in range(2):
            xn, mn, pn, cn = oracle_step(x, m, g, mode, HYP)
            dl.dlion_step(x, m, g, mode, HYP["beta1"], HYP["beta2"], HYP["lr"], HYP["lam"],
                          packed=packed, counts=counts)
            torch.cuda.synchronize()
            compare_all(f"fused d={d} N={N} step={step}", x, m, packed, counts, xn, mn, pn, cn)
        # the same through the separate calls
        x2 = x.clone()
        xn, mn, pn, cn = oracle_step(x, m, g, mode, HYP)
        packed.fill_(-1)
        counts.fill_(-1)
        dl.dlion_worker_step(m, g, packed, HYP["beta1"], HYP["beta2"])
        dl.dlion_aggregate(packed, d, counts)
        dl.dlion_apply(x, counts, N, mode, HYP["lr"], HYP["lam"])
        torch.cuda.synchronize()
        compare_all(f"unfused d={d} N={N}", x, m, packed, counts, xn, mn, pn, cn)
        x2b, x2o = offset_view((d,), torch.float32, 3)
        x2o.copy_(x2)
        dl.dlion_aggregate_apply(x2o, packed, mode, HYP["lr"], HYP["lam"])
        torch.cuda.synchronize()
        assert_f32_equal(to_np(x2o), xn, "aggregate_apply: x")
        # nothing outside the views was written
        for buf, view in ((xb, x), (mb, m), (x2b, x2o)):
            assert torch.isnan(buf[0]) and torch.isnan(buf[-1])
        assert pb[0] == -1 and pb[-1] == -1 and cb[0] == -1 and cb[-1] == -1
        # averaging over all workers' blends (same layout)
        xn, mn = to_np(x), to_np(m)
        bn = oracle.global_lion_step(xn, mn, to_np(g), 0.9, 0.99, 3e-4, 0.1)
        bits = torch.full((W,), -1, dtype=torch.int64, device=DEV)
        dl.dlion_global_lion_step(x, m, g, 0.9, 0.99, 3e-4, 0.1, sign_bits=bits)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(bits), bn)
        assert_f32_equal(to_np(m), mn, "global lion: m")
        assert_f32_equal(to_np(x), xn, "global lion: x")


@pytest.mark.parametrize("per,tiles", [(1, 0), (3, 3), (8, 5)])
def test_step_split_into_launches_over_few_workers(per, tiles, tune):
    """Many workers at large d run as several launches over a few workers each, the votes carried in
    the counts array, block of tiles by block of tiles; forced here at small sizes (`per` workers per
    launch, `tiles` tiles per block, 0 = one block).  Same bits and state as one launch."""
    tune(pass_workers=per, block_tiles=tiles)
    rng = np.random.default_rng(4242 + per)
    for (d, N), mode, g_dtype in itertools.product(((1000, 4), (4099, 9), (257, 17), (70_001, 33), (700, 70)),
                                                   (dl.VOTE, dl.AVG), (torch.float32, torch.bfloat16)):
        announce("launches of", per, "workers:", g_dtype, "d", d, "N", N, "mode", mode)
        stride = d + 3
        x, m, g = draw_state(rng, N, d, g_dtype, stride, stride)
        W = dl.words_for(d)
        packed = strided_rows(N, W, W + 1, torch.int64, DEV)
        counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
        for step in range(2):
            xn, mn, pn, cn = oracle_step(x, m, g, mode, HYP)
            m_w = m.clone()
            packed_w = torch.full((N, W), -1, dtype=torch.int64, device=DEV)
            dl.dlion_worker_step(m_w, g, packed_w, HYP["beta1"], HYP["beta2"])
            dl.dlion_step(x, m, g, mode, HYP["beta1"], HYP["beta2"], HYP["lr"], HYP["lam"],
                          packed=packed if step else None, counts=counts)
            torch.cuda.synchronize()
            compare_all(f"fused d={d} N={N} step={step}", x, m, packed if step else None, counts, xn, mn, pn, cn)
            assert np.array_equal(to_np(packed_w), pn), "worker step: packed"
            assert_f32_equal(to_np(m_w), mn, "worker step: m")
        # per-worker coefficients: launches that begin inside a block of 64 workers
        b1 = rng.choice(np.array([0.0, 0.5, 0.9, 0.95], np.float32), N)
        b2 = rng.choice(np.array([0.25, 0.9, 0.99], np.float32), N)
        xn, mn, gn = to_np(x), to_np(m), to_np(g)
        pn = oracle.worker_step_pw(mn, gn, b1, b2)
        cn = oracle.aggregate_packed(pn, d)
        oracle.apply(xn, cn, N, mode, 3e-4, 0.1)
        dl.dlion_step_pw(x, m, g, mode, torch.from_numpy(b1).to(DEV), torch.from_numpy(b2).to(DEV), 3e-4, 0.1,
                         packed=packed, counts=counts)
        torch.cuda.synchronize()
        compare_all(f"step_pw d={d} N={N}", x, m, packed, counts, xn, mn, pn, cn)
    # tensor list
    numels = [1000, 5, 64, 256, 257, 1, 2304 * 8, 63]
    for N, mode in ((5, dl.VOTE), (18, dl.AVG)):
        announce("launches of", per, "workers: tensor list N", N)
        xs, ms, gs = make_list(rng, numels, N, torch.bfloat16)
        table = dl.SegTable(xs, ms, gs)
        Wt = table.total_words
        packed = torch.full((N, Wt), -1, dtype=torch.int64, device=DEV)
        counts = torch.full((64 * Wt,), -1, dtype=torch.int16, device=DEV)
        xn = [to_np(t) for t in xs]
        mn = [to_np(t) for t in ms]
        pn, cn = oracle.step_mt(xn, mn, [to_np(t) for t in gs], mode, 0.9, 0.99, 1e-4, 10.0)
        dl.dlion_step_mt(table, N, mode, 0.9, 0.99, 1e-4, 10.0, packed=packed, counts=counts)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(packed), pn) and np.array_equal(unpad_counts(counts, table), cn)
        for k in range(len(numels)):
            assert_f32_equal(to_np(xs[k]), xn[k], f"x[{k}]")
            assert_f32_equal(to_np(ms[k]), mn[k], f"m[{k}]")


def test_per_nibble_server_kernel_on_flat_buffers(tune):
    """Flat buffers take the bit-sliced server kernel at every N; the per-nibble one (which tensor
    lists use for the fused aggregate + update) is forced here so that its flat form stays checked."""
    tune(sliced_min_workers=100000)
    rng = np.random.default_rng(515)
    for N, d in ((1, 1), (2, 63), (3, 257), (8, 4096 + 3), (9, 70_001), (33, 1000), (300, 5000)):
        W = dl.words_for(d)
        bits = rng.random((N, W * 64)) < 0.6
        bits[:, d:] = False
        words = np.packbits(bits, axis=1, bitorder="little").view("<u8")
        want = oracle.aggregate_packed(np.ascontiguousarray(words), d)
        packed = strided_rows(N, W, W + 1, torch.int64, DEV)
        packed.copy_(torch.from_numpy(words.view(np.int64)))
        for mode in (dl.VOTE, dl.AVG):
            announce("per-nibble forced", "N", N, "d", d, "mode", mode)
            counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_aggregate(packed, d, counts)
            xv = rng.normal(0, 0.02, d).astype(np.float32)
            x = torch.from_numpy(xv).to(DEV)
            xn = xv.copy()
            oracle.apply(xn, want, N, mode, 0.25, 0.5)
            counts2 = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_aggregate_apply(x, packed, mode, 0.25, 0.5, counts=counts2)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(counts), want) and np.array_equal(to_np(counts2), want)
            assert_f32_equal(to_np(x), xn, f"N={N} d={d} mode={mode}: x")


@pytest.mark.parametrize("per,tiles", [(3, 3), (8, 0), (15, 2), (20, 0)])
def test_step_with_votes_carried_in_a_workspace(per, tiles, tune):
    """dlion_step_ws / dlion_step_pw_ws / dlion_step_mt_ws: the launches over a few workers hand the votes on through the
    caller's workspace, block of tiles by block of tiles (forced at small sizes).  Up to 8 launches of at
    most 15 workers use planes of 4-bit partial counts, anything beyond a running uint16 count: the
    cases cover both, with and without a counts output."""
    tune(pass_workers=per, block_tiles=tiles)
    rng = np.random.default_rng(99 + per)
    workspace = torch.full((4 << 20,), 0x5A, dtype=torch.uint8, device=DEV)
    small = torch.zeros(64, dtype=torch.uint8, device=DEV)                         # holds no block: not used
    for (d, N), mode, g_dtype in itertools.product(((1000, 4), (4099, 9), (70_001, 33), (700, 70)),
                                                   (dl.VOTE, dl.AVG), (torch.float32, torch.bfloat16)):
        announce("workspace carry", per, tiles, g_dtype, "d", d, "N", N, "mode", mode)
        x, m, g = draw_state(rng, N, d, g_dtype, d + 3, d + 3)
        W = dl.words_for(d)
        packed = strided_rows(N, W, W + 1, torch.int64, DEV)
        counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
        for step, (ws, want_packed, want_counts) in enumerate(((workspace, False, False), (workspace, True, False),
                                                               (workspace, True, True), (small, False, False),
                                                               (None, True, False))):
            xn, mn, pn, cn = oracle_step(x, m, g, mode, HYP)
            workspace.fill_(0x5A if step % 2 else 0xFF)             # scratch: whatever it held must not matter
            dl.dlion_step_ws(x, m, g, mode, HYP["beta1"], HYP["beta2"], HYP["lr"], HYP["lam"], ws,
                             packed=packed if want_packed else None, counts=counts if want_counts else None)
            torch.cuda.synchronize()
            compare_all(f"d={d} N={N} step={step}", x, m, packed if want_packed else None,
                        counts if want_counts else None, xn, mn, pn, cn)
        # each worker's own coefficients, same hand-over (dlion_step_pw_ws)
        b1 = rng.choice(np.array([0.0, 0.5, 0.9, 0.95], np.float32), N)
        b2 = rng.choice(np.array([0.25, 0.9, 0.99], np.float32), N)
        xn, mn, gn = to_np(x), to_np(m), to_np(g)
        pn = oracle.worker_step_pw(mn, gn, b1, b2)
        cn = oracle.aggregate_packed(pn, d)
        oracle.apply(xn, cn, N, mode, 3e-4, 0.1)
        dl.dlion_step_pw(x, m, g, mode, torch.from_numpy(b1).to(DEV), torch.from_numpy(b2).to(DEV), 3e-4, 0.1,
                         packed=packed, counts=counts, workspace=workspace)
        torch.cuda.synchronize()
        compare_all(f"step_pw_ws d={d} N={N}", x, m, packed, counts, xn, mn, pn, cn)
    # tensor list, ragged tensors included
    numels = [1000, 5, 64, 256, 257, 1, 2304 * 8, 63]
    for N, mode in ((5, dl.VOTE), (18, dl.AVG), (70, dl.VOTE)):
        announce("workspace carry: tensor list N", N)
        xs, ms, gs = make_list(rng, numels, N, torch.bfloat16)
        table = dl.SegTable(xs, ms, gs)
        Wt = table.total_words
        packed = torch.full((N, Wt), -1, dtype=torch.int64, device=DEV)
        counts = torch.full((64 * Wt,), -1, dtype=torch.int16, device=DEV)
        xn = [to_np(t) for t in xs]
        mn = [to_np(t) for t in ms]
        for step, (want_packed, want_counts) in enumerate(((False, False), (True, True))):
            pn, cn = oracle.step_mt(xn, mn, [to_np(t) for t in gs], mode, 0.9, 0.99, 1e-4, 10.0)
            dl.dlion_step_mt(table, N, mode, 0.9, 0.99, 1e-4, 10.0, packed=packed if want_packed else None,
                             counts=counts if want_counts else None, workspace=workspace)
            torch.cuda.synchronize()
            if want_packed:
                assert np.array_equal(to_np(packed), pn) and np.array_equal(unpad_counts(counts, table), cn)
            for k in range(len(numels)):
                assert_f32_equal(to_np(xs[k]), xn[k], f"x[{k}] step {step}")
                assert_f32_equal(to_np(ms[k]), mn[k], f"m[{k}] step {step}")


def test_workspace_sizes():
    assert dl.dlion_step_workspace_bytes(1000, 4) == 0 and dl.dlion_step_workspace_bytes(350_000_000, 8) == 0
    # 4 launches over 8 workers: 3 planes of one uint16 per lane and tile, 262144 tiles at a time
    assert dl.dlion_step_workspace_bytes(350_000_000, 32) == 262144 * 3 * 128
    assert dl.dlion_step_workspace_bytes(20_000_000, 16) == 78125 * 1 * 128
    # 16 launches: a running count, four uint16 per lane
    assert dl.dlion_step_workspace_bytes(350_000_000, 128) == 262144 * 512
    assert dl.dlion_step_mt_workspace_bytes(78125, 16) == dl.dlion_step_workspace_bytes(20_000_000, 16)


@pytest.mark.parametrize("kernel", ["bit-sliced", "per-nibble", "few-worker"])
def test_server_side_calls_cut_into_several_launches(kernel, tune):
    """Large problems run the server-side and update kernels as several launches over blocks of
    coordinates; forced here at small sizes (8 tiles per launch; a bit-sliced workgroup is at least 32)."""
    sliced = kernel == "bit-sliced"
    tune(block_tiles=8, sliced_min_workers=1 if sliced else 100000, sliced_waves=8 if sliced else -1,
         group_max_workers=120 if kernel == "few-worker" else 0)
    rng = np.random.default_rng(616)
    for N, d in ((3, 5000), (8, 70_001), (33, 20_000), (300, 9000)):
        W = dl.words_for(d)
        bits = rng.random((N, W * 64)) < 0.55
        bits[:, d:] = False
        words = np.packbits(bits, axis=1, bitorder="little").view("<u8")
        want = oracle.aggregate_packed(np.ascontiguousarray(words), d)
        packed = strided_rows(N, W, W + 1, torch.int64, DEV)
        packed.copy_(torch.from_numpy(words.view(np.int64)))
        counts = torch.full((d,), -1, dtype=torch.int16, device=DEV)
        dl.dlion_aggregate(packed, d, counts)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(counts), want), f"N={N} d={d}: counts"
        for mode in (dl.VOTE, dl.AVG):
            announce("several launches", kernel, "N", N, "d", d, "mode", mode)
            xv = rng.normal(0, 0.02, d).astype(np.float32)
            xn = xv.copy()
            oracle.apply(xn, want, N, mode, 0.25, 0.5)
            x1, x2, x3 = (torch.from_numpy(xv).to(DEV) for _ in range(3))
            counts2 = torch.full((d,), -1, dtype=torch.int16, device=DEV)
            dl.dlion_apply(x1, counts, N, mode, 0.25, 0.5)
            dl.dlion_aggregate_apply(x2, packed, mode, 0.25, 0.5, counts=counts2)
            P = dl.dlion_delta_planes(N, mode)
            delta = torch.full((P, W), -1, dtype=torch.int64, device=DEV)
            dl.dlion_aggregate_encode(packed, d, mode, delta)
            dl.dlion_apply_encoded(x3, delta, N, mode, 0.25, 0.5)
            torch.cuda.synchronize()
            assert np.array_equal(to_np(counts2), want)
            assert np.array_equal(to_np(delta), oracle.encode_delta(want, N, mode))
            for tag, x in (("apply", x1), ("aggregate_apply", x2), ("apply_encoded", x3)):
                assert_f32_equal(to_np(x), xn, f"{tag} N={N} d={d} mode={mode}: x")


def test_randomized_shapes_strides_and_flags():
    """Seeded random sweep over d, N, row strides (aligned or not), gradient dtype, aggregation and
    optional outputs, two steps each, fused and unfused, against the oracle."""
    rng = np.random.default_rng(20240400)
    for case in range(120):
        N = int(rng.choice([1, 2, 3, 4, 6, 8, 11, 16, 24, 40]))
        d = int(rng.choice([rng.integers(1, 300), rng.integers(300, 5000), rng.integers(5000, 40_000)]))
        g_dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
        mode = dl.AVG if rng.random() < 0.5 else dl.VOTE
        m_stride = d + int(rng.choice([0, 1, 2, 3, 4, 64 - d % 64, 257]))
        g_stride = d + int(rng.choice([0, 1, 2, 4, 8, 64 - d % 64, 100]))
        want_p, want_c = bool(rng.random() < 0.6), bool(rng.random() < 0.6)
        hyp = dict(beta1=float(rng.choice([0.0, 0.5, 0.9, 0.95])), beta2=float(rng.choice([0.9, 0.99, 0.999])),
                   lr=float(rng.choice([1e-5, 3e-4, 1e-2])), lam=float(rng.choice([0.0, 0.1, 10.0])))
        announce("random", case, "N", N, "d", d, g_dtype, "mode", mode, "strides", m_stride, g_stride,
                 "p", want_p, "c", want_c, hyp)
        x, m, g = draw_state(rng, N, d, g_dtype, m_stride, g_stride, scale=float(rng.choice([1e-3, 1.0])))
        W = dl.words_for(d)
        for step in range(2):
            xn, mn, pn, cn = oracle_step(x, m, g, mode, hyp)
            # unfused on copies
            x_u, m_u = x.clone(), m.clone()
            packed_u = torch.full((N, W), -1, dtype=torch.int64, device=DEV)
            dl.dlion_worker_step(m_u, g, packed_u, hyp["beta1"], hyp["beta2"])
            dl.dlion_aggregate_apply(x_u, packed_u, mode, hyp["lr"], hyp["lam"])
            # fused in place
            packed = torch.full((N, W), -1, dtype=torch.int64, device=DEV) if want_p else None
            counts = torch.full((d,), -1, dtype=torch.int16, device=DEV) if want_c else None
            dl.dlion_step(x, m, g, mode, hyp["beta1"], hyp["beta2"], hyp["lr"], hyp["lam"],
                          packed=packed, counts=counts)
            torch.cuda.synchronize()
            compare_all(f"random {case} fused", x, m, packed, counts, xn, mn, pn, cn)
            compare_all(f"random {case} unfused", x_u, m_u, packed_u, None, xn, mn, pn, cn)
            g.copy_(torch.from_numpy(rng.standard_t(3, (N, d)).astype(np.float32) * 1e-3).to(g_dtype))


def test_calls_follow_the_given_stream():
    """Work is enqueued on the stream that is passed (torch's current stream in the binding):
    a step issued on a side stream after an event sees the data written before that event."""
    rng = np.random.default_rng(8)
    N, d = 4, 300_003
    x, m, g = draw_state(rng, N, d, torch.float32, d + 1, d + 3)
    xn, mn, pn, cn = oracle_step(x, m, g, dl.VOTE, HYP)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    packed = torch.zeros((N, dl.words_for(d)), dtype=torch.int64, device=DEV)
    counts = torch.zeros(d, dtype=torch.int16, device=DEV)
    with torch.cuda.stream(side):
        packed.zero_()
        dl.dlion_step(x, m, g, dl.VOTE, HYP["beta1"], HYP["beta2"], HYP["lr"], HYP["lam"],
                      packed=packed, counts=counts)
        done = torch.cuda.Event()
        done.record()
    done.synchronize()
    compare_all("side stream", x, m, packed, counts, xn, mn, pn, cn)


def test_step_can_be_captured_in_a_graph(tune):
    """The calls allocate nothing and never synchronise, so a step (here split into several launches)
    can be captured once and replayed; every replay is checked, with eager work in between."""
    tune(pass_workers=3)
    rng = np.random.default_rng(31)
    N, d = 7, 70_001
    x, m, g = draw_state(rng, N, d, torch.bfloat16, d + 3, d + 5)
    packed = torch.zeros((N, dl.words_for(d)), dtype=torch.int64, device=DEV)
    counts = torch.zeros(d, dtype=torch.int16, device=DEV)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        dl.dlion_step(x, m, g, dl.AVG, HYP["beta1"], HYP["beta2"], HYP["lr"], HYP["lam"],
                      packed=packed, counts=counts)
    for replay in range(3):
        announce("graph replay", replay)
        xn, mn, pn, cn = oracle_step(x, m, g, dl.AVG, HYP)
        graph.replay()
        torch.cuda.synchronize()
        compare_all(f"replay {replay}", x, m, packed, counts, xn, mn, pn, cn)
        # eager work between the replays: new gradients in the same buffer
        g.copy_(torch.from_numpy(rng.standard_t(3, (N, d)).astype(np.float32) * 1e-3).to(torch.bfloat16))
        packed.fill_(-1)
        counts.fill_(-1)
        torch.cuda.synchronize()
