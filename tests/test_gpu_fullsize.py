"""GPU parity at the full sizes of the stated workloads, in the launch configuration bench.py times.

The CPU oracle cannot run 10^9..10^10 updates per step in seconds, but every
coordinate is independent of every other (apart from sharing a 64-bit packed
word with its neighbours), so the oracle is run on SAMPLED word-aligned chunks
of the full problem -- always including the first words and the ragged end --
fed with the very same initial state and gradients the GPU sees, step after
step.  Whole-array properties that hold at any size complete the check.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2404_00438_amd as dl
from paper_2404_00438_amd import workloads as wl
from helpers import assert_f32_equal, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CHUNK = 2048            # coordinates per sampled chunk (32 packed words)


def announce(*what):
    print("[case]", *what, flush=True)


BLOCK_COORDS = (262144 * 256, 524288 * 256)   # coordinates per launch: split steps, whole steps


def sample_chunks(d: int, n_chunks: int, seed: int, edges=()):
    """Word-aligned, disjoint [start, stop) ranges in increasing order: the first chunk, random ones, a
    chunk centred on every coordinate in ``edges`` (launch boundaries, 2^32-byte crossings, ...), the
    last tiles, and the one ending at d (the only one that may be ragged)."""
    rng = np.random.default_rng(seed)
    W = (d + 63) // 64
    words_per_chunk = CHUNK // 64
    starts = {0}
    while len(starts) < n_chunks - 1:
        starts.add(int(rng.integers(0, max(1, W - words_per_chunk))) * 64)
    for e in edges:
        if 0 < e < d:
            starts.add(max(0, (e - CHUNK // 2) // 64 * 64))
    last_start = max(0, (W - words_per_chunk)) * 64
    starts.add(max(0, last_start - 32 * 256))          # the last 32 tiles before the final chunk
    ranges = []
    for s_ in sorted(starts):
        if s_ >= last_start:
            continue
        stop = min(s_ + CHUNK, last_start)
        if ranges and s_ < ranges[-1][1]:              # overlap: extend the previous range
            ranges[-1] = (ranges[-1][0], max(ranges[-1][1], stop))
        else:
            ranges.append((s_, stop))
    return ranges + [(last_start, d)]                  # ragged end goes last


def launch_edges(d: int):
    """Coordinates where one launch of a step ends and the next begins, the first tiles of the last
    (partial) block, and where a row crosses 2^32 bytes (fp32: 2^30 elements, bf16: 2^31)."""
    edges = [1 << 30, 1 << 31]
    for block in BLOCK_COORDS:
        edges += list(range(block, d, block))
        edges.append(d // block * block + CHUNK // 2)
    return edges


def gather(t: torch.Tensor, ranges) -> torch.Tensor:
    """Concatenate the sampled coordinate ranges along the last axis."""
    return torch.cat([t[..., a:b] for a, b in ranges], dim=-1).contiguous()


def gather_words(t: torch.Tensor, ranges) -> torch.Tensor:
    return torch.cat([t[..., a // 64:(b + 63) // 64] for a, b in ranges], dim=-1).contiguous()


def popcount64_total(t: torch.Tensor) -> int:
    """Total number of set bits of an int64 tensor (SWAR, row by row to bound temporaries)."""
    if t.dim() == 2 and not t.is_contiguous():              # padded rows: never flatten (that would copy)
        return sum(popcount64_total(t[i]) for i in range(t.shape[0]))
    total = 0
    flat = t.reshape(-1)
    step = 1 << 26
    for i in range(0, flat.numel(), step):
        v = flat[i:i + step].clone()
        lo = (v & 0xFFFFFFFF)
        hi = (v >> 32) & 0xFFFFFFFF
        for h in (lo, hi):
            h = h - ((h >> 1) & 0x55555555)
            h = (h & 0x33333333) + ((h >> 2) & 0x33333333)
            h = (h + (h >> 4)) & 0x0F0F0F0F
            h = (h * 0x01010101 >> 24) & 0xFF
            total += int(h.sum().item())
    return total


def same_bits(a: torch.Tensor, b: torch.Tensor) -> bool:
    """Whole-array, bit-for-bit comparison on the device (fp32 compared as integers: NaNs included)."""
    if a.dtype == torch.float32:
        return all(torch.equal(a[i].view(torch.int32), b[i].view(torch.int32)) for i in range(a.shape[0])) \
            if a.dim() == 2 else torch.equal(a.view(torch.int32), b.view(torch.int32))
    return torch.equal(a, b)


def run_flat_workload(w: wl.Workload, n_chunks: int = 24, steps=None, padded=True, full_oracle_step=False):
    """All steps of a flat workload exactly as bench.py launches it (padded rows, the workspace form when
    the library would use one), the oracle following on sampled chunks; on the last step the instrumented
    variant (packed words and counts) and, on copies of the state, the unfused pipeline, whose x, m, packed
    words and counts must equal the fused step's over the WHOLE arrays; optionally one step of the oracle
    over the whole arrays on all host threads."""
    steps = w.steps if steps is None else steps
    d, N = w.d, w.N
    announce(w.name, "d", d, "N", N, "mode", w.mode, "steps", steps)
    ranges = sample_chunks(d, n_chunks, seed=d % 9973, edges=launch_edges(d))
    stride = wl.padded_stride(d) if padded else d
    x = wl.init_x(w, DEV)
    m = wl.init_m(w, DEV, row_stride=stride)
    g = torch.empty((N, stride), dtype=w.g_dtype, device=DEV)[:, :d]
    xh, mh = to_np(gather(x, ranges)), to_np(gather(m, ranges))
    W = dl.words_for(d)
    exact = True
    ws_bytes = dl.dlion_step_workspace_bytes(d, N)
    workspace = torch.full((ws_bytes,), 0xA5, dtype=torch.uint8, device=DEV) if ws_bytes else None
    hyp = (w.mode, w.beta1, w.beta2, w.lr, w.lam)
    for t in range(steps):
        wl.make_grads(w, t, DEV, out=g)
        gh = to_np(gather(g, ranges))
        ph, ch = oracle.step(xh, mh, gh, *hyp)
        last = t == steps - 1
        if last:
            # copies for the unfused pipeline and (optionally) the oracle over the whole arrays
            x_u, m_u = x.clone(), m.clone()
            x_a = x.clone()
            # where the library's static scratch is smaller than the workspace it would like, the entry
            # point that allocates nothing runs the same step in smaller blocks of tiles: checked below
            small_scratch = ws_bytes > (64 << 20)
            if small_scratch:
                x_n, m_n = x.clone(), m.clone()
            if full_oracle_step:
                x_full, m_full, g_full = to_np(x), to_np(m), to_np(g)
            # the instrumented variant on the last step: packed words and counts at full size
            packed = torch.empty((N, W), dtype=torch.int64, device=DEV)
            counts = torch.empty(d, dtype=torch.int16, device=DEV)
            dl.dlion_step_ws(x, m, g, *hyp, workspace, packed=packed, counts=counts)
        else:
            # exactly what bench.py launches (a null workspace is dlion_step)
            dl.dlion_step_ws(x, m, g, *hyp, workspace)
        torch.cuda.synchronize()
        exact &= assert_f32_equal(to_np(gather(m, ranges)), mh, f"{w.name} step {t}: m")
        exact &= assert_f32_equal(to_np(gather(x, ranges)), xh, f"{w.name} step {t}: x")
        print(f"  step {t} ok", flush=True)
    assert np.array_equal(to_np(gather_words(packed, ranges)), ph), f"{w.name}: packed words differ"
    assert np.array_equal(to_np(gather(counts, ranges)), ch), f"{w.name}: counts differ"
    if small_scratch:
        dl.dlion_step_noalloc(x_n, m_n, g, *hyp)
        torch.cuda.synchronize()
        assert same_bits(m_n, m) and same_bits(x_n, x), f"{w.name}: dlion_step_noalloc and dlion_step_ws differ somewhere"
        del x_n, m_n
        print("  dlion_step_noalloc (64 MiB of static scratch, smaller blocks) == dlion_step_ws", flush=True)
    # the unfused pipeline (three other kernels) on the copies: whole arrays, bit for bit
    packed_u = torch.empty((N, W), dtype=torch.int64, device=DEV)
    counts_u = torch.empty(d, dtype=torch.int16, device=DEV)
    dl.dlion_worker_step(m_u, g, packed_u, w.beta1, w.beta2)
    dl.dlion_aggregate(packed_u, d, counts_u)
    dl.dlion_apply(x_u, counts_u, N, w.mode, w.lr, w.lam)
    torch.cuda.synchronize()
    assert same_bits(packed_u, packed), f"{w.name}: fused and unfused packed words differ somewhere"
    assert same_bits(counts_u, counts), f"{w.name}: fused and unfused counts differ somewhere"
    assert same_bits(m_u, m), f"{w.name}: fused and unfused momentum differ somewhere"
    assert same_bits(x_u, x), f"{w.name}: fused and unfused weights differ somewhere"
    del counts_u, m_u
    print("  fused step == worker_step + aggregate + apply over the whole arrays", flush=True)
    # ... and the two other ways from the packed words to the weights: the fused aggregate + update (with its
    # counts), and the down-link message applied to the weights
    x_u.copy_(x_a)
    counts_a = torch.empty(d, dtype=torch.int16, device=DEV)
    dl.dlion_aggregate_apply(x_u, packed_u, w.mode, w.lr, w.lam, counts=counts_a)
    torch.cuda.synchronize()
    assert same_bits(counts_a, counts), f"{w.name}: counts of aggregate_apply differ somewhere"
    assert same_bits(x_u, x), f"{w.name}: aggregate_apply and the fused step differ somewhere"
    del counts_a
    delta = torch.empty((dl.dlion_delta_planes(N, w.mode), wl.padded_words(W)), dtype=torch.int64, device=DEV)[:, :W]
    dl.dlion_aggregate_encode(packed_u, d, w.mode, delta)
    dl.dlion_apply_encoded(x_a, delta, N, w.mode, w.lr, w.lam)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(gather_words(delta, ranges)), oracle.encode_delta(ch, N, w.mode)), f"{w.name}: planes"
    assert same_bits(x_a, x), f"{w.name}: the down-link message and the fused step differ somewhere"
    del packed_u, x_u, x_a, delta
    print("  fused step == aggregate_apply == aggregate_encode + apply_encoded over the whole arrays", flush=True)
    if full_oracle_step:
        threads = min(len(os.sched_getaffinity(0)), 16)
        p_full, c_full = oracle.step(x_full, m_full, g_full, *hyp, threads=threads)
        assert np.array_equal(to_np(packed), p_full), f"{w.name}: packed words differ from the whole-array oracle"
        assert np.array_equal(to_np(counts), c_full), f"{w.name}: counts differ from the whole-array oracle"
        exact &= assert_f32_equal(to_np(m), m_full, f"{w.name}: m, whole arrays")
        exact &= assert_f32_equal(to_np(x), x_full, f"{w.name}: x, whole arrays")
        del p_full, c_full, x_full, m_full, g_full
        print(f"  last step equals the oracle over all {d} x {N} updates", flush=True)
    # properties of the whole arrays
    c32 = counts.to(torch.int32) & 0xFFFF
    assert int(c32.max().item()) <= N and int(c32.min().item()) >= 0
    assert popcount64_total(packed) == int(c32.sum(dtype=torch.int64).item())
    tail = d - 64 * (W - 1)
    if tail < 64:
        assert int(((packed[:, W - 1] >> tail) != 0).sum().item()) == 0, "bits past d must be zero"
    assert bool(torch.isfinite(x).all()) and bool(torch.isfinite(m).all())
    print(f"{w.name}: sampled {sum(b - a for a, b in ranges)} coordinates per step in {len(ranges)} ranges, "
          f"fp32 state bit-identical: {exact}", flush=True)
    del packed, counts, g, m, x
    torch.cuda.empty_cache()


def test_gpt2_small_avg8_full_size():
    """d = 124 M flat, N = 8, averaging, bf16 Student-t gradients, 20 steps; the last step also against
    the oracle over the whole arrays."""
    run_flat_workload(wl.CONFIGS["gpt2s_avg8"], full_oracle_step=True)


def test_gpt350m_32_workers_vote_then_avg_full_size():
    """d = 350 M, N = 32, bf16 gradients with outliers: majority vote, then averaging on the same gradients."""
    run_flat_workload(wl.CONFIGS["gpt350m_vote32"])
    run_flat_workload(wl.CONFIGS["gpt350m_avg32"])


def test_stress_1p3b_full_size():
    """d = 1.3 B, N = 8: offsets beyond 2^32 bytes within one stream and 2^33 elements overall."""
    run_flat_workload(wl.CONFIGS["stress1p3b_vote8"])


def test_vit_b16_tensor_list_full_size():
    """ViT-B/16-shaped list of 148 tensors, N = 16, majority vote, fp32 gradients, 10 steps, launched as
    bench.py launches it (workspace form).  The oracle follows on every small tensor in full, on sampled
    chunks of the large ones and on the chunks around every launch boundary; the last step is also
    compared with the oracle over ALL tensors in full and with the unfused calls over the whole arrays."""
    w = wl.CONFIGS["vitb16_vote16"]
    numels = w.numels()
    N = w.N
    announce(w.name, "tensors", len(numels), "d", w.d, "N", N)
    xs = [wl.init_x(w, DEV, tensor=k) for k in range(len(numels))]
    ms = [wl.init_m(w, DEV, numel=n) for n in numels]
    gs = [torch.empty((N, n), dtype=w.g_dtype, device=DEV) for n in numels]
    table = dl.SegTable(xs, ms, gs)
    Wt = table.total_words
    ws_bytes = dl.dlion_step_mt_workspace_bytes(table.total_tiles, N)
    assert ws_bytes > 0
    workspace = torch.full((ws_bytes,), 0xA5, dtype=torch.uint8, device=DEV)
    # every small tensor in full, and sampled chunks of the big ones
    rng = np.random.default_rng(3)
    picks = []
    for k, n in enumerate(numels):
        if n <= 4096:
            picks.append((k, 0, n))
        elif rng.random() < 0.25:
            s = int(rng.integers(0, (n - CHUNK) // 64)) * 64
            picks.append((k, s, s + CHUNK))
            picks.append((k, n - CHUNK, n))
    # the tiles on both sides of every launch boundary (tile numbers run through the whole list)
    tile_begin = [table.host[k].tile_begin for k in range(len(numels))]
    for block in (262144, 524288):
        for edge in range(block, table.total_tiles, block):
            k = max(i for i in range(len(numels)) if tile_begin[i] <= edge)
            at = (edge - tile_begin[k]) * 256
            lo, hi = max(0, at - CHUNK // 2), min(numels[k], at + CHUNK // 2)
            if hi > lo:
                picks.append((k, lo, hi))
    xh = [to_np(xs[k][a:b]) for k, a, b in picks]
    mh = [to_np(ms[k][:, a:b]) for k, a, b in picks]
    exact = True
    hyp = (w.mode, w.beta1, w.beta2, w.lr, w.lam)
    for t in range(w.steps):
        for k in range(len(numels)):
            wl.make_grads(w, t, DEV, tensor=k, out=gs[k])
        gh = [to_np(gs[k][:, a:b]) for k, a, b in picks]
        ph, ch = oracle.step_mt(xh, mh, gh, *hyp)
        last = t == w.steps - 1
        if last:
            x_full, m_full, g_full = [to_np(t_) for t_ in xs], [to_np(t_) for t_ in ms], [to_np(t_) for t_ in gs]
            xs_u, ms_u = [t_.clone() for t_ in xs], [t_.clone() for t_ in ms]
            xs_a = [t_.clone() for t_ in xs]
            packed = torch.empty((N, Wt), dtype=torch.int64, device=DEV)
            counts = torch.empty(64 * Wt, dtype=torch.int16, device=DEV)
            dl.dlion_step_mt(table, N, *hyp, packed=packed, counts=counts, workspace=workspace)
        else:
            dl.dlion_step_mt(table, N, *hyp, workspace=workspace)
        torch.cuda.synchronize()
        for i, (k, a, b) in enumerate(picks):
            exact &= assert_f32_equal(to_np(ms[k][:, a:b]), mh[i], f"step {t} tensor {k}: m")
            exact &= assert_f32_equal(to_np(xs[k][a:b]), xh[i], f"step {t} tensor {k}: x")
        print(f"  step {t} ok", flush=True)
    got_p = torch.cat([packed[:, table.word_begin[k] + a // 64: table.word_begin[k] + (b + 63) // 64]
                       for k, a, b in picks], dim=1)
    got_c = torch.cat([counts[64 * table.word_begin[k] + a: 64 * table.word_begin[k] + b] for k, a, b in picks])
    assert np.array_equal(to_np(got_p), ph)
    assert np.array_equal(to_np(got_c), ch)
    c32 = counts.to(torch.int32) & 0xFFFF
    assert int(c32.max().item()) <= N
    assert popcount64_total(packed) == int(c32.sum(dtype=torch.int64).item())
    # the last step through the unfused calls on copies: whole arrays, bit for bit
    table_u = dl.SegTable(xs_u, ms_u, gs)
    packed_u = torch.empty((N, Wt), dtype=torch.int64, device=DEV)
    counts_u = torch.empty(64 * Wt, dtype=torch.int16, device=DEV)
    dl.dlion_worker_step_mt(table_u, packed_u, w.beta1, w.beta2)
    dl.dlion_aggregate_mt(table_u, packed_u, counts_u)
    dl.dlion_apply_mt(table_u, counts_u, N, w.mode, w.lr, w.lam)
    torch.cuda.synchronize()
    assert torch.equal(packed_u, packed) and torch.equal(counts_u, counts)
    for k in range(len(numels)):
        assert same_bits(ms_u[k], ms[k]) and same_bits(xs_u[k], xs[k]), f"tensor {k}: fused and unfused state differ"
    # the fused aggregate + update on the same packed words: a fourth kernel, whole arrays again
    counts_a = torch.empty(64 * Wt, dtype=torch.int16, device=DEV)
    dl.dlion_aggregate_apply_mt(dl.SegTable(xs_a, None, None), packed_u, w.mode, w.lr, w.lam, counts=counts_a)
    torch.cuda.synchronize()
    assert torch.equal(counts_a, counts)
    for k in range(len(numels)):
        assert same_bits(xs_a[k], xs[k]), f"tensor {k}: aggregate_apply_mt and the fused step differ"
    print("  fused step == worker_step + aggregate + apply == worker_step + aggregate_apply over all tensors", flush=True)
    # ... and against the oracle over all 148 tensors in full
    threads = min(len(os.sched_getaffinity(0)), 16)
    p_full, c_full = oracle.step_mt(x_full, m_full, g_full, *hyp, threads=threads)
    assert np.array_equal(to_np(packed), p_full)
    assert np.array_equal(unpad(counts, table), c_full)
    for k in range(len(numels)):
        exact &= assert_f32_equal(to_np(ms[k]), m_full[k], f"tensor {k}: m in full")
        exact &= assert_f32_equal(to_np(xs[k]), x_full[k], f"tensor {k}: x in full")
    print(f"{w.name}: {len(picks)} sampled ranges per step, last step against the oracle on all {w.d} x {N} updates; "
          f"fp32 state bit-identical: {exact}", flush=True)


def unpad(counts, table):
    """counts of a tensor list without the padding entries between a tensor's end and its next word"""
    c = to_np(counts)
    return np.concatenate([c[64 * table.word_begin[k]: 64 * table.word_begin[k] + table.numels[k]]
                           for k in range(table.K)])


def test_vote_only_256_streams_full_size():
    """Vote-only pass over N = 256 pre-packed random sign streams at d = 1.0 B."""
    w = wl.CONFIGS["packed256_1b"]
    d, N = w.d, w.N
    W = dl.words_for(d)
    announce(w.name, "d", d, "N", N, "W", W)
    packed = wl.random_packed(N, W, DEV, seed=w.seed, row_stride=wl.padded_words(W))   # as bench.py lays them out
    counts = torch.empty(d, dtype=torch.int16, device=DEV)
    dl.dlion_aggregate(packed, d, counts)
    torch.cuda.synchronize()
    # the bit-sliced kernel's workgroups own 8192 coordinates per wave, 16 waves each
    ranges = sample_chunks(d, 16, seed=11, edges=[8192 * 16 * k for k in (1, 2, 1000, 7629)] + [1 << 30])
    ph = to_np(gather_words(packed, ranges))
    want = oracle.aggregate_packed(ph, ph.shape[1] * 64)
    assert np.array_equal(to_np(gather(counts, ranges)), want)
    c32 = counts.to(torch.int32) & 0xFFFF
    assert int(c32.max().item()) <= N
    assert popcount64_total(packed) == int(c32.sum(dtype=torch.int64).item())
    # fused vote + apply on weights, both modes, against the oracle on the same chunks
    for mode in (dl.VOTE, dl.AVG):
        x = wl.init_x(w, DEV)
        xh = to_np(gather(x, ranges))
        oracle.apply(xh, want, N, mode, w.lr, w.lam)
        dl.dlion_aggregate_apply(x, packed, mode, w.lr, w.lam)
        torch.cuda.synchronize()
        assert_f32_equal(to_np(gather(x, ranges)), xh, f"aggregate_apply mode {mode}: x")
        del x
    print(f"{w.name}: counts bit-exact on {sum(b - a for a, b in ranges)} sampled coordinates; "
          f"sum(counts) equals the popcount of all {N * W} words", flush=True)


def test_unfused_and_wider_rows_full_size():
    """d = 1.3 B, N = 8: the unfused pipeline, the down-link planes, per-worker coefficients and
    Global Lion at a size where one stream is more than 2^32 bytes long, on sampled chunks."""
    w = wl.CONFIGS["stress1p3b_vote8"]
    d, N = w.d, w.N
    W = dl.words_for(d)
    announce("unfused + wider rows", "d", d, "N", N)
    ranges = sample_chunks(d, 16, seed=5, edges=launch_edges(d))
    x = wl.init_x(w, DEV)
    m = wl.init_m(w, DEV)
    m.normal_(0, 1e-3)
    g = wl.make_grads(w, 0, DEV)
    x0h, m0h, gh = to_np(gather(x, ranges)), to_np(gather(m, ranges)), to_np(gather(g, ranges))
    hyp = (w.beta1, w.beta2, w.lr, w.lam)

    # 1. worker_step -> aggregate -> apply, and aggregate_encode -> apply_encoded, both modes
    m1 = m.clone()
    packed = torch.empty((N, W), dtype=torch.int64, device=DEV)
    counts = torch.empty(d, dtype=torch.int16, device=DEV)
    dl.dlion_worker_step(m1, g, packed, w.beta1, w.beta2)
    dl.dlion_aggregate(packed, d, counts)
    torch.cuda.synchronize()
    mh = m0h.copy()
    ph = oracle.worker_step(mh, gh, w.beta1, w.beta2)
    ch = oracle.aggregate_packed(ph, ph.shape[1] * 64)[: x0h.shape[0]]
    assert np.array_equal(to_np(gather_words(packed, ranges)), ph)
    assert np.array_equal(to_np(gather(counts, ranges)), ch)
    assert_f32_equal(to_np(gather(m1, ranges)), mh, "worker_step: m")
    del m1
    for mode in (dl.VOTE, dl.AVG):
        xa = x.clone()
        dl.dlion_apply(xa, counts, N, mode, w.lr, w.lam)
        xh = x0h.copy()
        oracle.apply(xh, ch, N, mode, w.lr, w.lam)
        torch.cuda.synchronize()
        assert_f32_equal(to_np(gather(xa, ranges)), xh, f"apply mode {mode}: x")
        P = dl.dlion_delta_planes(N, mode)
        delta = torch.empty((P, W), dtype=torch.int64, device=DEV)
        dl.dlion_aggregate_encode(packed, d, mode, delta)
        xa.copy_(x)
        dl.dlion_apply_encoded(xa, delta, N, mode, w.lr, w.lam)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(gather_words(delta, ranges)), oracle.encode_delta(ch, N, mode))
        assert_f32_equal(to_np(gather(xa, ranges)), xh, f"apply_encoded mode {mode}: x")
        del xa, delta
    del packed, counts
    torch.cuda.empty_cache()
    print("  unfused pipeline and down-link ok", flush=True)

    # 2. per-worker coefficients, fused
    b1 = np.array([0.9, 0.5, 0.95, 0.8, 0.9, 0.0, 1.0, 0.99], np.float32)
    b2 = np.array([0.99, 0.75, 0.98, 0.8, 0.999, 0.5, 0.25, 0.99], np.float32)
    m2, x2 = m.clone(), x.clone()
    dl.dlion_step_pw(x2, m2, g, dl.VOTE, torch.from_numpy(b1).to(DEV), torch.from_numpy(b2).to(DEV), w.lr, w.lam)
    torch.cuda.synchronize()
    mh, xh = m0h.copy(), x0h.copy()
    ph = oracle.worker_step_pw(mh, gh, b1, b2)
    oracle.apply(xh, oracle.aggregate_packed(ph, ph.shape[1] * 64)[: xh.shape[0]], N, oracle.VOTE, w.lr, w.lam)
    assert_f32_equal(to_np(gather(m2, ranges)), mh, "step_pw: m")
    assert_f32_equal(to_np(gather(x2, ranges)), xh, "step_pw: x")
    del m2, x2
    torch.cuda.empty_cache()
    print("  per-worker coefficients ok", flush=True)

    # 3. Global Lion, in place on the originals
    bits = torch.empty(W, dtype=torch.int64, device=DEV)
    dl.dlion_global_lion_step(x, m, g, *hyp, sign_bits=bits)
    torch.cuda.synchronize()
    mh, xh = m0h.copy(), x0h.copy()
    bh = oracle.global_lion_step(xh, mh, gh, *hyp)
    assert np.array_equal(to_np(gather_words(bits, ranges)), bh)
    assert_f32_equal(to_np(gather(m, ranges)), mh, "global lion: m")
    assert_f32_equal(to_np(gather(x, ranges)), xh, "global lion: x")
    print("  Global Lion ok", flush=True)
