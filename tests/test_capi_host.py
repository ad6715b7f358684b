"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and lays out tensor lists."""
import ctypes
import os
import re

import pytest

from paper_2404_00438_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return binding.load_library()


def declared_symbols():
    with open(os.path.join(ROOT, "include", "dlion.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dlion_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert lib.dlion_version() >= 100
    seen = {lib.dlion_status_str(s) for s in range(5)}
    assert len(seen) == 5 and all(seen)
    assert lib.dlion_status_str(99) == b"unknown status"


A = 0x7F0000000000   # a 256-byte aligned fake device address; never dereferenced by validation


def test_bad_arguments_are_rejected_on_the_host(lib):
    EINVAL, EALIGN = 1, 2
    ws = lib.dlion_worker_step
    assert ws(A, 128, A, 128, 0, A, 2, 0, 4, 0.9, 0.99, None) == EINVAL          # d = 0
    assert ws(A, 128, A, 128, 0, A, 2, -5, 4, 0.9, 0.99, None) == EINVAL         # d < 0
    assert ws(A, 128, A, 128, 0, A, 2, 128, 0, 0.9, 0.99, None) == EINVAL        # N = 0
    assert ws(A, 128, A, 128, 0, A, 2, 128, 65536, 0.9, 0.99, None) == EINVAL    # N too large
    assert ws(None, 128, A, 128, 0, A, 2, 128, 4, 0.9, 0.99, None) == EINVAL     # null m
    assert ws(A, 128, None, 128, 0, A, 2, 128, 4, 0.9, 0.99, None) == EINVAL     # null g
    assert ws(A, 128, A, 128, 0, None, 2, 128, 4, 0.9, 0.99, None) == EINVAL     # null packed
    assert ws(A, 127, A, 128, 0, A, 2, 128, 4, 0.9, 0.99, None) == EINVAL        # m stride < d
    assert ws(A, 128, A, 100, 0, A, 2, 128, 4, 0.9, 0.99, None) == EINVAL        # g stride < d
    assert ws(A, 128, A, 128, 0, A, 1, 128, 4, 0.9, 0.99, None) == EINVAL        # packed stride < W
    assert ws(A, 128, A, 128, 7, A, 2, 128, 4, 0.9, 0.99, None) == EINVAL        # dtype enum
    assert ws(A + 2, 128, A, 128, 0, A, 2, 128, 4, 0.9, 0.99, None) == EALIGN    # m not 4-aligned
    assert ws(A, 128, A + 1, 128, 1, A, 2, 128, 4, 0.9, 0.99, None) == EALIGN    # bf16 g not 2-aligned
    assert ws(A, 128, A, 128, 0, A + 4, 2, 128, 4, 0.9, 0.99, None) == EALIGN    # packed not 8-aligned

    ag = lib.dlion_aggregate
    assert ag(A, 2, 128, 4, None, None) == EINVAL
    assert ag(A, 2, 128, 4, A + 1, None) == EALIGN
    assert ag(None, 2, 128, 4, A, None) == EINVAL
    assert ag(A, 1, 128, 4, A, None) == EINVAL

    ap = lib.dlion_apply
    assert ap(None, A, 128, 4, 0, 1e-4, 0.1, None) == EINVAL
    assert ap(A, None, 128, 4, 0, 1e-4, 0.1, None) == EINVAL
    assert ap(A, A, 128, 4, 2, 1e-4, 0.1, None) == EINVAL                         # mode enum
    assert ap(A + 1, A, 128, 4, 0, 1e-4, 0.1, None) == EALIGN

    aa = lib.dlion_aggregate_apply
    assert aa(None, A, 2, 128, 4, 0, 1e-4, 0.1, None, None) == EINVAL
    assert aa(A, A, 2, 128, 4, 3, 1e-4, 0.1, None, None) == EINVAL
    assert aa(A, A, 1, 128, 4, 0, 1e-4, 0.1, None, None) == EINVAL

    st = lib.dlion_step
    assert st(None, A, 128, A, 128, 0, 128, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    assert st(A, A, 128, A, 128, 0, 128, 4, 5, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    assert st(A, A, 128, A, 128, 0, 128, 4, 0, 0.9, 0.99, 1e-4, 0.1, A, 1, None, None) == EINVAL
    assert st(A, A, 128, A, 128, 0, 128, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, A + 1, None) == EALIGN
    assert st(A, A, 64, A, 128, 0, 128, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL


def test_tensor_list_layout_and_validation(lib):
    EINVAL = 1
    K = 5
    numels = [64, 1000, 5, 256, 257]
    arr = (binding.Seg * K)()
    for k, n in enumerate(numels):
        arr[k].x = A
        arr[k].m = A
        arr[k].g = A
        arr[k].m_stride = n
        arr[k].g_stride = n
        arr[k].numel = n
    tw, tt = ctypes.c_int64(), ctypes.c_int64()
    assert lib.dlion_mt_layout(arr, K, ctypes.byref(tw), ctypes.byref(tt)) == 0
    words = [(n + 63) // 64 for n in numels]
    tiles = [(n + 255) // 256 for n in numels]
    assert tw.value == sum(words) and tt.value == sum(tiles)
    assert [arr[k].word_begin for k in range(K)] == [sum(words[:k]) for k in range(K)]
    assert [arr[k].tile_begin for k in range(K)] == [sum(tiles[:k]) for k in range(K)]
    # a table that was not laid out, or tampered with, is refused before any launch
    arr[3].word_begin += 1
    assert lib.dlion_step_mt(arr, A, K, 0, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    arr[3].word_begin -= 1
    arr[2].numel = 0
    assert lib.dlion_mt_layout(arr, K, None, None) == EINVAL
    assert lib.dlion_step_mt(arr, A, K, 0, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    arr[2].numel = 5
    assert lib.dlion_step_mt(arr, None, K, 0, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    assert lib.dlion_step_mt(None, A, K, 0, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    assert lib.dlion_step_mt(arr, A, 0, 0, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    arr[1].m = None
    assert lib.dlion_step_mt(arr, A, K, 0, 4, 0, 0.9, 0.99, 1e-4, 0.1, None, 0, None, None) == EINVAL
    assert lib.dlion_aggregate_mt(arr, A, K, A, 2, 4, A, None) == EINVAL      # packed stride < total words
    assert lib.dlion_mt_layout(None, K, None, None) == EINVAL


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        binding.load_library(os.path.join(tmp_path, "libdlion.so"))


def test_wider_rows_validation(lib):
    EINVAL, EALIGN = 1, 2
    assert lib.dlion_delta_planes(3, 0) == 1 and lib.dlion_delta_planes(4, 0) == 2
    assert [lib.dlion_delta_planes(n, 1) for n in (1, 2, 3, 4, 7, 8, 255, 256, 65535)] == [1, 2, 2, 3, 3, 4, 8, 9, 16]
    assert lib.dlion_delta_planes(0, 0) == 0 and lib.dlion_delta_planes(4, 7) == 0
    enc = lib.dlion_aggregate_encode
    assert enc(None, 2, 128, 4, 0, A, 2, None) == EINVAL
    assert enc(A, 2, 128, 4, 0, None, 2, None) == EINVAL
    assert enc(A, 2, 128, 4, 0, A, 1, None) == EINVAL          # two planes need stride >= W
    assert enc(A, 2, 128, 4, 9, A, 2, None) == EINVAL
    assert enc(A, 2, 128, 4, 0, A + 4, 2, None) == EALIGN
    dec = lib.dlion_apply_encoded
    assert dec(None, A, 2, 128, 4, 0, 1e-4, 0.1, None) == EINVAL
    assert dec(A, None, 2, 128, 4, 0, 1e-4, 0.1, None) == EINVAL
    assert dec(A + 2, A, 2, 128, 4, 0, 1e-4, 0.1, None) == EALIGN
    assert dec(A, A, 1, 128, 4, 1, 1e-4, 0.1, None) == EINVAL  # three planes, stride < W
    pw = lib.dlion_worker_step_pw
    assert pw(A, 128, A, 128, 0, A, 2, 128, 4, None, A, None) == EINVAL
    assert pw(A, 128, A, 128, 0, A, 2, 128, 4, A, None, None) == EINVAL
    assert pw(A, 128, A, 128, 0, A, 2, 128, 4, A + 2, A, None) == EALIGN
    spw = lib.dlion_step_pw
    assert spw(A, A, 128, A, 128, 0, 128, 4, 0, None, A, 1e-4, 0.1, None, 0, None, None) == EINVAL
    assert spw(None, A, 128, A, 128, 0, 128, 4, 0, A, A, 1e-4, 0.1, None, 0, None, None) == EINVAL
    spww = lib.dlion_step_pw_ws
    assert spww(A, A, 128, A, 128, 0, 128, 4, 0, A, None, 1e-4, 0.1, None, 0, None, None, 0, None) == EINVAL
    assert spww(A, A, 128, A, 128, 0, 128, 4, 0, A, A, 1e-4, 0.1, None, 0, None, None, 64, None) == EINVAL
    assert spww(A, A, 128, A, 128, 0, 128, 4, 0, A, A, 1e-4, 0.1, None, 0, None, A, -1, None) == EINVAL
    assert spww(A, A, 128, A, 128, 0, 128, 4, 0, A, A, 1e-4, 0.1, None, 0, None, A + 8, 4096, None) == EALIGN
    gl = lib.dlion_global_lion_step
    assert gl(None, A, 128, A, 128, 0, 128, 4, 0.9, 0.99, 1e-4, 0.1, None, None) == EINVAL
    assert gl(A, A, 100, A, 128, 0, 128, 4, 0.9, 0.99, 1e-4, 0.1, None, None) == EINVAL
    assert gl(A, A, 128, A, 128, 3, 128, 4, 0.9, 0.99, 1e-4, 0.1, None, None) == EINVAL
    assert gl(A, A, 128, A, 128, 0, 128, 4, 0.9, 0.99, 1e-4, 0.1, A + 4, None) == EALIGN


def test_product_and_oracle_do_not_import_each_other():
    """The HIP path and the oracle share no code: neither package imports the other, and the C
    sources include nothing of each other's."""
    import ast
    import glob

    def imported(path):
        with open(path) as f:
            tree = ast.parse(f.read())
        names = set()
        for node in ast.walk(tree):
            if isinstance(node, ast.Import):
                names.update(a.name.split(".")[0] for a in node.names)
            elif isinstance(node, ast.ImportFrom) and node.module and node.level == 0:
                names.add(node.module.split(".")[0])
        return names

    for path in glob.glob(os.path.join(ROOT, "paper_2404_00438_amd", "*.py")):
        assert "oracle" not in imported(path), path
    for path in glob.glob(os.path.join(ROOT, "oracle", "*.py")):
        assert "paper_2404_00438_amd" not in imported(path), path
    for path in glob.glob(os.path.join(ROOT, "paper_2404_00438_amd", "csrc", "*")):
        with open(path) as f:
            assert "oracle" not in f.read().lower(), path
    with open(os.path.join(ROOT, "oracle", "dlion_oracle.c")) as f:
        text = f.read()
    includes = [line for line in text.splitlines() if line.lstrip().startswith("#include")]
    assert includes and all("dlion" not in line and "hip" not in line for line in includes), includes


def test_workspace_entry_point_validation(lib):
    """dlion_step_ws rejects a bad workspace before anything is launched; the size helper is host-only."""
    EINVAL, EALIGN = 1, 2

    def call(ws, nbytes):
        return lib.dlion_step_ws(A, A, 1024, A, 1024, 0, 1024, 4, 0, 0.9, 0.99, 1e-3, 0.1, None, 0, None, ws, nbytes, None)

    assert call(A, -1) == EINVAL              # negative size
    assert call(None, 4096) == EINVAL         # a size without a pointer
    assert call(A + 8, 4096) == EALIGN        # workspace not 16-byte aligned
    assert lib.dlion_step_workspace_bytes(1000, 4) == 0
    assert lib.dlion_step_workspace_bytes(-5, 32) == 0
    # 4 launches over 8 workers: 3 planes of 128 bytes per tile, 262144 tiles at a time
    assert lib.dlion_step_workspace_bytes(350_000_000, 32) == 262144 * 3 * 128
    # 16 launches: a running count, 512 bytes per tile
    assert lib.dlion_step_workspace_bytes(350_000_000, 128) == 262144 * 512
    assert lib.dlion_step_mt_workspace_bytes(0, 32) == 0 and lib.dlion_step_mt_workspace_bytes(1 << 31, 32) == 0
    assert lib.dlion_step_mt_workspace_bytes(78125, 16) == 78125 * 128

    def call_mt(ws, nbytes):
        return lib.dlion_step_mt_ws(None, A, 1, 0, 4, 0, 0.9, 0.99, 1e-3, 0.1, None, 0, None, ws, nbytes, None)

    assert call_mt(A, -1) == EINVAL and call_mt(None, 64) == EINVAL and call_mt(A + 8, 4096) == EALIGN
    assert call_mt(A, 4096) == EINVAL         # null table


def test_tuning_overrides_are_validated_and_restored(lib):
    """dlion_set_tuning: host-only state, every field -1 by default, out-of-range values refused."""
    t = binding.Tuning()
    lib.dlion_get_tuning(ctypes.byref(t))
    assert [getattr(t, f) for f, _ in binding.Tuning._fields_] == [-1] * len(binding.Tuning._fields_)
    try:
        binding.dlion_set_tuning(pass_workers=3, block_tiles=5, unroll=4)
        now = binding.dlion_get_tuning()
        assert (now.pass_workers, now.block_tiles, now.unroll, now.sliced_waves) == (3, 5, 4, -1)
        # the size helper follows the overrides: 11 launches of 3 workers need a running count
        assert lib.dlion_step_workspace_bytes(70_001, 33) == 5 * 512
        with binding.tuned(pass_workers=0):
            assert binding.dlion_get_tuning().pass_workers == 0 and binding.dlion_get_tuning().block_tiles == 5
            assert lib.dlion_step_workspace_bytes(350_000_000, 32) == 0
        assert binding.dlion_get_tuning().pass_workers == 3
        for bad in (dict(unroll=3), dict(sliced_waves=4), dict(blocks_per_cu=-2), dict(step_quads=2),
                    dict(block_tiles=-7), dict(pass_workers=-3), dict(group_max_workers=121), dict(group_blocks=65)):
            with pytest.raises(binding.DlionError):
                binding.dlion_set_tuning(**bad)
        assert binding.dlion_get_tuning().pass_workers == 3          # a refused struct changes nothing
        with pytest.raises(TypeError):
            binding.dlion_set_tuning(no_such_field=1)
    finally:
        binding.dlion_set_tuning(None)
    assert binding.dlion_get_tuning().pass_workers == -1 and binding.dlion_get_tuning().block_tiles == -1


class _Recorder:
    """Stands in for the loaded library: records calls, launches nothing."""

    def __init__(self, real):
        self.real, self.calls = real, []

    def __getattr__(self, name):
        if name in ("dlion_delta_planes", "dlion_mt_layout", "dlion_status_str"):
            return getattr(self.real, name)

        def fn(*args):
            self.calls.append(name)
            return 0
        return fn


def test_binding_checks_extents_before_calling_the_library(lib, monkeypatch):
    """The C ABI sees pointers, not tensor sizes: the binding must refuse short, strided, host or
    mismatched tensors itself.  Host tensors stand in for device ones here (the device check is
    switched off, and a recorder replaces the library so nothing is launched)."""
    import torch

    rec = _Recorder(lib)
    monkeypatch.setattr(binding, "load_library", lambda path=None: rec)
    monkeypatch.setattr(binding, "_stream", lambda s: 0)
    N, d = 4, 1000
    W = binding.words_for(d)
    x = torch.zeros(d)
    m = torch.zeros(N, d)
    g = torch.zeros(N, d)
    packed = torch.zeros(N, W, dtype=torch.int64)
    counts = torch.zeros(d, dtype=torch.int16)

    # host tensors are refused while the device check is on
    for call in (lambda: binding.dlion_aggregate(packed, d, counts),
                 lambda: binding.dlion_apply(x, counts, N, 0, 1e-3, 0.1),
                 lambda: binding.dlion_step(x, m, g, 0, 0.9, 0.99, 1e-3, 0.1),
                 lambda: binding.dlion_step_ws(x, m, g, 0, 0.9, 0.99, 1e-3, 0.1, torch.zeros(64, dtype=torch.uint8))):
        with pytest.raises(ValueError):
            call()
    assert rec.calls == []

    monkeypatch.setattr(binding, "_on_device", lambda t: True)
    binding.dlion_worker_step(m, g, packed, 0.9, 0.99)
    binding.dlion_aggregate(packed, d, counts)
    binding.dlion_apply(x, counts, N, 0, 1e-3, 0.1)
    binding.dlion_aggregate_apply(x, packed, 0, 1e-3, 0.1, counts=counts)
    binding.dlion_step(x, m, g, 0, 0.9, 0.99, 1e-3, 0.1, packed=packed, counts=counts)
    good = list(rec.calls)
    assert good == ["dlion_worker_step", "dlion_aggregate", "dlion_apply", "dlion_aggregate_apply", "dlion_step"]

    short_packed = torch.zeros(N, W - 1, dtype=torch.int64)
    short_counts = torch.zeros(d - 1, dtype=torch.int16)
    bad = [
        lambda: binding.dlion_worker_step(m, g, short_packed, 0.9, 0.99),
        lambda: binding.dlion_worker_step(m, g, packed, 0.9, 0.99, d=d + 1),        # d beyond the rows
        lambda: binding.dlion_worker_step(m, g, packed[:3], 0.9, 0.99),             # N mismatch
        lambda: binding.dlion_worker_step(m, torch.zeros(N, d + 1), packed, 0.9, 0.99),
        lambda: binding.dlion_aggregate(short_packed, d, counts),
        lambda: binding.dlion_aggregate(packed, d, short_counts),
        lambda: binding.dlion_aggregate(packed, d, torch.zeros(2 * d, dtype=torch.int16)[::2]),   # strided counts
        lambda: binding.dlion_aggregate(packed, d, torch.zeros(d, 1, dtype=torch.int16)),         # not 1-D
        lambda: binding.dlion_apply(x, short_counts, N, 0, 1e-3, 0.1),
        lambda: binding.dlion_aggregate_apply(x, short_packed, 0, 1e-3, 0.1),
        lambda: binding.dlion_aggregate_apply(x, packed, 0, 1e-3, 0.1, counts=short_counts),
        lambda: binding.dlion_step(x, m, g, 0, 0.9, 0.99, 1e-3, 0.1, packed=short_packed),
        lambda: binding.dlion_step(x, m, g, 0, 0.9, 0.99, 1e-3, 0.1, counts=short_counts),
        lambda: binding.dlion_step(x[:-1], m, g, 0, 0.9, 0.99, 1e-3, 0.1),
        lambda: binding.dlion_step(x, m, g[:, ::2], 0, 0.9, 0.99, 1e-3, 0.1),       # strided rows
        lambda: binding.dlion_step_ws(x, m, g, 0, 0.9, 0.99, 1e-3, 0.1, torch.zeros(8, 8)[:, ::2]),
        lambda: binding.dlion_aggregate_encode(packed, d, 0, torch.zeros(2, W - 1, dtype=torch.int64)),
        lambda: binding.dlion_aggregate_encode(packed, d, 0, torch.zeros(1, W, dtype=torch.int64)),   # N even: 2 planes
        lambda: binding.dlion_apply_encoded(x, torch.zeros(2, W - 1, dtype=torch.int64), N, 0, 1e-3, 0.1),
        lambda: binding.dlion_global_lion_step(x, m, g, 0.9, 0.99, 1e-3, 0.1, sign_bits=torch.zeros(W - 1, dtype=torch.int64)),
        lambda: binding.dlion_step_pw(x, m, g, 0, torch.zeros(N - 1), torch.zeros(N), 1e-3, 0.1),
    ]
    for k, call in enumerate(bad):
        with pytest.raises((ValueError, TypeError)):
            call()
        assert rec.calls == good, f"case {k} reached the library"

    # tensor lists: packed / counts against the table's totals, N against the table's rows
    xs = [torch.zeros(n) for n in (1000, 5, 300)]
    ms = [torch.zeros(N, n) for n in (1000, 5, 300)]
    gs = [torch.zeros(N, n) for n in (1000, 5, 300)]
    table = binding.SegTable(xs, ms, gs, device="cpu")
    Wt = table.total_words
    assert Wt == 16 + 1 + 5
    ok_packed = torch.zeros(N, Wt, dtype=torch.int64)
    ok_counts = torch.zeros(64 * Wt, dtype=torch.int16)
    binding.dlion_step_mt(table, N, 0, 0.9, 0.99, 1e-3, 0.1, packed=ok_packed, counts=ok_counts)
    good = list(rec.calls)
    bad = [
        lambda: binding.dlion_step_mt(table, N + 1, 0, 0.9, 0.99, 1e-3, 0.1),
        lambda: binding.dlion_step_mt(table, N, 0, 0.9, 0.99, 1e-3, 0.1, packed=torch.zeros(N, Wt - 1, dtype=torch.int64)),
        lambda: binding.dlion_step_mt(table, N, 0, 0.9, 0.99, 1e-3, 0.1, counts=torch.zeros(64 * Wt - 1, dtype=torch.int16)),
        lambda: binding.dlion_worker_step_mt(table, torch.zeros(N + 1, Wt, dtype=torch.int64), 0.9, 0.99),
        lambda: binding.dlion_aggregate_mt(table, ok_packed, torch.zeros(1000 + 5 + 300, dtype=torch.int16)),
        lambda: binding.dlion_apply_mt(table, ok_counts[:-64], N, 0, 1e-3, 0.1),
        lambda: binding.dlion_aggregate_apply_mt(table, ok_packed[:, :-1], 0, 1e-3, 0.1),
    ]
    for k, call in enumerate(bad):
        with pytest.raises((ValueError, TypeError)):
            call()
        assert rec.calls == good, f"tensor-list case {k} reached the library"


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU and says so when asked for more (no GPU needed for that)."""
    import subprocess
    import sys

    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and res.stdout.strip() == ""
