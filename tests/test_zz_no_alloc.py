"""The entry point that allocates nothing: dlion_step_noalloc against dlion_step_ws, through the C ABI.

Its workspace is a static device array inside the library that every call on the GPU shares and that keeps
the last call's contents, so the check is made on two calls in a row, the second on a smaller input.
"""
import numpy as np
import pytest
import torch

import paper_2404_00438_amd as dl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def draw(rng, N, d, g_dtype):
    x = torch.from_numpy(rng.normal(0, 0.02, d).astype(np.float32)).to(DEV)
    m = torch.from_numpy(rng.normal(0, 1e-3, (N, d)).astype(np.float32)).to(DEV)
    g = torch.from_numpy(rng.standard_t(3, (N, d)).astype(np.float32) * 1e-3).to(DEV).to(g_dtype)
    return x, m, g


def both_ways(x, m, g, mode, hyp, workspace, want_packed, want_counts):
    """One step through dlion_step_ws on copies and through dlion_step_noalloc in place; all outputs
    must be identical bit for bit (same kernels, same launch plan up to the block size)."""
    N, d = m.shape
    W = dl.words_for(d)
    x_ref, m_ref = x.clone(), m.clone()
    outs = []
    for _ in range(2):
        packed = torch.full((N, W), -1, dtype=torch.int64, device=DEV) if want_packed else None
        counts = torch.full((d,), -1, dtype=torch.int16, device=DEV) if want_counts else None
        outs.append((packed, counts))
    dl.dlion_step_ws(x_ref, m_ref, g, mode, *hyp, workspace, packed=outs[0][0], counts=outs[0][1])
    dl.dlion_step_noalloc(x, m, g, mode, *hyp, packed=outs[1][0], counts=outs[1][1])
    torch.cuda.synchronize()
    assert torch.equal(x.view(torch.int32), x_ref.view(torch.int32)), "x differs"
    assert torch.equal(m.view(torch.int32), m_ref.view(torch.int32)), "m differs"
    if want_packed:
        assert torch.equal(outs[0][0], outs[1][0]), "packed words differ"
    if want_counts:
        assert torch.equal(outs[0][1], outs[1][1]), "counts differ"


@pytest.mark.parametrize("per,tiles", [(3, 5), (8, 0), (2, 3)])
def test_noalloc_step_equals_workspace_step_forced_split(per, tiles, tune):
    """Small inputs with the split into launches over few workers forced, so that the static scratch
    really carries the votes: planes of partial counts (few launches) and running counts (many)."""
    tune(pass_workers=per, block_tiles=tiles)
    dl.dlion_noalloc_init()
    rng = np.random.default_rng(7 + per)
    workspace = torch.empty(8 << 20, dtype=torch.uint8, device=DEV)
    hyp = (0.9, 0.99, 3e-4, 0.1)
    # two calls in a row on the same scratch, the second with a smaller input (and fewer workers)
    for (N, d), mode, g_dtype in (((33, 70_001), dl.VOTE, torch.bfloat16), ((9, 4099), dl.AVG, torch.float32),
                                  ((70, 700), dl.VOTE, torch.bfloat16), ((4, 300), dl.AVG, torch.bfloat16)):
        print("[case] noalloc forced", per, tiles, "N", N, "d", d, "mode", mode, g_dtype, flush=True)
        x, m, g = draw(rng, N, d, g_dtype)
        both_ways(x, m, g, mode, hyp, workspace, True, True)
        both_ways(x, m, g, mode, hyp, workspace, False, False)


def test_noalloc_step_equals_workspace_step_default_plan():
    """The library's own plan at a size where it splits the step (16 workers, 17 M and then 5 M
    coordinates: the second, smaller call runs as one launch and must not be disturbed by what the
    first left in the scratch)."""
    rng = np.random.default_rng(5)
    hyp = (0.9, 0.99, 1e-4, 1.0)
    for N, d in ((16, 17_000_003), (16, 5_000_001)):
        print("[case] noalloc default plan N", N, "d", d, flush=True)
        x = torch.randn(d, device=DEV) * 0.02
        m = torch.randn((N, d), device=DEV) * 1e-3
        g = (torch.randn((N, d), device=DEV) * 1e-3).to(torch.bfloat16)
        ws_bytes = dl.dlion_step_workspace_bytes(d, N)
        assert (ws_bytes > 0) == (d > 16_000_000)
        workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=DEV)
        for mode in (dl.VOTE, dl.AVG):
            both_ways(x, m, g, mode, hyp, workspace, mode == dl.AVG, mode == dl.VOTE)
        del x, m, g, workspace
        torch.cuda.empty_cache()


def test_noalloc_step_validates_like_the_step():
    x = torch.zeros(1000, device=DEV)
    m = torch.zeros((4, 1000), device=DEV)
    g = torch.zeros((4, 1000), device=DEV)
    lib = dl.load_library()
    s = torch.cuda.current_stream().cuda_stream
    assert lib.dlion_step_noalloc(None, m.data_ptr(), 1000, g.data_ptr(), 1000, 0, 1000, 4, 0, 0.9, 0.99, 1e-3, 0.1,
                                  None, 0, None, s) == 1
    assert lib.dlion_step_noalloc(x.data_ptr(), m.data_ptr(), 999, g.data_ptr(), 1000, 0, 1000, 4, 0, 0.9, 0.99, 1e-3,
                                  0.1, None, 0, None, s) == 1
    assert lib.dlion_step_noalloc(x.data_ptr(), m.data_ptr(), 1000, g.data_ptr(), 1000, 0, 0, 4, 0, 0.9, 0.99, 1e-3,
                                  0.1, None, 0, None, s) == 1
