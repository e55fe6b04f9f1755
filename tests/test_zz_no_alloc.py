"""GPU test of the entry point that allocates nothing (duqpp_rotq_gemm_tiled_noalloc): through the C ABI, against
duqpp_rotq_gemm_tiled with a caller's workspace, bit for bit, on two calls in a row -- the second with a smaller
input, which finds the library's fixed scratch still holding the first call's bytes -- and on the error paths that
must not launch anything."""
import numpy as np
import pytest

import workloads as wl
from helpers import to_dev, to_dev_bf16

pytestmark = pytest.mark.gpu


def _case(torch, duqpp, name, T, K, N, shared=False):
    xb = wl.make_activations(name, T, K, (wl.OutlierSpec(min(8, K // 4), 50.0), wl.OutlierSpec(1, 1000.0, 1)))
    wb = wl.make_weights(name, N, K, 0.02)
    R = to_dev(wl.make_rotation_blocks(name, 1 if shared else K // 32), torch)
    x, w = to_dev_bf16(xb, torch), to_dev_bf16(wb, torch)
    bct, bst = duqpp.quantize_weights_tiled(w, R)
    return x, R, bct, bst


def test_noalloc_entry_point_matches_the_workspace_one_on_consecutive_calls():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    assert duqpp.noalloc_scratch_bytes() == 8 << 20
    # (T, K, N, output type, one shared rotation block): a prefill-sized call that nearly fills the scratch, then
    # smaller ones (ragged token tile, groups that need padding, a decode call), then a larger one again
    calls = [(1000, 14336, 520, duqpp.BF16, False), (77, 1184, 200, duqpp.F32, False), (1, 4096, 512, duqpp.F32, True),
             (16, 14336, 300, duqpp.BF16, False), (300, 2048, 264, duqpp.F32, False)]
    cases = [_case(torch, duqpp, f"noalloc-{i}", T, K, N, sh) for i, (T, K, N, dt, sh) in enumerate(calls)]
    # expected results first, from the entry point with a caller's workspace
    want = [duqpp.rotq_gemm_tiled(x, R, bct, bst, N, out_dtype=dt)
            for (x, R, bct, bst), (T, K, N, dt, sh) in zip(cases, calls)]
    outs = [torch.zeros_like(y) for y in want]
    torch.cuda.synchronize()
    for i, ((x, R, bct, bst), (T, K, N, dt, sh)) in enumerate(zip(cases, calls)):
        cb, sb = duqpp.tiled_bytes(T, K)
        assert (cb + 255) // 256 * 256 + (sb + 255) // 256 * 256 <= duqpp.noalloc_scratch_bytes()
        print(f"[noalloc] call {i}: T={T} K={K} N={N}", flush=True)
        duqpp.rotq_gemm_tiled_noalloc(x, R, bct, bst, N, out_dtype=dt, out=outs[i])      # back to back, same stream
    torch.cuda.synchronize()
    for i, (y, ref) in enumerate(zip(outs, want)):
        assert torch.equal(y, ref), i
        assert float(ref.float().abs().max()) > 0


def test_noalloc_entry_point_rejects_what_does_not_fit_and_bad_arguments():
    import torch

    import paper_2604_17789_amd as duqpp
    x, R, bct, bst = _case(torch, duqpp, "noalloc-big", 1100, 14336, 64)
    cb, sb = duqpp.tiled_bytes(1100, 14336)
    assert cb + sb > duqpp.noalloc_scratch_bytes()
    y = torch.full((1100, 64), 7.0, dtype=torch.float32, device=x.device)
    with pytest.raises(duqpp.DuqppError) as e:
        duqpp.rotq_gemm_tiled_noalloc(x, R, bct, bst, 64, out=y)
    assert e.value.status == -8 and "fixed scratch" in str(e.value)
    # a bad output type is refused before anything is launched (the output keeps its contents)
    x2, R2, bct2, bst2 = _case(torch, duqpp, "noalloc-dtype", 40, 256, 64)
    y2 = torch.full((40, 64), 7.0, dtype=torch.float32, device=x.device)
    st = duqpp.lib.duqpp_rotq_gemm_tiled_noalloc(x2.data_ptr(), x2.stride(0), R2.data_ptr(), R2.shape[0], bct2.data_ptr(),
                                                 bst2.data_ptr(), 40, 64, 256, y2.data_ptr(), 5, 64, None)
    assert st == -4
    torch.cuda.synchronize()
    assert bool((y == 7.0).all()) and bool((y2 == 7.0).all())


def test_noalloc_entry_point_under_graph_capture():
    """The callers it is for: a stream capture, where nothing may be allocated.  The per-device set-up is done ahead of
    the capture (duqpp_init); the captured call is replayed several times with the program's own eager work and
    synchronisations between the replays, each replay against the eager result of the workspace form."""
    import torch

    import paper_2604_17789_amd as duqpp
    duqpp.init()
    T, K, N = 24, 2048, 300
    x, R, bct, bst = _case(torch, duqpp, "noalloc-graph-0", T, K, N)
    y = torch.zeros((T, N), dtype=torch.float32, device=x.device)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            duqpp.rotq_gemm_tiled_noalloc(x, R, bct, bst, N, out=y)
    torch.cuda.synchronize()
    for rep in range(3):
        xn, _, _, _ = _case(torch, duqpp, f"noalloc-graph-{rep + 1}", T, K, N)
        x.copy_(xn)
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        want = duqpp.rotq_gemm_tiled(x, R, bct, bst, N)          # eager, with a workspace of its own
        torch.cuda.synchronize()
        assert torch.equal(y, want), rep
        assert float(want.abs().max()) > 0
