"""GPU test of the promise that the same inputs give bit-identical outputs on every call: each kernel is run three
times on the same inputs with other launches of other sizes in between (which change what the caches hold and when
the workgroups start), and every output must repeat byte for byte.  No fp32 atomics or arrival-order reductions may
hide in any path."""
import numpy as np
import pytest

import workloads as wl
from helpers import to_dev, to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch

    import paper_2604_17789_amd as duqpp
    assert torch.cuda.is_available()
    return torch, duqpp


def _disturb(torch, duqpp, state):
    """Unrelated work between the repeats: a rotate+quantise and a product of another size."""
    if "x" not in state:
        state["x"] = to_dev_bf16(wl.make_activations("det-other", 333, 1184, (wl.OutlierSpec(4, 50.0),)), torch)
        state["R"] = to_dev(wl.make_rotation_blocks("det-other", 1184 // 32), torch)
        w = to_dev_bf16(wl.make_weights("det-other", 520, 1184, 0.02), torch)
        state["b"] = duqpp.quantize_weights_tiled(w, state["R"])
    duqpp.rotq_gemm_tiled(state["x"], state["R"], state["b"][0], state["b"][1], 520)


# (T, N, K, kernel forced by name or 0 for the library's choice)
CASES = [(16, 4100, 14336, 0), (1, 14336, 4096, 0), (48, 300, 1184, 1), (100, 8200, 544, 1), (300, 523, 1056, 2),
         (300, 523, 1056, 3), (513, 1032, 288, 4), (2048, 4096, 2048, 0), (1100, 8304, 544, 4)]


@pytest.mark.parametrize("T,N,K,kernel", CASES)
def test_every_path_repeats_bit_for_bit(env, T, N, K, kernel):
    torch, duqpp = env
    name = f"det-{T}-{N}-{K}"
    x = to_dev_bf16(wl.make_activations(name, T, K, (wl.OutlierSpec(min(8, K // 4), 50.0), wl.OutlierSpec(1, 1000.0, 1))), torch)
    R = to_dev(wl.make_rotation_blocks(name, K // 32), torch)
    w = to_dev_bf16(wl.make_weights(name, N, K, 0.02), torch)
    Rp = duqpp.pack_rotation(R)
    bct, bst = duqpp.quantize_weights_tiled(w, R)
    print(f"[determinism] T={T} N={N} K={K} kernel={kernel}", flush=True)
    state, runs = {}, []
    for rep in range(3):
        out = {}
        out["rm"] = duqpp.rotate_quantize(x, R)
        out["tiled"] = duqpp.rotate_quantize_tiled(x, R)
        out["packed"] = duqpp.rotate_quantize_tiled_packed(x, Rp)
        out["weights"] = duqpp.quantize_weights_tiled(w, R)
        act, ast = out["tiled"]
        out["y32"] = (duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=duqpp.F32, kernel=kernel),)
        out["y16"] = (duqpp.mxfp4_gemm_tiled(act, ast, bct, bst, T, N, K, out_dtype=duqpp.BF16, kernel=kernel),)
        out["rowmajor"] = (duqpp.rotq_gemm(x, R, *duqpp.untile_operand(bct, bst, N, K)),)
        if T <= 128:
            out["one_kernel"] = (duqpp.rotq_gemm_fused_decode(x, Rp, bct, bst, N),)
        torch.cuda.synchronize()
        runs.append(out)
        _disturb(torch, duqpp, state)
        torch.cuda.synchronize()
    for key in runs[0]:
        for rep in (1, 2):
            for a, b in zip(runs[0][key], runs[rep][key]):
                assert torch.equal(a, b), (key, rep)
    assert float(runs[0]["y32"][0].abs().max()) > 0
