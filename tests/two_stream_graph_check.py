"""Run by test_gpu_tiled.py::test_two_stream_graph_matches_eager_launches in a process of its own: a HIP graph of
rotate+quantise launches on one stream and GEMM launches on another, tied by events, replayed three times with eager
work between the replays; every replay must give bit for bit what eager launches give."""
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import paper_2604_17789_amd as duqpp  # noqa: E402
import workloads as wl  # noqa: E402
from helpers import to_dev, to_dev_bf16  # noqa: E402

T, N, K, nsets, steps = 300, 520, 1184, 2, 7
R = to_dev(wl.make_rotation_blocks("graph2", K // 32), torch)
w = to_dev_bf16(wl.make_weights("graph2", N, K, 0.02), torch)
bct, bst = duqpp.quantize_weights_tiled(w, R)
cb, sb = duqpp.tiled_bytes(T, K)
sets = []
for k in range(nsets):
    x = to_dev_bf16(wl.make_activations(f"graph2-{k}", T, K, (wl.OutlierSpec(4, 50.0),)), torch)
    sets.append(dict(x=x, a=(torch.empty(cb, dtype=torch.uint8, device=x.device), torch.empty(sb, dtype=torch.uint8, device=x.device)),
                     y=torch.empty((T, N), dtype=torch.float32, device=x.device)))

def rq(s_):
    duqpp.rotate_quantize_tiled(s_["x"], R, out=s_["a"])

def gm(s_):
    duqpp.mxfp4_gemm_tiled(s_["a"][0], s_["a"][1], bct, bst, T, N, K, out=s_["y"])

for s_ in sets:
    rq(s_)
    gm(s_)
torch.cuda.synchronize()
sg, sr = torch.cuda.Stream(), torch.cuda.Stream()
sg.wait_stream(torch.cuda.current_stream())
g = torch.cuda.CUDAGraph()
with torch.cuda.stream(sg):
    with torch.cuda.graph(g, stream=sg):
        sr.wait_stream(sg)
        free = {}
        events = []                                    # kept alive until the capture has ended
        for i in range(steps):
            k = i % nsets
            with torch.cuda.stream(sr):
                if k in free:
                    sr.wait_event(free[k])
                rq(sets[k])
                ready = torch.cuda.Event()
                ready.record(sr)
            sg.wait_event(ready)
            gm(sets[k])
            free[k] = torch.cuda.Event()
            free[k].record(sg)
            events += [ready, free[k]]
        sg.wait_stream(sr)
torch.cuda.synchronize()
for rep in range(3):
    for k, s_ in enumerate(sets):
        s_["x"].copy_(to_dev_bf16(wl.make_activations(f"graph2-{k}-{rep}", T, K, (wl.OutlierSpec(4, 50.0),)), torch))
        s_["y"].zero_()
        s_["a"][0].zero_()
    g.replay()
    torch.cuda.synchronize()
    got = [(s_["y"].clone(), s_["a"][0].clone()) for s_ in sets]
    for s_ in sets:
        s_["y"].zero_()
        rq(s_)
        gm(s_)
    torch.cuda.synchronize()
    for s_, (y_g, a_g) in zip(sets, got):
        assert torch.equal(y_g, s_["y"]) and torch.equal(a_g, s_["a"][0]), rep
        assert float(s_["y"].abs().max()) > 0

print("two-stream graph: OK", flush=True)
