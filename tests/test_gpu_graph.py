"""bench.py times HIP-graph replays of a sequence of nm_conv2d launches.  The library
only enqueues kernels, so a captured sequence must reproduce the eager results on
every replay: a short dependent chain is captured once and replayed several times on
fresh inputs, with eager work and synchronisations in between, and every replay is
compared bit for bit with the eager run of the same inputs; the first one also goes
against the oracle layer by layer."""
import numpy as np
import pytest

from paper_2507_17301_amd import binding as nm
from paper_2507_17301_amd import workloads as wl
from gpu_util import FP32_TOL, BF16_TOL, say, norm_err, oracle_conv

pytestmark = pytest.mark.gpu

L = wl.ConvLayer
CHAIN = [
    L("g1_3x3", 12, 12, 64, 64, 3, 3, 1, 1, 1, 2, 4, 16),
    L("g2_1x1", 12, 12, 64, 128, 1, 1, 1, 0, 1, 2, 4, 16),
    L("g3_3x3_s2", 12, 12, 128, 64, 3, 3, 2, 1, 1, 1, 4, 16),
]


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_graph_replays_match_eager(bf16):
    import torch
    batch, replays = 3, 4
    tdt = torch.bfloat16 if bf16 else torch.float32
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    params = []
    for i, layer in enumerate(CHAIN):
        _, w, bias = wl.make_tensors(layer, batch, 8100 + i, with_input=False)
        params.append((w, bias, nm.nm_prune(w, layer.n, layer.m, layer.tile, ndt), torch.from_numpy(bias).cuda()))
    rng = np.random.default_rng(8200)
    inputs = [rng.random((batch, 12, 12, 64), dtype=np.float32) for _ in range(replays)]

    x_static = torch.zeros((batch, 12, 12, 64), dtype=tdt, device="cuda")
    acts = [x_static] + [torch.zeros((batch, l.Ho, l.Wo, l.Cout), dtype=tdt, device="cuda") for l in CHAIN]

    def run(stream=None):
        for i, layer in enumerate(CHAIN):
            nm.nm_conv2d(acts[i], params[i][2], params[i][3], layer.stride, layer.pad, layer.dil, True,
                         y=acts[i + 1], stream=stream)

    # eager results for every input (also the warm-up the capture needs)
    eager = []
    for r in range(replays):
        x_static.copy_(torch.from_numpy(inputs[r]).cuda().to(tdt))
        run()
        torch.cuda.synchronize()
        eager.append([a.clone() for a in acts[1:]])

    say(f"graph capture of {len(CHAIN)} launches, {'bf16' if bf16 else 'fp32'}")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(torch.cuda.current_stream())

    tol = BF16_TOL if bf16 else FP32_TOL
    for r in (2, 0, 3, 1, 0):                      # not in order, and one input twice
        x_static.copy_(torch.from_numpy(inputs[r]).cuda().to(tdt))
        for a in acts[1:]:
            a.fill_(float("nan"))                  # eager work between replays; stale outputs cannot pass
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, a in enumerate(acts[1:]):
            assert torch.equal(a, eager[r][i]), f"replay of input {r}, layer {CHAIN[i].name}"
    # the eager results themselves, layer by layer on the GPU's own previous activation
    prev = inputs[0]                               # (the oracle helper rounds bf16 inputs itself)
    for i, layer in enumerate(CHAIN):
        ref = oracle_conv(layer, prev, params[i][0], params[i][1], relu=True, bf16=bf16)
        got = eager[0][i].float().cpu().numpy()
        assert norm_err(got, ref) <= tol, layer.name
        prev = got
