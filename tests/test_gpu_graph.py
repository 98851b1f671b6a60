"""Every entry point enqueues plain kernel launches on the caller's stream and nothing else (no
allocation, no memset, no synchronisation), so a training step can be captured into a HIP graph.
The graph is replayed several times on fresh inputs, with eager work and synchronisations in
between, and every replay must reproduce the eager results bit for bit (the library is
deterministic)."""
import pytest
import torch

import paper_1911_10175_amd as st
import stgen
from oracle.st_ref import Geom

from tests.gpu_harness import desc_of, dev, workspace

pytestmark = pytest.mark.gpu

# (entry point, pass id for the workspace query, dense flag, first operand, second operand, output)
CALLS = (
    ("st_conv_fwd", st.ST_PASS_FWD, False, "x", "w", "y"),
    ("st_conv_fwd_dense", st.ST_PASS_FWD, True, "x", "w", "y"),
    ("st_conv_fwd_auto", st.ST_PASS_FWD_AUTO, False, "x", "w", "y"),
    ("st_conv_bwi", st.ST_PASS_BWI, False, "dy", "w", "dx"),
    ("st_conv_bwi_dense", st.ST_PASS_BWI, True, "dy", "w", "dx"),
    ("st_conv_bwi_auto", st.ST_PASS_BWI_AUTO, False, "dy", "w", "dx"),
    ("st_conv_bww", st.ST_PASS_BWW, False, "x", "dy", "dw"),
    ("st_conv_bww_dense", st.ST_PASS_BWW, True, "x", "dy", "dw"),
    ("st_conv_bww_dy", st.ST_PASS_BWW_DY, False, "x", "dy", "dw"),
    ("st_conv_bww_auto", st.ST_PASS_BWW_AUTO, False, "x", "dy", "dw"),
)


def draw(g: Geom, seed: int, px: float, pdy: float):
    x = stgen.relu_sparse((g.N, g.C, g.H, g.W), px, seed)
    w = stgen.he_normal((g.K, g.C, g.S, g.R), seed + 1)
    dy = stgen.bernoulli_masked((g.N, g.K, g.OH, g.OW), pdy, seed + 2, seed + 3)
    return {"x": dev(st.pack_activations(x)), "w": dev(st.pack_filters(w)), "dy": dev(st.pack_activations(dy))}


@pytest.mark.parametrize("g", [Geom(2, 64, 128, 14, 14, 3, 3, 1, 1, 1, 1), Geom(2, 64, 64, 9, 9, 1, 1, 1, 1, 0, 0),
                               Geom(1, 32, 32, 11, 11, 3, 3, 2, 2, 1, 1),
                               # 9408 pixels, 64 KB filter matrix: the dense 1x1 form that keeps the filters in
                               # LDS (more dynamic LDS than the default limit) for FWD and for BWI
                               Geom(3, 256, 64, 56, 56, 1, 1, 1, 1, 0, 0),
                               # FWD auto through the single main kernel that holds both forms (the replays see 10 %,
                               # 60 % and 95 % zeros: both sides of the break-even), BWW auto through its merged launches
                               Geom(8, 64, 128, 56, 56, 3, 3, 1, 1, 1, 1)],
                         ids=["3x3", "1x1", "3x3s2", "1x1-filters-in-lds", "3x3-single-auto-kernel"])
def test_graph_replays_match_eager(g):
    d = desc_of(g)
    shapes = {"y": (g.N, g.K // 16, g.OH, g.OW, 16), "dx": (g.N, g.C // 16, g.H, g.W, 16),
              "dw": (g.K // 16, g.C // 16, g.S, g.R, 16, 16)}
    static = draw(g, 100, 0.5, 0.5)
    outs = [torch.zeros(shapes[c[5]], device="cuda") for c in CALLS]
    wss = [workspace(d, c[1], c[2]) for c in CALLS]

    def enqueue(inputs, outputs, stream):
        for c, o, ws in zip(CALLS, outputs, wss):
            getattr(st, c[0])(d, inputs[c[3]], inputs[c[4]], o, ws, stream)

    # warm-up outside the capture (module loading), then capture one pass over all entry points
    enqueue(static, outs, torch.cuda.current_stream())
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue(static, outs, torch.cuda.current_stream())
    torch.cuda.synchronize()

    for rep, (seed, px, pdy) in enumerate(((200, 0.6, 0.3), (300, 0.1, 0.9), (400, 0.95, 0.95))):
        fresh = draw(g, seed, px, pdy)
        eager = [torch.full(shapes[c[5]], float("nan"), device="cuda") for c in CALLS]
        enqueue(fresh, eager, torch.cuda.current_stream())          # eager work between the replays
        torch.cuda.synchronize()
        for k in static:
            static[k].copy_(fresh[k])
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for c, o, e in zip(CALLS, outs, eager):
            assert torch.equal(o, e), f"replay {rep}: {c[0]} differs from the eager call"
