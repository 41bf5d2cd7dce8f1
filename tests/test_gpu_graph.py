"""The library's calls under HIP graph capture by the caller: every entry point only enqueues
kernels on the stream it is given (no allocation, copy, memset or synchronisation inside), so
a training step can be captured once and replayed.  One layer per implementation (implicit
GEMM, fused Winograd with its fix-up pass, unfused Winograd with its split GEMM round, product
of spectra), all three passes, captured into one graph; the graph is replayed several times
with the inputs changed and eager work run in between, and every replay must equal, bit for
bit, what the same calls give eagerly on the same inputs (the kernels are deterministic)."""
import pytest

from paper_1606_04884_amd import binding as B
from paper_1606_04884_amd import synth

pytestmark = pytest.mark.gpu

LAYERS = [
    ((3, 24, 17, 13, 40, 3, 3, 2, 1, 1, 1), B.ALGO_IGEMM),
    ((6, 64, 30, 30, 96, 3, 3, 1, 1, 1, 1), B.ALGO_WINOGRAD),
    ((8, 64, 16, 16, 128, 3, 3, 1, 1, 1, 1), B.ALGO_WINOGRAD4),
    ((8, 32, 27, 27, 48, 5, 5, 1, 1, 2, 2), B.ALGO_FFT),
]


def _make(dev):
    import torch
    recs = []
    for i, (geom, algo) in enumerate(LAYERS):
        N, C, H, W, K, R, S = geom[:7]
        P, Q = B.conv2d_output_dims(geom)
        r = dict(geom=B.make_desc(geom), algo=algo)
        r["x"] = torch.empty((N, C, H, W), device=dev)
        r["w"] = torch.empty((K, C, R, S), device=dev)
        r["b"] = torch.empty((K,), device=dev)
        r["dy"] = torch.empty((N, K, P, Q), device=dev)
        r["out"] = {k: torch.empty_like(r[s]) for k, s in (("y", "dy"), ("dx", "x"), ("dw", "w"), ("db", "b"))}
        need = max(B.conv2d_workspace_bytes(r["geom"], op, algo) for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT))
        assert need > 0 or algo == B.ALGO_IGEMM
        r["ws"] = B.alloc_workspace(need, dev)
        r["seed0"] = 9100 + 10 * i
        recs.append(r)
    return recs


def _fill(recs, variant):
    import torch
    for r in recs:
        for j, k in enumerate(("x", "w", "b", "dy")):
            t = r[k]
            std = 0.05 if k == "w" else 1.0
            t.copy_(torch.from_numpy(synth.normal(tuple(t.shape), r["seed0"] + 100 * variant + j, std=std)))


def _step(recs, out_key="out"):
    for r in recs:
        o = r[out_key]
        B.conv2d_fwd(r["geom"], r["x"], r["w"], r["b"], o["y"], ws=r["ws"], algo=r["algo"])
        B.conv2d_bwd_data(r["geom"], r["dy"], r["w"], o["dx"], ws=r["ws"], algo=r["algo"])
        B.conv2d_bwd_weight(r["geom"], r["x"], r["dy"], o["dw"], o["db"], ws=r["ws"], algo=r["algo"])


def test_captured_step_replays_bit_exactly():
    import torch
    dev = torch.device("cuda:0")
    recs = _make(dev)
    for r in recs:
        r["eager"] = {k: torch.empty_like(v) for k, v in r["out"].items()}
    _fill(recs, 0)
    _step(recs)                       # warm-up outside the capture: one-time kernel attributes are set here
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _step(recs)
    torch.cuda.synchronize()
    for variant in (1, 2, 3, 1):
        _fill(recs, variant)          # new inputs in the same buffers
        for r in recs:
            for t in r["out"].values():
                t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        _step(recs, "eager")          # the program's own eager work between replays
        torch.cuda.synchronize()
        for li, r in enumerate(recs):
            for k in ("y", "dx", "dw", "db"):
                assert torch.isfinite(r["out"][k]).all(), (variant, li, k)
                assert torch.equal(r["out"][k], r["eager"][k]), (variant, li, k)
