"""The whole path (predict, group_by_expert, score) recorded into a HIP graph: every replay must reproduce the
eager result bit for bit, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2511_10676_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,path", [(8, "decode"), (600, "prefill")])
def test_graph_replays_match_eager(T, path):
    L, d, r, E, k = 3, 256, 256, 64, 6
    g = torch.Generator(device="cuda"); g.manual_seed(T)
    xs = [torch.randn((L, T, d), device="cuda", generator=g).to(torch.bfloat16) for _ in range(3)]
    W1 = (torch.randn((L, r, d), device="cuda", generator=g) / d ** 0.5).to(torch.bfloat16)
    W2 = (torch.randn((L, E, r), device="cuda", generator=g) / r ** 0.5).to(torch.bfloat16)
    ref = torch.randint(0, E, (L, T, k), device="cuda", dtype=torch.int32)
    desc = B.make_desc(T, d, r, E, k, L, B.BF16)
    assert B.resolve_path(desc) == path

    def buffers():
        out = B.Prediction(torch.empty((L, T, k), dtype=torch.int32, device="cuda"),
                           torch.empty((L, T, k), dtype=torch.float32, device="cuda"), None, path)
        ws = torch.empty(max(B.predict_workspace_bytes(desc), 16), dtype=torch.uint8, device="cuda")
        grp = B.alloc_grouping(L, T, k, E, torch.device("cuda"))
        gws = torch.empty(max(B.group_workspace_bytes(L, T, k, E), 16), dtype=torch.uint8, device="cuda")
        cnt = torch.empty((L, 4), dtype=torch.int64, device="cuda")
        return out, ws, grp, gws, cnt

    def run(x, bufs):
        out, ws, grp, gws, cnt = bufs
        B.predict(x, W1, W2, k, out=out, workspace=ws)
        B.group_by_expert(out.idx, E, out=grp, workspace=gws)
        B.score(out.idx, ref, E, out=cnt)

    def snapshot(bufs):
        out, _, grp, _, cnt = bufs
        return [t.clone() for t in (out.idx, out.probs, grp.counts, grp.offsets, grp.token_pos, grp.active, cnt)]

    eager = []
    eb = buffers()
    for x in xs:
        run(x, eb)
        torch.cuda.synchronize()
        eager.append(snapshot(eb))

    x_static = xs[0].clone()
    gb = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(x_static, gb)                                  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(x_static, gb)
    for rep in range(2):
        for i, x in enumerate(xs):
            x_static.copy_(x)
            run(xs[(i + 1) % 3], eb)                       # eager work in between, on other buffers
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, want in zip(snapshot(gb), eager[i]):
                assert torch.equal(got, want), (rep, i)
