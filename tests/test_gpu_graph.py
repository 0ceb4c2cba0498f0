"""The per-token path under HIP graph capture: the library allocates nothing, never synchronises and
enqueues on the caller's stream, so a chain of layers can be captured once and replayed.  Replays are
checked against the eager results several times, with eager work and synchronisations in between."""
import pytest
import torch

from paper_2506_23225_amd import api, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("T,n_m", [(1, 4), (40, 4), (200, 4), (40, 16)])
def test_graph_replay_matches_eager(T, n_m):
    """(40 tokens, 16 masks: each layer is two launches of the tiled kernel with a hand-over through the
    workspace, which the caller allocates before the capture.)"""
    h, d, layers = 512, 528, 3
    packs, outs_eager = [], []
    x, W0, M0 = synth.make_inputs(h, d, n_m, T, dtype="bf16", seed=900 + T, device=DEV)
    desc = api.make_desc(T, h, d, n_m, x.dtype)
    down = api.make_desc(T, d, h, 1, x.dtype)
    gen = torch.Generator(device=DEV).manual_seed(1)
    for layer in range(layers):
        _, W, M = synth.make_inputs(h, d, n_m, 1, dtype="bf16", seed=910 + layer, device=DEV)
        Wo = (torch.randn(d, h, generator=gen, device=DEV) * 0.05).to(x.dtype)
        packs.append((api.mglu_pack_weights(desc, W), api.mglu_pack_masks(desc, M), api.mglu_pack_weights(down, Wo)))
    hidden = torch.empty(T, d, dtype=x.dtype, device=DEV)
    acts = [x.clone()] + [torch.empty(T, h, dtype=x.dtype, device=DEV) for _ in range(layers)]
    ws = torch.empty(max(api.mglu_workspace_bytes(desc), 16), dtype=torch.uint8, device=DEV)

    def chain():
        for layer, (Wp, Mp, Wop) in enumerate(packs):
            api.mglu_ffn_forward(desc, acts[layer], Wp, Mp, Wop, hidden=hidden, y=acts[layer + 1], workspace=ws)

    chain()                                   # eager: also the first call of every kernel involved
    torch.cuda.synchronize()
    want = [a.clone() for a in acts[1:]]

    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        chain()                               # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            chain()
    torch.cuda.current_stream().wait_stream(stream)
    for rep in range(4):
        for a in acts[1:]:
            a.fill_(float(rep))               # eager work between replays; the replay must overwrite it
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(acts[1:], want):
            assert torch.equal(got, ref), "replay %d differs from the eager result" % rep
