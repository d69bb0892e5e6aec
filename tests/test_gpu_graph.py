"""The decode step inside a HIP graph: callers that capture their decode loop replay
`chunk_score` -> `chunk_select_attention_decode` (and the three-call form) many times.  The
one-launch kernel keeps arrival counters in its workspace and resets them itself, so every
replay must start from a clean state; nothing in the entry points may allocate, synchronise
or record a memset.  Each replay is checked bit for bit against the same step run eagerly,
with eager work and synchronisations between the replays and changing inputs."""
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def snapshot(layer):
    return [t.clone() for t in (layer.score, layer.sel_idx, layer.sel_count, layer.sel_tokens, layer.out, layer.lse)]


def poison(layer):
    layer.score.fill_(float("nan"))
    layer.out.fill_(float("nan"))
    layer.lse.fill_(float("nan"))
    for buf in (layer.sel_idx, layer.sel_count, layer.sel_tokens):
        buf.fill_(-7)


@pytest.mark.parametrize("separate", [False, True], ids=["one_call", "three_calls"])
@pytest.mark.parametrize("cfg,kw", [("c2", dict(layer=17, n_ctx=16384 + 5, hq=8, hkv=2, token_budget=2048)),
                                    ("c3", dict(layer=9, batch=3, n_ctx=8192 + 100, hq=8, hkv=2, token_budget=1024))],
                         ids=["c2_reduced", "c3_reduced"])
def test_decode_step_replays_from_a_graph(L, cfg, kw, separate):
    case = gen.make_case(cfg, device="cuda", **kw)
    layer = L.DecodeLayer(case.K, case.V, case.chunk_off, case.n_chunks, case.hq, case.k_max, case.max_chunks,
                          case.token_budget)
    replay_against_eager(layer, case, separate)


@pytest.mark.parametrize("separate", [False, True], ids=["one_call", "three_calls"])
def test_compressed_store_step_replays_from_a_graph(L, separate):
    qc = gen.make_quant_case("c4", layer=9, n_ctx=32768 + 77, hq=8, hkv=2, token_budget=2048, device="cuda")
    c = qc.case
    layer = L.DecodeLayer(qc.kblob, qc.vblob, c.chunk_off, c.n_chunks, c.hq, c.k_max, c.max_chunks, c.token_budget,
                          qmeta=qc.qmeta, n_kv_heads=c.hkv, n_ctx=c.n_ctx)
    replay_against_eager(layer, c, separate)


def replay_against_eager(layer, case, separate):
    layer.build_abstract()
    step = layer.step_separate if separate else layer.step
    q = case.q.clone()                      # the graph reads its query from this buffer
    g = torch.Generator(device="cuda").manual_seed(3)
    queries = [case.q.clone()] + [(case.q.float() + 0.3 * torch.randn(case.q.shape, generator=g, device="cuda")).to(case.q.dtype)
                                  for _ in range(3)]

    # eager results for every query
    want = []
    for qi in queries:
        q.copy_(qi)
        poison(layer)
        step(q)
        torch.cuda.synchronize()
        want.append(snapshot(layer))
    assert not torch.equal(want[0][1], want[1][1]) or not torch.equal(want[0][4], want[1][4]), "the queries differ"

    # capture on a side stream (warm-up there first, as capture wants)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(q)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(q)
    torch.cuda.synchronize()

    for rep in range(2):
        for qi, w in zip(queries, want):
            q.copy_(qi)
            poison(layer)                   # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got = snapshot(layer)
            for name, a, b in zip(("score", "sel_idx", "sel_count", "sel_tokens", "out", "lse"), got, w):
                assert torch.equal(a, b), f"{name} differs on replay (pass {rep})"
    # and the eager path still works after the replays (the counters were left at zero)
    q.copy_(queries[2])
    poison(layer)
    step(q)
    torch.cuda.synchronize()
    for a, b in zip(snapshot(layer), want[2]):
        assert torch.equal(a, b)
