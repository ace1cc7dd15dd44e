"""The device calls are asynchronous on the caller's stream, allocate nothing and keep no state:
they must behave the same on a side stream, under graph capture (replayed several times with the
program's own work in between) and with two calls in flight on two streams."""
import numpy as np
import pytest
import torch

from paper_2403_20137_amd import kvbfp, synth

pytestmark = pytest.mark.gpu

D, N, P, HKV, G, S = 128, 32, 4, 2, 4, 900


def _inputs(seed, dtype=torch.bfloat16, B=2):
    gains = synth.outlier_gains(seed, 0, HKV, D)
    k = synth.kv_rows(B, S, HKV, D, "bf16", gains, seed, 2, "cuda")
    v = synth.kv_rows(B, S, HKV, D, "bf16", gains, seed, 3, "cuda")
    q = synth.queries(B, HKV * G, D, "bf16", seed, 4, "cuda")
    return k, v, q


def _eager(k, v, q, cache=None, stream=None):
    B = k.shape[0]
    layout = kvbfp.make_layout(D, N, P, HKV, B, S)
    cache = cache or kvbfp.alloc_cache(layout, "cuda")
    kvbfp.quantize_append(cache, k, v, stream=stream)
    out = kvbfp.decode_attention(cache, q, S, 0.09, stream=stream)
    return cache, out


def test_side_stream_gives_identical_bits():
    k, v, q = _inputs(5)
    _, want = _eager(k, v, q)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        _, got = _eager(k, v, q, stream=side)
    side.synchronize()
    assert torch.equal(got, want)


def test_graph_replays_match_eager():
    k, v, q = _inputs(6)
    layout = kvbfp.make_layout(D, N, P, HKV, 2, S)
    cache = kvbfp.alloc_cache(layout, "cuda")
    need = kvbfp.decode_workspace_bytes(layout, HKV * G, S)
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
    q_in = q.clone()
    out = torch.empty_like(q)
    k_new, v_new = k[:, -1:].contiguous(), v[:, -1:].contiguous()
    kvbfp.quantize_append(cache, k[:, :-1], v[:, :-1])
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=cap):
        kvbfp.quantize_append(cache, k_new, v_new, pos0=S - 1)
        kvbfp.decode_attention(cache, q_in, S, 0.09, out=out, workspace=ws)
    for rep in range(4):
        # the program's own eager work and synchronisation between replays
        qi = synth.queries(2, HKV * G, D, "bf16", 100 + rep, 4, "cuda")
        q_in.copy_(qi)
        scribble = torch.full_like(ws, rep + 1)       # someone else used the workspace meanwhile
        ws.copy_(scribble)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _, want = _eager(k, v, qi)
        torch.cuda.synchronize()
        assert torch.equal(out, want), "replay %d" % rep


def test_two_calls_in_flight_on_two_streams():
    ka, va, qa = _inputs(7)
    kb, vb, qb = _inputs(8)
    _, want_a = _eager(ka, va, qa)
    _, want_b = _eager(kb, vb, qb)
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(3):
        with torch.cuda.stream(sa):
            _, oa = _eager(ka, va, qa, stream=sa)
        with torch.cuda.stream(sb):
            _, ob = _eager(kb, vb, qb, stream=sb)
        outs.append((oa, ob))
    sa.synchronize()
    sb.synchronize()
    for oa, ob in outs:
        assert torch.equal(oa, want_a) and torch.equal(ob, want_b)
