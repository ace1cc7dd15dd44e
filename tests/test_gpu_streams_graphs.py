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


def test_graph_replays_of_the_paged_and_the_rotating_call_match_eager():
    k, v, q = _inputs(9)
    page, per_seq = 128, -(-S // 128)
    rng = np.random.default_rng(9)
    table = torch.as_tensor(rng.permutation(2 * per_seq).reshape(2, per_seq).astype(np.int32), device="cuda")
    pool = kvbfp.alloc_cache(kvbfp.make_layout(D, N, P, HKV, 2 * per_seq, page), "cuda")
    kvbfp.quantize_append_paged(pool, table, k, v)
    cache, _ = _eager(k, v, q)
    theta = (10000.0 ** (-np.arange(D // 2, dtype=np.float64) / (D // 2))).astype(np.float32)
    rp = [torch.from_numpy(x).cuda() for x in kvbfp.permute_rope(theta, np.tile(np.arange(D, dtype=np.int32), (HKV, 1)), 1)]
    ws = torch.empty((kvbfp.decode_workspace_bytes_paged(pool.layout, per_seq, 2, HKV * G, S),), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty((kvbfp.decode_workspace_bytes(cache.layout, HKV * G, S),), dtype=torch.uint8, device="cuda")
    q_in = q.clone()
    out_p, out_r = torch.empty_like(q), torch.empty_like(q)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=cap):
        kvbfp.decode_attention_paged(pool, table, q_in, S, 0.09, out=out_p, workspace=ws)
        kvbfp.decode_attention_rope(cache, q_in, S, 0.09, *rp, out=out_r, workspace=ws2)
    for rep in range(3):
        qi = synth.queries(2, HKV * G, D, "bf16", 200 + rep, 4, "cuda")
        q_in.copy_(qi)
        ws.fill_(rep + 1)
        ws2.fill_(rep + 7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_p = kvbfp.decode_attention(cache, qi, S, 0.09)
        want_r = kvbfp.decode_attention_rope(cache, qi, S, 0.09, *rp)
        torch.cuda.synchronize()
        assert torch.equal(out_p, want_p) and torch.equal(out_r, want_r), "replay %d" % rep
