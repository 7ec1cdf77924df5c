"""The library's calls record only kernels (no memset nodes, no allocation), so a caller may capture them into a
HIP graph: a captured append + decode step is replayed several times, with eager work and synchronisation between
the replays, and every replay must reproduce the eager result (to the last bf16 place: the order in which float
atomics add is not fixed)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_captured_append_and_decode_replay_like_the_eager_calls():
    import torch
    from paper_2602_08005_amd import binding as B
    from synthetic import generator as G
    from tests.helpers import Case, dev_bits, out_f64, f64, check_attention
    from tests.test_gpu_decode import _setup
    from oracle import deltakv_oracle as O
    L0 = 1999
    case = Case(9900, [L0 + 1, 700], Hkv=2, Hq=8, r=64, n_proto=16)
    cache = _setup(case)                       # holds both sequences in full (oracle-built)
    W = case.W
    wdk, wdv = dev_bits(W["w_down_k_bf16"]), dev_bits(W["w_down_v_bf16"])
    wuk, wuv = dev_bits(W["w_up_k_bf16"]), dev_bits(W["w_up_v_bf16"])
    scale = 1.0 / np.sqrt(128)
    # the step to capture: append token L0 of sequence 0 (recomputed on the GPU from its raw K, V), then attend
    kn, vn = dev_bits(case.K[0][L0:L0 + 1]), dev_bits(case.V[0][L0:L0 + 1])
    cu = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    lb = torch.tensor([L0], dtype=torch.int32, device="cuda")
    seq = torch.tensor(case.lens, dtype=torch.int32, device="cuda")
    q = dev_bits(case.q).clone()
    out_g, out_e = torch.empty_like(q), torch.empty_like(q)

    def step(out):
        B.compress(cache.dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.ref_inv_norm,
                   cache.block_tables, cache.ref_tables, wdk, wdv, kn, vn, cu, [0, 1], lb, [L0], cache.compress_ws)
        B.decode_attn(cache.dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.block_tables,
                      cache.ref_tables, wuk, wuv, q, seq, case.lens, scale, out, None, cache.decode_ws)

    side = torch.cuda.Stream()                 # warm-up outside the capture (function attributes are set on first use)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(out_e)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(out_g)
    for rep in range(3):
        q.copy_(dev_bits(G.make_queries(9900 + 7 * rep, 2, 8, 128)))
        # eager work between the replays: spoil what the step writes, then the eager step
        i0 = cache._idx_index(0, L0, L0 + 1).ravel()
        cache.idx_pool[torch.from_numpy(i0).cuda()] = -5
        step(out_e)
        torch.cuda.synchronize()
        cache.idx_pool[torch.from_numpy(i0).cuda()] = -5
        out_g.fill_(0x7FC0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, eager = out_f64(out_g), out_f64(out_e)
        # float atomics leave the summation order free: a replay agrees with the eager call to one bf16 ulp, and in
        # all but a few outputs exactly (a stale or dropped graph node would show as a large difference)
        assert np.max(np.abs(got - eager)) <= 2.0 ** -8 * np.maximum(np.abs(eager), 2.0 ** -20).max(), rep
        assert np.mean(got == eager) > 0.99, rep
        idx, _, _ = cache.get_sequence(0, L0, L0 + 1)
        assert np.array_equal(idx, case.res[0]["idx"][L0:L0 + 1])
        qh = f64(q.cpu().numpy().view(np.uint16))
        for b in range(2):
            want, _ = case.oracle_decode(b, scale, q=qh[b])
            check_attention(got[b], want, f"replay {rep}, seq {b}")
