"""GPU parity at the shapes and launch configurations of the named workloads (benchmark configs 2-5), on
sampled outputs the oracle can compute one by one, plus determinism, the status flag and the smoke entry."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _dev(bits):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


@pytest.mark.parametrize("joint,bits", [(False, 16), (True, 16), (False, 4), (True, 4)])
def test_long_context_decode_launch_configuration(joint, bits):
    """Config 3's launch shape: batch 8 x 131072 tokens, 8 kv-heads, 32 q-heads, rank 64 -- the same split count,
    wave count and LDS table size bench.py times.  One sequence is compressed for real; all 8 batch rows map to its
    pages (block tables may alias), each with its own query, and two rows are checked against the oracle."""
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import check_attention
    B, L, Hkv, Hq, r, s = 8, 131072, 8, 32, 64, 16
    dims = dk.make_dims(Hkv, Hq, r, n_pages=L // 16, n_ref_slots=L // s, latent_mode=dk.JOINT if joint else dk.SPLIT,
                        latent_bits=bits)
    ids = [np.arange(L // 16, dtype=np.int32)] * B
    cache = dk.PagedCache(dims, B, L, L, page_ids=ids, ref_slots=ids)
    W = G.make_projections(G.seed_for(3), 128, r, joint=joint)
    K, V, _ = G.make_kv(G.seed_for(3, 0, 0), L, Hkv, 128, n_proto=1024, threads=8)
    cache.compress(_dev(W["w_down_k_bf16"]), _dev(W["w_down_v_bf16"]), _dev(K), _dev(V), [0, L], [0])
    q_bits = G.make_queries(G.seed_for(3), B, Hq, 128)
    lens = [L] * B
    lens[5] = L - 7                      # one ragged row in the batch
    out = cache.decode_attn(_dev(W["w_up_k_bf16"]), _dev(W["w_up_v_bf16"]), _dev(q_bits), lens, 1 / np.sqrt(128))
    torch.cuda.synchronize()
    assert int(cache.decode_ws[:4].view(torch.int32)[0].item()) == 0
    f = O.bf16_bits_to_f64
    if bits == 4:          # the values the GPU's 4-bit records read back as
        idx, c0, s0, z0 = cache.get_sequence_q4(0, 0, L)
        zkf = zvf = f(s0)[..., None] * c0 + f(z0)[..., None]
        if not joint:
            _, c1, s1, z1 = cache.get_sequence_q4(0, 0, L, stream=1)
            zvf = f(s1)[..., None] * c1 + f(z1)[..., None]
    else:
        idx, zk, zv = cache.get_sequence(0, 0, L)
        zkf, zvf = f(zk), f(zv)
    got = f(out.cpu().numpy().view(np.uint16))
    for b in (2, 5):
        Lb = lens[b]
        want, _ = O.decode_attn_direct(f(q_bits[b]), idx[:Lb], zkf[:Lb], zvf[:Lb], f(K[:Lb:s]), f(V[:Lb:s]),
                                       f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), 1 / np.sqrt(128))
        check_attention(got[b], want, f"row {b}")
    # ordinals of a sample of tokens against the oracle's own retrieval (prefill at 131072 tokens)
    Kf, Vf = f(K), f(V)
    rng = np.random.default_rng(0)
    for i in rng.integers(1, L, 24):
        for h in (0, 7):
            if i % s == 0:
                assert idx[i, h] == i // s
                continue
            j, c = O.retrieve_one(np.concatenate([Kf, Vf], axis=2), int(i), h, s)
            if idx[i, h] != j:
                assert O.cosine_of(Kf, Vf, int(i), h, int(idx[i, h]), s) >= c - 1e-6


def test_irregular_paged_batch_matches_oracle_and_contiguous_layout():
    """Config 5's shape at reduced sequence count: lengths log-uniform, 4 kv-heads, 28 q-heads (7:1), rank 48, pages
    scattered over a shared pool; shortest / median / longest sequence against the oracle, and the same data laid
    out contiguously gives the same result."""
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import check_attention
    nseq, Hkv, Hq, r, s = 12, 4, 28, 48, 16
    lens = G.loguniform_lengths(G.seed_for(5, 0, 99), nseq, 4096, 65536)
    lens[3] = 65536
    lens[7] = 4096 + 5
    W = G.make_projections(G.seed_for(5), 128, r)
    q_bits = G.make_queries(G.seed_for(5), nseq, Hq, 128)
    KV = [G.make_kv(G.seed_for(5, 0, b + 1), int(lens[b]), Hkv, 128, n_proto=256, threads=8)[:2] for b in range(nseq)]
    outs = []
    for paged in (True, False):
        pages = [-(-int(x) // 16) for x in lens]
        n_pages = int(sum(pages) * 1.25) if paged else sum(pages)
        cp = np.concatenate([[0], np.cumsum(pages)])
        pp = G.page_permutation(5, sum(pages), n_pages) if paged else np.arange(sum(pages), dtype=np.int32)
        rp = G.page_permutation(6, sum(pages), n_pages) if paged else np.arange(sum(pages), dtype=np.int32)
        dims = dk.make_dims(Hkv, Hq, r, n_pages=n_pages, n_ref_slots=n_pages)
        cache = dk.PagedCache(dims, nseq, int(lens.max()), int(lens.max()),
                              page_ids=[pp[cp[b]:cp[b + 1]] for b in range(nseq)],
                              ref_slots=[rp[cp[b]:cp[b + 1]] for b in range(nseq)])
        for b in range(nseq):
            cache.compress(_dev(W["w_down_k_bf16"]), _dev(W["w_down_v_bf16"]), _dev(KV[b][0]), _dev(KV[b][1]),
                           [0, int(lens[b])], [0], first_seq=b)
        out = cache.decode_attn(_dev(W["w_up_k_bf16"]), _dev(W["w_up_v_bf16"]), _dev(q_bits), lens, 1 / np.sqrt(128))
        torch.cuda.synchronize()
        assert int(cache.decode_ws[:4].view(torch.int32)[0].item()) == 0
        outs.append(O.bf16_bits_to_f64(out.cpu().numpy().view(np.uint16)))
        if paged:
            f = O.bf16_bits_to_f64
            order = np.argsort(lens)
            for b in (int(order[0]), int(order[nseq // 2]), int(order[-1])):
                Lb = int(lens[b])
                idx, zk, zv = cache.get_sequence(b, 0, Lb)
                want, _ = O.decode_attn_direct(f(q_bits[b]), idx, f(zk), f(zv), f(KV[b][0][::s]), f(KV[b][1][::s]),
                                               f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), 1 / np.sqrt(128))
                check_attention(outs[0][b], want, f"sequence {b} ({Lb} tokens)")
    assert np.max(np.abs(outs[0] - outs[1])) <= 2.0 ** -7 * max(1.0, np.max(np.abs(outs[1])))


def test_decode_loop_appending_one_token_per_step():
    """Config 2's loop at reduced length: prefill, then each step appends one compressed token and attends over the
    whole cache; ordinals of every appended token and the outputs of the first, middle and last step are checked."""
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import check_attention
    L0, n, Hkv, Hq, r, s = 4096 + 9, 48, 8, 32, 64, 16
    dims = dk.make_dims(Hkv, Hq, r, n_pages=300, n_ref_slots=300)
    cache = dk.PagedCache(dims, 1, L0, L0 + n)
    W = G.make_projections(G.seed_for(2), 128, r)
    K, V, _ = G.make_kv(G.seed_for(2), L0 + n, Hkv, 128, n_proto=1024)
    q_bits = G.make_queries(G.seed_for(2), n, Hq, 128)
    wdk, wdv, wuk, wuv = (_dev(W[k]) for k in ("w_down_k_bf16", "w_down_v_bf16", "w_up_k_bf16", "w_up_v_bf16"))
    cache.compress(wdk, wdv, _dev(K[:L0]), _dev(V[:L0]), [0, L0], [0])
    outs = []
    for i in range(n):
        t = L0 + i
        cache.compress(wdk, wdv, _dev(K[t:t + 1]), _dev(V[t:t + 1]), [0, 1], [t])
        outs.append(cache.decode_attn(wuk, wuv, _dev(q_bits[i:i + 1]), [t + 1], 1 / np.sqrt(128)).clone())
    torch.cuda.synchronize()
    f = O.bf16_bits_to_f64
    ref = O.compress(f(K), f(V), f(W["w_down_k_bf16"]), f(W["w_down_v_bf16"]), s=s)
    idx, zk, zv = cache.get_sequence(0, 0, L0 + n)
    assert np.array_equal(idx, ref["idx"])
    for i in (0, n // 2, n - 1):
        Lc = L0 + i + 1
        want, _ = O.decode_attn_direct(f(q_bits[i]), ref["idx"][:Lc], f(ref["zb_k"][:Lc]), f(ref["zb_v"][:Lc]),
                                       ref["ref_k"][:-(-Lc // s)], ref["ref_v"][:-(-Lc // s)],
                                       f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), 1 / np.sqrt(128))
        check_attention(f(outs[i].cpu().numpy().view(np.uint16))[0], want, f"step {i}")


def test_prefill_32k_ordinals_and_latents_on_a_sample():
    """Config 4's shape (one 32768-token prompt, 8 kv-heads, rank 64, 1024 prototypes): the last 2048 tokens' ordinals
    and latents against the oracle."""
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.test_gpu_compress import _check_against_oracle
    L, Hkv, r, s = 32768, 8, 64, 16
    dims = dk.make_dims(Hkv, 32, r, n_pages=L // 16, n_ref_slots=L // s)
    cache = dk.PagedCache(dims, 1, L, L)
    W = G.make_projections(G.seed_for(4), 128, r)
    K, V, _ = G.make_kv(G.seed_for(4, 0), L, Hkv, 128, n_proto=1024, threads=8)
    cache.compress(_dev(W["w_down_k_bf16"]), _dev(W["w_down_v_bf16"]), _dev(K), _dev(V), [0, L], [0])
    torch.cuda.synchronize()
    t0 = L - 2048
    idx, zk, zv = cache.get_sequence(0, t0, L)
    _check_against_oracle(K, V, W, s, False, idx, zk, zv, t0=t0)


def test_prefill_32k_two_full_layers_every_ordinal_and_latent():
    """Config 4 at full size: two layers (different inputs) of one 32768-token prompt, every token's ordinal and latent
    against the oracle."""
    import torch
    import paper_2602_08005_amd as dk
    from synthetic import generator as G
    from tests.test_gpu_compress import _check_against_oracle
    L, Hkv, r, s = 32768, 8, 64, 16
    dims = dk.make_dims(Hkv, 32, r, n_pages=L // 16, n_ref_slots=L // s)
    cache = dk.PagedCache(dims, 1, L, L)
    W = G.make_projections(G.seed_for(4), 128, r)
    n_diff = 0
    for layer in (0, 1):
        K, V, _ = G.make_kv(G.seed_for(4, layer), L, Hkv, 128, n_proto=1024, threads=8)
        print("layer", layer, "compress", flush=True)
        cache.compress(_dev(W["w_down_k_bf16"]), _dev(W["w_down_v_bf16"]), _dev(K), _dev(V), [0, L], [0])
        torch.cuda.synchronize()
        idx, zk, zv = cache.get_sequence(0, 0, L)
        print("layer", layer, "oracle", flush=True)
        n_diff += _check_against_oracle(K, V, W, s, False, idx, zk, zv)
    assert n_diff <= 4          # (ordinals that differ are accepted only on ties of the oracle's own scores within 1e-6)


def test_decode_loop_full_size_32k_prompt_256_appended_tokens():
    """Config 2 at full size: a 32768-token prompt, then 256 steps that each append one compressed token and attend
    over the whole cache; every ordinal of prompt and appended tokens, and the outputs of steps 0, 127 and 255."""
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import check_attention
    L0, n, Hkv, Hq, r, s = 32768, 256, 8, 32, 64, 16
    dims = dk.make_dims(Hkv, Hq, r, n_pages=(L0 + n) // 16 + 1, n_ref_slots=(L0 + n) // s + 1)
    cache = dk.PagedCache(dims, 1, L0, L0 + n)
    W = G.make_projections(G.seed_for(2), 128, r)
    K, V, _ = G.make_kv(G.seed_for(2), L0 + n, Hkv, 128, n_proto=1024, threads=8)
    q_bits = G.make_queries(G.seed_for(2), n, Hq, 128)
    wdk, wdv, wuk, wuv = (_dev(W[k]) for k in ("w_down_k_bf16", "w_down_v_bf16", "w_up_k_bf16", "w_up_v_bf16"))
    Kd, Vd, qd = _dev(K), _dev(V), _dev(q_bits)
    cache.compress(wdk, wdv, Kd[:L0], Vd[:L0], [0, L0], [0])
    keep = {}
    for i in range(n):
        t = L0 + i
        cache.compress(wdk, wdv, Kd[t:t + 1], Vd[t:t + 1], [0, 1], [t])
        out = cache.decode_attn(wuk, wuv, qd[i:i + 1], [t + 1], 1 / np.sqrt(128))
        if i in (0, n // 2 - 1, n - 1):
            keep[i] = out.clone()
    torch.cuda.synchronize()
    assert cache.status() == 0
    f = O.bf16_bits_to_f64
    print("oracle", flush=True)
    ref = O.compress(f(K), f(V), f(W["w_down_k_bf16"]), f(W["w_down_v_bf16"]), s=s)
    idx, zk, zv = cache.get_sequence(0, 0, L0 + n)
    diff = np.argwhere(idx != ref["idx"])
    assert len(diff) <= 2, diff[:5]
    for (i, h) in diff:
        assert O.cosine_of(f(K), f(V), i, h, int(idx[i, h]), s) >= ref["cos"][i, h] - 1e-6
    for i, out in keep.items():
        Lc = L0 + i + 1
        # the oracle attends over the cache as the kernels wrote it (its own ordinals and latents but for near-ties)
        want, _ = O.decode_attn_direct(f(q_bits[i]), idx[:Lc], f(zk[:Lc]), f(zv[:Lc]),
                                       ref["ref_k"][:-(-Lc // s)], ref["ref_v"][:-(-Lc // s)],
                                       f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), 1 / np.sqrt(128))
        check_attention(f(out.cpu().numpy().view(np.uint16))[0], want, f"step {i}")


def test_repeated_calls_agree():
    """Two runs over the same cache agree to within one bf16 ulp (float atomics make the summation order free, so
    bit-identity is not guaranteed; a race would show up as a large difference)."""
    import torch
    from tests.helpers import Case, dev_bits, out_f64
    from tests.test_gpu_decode import _setup
    case = Case(8000, [9000, 5000], Hkv=4, Hq=16, r=64, n_proto=32)
    cache = _setup(case, page_perm_seed=3)
    args = (dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q), case.lens, 0.09)
    a = out_f64(cache.decode_attn(*args).clone())
    for _ in range(3):
        b = out_f64(cache.decode_attn(*args).clone())
        assert np.max(np.abs(a - b)) <= 2.0 ** -8 * np.maximum(np.abs(a), 2.0 ** -20).max()
        assert np.mean(a == b) > 0.99


def test_logits_outside_the_exponent_frame_are_recomputed_exactly():
    """A latent far outside anything a bounded residual produces pushes one logit hundreds of units above every
    reference-token logit, beyond what the streaming kernel's fixed exponent frame holds: the affected rows are
    recomputed by the rescue kernel (the status word records that it ran) and match the oracle like any other row;
    rows of the same call that stay inside the frame keep the streaming result.  A normal call afterwards clears
    the word."""
    import torch
    from oracle import deltakv_oracle as O
    from tests.helpers import Case, dev_bits, out_f64, check_attention
    from tests.test_gpu_decode import _setup
    from synthetic import generator as G
    f = O.bf16_bits_to_f64
    case = Case(8100, [600, 900], Hkv=1, Hq=4, r=16, n_proto=8)
    r0 = case.res[0]
    q = G.f32_to_bf16_bits(np.concatenate([np.full((1, 4, 128), 2.0), 0.1 * np.ones((1, 4, 128))]).astype(np.float32))
    qlat = f(case.W["w_up_k_bf16"]) @ f(q[0, 0])                  # direction in which a latent raises the logit
    zk_orig = r0["zb_k"]
    zk = zk_orig.copy()
    zk[333, 0, :] = G.f32_to_bf16_bits((300.0 * qlat / np.linalg.norm(qlat)).astype(np.float32))
    r0["zb_k"] = zk
    logits = f(zk[:, 0, :]) @ qlat + r0["ref_k"][r0["idx"][:, 0], 0] @ f(q[0, 0])
    ref_logits = r0["ref_k"][:, 0] @ f(q[0, 0])
    assert (logits.max() - ref_logits.max()) * 1.4427 > 200     # far past the 2^124 range of the biased exponent
    cache = _setup(case)
    lse = torch.zeros((2, 4), dtype=torch.float32, device="cuda")
    out = cache.decode_attn(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(q), case.lens, 1.0,
                            lse=lse)
    torch.cuda.synchronize()
    assert int(cache.decode_ws[:4].view(torch.int32)[0].item()) == 1
    got = out_f64(out)
    for b in range(2):
        want, wl = case.oracle_decode(b, 1.0, f(q[b]))
        check_attention(got[b], want, f"seq {b}", scale_with_magnitude=True)
        assert np.max(np.abs(lse[b].cpu().numpy() - wl)) <= 2e-2 * max(1.0, float(np.max(np.abs(wl))) / 64)
    cache.put_sequence(0, r0["idx"], zk_orig, r0["zb_v"], None, None)
    cache.decode_attn(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q), case.lens, 0.01)
    torch.cuda.synchronize()
    assert int(cache.decode_ws[:4].view(torch.int32)[0].item()) == 0


def test_smoke_entry_point():
    import __graft_entry__ as g
    g.smoke()


def test_longest_on_chip_table_and_the_first_sequence_beyond_it():
    """The per-reference weight table of a 160000-token sequence (10000 references x 4 query heads, rank 64) is the
    largest that still fits one CU's LDS; at 161000 tokens the oldest ordinals go to the table in global memory.
    The cache is built by the GPU's compress; attention is checked against the oracle for both whole sequences."""
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import check_attention
    L, Lbig, Hkv, Hq, r, s = 160000, 161000, 1, 4, 64, 16
    dims = dk.make_dims(Hkv, Hq, r, n_pages=-(-Lbig // 16), n_ref_slots=-(-Lbig // s))
    cache = dk.PagedCache(dims, 1, Lbig, Lbig)
    W = G.make_projections(77, 128, r)
    K, V, _ = G.make_kv(78, Lbig, Hkv, 128, n_proto=512, threads=8)
    cache.compress(_dev(W["w_down_k_bf16"]), _dev(W["w_down_v_bf16"]), _dev(K), _dev(V), [0, Lbig], [0])
    q_bits = G.make_queries(79, 1, Hq, 128)
    wuk, wuv, q = _dev(W["w_up_k_bf16"]), _dev(W["w_up_v_bf16"]), _dev(q_bits)
    f = O.bf16_bits_to_f64
    idx, zk, zv = cache.get_sequence(0, 0, Lbig)
    for n in (L, Lbig):
        out = cache.decode_attn(wuk, wuv, q, [n], 1 / np.sqrt(128))
        assert cache.status() == 0
        want, _ = O.decode_attn_direct(f(q_bits[0]), idx[:n], f(zk[:n]), f(zv[:n]), f(K[:n:s]), f(V[:n:s]),
                                       f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), 1 / np.sqrt(128))
        check_attention(f(out.cpu().numpy().view(np.uint16))[0], want, f"{n} tokens")
