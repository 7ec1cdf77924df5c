"""GPU parity of deltakv_compress_mlp (non-linear compressor, section 4.1; gated variant, section 5.3) against the
CPU oracle: reference ordinals as for the linear compressor, latents f_c(token) - f_c(reference) within one bf16 ulp
plus the fp32 evaluation error bound derived below, references copied exactly; then decode attention over the cache
the kernel wrote against the oracle's reconstruct-then-attend."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _bf16_ulp(x):
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def _oracle_mlp(M, kind):
    from oracle import deltakv_oracle as O
    m = {"kind": O.SWIGLU if kind == 1 else O.GELU, "w1": M["w1_f64"], "b1": M["b1_f32"].astype(np.float64),
         "w2": M["w2_f64"]}
    if kind == 1:
        m["wg"] = M["wg_f64"]
    return m


def _eval_bound(x_t, x_r, m):
    """Bound on the error of a latent evaluated in fp32 with bf16 hi+lo activations: every hidden unit j contributes
    at most 2^-21 (1 + |u_t| + |u_r|)(1 + |g_t| + |g_r|) |W2[j, c]| (pre-activations and activations carry a few
    fp32 ulps each, the split of the difference 2^-16 of itself, the accumulation 2^-24 per term)."""
    u_t, u_r = np.abs(x_t @ m["w1"] + m["b1"]), np.abs(x_r @ m["w1"] + m["b1"])
    s = 1.0 + u_t + u_r
    if "wg" in m:
        s = s * (1.0 + np.abs(x_t @ m["wg"]) + np.abs(x_r @ m["wg"]))
    return 2.0 ** -21 * (s @ np.abs(m["w2"]))


def _setup(seed, lens_before, lens_new, kind, hidden, Hkv=2, r=64, s=16, n_proto=16, perm=None, l2=False):
    import torch
    import paper_2602_08005_amd as dk
    from paper_2602_08005_amd import binding as B
    from synthetic import generator as G
    from tests.helpers import dev_bits
    nb = len(lens_new)
    total = [a + b for a, b in zip(lens_before, lens_new)]
    max_len = max(max(total), 1)
    pps, rps = -(-max_len // 16), -(-max_len // s)
    n_pages, n_slots = nb * pps + 3, nb * rps + 3
    page_ids = ref_slots = None
    if perm is not None:
        pp, rp = G.page_permutation(perm, nb * pps, n_pages), G.page_permutation(perm + 1, nb * rps, n_slots)
        page_ids = [pp[b * pps:(b + 1) * pps] for b in range(nb)]
        ref_slots = [rp[b * rps:(b + 1) * rps] for b in range(nb)]
    dims = dk.make_dims(Hkv, 4 * Hkv, r, n_pages, n_slots, ref_stride=s, latent_mode=dk.JOINT,
                        metric=dk.METRIC_L2 if l2 else dk.METRIC_COSINE)
    cache = dk.PagedCache(dims, nb, max(sum(lens_new), sum(lens_before), 1), max_len, page_ids=page_ids,
                          ref_slots=ref_slots)
    cache.latent_pool.fill_(0x7FC0)
    cache.idx_pool.fill_(-7)
    M = G.make_mlp_compressor(seed, 128, r, hidden, swiglu=kind == 1)
    KV = [G.make_kv(seed + 31 * b, max(total[b], 1), Hkv, 128, n_proto=n_proto)[:2] for b in range(nb)]
    w1, w2 = dev_bits(M["w1_bf16"]), dev_bits(M["w2_bf16"])
    wg = dev_bits(M["wg_bf16"]) if kind == 1 else None
    b1 = torch.from_numpy(M["b1_f32"]).cuda()
    for starts, counts in (([0] * nb, lens_before), (lens_before, lens_new)):
        if sum(counts) == 0:
            continue
        kn = np.concatenate([KV[b][0][starts[b]:starts[b] + counts[b]] for b in range(nb)])
        vn = np.concatenate([KV[b][1][starts[b]:starts[b] + counts[b]] for b in range(nb)])
        cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        print("compress_mlp", seed, kind, hidden, r, Hkv, counts, flush=True)
        cache.compress_mlp(kind, w1, wg, b1, w2, dev_bits(kn), dev_bits(vn), cu, np.asarray(starts, dtype=np.int32))
    torch.cuda.synchronize()
    return cache, KV, M, total


def _verify(cache, KV, M, total, kind, s=16, l2=False):
    from oracle import deltakv_oracle as O
    f = O.bf16_bits_to_f64
    m = _oracle_mlp(M, kind)
    out = []
    for b, L in enumerate(total):
        if L == 0:
            out.append(None)
            continue
        idx, zk, _ = cache.get_sequence(b, 0, L)
        K, V = KV[b][0][:L], KV[b][1][:L]
        Kf, Vf = f(K), f(V)
        ref = O.compress(Kf, Vf, None, None, s=s, mode=O.JOINT, mlp=m, metric=O.L2 if l2 else O.COSINE)
        out.append(ref)
        diff = np.argwhere(idx != ref["idx"])
        assert len(diff) <= max(2, L // 500), len(diff)
        for (i, h) in diff:                   # near-ties of the oracle's own scores only
            assert 0 <= idx[i, h] and idx[i, h] * s < i and not l2
            assert O.cosine_of(Kf, Vf, i, h, int(idx[i, h]), s) >= ref["cos"][i, h] - 1e-6
        x_t = np.concatenate([Kf, Vf], axis=2)                                    # [L, H, 256]
        hh = np.arange(Kf.shape[1])[None, :]
        x_r = x_t[np.clip(idx, 0, None) * s, hh]
        want = O.mlp_compressor(x_t, m) - O.mlp_compressor(x_r, m)
        want[::s] = 0.0
        same = idx == ref["idx"]
        assert np.max(np.abs(want[same] - ref["z_k"][same])) < 1e-12
        got = f(zk)
        tol = _bf16_ulp(want) + _eval_bound(x_t, x_r, m)
        bad = np.abs(got - O.f64_round_to_bf16(want)) > tol
        assert not bad.any(), (np.argwhere(bad)[:5], got[bad][:5], want[bad][:5])
        assert np.mean(got == O.f64_round_to_bf16(want)) > 0.97
        assert np.all(got[::s] == 0)
        n_ref = -(-L // s)
        rk, rv, _ = cache.get_refs(b, n_ref)
        assert np.array_equal(rk, K[::s]) and np.array_equal(rv, V[::s])
    return out


@pytest.mark.parametrize("kind,hidden,r,Hkv", [(0, 256, 64, 2), (1, 256, 64, 2), (0, 64, 16, 1), (1, 200, 48, 3),
                                               (0, 1000, 128, 2), (1, 512, 32, 9)])
def test_prefill_matches_oracle(kind, hidden, r, Hkv):
    """Hidden widths that are and are not multiples of the staged chunk; more kv-heads than a block has waves."""
    cache, KV, M, total = _setup(3100 + hidden + r, [0, 0, 0], [1500, 17, 1], kind, hidden, Hkv=Hkv, r=r)
    _verify(cache, KV, M, total, kind)


@pytest.mark.parametrize("kind", [0, 1])
def test_chunked_prefill_single_token_appends_and_scattered_pages(kind):
    cache, KV, M, total = _setup(3200 + kind, [700, 0, 33], [500, 40, 1], kind, 256, perm=9)
    _verify(cache, KV, M, total, kind)
    # one token for every sequence (the call shape the linear compressor has a short path for)
    cache, KV, M, total = _setup(3210 + kind, [100, 16, 31], [1, 1, 1], kind, 128, r=32)
    _verify(cache, KV, M, total, kind)


def test_squared_distance_retrieval_with_the_gated_compressor():
    cache, KV, M, total = _setup(3300, [0, 300], [900, 300], 1, 256, l2=True)
    _verify(cache, KV, M, total, 1, l2=True)


def test_unsupported_modes_and_bad_arguments_are_refused():
    import torch
    import paper_2602_08005_amd as dk
    from paper_2602_08005_amd import binding as B
    from synthetic import generator as G
    from tests.helpers import dev_bits
    M = G.make_mlp_compressor(1, 128, 64, 64)
    w1, w2, b1 = dev_bits(M["w1_bf16"]), dev_bits(M["w2_bf16"]), torch.from_numpy(M["b1_f32"]).cuda()
    kn = dev_bits(np.zeros((16, 2, 128), dtype=np.uint16))
    for kw in (dict(latent_mode=dk.SPLIT), dict(latent_mode=dk.JOINT, top_k=2), dict(latent_mode=dk.JOINT, latent_bits=4)):
        dims = dk.make_dims(2, 8, 64, 8, 8, **kw)
        cache = dk.PagedCache(dims, 1, 16, 16)
        cu, lb = np.array([0, 16], dtype=np.int32), np.array([0], dtype=np.int32)
        args = (cache.dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.ref_inv_norm,
                cache.block_tables, cache.ref_tables)
        tail = (kn, kn, torch.from_numpy(cu).cuda(), cu, torch.from_numpy(lb).cuda(), lb, cache.compress_ws)
        assert B.compress_mlp(*args, 0, w1, None, b1, w2, *tail, check=False) == B.E_UNSUPPORTED
    dims = dk.make_dims(2, 8, 64, 8, 8, latent_mode=dk.JOINT)
    cache = dk.PagedCache(dims, 1, 16, 16)
    args = (cache.dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.ref_inv_norm,
            cache.block_tables, cache.ref_tables)
    assert B.compress_mlp(*args, 1, w1, None, b1, w2, *tail, check=False) == B.E_INVALID_ARG    # gated without Wg
    assert B.compress_mlp(*args, 7, w1, None, b1, w2, *tail, check=False) == B.E_INVALID_ARG
    assert B.compress_mlp(*args, 0, w1, None, b1, w2, *tail, check=False) == B.OK


@pytest.mark.parametrize("kind", [0, 1])
def test_compress_then_decode_end_to_end(kind):
    """Attention over the cache the non-linear compressor wrote, against the oracle's reconstruct-then-attend on the
    oracle's own latents (linear decoder, section 4.1)."""
    import torch
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import dev_bits, out_f64, check_attention
    lens = [2000, 333]
    cache, KV, M, total = _setup(3400 + kind, [0, 0], lens, kind, 256, Hkv=2, r=64, n_proto=32)
    refs = _verify(cache, KV, M, total, kind)
    W = G.make_projections(3400, 128, 64, joint=True)
    f = O.bf16_bits_to_f64
    q_bits = G.make_queries(77, len(lens), 8, 128)
    scale = 1.0 / np.sqrt(128)
    out = cache.decode_attn(dev_bits(W["w_up_k_bf16"]), dev_bits(W["w_up_v_bf16"]), dev_bits(q_bits),
                            np.asarray(lens, dtype=np.int32), scale)
    torch.cuda.synchronize()
    got = out_f64(out)
    for b, L in enumerate(lens):
        idx, zk, _ = cache.get_sequence(b, 0, L)
        # the oracle attends over the latents as stored (bit-identical to its own for all but rounding-boundary cases)
        want, _ = O.decode_attn_direct(f(q_bits[b]), idx, f(zk), f(zk), refs[b]["ref_k"], refs[b]["ref_v"],
                                f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), scale)
        check_attention(got[b], want, what=f"mlp kind {kind} seq {b}")
