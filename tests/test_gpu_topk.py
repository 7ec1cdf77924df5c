"""Top-k retrieval with the mean of the retrieved references (section 4.1): decode attention over caches whose
tokens carry k = 2 or 4 reference ordinals, and the compress kernels' ordinals and latents, against the CPU oracle.
Bars: ordinals identical slot by slot; latents within one bf16 ulp; attention max-abs <= 2e-2, relative L2 <= 1e-2."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("top_k,joint,r,Hkv,Hq", [(4, False, 64, 2, 8), (2, False, 32, 2, 8), (4, True, 64, 2, 8),
                                                   (4, False, 48, 4, 28), (2, True, 128, 1, 4), (4, False, 16, 1, 16)])
def test_decode_over_caches_with_k_ordinal_slots(top_k, joint, r, Hkv, Hq):
    from tests.helpers import Case
    from tests.test_gpu_decode import _setup, _run, _compare
    case = Case(12000 + 10 * top_k + r, [3000, 777, 0, 1601, 1, 15, 17], Hkv=Hkv, Hq=Hq, r=r, n_proto=32, joint=joint,
                top_k=top_k)
    nonref = np.arange(3000) % 16 != 0
    assert case.res[0]["idx"].shape[2] == top_k and (case.res[0]["idx"][nonref][64:, :, top_k - 1] >= 0).all()
    assert (case.res[0]["idx"][1:16, :, 1:] == -1).all()            # one candidate only
    scale = 1.0 / np.sqrt(128)
    for perm in (None, 21):
        cache = _setup(case, page_perm_seed=perm)
        got, lse, status = _run(case, cache, scale)
        assert status == 0
        _compare(case, got, lse, scale)


def test_decode_k4_several_splits_selection_and_rescue():
    from paper_2602_08005_amd import binding as B
    from tests.helpers import Case, f64
    from tests.test_gpu_decode import _setup, _run, _compare
    from tests import test_gpu_subset as TS
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    case = Case(12100, [20000, 5000], Hkv=2, Hq=8, r=64, n_proto=64, top_k=4, metric=O.L2)
    cache = _setup(case)
    scale = 1.0 / np.sqrt(128)
    for splits in (0, 7):
        B.tune("splits", splits)
        try:
            got, lse, status = _run(case, cache, scale)
        finally:
            B.tune("splits", 0)
        assert status == 0
        _compare(case, got, lse, scale)
    rng = np.random.default_rng(2)
    positions = [np.sort(rng.choice(L, L // 4, replace=False)) for L in case.lens]
    got, lse, status = TS._run_subset(case, cache, scale, positions)
    assert status == 0
    TS._compare(case, got, lse, scale, positions)
    # a needle far outside the exponent frame: the rows are recomputed by the rescue branch, mean references included
    r0 = case.res[0]
    kh, _ = O.reconstruct(r0["idx"], f64(r0["zb_k"]), f64(r0["zb_v"]), r0["ref_k"], r0["ref_v"],
                          f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]))
    qn = np.stack([np.stack([12.0 * kh[1234 + 100 * g, g // 4] for g in range(8)]), f64(case.q[1])])
    q_bits = G.f32_to_bf16_bits(qn.astype(np.float32))
    got, lse, status = _run(case, cache, scale, q_bits=q_bits)
    assert status != 0                 # (out of the frame, or so far above its references that the list overflows)
    _compare(case, got, lse, scale, q_f64=f64(q_bits))


def _check_topk(cache, KV, W, total, s, joint, l2, top_k):
    """Ordinals of every slot identical to the oracle's ranking; latents (residual against the mean of the retrieved
    references) within one bf16 ulp of the oracle's and nearly all bit-identical; raw references copied exactly."""
    from oracle import deltakv_oracle as O
    from tests.test_gpu_compress import _bf16_ulp
    f = O.bf16_bits_to_f64
    for b, L in enumerate(total):
        if L == 0:
            continue
        K, V = KV[b][0][:L], KV[b][1][:L]
        ref = O.compress(f(K), f(V), f(W["w_down_k_bf16"]), f(W["w_down_v_bf16"]), s=s, mode=O.JOINT if joint else O.SPLIT,
                         metric=O.L2 if l2 else O.COSINE, top_k=top_k)
        idx, zk, zv = cache.get_sequence(b, 0, L)
        assert idx.shape == ref["idx"].shape == (L, K.shape[1], top_k)
        bad = np.argwhere(idx != ref["idx"])
        assert len(bad) == 0, (len(bad), bad[:5], idx[tuple(bad[0][:2])], ref["idx"][tuple(bad[0][:2])])
        # The kernel forms the mean of up to four raw rows in fp32 (three additions and one product, each rounding to
        # 2^-24 of the mean) before the residual; that moves a latent by up to 2^-22 * sum_d |mean_d| |W_dc| on top of
        # what the single-reference path carries (one bf16 ulp + 1e-6, the bar of the k = 1 tests).
        wk, wv = np.abs(f(W["w_down_k_bf16"])), np.abs(f(W["w_down_v_bf16"]))
        mk = np.abs(O.reference_mean(f(K), ref["idx"], s)) @ wk
        mv = np.abs(O.reference_mean(f(V), ref["idx"], s)) @ wv
        extra = {True: (mk + mv, mk + mv), False: (mk, mv)}[joint]
        for got, want, ex in ((zk, ref["z_k"], extra[0]), (zv, ref["z_v"], extra[1])):
            g = f(got)
            off = np.abs(g - O.f64_round_to_bf16(want)) > _bf16_ulp(want) + 1e-6 + 2.0 ** -22 * ex
            assert not off.any(), (np.argwhere(off)[:5], g[off][:5], want[off][:5])
            assert np.mean(g == O.f64_round_to_bf16(want)) > 0.98
        rk, rv, _ = cache.get_refs(b, -(-L // s))
        assert np.array_equal(rk, K[::s]) and np.array_equal(rv, V[::s])


def _plant(KV):
    """Duplicated references (equal scores: lower ordinal first), an exact copy of a reference, a zero vector."""
    K, V = KV[0]
    K[160], V[160] = K[32], V[32]
    K[320], V[320] = K[32], V[32]
    K[501], V[501] = K[160], V[160]
    K[777], V[777] = 0, 0


@pytest.mark.parametrize("top_k,joint,l2,r,s", [(4, False, True, 64, 16), (2, False, False, 32, 16), (4, True, False, 64, 16),
                                                (4, False, False, 48, 8), (2, True, True, 128, 32)])
def test_compress_topk_prefill_batched_append_and_single_tokens(top_k, joint, l2, r, s):
    import torch
    from tests.helpers import dev_bits
    from tests.test_gpu_compress import _compress_case
    before, new = [1500, 0, 700], [1203, 900, 37]
    cache, KV, W, total = _compress_case(13000 + top_k + r, before, new, Hkv=2, r=r, s=s, joint=joint, n_proto=12, perm=5,
                                         l2=l2, edit=_plant, top_k=top_k, capacity=2800)
    _check_topk(cache, KV, W, total, s, joint, l2, top_k)
    # then one token per sequence, five times (the general path: top-k appends do not take the two-kernel shortcut)
    wk, wv = dev_bits(W["w_down_k_bf16"]), dev_bits(W["w_down_v_bf16"])
    for step in range(5):
        t = [total[b] + step for b in range(3)]
        cache.compress(wk, wv, dev_bits(np.stack([KV[b][0][t[b]] for b in range(3)])),
                       dev_bits(np.stack([KV[b][1][t[b]] for b in range(3)])), [0, 1, 2, 3], t)
    torch.cuda.synchronize()
    _check_topk(cache, KV, W, [x + 5 for x in total], s, joint, l2, top_k)


def test_compress_k4_then_decode_end_to_end_and_one_long_prompt():
    """A 20000-token prompt (several 256-token tiles per block row, eight-wave similarity kernel) compressed with
    k = 4 by the GPU, checked slot by slot, then attended by the GPU over its own cache and compared with the oracle's
    attention over the oracle's cache."""
    import torch
    from oracle import deltakv_oracle as O
    from tests.helpers import dev_bits, out_f64, f64, check_attention
    from tests.test_gpu_compress import _compress_case
    from synthetic import generator as G
    cache, KV, W, total = _compress_case(13100, [0], [20000], Hkv=2, r=64, n_proto=64, top_k=4, l2=True)
    _check_topk(cache, KV, W, total, 16, False, True, 4)
    q = G.make_queries(13100, 1, 8, 128)
    scale = 1.0 / np.sqrt(128)
    out = cache.decode_attn(dev_bits(W["w_up_k_bf16"]), dev_bits(W["w_up_v_bf16"]), dev_bits(q), total, scale)
    assert cache.status() == 0
    K, V = KV[0][0][:20000], KV[0][1][:20000]
    ref = O.compress(f64(K), f64(V), f64(W["w_down_k_bf16"]), f64(W["w_down_v_bf16"]), s=16, metric=O.L2, top_k=4)
    want, _ = O.decode_attn_direct(f64(q[0]), ref["idx"], f64(ref["zb_k"]), f64(ref["zb_v"]), ref["ref_k"], ref["ref_v"],
                                   f64(W["w_up_k_bf16"]), f64(W["w_up_v_bf16"]), scale)
    check_attention(out_f64(out)[0], want, "k = 4 end to end")
