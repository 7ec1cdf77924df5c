"""Pins for the CPU oracle: values the paper prints, closed forms, invariants,
special cases that reduce to textbook / library routines, and brute force on
tiny inputs.  None of these use the HIP path."""
import math
import os

import numpy as np
import pytest

from oracle import deltakv_oracle as O
from synthetic import generator as G

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append([float(x) for x in line.split()])
    return out


def _f64(bits):
    return O.bf16_bits_to_f64(bits)


def _small_case(seed=1, L=96, H=2, D=16, r=8, s=4, n_proto=6, joint=False):
    K, V, cls = G.make_kv(seed, L, H, D, n_proto=n_proto, basis_dim=4)
    P = G.make_projections(seed, D, r, joint=joint, recipe="paired")
    return _f64(K), _f64(V), cls, P


# ---------------------------------------------------------------- P1: paper's printed values
@pytest.mark.parametrize("row", _rows("kr_worked_rows.txt"))
def test_keep_ratio_matches_paper_rows(row):
    n_full, n_layers, s, dc, bits, want, tol = row
    got = 100.0 * O.keep_ratio_eq5(int(n_full), int(n_layers), int(s), dc, latent_bits=int(bits))
    assert abs(got - want) <= tol, (got, want)


def test_compute_ratio_equation_closed_forms():
    """Equation (6): no dense layers -> the budget itself (the figure the appendix's table prints, 30.0 / 20.0);
    all layers dense -> 100 %; budget 1 -> 100 %; linear in the budget; and the table's two layer splits by hand."""
    assert O.compute_ratio_eq6(0, 32, 0.3) == pytest.approx(0.3) and O.compute_ratio_eq6(0, 32, 0.2) == pytest.approx(0.2)
    assert O.compute_ratio_eq6(32, 32, 0.3) == 1.0 and O.compute_ratio_eq6(5, 32, 1.0) == pytest.approx(1.0)
    assert O.compute_ratio_eq6(5, 32, 0.3) == pytest.approx(5 / 32 + 27 / 32 * 0.3)        # 40.9 %
    assert O.compute_ratio_eq6(4, 32, 0.2) == pytest.approx(0.125 + 0.875 * 0.2)            # 30.0 %
    a, b, c = (O.compute_ratio_eq6(5, 32, x) for x in (0.1, 0.2, 0.3))
    assert (b - a) == pytest.approx(c - b)


def test_dense_kv_size_statement():
    b, L, nl, hkv, d, bpv, lo, hi = _rows("dense_kv_size.txt")[0]
    gb = O.dense_kv_bytes(int(b), int(L), int(nl), int(hkv), int(d), int(bpv)) / 1e9
    assert lo < gb < hi
    assert abs(gb - 137.438953472) < 1e-6


def test_record_keep_ratio_closed_forms():
    # SPLIT r=64, D=128, s=16, int32 idx: (256 + 4 + 32)/512 ; JOINT: (128 + 4 + 32)/512
    assert O.record_keep_ratio(O.SPLIT, 64, 128, 16) == pytest.approx(292 / 512)
    assert O.record_keep_ratio(O.JOINT, 64, 128, 16) == pytest.approx(164 / 512)
    # without the index and with s=10, JOINT d_c/2d_k = 0.25 reproduces equation (5)'s bracket
    assert O.record_keep_ratio(O.JOINT, 64, 128, 10, idx_bytes=0) == pytest.approx(0.35)


# ---------------------------------------------------------------- bf16 rounding
def test_bf16_round_ties_to_even_and_matches_library_on_fp32_inputs():
    import torch
    # exact ties: 1 + 2^-8 is halfway between 1 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert O.f64_round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.f64_round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.f64_round_to_bf16(np.array([-(1.0 + 2.0 ** -8 + 2.0 ** -40)]))[0] == -(1.0 + 2.0 ** -7)
    # a value where rounding first to fp32 and then to bf16 gives the wrong answer
    x = 1.0 + 2.0 ** -8 + 2.0 ** -30          # fp32 rounds it to the tie, bf16 then to 1.0
    assert O.f64_round_to_bf16(np.array([x]))[0] == 1.0 + 2.0 ** -7
    rng = np.random.default_rng(0)
    v = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.f64_round_to_bf16(v.astype(np.float64))
    assert np.array_equal(got, want)
    bits = O.f64_to_bf16_bits(v.astype(np.float64))
    assert np.array_equal(O.bf16_bits_to_f64(bits), want)
    # subnormal bf16 and zero
    assert O.f64_round_to_bf16(np.array([2.0 ** -133, 2.0 ** -135, 0.0, -0.0])).tolist() == [2.0 ** -133, 0.0, 0.0, 0.0]


# ---------------------------------------------------------------- P2: brute-force retrieval
def _brute_retrieve(K, V, i, h, s):
    """Plain loops, strict '>' over ascending ordinals."""
    a = list(K[i, h]) + list(V[i, h])
    na = math.sqrt(math.fsum(x * x for x in a))
    best, bj = -math.inf, -1
    j = 0
    while j * s < i:
        b = list(K[j * s, h]) + list(V[j * s, h])
        nb = math.sqrt(math.fsum(x * x for x in b))
        c = 0.0 if (na == 0.0 or nb == 0.0) else math.fsum(x * y for x, y in zip(a, b)) / (na * nb)
        if c > best:
            best, bj = c, j
        j += 1
    return bj, best


def test_retrieval_equals_brute_force_with_ties():
    K, V, cls, P = _small_case(seed=3, L=70, H=2, D=8, r=4, s=4)
    # exact ties: make references 3 and 9 bit-identical copies of reference 1, and token 50 a scaled copy
    for j in (3, 9):
        K[j * 4], V[j * 4] = K[4].copy(), V[4].copy()
    K[50], V[50] = 2.0 * K[4], 2.0 * V[4]
    # a zero-norm token and a zero-norm reference
    K[33], V[33] = 0.0, 0.0
    K[8, 1], V[8, 1] = 0.0, 0.0
    res = O.compress(K, V, _f64(P["w_down_k_bf16"]), _f64(P["w_down_v_bf16"]), s=4)
    for i in range(70):
        for h in range(2):
            if i % 4 == 0:
                assert res["idx"][i, h] == i // 4
                continue
            bj, bc = _brute_retrieve(K, V, i, h, 4)
            oj = int(res["idx"][i, h])
            if oj != bj:   # only allowed when the two scores differ by rounding noise
                assert abs(O.cosine_of(K, V, i, h, oj, 4) - bc) < 1e-14 and False, (i, h, oj, bj)
            assert abs(res["cos"][i, h] - bc) < 1e-13
    assert res["idx"][50, 0] == 1 and res["idx"][50, 1] == 1          # lowest of the tied 1, 3, 9
    assert res["idx"][33, 0] == 0                                       # all scores 0 -> ordinal 0


def test_candidates_are_strictly_earlier():
    # token i may use ordinal j only if j*s < i: the token right after a reference can see it,
    # a reference never sees itself as a candidate, and nothing looks forward.
    assert [O.n_candidates(i, 4) for i in (1, 4, 5, 8, 9)] == [1, 1, 2, 2, 3]
    K, V, cls, P = _small_case(seed=5, L=40, H=1, D=8, r=4, s=4)
    K[21], V[21] = K[24].copy(), V[24].copy()      # identical to a LATER reference (ordinal 6)
    res = O.compress(K, V, _f64(P["w_down_k_bf16"]), _f64(P["w_down_v_bf16"]), s=4)
    assert res["idx"][21, 0] < 6
    assert np.all(res["idx"][:, 0] * 4 <= np.arange(40))


def test_near_ties_resolved_in_float64():
    rng = np.random.default_rng(7)
    L, s, D = 14, 4, 8
    K = rng.standard_normal((L, 1, D))
    V = rng.standard_normal((L, 1, D))
    base = np.concatenate([K[13, 0], V[13, 0]])
    for eps, winner in ((1e-7, 2), (1e-5, 2)):
        # ordinal 1 = base + small orthogonal perturbation (cos slightly < 1), ordinal 2 = exact direction
        pert = rng.standard_normal(2 * D)
        pert -= pert @ base / (base @ base) * base
        pert *= math.sqrt(2 * eps) * np.linalg.norm(base) / np.linalg.norm(pert)
        v1 = base + pert
        K[4, 0], V[4, 0] = v1[:D], v1[D:]
        K[8, 0], V[8, 0] = 3.0 * base[:D], 3.0 * base[D:]
        res = O.compress(K, V, np.eye(D)[:, :4], np.eye(D)[:, :4], s=s)
        assert res["idx"][13, 0] == winner
        c1 = O.cosine_of(K, V, 13, 0, 1, s)
        assert 0.2 * eps < 1.0 - c1 < 5 * eps


# ---------------------------------------------------------------- P3 / P12
def test_planted_copy_and_reference_round_trip():
    K, V, cls, P = _small_case(seed=11, L=64, H=2, D=16, r=8, s=4)
    K[37], V[37] = K[20].copy(), V[20].copy()            # token 37 := reference ordinal 5
    wd = _f64(P["w_down_k_bf16"])
    res = O.compress(K, V, wd, wd, s=4)
    assert np.all(res["idx"][37] == 5)
    assert np.allclose(res["cos"][37], 1.0, atol=1e-15)
    assert np.all(res["z_k"][37] == 0) and np.all(res["z_v"][37] == 0)
    ref_tok = np.arange(0, 64, 4)
    assert np.array_equal(res["idx"][ref_tok], np.repeat((ref_tok // 4)[:, None], 2, 1))
    assert np.all(res["z_k"][ref_tok] == 0) and np.all(res["zb_v"][ref_tok] == 0)
    assert np.array_equal(res["ref_k"], K[0::4]) and np.array_equal(res["ref_v"], V[0::4])
    wu = wd.T
    kh, vh = O.reconstruct(res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"], wu, wu)
    assert np.array_equal(kh[ref_tok], K[ref_tok]) and np.array_equal(vh[ref_tok], V[ref_tok])


# ---------------------------------------------------------------- P4: full-rank orthonormal
@pytest.mark.parametrize("joint", [False, True])
def test_full_rank_orthonormal_reconstructs_exactly(joint):
    D = 16
    r = 2 * D if joint else D
    K, V, cls, _ = _small_case(seed=13, L=80, H=2, D=D, r=8, s=4)
    P = G.make_projections(99, D, r, joint=joint, recipe="paired")   # distinct per stream: swapping them is caught
    assert joint or np.max(np.abs(P["w_down_k_f64"] - P["w_down_v_f64"])) > 0.1
    mode = O.JOINT if joint else O.SPLIT
    res = O.compress(K, V, P["w_down_k_f64"], P["w_down_v_f64"], s=4, mode=mode)
    kh, vh = O.reconstruct(res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"],
                           P["w_up_k_f64"], P["w_up_v_f64"])
    assert np.max(np.abs(kh - K)) < 1e-12 and np.max(np.abs(vh - V)) < 1e-12


def test_signed_permutation_projection_error_is_latent_rounding_only():
    D = 16
    K, V, cls, _ = _small_case(seed=17, L=80, H=2, D=D, r=8, s=4)
    rng = np.random.default_rng(1)
    W = np.zeros((D, D))
    W[np.arange(D), rng.permutation(D)] = rng.choice([-1.0, 1.0], D)
    res = O.compress(K, V, W, W, s=4)
    zk = O.bf16_bits_to_f64(res["zb_k"])
    zv = O.bf16_bits_to_f64(res["zb_v"])
    kh, vh = O.reconstruct(res["idx"], zk, zv, res["ref_k"], res["ref_v"], W.T, W.T)
    hh = np.arange(2)[None, :]
    rk = K - res["ref_k"][res["idx"], hh]
    # the reconstruction error is exactly the bf16 rounding error of each residual component
    assert np.array_equal(kh - res["ref_k"][res["idx"], hh], O.f64_round_to_bf16(rk @ W) @ W.T)
    assert np.max(np.abs(kh - K)) <= 2.0 ** -8 * np.max(np.abs(rk))   # half an ulp is below 2^-8 |x|
    assert np.max(np.abs(kh - K)) > 0


# ---------------------------------------------------------------- P11: subspace case
def test_subspace_residual_is_captured_exactly():
    # tokens = prototype + B c with no noise; if span(W_d) contains span(B) and the retrieved
    # reference has the same prototype, the rank-r latent reconstructs the token exactly.
    rng = np.random.default_rng(5)
    D, rb, r, s, L = 16, 3, 6, 4, 64
    Bm = G.orthonormal(rng, D, rb)
    extra = G.orthonormal(rng, D, D)
    Wd = np.linalg.qr(np.concatenate([Bm, extra[:, : r - rb]], axis=1))[0]      # spans B
    proto = 10.0 * rng.standard_normal((3, 2, D))
    cls = rng.integers(0, 3, L)
    cls[:12:4] = [0, 1, 2]                                  # each class has an early reference
    K = proto[cls, 0][:, None, :] + (rng.standard_normal((L, 1, rb)) @ Bm.T)
    V = proto[cls, 1][:, None, :] + (rng.standard_normal((L, 1, rb)) @ Bm.T)
    res = O.compress(K, V, Wd, Wd, s=s)
    late = np.arange(12, L)
    assert np.array_equal(cls[res["idx"][late, 0] * s], cls[late])     # same-prototype reference
    kh, vh = O.reconstruct(res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"], Wd.T, Wd.T)
    assert np.max(np.abs(kh[late] - K[late])) < 1e-12
    assert np.max(np.abs(vh[late] - V[late])) < 1e-12
    # and a projection that misses B does NOT reconstruct (the check can fail)
    Wbad = np.linalg.qr(extra[:, :r] - Bm @ (Bm.T @ extra[:, :r]))[0]
    res2 = O.compress(K, V, Wbad, Wbad, s=s)
    kh2, _ = O.reconstruct(res2["idx"], res2["z_k"], res2["z_v"], res2["ref_k"], res2["ref_v"], Wbad.T, Wbad.T)
    assert np.max(np.abs(kh2[late] - K[late])) > 1e-2


# ---------------------------------------------------------------- P10: idempotence
def test_projection_idempotence():
    K, V, cls, P = _small_case(seed=19, L=96, H=2, D=16, r=8, s=4)
    wd, wu = P["w_down_k_f64"], P["w_up_k_f64"]
    res = O.compress(K, V, wd, wd, s=4)
    kh, vh = O.reconstruct(res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"], wu, wu)
    hh = np.arange(2)[None, :]
    z2 = (kh - res["ref_k"][res["idx"], hh]) @ wd
    assert np.max(np.abs(z2 - res["z_k"])) < 1e-12


# ---------------------------------------------------------------- decode pins
def _decode_case(seed=23, L=90, Hkv=2, Gq=3, D=16, r=8, s=4, joint=False):
    K, V, cls, P = _small_case(seed=seed, L=L, H=Hkv, D=D, r=r, s=s, joint=joint)
    mode = O.JOINT if joint else O.SPLIT
    res = O.compress(K, V, _f64(P["w_down_k_bf16"]), _f64(P["w_down_v_bf16"]), s=s, mode=mode)
    q = _f64(G.make_queries(seed, 1, Hkv * Gq, D))[0]
    zk, zv = _f64(res["zb_k"]), _f64(res["zb_v"])
    wuk, wuv = _f64(P["w_up_k_bf16"]), _f64(P["w_up_v_bf16"])
    return K, V, res, q, zk, zv, wuk, wuv


def _torch_sdpa(q, K, V, scale):
    import torch
    import torch.nn.functional as F
    Hq = q.shape[0]
    Hkv = K.shape[1]
    qt = torch.from_numpy(q)[None, :, None, :]                                  # [1,Hq,1,D]
    kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)[None]
    vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)[None]
    return F.scaled_dot_product_attention(qt, kt, vt, scale=scale)[0, :, 0, :].numpy()


def test_stride_one_is_textbook_attention_vs_library():            # P6
    K, V, cls, P = _small_case(seed=29, L=50, H=2, D=16, r=8, s=1)
    wd = _f64(P["w_down_k_bf16"])
    res = O.compress(K, V, wd, wd, s=1)
    assert np.array_equal(res["idx"][:, 0], np.arange(50)) and np.all(res["z_k"] == 0)
    q = _f64(G.make_queries(29, 1, 6, 16))[0]
    scale = 0.37
    out, lse = O.decode_attn_direct(q, res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"],
                                    wd.T, wd.T, scale)
    want = _torch_sdpa(q, K, V, scale)
    assert np.max(np.abs(out - want)) < 1e-12
    # lse against scipy's logsumexp of the plain logits, GQA head map g -> g // 3
    from scipy.special import logsumexp
    for g in range(6):
        assert abs(lse[g] - logsumexp(scale * (K[:, g // 3] @ q[g]))) < 1e-12


def test_zero_residual_equals_dense_attention_over_gathered_references():   # P5
    K, V, res, q, zk, zv, wuk, wuv = _decode_case()
    z0 = np.zeros_like(zk)
    out, lse = O.decode_attn_direct(q, res["idx"], z0, z0, res["ref_k"], res["ref_v"], wuk, wuv, 0.25)
    hh = np.arange(2)[None, :]
    want = _torch_sdpa(q, res["ref_k"][res["idx"], hh], res["ref_v"][res["idx"], hh], 0.25)
    assert np.max(np.abs(out - want)) < 1e-12


def test_full_rank_decode_equals_dense_attention_over_raw_kv():
    D = 16
    K, V, cls, _ = _small_case(seed=31, L=70, H=2, D=D, r=8, s=4)
    P = G.make_projections(5, D, D, recipe="paired")
    res = O.compress(K, V, P["w_down_k_f64"], P["w_down_v_f64"], s=4)
    q = _f64(G.make_queries(31, 1, 4, D))[0]
    out, _ = O.decode_attn_direct(q, res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"],
                                  P["w_up_k_f64"], P["w_up_v_f64"], 1 / 4.0)
    assert np.max(np.abs(out - _torch_sdpa(q, K, V, 1 / 4.0))) < 1e-11


def test_single_token_and_zero_query_closed_forms():              # P7
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(L=1)
    out, lse = O.decode_attn_direct(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.3)
    for g in range(6):
        assert np.array_equal(out[g], V[0, g // 3])
        assert abs(lse[g] - 0.3 * (K[0, g // 3] @ q[g])) < 1e-13
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(L=77)
    out, lse = O.decode_attn_direct(0 * q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.3)
    kh, vh = O.reconstruct(res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv)
    for g in range(6):
        assert np.max(np.abs(out[g] - vh[:, g // 3].mean(0))) < 1e-13
        assert abs(lse[g] - math.log(77)) < 1e-13


@pytest.mark.parametrize("joint", [False, True])
def test_direct_equals_absorbed(joint):                              # P8
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=37, L=130, joint=joint)
    a, la = O.decode_attn_direct(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25)
    b, lb = O.decode_attn_absorbed(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25)
    assert np.max(np.abs(a - b)) < 1e-10 and np.max(np.abs(la - lb)) < 1e-10


def test_reconstruction_uses_the_indexed_reference_and_the_right_stream():
    # one token, hand-built cache: K_hat = ref_k[idx] + z_k W_uk, V_hat = ref_v[idx] + z_v W_uv
    rng = np.random.default_rng(3)
    ref_k, ref_v = rng.standard_normal((3, 1, 4)), rng.standard_normal((3, 1, 4))
    wuk, wuv = rng.standard_normal((2, 4)), rng.standard_normal((2, 4))
    idx = np.array([[2]], dtype=np.int32)
    zk, zv = np.array([[[1.0, -2.0]]]), np.array([[[0.5, 3.0]]])
    kh, vh = O.reconstruct(idx, zk, zv, ref_k, ref_v, wuk, wuv)
    assert np.allclose(kh[0, 0], ref_k[2, 0] + 1.0 * wuk[0] - 2.0 * wuk[1], atol=1e-15)
    assert np.allclose(vh[0, 0], ref_v[2, 0] + 0.5 * wuv[0] + 3.0 * wuv[1], atol=1e-15)


def test_lse_merge_of_two_halves_equals_whole():                   # P9
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=41, L=120)
    whole, lw = O.decode_attn_direct(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25)
    parts = []
    for sl in (slice(0, 45), slice(45, 120)):
        parts.append(O.decode_attn_direct(q, res["idx"][sl], zk[sl], zv[sl], res["ref_k"], res["ref_v"],
                                          wuk, wuv, 0.25))
    out, lse = O.merge_partials([p[0] for p in parts], [p[1] for p in parts])
    assert np.max(np.abs(out - whole)) < 1e-12 and np.max(np.abs(lse - lw)) < 1e-12


# ---------------------------------------------------------------- squared-L2 retrieval pins
def test_l2_retrieval_equals_brute_force_and_breaks_ties_low():
    K, V, cls, P = _small_case(seed=61, L=70, H=2, D=16, r=8, s=4)
    K, V = K.copy(), V.copy()
    K[12], V[12] = K[4], V[4]                      # reference 3 duplicates reference 1
    K[41], V[41] = K[4], V[4]                      # token 41 is an exact copy: distance 0 to ordinals 1 and 3
    res = O.compress(K, V, _f64(P["w_down_k_bf16"]), _f64(P["w_down_v_bf16"]), s=4, metric=O.L2)
    kv = np.concatenate([K, V], axis=2)
    for i in range(70):
        for h in range(2):
            if i % 4 == 0:
                assert res["idx"][i, h] == i // 4
                continue
            best, arg = None, None
            for j in range((i + 3) // 4):          # strictly earlier references, ascending
                d = sum((float(kv[i, h, n]) - float(kv[4 * j, h, n])) ** 2 for n in range(32))
                if best is None or d < best:
                    best, arg = d, j
            assert res["idx"][i, h] == arg and abs(res["cos"][i, h] + best) < 1e-12
    assert np.all(res["idx"][41] == 1) and np.all(res["z_k"][41] == 0)


def test_l2_and_cosine_agree_on_unit_norm_references_and_differ_on_a_scaled_copy():
    rng = np.random.default_rng(7)
    L, H, D, s = 61, 1, 8, 4
    K, V = rng.standard_normal((L, H, D)), rng.standard_normal((L, H, D))
    kv = np.concatenate([K, V], axis=2)
    kv[0::s] /= np.linalg.norm(kv[0::s], axis=2, keepdims=True)      # every reference has norm 1
    K, V = kv[..., :D].copy(), kv[..., D:].copy()
    W = np.eye(D)
    a = O.compress(K, V, W, W, s=s, metric=O.COSINE)
    b = O.compress(K, V, W, W, s=s, metric=O.L2)
    assert np.array_equal(a["idx"], b["idx"])      # ||a-b||^2 = |a|^2 + 1 - 2 a.b: same order as the cosine
    # a token that is 3x reference 2 has cosine 1 to it, but is nearer to a longer reference pointing elsewhere
    K2, V2 = K.copy(), V.copy()
    K2[8], V2[8] = 0.0, 0.0
    K2[8, 0, 0] = 1.0                              # reference 2 = e0
    K2[4], V2[4] = 0.0, 0.0
    K2[4, 0, 0], K2[4, 0, 1] = 2.9, 0.8            # reference 1: close to 3*e0 in distance, not in angle
    K2[30], V2[30] = 0.0, 0.0
    K2[30, 0, 0] = 3.0                             # token 30 = 3 * e0
    ca = O.compress(K2, V2, W, W, s=s, metric=O.COSINE)
    cb = O.compress(K2, V2, W, W, s=s, metric=O.L2)
    assert ca["idx"][30, 0] == 2 and cb["idx"][30, 0] == 1


# ---------------------------------------------------------------- subset decode pins
def test_subset_of_all_tokens_is_the_full_attention_and_order_is_free():
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=43, L=101)
    full, lf = O.decode_attn_direct(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25)
    a, la = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25, np.arange(101))
    assert np.array_equal(a, full) and np.array_equal(la, lf)
    sel = np.array([5, 99, 17, 64, 3, 42, 8, 0, 77])
    b, lb = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25, sel)
    c, lc = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25, np.sort(sel))
    assert np.max(np.abs(b - c)) < 1e-13 and np.max(np.abs(lb - lc)) < 1e-13


def test_subset_equals_explicit_softmax_over_the_reconstructed_rows():
    """Brute force from the definition: reconstruct everything, keep the selected rows, softmax by hand."""
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=47, L=88)
    sel = np.array([1, 2, 3, 30, 31, 64, 87])
    out, lse = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.2, sel)
    kh, vh = O.reconstruct(res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv)
    for g in range(6):
        h = g // 3
        logit = np.array([0.2 * float(kh[t, h] @ q[g]) for t in sel])
        w = np.exp(logit - logit.max())
        want = sum(w[i] * vh[t, h] for i, t in enumerate(sel)) / w.sum()
        assert np.max(np.abs(out[g] - want)) < 1e-13
        assert abs(lse[g] - (logit.max() + math.log(w.sum()))) < 1e-13


def test_subset_of_reference_tokens_is_dense_attention_over_raw_references():
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=53, L=90, s=4)
    sel = np.arange(0, 90, 4)[[0, 3, 4, 9, 22]]
    out, _ = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.25, sel)
    assert np.max(np.abs(out - _torch_sdpa(q, K[sel], V[sel], 0.25))) < 1e-12


def test_subset_single_token_empty_selection_and_merge_of_disjoint_subsets():
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=59, L=75)
    kh, vh = O.reconstruct(res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv)
    out, lse = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.3, [41])
    for g in range(6):
        assert np.max(np.abs(out[g] - vh[41, g // 3])) < 1e-14
        assert abs(lse[g] - 0.3 * float(kh[41, g // 3] @ q[g])) < 1e-13
    out0, lse0 = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.3, [])
    assert np.all(out0 == 0) and np.all(np.isneginf(lse0))
    a_sel, b_sel = np.array([0, 9, 33, 70]), np.array([2, 10, 11, 50, 74])
    parts = [O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.3, x)
             for x in (a_sel, b_sel)]
    both, lboth = O.decode_attn_subset(q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.3,
                                       np.concatenate([a_sel, b_sel]))
    out, lse = O.merge_partials([p[0] for p in parts], [p[1] for p in parts])
    assert np.max(np.abs(out - both)) < 1e-12 and np.max(np.abs(lse - lboth)) < 1e-12


# ---------------------------------------------------------------- 4-bit token-wise latents
def test_4bit_quantiser_exact_on_a_16_level_grid_and_degenerate_vectors():
    """Values that already sit on 16 levels with a bf16-representable origin and step come back exactly and their
    codes are the level numbers (the textbook affine quantiser); a constant vector and the zero vector are exact."""
    rng = np.random.default_rng(5)
    lv = rng.integers(0, 16, size=(7, 3, 32))
    lv[..., 0], lv[..., 1] = 0, 15                          # both ends present in every vector
    z = -1.5 + 0.25 * lv                                    # origin -1.5, step 0.25: exact in bf16 and fp32
    codes, sb, zb, back = O.quantize_tokenwise_4bit(z)
    assert np.array_equal(codes, lv) and np.array_equal(back, z)
    assert np.all(O.bf16_bits_to_f64(sb) == 0.25) and np.all(O.bf16_bits_to_f64(zb) == -1.5)
    c2, s2, z2, b2 = O.quantize_tokenwise_4bit(np.full((2, 8), 0.375))
    assert np.all(c2 == 0) and np.all(O.bf16_bits_to_f64(s2) == 0) and np.all(b2 == 0.375)
    c3, s3, z3, b3 = O.quantize_tokenwise_4bit(np.zeros((4, 16)))
    assert np.all(c3 == 0) and np.all(s3 == 0) and np.all(z3 == 0) and np.all(b3 == 0)


def test_4bit_quantiser_halfway_points_go_to_the_even_level_and_are_decided_in_fp64():
    """Values exactly half-way between two levels of a bf16-exact grid take the even level (0.5 -> 0, 1.5 -> 2,
    2.5 -> 2, ... 14.5 -> 14): round-half-up or round-half-away would give 1, 2, 3, ... 15.  A value a hair under a
    half-way point (2^-30 of the step, far below fp32 resolution) stays on the lower level although it rounds to the
    half-way point -- and from there up, when the lower level is odd -- once it is squeezed into fp32: the decision
    is taken on the float64 latent."""
    half = np.arange(15) + 0.5
    z = -2.0 + 0.125 * np.concatenate([[0.0, 15.0], half])          # origin -2, step 1/8: exact in bf16
    codes, sb, zb, back = O.quantize_tokenwise_4bit(z[None, :])
    assert O.bf16_bits_to_f64(sb)[0] == 0.125 and O.bf16_bits_to_f64(zb)[0] == -2.0
    assert codes[0, :2].tolist() == [0, 15]
    assert codes[0, 2:].tolist() == [0, 2, 2, 4, 4, 6, 6, 8, 8, 10, 10, 12, 12, 14, 14]
    assert np.array_equal(O.code_positions_4bit(z[None, :], sb, zb)[0, 2:], half)
    under = -2.0 + 0.125 * (half * (1.0 - 2.0 ** -30))
    assert np.all(under.astype(np.float32).astype(np.float64) == -2.0 + 0.125 * half)   # fp32 cannot tell them apart
    c2 = O.quantize_tokenwise_4bit(np.concatenate([[-2.0, -0.125], under])[None, :])[0]
    assert c2[0, 2:].tolist() == list(range(15))


def test_4bit_quantiser_error_bound_monotonicity_and_record_accounting():
    """|read back - z| <= half a step plus the bf16 rounding of scale and zero point; codes are monotone in z; the
    smallest value gets code 0 and the largest 15; keep ratio of the 4-bit record in closed form."""
    rng = np.random.default_rng(6)
    z = rng.standard_normal((500, 64)) * rng.uniform(0.01, 30.0, size=(500, 1))
    codes, sb, zb, back = O.quantize_tokenwise_4bit(z)
    step = O.bf16_bits_to_f64(sb)
    rng_ = z.max(-1) - z.min(-1)
    assert np.all(np.abs(step - rng_ / 15) <= rng_ / 15 * 2.0 ** -8)
    slack = 15 * step * 2.0 ** -8 + np.abs(z.min(-1)) * 2.0 ** -8 + 1e-6
    assert np.all(np.abs(back - z) <= (0.5 * step + slack)[:, None])
    order = np.argsort(z, axis=-1)
    sorted_codes = np.take_along_axis(codes, order, axis=-1).astype(int)
    assert np.all(np.diff(sorted_codes, axis=-1) >= 0)
    assert np.all(sorted_codes[:, 0] == 0) and np.all(sorted_codes[:, -1] == 15)
    assert O.record_keep_ratio_4bit(O.JOINT, 64, 128, 16) == pytest.approx((32 + 4 + 4 + 516 / 16) / 512)
    assert O.record_keep_ratio_4bit(O.SPLIT, 64, 128, 16) == pytest.approx((2 * 36 + 4 + 516 / 16) / 512)


def test_4bit_compress_keeps_ordinals_and_decodes_close_to_the_bf16_cache():
    """Quantisation touches the latents only: ordinals and references are those of the bf16 path, reference tokens
    keep an exactly zero latent, and attention over the 4-bit cache stays within the quantiser's error of the bf16
    one (a loose sanity bound; the GPU is compared with this oracle, not with the bf16 result)."""
    K, V, cls, P = _small_case(seed=73, L=120, H=2, D=16, r=8, s=4, joint=True)
    wk, wv = _f64(P["w_down_k_bf16"]), _f64(P["w_down_v_bf16"])
    a = O.compress(K, V, wk, wv, s=4, mode=O.JOINT)
    b = O.compress(K, V, wk, wv, s=4, mode=O.JOINT, latent_bits=4)
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["zb_k"], b["zb_k"])
    assert np.all(b["zq_k"][::4] == 0) and np.all(b["q_k"][::4] == 0)
    assert b["zq_v"] is b["zq_k"]
    step = O.bf16_bits_to_f64(b["qs_k"])
    assert np.all(np.abs(b["zq_k"] - b["z_k"]) <= 0.52 * step[..., None] + 1e-3 * np.abs(b["z_k"]).max())
    q = np.random.default_rng(1).standard_normal((6, 16))
    wuk, wuv = _f64(P["w_up_k_bf16"]), _f64(P["w_up_v_bf16"])
    o16, _ = O.decode_attn_direct(q, a["idx"], _f64(a["zb_k"]), _f64(a["zb_k"]), a["ref_k"], a["ref_v"], wuk, wuv, 0.25)
    o4, _ = O.decode_attn_direct(q, b["idx"], b["zq_k"], b["zq_v"], b["ref_k"], b["ref_v"], wuk, wuv, 0.25)
    assert np.max(np.abs(o16 - o4)) < 0.25 * np.abs(o16).max() + 0.05


# ---------------------------------------------------------------- raw (sink / recent) segment pins
def test_raw_segment_brute_force_and_special_cases():
    """Cached tokens + raw rows by hand from the definition; no raw rows = the plain call; no cached tokens = dense
    attention over the raw rows (library routine); the raw rows' place in the concatenation is immaterial."""
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=67, L=60)
    rng = np.random.default_rng(67)
    rk, rv = rng.standard_normal((7, 2, K.shape[2])), rng.standard_normal((7, 2, K.shape[2]))
    args = (q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.22)
    out, lse = O.decode_attn_with_raw(*args, rk, rv)
    kh, vh = O.reconstruct(res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv)
    for g in range(6):
        h = g // 3
        logit = [0.22 * float(kh[t, h] @ q[g]) for t in range(60)] + [0.22 * float(rk[t, h] @ q[g]) for t in range(7)]
        m = max(logit)
        w = [math.exp(x - m) for x in logit]
        want = (sum(w[t] * vh[t, h] for t in range(60)) + sum(w[60 + t] * rv[t, h] for t in range(7))) / sum(w)
        assert np.max(np.abs(out[g] - want)) < 1e-13 and abs(lse[g] - (m + math.log(sum(w)))) < 1e-13
    a, la = O.decode_attn_with_raw(*args, rk[:0], rv[:0])
    b, lb = O.decode_attn_direct(*args)
    assert np.array_equal(a, b) and np.array_equal(la, lb)
    c, _ = O.decode_attn_with_raw(*args, rk, rv, positions=[])
    assert np.max(np.abs(c - _torch_sdpa(q, rk, rv, 0.22))) < 1e-12
    e, le = O.decode_attn_with_raw(*args, rk[:0], rv[:0], positions=[])
    assert np.all(e == 0) and np.all(np.isneginf(le))


def test_raw_segment_is_the_merge_of_the_two_parts_and_equals_caching_exact_tokens():
    """(1) LSE merge of the cache-only result with dense attention over the raw rows.  (2) A reference token is
    reconstructed exactly (z = 0), so serving the reference tokens from the raw segment instead of from the cache
    changes nothing."""
    K, V, res, q, zk, zv, wuk, wuv = _decode_case(seed=71, L=64, s=4)
    rng = np.random.default_rng(71)
    rk, rv = rng.standard_normal((5, 2, K.shape[2])), rng.standard_normal((5, 2, K.shape[2]))
    args = (q, res["idx"], zk, zv, res["ref_k"], res["ref_v"], wuk, wuv, 0.3)
    sel = np.array([1, 4, 9, 10, 33, 63])
    out, lse = O.decode_attn_with_raw(*args, rk, rv, positions=sel)
    p0 = O.decode_attn_subset(*args, sel)
    p1 = O.dense_attention(q, rk, rv, 0.3)
    want, lwant = O.merge_partials([p0[0], p1[0]], [p0[1], p1[1]])
    assert np.max(np.abs(out - want)) < 1e-12 and np.max(np.abs(lse - lwant)) < 1e-12
    refs = np.arange(0, 64, 4)
    others = np.setdiff1d(np.arange(64), refs)
    a, la = O.decode_attn_with_raw(*args, K[refs], V[refs], positions=others)
    b, lb = O.decode_attn_direct(*args)
    assert np.max(np.abs(a - b)) < 1e-12 and np.max(np.abs(la - lb)) < 1e-12


def test_joint_latent_is_sum_of_stream_projections():
    K, V, cls, P = _small_case(seed=43, L=40, H=1, D=16, r=8, s=4, joint=True)
    wk, wv = P["w_down_k_f64"], P["w_down_v_f64"]
    res = O.compress(K, V, wk, wv, s=4, mode=O.JOINT)
    i = 13
    j = int(res["idx"][i, 0])
    want = np.concatenate([K[i, 0] - K[4 * j, 0], V[i, 0] - V[4 * j, 0]]) @ np.concatenate([wk, wv], 0)
    assert np.max(np.abs(res["z_k"][i, 0] - want)) < 1e-13
    assert res["z_v"] is res["z_k"] and res["zb_v"] is res["zb_k"]


def test_incremental_compress_matches_one_shot():
    K, V, cls, P = _small_case(seed=47, L=75, H=2, D=16, r=8, s=4)
    wd = _f64(P["w_down_k_bf16"])
    full = O.compress(K, V, wd, wd, s=4)
    part = O.compress(K, V, wd, wd, s=4, start=51)
    assert np.array_equal(part["idx"], full["idx"][51:])
    assert np.array_equal(part["zb_k"], full["zb_k"][51:]) and np.array_equal(part["zb_v"], full["zb_v"][51:])


def test_generator_recipe_statistics():
    # the inputs have the structure the recipe states: same-class tokens are close, others are not
    K, V, cls = G.make_kv(G.seed_for(1), 2048, 2, 128, n_proto=256)
    Kf = _f64(K)
    same = [(i, j) for i in range(300, 340) for j in range(0, 300) if cls[i, 0] == cls[j, 0]]
    assert len(same) > 5
    def cs(i, j):
        return Kf[i, 0] @ Kf[j, 0] / np.linalg.norm(Kf[i, 0]) / np.linalg.norm(Kf[j, 0])
    assert np.mean([cs(i, j) for i, j in same]) > 0.6
    assert abs(np.mean([cs(i, i - 1) for i in range(1, 400) if cls[i, 0] != cls[i - 1, 0]])) < 0.1
    # per-token energy: 128 (prototype) + 32 (basis part, variance 2 x 16) + 0.32 (noise)
    assert abs(np.mean(np.sum(Kf * Kf, -1)) - 160.3) < 4.0


def test_4bit_record_validity_criterion_accepts_fp32_decisions_and_rejects_planted_mistakes():
    """The criterion the GPU records are held to (tests.helpers.check_q4_records), exercised on the CPU: records
    produced from latents perturbed inside the error bound, with the decisions taken in fp32, pass; a code moved one
    level away from a point that is not half-way, a scale or zero point one bf16 step off where no rounding boundary
    is near, a code two levels from an exact half-way point, and a non-zero code under a zero scale all fail.  (At an
    exact half-way point of the float64 latent either neighbour passes: the computed latent may lie on either side.
    That the definition itself takes the even one is pinned on the oracle above.)"""
    from tests.helpers import check_q4_records
    rng = np.random.default_rng(11)
    z = rng.standard_normal((400, 3, 32)) * rng.uniform(0.05, 8.0, size=(400, 3, 1))
    d = np.full(z.shape, 1e-5) * np.abs(z).max(-1, keepdims=True)
    z32 = (z + rng.uniform(-1, 1, size=z.shape) * d).astype(np.float32)
    mn, mx = z32.min(-1), z32.max(-1)
    sb = O.f64_to_bf16_bits(((mx - mn) * np.float32(1 / 15)).astype(np.float64))
    zb = O.f64_to_bf16_bits(mn.astype(np.float64))
    sc, zp = O.bf16_bits_to_f64(sb).astype(np.float32), O.bf16_bits_to_f64(zb).astype(np.float32)
    codes = np.clip(np.rint((z32 - zp[..., None]) * (np.float32(1) / sc)[..., None]), 0, 15).astype(np.uint8)
    check_q4_records(z, d, codes, sb, zb)
    x = O.code_positions_4bit(z, sb, zb)
    i = np.unravel_index(np.argmin(np.abs(x - np.rint(x)) + (np.rint(x) > 14) + (np.rint(x) < 1)), x.shape)
    bad = codes.copy()
    bad[i] += 1                                              # a value sitting on a level, moved one level up
    with pytest.raises(AssertionError):
        check_q4_records(z, d, bad, sb, zb)
    for arr in (sb, zb):                                     # a stored parameter one bf16 step off, everywhere
        off = arr.copy()
        off += 1
        with pytest.raises(AssertionError):
            check_q4_records(z, d, codes, off if arr is sb else sb, off if arr is zb else zb)
    zg = (-2.0 + 0.125 * np.concatenate([[0.0, 15.0], np.arange(15) + 0.5]))[None, :]
    cg, sg, zg_b, _ = O.quantize_tokenwise_4bit(zg)
    tiny = np.full(zg.shape, 1e-12)
    check_q4_records(zg, tiny, cg, sg, zg_b)
    up = np.concatenate([[0, 15], np.arange(15) + 1]).astype(np.uint8)[None, :]
    check_q4_records(zg, tiny, up, sg, zg_b)                 # at an exact half-way point both neighbours are within eps
    with pytest.raises(AssertionError):
        check_q4_records(zg, tiny, (up + 1).clip(0, 15).astype(np.uint8), sg, zg_b)
    const = np.full((1, 8), 0.375)
    with pytest.raises(AssertionError):
        check_q4_records(const, np.full(const.shape, 1e-12), np.ones((1, 8), np.uint8), np.zeros(1, np.uint16),
                         O.f64_to_bf16_bits(np.array([0.375])))


# ---------------------------------------------------------------- top-k retrieval with the mean of the references
@pytest.mark.parametrize("metric", [O.COSINE, O.L2])
@pytest.mark.parametrize("top_k", [2, 4])
def test_topk_retrieval_is_brute_force_ranking_and_the_residual_is_against_the_mean(metric, top_k):
    """Section 4.1 (arg top-k, then the mean of the retrieved references), by hand in pure Python on a tiny case
    with duplicated references (equal scores: lower ordinal first), an exact copy of a reference, and tokens that
    have fewer candidates than k (they take all of them)."""
    import math
    K, V, cls, P = _small_case(seed=83, L=61, H=2, D=8, r=4, s=4, n_proto=3)
    K[8], V[8] = K[0], V[0]                       # reference 2 duplicates reference 0
    K[20], V[20] = K[4], V[4]                     # reference 5 duplicates reference 1
    K[27], V[27] = K[12], V[12]                   # token 27 is an exact copy of reference 3
    wk, wv = _f64(P["w_down_k_bf16"]), _f64(P["w_down_v_bf16"])
    res = O.compress(K, V, wk, wv, s=4, mode=O.SPLIT, metric=metric, top_k=top_k)
    L, H, D = K.shape
    assert res["idx"].shape == (L, H, top_k)
    for i in range(L):
        for h in range(H):
            got = [int(x) for x in res["idx"][i, h]]
            if i % 4 == 0:
                assert got == [i // 4] + [-1] * (top_k - 1)
                assert np.all(res["z_k"][i, h] == 0) and np.all(res["z_v"][i, h] == 0)
                continue
            a = [float(x) for x in K[i, h]] + [float(x) for x in V[i, h]]
            scored = []
            for j in range((i + 3) // 4):
                bvec = [float(x) for x in K[4 * j, h]] + [float(x) for x in V[4 * j, h]]
                if metric == O.L2:
                    sc = -math.fsum((x - y) ** 2 for x, y in zip(a, bvec))
                else:
                    den = math.sqrt(math.fsum(x * x for x in a)) * math.sqrt(math.fsum(y * y for y in bvec))
                    sc = math.fsum(x * y for x, y in zip(a, bvec)) / den if den > 0 else 0.0
                scored.append((sc, j))
            # exact duplicates must tie exactly whatever the summation order: compare on rounded scores
            ranked = sorted(scored, key=lambda t: (-round(t[0], 12), t[1]))[:top_k]
            want = [j for _, j in ranked] + [-1] * (top_k - len(ranked))
            assert got == want, (i, h, got, want)
            m = len(ranked)
            mean_k = sum(K[4 * j, h] for _, j in ranked) / m
            mean_v = sum(V[4 * j, h] for _, j in ranked) / m
            assert np.max(np.abs(res["z_k"][i, h] - (K[i, h] - mean_k) @ wk)) < 1e-12
            assert np.max(np.abs(res["z_v"][i, h] - (V[i, h] - mean_v) @ wv)) < 1e-12
    assert list(res["idx"][27, 0][:1]) == [3]                    # the exact copy is its own nearest reference
    if top_k == 4:                                               # token 1..3 see one candidate, 5..7 two, 9..11 three
        assert [int((res["idx"][t, 0] >= 0).sum()) for t in (1, 5, 9, 13)] == [1, 2, 3, 4]


def test_topk_first_slot_is_the_top1_choice_and_k_identical_references_give_a_zero_latent():
    K, V, cls, P = _small_case(seed=85, L=70, H=2, D=8, r=4, s=4, n_proto=4)
    wk, wv = _f64(P["w_down_k_bf16"]), _f64(P["w_down_v_bf16"])
    one = O.compress(K, V, wk, wv, s=4, mode=O.JOINT)
    four = O.compress(K, V, wk, wv, s=4, mode=O.JOINT, top_k=4)
    assert np.array_equal(four["idx"][:, :, 0], one["idx"])
    # every reference identical and the token a copy of them: the mean is that vector, the latent is zero
    K2, V2 = K.copy(), V.copy()
    K2[::4], V2[::4] = K[0], V[0]
    K2[33], V2[33] = K[0], V[0]
    res = O.compress(K2, V2, wk, wv, s=4, mode=O.JOINT, top_k=4)
    assert res["idx"][33, 0].tolist() == [0, 1, 2, 3] and np.all(res["z_k"][33] == 0)


@pytest.mark.parametrize("joint", [False, True])
def test_topk_full_rank_reconstruction_and_decode_against_dense_attention(joint):
    """With full-rank orthonormal projections the decoded residual added back to the mean reference is the raw
    token whatever k is, so decode over the k = 4 cache equals dense attention over the raw K, V (library routine)."""
    D = 16
    r = 2 * D if joint else D
    K, V, cls, _ = _small_case(seed=87, L=90, H=2, D=D, r=8, s=4)
    P = G.make_projections(98, D, r, joint=joint, recipe="paired")
    mode = O.JOINT if joint else O.SPLIT
    res = O.compress(K, V, P["w_down_k_f64"], P["w_down_v_f64"], s=4, mode=mode, top_k=4, metric=O.L2)
    kh, vh = O.reconstruct(res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"],
                           P["w_up_k_f64"], P["w_up_v_f64"])
    assert np.max(np.abs(kh - K)) < 1e-12 and np.max(np.abs(vh - V)) < 1e-12
    q = _f64(G.make_queries(87, 1, 4, D))[0]
    out, _ = O.decode_attn_direct(q, res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"],
                                  P["w_up_k_f64"], P["w_up_v_f64"], 0.25)
    assert np.max(np.abs(out - _torch_sdpa(q, K, V, 0.25))) < 1e-11
    # and with zero latents the reconstruction is the mean of the retrieved references, by hand for one token
    t, h = 57, 1
    js = [int(j) for j in res["idx"][t, h] if j >= 0]
    kz, _ = O.reconstruct(res["idx"], 0 * res["z_k"], 0 * res["z_v"], res["ref_k"], res["ref_v"],
                          P["w_up_k_f64"], P["w_up_v_f64"])
    assert len(js) == 4 and np.max(np.abs(kz[t, h] - sum(K[4 * j, h] for j in js) / 4)) < 1e-14


# ---------------------------------------------------------------- rotary position embedding on reconstructed keys
def test_rope_rotation_properties_and_complex_multiplication():
    """A rotation: norms kept, position 0 the identity; the score of a rotated query and key depends on the
    position DIFFERENCE only; dimension pair (i, i + D/2) is the complex number x_i + j x_{i+D/2} multiplied by
    exp(j pos theta_i) (numpy's complex arithmetic as the library routine); D = 2 by hand."""
    rng = np.random.default_rng(91)
    x, y = rng.standard_normal((5, 3, 16)), rng.standard_normal((5, 3, 16))
    pos = np.array([0, 1, 7, 1000, 131071])
    r = O.rope_rotate(x, pos[:, None], 10000.0)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    assert np.array_equal(r[0], x[0])
    a = np.sum(O.rope_rotate(x[1], 1234, 500.0) * O.rope_rotate(y[1], 1200, 500.0), axis=-1)
    b = np.sum(O.rope_rotate(x[1], 34, 500.0) * O.rope_rotate(y[1], 0, 500.0), axis=-1)
    assert np.max(np.abs(a - b)) < 1e-9
    theta = 10000.0 ** (-np.arange(8) * 2.0 / 16)
    z = (x[..., :8] + 1j * x[..., 8:]) * np.exp(1j * pos[:, None, None] * theta)
    assert np.max(np.abs(r - np.concatenate([z.real, z.imag], axis=-1))) < 1e-9
    two = O.rope_rotate(np.array([1.0, 0.0]), 3, 10000.0)                 # D = 2: one pair, theta = 1
    assert np.max(np.abs(two - np.array([np.cos(3.0), np.sin(3.0)]))) < 1e-15


def test_rope_decode_reduces_to_library_attention_over_rotated_raw_keys():
    """Full-rank orthonormal projections reconstruct the raw pre-RoPE keys exactly, so decode with rotation equals
    dense attention (library routine) over explicitly rotated raw K; with every position 0 it gives back the
    un-rotated decode."""
    D = 16
    K, V, cls, _ = _small_case(seed=93, L=75, H=2, D=D, r=8, s=4)
    P = G.make_projections(94, D, D, recipe="paired")
    res = O.compress(K, V, P["w_down_k_f64"], P["w_down_v_f64"], s=4)
    q = _f64(G.make_queries(93, 1, 4, D))[0]
    args = (res["idx"], res["z_k"], res["z_v"], res["ref_k"], res["ref_v"], P["w_up_k_f64"], P["w_up_v_f64"], 0.25)
    out, lse = O.decode_attn_rope(q, *args, base=100.0)
    want = _torch_sdpa(q, O.rope_rotate(K, np.arange(75)[:, None], 100.0), V, 0.25)
    assert np.max(np.abs(out - want)) < 1e-11
    flat, _ = O.decode_attn_rope(q, *args, base=100.0, positions=np.zeros(75, dtype=np.int64))
    plain, _ = O.decode_attn_direct(q, *args)
    assert np.max(np.abs(flat - plain)) < 1e-13
    assert np.max(np.abs(out - plain)) > 1e-3                      # the rotation matters


# ---------------------------------------------------------------- non-linear compressor
def _mlp(kind, n_in=32, hidden=24, r=8, seed=5):
    rng = np.random.default_rng(seed)
    m = {"kind": kind, "w1": rng.standard_normal((n_in, hidden)) / np.sqrt(n_in), "b1": 0.1 * rng.standard_normal(hidden),
         "w2": rng.standard_normal((hidden, r)) / np.sqrt(hidden)}
    if kind == O.SWIGLU:
        m["wg"] = rng.standard_normal((n_in, hidden)) / np.sqrt(n_in)
    return m


@pytest.mark.parametrize("kind", [O.GELU, O.SWIGLU])
def test_mlp_compressor_against_library_activations_and_difference_structure(kind):
    """f_c evaluated with torch's gelu / silu (library routines) on the same weights; the latent is the difference
    f_c(token) - f_c(reference): a token that equals its reference gets exactly zero, reference tokens get zero, and
    for a residual shrunk by 10^-6 the latent approaches the directional derivative (it is linear in small residuals)."""
    import torch
    m = _mlp(kind)
    rng = np.random.default_rng(8)
    x = rng.standard_normal((11, 32))
    tx = torch.from_numpy(x)
    u = tx @ torch.from_numpy(m["w1"]) + torch.from_numpy(m["b1"])
    if kind == O.GELU:
        h = torch.nn.functional.gelu(u)
    else:
        h = torch.nn.functional.silu(tx @ torch.from_numpy(m["wg"])) * u
    want = (h @ torch.from_numpy(m["w2"])).numpy()
    assert np.max(np.abs(O.mlp_compressor(x, m) - want)) < 1e-12
    K, V, cls, P = _small_case(seed=97, L=60, H=2, D=16, r=8, s=4, joint=True)
    K[13], V[13] = K[8], V[8]                      # token 13 is an exact copy of reference 2
    res = O.compress(K, V, None, None, s=4, mode=O.JOINT, mlp=m)
    assert res["idx"][13, 0] == 2 and np.all(res["z_k"][13] == 0) and np.all(res["z_k"][::4] == 0)
    # by hand for one token: f_c(x) - f_c(ref)
    t, h_ = 27, 1
    j = int(res["idx"][t, h_])
    xt = np.concatenate([K[t, h_], V[t, h_]])
    xr = np.concatenate([K[4 * j, h_], V[4 * j, h_]])
    assert np.max(np.abs(res["z_k"][t, h_] - (O.mlp_compressor(xt, m) - O.mlp_compressor(xr, m)))) < 1e-13
    eps = 1e-6
    small = (O.mlp_compressor(xr + eps * (xt - xr), m) - O.mlp_compressor(xr, m)) / eps
    smaller = (O.mlp_compressor(xr + 0.5 * eps * (xt - xr), m) - O.mlp_compressor(xr, m)) / (0.5 * eps)
    assert np.max(np.abs(small - smaller)) < 1e-5 * max(1.0, np.max(np.abs(small)))


def test_retrieve_one_agrees_with_the_batched_retrieval_and_brute_force():
    """`retrieve_one` (used by GPU tests to re-score single tokens) against `compress`' ordinals on every token of a
    small case, and against a brute-force loop over the candidates written out here for a few tokens."""
    K, V, cls, P = _small_case(seed=123, L=90, H=3, D=16, r=8, s=4)
    res = O.compress(K, V, P["w_down_k_f64"], P["w_down_v_f64"], s=4)
    kv = np.concatenate([K, V], axis=2)
    for i in range(90):
        for h in range(3):
            if i % 4 == 0:
                continue
            j, c = O.retrieve_one(kv, i, h, 4)
            assert j == res["idx"][i, h] and abs(c - res["cos"][i, h]) < 1e-12
    for i, h in ((1, 0), (37, 2), (89, 1)):
        best, arg = -np.inf, -1
        for j in range((i + 3) // 4):
            a, b = kv[i, h], kv[4 * j, h]
            c = float(a @ b) / (np.sqrt(float(a @ a)) * np.sqrt(float(b @ b)))
            if c > best:
                best, arg = c, j
        assert O.retrieve_one(kv, i, h, 4)[0] == arg
