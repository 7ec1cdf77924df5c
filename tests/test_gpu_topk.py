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
