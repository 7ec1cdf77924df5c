"""The allocation-free decode entry point (deltakv_decode_attn_static: workspace inside the library's device image)
against deltakv_decode_attn on a caller-provided workspace and against the oracle: two calls in a row on the same
GPU, the second with a smaller batch and shorter sequences, so that whatever the first call left in the shared array
is stale for the second."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _run(case, scale):
    import torch
    import paper_2602_08005_amd as dk
    from paper_2602_08005_amd import binding as B
    from tests.helpers import dev_bits, out_f64
    nb = len(case.lens)
    max_len = max(case.lens)
    pps, rps = -(-max_len // 16), -(-max_len // case.s)
    dims = dk.make_dims(case.Hkv, case.Hq, case.r, nb * pps + 2, nb * rps + 2, ref_stride=case.s,
                        latent_mode=dk.JOINT if case.joint else dk.SPLIT)
    cache = dk.PagedCache(dims, nb, 16, max_len)
    for b, L in enumerate(case.lens):
        r = case.res[b]
        cache.put_sequence(b, r["idx"], r["zb_k"], r["zb_v"], case.K[b][::case.s], case.V[b][::case.s])
    wuk, wuv, q = dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q)
    lens_dev = torch.tensor(case.lens, dtype=torch.int32, device="cuda")
    ref_lse = torch.zeros((nb, case.Hq), dtype=torch.float32, device="cuda")
    ref_out = cache.decode_attn(wuk, wuv, q, case.lens, scale, lse=ref_lse)
    out = torch.full_like(q, 0x7FC0)
    lse = torch.full((nb, case.Hq), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.decode_attn_static(dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.block_tables,
                         cache.ref_tables, wuk, wuv, q, lens_dev, case.lens, scale, out, lse)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return out_f64(out), lse.cpu().numpy(), out_f64(ref_out), ref_lse.cpu().numpy()


def test_static_workspace_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    from tests.helpers import Case, check_attention
    scale = 1.0 / np.sqrt(128)
    first = Case(4301, [5000, 1234, 3000], Hkv=2, Hq=8, r=64)
    second = Case(4302, [700, 33], Hkv=2, Hq=8, r=64)
    for case in (first, second):
        got, lse, ref, ref_lse = _run(case, scale)
        # same kernels, same launch plan: equal up to the order of the on-chip float additions
        assert np.max(np.abs(got - ref)) <= 2.0 ** -8 * max(1.0, float(np.max(np.abs(ref))))
        assert np.max(np.abs(lse - ref_lse)) <= 1e-5
        for b in range(len(case.lens)):
            want, wl = case.oracle_decode(b, scale)
            check_attention(got[b], want, f"seq {b}")
            assert np.max(np.abs(lse[b] - wl)) <= 2e-2


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    import torch
    import paper_2602_08005_amd as dk
    from paper_2602_08005_amd import binding as B
    # 64 sequences of 131072 tokens: the per-reference score table alone is larger than the static array
    L, nb = 131072, 64
    dims = dk.make_dims(8, 32, 64, 64, 64)
    lay = dk.paged_layout(dims, 1, 16, 1024)
    z = torch.zeros(4096, dtype=torch.int32, device="cuda")
    tab = torch.zeros((nb, L // 16), dtype=torch.int32, device="cuda")
    lens = np.full(nb, L, dtype=np.int32)
    rc = B.decode_attn_static(dk.make_dims(8, 32, 64, L // 16, L // 16), lay, z, z, z, tab, tab, z, z, z,
                              torch.from_numpy(lens).cuda(), lens, 0.1, z, None, check=False)
    assert rc == B.E_WORKSPACE
    with pytest.raises(dk.DeltaKVError, match="static workspace"):
        B.decode_attn_static(dk.make_dims(8, 32, 64, L // 16, L // 16), lay, z, z, z, tab, tab, z, z, z,
                             torch.from_numpy(lens).cuda(), lens, 0.1, z, None)
