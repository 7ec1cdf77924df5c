"""GPU parity of deltakv_decode_attn_rope (keys reconstructed from the pre-RoPE cache, rotated at their position,
then attended) against the CPU oracle.  Bar: max-abs <= 2e-2 on bf16 outputs, relative L2 <= 1e-2, lse within 2e-2."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _run_rope(case, cache, scale, base, q_rot_bits):
    import torch
    from tests.helpers import dev_bits, out_f64
    lse = torch.full((len(case.lens), case.Hq), 123.0, dtype=torch.float32, device="cuda")
    out = cache.decode_attn_rope(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(q_rot_bits),
                                 case.lens, scale, base, lse=lse)
    torch.cuda.synchronize()
    return out_f64(out), lse.cpu().numpy().astype(np.float64)


def _check(case, cache, scale, base):
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import f64, check_attention
    # the query is rotated at the position of the token being decoded (one past the cache), then stored as bf16
    q = f64(case.q)
    q_rot = np.stack([O.rope_rotate(q[b], max(case.lens[b], 1), base) for b in range(len(case.lens))])
    q_bits = G.f32_to_bf16_bits(q_rot.astype(np.float32))
    got, lse = _run_rope(case, cache, scale, base, q_bits)
    for b, L in enumerate(case.lens):
        if L == 0:
            assert np.all(got[b] == 0) and np.all(np.isneginf(lse[b]))
            continue
        r = case.res[b]
        want, wl = O.decode_attn_rope(f64(q_bits[b]), r["idx"], f64(r["zb_k"]), f64(r["zb_v"]), r["ref_k"], r["ref_v"],
                                      f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale, base=base)
        check_attention(got[b], want, f"seq {b} len {L}")
        assert np.max(np.abs(lse[b] - wl)) <= 2e-2, (b, np.max(np.abs(lse[b] - wl)))
        plain, _ = O.decode_attn_direct(f64(q_bits[b]), r["idx"], f64(r["zb_k"]), f64(r["zb_v"]), r["ref_k"], r["ref_v"],
                                        f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale)
        if L > 64:
            assert np.max(np.abs(want - plain)) > 1e-3       # the rotation matters in this case


@pytest.mark.parametrize("joint,r,Hkv,Hq,base", [(False, 64, 2, 8, 10000.0), (True, 64, 2, 8, 500000.0),
                                                 (False, 48, 4, 28, 10000.0), (True, 32, 1, 1, 100.0),
                                                 (False, 128, 1, 4, 1000000.0), (False, 16, 2, 12, 10000.0)])
def test_rope_decode_ragged_batch(joint, r, Hkv, Hq, base):
    from tests.helpers import Case
    from tests.test_gpu_decode import _setup
    case = Case(15000 + r + Hq, [3000, 777, 0, 1601, 1, 15, 17, 4100], Hkv=Hkv, Hq=Hq, r=r, n_proto=32, joint=joint)
    for perm in (None, 31):
        _check(case, _setup(case, page_perm_seed=perm), 1.0 / np.sqrt(128), base)


def test_rope_decode_long_sequence_several_splits_and_needle():
    from paper_2602_08005_amd import binding as B
    from oracle import deltakv_oracle as O
    from synthetic import generator as G
    from tests.helpers import Case, f64, check_attention
    from tests.test_gpu_decode import _setup
    case = Case(15100, [40000, 9000], Hkv=2, Hq=8, r=64, n_proto=64)
    cache = _setup(case)
    scale = 1.0 / np.sqrt(128)
    for splits in (0, 1, 11):
        B.tune("splits", splits)
        try:
            _check(case, cache, scale, 500000.0)
        finally:
            B.tune("splits", 0)
    # needle: the query is 8 x the rotated reconstructed key of one token per head -> outputs of order one
    r0 = case.res[0]
    kh, vh = O.reconstruct(r0["idx"], f64(r0["zb_k"]), f64(r0["zb_v"]), r0["ref_k"], r0["ref_v"],
                           f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]))
    t_star = [1234, 17, 39999, 640, 5, 20480, 777, 31601]
    qn = np.stack([8.0 * O.rope_rotate(kh[t_star[g], g // 4], t_star[g], 500000.0) for g in range(8)])
    q_bits = np.stack([G.f32_to_bf16_bits(qn.astype(np.float32)), case.q[1]])
    got, lse = _run_rope(case, cache, scale, 500000.0, q_bits)
    want, wl = O.decode_attn_rope(f64(q_bits[0]), r0["idx"], f64(r0["zb_k"]), f64(r0["zb_v"]), r0["ref_k"], r0["ref_v"],
                                  f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale, base=500000.0)
    assert np.max(np.abs(want)) > 1.0
    check_attention(got[0], want, "needle", scale_with_magnitude=True)
    assert np.max(np.abs(lse[0] - wl)) <= 2e-2 * max(1.0, float(np.max(np.abs(wl))) / 64)


def test_rope_decode_unsupported_shapes():
    import torch
    import paper_2602_08005_amd as dk
    from paper_2602_08005_amd import binding as B
    z = torch.zeros(4096, dtype=torch.int32, device="cuda")
    tab = torch.zeros((1, 64), dtype=torch.int32, device="cuda")
    for kw in (dict(n_q=32, n_kv=2), dict(top_k=4), dict(latent_bits=4, latent_mode=dk.JOINT)):
        n_kv, n_q = kw.pop("n_kv", 2), kw.pop("n_q", 8)
        dims = dk.make_dims(n_kv, n_q, 64, 64, 64, **kw)
        lay = dk.paged_layout(dims, 1, 16, 1024)
        ws = torch.empty(lay.decode_ws_bytes, dtype=torch.uint8, device="cuda")
        rc = B.decode_attn_rope(dims, lay, z, z, z, tab, tab, z, z, z, torch.tensor([64], dtype=torch.int32, device="cuda"),
                                [64], 0.1, 10000.0, z, None, ws, check=False)
        assert rc == B.E_UNSUPPORTED
