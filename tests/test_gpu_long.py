"""Sequences whose per-reference weight table does not fit one compute unit's LDS: the streaming kernel keeps a
window of the most recent ordinals on chip and accumulates the weights of older ordinals in global memory.  Parity
against the CPU oracle (a) on ordinary caches with the window forced down to a few dozen ordinals, in every record
format and call variant, and (b) at lengths past the on-chip limit, up to a million tokens, on records drawn at
random (decode does not care how ordinals and latents were chosen; compress is tested elsewhere).
Bar: max-abs <= 2e-2 on bf16 outputs, relative L2 <= 1e-2, lse within 2e-2."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("joint,rows", [(False, 64), (True, 16), (False, 1000)])
def test_forced_small_window_full_subset_and_raw(joint, rows):
    import torch
    from paper_2602_08005_amd import binding as B
    from tests.helpers import Case, dev_bits, out_f64, check_attention, f64
    from tests.test_gpu_decode import _setup, _run, _compare
    from tests import test_gpu_subset as TS
    from oracle import deltakv_oracle as O
    case = Case(9900 + rows, [3000, 777, 16, 1601, 4100], Hkv=2, Hq=8, r=64, n_proto=32, joint=joint)
    cache = _setup(case, page_perm_seed=11)
    scale = 1.0 / np.sqrt(128)
    B.tune("table_rows", rows)
    try:
        for splits in (0, 1, 5):
            B.tune("splits", splits)
            got, lse, status = _run(case, cache, scale)
            assert status == 0
            _compare(case, got, lse, scale)
        B.tune("splits", 0)
        rng = np.random.default_rng(rows)
        positions = [np.sort(rng.choice(L, L // 3, replace=False)) for L in case.lens]
        got, lse, status = TS._run_subset(case, cache, scale, positions)
        assert status == 0
        TS._compare(case, got, lse, scale, positions)
        # raw segment beside the cache
        nb = len(case.lens)
        raw_lens = [300, 0, 5, 77, 1]
        rk = rng.standard_normal((nb, 300, 2, 128)).astype(np.float32)
        rv = rng.standard_normal((nb, 300, 2, 128)).astype(np.float32)
        from synthetic import generator as G
        rkb, rvb = G.f32_to_bf16_bits(rk), G.f32_to_bf16_bits(rv)
        lse_t = torch.zeros((nb, 8), dtype=torch.float32, device="cuda")
        out = cache.decode_attn_raw(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q),
                                    case.lens, dev_bits(rkb), dev_bits(rvb), raw_lens, scale, lse=lse_t)
        torch.cuda.synchronize()
        got = out_f64(out)
        for b, L in enumerate(case.lens):
            r = case.res[b]
            idx, zk, zv, refk, refv = r["idx"], f64(r["zb_k"]), f64(r["zb_v"]), r["ref_k"], r["ref_v"]
            want, wl = O.decode_attn_with_raw(f64(case.q[b]), idx, zk, zv, refk, refv, f64(case.W["w_up_k_bf16"]),
                                              f64(case.W["w_up_v_bf16"]), scale, f64(rkb[b, :raw_lens[b]]),
                                              f64(rvb[b, :raw_lens[b]]))
            check_attention(got[b], want, f"raw seq {b}")
            assert np.max(np.abs(lse_t[b].cpu().numpy() - wl)) <= 2e-2
    finally:
        B.tune("table_rows", 0)
        B.tune("splits", 0)


def test_forced_small_window_4bit_records():
    from paper_2602_08005_amd import binding as B
    from tests.test_gpu_q4 import Q4Case, _setup, _check_decode
    B.tune("table_rows", 48)
    try:
        for joint in (True, False):
            case = Q4Case(9950 + joint, [2900, 0, 811, 1601], Hkv=2, Hq=8, r=64, joint=joint)
            _check_decode(case, _setup(case, perm=9), 1.0 / np.sqrt(128))
    finally:
        B.tune("table_rows", 0)


class RandomRecords:
    """A cache of L tokens per sequence drawn at random: bf16 reference rows ~ N(0,1), every non-reference token
    pointing at a uniformly drawn earlier reference (long-range by construction), bf16 latents ~ N(0, 0.25)."""

    def __init__(self, seed, lens, Hkv, Hq, r, joint):
        from synthetic import generator as G
        rng = np.random.default_rng(seed)
        self.lens, self.Hkv, self.Hq, self.r, self.joint, self.s = list(lens), Hkv, Hq, r, joint, 16
        self.W = G.make_projections(seed, 128, r, joint=joint)
        self.q = G.make_queries(seed, len(lens), Hq, 128)
        self.recs = []
        for L in lens:
            n_ref = -(-L // 16)
            t = np.arange(L)
            ncand = -(-t // 16)
            idx = (rng.random((L, Hkv)) * np.maximum(ncand, 1)[:, None]).astype(np.int32)
            idx[::16] = (t[::16] // 16)[:, None]
            zk = G.f32_to_bf16_bits((0.5 * rng.standard_normal((L, Hkv, r), dtype=np.float32)))
            zv = zk if joint else G.f32_to_bf16_bits((0.5 * rng.standard_normal((L, Hkv, r), dtype=np.float32)))
            zk[::16] = 0
            zv[::16] = 0
            refk = G.f32_to_bf16_bits(rng.standard_normal((n_ref, Hkv, 128), dtype=np.float32))
            refv = G.f32_to_bf16_bits(rng.standard_normal((n_ref, Hkv, 128), dtype=np.float32))
            self.recs.append((idx, zk, zv, refk, refv))


def _run_random_records(case, scale):
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from tests.helpers import dev_bits, out_f64, f64, check_attention
    nb, max_len = len(case.lens), max(case.lens)
    pps = -(-max_len // 16)
    dims = dk.make_dims(case.Hkv, case.Hq, case.r, nb * pps + 1, nb * pps + 1,
                        latent_mode=dk.JOINT if case.joint else dk.SPLIT)
    cache = dk.PagedCache(dims, nb, 16, max_len)
    for b, (idx, zk, zv, refk, refv) in enumerate(case.recs):
        cache.put_sequence(b, idx, zk, zv, refk, refv, chunk=65536)
    lse = torch.zeros((nb, case.Hq), dtype=torch.float32, device="cuda")
    out = cache.decode_attn(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q),
                            case.lens, scale, lse=lse)
    assert cache.status() == 0
    got, lse = out_f64(out), lse.cpu().numpy()
    for b, (idx, zk, zv, refk, refv) in enumerate(case.recs):
        want, wl = O.decode_attn_direct(f64(case.q[b]), idx, f64(zk), f64(zv), f64(refk), f64(refv),
                                        f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale)
        check_attention(got[b], want, f"seq {b} len {case.lens[b]}")
        assert np.max(np.abs(lse[b] - wl)) <= 2e-2
    return cache


@pytest.mark.parametrize("Hq,joint,lens", [(4, False, [200000, 40000]), (7, False, [100003]), (8, True, [90000, 100]),
                                           (16, False, [60000])])
def test_lengths_just_past_the_on_chip_table(Hq, joint, lens):
    """4 query heads per kv-head fit 39 000 ordinals (160 000 tokens) on chip, 7 or 8 heads 19 000, 16 heads 9 700."""
    _run_random_records(RandomRecords(31000 + Hq, lens, 1, Hq, 64, joint), 1.0 / np.sqrt(128))


@pytest.mark.parametrize("Hq,L", [(4, 1 << 20), (7, 1 << 19)])
def test_a_million_tokens_at_four_heads_and_half_a_million_at_seven(Hq, L):
    case = RandomRecords(32000 + Hq, [L], 1, Hq, 64, False)
    cache = _run_random_records(case, 1.0 / np.sqrt(128))
    # the same call with a selection of an eighth of the pages, clustered and scattered
    from tests import test_gpu_subset as TS
    rng = np.random.default_rng(5)
    pages = np.sort(rng.choice(L // 16, L // 128, replace=False))
    positions = [(pages[:, None] * 16 + np.arange(16)[None, :]).ravel()]
    import torch
    from oracle import deltakv_oracle as O
    from tests.helpers import dev_bits, out_f64, f64, check_attention
    scale = 1.0 / np.sqrt(128)
    lse = torch.zeros((1, Hq), dtype=torch.float32, device="cuda")
    out = cache.decode_attn_subset(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q),
                                   case.lens, positions, scale, lse=lse)
    assert cache.status() == 0
    idx, zk, zv, refk, refv = case.recs[0]
    want, wl = O.decode_attn_subset(f64(case.q[0]), idx, f64(zk), f64(zv), f64(refk), f64(refv),
                                    f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale, positions[0])
    check_attention(out_f64(out)[0], want, "subset")
    assert np.max(np.abs(lse.cpu().numpy()[0] - wl)) <= 2e-2
