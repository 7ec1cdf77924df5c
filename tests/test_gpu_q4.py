"""GPU parity for 4-bit token-wise latents (single-stream layout): decode attention over a cache of 4-bit records
against the oracle's attention over the values those records read back as (max-abs <= 2e-2, relative L2 <= 1e-2),
and the compression kernels' records against the oracle's quantiser."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


class Q4Case:
    """Sequences compressed by the oracle into 4-bit records (JOINT latents, or the two streams of SPLIT)."""

    def __init__(self, seed, lens, Hkv=2, Hq=8, r=64, s=16, n_proto=32, joint=True):
        from oracle import deltakv_oracle as O
        from synthetic import generator as G
        from tests.helpers import f64
        self.lens, self.Hkv, self.Hq, self.r, self.s, self.joint = list(lens), Hkv, Hq, r, s, joint
        self.W = G.make_projections(seed, 128, r, joint=joint)
        self.K, self.V, self.res = [], [], []
        for b, L in enumerate(self.lens):
            K, V, _ = G.make_kv(seed + 17 * b, max(L, 1), Hkv, 128, n_proto=n_proto)
            self.K.append(K[:L])
            self.V.append(V[:L])
            self.res.append(O.compress(f64(K[:L]), f64(V[:L]), f64(self.W["w_down_k_bf16"]), f64(self.W["w_down_v_bf16"]),
                                       s=s, mode=O.JOINT if joint else O.SPLIT, latent_bits=4) if L else None)
        self.q = G.make_queries(seed, len(self.lens), Hq, 128)


def _setup(case, perm=None):
    import paper_2602_08005_amd as dk
    from synthetic import generator as G
    B = len(case.lens)
    max_len = max(max(case.lens), 1)
    pps, rps = -(-max_len // 16), -(-max_len // case.s)
    n_pages, n_slots = B * pps + 5, B * rps + 5
    page_ids = ref_slots = None
    if perm is not None:
        pp, rp = G.page_permutation(perm, B * pps, n_pages), G.page_permutation(perm + 1, B * rps, n_slots)
        page_ids = [pp[b * pps:(b + 1) * pps] for b in range(B)]
        ref_slots = [rp[b * rps:(b + 1) * rps] for b in range(B)]
    dims = dk.make_dims(case.Hkv, case.Hq, case.r, n_pages, n_slots, ref_stride=case.s,
                        latent_mode=dk.JOINT if case.joint else dk.SPLIT, latent_bits=4)
    cache = dk.PagedCache(dims, B, 16, max_len, page_ids=page_ids, ref_slots=ref_slots)
    cache.latent_pool.fill_(0x7FC0)            # bf16 NaN in every scale / zero point that is not written
    cache.idx_pool.fill_(0x7FFFFFF0)
    for b, L in enumerate(case.lens):
        if L:
            r = case.res[b]
            extra = {} if case.joint else dict(codes_v=r["q_v"], scale_bits_v=r["qs_v"], zero_bits_v=r["qz_v"])
            cache.put_sequence_q4(b, r["idx"], r["q_k"], r["qs_k"], r["qz_k"], case.K[b][::case.s], case.V[b][::case.s],
                                  **extra)
    return cache


def _check_decode(case, cache, scale, positions=None):
    import torch
    from oracle import deltakv_oracle as O
    from tests.helpers import dev_bits, out_f64, f64, check_attention
    wuk, wuv, q = dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q)
    lse = torch.zeros((len(case.lens), case.Hq), dtype=torch.float32, device="cuda")
    if positions is None:
        out = cache.decode_attn(wuk, wuv, q, case.lens, scale, lse=lse)
    else:
        out = cache.decode_attn_subset(wuk, wuv, q, case.lens, positions, scale, lse=lse)
    torch.cuda.synchronize()
    assert int(cache.decode_ws[:4].view(torch.int32)[0].item()) == 0
    got, lse = out_f64(out), lse.cpu().numpy().astype(np.float64)
    for b, L in enumerate(case.lens):
        if L == 0:
            assert np.all(got[b] == 0)
            continue
        r = case.res[b]
        args = (f64(case.q[b]), r["idx"], r["zq_k"], r["zq_v"], r["ref_k"], r["ref_v"], f64(case.W["w_up_k_bf16"]),
                f64(case.W["w_up_v_bf16"]), scale)
        want, wl = O.decode_attn_direct(*args) if positions is None else O.decode_attn_subset(*args, positions[b])
        check_attention(got[b], want, f"seq {b}")
        assert np.max(np.abs(lse[b] - wl)) <= 2e-2


@pytest.mark.parametrize("r,Hkv,Hq", [(64, 2, 8), (48, 4, 28), (16, 1, 16), (128, 2, 4)])
def test_decode_over_4bit_records_ragged(r, Hkv, Hq):
    case = Q4Case(9100 + r, [3000, 777, 0, 1601], Hkv=Hkv, Hq=Hq, r=r)
    _check_decode(case, _setup(case, perm=7), 1.0 / np.sqrt(128))


@pytest.mark.parametrize("r,Hkv,Hq", [(64, 2, 8), (128, 1, 7), (64, 4, 28)])
def test_decode_over_4bit_records_two_streams(r, Hkv, Hq):
    case = Q4Case(9150 + r + Hq, [2900, 0, 811, 1601], Hkv=Hkv, Hq=Hq, r=r, joint=False)
    _check_decode(case, _setup(case, perm=9), 1.0 / np.sqrt(128))


@pytest.mark.parametrize("joint", [True, False])
def test_decode_over_4bit_records_long_sequence_and_selection(joint):
    case = Q4Case(9200, [36000], Hkv=1, Hq=4, r=64, n_proto=64, joint=joint)
    cache = _setup(case)
    _check_decode(case, cache, 1.0 / np.sqrt(128))
    rng = np.random.default_rng(3)
    _check_decode(case, cache, 1.0 / np.sqrt(128), positions=[np.sort(rng.choice(36000, 9000, replace=False))])


def _latent_error_bound(case, b, stream):
    """Bound on |z_gpu - z_oracle| per latent value, [L, H, r].  The kernels form the residual exactly in fp32, feed
    it to the matrix unit as bf16 hi + lo parts (what is dropped is below 2^-18 of the element) or to fp32 FMAs, and
    accumulate at most 2 x 256 products in fp32 (each addition rounds to 2^-24 of the running sum, itself at most the
    sum of the terms' magnitudes): (2^-18 + 512 * 2^-24) * sum_i |r_i| |W_ic| < 2^-14 * sum_i |r_i| |W_ic|."""
    from tests.helpers import f64
    res, s = case.res[b], case.s
    K, V = f64(case.K[b]), f64(case.V[b])
    tok_ref = res["idx"].astype(np.int64) * s
    hh = np.arange(case.Hkv)[None, :]
    t = np.arange(K.shape[0])[:, None]
    ak, av = np.abs(K[t, hh] - K[tok_ref, hh]), np.abs(V[t, hh] - V[tok_ref, hh])
    wk, wv = np.abs(f64(case.W["w_down_k_bf16"])), np.abs(f64(case.W["w_down_v_bf16"]))
    if case.joint:
        mag = ak @ wk + av @ wv
    else:
        mag = av @ wv if stream else ak @ wk
    return 2.0 ** -14 * mag + 1e-30


def _compare_records(case, cache, b, t0, t1, stream=0):
    """GPU-written 4-bit records of tokens t0..t1-1 against the oracle's definition: accepted iff they are what
    the definition gives for some latent within the kernels' arithmetic error of the oracle's float64 latent
    (tests.helpers.check_q4_records); the oracle's own record is the outcome in nearly all tokens."""
    from oracle import deltakv_oracle as O
    r = case.res[b]
    idx, codes, sb, zb = cache.get_sequence_q4(b, t0, t1, stream)
    assert np.array_equal(idx, r["idx"][t0:t1])
    sfx = "_v" if stream else "_k"
    z = r["z" + sfx][t0:t1]
    d = _latent_error_bound(case, b, stream)[t0:t1]
    from tests.helpers import check_q4_records
    check_q4_records(z, d, codes, sb, zb)
    scale, zero = O.bf16_bits_to_f64(sb), O.bf16_bits_to_f64(zb)
    # and the oracle's own record is the usual outcome: identical in nearly all tokens
    same = (sb == r["qs" + sfx][t0:t1]) & (zb == r["qz" + sfx][t0:t1])
    assert same.mean() > 0.99 and (codes[same] == r["q" + sfx][t0:t1][same]).mean() > 0.99
    back = scale[..., None] * codes + zero[..., None]
    return idx, back


@pytest.mark.parametrize("r,joint", [(64, True), (32, True), (128, True), (64, False), (128, False)])
def test_compress_writes_the_oracles_4bit_records_prefill_append_and_single_tokens(r, joint):
    import torch
    import paper_2602_08005_amd as dk
    from oracle import deltakv_oracle as O
    from tests.helpers import dev_bits, out_f64, f64, check_attention
    case = Q4Case(9300 + r, [2500, 1203], Hkv=2, Hq=8, r=r, n_proto=16, joint=joint)
    B, max_len = 2, 2500
    pps = -(-max_len // 16)
    dims = dk.make_dims(2, 8, r, B * pps + 3, B * pps + 3, latent_mode=dk.JOINT if joint else dk.SPLIT, latent_bits=4)
    cache = dk.PagedCache(dims, B, 4000, max_len)
    cache.latent_pool.fill_(0x7FC0)
    wk, wv = dev_bits(case.W["w_down_k_bf16"]), dev_bits(case.W["w_down_v_bf16"])
    first = [1701, 903]                        # prefill, then a batched ragged append that starts inside a page (and
    second = [2490, 1193]                      # inside a token pair of the value stream), then single-token appends
    for lo, hi in (([0, 0], first), (first, second)):
        kn = np.concatenate([case.K[b][lo[b]:hi[b]] for b in range(B)])
        vn = np.concatenate([case.V[b][lo[b]:hi[b]] for b in range(B)])
        cu = np.concatenate([[0], np.cumsum([hi[b] - lo[b] for b in range(B)])]).astype(np.int32)
        cache.compress(wk, wv, dev_bits(kn), dev_bits(vn), cu, np.asarray(lo, dtype=np.int32))
    for step in range(10):
        t = [second[0] + step, second[1] + step]
        cache.compress(wk, wv, dev_bits(np.stack([case.K[b][t[b]] for b in range(B)])),
                       dev_bits(np.stack([case.V[b][t[b]] for b in range(B)])), [0, 1, 2], t)
    torch.cuda.synchronize()
    backs = []
    for b in range(B):
        bk = _compare_records(case, cache, b, 0, case.lens[b])
        bv = bk if joint else _compare_records(case, cache, b, 0, case.lens[b], stream=1)
        backs.append((bk[0], bk[1], bv[1]))
    # attention over the GPU-built cache against the oracle's attention over the values ITS records read back as
    scale = 1.0 / np.sqrt(128)
    out = out_f64(cache.decode_attn(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q),
                                    case.lens, scale))
    torch.cuda.synchronize()
    for b in range(B):
        idx, back, back_v = backs[b]
        res = case.res[b]
        want, _ = O.decode_attn_direct(f64(case.q[b]), idx, back, back_v, res["ref_k"], res["ref_v"],
                                       f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale)
        check_attention(out[b], want, f"seq {b}")


def test_4bit_two_stream_layout_needs_rank_64_or_128():
    import paper_2602_08005_amd as dk
    from paper_2602_08005_amd import binding as B
    with pytest.raises(dk.DeltaKVError) as e:
        dk.paged_layout(dk.make_dims(2, 8, 48, 8, 8, latent_mode=dk.SPLIT, latent_bits=4), 1, 16, 16)
    assert e.value.code == B.E_UNSUPPORTED
    assert dk.paged_layout(dk.make_dims(2, 8, 64, 8, 8, latent_mode=dk.SPLIT, latent_bits=4), 1, 16, 16).n_streams == 2
    with pytest.raises(dk.DeltaKVError) as e:
        dk.paged_layout(dk.make_dims(2, 8, 64, 8, 8, latent_mode=dk.JOINT, latent_bits=8), 1, 16, 16)
    assert e.value.code == B.E_INVALID_ARG
