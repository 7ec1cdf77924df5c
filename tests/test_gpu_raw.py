"""GPU parity of deltakv_decode_attn_raw (compressed cache + a raw sink / recent segment) against the CPU oracle.
Bar: max-abs <= 2e-2 on bf16 outputs, plus relative L2 <= 1e-2; lse within 2e-2."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _raw_rows(seed, B, cap, Hkv, lens, gain=1.0):
    """Raw K, V bf16 bits [B, cap, Hkv, 128]; rows past lens[b] are poisoned with NaN bits (never read)."""
    from synthetic import generator as G
    K = np.full((B, cap, Hkv, 128), 0x7FC0, dtype=np.uint16)
    V = np.full((B, cap, Hkv, 128), 0x7FC0, dtype=np.uint16)
    for b in range(B):
        if lens[b]:
            k, v, _ = G.make_kv(seed + b, lens[b], Hkv, 128, n_proto=8)
            if gain != 1.0:
                x = (k.astype(np.uint32) << 16).view(np.float32) * np.float32(gain)
                u = x.view(np.uint32)
                k = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
            K[b, :lens[b]], V[b, :lens[b]] = k, v
    return K, V


def _run(case, cache, scale, rawK, rawV, raw_lens, positions=None):
    import torch
    from tests.helpers import dev_bits, out_f64
    lse = torch.full((len(case.lens), case.Hq), 123.0, dtype=torch.float32, device="cuda")
    out = cache.decode_attn_raw(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q),
                                case.lens, None if rawK is None else dev_bits(rawK),
                                None if rawV is None else dev_bits(rawV), raw_lens, scale,
                                positions_per_seq=positions, lse=lse)
    torch.cuda.synchronize()
    status = int(cache.decode_ws[:4].view(torch.int32)[0].item())
    return out_f64(out), lse.cpu().numpy().astype(np.float64), status


def _compare(case, got, lse, scale, rawK, rawV, raw_lens, positions=None):
    from tests.helpers import check_attention, f64
    from oracle import deltakv_oracle as O
    for b, L in enumerate(case.lens):
        r = case.res[b]
        pos = None
        if positions is not None:
            pos = np.asarray(positions[b], dtype=np.int64)
            pos = pos[pos < L]
        if L:
            idx, zk, zv, rk, rv = r["idx"], f64(r["zb_k"]), f64(r["zb_v"]), r["ref_k"], r["ref_v"]
        else:                                   # nothing cached: empty arrays of the right widths
            wz = case.W["w_up_k_bf16"].shape[0]
            idx, zk, zv = np.zeros((0, case.Hkv), dtype=np.int64), np.zeros((0, case.Hkv, wz)), np.zeros((0, case.Hkv, wz))
            rk = rv = np.zeros((1, case.Hkv, 128))
        want, wl = O.decode_attn_with_raw(f64(case.q[b]), idx, zk, zv, rk, rv,
                                          f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale,
                                          f64(rawK[b, :raw_lens[b]]), f64(rawV[b, :raw_lens[b]]), positions=pos)
        if np.all(np.isneginf(wl)):
            assert np.all(got[b] == 0) and np.all(np.isneginf(lse[b]))
            continue
        check_attention(got[b], want, f"seq {b}")
        assert np.max(np.abs(lse[b] - wl)) <= 2e-2, (b, np.max(np.abs(lse[b] - wl)))


@pytest.mark.parametrize("joint,Hkv,Hq,r", [(False, 2, 8, 64), (True, 2, 8, 48), (False, 4, 28, 48), (False, 1, 16, 32)])
def test_cache_plus_raw_segment_ragged(joint, Hkv, Hq, r):
    """Raw segments of 0, 1, a ragged chunk and several chunks beside caches of different lengths."""
    from tests.helpers import Case
    from tests.test_gpu_decode import _setup
    case = Case(9500 + Hq, [2500, 700, 1300, 333], Hkv=Hkv, Hq=Hq, r=r, n_proto=16, joint=joint)
    cache = _setup(case, page_perm_seed=3)
    raw_lens = [0, 1, 300, 777]
    rawK, rawV = _raw_rows(77, 4, 800, Hkv, raw_lens)
    scale = 1.0 / np.sqrt(128)
    got, lse, status = _run(case, cache, scale, rawK, rawV, raw_lens)
    assert status == 0
    _compare(case, got, lse, scale, rawK, rawV, raw_lens)


def test_raw_segment_with_a_selection_and_raw_only_sequences():
    """Subset of the cache + raw rows; an empty selection and an empty sequence attend their raw rows alone; a
    sequence with nothing at all gives zeros and lse = -inf."""
    from tests.helpers import Case, f64
    from oracle import deltakv_oracle as O
    from tests.test_gpu_decode import _setup
    case = Case(9600, [1500, 1500, 0, 0], Hkv=2, Hq=8, r=64, n_proto=16)
    cache = _setup(case)
    rng = np.random.default_rng(4)
    positions = [np.sort(rng.choice(1500, 400, replace=False)), np.array([], dtype=np.int64),
                 np.array([], dtype=np.int64), np.array([], dtype=np.int64)]
    raw_lens = [130, 64, 257, 0]
    rawK, rawV = _raw_rows(78, 4, 257, 2, raw_lens)
    got, lse, status = _run(case, cache, 0.1, rawK, rawV, raw_lens, positions)
    _compare(case, got, lse, 0.1, rawK, rawV, raw_lens, positions)
    want, _ = O.dense_attention(f64(case.q[2]), f64(rawK[2, :257]), f64(rawV[2, :257]), 0.1)
    assert np.max(np.abs(got[2] - want)) <= 2e-2
    assert np.all(got[3] == 0) and np.all(np.isneginf(lse[3]))


def test_raw_logits_far_above_and_far_below_the_cached_ones():
    """The two parts are merged at the larger exponent offset: raw keys scaled 64x dominate (the cached part
    underflows harmlessly), raw keys scaled 1/64 barely count; neither sets the status word."""
    from tests.helpers import Case
    from tests.test_gpu_decode import _setup
    for gain in (64.0, 1.0 / 64.0):
        case = Case(9700, [2000, 900], Hkv=2, Hq=8, r=64, n_proto=16)
        cache = _setup(case)
        raw_lens = [200, 40]
        rawK, rawV = _raw_rows(79, 2, 256, 2, raw_lens, gain=gain)
        got, lse, status = _run(case, cache, 0.5, rawK, rawV, raw_lens)
        assert status == 0
        _compare(case, got, lse, 0.5, rawK, rawV, raw_lens)


def test_no_raw_segment_is_the_plain_call_and_bad_arguments_are_rejected():
    import torch
    from paper_2602_08005_amd import binding as B
    from tests.helpers import Case, dev_bits, out_f64
    from tests.test_gpu_decode import _setup
    case = Case(9800, [1000, 400], Hkv=2, Hq=8, r=64, n_proto=16)
    cache = _setup(case)
    wk, wv, q = dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q)
    full = out_f64(cache.decode_attn(wk, wv, q, case.lens, 0.1))
    got, _, _ = _run(case, cache, 0.1, None, None, [0, 0])
    assert np.array_equal(full, got)
    rawK, rawV = _raw_rows(80, 2, 64, 2, [64, 64])
    zero, _, _ = _run(case, cache, 0.1, rawK, rawV, [0, 0])          # a segment with no valid rows
    assert np.array_equal(full, zero)
    seq = torch.tensor(case.lens, dtype=torch.int32, device="cuda")
    rl = torch.tensor([1, 1], dtype=torch.int32, device="cuda")
    out = torch.empty_like(q)
    big = torch.zeros((2, 4097, 2, 128), dtype=torch.int16, device="cuda")
    args = (cache.dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.block_tables,
            cache.ref_tables, wk, wv, q, seq, case.lens)
    assert B.decode_attn_raw(*args, big, big, rl, 0.1, out, None, cache.decode_ws, check=False) == B.E_UNSUPPORTED
    assert B.decode_attn_raw(*args, dev_bits(rawK), None, rl, 0.1, out, None, cache.decode_ws,
                             check=False) == B.E_INVALID_ARG
    assert B.decode_attn_raw(*args, dev_bits(rawK), dev_bits(rawV), None, 0.1, out, None, cache.decode_ws,
                             check=False) == B.E_INVALID_ARG
