"""GPU parity of deltakv_decode_attn_subset (attention over selected tokens only) against the CPU oracle.
Bar: max-abs <= 2e-2 on bf16 outputs, plus relative L2 <= 1e-2; lse within 2e-2."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _run_subset(case, cache, scale, positions, q_bits=None):
    import torch
    from tests.helpers import dev_bits, out_f64
    q = dev_bits(case.q if q_bits is None else q_bits)
    lse = torch.full((len(case.lens), case.Hq), 123.0, dtype=torch.float32, device="cuda")
    out = cache.decode_attn_subset(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), q, case.lens,
                                   positions, scale, lse=lse)
    torch.cuda.synchronize()
    status = int(cache.decode_ws[:4].view(torch.int32)[0].item())
    return out_f64(out), lse.cpu().numpy().astype(np.float64), status


def _oracle_subset(case, b, scale, positions):
    from tests.helpers import f64
    from oracle import deltakv_oracle as O
    r = case.res[b]
    pos = np.asarray(positions, dtype=np.int64)
    pos = pos[pos < case.lens[b]]
    return O.decode_attn_subset(f64(case.q[b]), r["idx"], f64(r["zb_k"]), f64(r["zb_v"]), r["ref_k"], r["ref_v"],
                                f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]), scale, pos)


def _compare(case, got, lse, scale, positions):
    from tests.helpers import check_attention
    for b in range(len(case.lens)):
        want, wl = _oracle_subset(case, b, scale, positions[b])
        if np.all(np.isneginf(wl)):
            assert np.all(got[b] == 0) and np.all(np.isneginf(lse[b]))
            continue
        check_attention(got[b], want, f"seq {b}")
        assert np.max(np.abs(lse[b] - wl)) <= 2e-2, (b, np.max(np.abs(lse[b] - wl)))


@pytest.mark.parametrize("joint", [False, True])
def test_random_quarter_of_the_tokens(joint):
    from tests.helpers import Case
    from tests.test_gpu_decode import _setup
    case = Case(9100 + joint, [3000, 1777], Hkv=2, Hq=8, r=64, n_proto=32, joint=joint)
    cache = _setup(case, page_perm_seed=5)
    rng = np.random.default_rng(1)
    positions = [np.sort(rng.choice(L, L // 4, replace=False)) for L in case.lens]
    scale = 1.0 / np.sqrt(128)
    got, lse, status = _run_subset(case, cache, scale, positions)
    assert status == 0
    _compare(case, got, lse, scale, positions)


def test_page_clustered_selection_over_several_splits():
    """Whole pages picked at random from a long sequence (the shape a page-level sparse attention produces)."""
    from tests.helpers import Case
    from tests.test_gpu_decode import _setup
    case = Case(9200, [40000], Hkv=1, Hq=4, r=64, n_proto=64)
    cache = _setup(case)
    rng = np.random.default_rng(2)
    pages = np.sort(rng.choice(2500, 700, replace=False))
    positions = [(pages[:, None] * 16 + np.arange(16)[None, :]).ravel()]
    scale = 1.0 / np.sqrt(128)
    got, lse, status = _run_subset(case, cache, scale, positions)
    assert status == 0
    _compare(case, got, lse, scale, positions)


def test_selecting_everything_equals_the_full_attention():
    import torch
    from tests.helpers import Case, dev_bits, out_f64
    from tests.test_gpu_decode import _setup
    case = Case(9300, [1111, 530], Hkv=4, Hq=28, r=48, n_proto=16)
    cache = _setup(case)
    scale = 0.09
    positions = [np.arange(L) for L in case.lens]
    got, lse, status = _run_subset(case, cache, scale, positions)
    assert status == 0
    _compare(case, got, lse, scale, positions)
    full = out_f64(cache.decode_attn(dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]),
                                     dev_bits(case.q), case.lens, scale))
    torch.cuda.synchronize()
    assert np.max(np.abs(full - got)) <= 2.0 ** -7 * max(np.abs(full).max(), 2.0 ** -10)


def test_reference_tokens_only_single_token_and_empty_selection():
    from tests.helpers import Case, f64
    from oracle import deltakv_oracle as O
    from tests.test_gpu_decode import _setup
    case = Case(9400, [900, 900, 900], Hkv=2, Hq=4, r=32, n_proto=8)
    cache = _setup(case)
    positions = [np.arange(0, 900, 16), np.array([517]), np.array([], dtype=np.int64)]
    got, lse, status = _run_subset(case, cache, 0.1, positions)
    _compare(case, got, lse, 0.1, positions)
    # reference tokens attend as their raw rows; a single token returns its reconstructed value row
    want_refs, _ = O.dense_attention(f64(case.q[0]), f64(case.K[0][::16]), f64(case.V[0][::16]), 0.1)
    assert np.max(np.abs(got[0] - want_refs)) <= 2e-2
    r = case.res[1]
    _, vh = O.reconstruct(r["idx"], f64(r["zb_k"]), f64(r["zb_v"]), r["ref_k"], r["ref_v"],
                          f64(case.W["w_up_k_bf16"]), f64(case.W["w_up_v_bf16"]))
    for g in range(4):
        assert np.max(np.abs(got[1, g] - vh[517, g // 2])) <= 2e-2
    assert np.all(got[2] == 0) and np.all(np.isneginf(lse[2]))


@pytest.mark.parametrize("joint", [False, True])
def test_selected_tokens_far_below_a_sink_reference(joint):
    """Reference 0 is made an attention sink: its key is aligned with the query so that its score lies more than 60
    nats above the logit of every selected token (none of which is the sink).  The streaming kernel's exponent frame
    hangs on the largest reference score, so all selected weights underflow there; the rows are recomputed by the
    rescue kernel against their own largest logit and match the oracle.  A second sequence of the same call, with
    an ordinary selection, keeps the streaming result."""
    from tests.helpers import Case, f64
    from tests.test_gpu_decode import _setup
    from synthetic import generator as G
    case = Case(9600 + joint, [1500, 800], Hkv=2, Hq=8, r=64, n_proto=16, joint=joint)
    scale = 0.1
    q = f64(case.q)
    for h in range(2):                     # sink key of kv-head h: along the mean of its four queries, length 200
        d = q[0, 4 * h:4 * h + 4].mean(0)
        sink = G.f32_to_bf16_bits((200.0 * d / np.linalg.norm(d)).astype(np.float32))
        case.K[0][0, h] = sink
        case.res[0]["ref_k"][0, h] = f64(sink)
    rng = np.random.default_rng(4)
    cand = np.flatnonzero((case.res[0]["idx"] != 0).all(axis=1))          # tokens that do not lean on the sink
    positions = [np.sort(rng.choice(cand, 300, replace=False)), np.sort(rng.choice(800, 200, replace=False))]
    r = case.res[0]
    kh = r["ref_k"][r["idx"], np.arange(2)[None, :]] + f64(r["zb_k"]) @ f64(case.W["w_up_k_bf16"])
    for g in range(8):
        sel = scale * kh[positions[0], g // 4] @ q[0, g]
        assert scale * float(r["ref_k"][0, g // 4] @ q[0, g]) - sel.max() > 60.0
    cache = _setup(case)
    got, lse, status = _run_subset(case, cache, scale, positions)
    assert status & 1
    _compare(case, got, lse, scale, positions)


def test_positions_past_the_sequence_are_ignored_and_bad_arguments_rejected():
    import torch
    from paper_2602_08005_amd import binding as B
    from tests.helpers import Case, dev_bits
    from tests.test_gpu_decode import _setup
    case = Case(9500, [333], Hkv=2, Hq=8, r=64, n_proto=8)
    cache = _setup(case)
    positions = [np.array([0, 5, 100, 332, 333, 334, 351, 5000])]
    got, lse, status = _run_subset(case, cache, 0.1, positions)
    _compare(case, got, lse, 0.1, positions)
    sp, sm, n_dev, n_host = cache.selection(positions)
    args = (cache.dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.block_tables,
            cache.ref_tables, dev_bits(case.W["w_up_k_bf16"]), dev_bits(case.W["w_up_v_bf16"]), dev_bits(case.q),
            torch.tensor([333], dtype=torch.int32, device="cuda"), [333])
    out = torch.empty(8 * 128, dtype=torch.int16, device="cuda")
    assert B.decode_attn_subset(*args, sp, sm, n_dev, [sp.shape[1] + 1], 0.1, out, None, cache.decode_ws,
                                check=False) == B.E_INVALID_ARG
    assert B.decode_attn_subset(*args, sp, sm, n_dev, [-1], 0.1, out, None, cache.decode_ws,
                                check=False) == B.E_INVALID_ARG
