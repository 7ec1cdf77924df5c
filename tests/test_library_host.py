"""CPU-side tests of the C-ABI library: it loads, exports every declared symbol, its layout arithmetic is
consistent, and invalid arguments are rejected before anything touches a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2602_08005_amd as dk
from paper_2602_08005_amd import binding as B
from oracle import deltakv_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "deltakv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(deltakv_[a-z0-9_]+)\s*\(", hdr))
    assert {"deltakv_compress", "deltakv_decode_attn", "deltakv_paged_layout"} <= declared
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)
    assert dk.version() == 1
    assert dk.strerror(0) == "ok" and "unsupported" in dk.strerror(B.E_UNSUPPORTED)


def test_layout_sizes_and_strides():
    d = dk.make_dims(8, 32, 64, n_pages=128, n_ref_slots=128)
    L = dk.paged_layout(d, 1, 2048, 2048)
    assert L.n_streams == 2 and L.alignment == 256
    assert L.latent_pool_bytes == 128 * 8 * 2 * 16 * 64 * 2
    assert L.idx_pool_bytes == 128 * 8 * 16 * 4
    assert L.ref_pool_bytes == 8 * 2 * 128 * 128 * 2
    assert L.ref_norm_pool_bytes == 8 * 128 * 4
    assert L.latent_page_stride == 8 * L.latent_head_stride and L.latent_head_stride == 2 * 16 * 64
    assert L.decode_ws_bytes > 0 and L.compress_ws_bytes > 0
    dj = dk.make_dims(8, 32, 64, 128, 128, latent_mode=dk.JOINT)
    Lj = dk.paged_layout(dj, 1, 2048, 2048)
    assert Lj.n_streams == 1 and Lj.latent_pool_bytes * 2 == L.latent_pool_bytes


@pytest.mark.parametrize("rank", [16, 48, 64, 128])
def test_block_offsets_are_permutations_with_the_documented_formula(rank):
    d = dk.make_dims(4, 28, rank, 8, 8)
    for stream in (0, 1):
        off = dk.latent_block_offsets(d, stream)
        assert off.shape == (16, rank)
        assert sorted(off.ravel().tolist()) == list(range(16 * rank))
        for tok, c in ((0, 0), (5, 9), (15, rank - 1), (7, 16 % rank)):
            want = ((c // 8) * 16 + tok) * 8 + c % 8 if stream == 0 else \
                ((c // 16) * 64 + (tok // 4) * 16 + c % 16) * 4 + tok % 4
            assert off[tok, c] == want
    with pytest.raises(dk.DeltaKVError):
        dk.latent_block_offsets(dk.make_dims(4, 28, rank, 8, 8, latent_mode=dk.JOINT), 1)


@pytest.mark.parametrize("rank,mode", [(16, "joint"), (64, "joint"), (64, "split"), (128, "split"), (48, "joint")])
def test_4bit_record_offsets_tile_the_block_without_overlap(rank, mode):
    """Every (token, column) owns its own nibble, scales and zero points their own half-words behind the codes, and
    the whole record block (rank / 2 + 4 bytes per token) is covered exactly once."""
    from paper_2602_08005_amd import binding as B
    d = dk.make_dims(4, 28, rank, 8, 8, latent_mode=dk.JOINT if mode == "joint" else dk.SPLIT, latent_bits=4)
    for stream in range(1 if mode == "joint" else 2):
        ce, cs, se, ze = B.q4_block_offsets(d, stream)
        assert ce.shape == (16, rank) and se.shape == (16,)
        nibbles = (ce.astype(np.int64) * 4 + cs // 4).ravel()              # nibble index inside the block
        assert len(set(nibbles.tolist())) == 16 * rank and set(cs.ravel().tolist()) == {0, 4, 8, 12}
        assert nibbles.min() == 0 and nibbles.max() == 16 * rank - 1       # the codes fill the first 8 * rank bytes
        tail = sorted(se.tolist() + ze.tolist())
        assert tail == list(range(4 * rank, 4 * rank + 32))                 # 16 scales + 16 zero points behind them
    with pytest.raises(dk.DeltaKVError):
        B.q4_block_offsets(dk.make_dims(4, 28, rank, 8, 8), 0)             # bf16 latents: not this layout


def test_keep_ratio_matches_record_accounting():
    for mode, om in ((dk.SPLIT, O.SPLIT), (dk.JOINT, O.JOINT)):
        for r, s in ((64, 16), (48, 16), (64, 10)):
            d = dk.make_dims(8, 32, r, 8, 8, latent_mode=mode, ref_stride=s)
            assert dk.keep_ratio(d) == pytest.approx(O.record_keep_ratio(om, r, 128, s, norm_bytes=4), rel=1e-12)
    # the figures quoted for this build's two modes (index and norm included)
    assert dk.keep_ratio(dk.make_dims(8, 32, 64, 8, 8)) == pytest.approx((256 + 4 + 516 / 16) / 512)
    for r in (16, 64, 128):                    # 4-bit token-wise latents, single-stream layout
        d4 = dk.make_dims(8, 32, r, 8, 8, latent_mode=dk.JOINT, latent_bits=4)
        assert dk.keep_ratio(d4) == pytest.approx(O.record_keep_ratio_4bit(O.JOINT, r, 128, 16), rel=1e-12)
        L4 = dk.paged_layout(d4, 1, 16, 16)
        assert L4.latent_head_stride * 2 == 8 * r + 64 and L4.latent_pool_bytes == 8 * 8 * (8 * r + 64)


def test_bad_dims_are_rejected():
    def rc(**kw):
        args = dict(n_kv_heads=8, n_q_heads=32, rank=64, n_pages=8, n_ref_slots=8)
        args.update(kw)
        out = B.Layout()
        return B._lib.deltakv_paged_layout(C.byref(dk.make_dims(**args)), 1, 16, 16, C.byref(out))
    assert rc() == B.OK
    assert rc(head_dim=64) == B.E_UNSUPPORTED
    assert rc(page_tokens=32) == B.E_UNSUPPORTED
    assert rc(rank=40) == B.E_UNSUPPORTED and rc(rank=256) == B.E_UNSUPPORTED
    assert rc(n_q_heads=30) == B.E_UNSUPPORTED
    assert rc(n_kv_heads=1, n_q_heads=32) == B.E_UNSUPPORTED
    assert rc(rank=0) == B.E_INVALID_ARG and rc(ref_stride=0) == B.E_INVALID_ARG
    assert rc(latent_mode=7) == B.E_INVALID_ARG
    assert rc(metric=1) == B.OK and rc(metric=2) == B.E_INVALID_ARG
    out = B.Layout()
    d = dk.make_dims(8, 32, 64, 8, 8)
    assert B._lib.deltakv_paged_layout(None, 1, 16, 16, C.byref(out)) == B.E_INVALID_ARG
    assert B._lib.deltakv_paged_layout(C.byref(d), 0, 16, 16, C.byref(out)) == B.E_INVALID_ARG
    assert B._lib.deltakv_paged_layout(C.byref(d), 1, 16, 0, C.byref(out)) == B.E_INVALID_ARG
    assert B._lib.deltakv_paged_layout(C.byref(d), 1, 16, 16, None) == B.E_INVALID_ARG


def test_entry_points_reject_null_and_inconsistent_arguments_without_a_device():
    d = dk.make_dims(2, 8, 64, 8, 8)
    L = dk.paged_layout(d, 2, 64, 128)
    buf = np.zeros(4096, dtype=np.uint8)
    p = buf.ctypes.data + (256 - buf.ctypes.data % 256) % 256      # 256-aligned host address (never dereferenced)
    sl = np.array([40, 128], dtype=np.int32)
    lib = B._lib
    vp = C.c_void_p
    def decode(**kw):
        a = dict(dims=C.byref(d), lay=C.byref(L), lat=p, idx=p, ref=p, bt=p, bts=8, rt=p, rts=8, wuk=p, wuv=p, q=p,
                 sl=p, slh=sl.ctypes.data, batch=2, scale=0.1, out=p, lse=None, ws=p, wsb=L.decode_ws_bytes, st=None)
        a.update(kw)
        return lib.deltakv_decode_attn(a["dims"], a["lay"], a["lat"], a["idx"], a["ref"], a["bt"], a["bts"], a["rt"],
                                       a["rts"], a["wuk"], a["wuv"], a["q"], a["sl"], a["slh"], a["batch"], a["scale"],
                                       a["out"], a["lse"], a["ws"], a["wsb"], a["st"])
    assert decode(lat=None) == B.E_INVALID_ARG
    assert decode(q=None) == B.E_INVALID_ARG
    assert decode(slh=None) == B.E_INVALID_ARG
    assert decode(batch=-1) == B.E_INVALID_ARG
    assert decode(batch=0) == B.OK
    assert decode(ws=None) == B.E_WORKSPACE
    assert decode(ws=p + 8) == B.E_WORKSPACE
    assert decode(wsb=64) == B.E_WORKSPACE
    assert decode(bts=4) == B.E_INVALID_ARG          # 128 tokens need 8 pages per sequence
    assert decode(rts=4) == B.E_INVALID_ARG
    assert decode(scale=float("nan")) == B.E_INVALID_ARG
    bad = np.array([40, -1], dtype=np.int32)
    assert decode(slh=bad.ctypes.data) == B.E_INVALID_ARG
    big = np.array([40, 129], dtype=np.int32)         # more tokens than the pools hold
    assert decode(slh=big.ctypes.data, bts=16, rts=16) == B.E_INVALID_ARG

    cu = np.array([0, 3, 5], dtype=np.int32)
    lb = np.array([10, 0], dtype=np.int32)
    def comp(**kw):
        a = dict(dims=C.byref(d), lay=C.byref(L), lat=p, idx=p, ref=p, nrm=p, bt=p, bts=8, rt=p, rts=8, wk=p, wv=p,
                 kn=p, vn=p, cu=p, cuh=cu.ctypes.data, lb=p, lbh=lb.ctypes.data, batch=2, ws=p, wsb=L.compress_ws_bytes,
                 st=None)
        a.update(kw)
        return lib.deltakv_compress(a["dims"], a["lay"], a["lat"], a["idx"], a["ref"], a["nrm"], a["bt"], a["bts"],
                                    a["rt"], a["rts"], a["wk"], a["wv"], a["kn"], a["vn"], a["cu"], a["cuh"], a["lb"],
                                    a["lbh"], a["batch"], a["ws"], a["wsb"], a["st"])
    assert comp(kn=None) == B.E_INVALID_ARG
    assert comp(nrm=None) == B.E_INVALID_ARG
    assert comp(cuh=None) == B.E_INVALID_ARG
    assert comp(batch=0) == B.OK
    assert comp(ws=None) == B.E_WORKSPACE
    assert comp(wsb=16) == B.E_WORKSPACE
    bad_cu = np.array([1, 3, 5], dtype=np.int32)
    assert comp(cuh=bad_cu.ctypes.data) == B.E_INVALID_ARG
    dec_cu = np.array([0, 3, 2], dtype=np.int32)
    assert comp(cuh=dec_cu.ctypes.data) == B.E_INVALID_ARG
    far = np.array([126, 0], dtype=np.int32)          # 126 + 3 tokens exceed the 8-page tables
    assert comp(lbh=far.ctypes.data) == B.E_INVALID_ARG
    empty = np.array([0, 0, 0], dtype=np.int32)
    assert comp(cuh=empty.ctypes.data, ws=None) == B.OK


def test_subset_and_raw_entry_points_reject_bad_arguments_without_a_device():
    d = dk.make_dims(2, 8, 64, 8, 8)
    L = dk.paged_layout(d, 2, 64, 128)
    buf = np.zeros(4096, dtype=np.uint8)
    p = buf.ctypes.data + (256 - buf.ctypes.data % 256) % 256      # aligned host address, never dereferenced
    sl = np.array([40, 128], dtype=np.int32)
    ns = np.array([2, 3], dtype=np.int32)
    lib = B._lib
    def subset(**kw):
        a = dict(sp=p, sm=p, ss=4, nd=p, nh=ns.ctypes.data, batch=2, ws=p)
        a.update(kw)
        return lib.deltakv_decode_attn_subset(C.byref(d), C.byref(L), p, p, p, p, 8, p, 8, p, p, p, p, sl.ctypes.data,
                                              a["sp"], a["sm"], a["ss"], a["nd"], a["nh"], a["batch"], 0.1, p, None,
                                              a["ws"], L.decode_ws_bytes, None)
    assert subset(sp=None) == B.E_INVALID_ARG
    assert subset(sm=None) == B.E_INVALID_ARG
    assert subset(nh=None) == B.E_INVALID_ARG
    assert subset(ss=0) == B.E_INVALID_ARG
    assert subset(ss=2) == B.E_INVALID_ARG            # a sequence lists 3 pages, the rows hold 2
    neg = np.array([2, -1], dtype=np.int32)
    assert subset(nh=neg.ctypes.data) == B.E_INVALID_ARG
    assert subset(batch=0) == B.OK
    assert subset(ws=None) == B.E_WORKSPACE

    def raw(**kw):
        a = dict(sp=None, sm=None, ss=0, nd=None, nh=None, rk=p, rv=p, rl=p, cap=16, batch=2, ws=p)
        a.update(kw)
        return lib.deltakv_decode_attn_raw(C.byref(d), C.byref(L), p, p, p, p, 8, p, 8, p, p, p, p, sl.ctypes.data,
                                           a["sp"], a["sm"], a["ss"], a["nd"], a["nh"], a["rk"], a["rv"], a["rl"],
                                           a["cap"], a["batch"], 0.1, p, None, a["ws"], L.decode_ws_bytes, None)
    assert raw(rk=None) == B.E_INVALID_ARG
    assert raw(rv=None) == B.E_INVALID_ARG
    assert raw(rl=None) == B.E_INVALID_ARG
    assert raw(cap=-1) == B.E_INVALID_ARG
    assert raw(rk=p + 8) == B.E_INVALID_ARG           # misaligned rows
    assert raw(cap=4097) == B.E_UNSUPPORTED
    assert raw(sp=p, sm=None) == B.E_INVALID_ARG      # a selection needs all of its arguments
    assert raw(batch=0) == B.OK
    assert raw(ws=None) == B.E_WORKSPACE
    assert raw(cap=0, rk=None, rv=None, rl=None, batch=0) == B.OK
