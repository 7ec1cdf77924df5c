"""Shared helpers of the GPU parity tests: build a case with the generator, compress it with the
oracle, and place it in a PagedCache."""
import numpy as np

from oracle import deltakv_oracle as O
from synthetic import generator as G

f64 = O.bf16_bits_to_f64


def dev_bits(bits):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()


def out_f64(t):
    return f64(t.detach().cpu().numpy().view(np.uint16))


class Case:
    """One sequence per entry of `lens`; raw K/V, oracle-compressed cache, projections."""

    def __init__(self, seed, lens, Hkv=8, Hq=32, r=64, s=16, n_proto=64, joint=False, D=128, top_k=1, metric=O.COSINE):
        self.lens, self.Hkv, self.Hq, self.r, self.s, self.D, self.joint = list(lens), Hkv, Hq, r, s, D, joint
        self.top_k, self.metric = top_k, metric
        self.W = G.make_projections(seed, D, r, joint=joint)
        self.K, self.V, self.res = [], [], []
        mode = O.JOINT if joint else O.SPLIT
        for b, L in enumerate(self.lens):
            K, V, _ = G.make_kv(seed + 17 * b, max(L, 1), Hkv, D, n_proto=n_proto)
            K, V = K[:L], V[:L]
            self.K.append(K)
            self.V.append(V)
            if L > 0:
                self.res.append(O.compress(f64(K), f64(V), f64(self.W["w_down_k_bf16"]), f64(self.W["w_down_v_bf16"]),
                                           s=s, mode=mode, top_k=top_k, metric=metric))
            else:
                self.res.append(None)
        self.q = G.make_queries(seed, len(self.lens), Hq, D)

    def oracle_decode(self, b, scale, q=None):
        r = self.res[b]
        qq = f64(self.q[b]) if q is None else q
        return O.decode_attn_direct(qq, r["idx"], f64(r["zb_k"]), f64(r["zb_v"]), r["ref_k"], r["ref_v"],
                                    f64(self.W["w_up_k_bf16"]), f64(self.W["w_up_v_bf16"]), scale)


def check_attention(got, want, what="", scale_with_magnitude=False):
    """Spec bar: max-abs <= 2e-2; plus a relative L2 bar so that near-zero outputs cannot pass vacuously.
    scale_with_magnitude: for cases built to have outputs well above 1 (a handful of attended tokens): the output
    is stored as bf16, whose half-step alone is 7.8e-3 between 2 and 4 and 1.6e-2 between 4 and 8, so the absolute
    bar grows in proportion once the largest expected output exceeds 2."""
    err = float(np.max(np.abs(got - want)))
    rel = float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))
    bar = 2e-2 * max(1.0, float(np.max(np.abs(want))) / 2.0) if scale_with_magnitude else 2e-2
    assert err <= bar, f"{what}: max-abs {err}"
    assert rel <= 1e-2, f"{what}: relative L2 {rel}"
    return err, rel


def check_q4_records(z, d, codes, sb, zb):
    """Validity of 4-bit token-wise records (codes [..., r], bf16 bits of scale and zero point [...]) for latents
    whose float64 values are z [..., r] and whose computed values lie within d [..., r] of them.  A record passes iff
    it is what the definition (scale = (max - min)/15 and zero = min stored as bf16; code = the nearest level of
    (z - zero)/scale, halves to even, clamped to 0..15) gives for SOME latent inside that error bound:
      * zero point: a bf16 value between bf16(min - dmax) and bf16(min + dmax) -- one value, two only where the minimum
        sits at a bf16 rounding boundary; scale likewise from (max - min -/+ 2 dmax)/15, with 2^-21 relative for an
        fp32 product with 1/15;
      * every code c, on the grid of the record's OWN scale and zero point: the unrounded position x = (z - zero)/scale
        has |x - c| <= 1/2 + eps (or lies beyond the end level that c clamps to), eps = d/scale + 2^-17 (a position
        formed in fp32 from a reciprocal: three roundings of a number below 16);
      * scale 0 (constant latent): all codes 0.
    A code one level off anywhere but at a half-way point fails."""
    f, bits = O.bf16_bits_to_f64, O.f64_to_bf16_bits
    dmax = d.max(axis=-1)
    mn, mx = z.min(axis=-1), z.max(axis=-1)
    zero, scale = f(zb), f(sb)
    assert np.all((zero >= f(bits(mn - dmax))) & (zero <= f(bits(mn + dmax)))), "zero point outside its rounding window"
    lo = np.maximum(mx - mn - 2 * dmax, 0.0) / 15.0 * (1 - 2.0 ** -21)
    hi = (mx - mn + 2 * dmax) / 15.0 * (1 + 2.0 ** -21)
    assert np.all((scale >= f(bits(lo))) & (scale <= f(bits(hi)))), "scale outside its rounding window"
    x = O.code_positions_4bit(z, sb, zb)
    c = codes.astype(np.float64)
    eps = d / np.where(scale > 0, scale, 1.0)[..., None] + 2.0 ** -17
    ok = (np.abs(x - c) <= 0.5 + eps) | ((c == 0) & (x <= 0.5 + eps)) | ((c == 15) & (x >= 14.5 - eps))
    ok = np.where((scale > 0)[..., None], ok, c == 0)
    assert np.all(ok), f"{int((~ok).sum())} codes off their level (worst |x - c| = {float(np.abs(x - c)[~ok].max())})"
