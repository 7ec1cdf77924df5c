"""CPU oracle for the DeltaKV hot path (TEST INFRASTRUCTURE, not product code).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module.  It shares no code with the HIP path and imports nothing from it.

Everything is plain numpy in float64 over the exact values of the bf16 inputs.
Library matmuls are used as single steps; there is no tiling, fusion or
reordering beyond what the definitions state.

What it follows (paper: "DeltaKV: Residual-Based KV Cache Compression via
Long-Range Similarity"):

* strided reference set T = {kv_t : t mod s = 0, t < i}        -- section 4.1
* retrieval of the nearest references (arg top-k; k = 1 by
  default) and the mean of the retrieved set as the reference    -- section 4.1
* residual against the retrieved reference, then the
  down-projection encoder                                        -- section 4.1 (compressor), appendix B.2 (lifecycle steps 1-3)
* reconstruction KV_hat = f_d(z) + KV_ref with the bias-free
  linear decoder f_d(z) = z W_d                                  -- section 4.1 (reconstruction), section 5.3 (light decompressor)
* keep-ratio accounting KR                                       -- appendix D, equation (5)
* attention over a selected subset of the cached tokens
  (selective decompression under a sparse attention mask)        -- section 4.2, appendix B.2

Readings where the paper is silent or differs from the build target are listed
in the repository's design notes; the ones that shape this file:
  - similarity is cosine over the per-(token, kv-head) vector K||V (256 values
    for head_dim 128); a zero-norm vector scores 0 against everything; the
    paper's own metric, squared L2 distance over the same vector, is the
    alternative (metric = L2);
  - k = 1 unless top_k says otherwise; ties go to the lowest reference ordinal; a token with fewer
    candidates than k takes all of them (the paper does not say);
  - positions are 0-indexed, token 0 is a reference, candidates are strictly
    earlier (ordinal j is token j*s < i);
  - a reference token is stored raw and attends as itself: idx = own ordinal,
    latent = 0;
  - SPLIT mode keeps one latent per stream (z_K = r_K W_dK, z_V = r_V W_dV),
    JOINT mode one latent per token-head (z = r_K W_dK + r_V W_dV, the paper's
    single latent over Concat(K, V));
  - latents are stored in bf16, rounded to nearest even from the float64 value.

Pins (tests/test_oracle_*.py): the paper's two worked KR rows and its dense-KV
size statement; brute-force retrieval with constructed ties; planted copies;
full-rank orthonormal reconstruction; zero residual == dense attention over the
gathered references; s = 1 == textbook attention (cross-checked with
torch.nn.functional.scaled_dot_product_attention); L = 1 and q = 0 closed
forms; direct == absorbed formulation; two-half log-sum-exp merge.  Absolute
latent / attention values for arbitrary inputs are printed nowhere in the paper:
for those, parity is pinned only through the invariants above.
"""
from __future__ import annotations

import numpy as np

SPLIT = 0
JOINT = 1


# ----------------------------------------------------------------------------
# bf16 <-> float64 (exact widening; direct round-to-nearest-even narrowing)
# ----------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (ties to even) of each float64, returned as float64.

    bf16 keeps 8 significant bits; its smallest subnormal is 2**-133.  The
    rounding is done once, directly from float64 (no intermediate fp32 step).
    """
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m * 2**e, 0.5 <= |m| < 1
    q = np.maximum(e - 8, -133)              # exponent of one unit in the last place
    y = np.rint(np.ldexp(x, -q))             # np.rint rounds half to even
    out = np.ldexp(y, q)
    big = np.abs(out) > 3.3895313892515355e38  # largest finite bf16
    out = np.where(big, np.copysign(np.inf, x), out)
    return np.where(np.isfinite(x), out, x)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    r = f64_round_to_bf16(x).astype(np.float32)          # exact: value is a bf16
    return (r.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------
# Keep-ratio accounting (appendix D, equation (5)) and cache sizes
# ----------------------------------------------------------------------------
def keep_ratio_eq5(n_full_layers: int, n_layers: int, s: int, dc_over_2dk: float,
                   latent_bits: int = 16, raw_bits: int = 16) -> float:
    """KR = L_full/L + L_sparse/L * (1/s + d_c/(2 d_k)); a latent stored in fewer
    bits than the raw cache scales the second term (section 5.3, 4-bit residuals)."""
    n_sparse = n_layers - n_full_layers
    per_layer = 1.0 / s + dc_over_2dk * (latent_bits / raw_bits)
    return n_full_layers / n_layers + n_sparse / n_layers * per_layer


def compute_ratio_eq6(n_full_layers: int, n_layers: int, budget: float) -> float:
    """CR = L_full/L * 100 % + L_sparse/L * r (appendix D, equation (6)): the dense layers attend every
    token, the compressed layers the fraction r that the sparse attention selects.  (The appendix's own
    worked table prints r itself -- 30.0 and 20.0 -- in its CR column, which is the second term's factor,
    not the value of the equation; the equation is what this function evaluates.)"""
    return n_full_layers / n_layers + (n_layers - n_full_layers) / n_layers * budget


def dense_kv_bytes(batch: int, seq_len: int, n_layers: int, n_kv_heads: int, head_dim: int,
                   bytes_per_value: int = 2) -> int:
    return batch * seq_len * n_layers * 2 * n_kv_heads * head_dim * bytes_per_value


def record_keep_ratio_4bit(mode: int, rank: int, head_dim: int, s: int) -> float:
    """As record_keep_ratio for 4-bit token-wise latents: rank/2 bytes of codes plus a bf16 scale and a
    bf16 zero point per latent, an int32 ordinal per token, and the raw bf16 reference (+ its fp32
    float) every s-th token."""
    streams = 1 if mode == JOINT else 2
    rec = streams * (rank / 2 + 4) + 4
    raw = 2 * head_dim * 2
    return (rec + (raw + 4) / s) / raw


def record_keep_ratio(mode: int, rank: int, head_dim: int, s: int, idx_bytes: int = 4,
                      value_bytes: int = 2, norm_bytes: int = 0) -> float:
    """Bytes kept per (token, kv-head) over the dense 2*head_dim values when every
    token stores a latent record (and an index) and every s-th token is also
    kept raw."""
    lat = (rank if mode == JOINT else 2 * rank) * value_bytes
    raw = 2 * head_dim * value_bytes
    return (lat + idx_bytes + (raw + norm_bytes) / s) / raw


# ----------------------------------------------------------------------------
# Retrieval (section 4.1: reference set T and arg top-k with k = 1)
# ----------------------------------------------------------------------------
def cosine_scores(a: np.ndarray, refs: np.ndarray) -> np.ndarray:
    """cos(a, refs[j]) for one vector a [n] against refs [m, n]; 0 where a norm is 0."""
    a = np.asarray(a, dtype=np.float64)
    refs = np.asarray(refs, dtype=np.float64)
    na = np.sqrt(np.dot(a, a))
    nb = np.sqrt(np.einsum("jn,jn->j", refs, refs))
    den = na * nb
    dots = refs @ a
    return np.where(den > 0.0, dots / np.where(den > 0.0, den, 1.0), 0.0)


def n_candidates(i: int, s: int) -> int:
    """Number of reference ordinals j with j*s < i."""
    return (i + s - 1) // s


def retrieve_one(kv: np.ndarray, i: int, h: int, s: int):
    """Best reference ordinal for token i, head h of kv [L, H, 2D]; returns (j, cos)."""
    m = n_candidates(i, s)
    c = cosine_scores(kv[i, h], kv[0:m * s:s, h])
    j = int(np.argmax(c))            # first occurrence of the maximum == lowest ordinal
    return j, float(c[j])


COSINE = 0
L2 = 1


def l2_scores(a: np.ndarray, refs: np.ndarray) -> np.ndarray:
    """-||a - refs[j]||^2 for one vector a [n] against refs [m, n]: section 4.1 retrieves the nearest tokens of the
    reference set by L2 distance (the largest of these scores is the nearest reference)."""
    a = np.asarray(a, dtype=np.float64)
    d = np.asarray(refs, dtype=np.float64) - a[None, :]
    return -np.einsum("jn,jn->j", d, d)


def code_positions_4bit(z: np.ndarray, scale_bits: np.ndarray, zero_bits: np.ndarray) -> np.ndarray:
    """Unrounded level positions (z - zero) / scale of latents z [..., r] on the 16-level grid of a stored
    record (bf16 scale and zero point, [...]); 0 where the scale is 0.  float64."""
    scale = bf16_bits_to_f64(scale_bits)[..., None]
    zero = bf16_bits_to_f64(zero_bits)[..., None]
    z = np.asarray(z, dtype=np.float64)
    return np.where(scale > 0.0, (z - zero) / np.where(scale > 0.0, scale, 1.0), 0.0)


def quantize_tokenwise_4bit(z: np.ndarray):
    """Token-wise asymmetric 4-bit quantisation of latent vectors (section 5.3, "Compatibility with
    Quantization": the token-wise scheme of KIVI applied to the compressed residuals only).  One group
    = the r values of one (token, head) latent; 16 levels between the group's smallest and largest value:
        scale = (max - min) / 15          zero = min             (both then stored as bf16)
        code  = clamp(round((z - zero) / scale), 0, 15)          (all codes 0 if scale = 0)
        value read back = scale * code + zero
    evaluated in float64 with the stored (bf16) scale and zero point, which are what a reader of the record
    has; round = to nearest, halves to the even level.
    z: [..., r].  Returns codes uint8 [..., r], scale bits uint16 [...], zero bits uint16 [...], and
    the values read back, float64 [..., r]."""
    z = np.asarray(z, dtype=np.float64)
    mn, mx = z.min(axis=-1), z.max(axis=-1)
    scale_b = f64_to_bf16_bits((mx - mn) / 15.0)
    zero_b = f64_to_bf16_bits(mn)
    pos = code_positions_4bit(z, scale_b, zero_b)
    codes = np.clip(np.rint(pos), 0, 15).astype(np.uint8)          # np.rint: halves to even
    back = bf16_bits_to_f64(scale_b)[..., None] * codes.astype(np.float64) + bf16_bits_to_f64(zero_b)[..., None]
    return codes, scale_b, zero_b, back


GELU = 0
SWIGLU = 1


def mlp_compressor(x: np.ndarray, mlp: dict) -> np.ndarray:
    """The non-linear compressor f_c of section 4.1 applied to vectors x [..., n_in] (n_in = 2 * head_dim: the
    per-head K||V vector).  mlp = {"kind", "w1" [n_in, d_h], "b1" [d_h], "w2" [d_h, r]} and, for SwiGLU, "wg"
    [n_in, d_h]:
        GELU   (the section's own form)          f_c(x) = GeLU(x W1 + b1) W2          (GeLU with the exact erf)
        SWIGLU (section 5.3, the heavy variant)  f_c(x) = (SiLU(x Wg) * (x W1 + b1)) W2
    The output bias of the section's formula is left out: the latent is a difference of two f_c values, in which it
    cancels.  float64."""
    from scipy.special import erf
    x = np.asarray(x, dtype=np.float64)
    u = x @ mlp["w1"] + mlp["b1"]
    if mlp["kind"] == GELU:
        h = 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))
    else:
        g = x @ mlp["wg"]
        h = g / (1.0 + np.exp(-g)) * u
    return h @ mlp["w2"]


def reference_mean(X: np.ndarray, idx: np.ndarray, s: int) -> np.ndarray:
    """Mean of the raw rows of the references each (token, head) retrieved (section 4.1, the reference
    representation: the mean of the retrieved set).  X [L, H, D] raw states; idx [n, H, k] reference
    ordinals (ordinal j is token j*s), -1 in unused slots; every (token, head) has at least one.
    Returns [n, H, D]."""
    idx = np.asarray(idx)
    valid = idx >= 0                                         # [n, H, k]
    tok = np.where(valid, idx, 0).astype(np.int64) * s
    hh = np.arange(X.shape[1])[None, :, None]
    rows = X[tok, hh] * valid[..., None]                     # [n, H, k, D]
    return rows.sum(axis=2) / valid.sum(axis=2)[..., None]


def compress(K: np.ndarray, V: np.ndarray, w_down_k: np.ndarray, w_down_v: np.ndarray,
             s: int = 16, mode: int = SPLIT, start: int = 0, token_block: int = 2048, metric: int = COSINE,
             latent_bits: int = 16, top_k: int = 1, mlp: dict = None):
    """Compress tokens start..L-1 of one sequence.

    K, V: float64 [L, H, D] -- the raw states of the WHOLE sequence so far (the
    references are the raw tokens at multiples of s).  w_down_*: float64 [D, r].

    Returns a dict of per-token results for tokens start..L-1 (index 0 of each
    array is token `start`):
      idx      int32   [n, H]      reference ordinal (own ordinal for reference tokens); with top_k > 1
                                   [n, H, top_k]: the top_k nearest references in order of rank (section 4.1,
                                   arg top-k; equal scores go to the lower ordinal first), -1 in the slots of a
                                   token that has fewer candidates than top_k; a reference token holds its own
                                   ordinal in slot 0 and -1 elsewhere.  The residual is taken against the MEAN of
                                   the retrieved references' raw rows (section 4.1, reference representation).
      cos      float64 [n, H]      the winning score: cosine (1.0 stored for reference tokens), or with
                                   metric = L2 minus the squared distance to the chosen reference
      z_k, z_v float64 [n, H, r]   unrounded latents (JOINT: z_v is z_k)
      zb_k, zb_v uint16 [n, H, r]  bf16 bits of the stored latents
    with latent_bits = 4 (4-bit token-wise latents) additionally
      q_k, q_v   uint8  [n, H, r]  codes;  qs_*, qz_* uint16 [n, H]: bf16 bits of scale and zero point
      zq_k, zq_v float64 [n, H, r] the latents as read back from the 4-bit record (what decode uses)
    and the reference pool of the whole sequence:
      ref_k, ref_v float64 [ceil(L/s), H, D]
    With `mlp` (see mlp_compressor; JOINT mode) the latent is f_c(token) - f_c(reference) instead of the projected
    residual; w_down_* are then ignored.
    """
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    L, H, D = K.shape
    r = mlp["w2"].shape[1] if mlp is not None else w_down_k.shape[1]
    n = L - start
    kv = np.concatenate([K, V], axis=2)                    # [L, H, 2D]
    refs = kv[0::s]                                        # ordinal j <-> token j*s
    ref_norm = np.sqrt(np.einsum("jhn,jhn->jh", refs, refs))
    idx = np.zeros((n, H), dtype=np.int32)
    idx_k = np.full((n, H, top_k), -1, dtype=np.int32)
    cos = np.zeros((n, H), dtype=np.float64)
    pos = np.arange(start, L)
    is_ref = (pos % s) == 0
    for b0 in range(0, n, token_block):
        b1 = min(n, b0 + token_block)
        p = pos[b0:b1]
        ncand = (p + s - 1) // s                           # candidates j < ncand
        mmax = int(ncand.max()) if len(p) else 0
        for h in range(H):
            a = kv[p, h]                                   # [nb, 2D]
            na = np.sqrt(np.einsum("in,in->i", a, a))
            if mmax == 0:
                continue
            if metric == L2:                               # the definition, token by token
                c = np.stack([l2_scores(a[i], refs[:mmax, h]) for i in range(len(p))])
            else:
                dots = a @ refs[:mmax, h].T                # [nb, mmax]
                den = na[:, None] * ref_norm[None, :mmax, h]
                c = np.where(den > 0.0, dots / np.where(den > 0.0, den, 1.0), 0.0)
            c = np.where(np.arange(mmax)[None, :] < ncand[:, None], c, -np.inf)
            j = np.argmax(c, axis=1)                       # lowest ordinal among equal maxima
            idx[b0:b1, h] = j
            cos[b0:b1, h] = c[np.arange(b1 - b0), j]
            if top_k > 1:
                # descending score, equal scores in ascending ordinal (a stable sort of the negated scores keeps
                # the ascending order of the columns among equals); slots beyond the candidates stay -1
                rank = np.argsort(-c, axis=1, kind="stable")[:, :top_k]
                ok = np.arange(rank.shape[1])[None, :] < ncand[:, None]
                idx_k[b0:b1, h, :rank.shape[1]] = np.where(ok, rank, -1)
    # reference tokens point at themselves and carry a zero latent
    idx[is_ref] = (pos[is_ref] // s)[:, None]
    cos[is_ref] = 0.0 if metric == L2 else 1.0
    hh = np.arange(H)[None, :]
    if top_k > 1:
        idx_k[:, :, 0] = np.where(is_ref[:, None], idx, idx_k[:, :, 0])
        idx_k[is_ref, :, 1:] = -1
        r_k = K[pos[:, None], hh] - reference_mean(K, idx_k, s)
        r_v = V[pos[:, None], hh] - reference_mean(V, idx_k, s)
    else:
        tok_ref = idx.astype(np.int64) * s                 # token position of the chosen reference
        r_k = K[pos[:, None], hh] - K[tok_ref, hh]         # [n, H, D]
        r_v = V[pos[:, None], hh] - V[tok_ref, hh]
    if mlp is not None:
        # non-linear compressor (section 4.1): the token's K||V and its reference's are compressed SEPARATELY and the
        # latent is the difference, z = f_c(kv) - f_c(kv_ref); one latent per (token, head), i.e. JOINT mode
        assert mode == JOINT, "the non-linear compressor produces the single latent over K||V"
        x_tok = np.concatenate([K[pos[:, None], hh], V[pos[:, None], hh]], axis=-1)
        x_ref = x_tok - np.concatenate([r_k, r_v], axis=-1)
        z_k = mlp_compressor(x_tok, mlp) - mlp_compressor(x_ref, mlp)
        z_v = z_k
    elif mode == SPLIT:
        z_k = r_k @ w_down_k
        z_v = r_v @ w_down_v
    else:
        z_k = r_k @ w_down_k + r_v @ w_down_v
        z_v = z_k
    z_k[is_ref] = 0.0
    if mode == SPLIT:
        z_v[is_ref] = 0.0
    out = {
        "idx": idx_k if top_k > 1 else idx, "cos": cos, "z_k": z_k, "z_v": z_v,
        "zb_k": f64_to_bf16_bits(z_k), "ref_k": K[0::s].copy(), "ref_v": V[0::s].copy(),
        "mode": mode, "s": s, "start": start,
    }
    out["zb_v"] = out["zb_k"] if mode == JOINT else f64_to_bf16_bits(z_v)
    if latent_bits == 4:
        out["q_k"], out["qs_k"], out["qz_k"], out["zq_k"] = quantize_tokenwise_4bit(z_k)
        if mode == JOINT:
            out["q_v"], out["qs_v"], out["qz_v"], out["zq_v"] = out["q_k"], out["qs_k"], out["qz_k"], out["zq_k"]
        else:
            out["q_v"], out["qs_v"], out["qz_v"], out["zq_v"] = quantize_tokenwise_4bit(z_v)
    return out


def cosine_of(K: np.ndarray, V: np.ndarray, i: int, h: int, j: int, s: int) -> float:
    """cos between token i and reference ordinal j for head h (float64)."""
    a = np.concatenate([K[i, h], V[i, h]]).astype(np.float64)
    b = np.concatenate([K[j * s, h], V[j * s, h]]).astype(np.float64)
    return float(cosine_scores(a, b[None, :])[0])


# ----------------------------------------------------------------------------
# Reconstruction and decode attention
# ----------------------------------------------------------------------------
def reconstruct(idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v):
    """KV_hat = reference + z W_up for every (token, head).  Shapes: idx [L,H] (one reference) or
    [L,H,k] (the mean of the references in the slots that are not -1: section 4.1, the decoded
    residual is added back to the mean reference), z_* [L,H,r], ref_* [n_ref,H,D], w_up_* [r,D];
    all float64."""
    if idx.ndim == 3:
        base_k, base_v = reference_mean(ref_k, idx, 1), reference_mean(ref_v, idx, 1)
    else:
        hh = np.arange(idx.shape[1])[None, :]
        base_k, base_v = ref_k[idx, hh], ref_v[idx, hh]
    k_hat = base_k + z_k @ w_up_k
    v_hat = base_v + z_v @ w_up_v
    return k_hat, v_hat


def dense_attention(q, K, V, scale):
    """Softmax attention of one query token over L cached tokens with grouped
    query heads: q [Hq, D], K/V [L, Hkv, D]; q-head g reads kv-head g // (Hq/Hkv).
    Returns out [Hq, D] and the natural-log log-sum-exp of the scaled logits [Hq]."""
    q = np.asarray(q, dtype=np.float64)
    Hq, D = q.shape
    L, Hkv, _ = K.shape
    G = Hq // Hkv
    out = np.zeros((Hq, D))
    lse = np.zeros(Hq)
    for g in range(Hq):
        h = g // G
        logit = scale * (K[:, h, :] @ q[g])
        m = np.max(logit)
        e = np.exp(logit - m)
        den = np.sum(e)
        out[g] = (e / den) @ V[:, h, :]
        lse[g] = m + np.log(den)
    return out, lse


def decode_attn_direct(q, idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v, scale):
    """Reconstruct every cached token, then attend (the definition)."""
    k_hat, v_hat = reconstruct(idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v)
    return dense_attention(q, k_hat, v_hat, scale)


def rope_rotate(x, positions, base: float = 10000.0):
    """Rotary position embedding of x [..., D] at integer positions [...] (broadcast against x's leading axes):
    dimension pair (i, i + D/2) is rotated by the angle position * base**(-2i/D), i = 0 .. D/2 - 1 (the
    "rotate-half" pairing of the Llama / Qwen families the paper evaluates).  float64."""
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    half = D // 2
    inv_freq = base ** (-np.arange(half, dtype=np.float64) * 2.0 / D)
    ang = np.asarray(positions, dtype=np.float64)[..., None] * inv_freq              # [..., D/2]
    c, s_ = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s_, x2 * c + x1 * s_], axis=-1)


def decode_attn_rope(q_rot, idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v, scale, base: float = 10000.0, positions=None):
    """Decode attention when the model applies rotary position embedding to keys: the cache holds PRE-RoPE
    states (section 4.1: every operation of the method works on pre-RoPE key-value states, to keep the
    representations position-invariant), so a key is reconstructed, K_hat = reference + z W_uK, and THEN rotated
    at its token's position before it meets the query (appendix B.5 names the fused de-/re-rotation as future
    work).  q_rot [Hq, D] is the query already rotated at its own position; cached token t has position t unless
    `positions` [L] says otherwise; values carry no rotation.  The definition: reconstruct, rotate, attend."""
    k_hat, v_hat = reconstruct(idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v)
    pos = np.arange(k_hat.shape[0]) if positions is None else np.asarray(positions)
    return dense_attention(q_rot, rope_rotate(k_hat, pos[:, None], base), v_hat, scale)


def decode_attn_subset(q, idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v, scale, positions):
    """Attention over the selected cached tokens only: section 4.2 ("Inference with Sparse
    Attention": selective decompression reconstructs just the KV pairs the sparse attention mask
    asks for) and appendix B.2 (view construction: index resolution, batch reconstruction).
    positions: distinct token positions; the definition is reconstruct-those-then-attend.
    An empty selection gives out = 0 and lse = -inf."""
    pos = np.asarray(positions, dtype=np.int64).reshape(-1)
    if pos.size == 0:
        return np.zeros((q.shape[0], ref_v.shape[-1])), np.full(q.shape[0], -np.inf)
    return decode_attn_direct(q, idx[pos], z_k[pos], z_v[pos], ref_k, ref_v, w_up_k, w_up_v, scale)


def decode_attn_with_raw(q, idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v, scale, raw_k, raw_v, positions=None):
    """Attention over the cached tokens (all of them, or the selected positions) together with a
    segment of tokens held raw: appendix B.2 keeps sink and recent tokens at full precision in a
    pool of their own, and the attention view stitches those static slots together with the
    reconstructed ones.  raw_k / raw_v [n_raw, Hkv, D] are tokens that are NOT in the cache; the
    definition is: reconstruct the cached tokens, put the raw rows beside them, attend.
    Nothing at all to attend gives out = 0 and lse = -inf."""
    pos = np.arange(idx.shape[0]) if positions is None else np.asarray(positions, dtype=np.int64).reshape(-1)
    k_hat, v_hat = reconstruct(idx[pos], z_k[pos], z_v[pos], ref_k, ref_v, w_up_k, w_up_v)
    K = np.concatenate([k_hat, np.asarray(raw_k, dtype=np.float64)], axis=0)
    V = np.concatenate([v_hat, np.asarray(raw_v, dtype=np.float64)], axis=0)
    if K.shape[0] == 0:
        return np.zeros((q.shape[0], ref_v.shape[-1])), np.full(q.shape[0], -np.inf)
    return dense_attention(q, K, V, scale)


def decode_attn_absorbed(q, idx, z_k, z_v, ref_k, ref_v, w_up_k, w_up_v, scale):
    """Same quantity through the linearity of the decoder: the query is pulled
    through W_up once, scores split into a per-reference part and a latent part,
    and the value sum splits into a per-reference weight sum and a latent sum.
    Written independently of decode_attn_direct; used only as a cross-check."""
    q = np.asarray(q, dtype=np.float64)
    Hq, D = q.shape
    L, Hkv = idx.shape
    n_ref = ref_k.shape[0]
    G = Hq // Hkv
    out = np.zeros((Hq, D))
    lse = np.zeros(Hq)
    for g in range(Hq):
        h = g // G
        q_lat = w_up_k @ q[g]                              # [r]
        s_ref = ref_k[:, h, :] @ q[g]                      # [n_ref]
        logit = scale * (s_ref[idx[:, h]] + z_k[:, h, :] @ q_lat)
        m = np.max(logit)
        e = np.exp(logit - m)
        den = np.sum(e)
        w = np.bincount(idx[:, h], weights=e, minlength=n_ref)
        out[g] = (w @ ref_v[:, h, :] + (e @ z_v[:, h, :]) @ w_up_v) / den
        lse[g] = m + np.log(den)
    return out, lse


def merge_partials(outs, lses):
    """Combine attention results over disjoint token sets from their outputs and
    log-sum-exps (what a split-KV kernel's final step must equal)."""
    lses = np.asarray(lses, dtype=np.float64)              # [n_parts, Hq]
    outs = np.asarray(outs, dtype=np.float64)              # [n_parts, Hq, D]
    m = np.max(lses, axis=0)
    w = np.exp(lses - m[None, :])
    den = np.sum(w, axis=0)
    out = np.einsum("ph,phd->hd", w, outs) / den[:, None]
    return out, m + np.log(den)
