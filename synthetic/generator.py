"""Seeded synthetic inputs for the DeltaKV hot path.

This module only *draws inputs*: raw K/V states, queries, projection matrices,
sequence lengths and page permutations.  It holds none of the method's
arithmetic (no retrieval, residual, projection or attention) and is the one
module that both the CPU oracle's tests and the HIP path's tests/bench may use,
so that both sides see bit-identical bf16 buffers.

Recipe (stands in for the real-model KV the paper analyses in its section 3:
a dominant component shared between distant tokens plus a low-energy
token-specific part).  Per kv-head h and per stream in {K, V}:

    x[t] = proto[h, stream][c[t, h]] + B[h, stream] @ coef[t, h, stream] + 0.05 * eps

with proto ~ N(0,1)^{n_proto x D}, class id c[t, h] uniform (one id per
(token, head), shared by K and V), B an orthonormal D x 16 basis, coef ~
N(0, variance 2)^16 and eps ~ N(0,1)^D.  Everything is drawn in fp32 from
numpy's counter-based Philox generator and rounded to bf16 (round to nearest
even); buffers are returned as uint16 bit patterns.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 260208005


def seed_for(config: int, layer: int = 0, extra: int = 0) -> int:
    return BASE_SEED + 1000 * int(config) + int(layer) + 1_000_000 * int(extra)


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def orthonormal(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """rows x cols matrix with orthonormal columns (fp64), cols <= rows."""
    a = rng.standard_normal((rows, cols))
    qm, rm = np.linalg.qr(a)
    return qm * np.sign(np.diag(rm))[None, :]


def make_kv(seed: int, n_tokens: int, n_kv_heads: int, head_dim: int = 128, n_proto: int = 256,
            basis_dim: int = 16, coef_var: float = 2.0, noise: float = 0.05, threads: int = 8,
            chunk: int = 16384):
    """Raw K and V, each uint16 bf16 bits of shape [n_tokens, n_kv_heads, head_dim].

    Also returns the class ids c[t, h] (int32), which tests use to reason about
    which reference a token should retrieve.
    """
    H, D = n_kv_heads, head_dim
    g0 = _rng(seed, 0)
    proto = g0.standard_normal((2, H, n_proto, D), dtype=np.float32)
    basis = np.stack([[orthonormal(g0, D, basis_dim).astype(np.float32) for _ in range(H)]
                      for _ in range(2)])                       # [2, H, D, basis_dim]
    K = np.empty((n_tokens, H, D), dtype=np.uint16)
    V = np.empty((n_tokens, H, D), dtype=np.uint16)
    cls = np.empty((n_tokens, H), dtype=np.int32)
    sd = np.float32(np.sqrt(coef_var))

    def work(ci: int):
        t0 = ci * chunk
        t1 = min(n_tokens, t0 + chunk)
        n = t1 - t0
        g = _rng(seed, 1 + ci)
        c = g.integers(0, n_proto, size=(n, H), dtype=np.int32)
        cls[t0:t1] = c
        for s, out in ((0, K), (1, V)):
            coef = g.standard_normal((n, H, basis_dim), dtype=np.float32) * sd
            eps = g.standard_normal((n, H, D), dtype=np.float32)
            x = eps * np.float32(noise)
            for h in range(H):
                x[:, h, :] += proto[s, h][c[:, h]]
                x[:, h, :] += coef[:, h, :] @ basis[s, h].T
            out[t0:t1] = f32_to_bf16_bits(x)

    n_chunks = (n_tokens + chunk - 1) // chunk
    if n_chunks <= 1 or threads <= 1:
        for ci in range(n_chunks):
            work(ci)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(n_chunks)))
    return K, V, cls


def make_queries(seed: int, batch: int, n_q_heads: int, head_dim: int = 128) -> np.ndarray:
    """q ~ N(0,1), bf16 bits, shape [batch, n_q_heads, head_dim]."""
    g = _rng(seed, 7_000_001)
    return f32_to_bf16_bits(g.standard_normal((batch, n_q_heads, head_dim), dtype=np.float32))


def make_projections(seed: int, head_dim: int, rank: int, joint: bool = False, recipe: str = "independent"):
    """Random orthonormal down-projections and up-projections.

    recipe:
      "independent" (default; what the parity tests feed both sides): the four matrices are separate draws, so a
                   path that read one of them in place of another gives a different result.  SPLIT: W_dK and W_dV
                   are two orthonormal head_dim x rank draws and W_uK, W_uV the transposes of two further draws;
                   JOINT: [W_dK; W_dV] is one orthonormal (2*head_dim) x rank draw and [W_uK | W_uV] the transpose
                   of another.
      "paired"     distinct streams, each with W_u = W_d^T (reconstruction is the orthogonal projection of the
                   residual): SPLIT two draws, JOINT the two halves of one (2*head_dim) x rank draw.
      "baseline"   the benchmark's stated weights: SPLIT one orthonormal head_dim x rank matrix used for both
                   streams (W_dK = W_dV), W_u = W_d^T; JOINT as "paired".

    Returns a dict with fp64 ("*_f64", unrounded) and bf16-bit ("*_bf16")
    versions of w_down_k, w_down_v [head_dim, rank] and w_up_k, w_up_v [rank, head_dim].
    """
    if recipe not in ("independent", "paired", "baseline"):
        raise ValueError(recipe)
    g = _rng(seed, 7_000_002)
    D = head_dim
    if joint:
        w = orthonormal(g, 2 * D, rank)
        wdk, wdv = w[:D].copy(), w[D:].copy()
    else:
        wdk = orthonormal(g, D, rank)
        wdv = wdk.copy() if recipe == "baseline" else orthonormal(g, D, rank)
    if recipe == "independent":
        if joint:
            u = orthonormal(g, 2 * D, rank)
            wuk, wuv = u[:D].T.copy(), u[D:].T.copy()
        else:
            wuk, wuv = orthonormal(g, D, rank).T.copy(), orthonormal(g, D, rank).T.copy()
    else:
        wuk, wuv = wdk.T.copy(), wdv.T.copy()
    out = {"w_down_k_f64": wdk, "w_down_v_f64": wdv, "w_up_k_f64": wuk, "w_up_v_f64": wuv}
    for k in ("w_down_k", "w_down_v", "w_up_k", "w_up_v"):
        out[k + "_bf16"] = f32_to_bf16_bits(out[k + "_f64"].astype(np.float32))
    return out


def make_mlp_compressor(seed: int, head_dim: int, rank: int, hidden: int, swiglu: bool = False):
    """Random weights of a non-linear compressor over the per-head K||V vector (2 * head_dim inputs): W1 (and, for
    SwiGLU, Wg) ~ N(0, 1 / n_in), b1 ~ N(0, 0.01), W2 ~ N(0, 1 / hidden).  Returns fp64 ("*_f64": the values of the
    bf16-rounded weights) and bf16-bit ("*_bf16") arrays; b1 stays fp32 ("b1_f32")."""
    g = _rng(seed, 7_000_005)
    n_in = 2 * head_dim
    out = {}
    names = ["w1", "w2"] + (["wg"] if swiglu else [])
    shapes = {"w1": (n_in, hidden), "wg": (n_in, hidden), "w2": (hidden, rank)}
    for k in names:
        w = g.standard_normal(shapes[k]).astype(np.float32) / np.float32(np.sqrt(shapes[k][0]))
        out[k + "_bf16"] = f32_to_bf16_bits(w)
        out[k + "_f64"] = bf16_bits_to_f32(out[k + "_bf16"]).astype(np.float64)
    out["b1_f32"] = (0.1 * g.standard_normal(hidden)).astype(np.float32)
    return out


def loguniform_lengths(seed: int, n_seqs: int, lo: int, hi: int) -> np.ndarray:
    """Sequence lengths floor(exp(U(ln lo, ln hi))), int32."""
    g = _rng(seed, 7_000_003)
    u = g.uniform(np.log(lo), np.log(hi), size=n_seqs)
    return np.clip(np.floor(np.exp(u)), lo, hi).astype(np.int32)


def page_permutation(seed: int, n_needed: int, pool_pages: int) -> np.ndarray:
    """n_needed distinct page ids drawn at random from [0, pool_pages), int32."""
    g = _rng(seed, 7_000_004)
    return g.permutation(pool_pages)[:n_needed].astype(np.int32)
