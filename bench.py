#!/usr/bin/env python3
"""Benchmark of the DeltaKV hot path on one MI355X.

Default workload ("cfg3", the long-context decode configuration the headline metric is quoted on):
batch 8 x 131072 cached tokens, 32 layers run one after the other, 8 kv-heads x 128, 32 query heads,
latent rank 64, bf16, SPLIT latents.  One *step* = one decode-attention pass over the compressed cache
of every layer (32 library calls), i.e. one new token for each of the 8 sequences.

Inputs are seeded and synthetic (synthetic/generator.py).  Layer 0's cache is built for real by the
library's own compress kernels from generated K/V; the other 31 layers are distinct device copies of
that cache (same access pattern, separate memory, so nothing is reused across layers), each with its
own queries.  All inputs are resident in HBM before the timed region.

Prints ONE JSON line (metric, value, roofline of the dominant kernel, cpu_baseline = the CPU oracle
timed on a bounded sample in the same run).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def measured_traffic(key):
    """HBM bytes per launch of a workload's dominant kernel as counted by rocprofv3 (FETCH_SIZE / WRITE_SIZE runs
    scaled by a plain copy of known size).  The figures live in a tracked summary, profiles/hbm_traffic.md, one table
    row per workload key with the commit they were measured at; a shape that has no row reports null."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 3 and cells[0] == key:
                    return int(cells[2].replace("_", "").replace(",", ""))
    except (OSError, ValueError):
        pass
    return None


def timing_begin_sampled(B, calls):
    """Start the library's per-kernel HIP-event timing for a timed region of `calls` library calls.  An event costs a
    few microseconds of stream time (32 decode calls with five events each: 3.7 % of the step at cfg3), so in long
    regions only every 8th (4th) call is instrumented; the averages are over those calls."""
    period = 8 if calls >= 64 else (4 if calls >= 16 else 1)
    B.tune("timing_period", period)
    B.timing_begin()
    return period


def timing_end_sampled(B, period):
    kern = B.timing_end()
    B.tune("timing_period", 1)
    note = ("HIP events around every kernel of every call of the timed region" if period == 1 else
            f"HIP events around every kernel of every {period}th call of the timed region")
    return kern, note


def log(*a):
    print(*a, file=sys.stderr, flush=True)


MFMA_BF16_PEAK_TFLOPS = 2500.0


def prefill_workload(args, torch, dk, B, G):
    """One 32768-token prompt compressed layer after layer (every token: cosine top-1 retrieval over every 16th
    earlier token, residual, W_down projection)."""
    L, NL, Hkv, Hq, r, D, s = 32768 if args.seq_len == 131072 else args.seq_len, args.layers, args.kv_heads, \
        args.q_heads, args.rank, 128, 16
    mlp = None
    if getattr(args, "mlp", None):                               # non-linear compressor: "gelu:256", "swiglu:256"
        kind_name, hidden = args.mlp.split(":")
        mlp = (1 if kind_name == "swiglu" else 0, int(hidden))
    joint = args.mode == "joint" or mlp is not None
    l2 = args.metric == "l2"
    dims = dk.make_dims(Hkv, Hq, r, n_pages=-(-L // 16), n_ref_slots=-(-L // s),
                        latent_mode=dk.JOINT if joint else dk.SPLIT, metric=dk.METRIC_L2 if l2 else dk.METRIC_COSINE)
    cache = dk.PagedCache(dims, 1, L, L)
    W = G.make_projections(G.seed_for(4), D, r, joint=joint, recipe="baseline")
    dev = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    wdk, wdv = dev(W["w_down_k_bf16"]), dev(W["w_down_v_bf16"])
    if mlp:
        M = G.make_mlp_compressor(G.seed_for(4), D, r, mlp[1], swiglu=mlp[0] == 1)
        mw1, mw2, mb1 = dev(M["w1_bf16"]), dev(M["w2_bf16"]), torch.from_numpy(M["b1_f32"]).cuda()
        mwg = dev(M["wg_bf16"]) if mlp[0] == 1 else None
    n_in = 4                                                     # distinct input sets, used round-robin
    kv = []
    for i in range(n_in):
        K, V, _ = G.make_kv(G.seed_for(4, i), L, Hkv, D, n_proto=args.protos, threads=16)
        kv.append((dev(K), dev(V)))
    cu = torch.tensor([0, L], dtype=torch.int32, device="cuda")
    lb = torch.tensor([0], dtype=torch.int32, device="cuda")

    def step():
        for layer in range(NL):
            kd, vd = kv[layer % n_in]
            if mlp:
                B.compress_mlp(dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool,
                               cache.ref_inv_norm, cache.block_tables, cache.ref_tables, mlp[0], mw1, mwg, mb1, mw2,
                               kd, vd, cu, [0, L], lb, [0], cache.compress_ws)
                continue
            B.compress(dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.ref_inv_norm,
                       cache.block_tables, cache.ref_tables, wdk, wdv, kd, vd, cu, [0, L], lb, [0], cache.compress_ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    period = timing_begin_sampled(B, NL * args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kern, timing_note = timing_end_sampled(B, period)
    ms_per_step = elapsed * 1e3 / args.steps
    # exact count of multiply-adds of the causal similarity search: token i scores ceil(i/s) references, 2*D values each
    cand = sum(-(-i // s) for i in range(L) if i % s)
    flops = 2.0 * cand * 2 * D * Hkv
    ms_sim = kern["sim_top2"][0] / max(kern["sim_top2"][1], 1)
    tflops = flops / (ms_sim * 1e-3) / 1e12
    # parity of the last layer's ordinals against the oracle on a sample of tokens
    from oracle import deltakv_oracle as O
    f = O.bf16_bits_to_f64
    Kh, Vh, _ = G.make_kv(G.seed_for(4, (NL - 1) % n_in), L, Hkv, D, n_proto=args.protos, threads=16)
    idx, zk, zv = cache.get_sequence(0, 0, L)
    t0 = time.perf_counter()
    nsamp = min(L, 32768 if not l2 else 8192)    # the L2 oracle evaluates the definition token by token (slower)
    nsamp = min(nsamp, getattr(args, "parity_tokens", None) or nsamp)
    om = None
    if mlp:
        om = {"kind": O.SWIGLU if mlp[0] == 1 else O.GELU, "w1": M["w1_f64"], "b1": M["b1_f32"].astype(np.float64),
              "w2": M["w2_f64"]}
        if mlp[0] == 1:
            om["wg"] = M["wg_f64"]
    ref = O.compress(f(Kh), f(Vh), f(W["w_down_k_bf16"]), f(W["w_down_v_bf16"]), s=s,
                     mode=O.JOINT if joint else O.SPLIT, start=L - nsamp, metric=O.L2 if l2 else O.COSINE, mlp=om)
    t_or = time.perf_counter() - t0
    mism = int(np.sum(ref["idx"] != idx[L - nsamp:]))
    same = ref["idx"] == idx[L - nsamp:]
    lat_off = int(np.sum((f(zk[L - nsamp:]) != O.f64_round_to_bf16(ref["z_k"]))[same]))
    result = {
        "metric": "compress tokens/s (prefill compression of one 32768-token prompt, all layers)",
        "value": round(L / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"prefill compression: 1 x {L} tokens, {NL} layers, {Hkv} kv-heads x {D}, rank {r}, "
                               f"{'JOINT' if joint else 'SPLIT'} latents"
                               f"{' from the ' + args.mlp + ' non-linear compressor' if mlp else ''}, references every {s}th earlier token, "
                               f"{'squared-L2' if l2 else 'cosine'} top-1"},
        "roofline": {"bound": "mfma", "kernel": "k_sim_top2", "achieved": round(tflops, 1),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": measured_traffic("prefill32k_sim_top2") if (L, Hkv, r, NL) == (32768, 8, 64, 32) and not joint and not l2 else None,
                     "flops_per_launch": flops, "avg_launch_ms": round(ms_sim, 4)},
        "cpu_baseline": {"value": round(nsamp / t_or / NL, 1), "unit": "tokens/s", "cores":
                         int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                         "sample": f"last {nsamp} tokens of one layer ({t_or:.2f} s), scaled to the layer's {L} tokens by "
                                   f"token count and to {NL} layers"},
        "kernel_ms": {k: round(ms / n, 4) for k, (ms, n) in kern.items() if n},
        "kernel_timing": timing_note,
        "parity": {"what": f"ordinals of the last {nsamp} tokens of the last layer vs CPU oracle", "mismatches": mism,
                   "latents_not_the_correctly_rounded_value": lat_off, "latents_compared": int(same.sum()) * r},
    }
    return result


def _oracle_decode_seq(cache, b, L, K, V, W, q_bits_row, s, scale):
    """CPU oracle decode of sequence b from the GPU-built cache (ordinals/latents read back) and raw references."""
    from oracle import deltakv_oracle as O
    f = O.bf16_bits_to_f64
    i0, zk0, zv0 = cache.get_sequence(b, 0, L)
    t0 = time.perf_counter()
    want, _ = O.decode_attn_direct(f(q_bits_row), i0, f(zk0), f(zv0), f(K[:L:s]), f(V[:L:s]),
                                   f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), scale)
    return want, time.perf_counter() - t0


def ragged_workload(args, torch, dk, B, G):
    """64 sequences, lengths log-uniform in [4096, 65536], 4 kv-heads x 128, 28 query heads, rank 48; latents and
    ordinals live in 16-token pages scattered randomly over a shared pool 1.25x the needed size."""
    nseq, Hkv, Hq, r, D, s = 64, 4, 28, 48, 128, 16
    scale = 1.0 / np.sqrt(D)
    joint = args.mode == "joint"
    n_streams = 1 if joint else 2
    lens = G.loguniform_lengths(G.seed_for(5), nseq, 4096, 65536)
    pages = [-(-int(L) // 16) for L in lens]
    refs = [-(-int(L) // s) for L in lens]
    n_pages, n_slots = int(sum(pages) * 1.25), int(sum(refs) * 1.25)
    pp = G.page_permutation(G.seed_for(5), sum(pages), n_pages)
    rp = G.page_permutation(G.seed_for(5, 1), sum(refs), n_slots)
    if args.contiguous:
        pp, rp = np.arange(sum(pages), dtype=np.int32), np.arange(sum(refs), dtype=np.int32)
    cp, cr = np.concatenate([[0], np.cumsum(pages)]), np.concatenate([[0], np.cumsum(refs)])
    dims = dk.make_dims(Hkv, Hq, r, n_pages=n_pages, n_ref_slots=n_slots, latent_mode=dk.JOINT if joint else dk.SPLIT)
    Lmax = int(lens.max())
    cache = dk.PagedCache(dims, nseq, Lmax, Lmax, page_ids=[pp[cp[b]:cp[b + 1]] for b in range(nseq)],
                          ref_slots=[rp[cr[b]:cr[b + 1]] for b in range(nseq)])
    W = G.make_projections(G.seed_for(5), D, r, joint=joint, recipe="baseline")
    dev = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    wdk, wdv, wuk, wuv = (dev(W[k]) for k in ("w_down_k_bf16", "w_down_v_bf16", "w_up_k_bf16", "w_up_v_bf16"))
    order = np.argsort(lens)
    keep = {int(order[0]): None, int(order[nseq // 2]): None, int(order[-1]): None}
    for b in range(nseq):
        K, V, _ = G.make_kv(G.seed_for(5, 0, b + 1), int(lens[b]), Hkv, D, n_proto=args.protos, threads=16)
        if b in keep:
            keep[b] = (K, V)
        cache.compress(wdk, wdv, dev(K), dev(V), [0, int(lens[b])], [0], first_seq=b)
    q_bits = G.make_queries(G.seed_for(5), nseq, Hq, D)
    q = dev(q_bits)
    out = torch.empty_like(q)
    sl = torch.from_numpy(lens.astype(np.int32)).cuda()
    torch.cuda.synchronize()

    def step():
        B.decode_attn(dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.block_tables,
                      cache.ref_tables, wuk, wuv, q, sl, lens, scale, out, None, cache.decode_ws)

    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    period = timing_begin_sampled(B, args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kern, timing_note = timing_end_sampled(B, period)
    ms = elapsed * 1e3 / args.steps
    units = int(lens.sum()) * Hkv
    stream_bytes = units * (n_streams * r * 2 + 4)
    path_bytes = units * (n_streams * r * 2 + 4 + 2 * D * 2 / s)
    ms_stream = kern["stream"][0] / max(kern["stream"][1], 1)
    worst, t_or = 0.0, 0.0
    f64 = None
    from oracle import deltakv_oracle as O
    for b, (K, V) in keep.items():
        want, t = _oracle_decode_seq(cache, b, int(lens[b]), K, V, W, q_bits[b], s, scale)
        got = O.bf16_bits_to_f64(out[b].cpu().numpy().view(np.uint16))
        worst = max(worst, float(np.max(np.abs(got - want))))
        t_or += t
    samp_tokens = sum(int(lens[b]) for b in keep)
    result = {
        "metric": "decode-attn tokens/s over compressed cache (irregular paged batch)",
        "value": round(nseq / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"irregular paged batch: {nseq} sequences, lengths log-uniform in [4096, 65536] "
                               f"({int(lens.sum())} tokens), {Hkv} kv-heads x {D}, {Hq} q-heads, rank {r}, "
                               f"{args.mode.upper()} latents, pages scattered over a pool 1.25x the needed size, 1 layer"},
        "roofline": {"bound": "hbm", "kernel": "k_stream", "achieved": round(stream_bytes / (ms_stream * 1e-3) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(stream_bytes / (ms_stream * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic("ragged_split") if args.mode == "split" and not args.contiguous else None,
                     "algorithmic_bytes_per_launch": stream_bytes, "avg_launch_ms": round(ms_stream, 5)},
        "cpu_baseline": {"value": round(nseq / (t_or * int(lens.sum()) / samp_tokens), 3), "unit": "tokens/s",
                         "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                         "sample": f"shortest, median and longest sequence ({samp_tokens} tokens, {t_or:.2f} s), "
                                   "scaled by token count"},
        "path_hbm_frac": round(path_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "kernel_ms": {k: round(v / n, 5) for k, (v, n) in kern.items() if n},
        "kernel_timing": timing_note,
        "parity": {"what": "shortest, median, longest sequence vs CPU oracle", "max_abs_err": worst},
    }
    return result


def append_workload(args, torch, dk, B, G):
    """Llama-3.1-8B-shaped single layer: batch 1, 32768-token context, 256 decode steps, each appending one
    compressed token and then attending over the whole cache."""
    L0, nsteps, Hkv, Hq, r, D, s = 32768, 256, args.kv_heads, args.q_heads, args.rank, 128, 16
    scale = 1.0 / np.sqrt(D)
    joint = args.mode == "joint"
    Lmax = L0 + nsteps
    l2 = args.metric == "l2"
    dims = dk.make_dims(Hkv, Hq, r, n_pages=-(-Lmax // 16), n_ref_slots=-(-Lmax // s),
                        latent_mode=dk.JOINT if joint else dk.SPLIT, metric=dk.METRIC_L2 if l2 else dk.METRIC_COSINE)
    cache = dk.PagedCache(dims, 1, L0, Lmax)
    W = G.make_projections(G.seed_for(2), D, r, joint=joint, recipe="baseline")
    dev = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    wdk, wdv, wuk, wuv = (dev(W[k]) for k in ("w_down_k_bf16", "w_down_v_bf16", "w_up_k_bf16", "w_up_v_bf16"))
    K, V, _ = G.make_kv(G.seed_for(2), Lmax, Hkv, D, n_proto=args.protos, threads=16)
    Kd, Vd = dev(K), dev(V)
    q_bits = G.make_queries(G.seed_for(2), nsteps, Hq, D)
    qd = dev(q_bits)
    outs = torch.empty_like(qd)
    cu = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
    lbs = [torch.tensor([L0 + i], dtype=torch.int32, device="cuda") for i in range(nsteps)]
    sls = [torch.tensor([L0 + i + 1], dtype=torch.int32, device="cuda") for i in range(nsteps)]

    def run(timed):
        cache.compress(wdk, wdv, Kd[:L0], Vd[:L0], [0, L0], [0])          # prefill (not timed)
        torch.cuda.synchronize()
        if timed:
            B.timing_begin()
        t0 = time.perf_counter()
        for i in range(nsteps):
            t = L0 + i
            B.compress(dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.ref_inv_norm,
                       cache.block_tables, cache.ref_tables, wdk, wdv, Kd[t:t + 1], Vd[t:t + 1], cu, [0, 1], lbs[i], [t],
                       cache.compress_ws)
            B.decode_attn(dims, cache.layout, cache.latent_pool, cache.idx_pool, cache.ref_pool, cache.block_tables,
                          cache.ref_tables, wuk, wuv, qd[i:i + 1], sls[i], [t + 1], scale, outs[i:i + 1], None,
                          cache.decode_ws)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    for _ in range(max(args.warmup, 1)):
        run(False)
    elapsed = run(True)
    kern = B.timing_end()
    us = elapsed * 1e6 / nsteps
    # parity at steps 0, 127, 255: ordinals of the appended tokens and the attention output
    from oracle import deltakv_oracle as O
    f = O.bf16_bits_to_f64
    ref = O.compress(f(K), f(V), f(W["w_down_k_bf16"]), f(W["w_down_v_bf16"]), s=s,
                     mode=O.JOINT if joint else O.SPLIT, start=L0, metric=O.L2 if l2 else O.COSINE)
    idx, zk, zv = cache.get_sequence(0, L0, Lmax)
    mism = int(np.sum(idx != ref["idx"]))
    worst, t_or = 0.0, 0.0
    i_all, zk_all, zv_all = cache.get_sequence(0, 0, Lmax)
    for i in (0, 127, 255):
        Lc = L0 + i + 1
        t0 = time.perf_counter()
        want, _ = O.decode_attn_direct(f(q_bits[i]), i_all[:Lc], f(zk_all[:Lc]), f(zv_all[:Lc]), f(K[:Lc:s]), f(V[:Lc:s]),
                                       f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"]), scale)
        t_or += time.perf_counter() - t0
        got = f(outs[i].cpu().numpy().view(np.uint16))
        worst = max(worst, float(np.max(np.abs(got - want))))
    units = (L0 + nsteps // 2) * Hkv
    n_streams = 1 if joint else 2
    result = {
        "metric": "decode tokens/s, single sequence (append one compressed token, then attend)",
        "value": round(1e6 / us, 1), "unit": "tokens/s", "n_gpus": 1, "steps": nsteps, "warmup": args.warmup,
        "ms_per_step": round(us / 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"single layer, batch 1, context {L0} -> {Lmax} over {nsteps} steps, {Hkv} kv-heads x {D}, "
                               f"{Hq} q-heads, rank {r}, {args.mode.upper()} latents"},
        "roofline": {"bound": "hbm", "kernel": "k_stream", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": None, "traffic": None,
                     "note": "latency-bound: 76 MB per step would take 9.6 us at 8 TB/s",
                     "algorithmic_bytes_per_launch": units * (n_streams * r * 2 + 4)},
        "cpu_baseline": {"value": round(3 / t_or, 3), "unit": "tokens/s",
                         "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                         "sample": f"decode attention at steps 0, 127, 255 ({t_or:.2f} s); the append's retrieval is not included"},
        "kernel_us": {k: round(v / n * 1e3, 2) for k, (v, n) in kern.items() if n},
        "parity": {"what": "ordinals of all 256 appended tokens; attention output at steps 0, 127, 255",
                   "ordinal_mismatches": mism, "max_abs_err": worst},
    }
    if kern["stream"][1]:
        ms_stream = kern["stream"][0] / kern["stream"][1]
        ach = result["roofline"]["algorithmic_bytes_per_launch"] / (ms_stream * 1e-3) / 1e9
        result["roofline"]["achieved"], result["roofline"]["frac"] = round(ach, 1), round(ach / HBM_PEAK_GBS, 4)
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--seq-len", type=int, default=131072)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--kv-heads", type=int, default=8)
    ap.add_argument("--q-heads", type=int, default=32)
    ap.add_argument("--rank", type=int, default=64)
    ap.add_argument("--protos", type=int, default=1024)
    ap.add_argument("--mode", choices=["split", "joint"], default="split",
                    help="split: one rank-r latent per stream (default, the literal config shapes); "
                         "joint: one rank-r latent per (token, kv-head) over K||V")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run 5 plain device copies of this many MiB (to scale rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--mlp", default=None, help="prefill32k with the non-linear compressor: gelu:HIDDEN or swiglu:HIDDEN "
                    "(JOINT latents)")
    ap.add_argument("--workload", choices=["decode128k", "prefill32k", "ragged", "append32k"], default="decode128k",
                    help="decode128k: the headline long-context decode (default); prefill32k: compression of one "
                         "32768-token prompt over the layers (reports compress tokens/s and the similarity GEMM's "
                         "fraction of the MFMA roofline)")
    ap.add_argument("--metric", choices=["cosine", "l2"], default="cosine",
                    help="retrieval metric of the compression workloads (prefill32k, append32k)")
    ap.add_argument("--contiguous", action="store_true", help="ragged workload: identity page placement (experiment)")
    ap.add_argument("--select", type=float, default=0.0, metavar="FRACTION",
                    help="decode128k: attend only a selected subset (deltakv_decode_attn_subset): this fraction of "
                         "each sequence's pages, drawn at random per layer, all 16 tokens of a drawn page")
    ap.add_argument("--select-tokens", action="store_true",
                    help="with --select: draw single tokens instead of whole pages (same number of tokens)")
    ap.add_argument("--latent-bits", type=int, choices=[16, 4], default=16,
                    help="decode128k: 4 = 4-bit token-wise latents")
    ap.add_argument("--top-k", type=int, choices=[1, 2, 4], default=1,
                    help="decode128k: references retrieved per token (the reference is their mean; section 4.1)")
    ap.add_argument("--rope", type=float, default=0.0, metavar="BASE",
                    help="decode128k: deltakv_decode_attn_rope with this base (keys rotated at their position after "
                         "reconstruction; the queries are taken as already rotated)")
    ap.add_argument("--raw", type=int, default=0, metavar="TOKENS",
                    help="decode128k: also attend this many uncompressed (sink / recent) tokens per sequence")
    ap.add_argument("--tune", action="append", default=[], help="name=value launch-shape override (repeatable)")
    ap.add_argument("--no-extras", dest="extras", action="store_false",
                    help="decode128k: do not append the short runs of the other configurations ('workloads')")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="do not record per-kernel events (roofline.achieved is then null)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no collectives, no sharding here)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_08005_amd as dk
    from paper_2602_08005_amd import binding as B
    from synthetic import generator as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.arange(n // 4, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "copies": 5}))
        return
    for kv in args.tune:
        name, val = kv.split("=")
        B.tune(name, int(val))
    torch.cuda.set_device(0)
    if args.workload == "prefill32k":
        result = prefill_workload(args, torch, dk, B, G)
    elif args.workload == "ragged":
        result = ragged_workload(args, torch, dk, B, G)
    elif args.workload == "append32k":
        result = append_workload(args, torch, dk, B, G)
    else:
        result = decode_workload(args, torch, dk, B, G)
        plain = (args.batch, args.seq_len, args.layers, args.kv_heads, args.q_heads, args.rank, args.mode, args.latent_bits,
                 args.select, args.raw, args.top_k, args.rope) == (8, 131072, 32, 8, 32, 64, "split", 16, 0.0, 0, 1, 0.0)
        if args.extras and plain:             # the headline run also carries short runs of the other configurations
            result["workloads"] = extra_workloads(args, torch, dk, B, G)
    print(json.dumps(result))


def extra_workloads(args, torch, dk, B, G):
    """Short runs of the other configurations, reported inside the headline's JSON line: the long-context decode with
    JOINT latents, the irregular paged batch, the 32768-token prefill compression and the single-sequence append
    loop, the decode over 4-bit latents, the decode path with rotary position embedding and the prefill with the
    non-linear compressor.  Each entry carries its throughput, the roofline of its dominant kernel and its parity figure against the
    CPU oracle (on a smaller sample than the workload's own command line takes)."""
    import copy
    import gc
    out = {}
    runs = [("decode128k_joint", decode_workload, dict(mode="joint", steps=5, warmup=1, parity_seqs=2)),
            ("ragged", ragged_workload, dict(workload="ragged", steps=20, warmup=2)),
            ("prefill32k", prefill_workload, dict(workload="prefill32k", steps=3, warmup=1, parity_tokens=4096)),
            ("append32k", append_workload, dict(workload="append32k", warmup=1)),
            ("decode128k_joint_q4", decode_workload, dict(mode="joint", latent_bits=4, steps=5, warmup=1, parity_seqs=1)),
            ("decode128k_rope", decode_workload, dict(rope=500000.0, steps=3, warmup=1, parity_seqs=1)),
            ("prefill32k_mlp_gelu", prefill_workload, dict(workload="prefill32k", mlp="gelu:256", steps=3, warmup=1,
                                                           parity_tokens=2048))]
    for name, fn, over in runs:
        gc.collect()
        torch.cuda.empty_cache()
        a = copy.copy(args)
        for k, v in over.items():
            setattr(a, k, v)
        t0 = time.time()
        r = fn(a, torch, dk, B, G)
        keep = ("value", "unit", "steps", "ms_per_step", "config", "roofline", "path_hbm_frac", "kernel_ms", "kernel_us",
                "kernel_timing", "parity", "status_flag", "cpu_baseline", "metric")
        out[name] = {k: r[k] for k in keep if k in r}
        out[name]["command"] = "python bench.py " + {"decode128k_joint": "--mode joint", "ragged": "--workload ragged",
                                                     "prefill32k": "--workload prefill32k",
                                                     "append32k": "--workload append32k",
                                                     "decode128k_joint_q4": "--mode joint --latent-bits 4",
                                                     "decode128k_rope": "--rope 500000",
                                                     "prefill32k_mlp_gelu": "--workload prefill32k --mlp gelu:256"}[name]
        log(f"[bench] extra workload {name}: {r['value']} {r['unit']} ({time.time() - t0:.1f} s wall)")
    return out


def decode_workload(args, torch, dk, B, G):
    Bt, L, NL, Hkv, Hq, r, D, s = args.batch, args.seq_len, args.layers, args.kv_heads, args.q_heads, args.rank, 128, 16
    scale = 1.0 / np.sqrt(D)
    pages_per_seq, refs_per_seq = -(-L // 16), -(-L // s)
    joint = args.mode == "joint"
    n_streams = 1 if joint else 2
    q4 = args.latent_bits == 4
    dims = dk.make_dims(Hkv, Hq, r, n_pages=Bt * pages_per_seq, n_ref_slots=Bt * refs_per_seq,
                        latent_mode=dk.JOINT if joint else dk.SPLIT, latent_bits=args.latent_bits, top_k=args.top_k,
                        metric=dk.METRIC_L2 if args.metric == "l2" else dk.METRIC_COSINE)
    # latent record(s) (codes + bf16 scale and zero point, or bf16 latents) + int32 ordinal(s), per (token, kv-head)
    rec_bytes = n_streams * (r // 2 + 4 if q4 else r * 2) + 4 * args.top_k
    t_setup = time.time()
    cache = dk.PagedCache(dims, Bt, L, L)
    W = G.make_projections(G.seed_for(3), D, r, joint=joint, recipe="baseline")
    dev = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    wdk, wdv = dev(W["w_down_k_bf16"]), dev(W["w_down_v_bf16"])
    wuk, wuv = dev(W["w_up_k_bf16"]), dev(W["w_up_v_bf16"])

    # ---- layer 0: generate K/V per sequence and compress it on the GPU (also the compress measurement)
    host_refs = []                                    # raw reference rows of every sequence (what the oracle's decode needs)
    comp_ms = 0.0
    comp_kern = {}
    for b in range(Bt):
        K, V, _ = G.make_kv(G.seed_for(3, 0, b), L, Hkv, D, n_proto=args.protos, threads=16)
        host_refs.append((K[::s].copy(), V[::s].copy()))
        kd, vd = dev(K), dev(V)
        torch.cuda.synchronize()
        B.timing_begin()
        t0 = time.perf_counter()
        cache.compress(wdk, wdv, kd, vd, [0, L], [0], first_seq=b)
        torch.cuda.synchronize()
        comp_ms += (time.perf_counter() - t0) * 1e3
        for k, (ms, n) in B.timing_end().items():
            if n:
                comp_kern[k] = comp_kern.get(k, 0.0) + ms
        del kd, vd
        log(f"[bench] sequence {b}: generated + compressed ({comp_ms:.1f} ms of compress so far)")
    compress_tok_s = Bt * L / (comp_ms * 1e-3)

    # ---- replicate to NL layers (distinct memory), one query set per layer
    lat = [cache.latent_pool] + [cache.latent_pool.clone() for _ in range(NL - 1)]
    idx = [cache.idx_pool] + [cache.idx_pool.clone() for _ in range(NL - 1)]
    ref = [cache.ref_pool] + [cache.ref_pool.clone() for _ in range(NL - 1)]
    qs = [dev(G.make_queries(G.seed_for(3, layer), Bt, Hq, D)) for layer in range(NL)]
    outs = [torch.empty_like(q) for q in qs]
    seq_lens_host = np.full(Bt, L, dtype=np.int32)
    seq_lens = torch.from_numpy(seq_lens_host).cuda()
    torch.cuda.synchronize()
    log(f"[bench] setup done in {time.time() - t_setup:.1f} s; "
        f"{torch.cuda.memory_allocated() / 1e9:.1f} GB resident")

    # ---- optional subset attention: one selection per layer (seeded), resident on the device before timing
    selections = None
    n_pages_seq = L // 16
    if args.select > 0:
        n_pick = max(1, int(round(args.select * n_pages_seq)))
        selections = []
        for layer in range(NL):
            rng = np.random.Generator(np.random.Philox(G.seed_for(3, layer) + 77))
            pos = []
            for b in range(Bt):
                if args.select_tokens:
                    pos.append(np.sort(rng.choice(L, n_pick * 16, replace=False)))
                else:
                    pg = np.sort(rng.choice(n_pages_seq, n_pick, replace=False))
                    pos.append((pg[:, None] * 16 + np.arange(16)[None, :]).ravel())
            selections.append(cache.selection(pos) + (pos,))
        sel_pages_touched = float(np.mean([int(sel[3].sum()) for sel in selections])) / Bt

    # ---- optional raw segment (sink + recent tokens kept uncompressed), the same rows for every layer
    raw = None
    if args.raw > 0:
        rk = np.stack([G.make_kv(G.seed_for(3, 900, b), args.raw, Hkv, D, n_proto=args.protos)[0] for b in range(Bt)])
        rv = np.stack([G.make_kv(G.seed_for(3, 900, b), args.raw, Hkv, D, n_proto=args.protos)[1] for b in range(Bt)])
        raw = (dev(rk), dev(rv), torch.full((Bt,), args.raw, dtype=torch.int32, device="cuda"), rk, rv)

    def step():
        for layer in range(NL):
            if args.rope > 0:
                B.decode_attn_rope(dims, cache.layout, lat[layer], idx[layer], ref[layer], cache.block_tables,
                                   cache.ref_tables, wuk, wuv, qs[layer], seq_lens, seq_lens_host, scale, args.rope,
                                   outs[layer], None, cache.decode_ws)
            elif raw is not None:
                sel = None if selections is None else selections[layer][:4]
                B.decode_attn_raw(dims, cache.layout, lat[layer], idx[layer], ref[layer], cache.block_tables,
                                  cache.ref_tables, wuk, wuv, qs[layer], seq_lens, seq_lens_host, raw[0], raw[1],
                                  raw[2], scale, outs[layer], None, cache.decode_ws, selection=sel)
            elif selections is None:
                B.decode_attn(dims, cache.layout, lat[layer], idx[layer], ref[layer], cache.block_tables,
                              cache.ref_tables, wuk, wuv, qs[layer], seq_lens, seq_lens_host, scale, outs[layer],
                              None, cache.decode_ws)
            else:
                sp, sm, n_dev, n_host, _ = selections[layer]
                B.decode_attn_subset(dims, cache.layout, lat[layer], idx[layer], ref[layer], cache.block_tables,
                                     cache.ref_tables, wuk, wuv, qs[layer], seq_lens, seq_lens_host, sp, sm, n_dev,
                                     n_host, scale, outs[layer], None, cache.decode_ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    timing = not args.no_kernel_timing
    if timing:
        period = timing_begin_sampled(B, NL * args.steps)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kern, timing_note = timing_end_sampled(B, period) if timing else ({}, None)
    status = int(cache.decode_ws[:4].view(torch.int32)[0].item())
    ms_per_step = elapsed * 1e3 / args.steps
    tok_s = Bt * args.steps / elapsed

    # ---- roofline of the dominant kernel (the streaming pass over latents + indices)
    units = Bt * L * Hkv                                  # (token, kv-head) records per launch
    stream_bytes = units * rec_bytes                              # latent record(s) + int32 ordinal
    path_bytes = units * (rec_bytes + 2 * D * 2 / s)              # + each raw reference K and V read once
    if selections is not None:
        # subset attention: the selected tokens' records (the method's bytes), each raw reference still read once
        sel_units = Bt * n_pick * 16 * Hkv
        stream_bytes = sel_units * rec_bytes
        path_bytes = stream_bytes + units * (2 * D * 2 / s)
    if raw is not None:
        path_bytes += Bt * args.raw * Hkv * 2 * D * 2             # raw K and V rows, read once
    roof = {"bound": "hbm", "kernel": "k_rope_attn" if args.rope > 0 else "k_stream", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": None, "traffic": None, "algorithmic_bytes_per_launch": stream_bytes}
    if (Bt, L, Hkv, Hq, r) == (8, 131072, 8, 32, 64) and raw is None:        # the rows of profiles/hbm_traffic.md
        key = "decode128k_" + args.mode + ("_q4" if q4 else "") + (f"_top{args.top_k}" if args.top_k > 1 else "") \
            + ("_rope" if args.rope > 0 else "")
        if selections is not None:
            key += f"_select{args.select:g}" + ("_tokens" if args.select_tokens else "")
        roof["traffic"] = measured_traffic(key)
    kernel_ms = {}
    if timing:
        for k, (ms, n) in kern.items():
            if n:
                kernel_ms[k] = round(ms / n, 5)
        ms_stream = kern["stream"][0] / max(kern["stream"][1], 1)
        roof["achieved"] = round(stream_bytes / (ms_stream * 1e-3) / 1e9, 1)
        roof["frac"] = round(roof["achieved"] / HBM_PEAK_GBS, 4)
        roof["avg_launch_ms"] = round(ms_stream, 5)
    path_gbs = path_bytes * NL / (ms_per_step * 1e-3) / 1e9

    # ---- CPU oracle on a bounded sample: layer 0 of every sequence = 1/layers of a step (about 10 s of CPU work)
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import deltakv_oracle as O
        f = O.bf16_bits_to_f64
        t_layer, worst_abs, worst_rel = 0.0, 0.0, 0.0
        n_par = min(Bt, getattr(args, "parity_seqs", None) or Bt)
        for b in range(n_par):
            if q4:      # the values the GPU's own 4-bit records read back as (scale * code + zero)
                i0, c0, s0, z0 = cache.get_sequence_q4(b, 0, L)
                zkf = zvf = f(s0)[..., None] * c0 + f(z0)[..., None]
                if not joint:
                    _, c1, s1, z1 = cache.get_sequence_q4(b, 0, L, stream=1)
                    zvf = f(s1)[..., None] * c1 + f(z1)[..., None]
            else:
                i0, zk0, zv0 = cache.get_sequence(b, 0, L)
                zkf, zvf = f(zk0), f(zv0)
            rk, rv = (f(x) for x in host_refs[b])
            qh = f(qs[0][b].cpu().numpy().view(np.uint16))
            wuk_f, wuv_f = f(W["w_up_k_bf16"]), f(W["w_up_v_bf16"])
            sel_b = None if selections is None else selections[0][4][b]
            t0 = time.perf_counter()
            if args.rope > 0:
                want, _ = O.decode_attn_rope(qh, i0, zkf, zvf, rk, rv, wuk_f, wuv_f, scale, base=args.rope)
            elif raw is not None:
                want, _ = O.decode_attn_with_raw(qh, i0, zkf, zvf, rk, rv, wuk_f, wuv_f, scale, f(raw[3][b]), f(raw[4][b]),
                                                 positions=sel_b)
            elif selections is None:
                want, _ = O.decode_attn_direct(qh, i0, zkf, zvf, rk, rv, wuk_f, wuv_f, scale)
            else:
                want, _ = O.decode_attn_subset(qh, i0, zkf, zvf, rk, rv, wuk_f, wuv_f, scale, sel_b)
            t_layer += time.perf_counter() - t0
            got = f(outs[0][b].cpu().numpy().view(np.uint16))
            worst_abs = max(worst_abs, float(np.max(np.abs(got - want))))
            worst_rel = max(worst_rel, float(np.linalg.norm(got - want) / np.linalg.norm(want)))
            del i0, zkf, zvf
        parity = {"what": f"layer 0, {n_par} of {Bt} sequences, all query heads vs CPU oracle (worst sequence)",
                  "max_abs_err": worst_abs, "rel_l2_err": worst_rel}
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": round(n_par / (t_layer * NL), 5), "unit": "tokens/s", "cores": threads, "kind": "oracle",
               "sample": f"decode attention of layer 0 for {n_par} of the {Bt} sequences = {n_par}/{Bt} of 1 of {NL} "
                         f"layers of one step ({t_layer:.2f} s), extrapolated linearly to the step"}

    result = {
        "metric": "decode-attn tokens/s over compressed cache + % HBM roofline; compress tokens/s",
        "value": round(tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"long-context decode: batch {Bt} x {L} tokens, {NL} layers sequential, "
                               f"{Hkv} kv-heads x {D}, {Hq} q-heads, rank {r}, {args.mode.upper()} latents"
                               f"{' (4-bit token-wise)' if q4 else ''}, stride {s}, 16-token pages"
                               + (f", top-{args.top_k} references per token ({args.metric}), mean" if args.top_k > 1 else "")
                               + (f", keys rotated after reconstruction (RoPE base {args.rope:g}; every token's key "
                                  f"rebuilt, its reference's raw K and V rows gathered)" if args.rope > 0 else ""),
                   "latent_mode": args.mode.upper(), "latent_bits": args.latent_bits,
                   "keep_ratio": round(dk.keep_ratio(dims), 4),
                   "layers_are_copies_of_layer0": True,
                   **({} if raw is None else {"raw_segment": f"{args.raw} uncompressed tokens per sequence attended "
                                                                "together with the cache"}),
                   **({} if selections is None else {
                       "subset": f"{n_pick * 16} of {L} tokens per sequence selected "
                                 f"({'single tokens' if args.select_tokens else 'whole pages'}, drawn per layer), "
                                 f"{sel_pages_touched:.0f} pages touched per sequence"})},
        "roofline": roof,
        "cpu_baseline": cpu,
        "path_hbm_frac": round(path_gbs / HBM_PEAK_GBS, 4),
        "path_algorithmic_GBps": round(path_gbs, 1),
        "kernel_ms": kernel_ms,
        "kernel_timing": timing_note,
        "compress": {"tokens_per_s": round(compress_tok_s, 1), "tokens": Bt * L,
                     "kernel_ms_total": {k: round(v, 3) for k, v in comp_kern.items()},
                     "what": f"prefill compression of {Bt} x {L} tokens for one layer, batch-1 calls"},
        "parity": parity, "status_flag": None if args.rope > 0 else status,   # (the rope path keeps no status word)
        "context": "paper: 29% KV memory and up to 2x vLLM decode throughput, whole model on 1x RTX PRO 6000 (not comparable)",
    }
    return result


if __name__ == "__main__":
    main()
