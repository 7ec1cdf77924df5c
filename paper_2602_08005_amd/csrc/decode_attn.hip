// Fused decode attention over the DeltaKV compressed cache, gfx950.
//
// Section 4.1 ("Reconstruction") defines KV_hat = f_d(z) + KV_ref; section 5.3 gives the bias-free
// linear decoder f_d(z) = z W_u.  With a linear decoder the attention over reconstructed tokens
//     logit_t = scale * q . (K_ref[idx_t] + z_K,t W_uK)
//     out     = sum_t p_t (V_ref[idx_t] + z_V,t W_uV) / sum_t p_t
// regroups exactly into
//     logit_t = S_ref[idx_t] + (W_uK q) . z_K,t          S_ref[j] = scale * q . K_ref[j]
//     out     = ( sum_j w_j V_ref[j] + (sum_t p_t z_V,t) W_uV ) / sum_t p_t ,  w_j = sum_{t: idx_t = j} p_t
// so each raw reference is read once per step (not once per token that points at it) and the per-token
// work is two small contractions against the latent streams.  Four kernels per call:
//   ref_scores  : S_ref for every reference ordinal (MFMA, q x K_ref tiles), chunk maxima, W_uK q
//   stream      : the HBM-bound pass over latents + indices; scores and the weighted latent sum on MFMA,
//                 w_j accumulated in a 32-bit fixed-point LDS table with integer atomics (plus a short list for the
//                 rare amounts that do not fit an entry), one partial set per (sequence, split) item
//   ref_values  : sum_j w_j V_ref[j] per reference chunk
//   finalize    : merges splits/chunks, up-projects the latent sum through W_uV, normalises, writes bf16
// (a fifth, raw_attn, runs first when the call brings a segment of uncompressed sink / recent tokens)
// All softmax weights use one fixed exponent offset per (sequence, q-head): m_ref = max_j S_ref[j].  A
// reference token is cached with idx = own ordinal and z = 0, so its logit IS S_ref[j]; the true maximum
// is therefore >= m_ref, partial sums from different waves/splits add without rescaling, and the sum of
// weights is >= 2^-64 > 0 (attention over a selection has no such floor: see the rescue kernel).
#include "decode_common.h"

namespace dkv {



// ------------------------------------------------------------------------------------------------
// ref_scores: grid (ceil(n_chunk_max / CPB), Hkv, B), 256 threads; a block scores CPB consecutive chunks of
// kRefChunk references.  Each wave scores 16 references per MFMA step: D[g][j] = sum_d q[g][d] K_ref[j][d].
// A wave's life is a chain of dependent round trips to memory (q and slots, reference rows, stores), about 10 us
// whatever the load of the machine, and blocks are handed to the compute units at a limited rate; a grid of
// thousands of one-chunk blocks therefore spends most of its time being dispatched, with a quarter of the wave
// slots occupied.  Large calls over sequences of about equal length use CPB = 4: a quarter of the blocks, each with
// the rows of its next chunk in flight while it scores the current one (chosen by the host).
// ------------------------------------------------------------------------------------------------
template <int CPB>
__global__ __launch_bounds__(256) void k_ref_scores(DecodeParams P) {
  const int chunk0 = blockIdx.x * CPB, h = blockIdx.y, b = blockIdx.z;
  // the status word is cleared here rather than by a memset node, so that a caller may capture the call
  if (chunk0 == 0 && h == 0 && b == 0) {
    if (threadIdx.x == 0) *P.status = 0;
    // List of the non-empty (sequence, split) items for the streaming kernel's grid.  Blocks start in list order,
    // so the list goes from the sequences with the largest splits to those with the smallest (longest processing
    // time first: the short blocks fill the gaps at the end of a ragged batch); a batch of more than 256
    // sequences keeps sequence order.  Thread t counts the items of its run of sequences, finds how many items
    // come before its run, and writes its run.
    __shared__ int run_items[256];
    __shared__ int run_size[256];
    const int per = ceil_div(P.batch, 256), b_lo = min((int)threadIdx.x * per, P.batch), b_hi = min(b_lo + per, P.batch);
    int cnt = 0, size = 0;
    for (int bb = b_lo; bb < b_hi; ++bb) {
      const int wp = work_pages_of(P, bb, seq_len_of(P, bb));
      cnt += used_splits(wp, P.S, P.pages_per_split);
      size = wp > 0 ? plan_splits(wp, P.S, P.pages_per_split).per : 0;     // pages per split (used when per == 1)
    }
    run_items[threadIdx.x] = cnt;
    run_size[threadIdx.x] = per == 1 ? size : 0;      // all equal: sequence order
    __syncthreads();
    int at = 0, total = 0;
    const int n_runs = ceil_div(P.batch, per);          // threads beyond hold no sequence
    for (int t = 0; t < n_runs; ++t) {
      const int n = run_items[t], sz = run_size[t];
      const bool before = sz > run_size[threadIdx.x] || (sz == run_size[threadIdx.x] && t < (int)threadIdx.x);
      at += before ? n : 0;
      total += n;
    }
    if (threadIdx.x == 0) P.items[0] = total;
    for (int bb = b_lo; bb < b_hi; ++bb) {
      const int ns = used_splits(work_pages_of(P, bb, seq_len_of(P, bb)), P.S, P.pages_per_split);
      for (int s = 0; s < ns; ++s) P.items[1 + at + s] = bb * kMaxSplits + s;
      at += ns;
    }
  }
  // (as are the rescue flags of this pair's query heads, by the pair's first block)
  if (chunk0 == 0 && (int)threadIdx.x < P.G) P.rescue[(int64_t)b * P.Hq + (int64_t)h * P.G + threadIdx.x] = 0;
  const int L = seq_len_of(P, b);
  const int n_ref = refs_below(L, P.stride);
  if (chunk0 * kRefChunk >= n_ref) return;
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63, ln = l & 15, lg = l >> 4;
  __shared__ float red[2][4][16];

  // A operand: q rows of this kv-head's group (rows >= G are zero)
  bf16x8 qa[4];
  {
    const uint16_t* qrow = P.q + ((int64_t)b * P.Hq + (int64_t)h * P.G + (ln < P.G ? ln : 0)) * kHeadDim;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 v = *reinterpret_cast<const uint4*>(qrow + (4 * kk + lg) * 8);
      if (ln >= P.G) v = make_uint4(0, 0, 0, 0);
      qa[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }
  const int64_t bh = (int64_t)b * P.Hkv + h;
  const uint16_t* kbase = P.ref + (int64_t)h * P.ref_head_stride;   // K half
  // A wave owns 64 references of every chunk: four 16-reference steps.  The pool slots of all the block's chunks
  // are fetched first; the sixteen 16-byte row loads of chunk c+1 are issued before chunk c is scored (rows past
  // the end re-read the last reference and are dropped afterwards).
  constexpr int NSTEP = kRefChunk / 64;
  constexpr int NBUF = CPB > 1 ? 2 : 1;
  int slot[CPB][NSTEP];
#pragma unroll
  for (int cc = 0; cc < CPB; ++cc)
#pragma unroll
    for (int step = 0; step < NSTEP; ++step) {
      const int j = min((chunk0 + cc) * kRefChunk + w * 64 + step * 16 + ln, n_ref - 1);
      slot[cc][step] = P.ref_tables[(int64_t)b * P.rt_stride + j];
    }
  uint4 kv[NBUF][NSTEP][4];
  auto issue = [&](const int (&sl)[NSTEP], uint4 (&dst)[NSTEP][4]) {
#pragma unroll
    for (int step = 0; step < NSTEP; ++step) {
      const uint16_t* krow = kbase + (int64_t)clampi(sl[step], 0, (int)P.n_ref_slots - 1) * kHeadDim;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) dst[step][kk] = *reinterpret_cast<const uint4*>(krow + (4 * kk + lg) * 8);
    }
  };
  issue(slot[0], kv[0]);
#pragma unroll
  for (int cc = 0; cc < CPB; ++cc) {
    const int chunk = chunk0 + cc, j0 = chunk * kRefChunk;
    if (j0 >= n_ref) break;                                  // uniform over the block
    if (cc + 1 < CPB) issue(slot[cc + 1 < CPB ? cc + 1 : cc], kv[(cc + 1) % NBUF]);
    float mx[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int step = 0; step < NSTEP; ++step) {
      const int j = j0 + w * 64 + step * 16 + ln;
      const bool valid = j < n_ref;
      float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[kk], __builtin_bit_cast(bf16x8, kv[cc % NBUF][step][kk]), acc, 0, 0, 0);
      // lane holds rows g = 4*lg + i of column j
      float4 o;
      o.x = acc[0] * P.qk_scale_log2; o.y = acc[1] * P.qk_scale_log2;
      o.z = acc[2] * P.qk_scale_log2; o.w = acc[3] * P.qk_scale_log2;
      if (valid && 4 * lg < P.Gp) {
        *reinterpret_cast<float4*>(P.sref + (bh * P.n_ref_max + j) * P.Gp + 4 * lg) = o;
        // long sequences: the table that takes the weights of ordinals older than the blocks' LDS windows starts at 0
        if (P.spill_on) *reinterpret_cast<float4*>(P.spill + (bh * P.n_ref_max + j) * P.Gp + 4 * lg) = make_float4(0.f, 0.f, 0.f, 0.f);
      }
      if (valid) {
        mx[0] = fmaxf(mx[0], o.x); mx[1] = fmaxf(mx[1], o.y);
        mx[2] = fmaxf(mx[2], o.z); mx[3] = fmaxf(mx[3], o.w);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) mx[i] = wave16_max(mx[i]);
    if (ln == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) red[cc & 1][w][4 * lg + i] = mx[i];
    }
    __syncthreads();      // (the buffer written two chunks later was read before the barrier in between)
    if (threadIdx.x < P.Gp) {
      const float (&r)[4][16] = red[cc & 1];
      float m = fmaxf(fmaxf(r[0][threadIdx.x], r[1][threadIdx.x]), fmaxf(r[2][threadIdx.x], r[3][threadIdx.x]));
      P.cmax[(bh * P.n_chunk_max + chunk) * P.Gp + threadIdx.x] = m;
    }
  }

  // first block of the pair: q_lat[g][c] = scale*log2e * sum_d q[g][d] W_uK[c][d], stored bf16; the 16-column
  // blocks go round the four waves (each block is a round trip to memory of its own)
  if (chunk0 == 0) {
    for (int nb = w; nb < P.R / 16; nb += 4) {
      const uint16_t* wrow = P.w_up_k + (int64_t)(nb * 16 + ln) * kHeadDim;
      float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        uint4 v = *reinterpret_cast<const uint4*>(wrow + (4 * kk + lg) * 8);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[kk], __builtin_bit_cast(bf16x8, v), acc, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int g = 4 * lg + i;
        if (g < P.G) {
          const float v = acc[i] * P.qk_scale_log2;
          const uint32_t hi = f32_to_bf16_bits(v);
          const int64_t at = ((int64_t)b * P.Hq + (int64_t)h * P.G + g) * P.R + nb * 16 + ln;
          P.qlat[at] = (uint16_t)hi;
          P.qlat[P.qlat_lo_offset + at] = (uint16_t)f32_to_bf16_bits(v - __uint_as_float(hi << 16));
        }
      }
    }
  }
}


// ------------------------------------------------------------------------------------------------
// ref_values: grid (n_chunk_max, Hkv, B), 256 threads.  opart[chunk][g][d] = sum_{j in chunk} w_j[g] V_ref[j][d]
// lane = (row-in-group l/16, 8-wide d chunk l%16); a wave reads four 256-byte V rows per load.
// ------------------------------------------------------------------------------------------------
template <int GP>
__global__ __launch_bounds__(256) void k_ref_values(DecodeParams P) {
  const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int L = seq_len_of(P, b);
  const int n_ref = refs_below(L, P.stride);
  const int j0 = chunk * kRefChunk;
  if (j0 >= n_ref) return;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 15, lg = l >> 4;
  const int n_pages = work_pages_of(P, b, L);
  const SplitPlan sp = plan_splits(n_pages, P.S, P.pages_per_split);
  const int64_t bh = (int64_t)b * P.Hkv + h;
  const uint16_t* vbase = P.ref + (int64_t)h * P.ref_head_stride + P.ref_kv_stride;   // V half
  __shared__ float red[4][GP][kHeadDim];
  __shared__ float wsum[kRefChunk][GP];
  __shared__ int slots[kRefChunk];

  // phase 1a: thread t loads the split partials of reference j0+t (coalesced across threads), its scores and its
  // slot.  All loads are issued before the reduction below needs its own, so the two latencies overlap.  The loads
  // of a split's entries are unconditional within the splits in use (an entry the split did not write holds stale
  // values and is dropped by the select): behind a per-thread branch each load would wait for the one before it.
  const int j = j0 + tid;
  float wfix[GP], wplain[GP], sj[GP];          // fixed-point sums, sums of tables already in plain units, scores
#pragma unroll
  for (int g = 0; g < GP; ++g) { wfix[g] = 0.f; wplain[g] = 0.f; sj[g] = 0.f; }
  // rows past the sequence's last reference carry weight 0; they re-read the last valid reference's row (never a
  // slot the caller did not admit: 0 * garbage could be NaN)
  const int slot = clampi(P.ref_tables[(int64_t)b * P.rt_stride + min(j, n_ref - 1)], 0, (int)P.n_ref_slots - 1);
  if (j < n_ref) {
    // splits in groups of four: within a group every load is issued before the first is used
    for (int s0 = 0; s0 < sp.n_splits; s0 += 4) {
      float4 t[4][GP / 4];
      bool on[4], pl[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int s = min(s0 + u, sp.n_splits - 1);            // (a repeated split is dropped below)
        const int p1 = min(n_pages, (s + 1) * sp.per);
        const int n_cov = s * sp.per < p1 ? refs_covered(P, b, L, p1) : 0;     // ordinals the split can touch
        const int lo = n_cov - min(n_cov, P.tab_cap);          // first ordinal of its table window
        on[u] = s0 + u < sp.n_splits && j >= lo && j < n_cov;
        pl[u] = P.wflag[bh * P.S + s] != 0;                    // its table already holds plain weights (rare)
        // row of ordinal j in the window (clamped: the load is unconditional, a row outside is dropped)
        const float* wp = P.wpart + ((bh * P.S + s) * P.tab_cap + clampi(j - lo, 0, P.tab_cap - 1)) * GP;
#pragma unroll
        for (int g4 = 0; g4 < GP; g4 += 4) t[u][g4 / 4] = *reinterpret_cast<const float4*>(wp + g4);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int g4 = 0; g4 < GP; g4 += 4) {
          const float tt[4] = {t[u][g4 / 4].x, t[u][g4 / 4].y, t[u][g4 / 4].z, t[u][g4 / 4].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            wfix[g4 + e] += on[u] && !pl[u] ? tt[e] : 0.f;
            wplain[g4 + e] += on[u] && pl[u] ? tt[e] : 0.f;
          }
        }
    }
    if (P.spill_on) {                          // plain weights from blocks whose window starts after ordinal j
      const float* sp2 = P.spill + (bh * P.n_ref_max + j) * GP;
#pragma unroll
      for (int g4 = 0; g4 < GP; g4 += 4) {
        const float4 t = *reinterpret_cast<const float4*>(sp2 + g4);
        wplain[g4] += t.x; wplain[g4 + 1] += t.y; wplain[g4 + 2] += t.z; wplain[g4 + 3] += t.w;
      }
    }
    const float* sp_ = P.sref + (bh * P.n_ref_max + j) * GP;
#pragma unroll
    for (int g4 = 0; g4 < GP; g4 += 4) {
      const float4 t = *reinterpret_cast<const float4*>(sp_ + g4);
      sj[g4] = t.x; sj[g4 + 1] = t.y; sj[g4 + 2] = t.z; sj[g4 + 3] = t.w;
    }
  }
  // per query head, the base of the table units (the same value the stream kernel used)
  __shared__ float cpart[256];
  __shared__ float shift_s[GP];
  {
    const int nch = ceil_div(n_ref, kRefChunk);
    float m = -INFINITY;
    for (int c = tid / GP; c < nch; c += 256 / GP) m = fmaxf(m, P.cmax[(bh * P.n_chunk_max + c) * GP + tid % GP]);
    cpart[tid] = m;
    __syncthreads();
    if (tid < GP) {
      for (int k = 1; k < 256 / GP; ++k) m = fmaxf(m, cpart[k * GP + tid]);
      shift_s[tid] = table_shift_base(m, exp_bias(P.sel_pages != nullptr));
    }
    __syncthreads();
  }
  // phase 1b: the fixed-point sums are scaled back by the power of two the stream kernel divided out
#pragma unroll
  for (int g = 0; g < GP; ++g)
    wsum[tid][g] = __builtin_ldexpf(wfix[g], -table_shift(sj[g], shift_s[g])) + wplain[g];
  slots[tid] = slot;
  __syncthreads();

  // phase 2: lane = (row-in-group lg, 8-wide d chunk ln); a wave reads four 256-byte V rows per load and
  // keeps UN such loads in flight
  float acc[GP][8];
#pragma unroll
  for (int g = 0; g < GP; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  constexpr int UN = GP >= 16 ? 2 : (GP == 8 ? 4 : 8);     // row loads in flight per wave
  for (int it0 = 0; it0 < kRefChunk / 16; it0 += UN) {
    uint4 v[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int row = w * (kRefChunk / 4) + (it0 + u) * 4 + lg;
      v[u] = *reinterpret_cast<const uint4*>(vbase + (int64_t)slots[row] * kHeadDim + ln * 8);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int row = w * (kRefChunk / 4) + (it0 + u) * 4 + lg;
      float wj[GP];
#pragma unroll
      for (int g = 0; g < GP; ++g) wj[g] = wsum[row][g];     // zero for rows past the end
      const uint32_t vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const float lo = bf16lo(vv[e2]), hi = bf16hi(vv[e2]);
#pragma unroll
        for (int g = 0; g < GP; ++g) {
          acc[g][2 * e2] += wj[g] * lo;
          acc[g][2 * e2 + 1] += wj[g] * hi;
        }
      }
    }
  }
  // sum the four row groups of the wave, then the four waves
#pragma unroll
  for (int g = 0; g < GP; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[g][e];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      acc[g][e] = v;
    }
  if (lg == 0) {
#pragma unroll
    for (int g = 0; g < GP; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) red[w][g][ln * 8 + e] = acc[g][e];
  }
  __syncthreads();
  float* op = P.opart + (bh * P.n_chunk_max + chunk) * GP * kHeadDim;
  for (int i = tid; i < GP * kHeadDim; i += 256) {
    const int g = i / kHeadDim, d = i % kHeadDim;
    op[i] = red[0][g][d] + red[1][g][d] + red[2][g][d] + red[3][g][d];
  }
}

// ------------------------------------------------------------------------------------------------
// raw_attn: grid (chunks of the longest raw segment, Hkv, B), 256 threads.  Appendix B.2 keeps sink and recent
// tokens uncompressed in a pool of their own and attends them together with the reconstructed ones.  A block
// takes kRawChunk raw tokens of one (sequence, kv-head): scores of the group's query heads on the matrix unit
// (as ref_scores), weights 2^(x - m) against the chunk's own largest logit m, then sum_t w_t V_t in fp32 (as
// ref_values).  It depends on nothing the other kernels compute; finalize merges its (m, sum w, sum w V).
// ------------------------------------------------------------------------------------------------
template <int GP>
__global__ __launch_bounds__(256) void k_raw_attn(DecodeParams P) {
  const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int n_raw = clampi(P.raw_lens[b], 0, P.raw_cap);
  const int t0 = chunk * kRawChunk;
  if (t0 >= n_raw) return;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 15, lg = l >> 4;
  __shared__ float sc[kRawChunk][GP];          // scores, then weights
  __shared__ float red[4][GP][kHeadDim];
  __shared__ float mred[4][16];
  __shared__ float msh[GP];
  const int64_t row_stride = (int64_t)P.Hkv * kHeadDim;
  const uint16_t* kseg = P.raw_k + ((int64_t)b * P.raw_cap * P.Hkv + h) * kHeadDim;
  const uint16_t* vseg = P.raw_v + ((int64_t)b * P.raw_cap * P.Hkv + h) * kHeadDim;

  bf16x8 qa[4];
  {
    const uint16_t* qrow = P.q + ((int64_t)b * P.Hq + (int64_t)h * P.G + (ln < P.G ? ln : 0)) * kHeadDim;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 v = *reinterpret_cast<const uint4*>(qrow + (4 * kk + lg) * 8);
      if (ln >= P.G) v = make_uint4(0, 0, 0, 0);
      qa[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }
  // scores: wave w, step st <-> tokens t0 + 64 w + 16 st + ln (rows past the end re-read the last token)
  float mx[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
  for (int st = 0; st < 4; ++st) {
    const int tl = w * 64 + st * 16 + ln;
    const bool valid = t0 + tl < n_raw;
    const uint16_t* krow = kseg + (int64_t)min(t0 + tl, n_raw - 1) * row_stride;
    float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const uint4 kv = *reinterpret_cast<const uint4*>(krow + (4 * kk + lg) * 8);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[kk], __builtin_bit_cast(bf16x8, kv), acc, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x = valid ? acc[i] * P.qk_scale_log2 : -INFINITY;
      if (4 * lg + i < GP) sc[tl][4 * lg + i] = x;      // lane holds heads 4*lg + i of token ln
      mx[i] = fmaxf(mx[i], x);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) mx[i] = wave16_max(mx[i]);
  if (ln == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) mred[w][4 * lg + i] = mx[i];
  }
  __syncthreads();
  if (tid < GP) msh[tid] = fmaxf(fmaxf(mred[0][tid], mred[1][tid]), fmaxf(mred[2][tid], mred[3][tid]));
  __syncthreads();
  // weights of token tid (the chunk holds a valid token, so every m is finite; rows past the end get 0)
  float lsum[GP];
#pragma unroll
  for (int g = 0; g < GP; ++g) {
    const float p = __builtin_amdgcn_exp2f(sc[tid][g] - msh[g]);
    sc[tid][g] = p;
    lsum[g] = p;
  }
#pragma unroll
  for (int g = 0; g < GP; ++g) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) lsum[g] += __shfl_xor(lsum[g], o);
  }
  __syncthreads();                                   // all weights written; mred is free again
  if (l == 0) {
#pragma unroll
    for (int g = 0; g < GP; ++g) mred[w][g] = lsum[g];
  }
  // values: lane = (row-in-group lg, 8-wide d chunk ln); a wave reads four 256-byte V rows per load
  float acc[GP][8];
#pragma unroll
  for (int g = 0; g < GP; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  constexpr int UN = GP >= 16 ? 2 : (GP == 8 ? 4 : 8);
  for (int it0 = 0; it0 < kRawChunk / 16; it0 += UN) {
    uint4 v[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int row = w * (kRawChunk / 4) + (it0 + u) * 4 + lg;
      v[u] = *reinterpret_cast<const uint4*>(vseg + (int64_t)min(t0 + row, n_raw - 1) * row_stride + ln * 8);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int row = w * (kRawChunk / 4) + (it0 + u) * 4 + lg;
      float wj[GP];
#pragma unroll
      for (int g = 0; g < GP; ++g) wj[g] = sc[row][g];
      const uint32_t vv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const float lo = bf16lo(vv[e2]), hi = bf16hi(vv[e2]);
#pragma unroll
        for (int g = 0; g < GP; ++g) {
          acc[g][2 * e2] += wj[g] * lo;
          acc[g][2 * e2 + 1] += wj[g] * hi;
        }
      }
    }
  }
#pragma unroll
  for (int g = 0; g < GP; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[g][e];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      acc[g][e] = v;
    }
  if (lg == 0) {
#pragma unroll
    for (int g = 0; g < GP; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) red[w][g][ln * 8 + e] = acc[g][e];
  }
  __syncthreads();
  const int64_t part = ((int64_t)b * P.Hkv + h) * kRawMaxChunks + chunk;
  float* op = P.rawo + part * GP * kHeadDim;
  for (int i = tid; i < GP * kHeadDim; i += 256) {
    const int g = i / kHeadDim, d = i % kHeadDim;
    op[i] = red[0][g][d] + red[1][g][d] + red[2][g][d] + red[3][g][d];
  }
  if (tid < GP) {
    float* ml = P.rawml + (part * GP + tid) * 2;
    ml[0] = msh[tid];
    ml[1] = mred[0][tid] + mred[1][tid] + mred[2][tid] + mred[3][tid];
  }
}

// Last step of an output row (thread = output dim d): the cached part arrives as (sum of weights lsum, weighted value
// sum o, both in units of 2^frame); the raw-segment chunks are merged at the largest of all frames, so no factor
// exceeds 1; then normalise and store.  Nothing to attend (no weight anywhere) gives out = 0 and lse = -inf.
__device__ inline void finish_output(const DecodeParams& P, int b, int gh, int h, int g, int d, float lsum, float o,
                                     float frame, int n_raw) {
  const int Gp = P.Gp;
  const int64_t bh = (int64_t)b * P.Hkv + h;
  const int64_t orow = ((int64_t)b * P.Hq + gh) * kHeadDim;
  if (n_raw > 0) {
    const int nrc = ceil_div(n_raw, kRawChunk);
    const float* ml = P.rawml + ((bh * kRawMaxChunks) * Gp + g) * 2;
    float top = lsum > 0.f ? frame : -INFINITY;
    for (int c = 0; c < nrc; ++c) top = fmaxf(top, ml[(int64_t)c * Gp * 2]);
    const float fc = lsum > 0.f ? __builtin_amdgcn_exp2f(frame - top) : 0.f;
    lsum *= fc;
    o *= fc;
    const float* ro = P.rawo + ((bh * kRawMaxChunks) * Gp + g) * kHeadDim + d;
    for (int c = 0; c < nrc; ++c) {
      const float f = __builtin_amdgcn_exp2f(ml[(int64_t)c * Gp * 2] - top);
      lsum += f * ml[(int64_t)c * Gp * 2 + 1];
      o += f * ro[(int64_t)c * Gp * kHeadDim];
    }
    frame = top;
  }
  const bool any = lsum > 0.f;
  P.out[orow + d] = any ? (uint16_t)f32_to_bf16_bits(o / lsum) : (uint16_t)0;
  if (d == 0 && P.lse) P.lse[(int64_t)b * P.Hq + gh] = any ? (frame + __log2f(lsum)) * kLn2 : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
// rescue (a branch of finalize: the block of one output row, 128 threads).  The streaming path keeps every softmax weight in one fixed frame per
// (sequence, q-head), 2^(x - m_ref - bias) with m_ref the largest per-reference score; that holds logits up to 86
// nats above m_ref (55 nats either way for a selection), which is where reconstructed keys of small residuals live.
// A row whose weights left that range (finalize saw a sum at or beyond 2^60, or below 2^-100), or whose block ran out of room for oversized table
// amounts, is recomputed here from the cache by the definition: pass 1 finds the exact largest logit of the row,
// pass 2 accumulates weights against it (all <= 1), sum_t p_t V_ref[idx_t] and sum_t p_t z_V,t directly.  Slow
// (every latent value is fetched on its own) and always right; logits use the same operands as the streaming
// kernel (per-reference scores and W_uK q of ref_scores, in log2 units).
// ------------------------------------------------------------------------------------------------
// Latent value c of token `tok` in the (page, head, stream) block that starts at `blk` (any of the four layouts).
__device__ inline float latent_value(const DecodeParams& P, const uint16_t* blk, int tok, int c, bool value_stream) {
  if (!P.q4) {
    const int at = value_stream ? ((c >> 4) * 64 + (tok >> 2) * 16 + (c & 15)) * 4 + (tok & 3)
                                : ((c >> 3) * kPage + tok) * 8 + (c & 7);
    return bf16lo(blk[at]);
  }
  const uint32_t* words = reinterpret_cast<const uint32_t*>(blk);
  uint32_t code;
  if (value_stream) {
    const uint32_t w = words[2 * ((c >> 6) * 64 + (tok >> 2) * 16 + (c & 15)) + ((tok & 3) >> 1)];
    code = (w >> (4 * ((c >> 4) & 3) + 16 * (tok & 1))) & 15u;
  } else {
    const uint32_t w = words[(c >> 3) * kPage + tok];
    code = (w >> (4 * ((c & 7) >> 1) + 16 * (c & 1))) & 15u;
  }
  const uint16_t* sz = blk + 4 * P.R + (tok >> 2) * 8 + (tok & 3);      // four scales, then four zero points
  return bf16lo(sz[0]) * (float)code + bf16lo(sz[4]);
}

__device__ __forceinline__ void rescue_row(const DecodeParams& P, int b, int gh) {
  constexpr int NT = 128;               // threads of the block = tokens per tile
  const int tid = threadIdx.x;
  const int G = P.G, Gp = P.Gp, R = P.R;
  const int h = gh / G, g = gh % G;
  const int L = seq_len_of(P, b);
  const int n_ent = work_pages_of(P, b, L);                  // entries of the page list (>= 1: the row was flagged)
  const int n_raw = P.raw_k ? clampi(P.raw_lens[b], 0, P.raw_cap) : 0;
  const int n_ref = refs_below(L, P.stride);
  const int64_t bh = (int64_t)b * P.Hkv + h;
  __shared__ float ql[kHeadDim];        // W_uK q of this head (hi + lo), log2 units
  __shared__ float pw[NT];              // weights of the current tile
  __shared__ int psl[4][NT];            // reference pool slots of each token of the tile (-1: ordinal slot unused)
  __shared__ float red[NT];
  if (tid < R) {
    const int64_t at = ((int64_t)b * P.Hq + gh) * R + tid;
    ql[tid] = bf16lo(P.qlat[at]) + bf16lo(P.qlat[P.qlat_lo_offset + at]);
  }
  __syncthreads();
  const float* sref = P.sref + bh * P.n_ref_max * Gp + g;
  const int last_logical = ceil_div(L, kPage) - 1;
  // token i of the row = (list entry i / 16, slot i % 16); returns whether it takes part, its logit and ordinal
  // (ords: the token's reference ordinals, -1 in unused slots; the reference part of the logit is the mean score)
  auto token = [&](int i, float& x, int (&ords)[4], const uint16_t*& blk) {
    const int e = i >> 4, tok = i & 15;
    if (e >= n_ent) return false;
    int logical = e;
    uint32_t mask = 0xffffu;
    if (P.sel_pages) {
      logical = P.sel_pages[(int64_t)b * P.sel_stride + e];
      mask = (uint32_t)P.sel_masks[(int64_t)b * P.sel_stride + e];
      if ((uint32_t)logical > (uint32_t)last_logical) return false;
    }
    if (logical * kPage + tok >= L || !((mask >> tok) & 1u)) return false;
    const int page = clampi(P.block_tables[(int64_t)b * P.bt_stride + logical], 0, (int)P.n_pages_pool - 1);
    const int32_t* ip = P.idx + (int64_t)page * P.idx_page_stride + (int64_t)h * P.idx_head_stride + tok;
    float sacc = 0.f;
    int cnt = 0;
    for (int i2 = 0; i2 < 4; ++i2) {
      const int raw = i2 < P.top_k ? ip[i2 * kPage] : -1;
      // one slot per token: the stored value is clamped, never trusted; several: a negative one marks an unused slot
      const bool used = i2 < P.top_k && (P.top_k == 1 || raw >= 0);
      ords[i2] = used ? (int)min((uint32_t)raw, (uint32_t)(n_ref - 1)) : -1;
      if (used) { sacc += sref[(int64_t)ords[i2] * Gp]; ++cnt; }
    }
    blk = P.latent + (int64_t)page * P.latent_page_stride + (int64_t)h * P.latent_head_stride;
    float acc = 0.f;
    for (int c = 0; c < R; ++c) acc += ql[c] * latent_value(P, blk, tok, c, false);
    x = sacc / (float)max(cnt, 1) + acc;
    return true;
  };
  const int n_tok = n_ent * kPage;
  // pass 1: the row's largest logit
  float m = -INFINITY;
  for (int i = tid; i < n_tok; i += NT) {
    float x; int ords[4]; const uint16_t* blk;
    if (token(i, x, ords, blk)) m = fmaxf(m, x);
  }
  red[tid] = m;
  __syncthreads();
  for (int o2 = NT / 2; o2 > 0; o2 >>= 1) {
    if (tid < o2) red[tid] = fmaxf(red[tid], red[tid + o2]);
    __syncthreads();
  }
  m = red[0];
  __syncthreads();
  // pass 2: tiles of 128 tokens; a thread owns an output dim and (the first R threads) a latent column
  float lsum = 0.f, o = 0.f, zs = 0.f;
  const uint16_t* vbase = P.ref + (int64_t)h * P.ref_head_stride + P.ref_kv_stride;
  const int64_t vstream = P.joint ? 0 : P.latent_stream_stride;
  for (int i0 = 0; i0 < n_tok; i0 += NT) {
    float x; int ords[4] = {-1, -1, -1, -1}; const uint16_t* blk = nullptr;
    const bool on = token(i0 + tid, x, ords, blk);
    pw[tid] = on ? __builtin_amdgcn_exp2f(x - m) : 0.f;
    for (int i2 = 0; i2 < 4; ++i2)
      psl[i2][tid] = on && ords[i2] >= 0 ? clampi(P.ref_tables[(int64_t)b * P.rt_stride + ords[i2]], 0, (int)P.n_ref_slots - 1) : -1;
    __syncthreads();
    const int n_here = min(NT, n_tok - i0);
    for (int t = 0; t < n_here; ++t) {
      const float p = pw[t];
      if (p == 0.f) continue;                                  // tokens that take no part may hold anything
      float vsum = 0.f;                                        // mean of the token's reference value rows
      int cnt = 0;
      for (int i2 = 0; i2 < 4; ++i2)
        if (psl[i2][t] >= 0) { vsum += bf16lo(vbase[(int64_t)psl[i2][t] * kHeadDim + tid]); ++cnt; }
      o += p * vsum / (float)max(cnt, 1);
      lsum += p;
      if (tid < R) {
        const int i = i0 + t, e = i >> 4;
        const int logical = P.sel_pages ? P.sel_pages[(int64_t)b * P.sel_stride + e] : e;
        const int page = clampi(P.block_tables[(int64_t)b * P.bt_stride + logical], 0, (int)P.n_pages_pool - 1);
        const uint16_t* vb = P.latent + (int64_t)page * P.latent_page_stride + (int64_t)h * P.latent_head_stride + vstream;
        zs += p * latent_value(P, vb, i & 15, tid, !P.joint);
      }
    }
    __syncthreads();
  }
  // up-projection of the weighted latent sum
  red[tid] = zs;
  __syncthreads();
  for (int c = 0; c < R; ++c) o += red[c] * bf16lo(P.w_up_v[(int64_t)c * kHeadDim + tid]);
  finish_output(P, b, gh, h, g, tid, lsum, o, m, n_raw);
}

// ------------------------------------------------------------------------------------------------
// finalize: grid (Hq, B), 128 threads (thread = output dim d); one block per query head.
// ------------------------------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(128) void k_finalize(DecodeParams P) {
  const int gh = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int G = P.G, Gp = P.Gp;
  // the thread's column of W_uV does not depend on anything computed here: all R loads are issued first and land
  // under the latency of the partial-sum loads below
  uint16_t wcol[R];
#pragma unroll
  for (int cc = 0; cc < R; ++cc) wcol[cc] = P.w_up_v[(int64_t)cc * kHeadDim + d];
  const int rescue_flag = P.rescue[(int64_t)b * P.Hq + gh];      // set by a streaming block that lost weights
  const int h = gh / G, g = gh % G;
  const int L = seq_len_of(P, b);
  const int64_t orow = ((int64_t)b * P.Hq + gh) * kHeadDim;
  const int n_pages = work_pages_of(P, b, L);
  const int n_raw = P.raw_k ? clampi(P.raw_lens[b], 0, P.raw_cap) : 0;
  if (n_pages <= 0 && n_raw <= 0) {         // nothing to attend: empty sequence or selection, no raw tokens
    P.out[orow + d] = 0;
    if (P.lse && d == 0) P.lse[(int64_t)b * P.Hq + gh] = -INFINITY;
    return;
  }
  __shared__ float zsum[128];
  __shared__ float redm[2];
  const int64_t bh = (int64_t)b * P.Hkv + h;
  // the cached tokens: weights 2^(x - frame), frame = m_ref + bias
  float lsum = 0.f, o = 0.f, frame = -INFINITY;
  if (n_pages > 0) {                        // uniform over the block
    const int n_ref = refs_below(L, P.stride);
    const int nch = ceil_div(n_ref, kRefChunk);
    const SplitPlan sp = plan_splits(n_pages, P.S, P.pages_per_split);
    int n_used = 0;
    for (int s = 0; s < sp.n_splits; ++s)
      if (s * sp.per < n_pages) n_used = s + 1;
    // loads of all split slots are unconditional (slots past the used ones hold stale values and are dropped
    // afterwards): behind a branch each load would wait for the one before it
    {
      float lp[kMaxSplits];
#pragma unroll
      for (int s = 0; s < kMaxSplits; ++s) lp[s] = P.lpart[(bh * P.S + min(s, P.S - 1)) * Gp + g];
#pragma unroll
      for (int s = 0; s < kMaxSplits; ++s) lsum += s < n_used ? lp[s] : 0.f;
    }
    float mref = -INFINITY;
    for (int c = d; c < nch; c += 128) mref = fmaxf(mref, P.cmax[(bh * P.n_chunk_max + c) * Gp + g]);
#pragma unroll
    for (int o2 = 1; o2 < 64; o2 <<= 1) mref = fmaxf(mref, __shfl_xor(mref, o2));
    if ((d & 63) == 0) redm[d >> 6] = mref;
    {
      const int dd = d < R ? d : R - 1;
      float ap[kMaxSplits];
#pragma unroll
      for (int s = 0; s < kMaxSplits; ++s) ap[s] = P.accpart[((bh * P.S + min(s, P.S - 1)) * Gp + g) * R + dd];
      float a = 0.f;
#pragma unroll
      for (int s = 0; s < kMaxSplits; ++s) a += s < n_used ? ap[s] : 0.f;
      if (d < R) zsum[d] = a;
    }
    // the chunk partials do not depend on anything above either: their loads go out before the barrier, sixteen at a
    // time (a 131072-token sequence has 32 chunks: two round trips instead of the four behind the barrier)
    {
      const float* op = P.opart + (bh * P.n_chunk_max * Gp + g) * kHeadDim + d;
      const int64_t cstride = (int64_t)Gp * kHeadDim;
      int c = 0;
      for (; c + 16 <= nch; c += 16) {
        float t[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) t[u] = op[(c + u) * cstride];
#pragma unroll
        for (int u = 0; u < 16; ++u) o += t[u];
      }
      for (; c + 4 <= nch; c += 4) {
        float t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = op[(c + u) * cstride];
#pragma unroll
        for (int u = 0; u < 4; ++u) o += t[u];
      }
      for (; c < nch; ++c) o += op[c * cstride];
    }
    __syncthreads();
    frame = fmaxf(redm[0], redm[1]) + exp_bias(P.sel_pages != nullptr);
#pragma unroll
    for (int cc = 0; cc < R; ++cc) o += zsum[cc] * bf16lo(wcol[cc]);
    // The fixed exponent frame holds weights between 2^-126 and 2^127.  A weight of 2^60 or more (any such weight
    // makes the sum at least that large) risks overflow of the fp32 sums; a sum below 2^-100 means every attended
    // token lies so far under the largest reference score that weights of some weight may have been flushed to
    // zero (only a selection can do that: a reference token of the full cache weighs 2^-64 or more; with the sum
    // at 2^-100 or more a flushed weight is below 2^-26 of it).  Such a row, and the rows of a (sequence, kv-head)
    // whose streaming block ran out of room for oversized table amounts, are recomputed by the rescue branch
    // with the row's exact maximum as its offset (uniform over the block: every thread holds the same sum).
    if (!(lsum >= kSumLo && lsum < kSumHi) || rescue_flag != 0) {
      if (d == 0 && !(lsum >= kSumLo && lsum < kSumHi)) atomicOr(P.status, 1);
      __syncthreads();
      rescue_row(P, b, gh);
      return;
    }
  }
  finish_output(P, b, gh, h, g, d, lsum, o, frame, n_raw);
}

// ------------------------------------------------------------------------------------------------
// host launcher
// ------------------------------------------------------------------------------------------------

size_t stream_lds_bytes(int n_rows, int Gp, int R, int nw, bool joint) {
  size_t b = (size_t)(((n_rows * Gp + 3) & ~3) + Gp * R + 16 + nw * 16) * sizeof(float);
  if (joint) b += (size_t)nw * 16 * (R + 8) * 2;
  b += (size_t)(4 + 2 * kOvfCap) * 4;   // overflow list of the fixed-point table
  return b;
}

hipError_t launch_decode(const DecodeParams& P, int batch, int n_items, int nw, size_t lds, hipStream_t st) {
  hipError_t e;
  dim3 gchunk(P.n_chunk_max, P.Hkv, batch);
  timing_mark(-1, st);
  if (P.raw_k && P.raw_cap > 0) {
    dim3 graw(ceil_div(P.raw_cap, kRawChunk), P.Hkv, batch);
    switch (P.Gp) {
      case 4: hipLaunchKernelGGL(k_raw_attn<4>, graw, dim3(256), 0, st, P); break;
      case 8: hipLaunchKernelGGL(k_raw_attn<8>, graw, dim3(256), 0, st, P); break;
      case 16: hipLaunchKernelGGL(k_raw_attn<16>, graw, dim3(256), 0, st, P); break;
      default: return hipErrorInvalidValue;
    }
    if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of raw_attn");
    timing_mark(K_RAW, st);
  }
  if (P.ref_cpb == 4)
    hipLaunchKernelGGL(k_ref_scores<4>, dim3(ceil_div(P.n_chunk_max, 4), P.Hkv, batch), dim3(256), 0, st, P);
  else
    hipLaunchKernelGGL(k_ref_scores<1>, gchunk, dim3(256), 0, st, P);
  if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of ref_scores");
  timing_mark(K_REF_SCORES, st);
  dim3 gs(n_items > 0 ? n_items * P.Hkv : 1);
  if (nw != 8) return hipErrorInvalidValue;
  // one translation unit per family of streaming-kernel variants (they compile side by side)
  if (P.q4)
    e = P.joint ? stream_q4_joint(P, gs, lds, st) : stream_q4_split(P, gs, lds, st);
  else if (P.sel_pages)
    e = P.joint ? stream_joint_subset(P, gs, lds, st) : stream_split_subset(P, gs, lds, st);
  else
    e = P.joint ? stream_joint_full(P, gs, lds, st) : stream_split_full(P, gs, lds, st);
  if (e != hipSuccess) return e;
  timing_mark(K_STREAM, st);
  switch (P.Gp) {
    case 4: hipLaunchKernelGGL(k_ref_values<4>, gchunk, dim3(256), 0, st, P); break;
    case 8: hipLaunchKernelGGL(k_ref_values<8>, gchunk, dim3(256), 0, st, P); break;
    case 16: hipLaunchKernelGGL(k_ref_values<16>, gchunk, dim3(256), 0, st, P); break;
    default: return hipErrorInvalidValue;
  }
  if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of ref_values");
  timing_mark(K_REF_VALUES, st);
  switch (P.R) {
    case 16: hipLaunchKernelGGL(k_finalize<16>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    case 32: hipLaunchKernelGGL(k_finalize<32>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    case 48: hipLaunchKernelGGL(k_finalize<48>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    case 64: hipLaunchKernelGGL(k_finalize<64>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    case 80: hipLaunchKernelGGL(k_finalize<80>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    case 96: hipLaunchKernelGGL(k_finalize<96>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    case 112: hipLaunchKernelGGL(k_finalize<112>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    case 128: hipLaunchKernelGGL(k_finalize<128>, dim3(P.Hq, batch), dim3(128), 0, st, P); break;
    default: return hipErrorInvalidValue;
  }
  e = note_hip_error(hipGetLastError(), "launch of finalize");
  timing_mark(K_FINALIZE, st);
  return e;
}

}  // namespace dkv
