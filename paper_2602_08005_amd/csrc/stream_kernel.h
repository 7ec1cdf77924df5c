// The streaming kernel of the decode call (latent + ordinal pass) and its launcher templates.  Included by the
// stream_*.hip translation units, each of which instantiates one family of variants, so that they compile in parallel.
#pragma once
#include "decode_common.h"

namespace dkv {

// ------------------------------------------------------------------------------------------------
// stream: 1-D grid over the (sequence, split) items that ref_scores lists, times kv-heads; NW waves.
// Dynamic LDS: [n_tab] fixed-point w table, then small reduction buffers and the overflow list.
// ------------------------------------------------------------------------------------------------
template <int R, bool Q4>
struct Tile {
  static constexpr int NKK = (R + 31) / 32;
  static constexpr int NB = R / 16;
  uint4 zk[NKK];   // scores operand: token l%16, latent chunk l/16 + 4*kk
  uint2 zv[NB];    // value operand: column l%16 + 16*nb, tokens 4*(l/16)..+3
};
// 4-bit token-wise latents (section 5.3; one stream, JOINT mode): eight codes per dword instead of eight bf16
// values per 16 bytes, plus the bf16 scales and zero points of the lane's four tokens 4*(l/16)..+3.
template <int R>
struct Tile<R, true> {
  static constexpr int NKK = (R + 31) / 32;
  static constexpr int NB = R / 16;
  static constexpr int NQ = (NB + 3) / 4;
  uint32_t zc[NKK];   // codes of token l%16, latent chunk l/16 + 4*kk (value c%8 at bits 4*((c%8)/2) + 16*(c%2))
  uint4 sz;           // scales of tokens 4*(l/16)..+3 (x, y), their zero points (z, w), bf16 pairs
  uint2 zv[NB];       // value operand, built on chip
  // two-stream layout only: codes of the value stream, columns l%16 + 16*nb of tokens 4*(l/16)..+3 (.x: first and
  // second token at bits 4*(nb%4) and 16 + 4*(nb%4), .y: third and fourth), and that stream's scales / zero points
  uint2 zvc[NQ];
  uint4 szv;
};

// Loads of the streaming loop take their address as (uniform 64-bit base of the page) + (32-bit offset of the
// lane), which the hardware forms itself (scalar base + vector offset): no vector arithmetic per load.  The bf16
// latent loads are non-temporal: every record is read once, and letting two gigabytes of them flow through the L2
// as ordinary lines kept evicting the per-reference score rows that the gathers come back to (11 % of the
// kernel's time).  The same hint on the ordinals, or on the small 4-bit records, changed nothing; and a cache that
// fits the chip's last-level cache and is read again by the next call (a single sequence's decode loop) is better
// off with ordinary loads, so the host picks the variant (NT) by the size of what the call streams.
// DENSE (see k_stream): the lane needs the scale and zero point of ONE token, 4*(l/16) + (l%16)/4: two 2-byte loads
// into sz.x / sz.z (szv likewise) instead of the group's sixteen bytes and the selects that pick a token out of them.
template <int R, bool JOINT, bool NT, bool DENSE = false>
__device__ inline void load_latents(const char* lat_h, uint32_t page_bytes, uint32_t stream_bytes, int page,
                                    uint32_t l, Tile<R, true>& t) {
  const char* base = lat_h + (uint64_t)(uint32_t)page * page_bytes;
  const uint32_t lg = l >> 4, te2 = ((l & 15u) >> 2) * 2u;
#pragma unroll
  for (int kk = 0; kk < Tile<R, true>::NKK; ++kk) {
    if (4 * kk + lg < R / 8)
      t.zc[kk] = *reinterpret_cast<const uint32_t*>(base + (l * 4u + kk * 256u));
    else
      t.zc[kk] = 0u;
  }
  if constexpr (DENSE) {
    t.sz.x = *reinterpret_cast<const uint16_t*>(base + (8u * R + lg * 16u + te2));
    t.sz.z = *reinterpret_cast<const uint16_t*>(base + (8u * R + lg * 16u + 8u + te2));
  } else {
    t.sz = *reinterpret_cast<const uint4*>(base + (8u * R + lg * 16u));
  }
  if (!JOINT) {
    const char* vb = base + stream_bytes;
#pragma unroll
    for (int q = 0; q < Tile<R, true>::NQ; ++q) t.zvc[q] = *reinterpret_cast<const uint2*>(vb + (l * 8u + q * 512u));
    if constexpr (DENSE) {
      t.szv.x = *reinterpret_cast<const uint16_t*>(vb + (8u * R + lg * 16u + te2));
      t.szv.z = *reinterpret_cast<const uint16_t*>(vb + (8u * R + lg * 16u + 8u + te2));
    } else {
      t.szv = *reinterpret_cast<const uint4*>(vb + (8u * R + lg * 16u));
    }
  }
}
template <int R, bool JOINT, bool NT, bool DENSE = false>
__device__ inline void load_latents(const char* lat_h, uint32_t page_bytes, uint32_t stream_bytes, int page,
                                    uint32_t l, Tile<R, false>& t) {
  const char* base = lat_h + (uint64_t)(uint32_t)page * page_bytes;
  const uint32_t lg = l >> 4;
#pragma unroll
  for (int kk = 0; kk < Tile<R, false>::NKK; ++kk) {
    if (4 * kk + lg < R / 8)
      t.zk[kk] = NT ? __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(base + (l * 16u + kk * 1024u))))
                    : *reinterpret_cast<const uint4*>(base + (l * 16u + kk * 1024u));
    else
      t.zk[kk] = make_uint4(0, 0, 0, 0);
  }
  if (!JOINT) {
    const char* vb = base + stream_bytes;
#pragma unroll
    for (int nb = 0; nb < Tile<R, false>::NB; ++nb)
      t.zv[nb] = NT ? __builtin_bit_cast(uint2, __builtin_nontemporal_load(reinterpret_cast<const uint2v*>(vb + (l * 8u + nb * 512u))))
                    : *reinterpret_cast<const uint2*>(vb + (l * 8u + nb * 512u));
  }
}
// One ordinal per lane: lane (row lg = l/16, quad position l%4) holds the ordinal of token 4*lg + l%4, so the four
// tokens a lane works on sit in the four lanes of its own quad and are fetched with quad-broadcast DPP moves when
// needed (one register per page in flight instead of four).
__device__ inline int load_ordinal(const char* idx_h, uint32_t page_bytes, int page, uint32_t l) {
  return *reinterpret_cast<const int*>(idx_h + (uint64_t)(uint32_t)page * page_bytes + (((l >> 4) * 4u + (l & 3u)) * 4u));
}
// Top-k retrieval (section 4.1: the reference of a token is the mean of its k nearest references): the index pool
// holds KS ordinal slots per token, [slot][token] inside a (page, head) block, -1 in the slots a token does not use.
// The kernel variant for k > 1 always works on four slots; with k = 2 slots 2 and 3 re-read slot 1 and are ignored.
// DENSE (see k_stream): the lane holds the ordinal of token 4*(l/16) + (l%16)/4 instead.
template <int KS, bool DENSE = false>
__device__ inline void load_ordinals(const char* idx_h, uint32_t page_bytes, int page, uint32_t l, int top_k, int (&out)[KS]) {
  const char* base = idx_h + (uint64_t)(uint32_t)page * page_bytes + (((l >> 4) * 4u + (DENSE ? (l & 15u) >> 2 : l & 3u)) * 4u);
#pragma unroll
  for (int i = 0; i < KS; ++i) out[i] = *reinterpret_cast<const int*>(base + (uint32_t)min(i, top_k - 1) * (kPage * 4u));
}
template <int E>
__device__ inline int quad_bcast(int v) {   // value held by lane E of the caller's quad
  return __builtin_amdgcn_update_dpp(0, v, E * 0x55, 0xf, 0xf, true);
}

// Grid: 1-D, one block per (item, kv-head) with the head fastest, where the items are the non-empty
// (sequence, split) pairs listed by ref_scores: no block of the grid is empty, whatever the mix of lengths.  (Empty
// blocks are not free here: each needs a whole compute unit's LDS before it can start and exit.)  Blocks of the kv-heads
// of one item run side by side and sweep the same pages; with eight kv-heads, block id % 8 = head, so all splits of a
// (sequence, head) also share one XCD's L2 copy of that pair's per-reference score table.
// SPILL: sequences whose per-reference weight table does not fit the LDS (beyond roughly 160 000 tokens at four query
// heads per kv-head).  The LDS table then covers a window of the P.tab_cap most recent ordinals the block can touch
// -- its own tokens' ordinals among them: every 16th token is a reference pointing at itself -- and weights of older
// ordinals are added, as plain floats with hardware float atomics, to one table per (sequence, kv-head) in global
// memory that all splits share (zeroed by ref_scores, read by ref_values).
// DENSE (at most four query heads per kv-head, one ordinal slot): the score product leaves a lane with four tokens of
// ONE head, and only the 16 lanes of heads 0..3 hold anything; everything that is done once per (token, head) --
// exponential, table units, rounding, the LDS atomic and the check of its return value, about two thirds of the
// kernel's vector instructions -- then runs four times per lane on a quarter of the lanes.  The dense variant first
// spreads the 64 (token, head) pairs of a page over the 64 lanes (three DPP row shifts: lane (lg, 4e + g) takes token
// 4 lg + e of head g from lane (lg, g)), does that work once per lane, and shifts the weights back into the operand
// layout of the value product (three row shifts the other way).  Ordinals and per-reference scores are loaded
// directly in the dense mapping.
template <int R, int NW, int PIPE_LG, bool JOINT, bool SUBSET, bool Q4, bool NT, bool SPILL, int KS, bool DENSE = false>
__global__ __launch_bounds__(NW * 64) void k_stream(DecodeParams P) {
  static_assert(KS == 1 || (KS == 4 && !SPILL && !Q4), "four ordinal slots: bf16 latents, on-chip table only");

  static_assert(!Q4 || JOINT || R % 64 == 0, "two-stream 4-bit latents: four 16-column blocks share a dword");
  typedef Tile<R, Q4> TileT;
  extern __shared__ float smem[];
  const int item_q = blockIdx.x / P.Hkv, h = blockIdx.x % P.Hkv;
  if (item_q >= P.items[0]) return;
  const int item = P.items[1 + item_q];
  const int b = min(item / kMaxSplits, P.batch - 1), s = item % kMaxSplits;
  const int pair = b * P.Hkv + h;
  const int L = seq_len_of(P, b);
  if (L <= 0) return;
  const int n_pages = work_pages_of(P, b, L);             // entries of the sequence's page list
  if (n_pages <= 0) return;
  const SplitPlan sp = plan_splits(n_pages, P.S, P.pages_per_split);
  if (s >= sp.n_splits) return;
  const int p0 = s * sp.per, p1 = min(n_pages, p0 + sp.per);
  if (p0 >= p1) return;
  const int n_cov = refs_covered(P, b, L, p1);          // ordinals this split can touch
  const int n_ref = refs_below(L, P.stride);
  const int Gp = P.Gp, G = P.G;
  const int n_win = SPILL ? min(n_cov, P.tab_cap) : n_cov;   // ordinals [win_lo, n_cov) live in the LDS table
  const int win_lo = n_cov - n_win;
  const int n_tab = n_win * Gp;
  float* tab = smem;
  float* accbuf = smem + ((n_tab + 3) & ~3);              // [Gp][R]
  float* lbuf = accbuf + Gp * R;                          // [16]
  float* xbuf = lbuf + 16;                                // [NW][16]; the first 16 hold each head's table-unit base
  const int tid = threadIdx.x;
  const uint32_t l = tid & 63, ln = l & 15, lg = l >> 4;
  const uint32_t hd = DENSE ? (ln & 3u) : ln;             // the query head of the lane's per-(token, head) arithmetic
  const uint32_t te = ln >> 2;                            // DENSE: the lane's token is 4 lg + te
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  // JOINT: per-wave [16 tokens][R + 8] bf16 scratch used to turn the single latent stream (stored in
  // scores-operand order) into the value-operand order of the P.z product
  constexpr int TRP = R + 8;
  uint16_t* tr = reinterpret_cast<uint16_t*>(xbuf + NW * 16) + w * 16 * TRP;
  // overflow list of the fixed-point table: [0] = number of records, then entry indices, then amounts
  uint32_t* ovf = reinterpret_cast<uint32_t*>(xbuf + NW * 16) + (JOINT ? NW * 16 * TRP / 2 : 0);
  uint32_t* pgctr = ovf + 1;            // next undrawn page position of the block
  uint32_t* ovf_ent = ovf + 4;
  float* ovf_val = reinterpret_cast<float*>(ovf_ent + kOvfCap);
  uint32_t* utab = reinterpret_cast<uint32_t*>(tab);
  // The chunk maxima of the per-reference scores (n_cm floats, at most a few hundred) are fetched with one load
  // per thread and staged in the still unused overflow list; read one after the other from global memory they cost a
  // round trip each, 32 in a row at 131072 tokens, which was most of a block's set-up time.
  const int64_t bh = (int64_t)b * P.Hkv + h;
  const int n_cm = ceil_div(n_ref, kRefChunk) * Gp;
  const bool cm_staged = n_cm <= kOvfCap;
  float cm_mine = -INFINITY;
  if (cm_staged && tid < n_cm) cm_mine = P.cmax[bh * P.n_chunk_max * Gp + tid];
  if (!cm_staged) {
    // long sequences (more chunk maxima than the list holds; the table then has thousands of entries): every thread
    // reduces a strided share -- NW * 64 is a multiple of Gp, so a thread's entries all belong to one head -- and the
    // partial maxima are staged in the table area, which is cleared afterwards
    for (int i = tid; i < n_cm; i += NW * 64) cm_mine = fmaxf(cm_mine, P.cmax[bh * P.n_chunk_max * Gp + i]);
    tab[tid] = cm_mine;
    __syncthreads();
  }
  float mref = -INFINITY;                                  // exponent offset for q-head g = hd (see below)
  if (!cm_staged) {
    const int gcol = hd < (uint32_t)Gp ? hd : Gp - 1;
    for (int k = gcol; k < NW * 64; k += Gp) mref = fmaxf(mref, tab[k]);
    __syncthreads();
  }
  for (int i = tid; i < n_tab; i += NW * 64) utab[i] = 0u;
  for (int i = tid; i < Gp * R + 16; i += NW * 64) accbuf[i] = 0.f;
  if (tid == 0) { ovf[0] = 0u; pgctr[0] = 0u; }
  if (cm_staged) {
    if (tid < n_cm) ovf_val[tid] = cm_mine;
    __syncthreads();
  }

  const uint32_t gq = hd < (uint32_t)Gp ? hd : Gp - 1;    // column of the score table this lane reads
  const bool ghead = hd < (uint32_t)G;                    // the lane does per-(token, head) work
  const bool ghead_op = ln < (uint32_t)G;                 // the lane's column of the matrix operands is a query head
  // exponent offset for q-head g = hd: the largest chunk maximum (the staged copy is free again after the barrier
  // that ends the set-up)
  if (cm_staged) {
    const int nch = ceil_div(n_ref, kRefChunk);
    for (int c = 0; c < nch; ++c) mref = fmaxf(mref, ovf_val[c * Gp + gq]);
  }
  const float cinit = -(mref + exp_bias(SUBSET));
  const float cshift = table_shift_base(mref, exp_bias(SUBSET));
  if (tid < 16) { xbuf[tid] = cshift; xbuf[16 + tid] = 0.f; }
  float* zbuf = xbuf + 16;                                // [16] 4-bit latents: sum of weight x zero-point term per head
  // B operand of the score product: (W_uK q) for head g = ln, latent chunk 4*kk + lg
  // (stored as bf16 hi + lo parts, so that the latent part of the logit keeps fp32-like accuracy)
  bf16x8 qb[TileT::NKK], qbl[TileT::NKK];
  {
    const uint16_t* qrow = P.qlat + ((int64_t)b * P.Hq + (int64_t)h * G + (ghead_op ? ln : 0)) * R;
#pragma unroll
    for (int kk = 0; kk < TileT::NKK; ++kk) {
      uint4 v = make_uint4(0, 0, 0, 0), vl = v;
      if (ghead_op && 4 * kk + lg < R / 8) {
        v = *reinterpret_cast<const uint4*>(qrow + (4 * kk + lg) * 8);
        vl = *reinterpret_cast<const uint4*>(qrow + P.qlat_lo_offset + (4 * kk + lg) * 8);
      }
      qb[kk] = __builtin_bit_cast(bf16x8, v);
      qbl[kk] = __builtin_bit_cast(bf16x8, vl);
    }
  }
  // 4-bit latents: a value reads back as scale * code + zero; the operand holds 16 + code (exact in bf16), so
  //   q . z = scale * (q . (16 + code)) + (zero - 16 * scale) * sum(q)        and
  //   sum_t p_t z_t = sum_t (p_t scale_t) (16 + code_t) + (sum_t p_t (zero_t - 16 scale_t)) * (1, ..., 1)
  // qsum = sum over the latent dims of this lane's query head
  float qsum = 0.f;
  if (Q4) {
#pragma unroll
    for (int kk = 0; kk < TileT::NKK; ++kk) {
      const uint4 a = __builtin_bit_cast(uint4, qb[kk]), c = __builtin_bit_cast(uint4, qbl[kk]);
      const uint32_t u[8] = {a.x, a.y, a.z, a.w, c.x, c.y, c.z, c.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) qsum += bf16lo(u[e]) + bf16hi(u[e]);
    }
    qsum += __shfl_xor(qsum, 16);
    qsum += __shfl_xor(qsum, 32);
    if (DENSE) qsum = __shfl(qsum, (int)hd);              // of the lane's own head (lanes 0..3 hold heads 0..3)
  }
  float zacc = 0.f;
  // bf16 pair (16.0, 16.0); kept in a vector register (opaque to the compiler) so that (x & mask) | c16 is a single
  // and-or instruction: such an instruction can take only one literal constant
  uint32_t c16 = 0x41804180u;
  if (Q4) asm volatile("" : "+v"(c16));
  // uniform bases of this (sequence, kv-head): score table row block, latent and ordinal pools at head h
  const char* sref_bh = reinterpret_cast<const char*>(P.sref + bh * P.n_ref_max * Gp);
  const char* lat_h = reinterpret_cast<const char*>(P.latent + (int64_t)h * P.latent_head_stride);
  const char* idx_h = reinterpret_cast<const char*>(P.idx + (int64_t)h * P.idx_head_stride);
  const uint32_t lat_page_bytes = (uint32_t)P.latent_page_stride * 2u, lat_stream_bytes = (uint32_t)P.latent_stream_stride * 2u;
  const uint32_t idx_page_bytes = (uint32_t)P.idx_page_stride * 4u;
  const int gsh2 = group_shift(Gp) + 2;                   // ordinal -> byte offset of its table row
  const uint32_t gq4 = gq * 4u, ln4 = hd * 4u;            // (byte offset of the lane's head inside a table row)
  const uint32_t id_hi = (uint32_t)(n_cov - 1);
  float* spill_bh = SPILL ? P.spill + bh * P.n_ref_max * Gp : nullptr;
  __syncthreads();

  float4v acc[TileT::NB];
#pragma unroll
  for (int nb = 0; nb < TileT::NB; ++nb) acc[nb] = float4v{0.f, 0.f, 0.f, 0.f};
  float lsum = 0.f;
  // lanes that hold no query head start their accumulator at -inf, so their weights are exactly 0
  // (the accumulator belongs to the operand column ln; for ln < 4 that is the lane's own head in either mapping)
  const float cstart = (Q4 ? ghead : ghead_op) ? cinit : -INFINITY;

  // Per-reference scores of a page: the lane fetches, with ONE 16-byte load, four heads of the row of the token
  // whose ordinal it holds (token 4*lg + l%4; heads 4*(ln/4)..+3), and compute() turns the quad's 4x4 block
  // (token x head) around with cross-lane moves so that every lane ends up with its own head for the quad's
  // four tokens.  Scattered 4-byte gathers -- four per lane and page -- kept the CU's address and data-return
  // units busy most of the time; quads that hold no query head do not load at all.
  const uint32_t quad4 = (ln >> 2) * 4u;
  const bool quad_live = quad4 < (uint32_t)G;
  const uint32_t quad_off = (quad4 < (uint32_t)Gp ? quad4 : 0u) * 4u;
  const int top_k = KS == 1 ? 1 : P.top_k;
  auto gather = [&](int (&id)[KS], float4 (&sr)[KS]) {
    // stored ordinals are clamped (unsigned min: negatives become the last ordinal), never trusted; with several
    // slots the raw values stay as they are (a negative one marks an unused slot) and only the address is clamped
#pragma unroll
    for (int i = 0; i < KS; ++i) {
      const uint32_t idc = min((uint32_t)id[i], id_hi);
      if (KS == 1) id[i] = (int)idc;
      sr[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if constexpr (DENSE) {          // the lane's own (token, head): one float
        sr[i].x = *reinterpret_cast<const float*>(sref_bh + ((idc << gsh2) + gq4));
      } else {
        if (quad_live) sr[i] = *reinterpret_cast<const float4*>(sref_bh + ((idc << gsh2) + quad_off));
      }
    }
  };
  auto quad_xchg = [](float v, int ctrl_is_pair) {   // value of the lane at position ^1 (pair) or ^2 of the quad
    const int i = __builtin_bit_cast(int, v);
    const int r = ctrl_is_pair ? __builtin_amdgcn_update_dpp(0, i, 0xB1, 0xf, 0xf, true)    // quad_perm [1,0,3,2]
                               : __builtin_amdgcn_update_dpp(0, i, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
    return __builtin_bit_cast(float, r);
  };
  const bool pos_odd = (ln & 1u) != 0u, pos_hi = (ln & 2u) != 0u;
  auto quad_transpose = [&](float4 v, float (&out)[4]) {   // lane q of a quad holds row q -> holds column q
    const float r0 = quad_xchg(pos_odd ? v.x : v.y, 1);
    const float r1 = quad_xchg(pos_odd ? v.z : v.w, 1);
    if (pos_odd) { v.x = r0; v.z = r1; } else { v.y = r0; v.w = r1; }
    const float r2 = quad_xchg(pos_hi ? v.x : v.z, 0);
    const float r3 = quad_xchg(pos_hi ? v.y : v.w, 0);
    if (pos_hi) { v.x = r2; v.y = r3; } else { v.z = r2; v.w = r3; }
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  };
  // Table updates of the previous page whose returned old values have not been looked at yet: an entry that
  // wrapped is recorded in the overflow list (rare).  The check runs one page late, in the shadow of the next
  // page's score MFMAs, so the atomics' return latency is never waited for.
  constexpr int NU = DENSE ? KS : 4 * KS;  // table updates per lane and page: four tokens x ordinal slots (DENSE: one token)
  uint32_t pend_old[NU], pend_fix[NU];
  uint32_t pend_ids[(NU + 1) / 2];      // table rows of the page's updates (16 bits each: a table fits the LDS)
#pragma unroll
  for (int n = 0; n < NU; ++n) { pend_old[n] = 0u; pend_fix[n] = 0u; }
#pragma unroll
  for (int n = 0; n < (NU + 1) / 2; ++n) pend_ids[n] = 0u;
  auto list_push = [&](uint32_t ent, float amount) {
    const uint32_t slot = atomicAdd(&ovf[0], 1u);
    if (slot < (uint32_t)kOvfCap) {
      ovf_ent[slot] = ent;
      ovf_val[slot] = amount;
    }
  };
  auto check_pending = [&]() {
    bool any = false;
#pragma unroll
    for (int n = 0; n < NU; ++n) any |= pend_old[n] + pend_fix[n] < pend_fix[n];
    if (any) {      // one branch per page; lanes without a query head keep all-zero state
#pragma unroll
      for (int e = 0; e < NU; ++e) {
        const uint32_t j = (e & 1) ? pend_ids[e >> 1] >> 16 : pend_ids[e >> 1] & 0xffffu;
        // 2^32 table units: marked (top bit) for conversion to a plain weight when the block flushes.  No
        // memory load may sit on this path: a conditional load in the loop would cost every wait its exact count.
        if (pend_old[e] + pend_fix[e] < pend_fix[e]) list_push((((j << gsh2) + ln4) >> 2) | 0x80000000u, 4294967296.f);
      }
    }
  };
  // DENSE: row shifts with a bank mask (a bank = four lanes of a row): only the lanes of one quad take the shifted value
  auto shr_into = [](float keep, float src, auto N) {       // lanes of quad N take src of the lane 4 N places down
    constexpr int n = decltype(N)::value;
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, keep), __builtin_bit_cast(int, src),
                                                                 0x110 + 4 * n, 0xf, 1 << n, false));
  };
  // every lane takes src of the lane 4 N places up in its row (0 past the row's end).  Only quad 0 needs the result:
  // the other lanes hold rows 4..15 of the weights operand, whose products land in accumulator rows of query heads
  // that do not exist and are never read.
  auto shl_quads = [](float src, auto N) {
    constexpr int n = decltype(N)::value;
    const int v = __builtin_bit_cast(int, src);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(v, v, 0x100 + 4 * n, 0xf, 0xf, true));
  };
  // FULL: all 16 tokens of the page take part (no masking code at all); otherwise bit t of `mask` says whether
  // token t does (a valid token of the sequence and, in subset attention, a selected one).
  auto compute = [&](auto full_tag, TileT& t, const int (&idv)[KS], const float4 (&srvv)[KS], const uint32_t mask) {
    constexpr bool FULL = decltype(full_tag)::value;
    const int id = idv[0];
    float sr[4];                       // per-reference score part of the quad's four tokens, this lane's head
    // several ordinal slots: score of every slot (the table units of an entry hang on ITS reference's score), table
    // row and validity of every (token, slot), 1 / (references the token uses); sr = mean over the used slots
    float sri[KS][4];
    uint32_t rown[4][KS];
    bool usedn[4][KS];
    float inv_m[4] = {1.f, 1.f, 1.f, 1.f};
    if constexpr (DENSE && KS == 1) {
      sr[0] = srvv[0].x;                 // of the lane's own (token, head)
    } else if constexpr (DENSE) {        // several slots: mean of the scores of the slots the lane's token uses
      float cnt = 0.f;
      sr[0] = 0.f;
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        sri[i][0] = srvv[i].x;
        usedn[0][i] = i < top_k && idv[i] >= 0;
        rown[0][i] = min((uint32_t)idv[i], id_hi);
        cnt += usedn[0][i] ? 1.f : 0.f;
        sr[0] += usedn[0][i] ? sri[i][0] : 0.f;
      }
      inv_m[0] = __builtin_amdgcn_rcpf(fmaxf(cnt, 1.f));
      sr[0] *= inv_m[0];
    } else if constexpr (KS == 1) {
      quad_transpose(srvv[0], sr);
    } else {
#pragma unroll
      for (int i = 0; i < KS; ++i) quad_transpose(srvv[i], sri[i]);
      float cnt[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int e = 0; e < 4; ++e) sr[e] = 0.f;
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        const int raw[4] = {quad_bcast<0>(idv[i]), quad_bcast<1>(idv[i]), quad_bcast<2>(idv[i]), quad_bcast<3>(idv[i])};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          usedn[e][i] = i < top_k && raw[e] >= 0;
          rown[e][i] = min((uint32_t)raw[e], id_hi);
          cnt[e] += usedn[e][i] ? 1.f : 0.f;
          sr[e] += usedn[e][i] ? sri[i][e] : 0.f;
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        inv_m[e] = __builtin_amdgcn_rcpf(fmaxf(cnt[e], 1.f));
        sr[e] *= inv_m[e];
      }
    }
    uint4 zk[TileT::NKK];                      // the scores operand as bf16
    float sc[4] = {1.f, 1.f, 1.f, 1.f}, zf[4] = {0.f, 0.f, 0.f, 0.f};   // 4-bit: scale, zero - 16 * scale per token
    if constexpr (Q4) {
#pragma unroll
      for (int kk = 0; kk < TileT::NKK; ++kk) {
        const uint32_t wd = t.zc[kk];            // bf16 (16 + code) = 0x4180 | code << 3
        zk[kk].x = ((wd << 3) & 0x00780078u) | c16;
        zk[kk].y = ((wd >> 1) & 0x00780078u) | c16;
        zk[kk].z = ((wd >> 5) & 0x00780078u) | c16;
        zk[kk].w = ((wd >> 9) & 0x00780078u) | c16;
      }
      if constexpr (DENSE) {                     // scale and zero point of the lane's own token 4 lg + te, in slot 0
        sc[0] = bf16lo(t.sz.x);              // (loaded for this token alone: bf16 bits in the low half)
        zf[0] = bf16lo(t.sz.z) - 16.f * sc[0];
        if (!FULL) {
          const bool on = (mask >> (4 * lg + te)) & 1u;
          sc[0] = on ? sc[0] : 0.f;
          zf[0] = on ? zf[0] : 0.f;
        }
      } else {
      sc[0] = bf16lo(t.sz.x); sc[1] = bf16hi(t.sz.x); sc[2] = bf16lo(t.sz.y); sc[3] = bf16hi(t.sz.y);
      zf[0] = bf16lo(t.sz.z) - 16.f * sc[0]; zf[1] = bf16hi(t.sz.z) - 16.f * sc[1];
      zf[2] = bf16lo(t.sz.w) - 16.f * sc[2]; zf[3] = bf16hi(t.sz.w) - 16.f * sc[3];
      if (!FULL) {                               // records of tokens that do not take part may hold anything
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool on = (mask >> (4 * lg + e)) & 1u;
          sc[e] = on ? sc[e] : 0.f;
          zf[e] = on ? zf[e] : 0.f;
        }
      }
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < TileT::NKK; ++kk) zk[kk] = t.zk[kk];
    }
    const float d0 = Q4 ? 0.f : cstart;
    float4v d = {d0, d0, d0, d0};
#pragma unroll
    for (int kk = 0; kk < TileT::NKK; ++kk) {
      d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, zk[kk]), qbl[kk], d, 0, 0, 0);
      d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, zk[kk]), qb[kk], d, 0, 0, 0);
    }
    check_pending();
    float p[4];
    if constexpr (DENSE) {
      // the lane's own score: token 4 lg + te of head hd, from lane (lg, hd)
      float dd = d[0];
      dd = shr_into(dd, d[1], std::integral_constant<int, 1>{});
      dd = shr_into(dd, d[2], std::integral_constant<int, 2>{});
      dd = shr_into(dd, d[3], std::integral_constant<int, 3>{});
      float x = Q4 ? cstart + (sr[0] + (sc[0] * dd + zf[0] * qsum)) : dd + sr[0];
      if (!FULL) x = ((mask >> (4 * lg + te)) & 1u) ? x : -INFINITY;
      p[0] = __builtin_amdgcn_exp2f(x);
      lsum += p[0];
    } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float x = Q4 ? cstart + (sr[e] + (sc[e] * d[e] + zf[e] * qsum)) : d[e] + sr[e];
      if (!FULL) x = ((mask >> (4 * lg + e)) & 1u) ? x : -INFINITY;   // select, not arithmetic: garbage may be NaN
      p[e] = __builtin_amdgcn_exp2f(x);
      lsum += p[e];
    }
    }
    if constexpr (KS > 1 && DENSE) {
      if (ghead) {     // one table update per used slot of the lane's token: weight p / m in the units of the slot's reference
        constexpr float kLim = 4294967040.f;     // largest float below 2^32
        float f[NU];
        uint32_t off[NU];
        float fmax_all = 0.f;
#pragma unroll
        for (int i = 0; i < KS; ++i) {
          f[i] = usedn[0][i] ? __builtin_ldexpf(p[0] * inv_m[0], table_shift(sri[i][0], cshift)) : 0.f;
          off[i] = (rown[0][i] << gsh2) + ln4;
          fmax_all = fmaxf(fmax_all, f[i]);
        }
        if (!(fmax_all < kLim)) {                  // an addend does not fit (rare): the whole weight goes to the list
#pragma unroll
          for (int n = 0; n < NU; ++n)
            if (!(f[n] < kLim)) list_push(off[n] >> 2, p[0] * inv_m[0]);
        }
#pragma unroll
        for (int n = 0; n < NU; ++n) {
          pend_fix[n] = f[n] < kLim ? (uint32_t)(f[n] + 0.5f) : 0u;
          pend_old[n] = atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(utab) + off[n]), pend_fix[n]);
        }
#pragma unroll
        for (int n = 0; n < NU / 2; ++n) pend_ids[n] = (off[2 * n] >> gsh2) | ((off[2 * n + 1] >> gsh2) << 16);
      }
    } else if constexpr (KS > 1) {
      if (ghead) {     // one table update per (token, used slot): weight p / m in the units of the slot's reference
        constexpr float kLim = 4294967040.f;     // largest float below 2^32
        float f[NU];
        uint32_t off[NU];
        float fmax_all = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int i = 0; i < KS; ++i) {
            const int n = e * KS + i;
            f[n] = usedn[e][i] ? __builtin_ldexpf(p[e] * inv_m[e], table_shift(sri[i][e], cshift)) : 0.f;
            off[n] = (rown[e][i] << gsh2) + ln4;
            fmax_all = fmaxf(fmax_all, f[n]);
          }
        if (!(fmax_all < kLim)) {                  // an addend does not fit (rare): the whole weight goes to the list
#pragma unroll
          for (int n = 0; n < NU; ++n)
            if (!(f[n] < kLim)) list_push(off[n] >> 2, p[n / KS] * inv_m[n / KS]);
        }
#pragma unroll
        for (int n = 0; n < NU; ++n) {
          pend_fix[n] = f[n] < kLim ? (uint32_t)(f[n] + 0.5f) : 0u;
          pend_old[n] = atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(utab) + off[n]), pend_fix[n]);
        }
#pragma unroll
        for (int n = 0; n < NU / 2; ++n) pend_ids[n] = (off[2 * n] >> gsh2) | ((off[2 * n + 1] >> gsh2) << 16);
      }
    } else if constexpr (DENSE) {
      // (merging the pages of a draw into one basic block -- update unconditional, returned values checked once per draw
      // -- was measured: no faster for bf16 latents, 12 % slower for 4-bit ones)
      if (ghead) {     // one fixed-point table update per lane
        constexpr float kLim = 4294967040.f;     // largest float below 2^32
        float f = __builtin_ldexpf(p[0], table_shift(sr[0], cshift));
        uint32_t off = ((uint32_t)id << gsh2) + ln4;
        if constexpr (SPILL) {     // ordinals older than the window: plain weights into the pair's table in global memory
          if (id < win_lo) {
            if (p[0] != 0.f) unsafeAtomicAdd(reinterpret_cast<float*>(reinterpret_cast<char*>(spill_bh) + off), p[0]);
            f = 0.f;
            off = ln4;             // a zero addend to the window's first row
          } else {
            off -= (uint32_t)win_lo << gsh2;
          }
        }
        if (!(f < kLim)) list_push(off >> 2, p[0]);     // the addend does not fit (rare): the whole weight goes to the list
        pend_fix[0] = f < kLim ? (uint32_t)(f + 0.5f) : 0u;
        pend_old[0] = atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(utab) + off), pend_fix[0]);
        pend_ids[0] = off >> gsh2;               // (window-relative row)
      }
    } else {
    // (cross-lane moves read 0 from lanes that are switched off, so they stay outside the per-head branch)
    const int ids[4] = {quad_bcast<0>(id), quad_bcast<1>(id), quad_bcast<2>(id), quad_bcast<3>(id)};
    if (ghead) {       // fixed-point table update (weights of masked tokens are 0; their clamped ordinal is valid)
      constexpr float kLim = 4294967040.f;     // largest float below 2^32
      float f[4];
      uint32_t off[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f[e] = __builtin_ldexpf(p[e], table_shift(sr[e], cshift));
        off[e] = ((uint32_t)ids[e] << gsh2) + ln4;
      }
      if constexpr (SPILL) {     // ordinals older than the window: plain weights into the pair's table in global memory
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (ids[e] < win_lo) {
            if (p[e] != 0.f) unsafeAtomicAdd(reinterpret_cast<float*>(reinterpret_cast<char*>(spill_bh) + off[e]), p[e]);
            f[e] = 0.f;
            off[e] = ln4;          // a zero addend to the window's first row
          } else {
            off[e] -= (uint32_t)win_lo << gsh2;
          }
        }
      }
      if (!(fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])) < kLim)) {   // an addend does not fit (rare): the whole
#pragma unroll                                                      // weight goes to the list
        for (int e = 0; e < 4; ++e)
          if (!(f[e] < kLim)) list_push(off[e] >> 2, p[e]);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pend_fix[e] = f[e] < kLim ? (uint32_t)(f[e] + 0.5f) : 0u;      // to nearest: no one-sided loss per token
        pend_old[e] = atomicAdd(reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(utab) + off[e]), pend_fix[e]);
      }
      if constexpr (SPILL) {     // window-relative rows, recovered from the offsets
        pend_ids[0] = (off[0] >> gsh2) | ((off[1] >> gsh2) << 16);
        pend_ids[1] = (off[2] >> gsh2) | ((off[3] >> gsh2) << 16);
      } else {
        pend_ids[0] = (uint32_t)ids[0] | ((uint32_t)ids[1] << 16);
        pend_ids[1] = (uint32_t)ids[2] | ((uint32_t)ids[3] << 16);
      }
    }
    }
    // 4-bit: the value product takes p * scale (rounded to bf16 for the matrix unit) against 16 + code; the scalar
    // that takes the offset back out must use the SAME rounded weights, or the two large terms would not cancel
    // exactly and the bf16 rounding of the weights would show the latent's whole range in every output.  The offset
    // taken out is 23.5, the centre of 16 + code, so that what the rounding of a weight multiplies is the centred
    // code (-7.5 .. 7.5), as it multiplies a centred latent in the bf16 layouts; the 7.5 scale goes with the zero point.
    float pzero = 0.f;                           // sum_e p[e] * (zero[e] + 7.5 scale[e])
    if constexpr (DENSE) {
      // the same per lane for its own token; then the weights go back to the operand layout of the value product:
      // lane (lg, g) of quad 0 collects tokens 4 lg + 0..3 of head g from lanes (lg, 4 e + g); the other lanes do not matter
      if constexpr (Q4 && JOINT) {
        pzero = p[0] * (zf[0] + 23.5f * sc[0]);
        p[0] *= sc[0];
      }
      if constexpr (Q4 && !JOINT) {
        const float sv = bf16lo(t.szv.x), zv0 = bf16lo(t.szv.z);
        const bool on = FULL || ((mask >> (4 * lg + te)) & 1u);
        pzero = p[0] * (on ? zv0 + 7.5f * sv : 0.f);
        p[0] *= on ? sv : 0.f;
      }
      if constexpr (Q4) zacc += pzero - 23.5f * bf16lo(pack_bf16(p[0], 0.f));     // (the weight as the matrix unit sees it)
      const float pd = p[0];
      p[1] = shl_quads(pd, std::integral_constant<int, 1>{});
      p[2] = shl_quads(pd, std::integral_constant<int, 2>{});
      p[3] = shl_quads(pd, std::integral_constant<int, 3>{});
    }
    if constexpr (Q4 && JOINT && !DENSE) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pzero += p[e] * (zf[e] + 23.5f * sc[e]); // zf = zero - 16 scale
        p[e] *= sc[e];
      }
    }
    if constexpr (Q4 && !JOINT) {  // the same with the value stream's own scales and zero points
      if constexpr (!DENSE) {
      float sv[4] = {bf16lo(t.szv.x), bf16hi(t.szv.x), bf16lo(t.szv.y), bf16hi(t.szv.y)};
      float zv0[4] = {bf16lo(t.szv.z), bf16hi(t.szv.z), bf16lo(t.szv.w), bf16hi(t.szv.w)};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool on = FULL || ((mask >> (4 * lg + e)) & 1u);
        pzero += p[e] * (on ? zv0[e] + 7.5f * sv[e] : 0.f);
        p[e] *= on ? sv[e] : 0.f;
      }
      }
#pragma unroll
      for (int nb = 0; nb < TileT::NB; ++nb) {
        const uint2 wv = t.zvc[nb >> 2];
        const int j = nb & 3;                       // bf16 (16 + code) = 0x4180 | code << 3
        t.zv[nb].x = ((j == 0 ? wv.x << 3 : wv.x >> (4 * j - 3)) & 0x00780078u) | c16;
        t.zv[nb].y = ((j == 0 ? wv.y << 3 : wv.y >> (4 * j - 3)) & 0x00780078u) | c16;
      }
    }
    uint2 pk;
    pk.x = pack_bf16(p[0], p[1]);
    pk.y = pack_bf16(p[2], p[3]);
    if constexpr (Q4 && !DENSE) zacc += pzero - 23.5f * ((bf16lo(pk.x) + bf16hi(pk.x)) + (bf16lo(pk.y) + bf16hi(pk.y)));
    const short4v pa = __builtin_bit_cast(short4v, pk);
    if (JOINT) {
#pragma unroll
      for (int kk = 0; kk < TileT::NKK; ++kk)
        if (4 * kk + lg < R / 8) *reinterpret_cast<uint4*>(tr + ln * TRP + (4 * kk + lg) * 8) = zk[kk];
      __builtin_amdgcn_wave_barrier();
      // LDS transpose load (ds_read_b64_tr_b16; behaviour checked on the hardware): within each 16-lane group
      // lane j supplies the address of a 4-element chunk and lane i receives element i%4 of the chunks
      // supplied by lanes i/4, i/4+4, i/4+8, i/4+12.  Lane j of group lg points at token 4*lg + j/4, columns
      // 16*nb + 4*(j%4)..+3, so lane i ends up with tokens 4*lg..4*lg+3 of column 16*nb + i: the value operand.
#pragma unroll
      for (int nb = 0; nb < TileT::NB; ++nb) {
        typedef short s4 __attribute__((ext_vector_type(4)));
        const uint16_t* src = tr + (4 * lg + (ln >> 2)) * TRP + nb * 16 + (ln & 3) * 4;
        const s4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)src);
        t.zv[nb] = __builtin_bit_cast(uint2, v);
      }
      __builtin_amdgcn_wave_barrier();
    }
    if (!FULL) {             // zero the value-operand slots of tokens that do not take part (they may hold garbage)
      const uint32_t m4 = mask >> (4 * lg);       // this lane's four tokens
      const uint32_t keep_x = ((m4 & 1u) ? 0x0000ffffu : 0u) | ((m4 & 2u) ? 0xffff0000u : 0u);
      const uint32_t keep_y = ((m4 & 4u) ? 0x0000ffffu : 0u) | ((m4 & 8u) ? 0xffff0000u : 0u);
#pragma unroll
      for (int nb = 0; nb < TileT::NB; ++nb) {
        t.zv[nb].x &= keep_x;
        t.zv[nb].y &= keep_y;
      }
    }
#pragma unroll
    for (int nb = 0; nb < TileT::NB; ++nb) {
      acc[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(short4v, t.zv[nb]), acc[nb], 0, 0, 0);
    }
  };

  // Software pipeline over the pages a wave draws.  While page i is computed, the ordinals of
  // page i+LI, the latents of page i+LZ and the per-reference score gather of page i+LG are in flight.  The
  // vector-memory counter retires in order, so a wait for some load is a wait for everything issued before it:
  //   * compute(i) waits for gather(i), issued LG iterations earlier -> LG pages of loads may stay outstanding;
  //   * gather(i+LG) needs the ordinals of page i+LG as addresses; they were issued LI-LG iterations earlier,
  //     so LI-LG >= LG keeps that wait from draining the pipe.
  // Every load in the loop is unconditional (positions past the block's range re-read its last page and are
  // computed with zero valid tokens), so the compiler can set the wait counts exactly.
  // The waves of a block draw their pages from a shared counter, ST consecutive pages at a time, instead of owning a
  // fixed share: with fixed shares the wave that is older on its SIMD ran a third faster than the younger one and
  // the block waited for the slow half with half-empty SIMDs.  A draw made in one loop iteration is turned into
  // pool pages in the next and computed two iterations after that, so the counter's latency is never waited for.
  {
    constexpr int LG = PIPE_LG, LZ = PIPE_LG + 1, LI = 2 * PIPE_LG + 1, ST = LI + 1;
    const int32_t* bt = P.block_tables + (int64_t)b * P.bt_stride;
    const int n_blk = p1 - p0;                               // pages of this block
    // Blocks start at different points of their (cyclic) page range: ranges of different sequences and splits
    // begin at large power-of-two distances, and blocks that advance in lockstep from such addresses would
    // keep hitting the same HBM channels.  The order is free because every partial sum simply adds.  The block
    // that holds the sequence's partial last page does not rotate, so that page comes last and every earlier
    // draw is made of full pages only: the steady-state loop carries no masking code.
    // (Subset attention runs the masked loop body throughout.)
    const bool has_partial = !SUBSET && (L & (kPage - 1)) != 0 && p1 == n_pages;
    const int rot = has_partial ? 0 : (int)(((uint32_t)pair * 2654435761u + (uint32_t)s * 40503u) >> 8) % n_blk;
    const int n_full = SUBSET ? 0 : n_blk - (has_partial ? 1 : 0);
    // Draw c (positions c*ST .. c*ST+ST-1) covers pages c%NW, c%NW + NW, ... of the (c/NW)-th group of NW*ST pages,
    // so the NW draws that the waves of a block hold at about the same time interleave page by page and the
    // block sweeps one contiguous region; positions of the last, incomplete group that map past the range are
    // empty.
    constexpr int GRP = NW * ST;
    const int n_pos = ceil_div(n_blk, GRP) * GRP;
    auto pos_page = [&](int x) {
      const int c = x / ST, u = x - c * ST;
      return (c / NW) * GRP + (c % NW) + NW * u;
    };
    auto local_page = [&](int x) {                            // page of position x in rotated order
      const int pgi = pos_page(x);
      int xx = (pgi < n_blk ? pgi : n_blk - 1) + rot;
      return xx >= n_blk ? xx - n_blk : xx;
    };
    // list entry -> logical page and the mask of its tokens that take part
    const int32_t* selp = SUBSET ? P.sel_pages + (int64_t)b * P.sel_stride : nullptr;
    const int32_t* selm = SUBSET ? P.sel_masks + (int64_t)b * P.sel_stride : nullptr;
    const int last_logical = ceil_div(L, kPage) - 1;
    auto logical_of = [&](int entry) { return SUBSET ? clampi(selp[entry], 0, last_logical) : entry; };
    auto mask_vec = [&](int base) {                           // lane u: mask of position base + u
      const int x = base + (int)l;
      const int entry = p0 + local_page(x);
      const int left = L - logical_of(entry) * kPage;         // valid tokens of the page (>= 1)
      uint32_t m = left >= kPage ? 0xffffu : (1u << left) - 1u;
      if (SUBSET) {
        m &= (uint32_t)selm[entry];
        if ((uint32_t)selp[entry] > (uint32_t)last_logical) m = 0u;   // a listed page outside the sequence
      }
      return (int)(pos_page(x) < n_blk ? m : 0u);
    };
    // Pool pages of a draw come from the block table with ONE vector load (lane u holds the page of position
    // base + u) and are handed to the stages with v_readlane at a constant lane.  A scalar load per stage would sit
    // in the same out-of-order counter as the LDS atomics and force a full wait-for-everything each time.
    auto page_vec = [&](int base) {
      return clampi(bt[logical_of(p0 + local_page(base + (int)l))], 0, (int)P.n_pages_pool - 1);
    };
    auto draw = [&]() {                                       // next ST positions of the block (wave-uniform)
      uint32_t v = 0;
      if (l == 0) v = atomicAdd(pgctr, (uint32_t)ST);
      return (int)__builtin_amdgcn_readfirstlane(v);
    };
    TileT t[ST];
    int id[ST][KS];
    float4 sr[ST][KS];
    int pg[ST];          // pg[k % ST] = pool page of the wave's k-th page, kept LI+1 pages ahead
    int cb = draw(), cb1 = draw(), cb2 = draw();              // positions of this, the next and the next-but-one draw
    {
      const int pv0 = page_vec(cb);
#pragma unroll
      for (int u = 0; u < ST; ++u) pg[u] = __builtin_amdgcn_readlane(pv0, u);
    }
    int pgit_next = page_vec(cb1);
    int mk_next = mask_vec(cb);                               // masks of the draw about to be computed
#pragma unroll
    for (int u = 0; u < LI; ++u) load_ordinals<KS, DENSE>(idx_h, idx_page_bytes, pg[u], l, top_k, id[u]);
#pragma unroll
    for (int u = 0; u < LZ; ++u) load_latents<R, JOINT, NT, DENSE>(lat_h, lat_page_bytes, lat_stream_bytes, pg[u], l, t[u]);
#pragma unroll
    for (int u = 0; u < LG; ++u) gather(id[u], sr[u]);
    auto body = [&](auto full_tag) {
      const int pgit = pgit_next;                             // pages of the next draw
      pgit_next = page_vec(cb2);
      const int mk = mk_next;                                 // masks of this draw
      mk_next = mask_vec(cb1);
      const int cb3 = draw();
#pragma unroll
      for (int u = 0; u < ST; ++u) {
        load_ordinals<KS, DENSE>(idx_h, idx_page_bytes, pg[(u + LI) % ST], l, top_k, id[(u + LI) % ST]);
        load_latents<R, JOINT, NT, DENSE>(lat_h, lat_page_bytes, lat_stream_bytes, pg[(u + LZ) % ST], l, t[(u + LZ) % ST]);
        pg[u] = __builtin_amdgcn_readlane(pgit, u);
        gather(id[(u + LG) % ST], sr[(u + LG) % ST]);
        compute(full_tag, t[u], id[u], sr[u],
                decltype(full_tag)::value ? 0xffffu : (uint32_t)__builtin_amdgcn_readlane(mk, u));
      }
      cb = cb1; cb1 = cb2; cb2 = cb3;
    };
    while (cb - cb % GRP + GRP <= n_full) body(std::true_type{});    // the draw's whole group is made of full pages
    while (cb < n_pos) body(std::false_type{});
    check_pending();
  }

  // ---- block reduction of the per-wave partials -------------------------------------------------
  if (DENSE) {                     // the four tokens of a lane group's head sit in four quads
    lsum += __shfl_xor(lsum, 4);
    lsum += __shfl_xor(lsum, 8);
  }
  lsum += __shfl_xor(lsum, 16);
  lsum += __shfl_xor(lsum, 32);
  if (l < (DENSE ? 4u : 16u)) atomicAdd(&lbuf[l], lsum);
  if (Q4) {
    if (DENSE) {
      zacc += __shfl_xor(zacc, 4);
      zacc += __shfl_xor(zacc, 8);
    }
    zacc += __shfl_xor(zacc, 16);
    zacc += __shfl_xor(zacc, 32);
    if (l < (DENSE ? 4u : 16u)) atomicAdd(&zbuf[l], zacc);
  }
#pragma unroll
  for (int nb = 0; nb < TileT::NB; ++nb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = 4 * lg + i;
      if (g < G) atomicAdd(&accbuf[g * R + nb * 16 + ln], acc[nb][i]);
    }
  __syncthreads();
  const int64_t part = bh * P.S + s;
  if (tid < Gp) P.lpart[part * Gp + tid] = lbuf[tid];
  if (tid == 0) P.wflag[part] = ovf[0] != 0u;
  for (int i = tid; i < Gp * R; i += NW * 64) P.accpart[part * Gp * R + i] = accbuf[i] + (Q4 ? zbuf[i / R] : 0.f);
  // the table leaves the block as floats, normally still in the per-entry units of table_shift()
  float* wp = P.wpart + part * P.tab_cap * Gp;              // window entry i <-> table element win_lo * Gp + i
  const uint32_t n_ovf = ovf[0];
  if (n_ovf == 0) {
    for (int i = tid * 4; i < n_tab; i += NW * 64 * 4) {
      const uint4 u = *reinterpret_cast<const uint4*>(utab + i);
      typedef float float4n __attribute__((ext_vector_type(4)));
      const float4n o = {(float)u.x, (float)u.y, (float)u.z, (float)u.w};
      if (NT) __builtin_nontemporal_store(o, reinterpret_cast<float4n*>(wp + i));   // large calls: keep the flush out of L2 too
      else *reinterpret_cast<float4n*>(wp + i) = o;
    }
  } else {
    // rare: turn the table into plain weights (entry i = (j, g) has the units of score-table element i)
    const float* sref_tab = P.sref + (bh * P.n_ref_max + win_lo) * Gp;
    for (int i = tid; i < n_tab; i += NW * 64)
      tab[i] = __builtin_ldexpf((float)utab[i], -table_shift(sref_tab[i], xbuf[i & (Gp - 1)]));
    __syncthreads();
    const uint32_t n_rec = n_ovf < (uint32_t)kOvfCap ? n_ovf : (uint32_t)kOvfCap;
    for (uint32_t i = tid; i < n_rec; i += NW * 64) {
      const uint32_t ent = ovf_ent[i] & 0x7fffffffu;
      float amount = ovf_val[i];
      if (ovf_ent[i] >> 31) amount = __builtin_ldexpf(amount, -table_shift(sref_tab[ent], xbuf[ent & (Gp - 1)]));
      atomicAdd(&tab[ent], amount);
    }
    if (n_ovf > (uint32_t)kOvfCap) {       // list exhausted, weights were lost: the pair's rows go to the rescue kernel
      if (tid == 0) atomicOr(P.status, 2);
      if (tid < G) P.rescue[(int64_t)b * P.Hq + (int64_t)h * G + tid] = 1;
    }
    __syncthreads();
    for (int i = tid * 4; i < n_tab; i += NW * 64 * 4)
      *reinterpret_cast<float4*>(wp + i) = *reinterpret_cast<const float4*>(tab + i);
  }
}

// ------------------------------------------------------------------------------------------------
// host launcher
// ------------------------------------------------------------------------------------------------
template <int R, int NW, bool JOINT, bool SUBSET, bool Q4, bool NT = false, bool SPILL = false, int KS = 1, bool DENSE = false>
static hipError_t launch_stream(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st) {
  if constexpr (!DENSE) {                  // at most four query heads per kv-head: one (token, head) pair per lane
    if (P.Gp == 4 && (KS > 1 || P.top_k <= 1)) return launch_stream<R, NW, JOINT, SUBSET, Q4, NT, SPILL, KS, true>(P, grid, lds, st);
  }
  if constexpr (KS == 1 && !Q4 && !SPILL) {      // several ordinal slots per token: bf16 latents, on-chip table
    if (P.top_k > 1) {
      if (P.spill_on) return hipErrorInvalidValue;
      return P.nt ? launch_stream<R, NW, JOINT, SUBSET, Q4, true, false, 4, DENSE>(P, grid, lds, st)
                  : launch_stream<R, NW, JOINT, SUBSET, Q4, false, false, 4, DENSE>(P, grid, lds, st);
    }
  }
  if constexpr (!SPILL && KS == 1) {        // (a spilling call is a long-sequence call: its bf16 latent loads are non-temporal)
    if (P.spill_on) return launch_stream<R, NW, JOINT, SUBSET, Q4, !Q4, true, 1, DENSE>(P, grid, lds, st);
  }
  if constexpr (!Q4 && !NT && KS == 1) {
    if (P.nt) return launch_stream<R, NW, JOINT, SUBSET, Q4, true, false, 1, DENSE>(P, grid, lds, st);
  }
  // Gather lead of the software pipeline (pages of loads kept in flight per wave), bounded by the 6-bit
  // load counter (loads per page) and by the register file (registers per page in flight).
  constexpr int NKK = (R + 31) / 32, NB = R / 16;
  constexpr int NQ = (NB + 3) / 4;
  constexpr int lat_loads = Q4 ? NKK + (DENSE ? 2 : 1) + (JOINT ? 0 : NQ + (DENSE ? 2 : 1))
                               : NKK + (JOINT ? 0 : NB);                                        // latent loads per page
  constexpr int tile_regs = Q4 ? NKK + 4 + (JOINT ? 0 : 2 * NQ + 4) : 4 * NKK + (JOINT ? 0 : 2 * NB);
  // live registers ~ (LG+2) latent tiles + (2LG+2) ordinals + (LG+1) score quads + ~100 for the rest
  // operands built per page in extra registers (the constants are fitted to what the compiler keeps without spilling)
  // (four ordinal slots: 2 x 16 pending table updates, 16 slot scores, 16 table rows per page being computed)
  // (the dense four-slot variant would have registers for a gather lead of two pages at rank 64; measured: 470 us
  // against 459 with one)
  constexpr int transient = (JOINT || Q4 ? 2 * NB : 0) + (Q4 ? 4 * NKK + (JOINT ? 40 : 16) : 0) + (KS > 1 ? 64 : 0);
  constexpr int by_regs = ((NW >= 16 ? 110 : 216) - transient - 112 - 2 * tile_regs) / (tile_regs + 6 * KS);
  // loads outstanding at once: (2LG+1) ordinals + (LG+1) pages of latents + LG pages of 4 score gathers (+ the page
  // vector); the hardware counter has 6 bits
  constexpr int by_counter = (56 - KS - lat_loads) / (6 * KS + lat_loads);
  constexpr int lg0 = by_counter < by_regs ? by_counter : by_regs;
  constexpr int ST = lg0 < 1 ? 1 : (lg0 > 8 ? 8 : lg0);
  static size_t attr_bytes = 48 * 1024;
  if (lds > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_stream<R, NW, ST, JOINT, SUBSET, Q4, NT, SPILL, KS, DENSE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)device_lds_limit());
    if (e != hipSuccess) return note_hip_error(e, "hipFuncSetAttribute(stream kernel LDS)");
    attr_bytes = device_lds_limit();
  }
  hipLaunchKernelGGL((k_stream<R, NW, ST, JOINT, SUBSET, Q4, NT, SPILL, KS, DENSE>), grid, dim3(NW * 64), lds, st, P);
  return note_hip_error(hipGetLastError(), "launch of the stream kernel");
}

template <int NW, bool JOINT, bool SUBSET, bool Q4 = false>
static hipError_t dispatch_stream(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st) {
  switch (P.R) {
    case 16: return launch_stream<16, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
    case 32: return launch_stream<32, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
    case 48: return launch_stream<48, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
    case 64: return launch_stream<64, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
    case 80: return launch_stream<80, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
    case 96: return launch_stream<96, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
    case 112: return launch_stream<112, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
    case 128: return launch_stream<128, NW, JOINT, SUBSET, Q4>(P, grid, lds, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace dkv
