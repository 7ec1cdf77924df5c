// Decode attention over the DeltaKV cache when keys carry a rotary position embedding, gfx950.
//
// Section 4.1: every operation of the method works on PRE-RoPE key-value states; appendix B.5 names the fused
// de-/re-rotation as future work.  The cache therefore holds un-rotated keys, and a key has to be reconstructed,
// K_hat_t = K_ref[idx_t] + z_K,t W_uK, and then rotated at its token's position before it meets the (already rotated)
// query.  The rotation depends on the token, not on its reference, so the per-reference score table of the plain
// kernels does not exist here: every token's key is rebuilt.  Per 16-token page and wave:
//   * the raw K and V rows of the page's sixteen references go from the reference pool straight into LDS
//     (global_load_lds, chunk-major), one page ahead;
//   * z_K W_uK on the matrix unit (A = the latent tile in its stored operand order, B = W_uK^T from LDS), the raw K
//     rows are added from LDS through transposing reads, which deliver them in the accumulator's layout;
//   * the rotation is lane-local (dimension pairs (d, d + 64) sit in one lane); cos / sin of position * theta come
//     from a per-call table of the page's first position (fp64 sincos, a small prologue kernel) combined with the
//     lane's sixteen in-page values by the angle-addition formulas;
//   * q . K_rot in fp32 on the vector unit, reduced over the sixteen lanes that share a row with DPP moves;
//   * online softmax per wave (the running maximum moves only when a page beats it by 2^6), P (bf16 hi + lo) times
//     the raw V rows and P times z_V on the matrix unit: values carry no rotation, so their latent part still
//     factors and is up-projected once, by the merge kernel.
// Splits of a sequence and the waves of a block are merged by their (maximum, sum) pairs.
#include "decode_common.h"

namespace dkv {

constexpr int kRopeTileElems = 16 * kHeadDim;          // one staged K or V tile: 16 rows of 128 bf16, chunk-major
constexpr float kRopeLazy = 6.0f;                      // log2 units a page may exceed the running maximum by

// hi table: (cos, sin)(16 * P * theta_p) for logical page P and dimension pair p, theta_p = base^(-p / 64).
__global__ __launch_bounds__(256) void k_rope_table(float2* tab, int n_pages, float base) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n_pages * 64) return;
  const int P = i >> 6, p = i & 63;
  const double theta = pow((double)base, -(double)p / 64.0);
  double s, c;
  sincos(16.0 * (double)P * theta, &s, &c);
  tab[i] = make_float2((float)c, (float)s);
}

__device__ inline float row16_sum(float v) {           // sum over the 16 lanes of a row, result in every lane
  int x = __builtin_bit_cast(int, v);
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]
  x = __builtin_bit_cast(int, v);
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]
  x = __builtin_bit_cast(int, v);
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, x, 0x141, 0xf, 0xf, true));   // row_half_mirror
  x = __builtin_bit_cast(int, v);
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, x, 0x140, 0xf, 0xf, true));   // row_mirror
  return v;
}

// Grid (pairs padded to a multiple of 8) x S blocks, 256 or 512 threads.  GP: query heads per kv-head padded to 4 or 8 (the lane keeps its row's share of
// every head's query in registers).
// Eight waves per block share the staged W_uK^T when the rank is at most 64 (150 KB of LDS), four beyond.
template <int R, bool JOINT, int GP>
__global__ __launch_bounds__((R <= 64 ? 8 : 4) * 64) void k_rope_attn(DecodeParams P, const float2* hi_tab, float rope_base) {
  constexpr int kRopeWaves = R <= 64 ? 8 : 4;
  // W_uK^T rows in LDS: for ranks with a power-of-two number of 16-byte chunks the chunks of row d are XOR-swizzled
  // by d (operand fetches of 16 rows then hit distinct banks: 2.4 times the LDS rate of rows padded by 16 bytes,
  // measured); other ranks keep padded rows
  constexpr bool kSwz = (R & (R - 1)) == 0;
  constexpr int kSwzMask = kSwz ? R / 8 - 1 : 0;
  constexpr int NKK = (R + 31) / 32, NB = R / 16, WP = kSwz ? R : R + 8;
  extern __shared__ uint16_t lds[];
  uint16_t* wt = lds;                                               // [128][WP]   W_uK^T
  uint16_t* tiles = wt + kHeadDim * WP;                             // [waves][2 buffers][K tile, V tile]
  float* red = reinterpret_cast<float*>(tiles + kRopeWaves * 4 * kRopeTileElems);   // cross-wave merge area
  // Blocks are handed to the eight XCDs round-robin by linear index, and every XCD has an L2 of its own.  All splits
  // of one (sequence, kv-head) pair go to ONE XCD, pair after pair: the pair's raw reference rows, which every token
  // of the pair gathers, then stay in that L2 instead of being fetched by all eight.
  const int xcd = blockIdx.x & 7, k_in = blockIdx.x >> 3;
  const int pair = xcd + 8 * (k_in / P.S), s = k_in % P.S;
  if (pair >= P.batch * P.Hkv) return;                              // (the pair count is padded to a multiple of 8)
  const int h = pair % P.Hkv, b = pair / P.Hkv;
  const int tid = threadIdx.x, l = tid & 63, ln = l & 15, lg = l >> 4;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int L = seq_len_of(P, b);
  const int n_pages = ceil_div(L, kPage);
  const SplitPlan sp = plan_splits(n_pages, P.S, P.pages_per_split);
  const int G = P.G;
  const int64_t bh = (int64_t)b * P.Hkv + h;
  const int64_t part = bh * P.S + s;
  float* pm = P.lpart + part * GP * 2;                              // [GP][2]: running maximum, sum of weights
  const int p0 = s * sp.per, p1 = min(n_pages, p0 + sp.per);
  if (s >= sp.n_splits || p0 >= p1) {                               // an unused split slot: marked empty for the merge
    if (tid < GP) { pm[2 * tid] = -INFINITY; pm[2 * tid + 1] = 0.f; }
    return;
  }
  // W_uK^T into LDS: element (d, c) <- w_up_k[c][d]
  for (int i = tid; i < kHeadDim * R; i += kRopeWaves * 64) {
    const int c = i / kHeadDim, d = i % kHeadDim;
    wt[d * WP + ((((c >> 3) ^ (d & kSwzMask)) << 3) | (c & 7))] = P.w_up_k[i];
  }
  // the lane's share of the queries: q[g][16 nb + ln] for nb = 0..7, times scale * log2(e)
  float qv[GP][8];
#pragma unroll
  for (int g = 0; g < GP; ++g)
#pragma unroll
    for (int nb = 0; nb < 8; ++nb)
      qv[g][nb] = g < G ? bf16lo(P.q[((int64_t)b * P.Hq + (int64_t)h * G + g) * kHeadDim + 16 * nb + ln]) * P.qk_scale_log2 : 0.f;
  // in-page part of the rotation: (cos, sin)(j * theta_p) for the lane's tokens j = 4 lg + i and pairs p = 16 nb + ln
  float lc[4][4], ls[4][4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) {
    const float theta = powf(rope_base, -(float)(16 * nb + ln) / 64.f);
#pragma unroll
    for (int i = 0; i < 4; ++i) sincosf((float)(4 * lg + i) * theta, &ls[i][nb], &lc[i][nb]);
  }
  __syncthreads();

  const char* lat_h = reinterpret_cast<const char*>(P.latent + (int64_t)h * P.latent_head_stride);
  const uint32_t lat_page_bytes = (uint32_t)P.latent_page_stride * 2u, lat_stream_bytes = (uint32_t)P.latent_stream_stride * 2u;
  const int32_t* idx_h = P.idx + (int64_t)h * P.idx_head_stride;
  const int32_t* bt = P.block_tables + (int64_t)b * P.bt_stride;
  const int32_t* rt = P.ref_tables + (int64_t)b * P.rt_stride;
  const uint16_t* kpool = P.ref + (int64_t)h * P.ref_head_stride;
  const uint16_t* vpool = kpool + P.ref_kv_stride;
  const int n_ref = refs_below(L, P.stride);
  uint16_t* my_tiles = tiles + w * 4 * kRopeTileElems;

  // accumulators: o[nb][i] = sum_t p_t V_ref[idx_t][16 nb + ln] for head 4 lg + i; z likewise over latent columns
  float4v acc_o[8], acc_z[NB];
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) acc_o[nb] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) acc_z[nb] = float4v{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;                   // of head ln (lanes ln >= G idle), this lane's token rows

  // page i of the wave: logical page p0 + w + 4 i
  const int n_mine = (p1 - p0 - w + kRopeWaves - 1) / kRopeWaves;
  auto logical = [&](int i) { return p0 + w + kRopeWaves * min(i, max(n_mine - 1, 0)); };
  auto pool_page = [&](int i) { return clampi(bt[logical(i)], 0, (int)P.n_pages_pool - 1); };
  auto load_ord = [&](int i) {            // ordinal of token ln of the page (clamped, never trusted)
    return (int)min((uint32_t)idx_h[(int64_t)pool_page(i) * P.idx_page_stride + ln], (uint32_t)(n_ref - 1));
  };
  auto issue_rows = [&](int slot, int buf) {               // raw K and V rows of the lane's token -> LDS, chunk-major
    const uint16_t* kr = kpool + (int64_t)slot * kHeadDim;
    const uint16_t* vr = vpool + (int64_t)slot * kHeadDim;
    uint16_t* kt = my_tiles + buf * 2 * kRopeTileElems;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(kr + (lg + 4 * j) * 8),
                                       (void __attribute__((address_space(3)))*)(kt + j * 512), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(vr + (lg + 4 * j) * 8),
                                       (void __attribute__((address_space(3)))*)(kt + kRopeTileElems + j * 512), 16, 0, 0);
    }
  };
  struct Lat { uint4 zk[NKK]; uint2 zv[NB]; };
  auto load_lat = [&](int i, Lat& t) {
    const char* base = lat_h + (uint64_t)(uint32_t)pool_page(i) * lat_page_bytes;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk)
      t.zk[kk] = 4 * kk + lg < R / 8 ? __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(base + (l * 16u + kk * 1024u))))
                                     : make_uint4(0, 0, 0, 0);          // (streamed once: kept out of the L2's way)
    if (!JOINT) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        t.zv[nb] = __builtin_bit_cast(uint2, __builtin_nontemporal_load(reinterpret_cast<const uint2v*>(base + lat_stream_bytes + (l * 8u + nb * 512u))));
    }
  };

  if (n_mine > 0) {
    int ord_next = load_ord(1);
    int slot_cur = clampi(rt[load_ord(0)], 0, (int)P.n_ref_slots - 1);
    Lat lat_cur, lat_next;
    load_lat(0, lat_cur);
    issue_rows(slot_cur, 0);
    for (int i = 0; i < n_mine; ++i) {
      const int buf = i & 1;
      const int lp = logical(i);
      // ---- the page's raw rows, in the accumulator layout: lane (ln, lg) gets tokens 4 lg .. +3 of column 16 nb + ln
      const uint16_t* kt = my_tiles + buf * 2 * kRopeTileElems;
      const uint16_t* vt = kt + kRopeTileElems;
      uint2 kref[8], vref[8];
      {
        const int T = 4 * lg + (ln >> 2);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
          typedef short s4 __attribute__((ext_vector_type(4)));
          const int at = ((2 * nb + ((ln & 3) >> 1)) * 16 + T) * 8 + 4 * (ln & 1);
          kref[nb] = __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(kt + at)));
          vref[nb] = __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(vt + at)));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // ---- next page: its rows go to the other buffer, its latents and the ordinals of the page after it to registers
      const int slot_next = clampi(rt[ord_next], 0, (int)P.n_ref_slots - 1);
      issue_rows(slot_next, buf ^ 1);
      ord_next = load_ord(i + 2);
      load_lat(i + 1, lat_next);
      const float2* hp = hi_tab + (int64_t)lp * 64 + ln;
      float hc[4], hs[4];
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) { const float2 t = hp[16 * nb]; hc[nb] = t.x; hs[nb] = t.y; }

      // ---- K_hat = K_ref + z_K W_uK  (D[token 4 lg + i][d = 16 nb + ln])
      float4v kh[8];
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        kh[nb] = float4v{bf16lo(kref[nb].x), bf16hi(kref[nb].x), bf16lo(kref[nb].y), bf16hi(kref[nb].y)};
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
          const bf16x8 wb = 4 * kk + lg < R / 8
              ? *reinterpret_cast<const bf16x8*>(wt + (16 * nb + ln) * WP + ((4 * kk + lg) ^ ((int)ln & kSwzMask)) * 8)
              : __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
          kh[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lat_cur.zk[kk]), wb, kh[nb], 0, 0, 0);
        }
      }
      // ---- rotate at position 16 lp + 4 lg + i and score against every head
      float x[GP][4];
#pragma unroll
      for (int g = 0; g < GP; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[g][e] = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
          const float c = hc[nb] * lc[e][nb] - hs[nb] * ls[e][nb];
          const float sn = hs[nb] * lc[e][nb] + hc[nb] * ls[e][nb];
          const float x1 = kh[nb][e], x2 = kh[nb + 4][e];
          const float y1 = x1 * c - x2 * sn, y2 = x2 * c + x1 * sn;
#pragma unroll
          for (int g = 0; g < GP; ++g) x[g][e] += qv[g][nb] * y1 + qv[g][nb + 4] * y2;
        }
      // the lane keeps the logits of ITS head (row position ln) for its four tokens
      float xm[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float mine = 0.f;
#pragma unroll
        for (int g = 0; g < GP; ++g) {
          const float tot = row16_sum(x[g][e]);
          mine = ln == g ? tot : mine;
        }
        const bool valid = lp * kPage + 4 * lg + e < L && ln < G;
        xm[e] = valid ? mine : -INFINITY;
      }
      // ---- online softmax: head ln over the page's 16 tokens (rows lg hold four each)
      float pmax = fmaxf(fmaxf(xm[0], xm[1]), fmaxf(xm[2], xm[3]));
      pmax = fmaxf(pmax, __shfl_xor(pmax, 16));
      pmax = fmaxf(pmax, __shfl_xor(pmax, 32));
      const bool move = pmax > m_run + kRopeLazy || (m_run == -INFINITY && pmax > -INFINITY);
      if (__builtin_amdgcn_ballot_w64(move) != 0) {         // rare after the first pages
        const float m_new = move ? pmax : m_run;
        const float alpha = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
        m_run = m_new;
        float ar[4];                                       // factors of the accumulator rows: heads 4 lg + i
#pragma unroll
        for (int e = 0; e < 4; ++e) ar[e] = __shfl(alpha, 4 * lg + e);
#pragma unroll
        for (int nb = 0; nb < 8; ++nb)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc_o[nb][e] *= ar[e];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc_z[nb][e] *= ar[e];
      }
      float p[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        p[e] = __builtin_amdgcn_exp2f(xm[e] - m_run);       // (-inf - finite = -inf -> 0; idle lanes: -inf - -inf = NaN)
        p[e] = xm[e] == -INFINITY ? 0.f : p[e];
        l_run += p[e];
      }
      uint2 ph, pl;
      ph.x = pack_bf16(p[0], p[1]);
      ph.y = pack_bf16(p[2], p[3]);
      pl.x = pack_bf16(p[0] - bf16lo(ph.x), p[1] - bf16hi(ph.x));
      pl.y = pack_bf16(p[2] - bf16lo(ph.y), p[3] - bf16hi(ph.y));
      const short4v pa = __builtin_bit_cast(short4v, ph), pb = __builtin_bit_cast(short4v, pl);
      // ---- P V_ref (hi + lo weights) and P z_V
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        acc_o[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(short4v, vref[nb]), acc_o[nb], 0, 0, 0);
        acc_o[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pb, __builtin_bit_cast(short4v, vref[nb]), acc_o[nb], 0, 0, 0);
      }
      uint2 zv[NB];
      if (JOINT) {      // the single stream is stored in scores-operand order: through LDS into value-operand order
        uint16_t* tr = const_cast<uint16_t*>(kt);          // the K tile of this page has been consumed
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
          if (4 * kk + lg < R / 8) *reinterpret_cast<uint4*>(tr + ((4 * kk + lg) * 16 + ln) * 8) = lat_cur.zk[kk];
        __builtin_amdgcn_wave_barrier();
        const int T = 4 * lg + (ln >> 2);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          typedef short s4 __attribute__((ext_vector_type(4)));
          const int at = ((2 * nb + ((ln & 3) >> 1)) * 16 + T) * 8 + 4 * (ln & 1);
          zv[nb] = __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4 __attribute__((address_space(3)))*)(tr + at)));
        }
        __builtin_amdgcn_wave_barrier();
      } else {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) zv[nb] = lat_cur.zv[nb];
      }
      if (lp * kPage + kPage > L) {          // the sequence's last page: records past its end may hold anything
        const int left = L - lp * kPage - 4 * lg;            // valid tokens among this lane's four
        const uint32_t keep_x = (left > 0 ? 0x0000ffffu : 0u) | (left > 1 ? 0xffff0000u : 0u);
        const uint32_t keep_y = (left > 2 ? 0x0000ffffu : 0u) | (left > 3 ? 0xffff0000u : 0u);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { zv[nb].x &= keep_x; zv[nb].y &= keep_y; }
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        acc_z[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(short4v, zv[nb]), acc_z[nb], 0, 0, 0);
      lat_cur = lat_next;
    }
  }
  // ---- merge the waves of the block (each holds (m, l) per head in lanes ln < G of every row, partial over rows)
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  __builtin_amdgcn_s_waitcnt(0);                            // no direct-to-LDS load of a prefetched page still in flight
  __syncthreads();
  float* wm = red;                                           // [waves][16] maxima, [waves][16] sums
  float* wo = red + 2 * kRopeWaves * 16;                     // [GP][128 + R] merged output rows
  if (lg == 0) { wm[w * 16 + ln] = m_run; wm[kRopeWaves * 16 + w * 16 + ln] = l_run; }
  for (int i = tid; i < GP * (kHeadDim + R); i += kRopeWaves * 64) wo[i] = 0.f;
  __syncthreads();
  float mb[4], fb[4];                                        // block maximum and this wave's factor, heads 4 lg + i
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int g = 4 * lg + e;
    float mm = -INFINITY;
    for (int ww = 0; ww < kRopeWaves; ++ww) mm = fmaxf(mm, wm[ww * 16 + g]);
    mb[e] = mm;
    const float mine = wm[w * 16 + g];
    fb[e] = mine == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mine - mm);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int g = 4 * lg + e;
    if (g < GP) {
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) atomicAdd(&wo[g * (kHeadDim + R) + 16 * nb + ln], acc_o[nb][e] * fb[e]);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) atomicAdd(&wo[g * (kHeadDim + R) + kHeadDim + 16 * nb + ln], acc_z[nb][e] * fb[e]);
    }
  }
  __syncthreads();
  if (tid < GP) {
    float mm = -INFINITY, ll = 0.f;
    for (int ww = 0; ww < kRopeWaves; ++ww) mm = fmaxf(mm, wm[ww * 16 + tid]);
    for (int ww = 0; ww < kRopeWaves; ++ww) {
      const float mw = wm[ww * 16 + tid];
      ll += mw == -INFINITY ? 0.f : wm[kRopeWaves * 16 + ww * 16 + tid] * __builtin_amdgcn_exp2f(mw - mm);
    }
    pm[2 * tid] = mm;
    pm[2 * tid + 1] = ll;
  }
  float* po = P.accpart + part * GP * (kHeadDim + R);
  for (int i = tid; i < GP * (kHeadDim + R); i += kRopeWaves * 64) po[i] = wo[i];
}

// merge: grid (Hq, B), 128 threads (thread = output dim).
__global__ __launch_bounds__(128) void k_rope_merge(DecodeParams P) {
  const int gh = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int G = P.G, Gp = P.Gp, R = P.R;
  const int h = gh / G, g = gh % G;
  const int64_t orow = ((int64_t)b * P.Hq + gh) * kHeadDim;
  const int L = seq_len_of(P, b);
  if (L <= 0) {
    P.out[orow + d] = 0;
    if (P.lse && d == 0) P.lse[(int64_t)b * P.Hq + gh] = -INFINITY;
    return;
  }
  const int64_t bh = (int64_t)b * P.Hkv + h;
  __shared__ float zs[kHeadDim];
  float M = -INFINITY;
  for (int s = 0; s < P.S; ++s) M = fmaxf(M, P.lpart[((bh * P.S + s) * Gp + g) * 2]);
  float lsum = 0.f, o = 0.f, z = 0.f;
  for (int s = 0; s < P.S; ++s) {
    const float* pm = P.lpart + ((bh * P.S + s) * Gp + g) * 2;
    if (pm[0] == -INFINITY) continue;
    const float f = __builtin_amdgcn_exp2f(pm[0] - M);
    const float* po = P.accpart + ((bh * P.S + s) * Gp + g) * (kHeadDim + R);
    lsum += f * pm[1];
    o += f * po[d];
    if (d < R) z += f * po[kHeadDim + d];
  }
  zs[d] = d < R ? z : 0.f;
  __syncthreads();
  for (int c = 0; c < R; ++c) o += zs[c] * bf16lo(P.w_up_v[(int64_t)c * kHeadDim + d]);
  P.out[orow + d] = (uint16_t)f32_to_bf16_bits(o / lsum);
  if (P.lse && d == 0) P.lse[(int64_t)b * P.Hq + gh] = (M + __log2f(lsum)) * kLn2;
}

size_t rope_lds_bytes(int R, int Gp) {
  const int kRopeWaves = R <= 64 ? 8 : 4;
  return (size_t)(kHeadDim * (R + 8) + kRopeWaves * 4 * kRopeTileElems) * 2 + (size_t)(2 * kRopeWaves * 16 + Gp * (kHeadDim + R)) * 4;   // (an upper bound for the swizzled ranks, whose rows carry no padding)
}

template <int R, bool JOINT, int GP>
static hipError_t launch_rope_one(const DecodeParams& P, const float2* tab, float base, dim3 grid, hipStream_t st) {
  const size_t lds = rope_lds_bytes(R, GP);
  static bool attr_set = false;
  if (!attr_set && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_rope_attn<R, JOINT, GP>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return note_hip_error(e, "hipFuncSetAttribute(rope attention LDS)");
    attr_set = true;
  }
  hipLaunchKernelGGL((k_rope_attn<R, JOINT, GP>), grid, dim3((R <= 64 ? 8 : 4) * 64), lds, st, P, tab, base);
  return note_hip_error(hipGetLastError(), "launch of rope attention");
}
template <int R>
static hipError_t launch_rope_r(const DecodeParams& P, const float2* tab, float base, dim3 grid, hipStream_t st) {
  if (P.Gp == 4) return P.joint ? launch_rope_one<R, true, 4>(P, tab, base, grid, st) : launch_rope_one<R, false, 4>(P, tab, base, grid, st);
  if (P.Gp == 8) return P.joint ? launch_rope_one<R, true, 8>(P, tab, base, grid, st) : launch_rope_one<R, false, 8>(P, tab, base, grid, st);
  return hipErrorInvalidValue;
}

hipError_t launch_rope(const DecodeParams& P, float2* tab, int n_pages_max, float base, int batch, hipStream_t st) {
  hipError_t e;
  timing_mark(-1, st);
  hipLaunchKernelGGL(k_rope_table, dim3(ceil_div(n_pages_max * 64, 256)), dim3(256), 0, st, tab, n_pages_max, base);
  if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of rope table");
  timing_mark(K_REF_SCORES, st);
  dim3 grid((batch * P.Hkv + 7) / 8 * 8 * P.S);              // (pair, split) slots, pairs padded to whole XCD rounds
  switch (P.R) {
    case 16: e = launch_rope_r<16>(P, tab, base, grid, st); break;
    case 32: e = launch_rope_r<32>(P, tab, base, grid, st); break;
    case 48: e = launch_rope_r<48>(P, tab, base, grid, st); break;
    case 64: e = launch_rope_r<64>(P, tab, base, grid, st); break;
    case 80: e = launch_rope_r<80>(P, tab, base, grid, st); break;
    case 96: e = launch_rope_r<96>(P, tab, base, grid, st); break;
    case 112: e = launch_rope_r<112>(P, tab, base, grid, st); break;
    case 128: e = launch_rope_r<128>(P, tab, base, grid, st); break;
    default: e = hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  timing_mark(K_STREAM, st);
  hipLaunchKernelGGL(k_rope_merge, dim3(P.Hq, batch), dim3(128), 0, st, P);
  e = note_hip_error(hipGetLastError(), "launch of rope merge");
  timing_mark(K_FINALIZE, st);
  return e;
}

}  // namespace dkv
