// Residual compression of new tokens into the DeltaKV cache, gfx950.
//
// Section 4.1: reference set T = {t : t mod s = 0, t < i}; retrieval of the nearest reference
// (top-1 over the per-head vector K||V, by cosine or -- the section's own metric -- by squared L2 distance;
// lowest ordinal on ties); appendix B.2
// "lifecycle management": residual against the assigned reference -> down-projection -> write to the
// latent pool; appendix B.3: the reference search is a dense matrix product.
//
// Five kernels per call:
//   admit_refs : new tokens at multiples of s are copied raw into the reference pool, with one float per
//                reference: 1/||b|| for the cosine, ||b||^2 / 2 for the L2 metric (argmin ||a-b||^2 =
//                argmax a.b - ||b||^2/2, so both metrics are one product and one per-reference term)
//   sim_top2   : MFMA GEMM [new tokens x 256] . [references x 256]^T per kv-head with a fused epilogue that
//                scales by the reference's inverse norm, applies the causal candidate mask and keeps
//                (best, second best, arg best) per token -- scores never leave the chip
//   resolve    : merges reference-range splits; a token whose two best fp32 scores are closer than the fp32
//                error bound is queued for exact re-scoring, every other token gets its ordinal (with a single
//                split the similarity kernel does this itself and the kernel is not launched)
//   exact      : queued tokens, 16 at a time, against all their candidates on the fp64 matrix unit
//                (v_mfma_f64_16x16x4) with the definition's formula, so the stored ordinal is the exact
//                arg-max with lowest-ordinal tie-break
//   project    : residual in fp32 (exact for bf16 inputs), split into bf16 hi+lo parts, W_down on MFMA,
//                bf16 latents + ordinals written into the token's page
#include <type_traits>

#include "common.h"
#include "launch.h"

namespace dkv {

// the per-reference float of the similarity epilogue from the lane's share of sum b^2 (all 64 lanes call)
__device__ inline float ref_term(float ss_lane, double dd_lane, int metric) {
  if (metric) {                       // ||b||^2 / 2, summed in fp64 (exact for bf16 inputs), one rounding to fp32
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) dd_lane += __shfl_xor(dd_lane, o);
    return (float)(0.5 * dd_lane);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) ss_lane += __shfl_xor(ss_lane, o);
  return ss_lane > 0.f ? 1.0f / sqrtf(ss_lane) : 0.f;
}

// Whether the two best fp32 scores of a token are far enough apart to trust their order.
//   cosine: a score is 256 exact products summed in fp32 times the stored inverse norm: within
//           256 * 2^-24 |a| = 1.53e-5 |a| of the exact value; pairs closer than twice that (plus slack) fail.
//   L2:     score = a.b - ||b||^2/2 with error <= 1.53e-5 |a||b| + 2^-24 (||b||^2 + |a||b|).  Any reference that
//           could still win is at most as far from a as the fp32 winner, so |b| <= |a| + |a - b_best| with
//           |a - b_best|^2 = |a|^2 - 2 best (5 % slack for the fp32 evaluation of that bound).
__device__ inline bool gap_is_safe(float best, float second, float na2, int metric) {
  const float na = sqrtf(na2);
  if (metric) {
    const float nb = 1.05f * (na + sqrtf(fmaxf(na2 - 2.f * best, 0.f)));
    return best - second > 4e-5f * na * nb + 2e-7f * nb * nb;
  }
  return best - second > 4e-5f * na;
}

constexpr int kKeyIdxMask = 0xFFFFFF;   // low 24 bits of an exact-pass key hold (2^24 - 1 - ordinal)
// Values of the per-round `ord` array besides an ordinal: -1 = queued for the exact pass (the ordinal is in the
// round's exact_key), kOrdNone = the token has no reference of this rank (fewer candidates than top_k; every slot
// but the first of a reference token).
constexpr int kOrdNone = -2;

// Top-k retrieval (section 4.1, arg top-k) runs as top_k rounds of the top-1 search: round r finds the best
// candidate that rounds 0..r-1 did not take, so the r-th slot holds the token's (r+1)-th nearest reference with
// equal scores in ascending ordinal.  The final ordinal round rr assigned to (token n, head h), or -1 for none.
__device__ inline int round_ordinal(const CompressParams& P, int rr, int64_t n, int h) {
  const int64_t at = (int64_t)rr * P.round_stride + n * P.Hkv + h;
  const int o = P.ord_all[at];
  if (o >= 0) return o;
  if (o == kOrdNone) return -1;
  return kKeyIdxMask - (int)(P.exact_key_all[at] & kKeyIdxMask);
}

// 4-bit token-wise latents (section 5.3): scale = bf16((max - min) / 15), zero = bf16(min), code =
// clamp(round_half_even((z - zero) / scale), 0, 15), all in fp32 (the decision precision of the format).
struct Q4Params {
  uint32_t scale_bits, zero_bits;
  float zero, inv;
};
__device__ inline Q4Params q4_params(float mn, float mx) {
  Q4Params q;
  q.scale_bits = f32_to_bf16_bits((mx - mn) * (1.0f / 15.0f));
  q.zero_bits = f32_to_bf16_bits(mn);
  const float scale = __uint_as_float(q.scale_bits << 16);
  q.zero = __uint_as_float(q.zero_bits << 16);
  q.inv = scale > 0.f ? 1.0f / scale : 0.f;
  return q;
}
__device__ inline uint32_t q4_code(float z, const Q4Params& q) {
  return (uint32_t)fminf(fmaxf(rintf((z - q.zero) * q.inv), 0.f), 15.f);
}

// The ordinal of a non-reference token from its merged fp32 result, or -1 after queueing it for the exact pass.
__device__ inline int decide_ordinal(const CompressParams& P, int64_t n, int b, int h, float best, float second, int arg,
                                     float na2) {
  if (arg >= 0 && gap_is_safe(best, second, na2, P.metric)) return arg;
  const int at = atomicAdd(&P.flag_count[b * P.Hkv + h], 1);
  P.flag_list[(int64_t)h * P.n_new_total + P.cu_new[b] + at] = (int)n;
  P.exact_key[n * P.Hkv + h] = kKeyIdxMask;          // (lowest score, ordinal 0); raised by the exact pass
  return -1;
}

__device__ inline int find_seq(const int32_t* cu, int batch, int n) {   // largest b with cu[b] <= n
  int lo = 0, hi = batch - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= n) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// ------------------------------------------------------------------------------------------------
// admit_refs: one wave per (new reference token, kv-head); grid (ceil(max new refs * Hkv / 4), B), 256 threads.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_admit_refs(CompressParams P) {
  if (blockIdx.x == 0 && blockIdx.y == 0)   // queue counters of the exact pass, every round's (cleared here, not by a memset node)
    for (int i = threadIdx.x; i < P.top_k * P.batch * P.Hkv; i += 256) P.flag_count_all[i] = 0;
  // W_down^T of both streams with padded rows, the form the projection kernel stages into LDS with wide copies:
  // element (stream, c, d) <- w_down[d][c]; the pad columns are zeroed
  if (blockIdx.y == 0 && P.mlp_kind < 0)   // (the non-linear compressor brings no W_down: its weights are packed by mlp_prep)
    for (int i = blockIdx.x * 256 + threadIdx.x; i < 2 * P.R * kWPad; i += gridDim.x * 256) {
      const int st = i / (P.R * kWPad), rem = i % (P.R * kWPad), c = rem / kWPad, d = rem % kWPad;
      P.wt[i] = d < kHeadDim ? (st ? P.w_down_v : P.w_down_k)[d * P.R + c] : (uint16_t)0;
    }
  const int b = blockIdx.y;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int l = threadIdx.x & 63;
  const int lb = P.len_before[b], la = lb + P.cu_new[b + 1] - P.cu_new[b];
  const int ord = refs_below(lb, P.stride) + item / P.Hkv, h = item % P.Hkv;   // first new reference: ceil(lb / s)
  const int64_t pos = (int64_t)ord * P.stride;
  if (pos >= la || ord >= P.rt_stride) return;
  const int64_t n = P.cu_new[b] + (pos - lb);
  const int slot = clampi(P.ref_tables[(int64_t)b * P.rt_stride + ord], 0, (int)P.n_ref_slots - 1);
  const uint32_t kx = reinterpret_cast<const uint32_t*>(P.k_new + (n * P.Hkv + h) * kHeadDim)[l];
  const uint32_t vx = reinterpret_cast<const uint32_t*>(P.v_new + (n * P.Hkv + h) * kHeadDim)[l];
  uint16_t* rk = P.ref + (int64_t)h * P.ref_head_stride + (int64_t)slot * kHeadDim;
  reinterpret_cast<uint32_t*>(rk)[l] = kx;
  reinterpret_cast<uint32_t*>(rk + P.ref_kv_stride)[l] = vx;
  const float ss = bf16lo(kx) * bf16lo(kx) + bf16hi(kx) * bf16hi(kx) + bf16lo(vx) * bf16lo(vx) + bf16hi(vx) * bf16hi(vx);
  const double dd = (double)bf16lo(kx) * bf16lo(kx) + (double)bf16hi(kx) * bf16hi(kx) + (double)bf16lo(vx) * bf16lo(vx) +
                    (double)bf16hi(vx) * bf16hi(vx);
  const float term = ref_term(ss, dd, P.metric);
  if (l == 0) P.ref_inv_norm[(int64_t)h * P.ref_norm_head_stride + slot] = term;
}

// ------------------------------------------------------------------------------------------------
// sim_top2: grid (B*Hkv, NS, tiles_max), 4 or 8 waves, wave tile (16*TB) tokens x 64 references.
// ------------------------------------------------------------------------------------------------
constexpr int kNT = 64;                 // references per LDS tile
constexpr int kRowPad = 264;            // bf16 elements per staged reference row (256 + 8: shifts banks)

struct Top2 {
  float best, second;
  int idx;
};
__device__ inline void top2_push(Top2& t, float v, int j) {   // strict '>' keeps the earliest ordinal
  const bool gt = v > t.best;
  t.second = __builtin_amdgcn_fmed3f(t.best, t.second, v);
  t.idx = gt ? j : t.idx;
  t.best = fmaxf(t.best, v);
}
__device__ inline void top2_merge(Top2& a, float ob, float os, int oi) {
  const bool take = (ob > a.best) || (ob == a.best && oi >= 0 && (a.idx < 0 || oi < a.idx));
  const float lo = fminf(a.best, ob);
  a.second = fmaxf(fmaxf(a.second, os), lo);
  a.best = fmaxf(a.best, ob);
  a.idx = take ? oi : a.idx;
}

// The product is issued as D[reference][token] (A = 16 staged reference rows from LDS, B = this wave's token
// rows, resident in registers): a lane then owns ONE token per 16-token block and sees four references per
// MFMA result, so the running (best, second, arg best) is one small state per token block instead of one per
// accumulator row, and only the four lane groups have to be merged at the end.
//
// One wave per SIMD with the whole register file (token operands 128 registers, two operand sets, two
// accumulator sets), software-pipelined by hand: while the 8*TB MFMAs of step q run, the LDS reads of step
// q+1's operands are in flight and the VALU epilogue of step q-1 (scale, mask, top-2) is issued in the MFMA
// shadow; reference tiles are staged through three LDS buffers so that one barrier per tile suffices.
// EXC (rounds after the first of a top-k search): candidates that an earlier round took are left out.
template <int TB, bool L2M, int NW, bool EXC>
__global__ __launch_bounds__(NW * 64) void k_sim_top2(CompressParams P) {
  constexpr int WM = 16 * TB, MT = NW * WM;
  constexpr int LPW = 32 / NW;                                // direct loads of reference rows per wave and tile
  constexpr int kTile = kNT * 256;                           // bf16 elements of one staged tile (64 rows x 512 B)
  extern __shared__ uint16_t lds_raw[];
  float* nrm = reinterpret_cast<float*>(lds_raw + 3 * kTile);   // [3][kNT]

  // Blocks are handed out in the order of their linear index, x fastest: (sequence, kv-head) runs fastest and the
  // token tile slowest, last tile first, so the tiles with the most candidate references (the causal search gets
  // longer with position) of ALL heads start first and the short ones fill the gaps at the end.
  const int tt = (int)gridDim.z - 1 - (int)blockIdx.z, split = blockIdx.y;
  const int b = blockIdx.x / P.Hkv, h = blockIdx.x % P.Hkv;
  const int n_new = P.cu_new[b + 1] - P.cu_new[b];
  if (tt * MT >= n_new) return;
  const int tid = threadIdx.x, l = tid & 63, ln = l & 15, lg = l >> 4;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lb = P.len_before[b];
  const int rows_valid = min(MT, n_new - tt * MT);
  const int pos_last = lb + tt * MT + rows_valid - 1;
  const int ncand_tile = min(refs_below(pos_last, P.stride), P.rt_stride);   // ordinals any row may use
  // this split's reference range, in whole tiles
  const int tiles_all = ceil_div(ncand_tile, kNT);
  const int tiles_per = ceil_div(tiles_all, P.NS);
  const int t_begin = split * tiles_per, t_end = min(tiles_all, t_begin + tiles_per);
  const int n_t = t_end - t_begin;

  // B operands: this wave's token rows (lane ln <-> token ln of each block), K (kk 0..3) then V (kk 4..7)
  bf16x8 tok[TB][8];
  float na2[TB];
  int ncand_tok[TB];          // candidates of the lane's token: ordinals j with j*s < pos, capped by the tile's
  const int row0 = tt * MT + w * WM;
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    const int r = row0 + tb * 16 + ln;
    const bool ok = r < n_new;
    ncand_tok[tb] = ok ? min(refs_below(lb + r, P.stride), ncand_tile) : 0;
    const int64_t n = P.cu_new[b] + (ok ? r : 0);
    const uint16_t* kr = P.k_new + (n * P.Hkv + h) * kHeadDim;
    const uint16_t* vr = P.v_new + (n * P.Hkv + h) * kHeadDim;
    float ss = 0.f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 x = *reinterpret_cast<const uint4*>(kr + (4 * kk + lg) * 8);
      uint4 y = *reinterpret_cast<const uint4*>(vr + (4 * kk + lg) * 8);
      if (!ok) { x = make_uint4(0, 0, 0, 0); y = x; }
      tok[tb][kk] = __builtin_bit_cast(bf16x8, x);
      tok[tb][4 + kk] = __builtin_bit_cast(bf16x8, y);
      const uint32_t uu[8] = {x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += bf16lo(uu[e]) * bf16lo(uu[e]) + bf16hi(uu[e]) * bf16hi(uu[e]);
    }
    ss += __shfl_xor(ss, 16);
    ss += __shfl_xor(ss, 32);
    na2[tb] = ss;
  }
  Top2 st[TB];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) st[tb] = Top2{-INFINITY, -INFINITY, -1};
  // ordinals taken by earlier rounds, as the codes this lane's epilogue sees them (a lane group sees the ordinals
  // with (j % 16) / 4 = lg; code = (j / 16) * 4 + j % 4); -1 (no code is negative) where there is none
  int exc[TB][3];
  if constexpr (EXC) {
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int r = row0 + tb * 16 + ln;
      const int64_t n = P.cu_new[b] + (r < n_new ? r : 0);
#pragma unroll
      for (int e = 0; e < 3; ++e) {
        const int x = e < P.round ? round_ordinal(P, e, n, h) : -1;
        exc[tb][e] = (x >= 0 && ((x >> 2) & 3) == lg) ? (((x >> 4) << 2) | (x & 3)) : -1;
      }
    }
  }

  const uint16_t* refk = P.ref + (int64_t)h * P.ref_head_stride;
  const uint16_t* refv = refk + P.ref_kv_stride;
  const float* rnorm = P.ref_inv_norm + (int64_t)h * P.ref_norm_head_stride;
  const int32_t* rtab = P.ref_tables + (int64_t)b * P.rt_stride;

  // Reference tiles go from global memory straight into LDS (global_load_lds_dwordx4: lane l's 16 bytes land at
  // a wave-uniform base + 16*l; placement checked on the hardware), no staging registers.  A tile is 64 rows of
  // 32 sixteen-byte chunks (K half then V half), unpadded; chunk c of row r is stored at position c ^ (r & 15),
  // which the loads realise by permuting their SOURCE chunk, so that the 16 rows read by one operand fetch hit
  // distinct banks.  Wave w issues loads i = 0..7 of a tile; load (w, i) fills rows 2*(8w+i) and 2*(8w+i)+1.
  // Every wave also copies the 64 inverse norms (same values to the same place: keeps all waves' load counts equal).
  const int my_row = l >> 5;                                  // which of the two rows of a load this lane fills
  const int my_pos = l & 31;                                  // position inside the row
  auto load_slots = [&](int t, int (&slot)[LPW + 1]) {        // pool slots of the rows this lane will fill
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const int r = 2 * (LPW * w + i) + my_row;
      slot[i] = rtab[(uint32_t)min(t * kNT + r, ncand_tile - 1)];   // rows past the end repeat the last reference
    }                                                                // (they are masked by the candidate count)
    slot[LPW] = rtab[(uint32_t)min(t * kNT + l, ncand_tile - 1)];
  };
  auto issue_tile = [&](int buf, const int (&slot)[LPW + 1]) {
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const int r = 2 * (LPW * w + i) + my_row;
      const int c = my_pos ^ (r & 15);
      // unsigned clamp (a negative table entry lands on the last slot): one instruction, zero-extended address
      const uint16_t* src = (c < 16 ? refk : refv) + (uint64_t)min((uint32_t)slot[i], (uint32_t)P.n_ref_slots - 1u) * kHeadDim + (c & 15) * 8;
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                       (void __attribute__((address_space(3)))*)(lds_raw + buf * kTile + (LPW * w + i) * 512),
                                       16, 0, 0);
    }
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(rnorm + min((uint32_t)slot[LPW], (uint32_t)P.n_ref_slots - 1u)),
                                     (void __attribute__((address_space(3)))*)(nrm + buf * kNT), 4, 0, 0);
  };
  // s_waitcnt for the vector-memory counter only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14)
  auto wait_vm = [](auto N) {
    constexpr int n = decltype(N)::value;
    __builtin_amdgcn_s_waitcnt((n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14));
  };

  if (n_t > 0) {
    // Per tile and wave: LPW + 1 (= 9 with four waves) slot loads (S) then as many direct loads (D).  Order of issue: S(0) S(1) D(0) S(2) D(1) |
    // tile ti: S(ti+3) D(ti+2) ... so D(ti+1), needed at the end of tile ti, has two tiles of work to land in,
    // and everything issued after it is S(ti+3), D(ti+2): 18 loads.
    int slot_a[LPW + 1], slot_b[LPW + 1];                     // slots of tiles ti+2 (a) and ti+3 (b)
    load_slots(t_begin, slot_a);
    load_slots(t_begin + (n_t > 1 ? 1 : 0), slot_b);
    issue_tile(0, slot_a);
    load_slots(t_begin + min(2, n_t - 1), slot_a);
    issue_tile(1, slot_b);
    wait_vm(std::integral_constant<int, 2 * (LPW + 1)>{});   // D(0) has landed (S(2), D(1) may be outstanding)
    __syncthreads();
    const int pos_first = lb + row0;                         // smallest position in this wave's rows

    struct Step { float inv[4]; int jb; int code0; };
    bf16x8 aop[2][8];
    float4v acc[2][TB];
    Step inext, icur, iprev;                                  // of the step being prefetched / computed / finished
    const int swz = ln;
    // operands and inverse norms of step (ti, cb): every LDS read of a tile happens before the barrier that
    // lets other waves overwrite its buffer
    // (The per-reference floats of a step come from `invt`, read once per tile: the compiler puts a wait for EVERY
    // outstanding global load in front of an LDS read of memory that direct-to-LDS loads write.  In front of each
    // step that wait exposed the whole latency of the loads issued a moment earlier, several hundred cycles per
    // tile and wave; at the top of a tile, before the tile's own loads are issued, only loads a tile old are in
    // flight.)
    auto prefetch = [&](int ti, int cb, bf16x8 (&dst)[8], Step& s, const float4* invt) {
      const int buf = ti % 3;
      const uint16_t* base = lds_raw + buf * kTile + (cb * 16 + ln) * 256;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) dst[kk] = *reinterpret_cast<const bf16x8*>(base + (((4 * kk + lg) ^ swz) * 8));
      if (invt) { s.inv[0] = invt[cb].x; s.inv[1] = invt[cb].y; s.inv[2] = invt[cb].z; s.inv[3] = invt[cb].w; }
      s.jb = (t_begin + ti) * kNT + cb * 16 + 4 * lg;
      s.code0 = ((t_begin + ti) * 4 + cb) * 4;               // wave-uniform; the ordinal is rebuilt from it at the end
    };
    auto mfmas = [&](const bf16x8 (&a)[8], float4v (&c)[TB]) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) c[tb] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) c[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kk], tok[tb][kk], c[tb], 0, 0, 0);
    };
    // lane holds references s.jb + i (i = 0..3) of token ln in every block
    auto taken = [&](int tb, int code) { return EXC && (code == exc[tb][0] || code == exc[tb][1] || code == exc[tb][2]); };
    auto epilogue_full = [&](const float4v (&c)[TB], const Step& s) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
          top2_push(st[tb], taken(tb, s.code0 + i) ? -INFINITY : (L2M ? c[tb][i] - s.inv[i] : c[tb][i] * s.inv[i]), s.code0 + i);
    };
    auto epilogue_masked = [&](const float4v (&c)[TB], const Step& s) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        const int left = ncand_tok[tb] - s.jb;               // this lane's references i < left are candidates
#pragma unroll
        for (int i = 0; i < 4; ++i)
          top2_push(st[tb], i < left && !taken(tb, s.code0 + i) ? (L2M ? c[tb][i] - s.inv[i] : c[tb][i] * s.inv[i]) : -INFINITY,
                    s.code0 + i);
      }
    };
    // a step needs no mask if even its last reference is a candidate of the wave's first (lowest) token
    auto is_full = [&](int ti, int cb) {
      const int jb0 = (t_begin + ti) * kNT + cb * 16;
      return (int64_t)(jb0 + 15) * P.stride < pos_first && jb0 + 16 <= ncand_tile;
    };

    // pipeline prologue: operands of step (0, 0); a dummy "previous step" whose scores are all masked
    prefetch(0, 0, aop[0], icur, nullptr);
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[1][tb] = float4v{0.f, 0.f, 0.f, 0.f};
    iprev.inv[0] = iprev.inv[1] = iprev.inv[2] = iprev.inv[3] = 0.f;
    iprev.jb = 0x3fffffff;
    iprev.code0 = 0;
    bool prev_full = false;

    // one tile: S(ti+3) into `fill`, D(ti+2) from `use`, four steps with the barrier before the last one
    auto tile_body = [&](int ti, const int (&use)[LPW + 1], int (&fill)[LPW + 1]) {
      // per-reference floats of the tile's four steps (the barrier that let step (ti, 0) be prefetched made them visible)
      float4 invt[4];
      __builtin_amdgcn_sched_barrier(0);       // not earlier than here: the loads of a whole tile ago must have had their time ...
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) invt[cb] = *reinterpret_cast<const float4*>(nrm + (ti % 3) * kNT + cb * 16 + 4 * lg);
      __builtin_amdgcn_sched_barrier(0);       // ... and only then the tile's own loads
      icur.inv[0] = invt[0].x; icur.inv[1] = invt[0].y; icur.inv[2] = invt[0].z; icur.inv[3] = invt[0].w;
      // loads are unconditional (past the end they re-load the last tile into a buffer nobody reads), so that
      // the number of loads in flight -- and with it the wait count below -- is the same in every iteration
      load_slots(t_begin + min(ti + 3, n_t - 1), fill);
      issue_tile((ti + 2) % 3, use);
      auto step = [&](auto CB) {
        constexpr int cb = decltype(CB)::value, cur = cb & 1, nxt = cur ^ 1;
        if (cb < 3) prefetch(ti, cb + 1, aop[nxt], inext, invt);
        else if (ti + 1 < n_t) prefetch(ti + 1, 0, aop[nxt], inext, nullptr);
        // one basic block per variant: the MFMAs of this step and the epilogue of the previous one interleave
        if (prev_full) {
          mfmas(aop[cur], acc[cur]);
          epilogue_full(acc[nxt], iprev);
        } else {
          mfmas(aop[cur], acc[cur]);
          epilogue_masked(acc[nxt], iprev);
        }
        prev_full = is_full(ti, cb);
        iprev = icur;
        icur = inext;
      };
      step(std::integral_constant<int, 0>{});
      step(std::integral_constant<int, 1>{});
      step(std::integral_constant<int, 2>{});
      // before step 3 prefetches the first operands of tile ti+1: its direct loads (issued one tile ago) must
      // have landed in every wave; after it nobody reads tile ti's buffer any more
      wait_vm(std::integral_constant<int, 2 * (LPW + 1)>{});
      __syncthreads();
      step(std::integral_constant<int, 3>{});
    };
    for (int ti = 0; ti < n_t; ti += 2) {
      tile_body(ti, slot_a, slot_b);
      if (ti + 1 < n_t) tile_body(ti + 1, slot_b, slot_a);
    }
    if (prev_full) epilogue_full(acc[1], iprev); else epilogue_masked(acc[1], iprev);
    wait_vm(std::integral_constant<int, 0>{});               // no LDS write may be in flight when the block ends
  }
  // rebuild ordinals, merge the four lane groups of every token; ties go to the lower ordinal
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    Top2 t = st[tb];
    t.idx = (t.best == -INFINITY || t.idx < 0) ? -1 : (t.idx >> 2) * 16 + 4 * lg + (t.idx & 3);
#pragma unroll
    for (int o = 16; o < 64; o <<= 1) {
      const float ob = __shfl_xor(t.best, o), os = __shfl_xor(t.second, o);
      const int oi = __shfl_xor(t.idx, o);
      top2_merge(t, ob, os, oi);
    }
    const int r = row0 + tb * 16 + ln;
    if (lg == 0 && r < n_new) {
      const int64_t n = P.cu_new[b] + r;
      if (P.NS == 1) {        // the whole reference range was this block's: decide here, no resolve kernel
        const int pos = lb + r;
        int o;
        if (pos % P.stride == 0) o = P.round == 0 ? pos / P.stride : kOrdNone;   // a reference token: itself, once
        else if (P.round >= min(refs_below(pos, P.stride), P.rt_stride)) o = kOrdNone;   // fewer candidates than rounds
        else o = decide_ordinal(P, n, b, h, t.best, t.second, t.idx, na2[tb]);
        P.ord[n * P.Hkv + h] = o;
      } else {
        float4 o;
        o.x = t.best; o.y = t.second; o.z = __int_as_float(t.idx); o.w = na2[tb];
        *reinterpret_cast<float4*>(P.part + ((n * P.Hkv + h) * P.NS + split) * 4) = o;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// resolve: one thread per (new token, kv-head); grid ceil(n_new*Hkv/256).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_resolve(CompressParams P) {
  const int item = blockIdx.x * 256 + threadIdx.x;
  if (item >= P.n_new_total * P.Hkv) return;
  const int n = item / P.Hkv, h = item % P.Hkv;
  const int b = find_seq(P.cu_new, P.batch, n);
  const int pos = P.len_before[b] + (n - P.cu_new[b]);
  int ord;
  if (pos % P.stride == 0) {
    ord = P.round == 0 ? pos / P.stride : kOrdNone;
  } else if (P.round >= min(refs_below(pos, P.stride), P.rt_stride)) {
    ord = kOrdNone;
  } else {
    // merge the reference-range splits (ascending ranges: strict '>' keeps the lowest ordinal)
    float bb = -INFINITY, b2 = -INFINITY, na2 = 0.f;
    int bi = -1;
    const float4* pp = reinterpret_cast<const float4*>(P.part) + (int64_t)item * P.NS;
    for (int s = 0; s < P.NS; ++s) {
      const float4 o = pp[s];
      na2 = o.w;
      const int oi = __float_as_int(o.z);
      if (oi < 0) continue;
      if (o.x > bb) { b2 = fmaxf(bb, o.y); bb = o.x; bi = oi; }
      else b2 = fmaxf(b2, o.x);
    }
    ord = decide_ordinal(P, n, b, h, bb, b2, bi, na2);
  }
  P.ord[item] = ord;
}

// ------------------------------------------------------------------------------------------------
// exact: grid (kExactX, kExactSplits, B*Hkv), 256 threads.  A block takes 16 queued tokens of its
// (sequence, kv-head) at a time and every kExactSplits*4-th 16-reference tile per wave.
// D[token][ref] = sum_d a[token][d] b[ref][d] in fp64 on v_mfma_f64_16x16x4 (operand layout checked on the
// hardware with one-hot inputs): lane (ln, lg) supplies element e of its 8-wide chunk as the k = lg slot of
// step (kk, e), identically for both operands.  Waves publish their best with a 64-bit atomic max on the key
// (cosine in 2^-38 steps above -1) << 24 | (2^24-1 - ordinal): the larger cosine wins, then the lower ordinal.
// With the L2 metric the 40 score bits are the complement of the leading bits of the fp64 squared distance
// |a|^2 - 2 a.b + |b|^2 (sign, exponent, 28 mantissa bits: distances closer than 2^-28 relative tie).
// ------------------------------------------------------------------------------------------------
constexpr int kExactX = 2;    // few blocks: an idle block of this kernel still costs a dispatch with ~240 registers per lane
constexpr int kExactSplits = 32;  // each wave then scores one 16-reference tile per 2048 candidates
typedef double double4v __attribute__((ext_vector_type(4)));

__device__ inline double bf16_elem_f64(const uint4& c, int e) {
  const uint32_t u = (e < 2) ? c.x : (e < 4) ? c.y : (e < 6) ? c.z : c.w;
  return (double)((e & 1) ? bf16hi(u) : bf16lo(u));
}

__global__ __launch_bounds__(256) void k_exact(CompressParams P) {
  const int b = blockIdx.z / P.Hkv, h = blockIdx.z % P.Hkv;
  const int cnt = P.flag_count[blockIdx.z];
  const int n_tiles = ceil_div(cnt, 16);
  if ((int)blockIdx.x >= n_tiles) return;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 15, lg = l >> 4;
  const int lb = P.len_before[b];
  const int32_t* list = P.flag_list + (int64_t)h * P.n_new_total + P.cu_new[b];
  const int32_t* rtab = P.ref_tables + (int64_t)b * P.rt_stride;
  const uint16_t* refk = P.ref + (int64_t)h * P.ref_head_stride;
  const uint16_t* refv = refk + P.ref_kv_stride;
  const int lane_tile0 = blockIdx.y * 4 + w, tile_step = kExactSplits * 4;

  for (int tile = blockIdx.x; tile < n_tiles; tile += kExactX) {
    // lane ln <-> queued token tile*16 + ln (rows past the end repeat the last one and are not published)
    const int qi = min(tile * 16 + ln, cnt - 1);
    const int n = list[qi];
    const int pos = lb + (n - P.cu_new[b]);
    const uint16_t* ak = P.k_new + ((int64_t)n * P.Hkv + h) * kHeadDim;
    const uint16_t* av = P.v_new + ((int64_t)n * P.Hkv + h) * kHeadDim;
    uint4 a[8];
    double na2 = 0.0;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      a[kk] = *reinterpret_cast<const uint4*>(ak + (4 * kk + lg) * 8);
      a[4 + kk] = *reinterpret_cast<const uint4*>(av + (4 * kk + lg) * 8);
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
#pragma unroll
      for (int e = 0; e < 8; ++e) { const double x = bf16_elem_f64(a[kk], e); na2 += x * x; }
    na2 += __shfl_xor(na2, 16);
    na2 += __shfl_xor(na2, 32);
    const double na = sqrt(na2);
    int pmax = pos;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) pmax = max(pmax, __shfl_xor(pmax, o));
    const int ncand = min(refs_below(pmax, P.stride), P.rt_stride);
    // accumulator register i of the fp64 MFMA holds token row 4*i + lg (rows are interleaved over the lane
    // groups, unlike the 32-bit variants where a lane group holds four consecutive rows)
    double na_row[4];
    int pos_row[4], n_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      na_row[i] = __shfl(na, 4 * i + lg);
      pos_row[i] = __shfl(pos, 4 * i + lg);
      n_row[i] = __shfl(n, 4 * i + lg);
    }
    double na2_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) na2_row[i] = __shfl(na2, 4 * i + lg);
    int exc_row[4][3];                     // ordinals earlier rounds of a top-k search took (-1: none)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 3; ++e) exc_row[i][e] = e < P.round ? round_ordinal(P, e, n_row[i], h) : -1;
    double cbest[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    int jbest[4] = {0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff};
    for (int rt = lane_tile0; rt * 16 < ncand; rt += tile_step) {
      const int j = rt * 16 + ln;
      const int slot = clampi(rtab[min(j, ncand - 1)], 0, (int)P.n_ref_slots - 1);
      uint4 bq[8];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bq[kk] = *reinterpret_cast<const uint4*>(refk + (int64_t)slot * kHeadDim + (4 * kk + lg) * 8);
        bq[4 + kk] = *reinterpret_cast<const uint4*>(refv + (int64_t)slot * kHeadDim + (4 * kk + lg) * 8);
      }
      double nb2 = 0.0;
      double4v acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const double x = bf16_elem_f64(a[kk], e), y = bf16_elem_f64(bq[kk], e);
          nb2 += y * y;
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, acc, 0, 0, 0);
        }
      nb2 += __shfl_xor(nb2, 16);
      nb2 += __shfl_xor(nb2, 32);
      const double nb = sqrt(nb2);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const double den = na_row[i] * nb;
        const double c = P.metric ? -fmax(na2_row[i] - 2.0 * acc[i] + nb2, 0.0) : (den > 0.0 ? acc[i] / den : 0.0);
        const bool ok = j < ncand && (int64_t)j * P.stride < pos_row[i] && j != exc_row[i][0] && j != exc_row[i][1] &&
                        j != exc_row[i][2];
        if (ok && c > cbest[i]) { cbest[i] = c; jbest[i] = j; }   // ascending j per lane: strict '>'
      }
    }
    // best over the 16 reference lanes (ties go to the lower ordinal), then one atomic per token row
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) {
        const double oc = __shfl_xor(cbest[i], o);
        const int oj = __shfl_xor(jbest[i], o);
        if (oc > cbest[i] || (oc == cbest[i] && oj < jbest[i])) { cbest[i] = oc; jbest[i] = oj; }
      }
      if (ln == 0 && tile * 16 + 4 * i + lg < cnt && jbest[i] != 0x7fffffff) {
        const double cc = fmin(fmax(cbest[i], -1.0), 1.0) + 1.0;                      // [0, 2]
        const unsigned long long q = P.metric
            ? ((1ull << 40) - 1) - ((unsigned long long)__double_as_longlong(-cbest[i]) >> 24)   // -cbest >= 0
            : (unsigned long long)(cc * 274877906944.0 + 0.5);                         // 2^-38 steps, q <= 2^39
        const unsigned long long key = (q << 24) | (unsigned long long)(kKeyIdxMask - (jbest[i] & kKeyIdxMask));
        atomicMax(reinterpret_cast<unsigned long long*>(P.exact_key) + ((int64_t)n_row[i] * P.Hkv + h), key);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// project: grid (ceil(page_tiles_max / pages per block), B), 256 threads; wave w handles kv-heads w, w+4, ...
// A wave owns one page of one sequence: lane (ln, lg) <-> token slot ln of the page, 8-wide chunk.
// ------------------------------------------------------------------------------------------------

// KS = 4 (top-k retrieval, section 4.1): the residual is taken against the MEAN of the raw rows of the references
// the rounds assigned to the token (one to four), and every ordinal slot of the token is written.
template <int R, int KS>
__global__ __launch_bounds__(256) void k_project(CompressParams P) {
  constexpr int NB = R / 16;
  extern __shared__ uint16_t wlds[];   // [2][R][kWPad]: W_dK^T, W_dV^T
  const int b = blockIdx.y;
  const int lb = P.len_before[b];
  const int n_new = P.cu_new[b + 1] - P.cu_new[b];
  const int la = lb + n_new;
  const int page_first = lb / kPage;
  const int lp0 = page_first + blockIdx.x * P.proj_ppb;   // first logical page of the block
  if (n_new <= 0 || lp0 * kPage >= la) return;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 15, lg = l >> 4;
  // stage W_down^T of both streams (transposed and padded by admit_refs) with 16-byte copies; a block of a long
  // call takes several consecutive pages, so that the staging (half as many bytes as a page brings) is shared
  for (int i = tid; i < 2 * R * kWPad / 8; i += 256)
    reinterpret_cast<uint4*>(wlds)[i] = reinterpret_cast<const uint4*>(P.wt)[i];
  __syncthreads();
  for (int lp = lp0; lp < lp0 + P.proj_ppb && lp * kPage < la; ++lp) {
  const int pos = lp * kPage + ln;
  const bool tok_ok = pos >= lb && pos < la;
  const int64_t n = P.cu_new[b] + (tok_ok ? pos - lb : 0);
  const bool is_ref = (pos % P.stride) == 0;
  int page = P.block_tables[(int64_t)b * P.bt_stride + min(lp, P.bt_stride - 1)];
  page = clampi(page, 0, (int)P.n_pages_pool - 1);
  const int32_t* rtab = P.ref_tables + (int64_t)b * P.rt_stride;

  // ordinal and reference slot of the lane's token for kv-head h: the fp32 decision, or (negative) the exact pass's
  // key; both are loaded unconditionally (no load behind a branch), and one head ahead of their use, so that the
  // chain ordinal -> table entry -> reference row of the next head runs under the current head's arithmetic
  auto fetch_ord = [&](int h) {
    const int hh = min(h, P.Hkv - 1);
    const int o = P.ord_all[n * P.Hkv + hh];                      // (round 0)
    const int oe = kKeyIdxMask - (int)(P.exact_key_all[n * P.Hkv + hh] & kKeyIdxMask);
    return clampi(o < 0 ? oe : o, 0, P.rt_stride - 1);
  };
  int ord_next = fetch_ord(w);
  int slot_next = rtab[ord_next];
  for (int h = w; h < P.Hkv; h += 4) {
    const uint16_t* kr = P.k_new + (n * P.Hkv + h) * kHeadDim;
    const uint16_t* vr = P.v_new + (n * P.Hkv + h) * kHeadDim;
    const int ord = ord_next;
    // residual against the chosen raw reference, fp32 (exact for bf16 inputs), split into bf16 hi + lo
    const int slot = clampi(slot_next, 0, (int)P.n_ref_slots - 1);
    ord_next = fetch_ord(h + 4);
    slot_next = rtab[ord_next];
    const uint16_t* rk = P.ref + (int64_t)h * P.ref_head_stride + (int64_t)slot * kHeadDim;
    const uint16_t* rv = rk + P.ref_kv_stride;
    const bool zero = !tok_ok || is_ref;
    // several references: slot 0 is `ord` above; the others, where the token has them
    int ords[KS];
    const uint16_t* rks[KS];
    float inv_m = 1.f;
    if constexpr (KS > 1) {
      int cnt = 1;
      ords[0] = ord;
      rks[0] = rk;
#pragma unroll
      for (int i = 1; i < KS; ++i) {
        const int o = i < P.top_k ? round_ordinal(P, i, n, h) : -1;
        ords[i] = o < 0 ? -1 : min(o, P.rt_stride - 1);
        const int sl = clampi(rtab[max(ords[i], 0)], 0, (int)P.n_ref_slots - 1);
        rks[i] = P.ref + (int64_t)h * P.ref_head_stride + (int64_t)sl * kHeadDim;
        cnt += ords[i] >= 0 ? 1 : 0;
      }
      inv_m = 1.0f / (float)cnt;
    }
    bf16x8 res[2][4][2];   // [stream][kk][hi/lo]
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const uint4 x = *reinterpret_cast<const uint4*>((st ? vr : kr) + (4 * kk + lg) * 8);
        const uint4 y = *reinterpret_cast<const uint4*>((st ? rv : rk) + (4 * kk + lg) * 8);
        const uint32_t xu[4] = {x.x, x.y, x.z, x.w}, yu[4] = {y.x, y.y, y.z, y.w};
        float m0[4], m1[4];                  // the reference the residual is taken against, fp32
#pragma unroll
        for (int e = 0; e < 4; ++e) { m0[e] = bf16lo(yu[e]); m1[e] = bf16hi(yu[e]); }
        if constexpr (KS > 1) {              // mean of the rows in use (sum in fp32, one rounding per addition)
#pragma unroll
          for (int i = 1; i < KS; ++i) {
            const uint4 yi = *reinterpret_cast<const uint4*>(rks[i] + (st ? P.ref_kv_stride : 0) + (4 * kk + lg) * 8);
            const uint32_t yiu[4] = {yi.x, yi.y, yi.z, yi.w};
            const bool on = ords[i] >= 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) { m0[e] += on ? bf16lo(yiu[e]) : 0.f; m1[e] += on ? bf16hi(yiu[e]) : 0.f; }
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) { m0[e] *= inv_m; m1[e] *= inv_m; }
        }
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float r0 = bf16lo(xu[e]) - m0[e], r1 = bf16hi(xu[e]) - m1[e];
          if (zero) { r0 = 0.f; r1 = 0.f; }
          hi[e] = pack_bf16(r0, r1);
          lo[e] = pack_bf16(r0 - bf16lo(hi[e]), r1 - bf16hi(hi[e]));
        }
        res[st][kk][0] = __builtin_bit_cast(bf16x8, make_uint4(hi[0], hi[1], hi[2], hi[3]));
        res[st][kk][1] = __builtin_bit_cast(bf16x8, make_uint4(lo[0], lo[1], lo[2], lo[3]));
      }
    uint16_t* lat = P.latent + (int64_t)page * P.latent_page_stride + (int64_t)h * P.latent_head_stride;
    // stream 0 (scores-operand order): D^T[c][token], lane holds 4 consecutive c of token ln
    float4v q4acc[NB];                 // 4-bit latents: the token's whole latent is needed before any of it is stored
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 wk = *reinterpret_cast<const bf16x8*>(wlds + (nb * 16 + ln) * kWPad + (4 * kk + lg) * 8);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wk, res[0][kk][0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wk, res[0][kk][1], acc, 0, 0, 0);
        if (P.joint) {
          const bf16x8 wv = *reinterpret_cast<const bf16x8*>(wlds + (R + nb * 16 + ln) * kWPad + (4 * kk + lg) * 8);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, res[1][kk][0], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, res[1][kk][1], acc, 0, 0, 0);
        }
      }
      q4acc[nb] = acc;
      if (tok_ok && !P.q4) {
        const int c = nb * 16 + 4 * lg;
        uint2 o;
        o.x = pack_bf16(acc[0], acc[1]);
        o.y = pack_bf16(acc[2], acc[3]);
        *reinterpret_cast<uint2*>(lat + ((c >> 3) * kPage + ln) * 8 + (c & 7)) = o;
      }
    }
    if (P.q4) {
      // the token's values sit in the four lanes (ln, lg = 0..3); value c = 16 nb + 4 lg + i is element
      // e = 4 (lg & 1) + i of chunk 2 nb + lg / 2 and goes to bits 4 (e / 2) + 16 (e & 1) of the chunk's dword
      float mn = INFINITY, mx = -INFINITY;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i) { mn = fminf(mn, q4acc[nb][i]); mx = fmaxf(mx, q4acc[nb][i]); }
      mn = fminf(mn, __shfl_xor(mn, 16)); mx = fmaxf(mx, __shfl_xor(mx, 16));
      mn = fminf(mn, __shfl_xor(mn, 32)); mx = fmaxf(mx, __shfl_xor(mx, 32));
      const Q4Params qp = q4_params(mn, mx);
      char* blk = reinterpret_cast<char*>(lat);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        uint32_t part = q4_code(q4acc[nb][0], qp) | (q4_code(q4acc[nb][1], qp) << 16) |
                        (q4_code(q4acc[nb][2], qp) << 4) | (q4_code(q4acc[nb][3], qp) << 20);
        part <<= 8 * (lg & 1);
        part |= __shfl_xor(part, 16);
        if (tok_ok && (lg & 1) == 0)
          *reinterpret_cast<uint32_t*>(blk + 4 * ((2 * nb + (lg >> 1)) * kPage + ln)) = part;
      }
      if (tok_ok && lg == 0) {
        uint16_t* sz = reinterpret_cast<uint16_t*>(blk + 8 * R + (ln >> 2) * 16 + (ln & 3) * 2);
        sz[0] = (uint16_t)qp.scale_bits;
        sz[4] = (uint16_t)qp.zero_bits;
      }
    }
    if (!P.joint) {
      // stream 1 (value-operand order): D[token][c], lane holds tokens 4*lg..4*lg+3 of column ln
      uint16_t* latv = lat + P.latent_stream_stride;
      const int t0 = lp * kPage + 4 * lg;                    // position of this lane's first token
      const bool all4 = t0 >= lb && t0 + 3 < la;
      float4v q4v[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const bf16x8 wv = *reinterpret_cast<const bf16x8*>(wlds + (R + nb * 16 + ln) * kWPad + (4 * kk + lg) * 8);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(res[1][kk][0], wv, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(res[1][kk][1], wv, acc, 0, 0, 0);
        }
        q4v[nb] = acc;
        if (P.q4) continue;
        uint16_t* dst = latv + (nb * 64 + l) * 4;
        if (all4) {
          uint2 o;
          o.x = pack_bf16(acc[0], acc[1]);
          o.y = pack_bf16(acc[2], acc[3]);
          *reinterpret_cast<uint2*>(dst) = o;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (t0 + i >= lb && t0 + i < la) dst[i] = (uint16_t)f32_to_bf16_bits(acc[i]);
        }
      }
      if (P.q4) {
        // Value stream, 4-bit: token 4 lg + i has its values in the 16 lanes (ln = 0..15, this lg) x NB registers.
        // The lane's codes for columns ln + 16 nb of its four tokens fill its own dword pair (.x: first and second
        // token at bits 4 (nb % 4) and 16 + 4 (nb % 4), .y: third and fourth) of column group nb / 4; tokens that
        // were written by an earlier call share those dwords and keep their bits.
        Q4Params qv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float mn = INFINITY, mx = -INFINITY;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) { mn = fminf(mn, q4v[nb][i]); mx = fmaxf(mx, q4v[nb][i]); }
#pragma unroll
          for (int o = 1; o < 16; o <<= 1) { mn = fminf(mn, __shfl_xor(mn, o)); mx = fmaxf(mx, __shfl_xor(mx, o)); }
          qv[i] = q4_params(mn, mx);
        }
        bool fresh[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) fresh[i] = t0 + i >= lb && t0 + i < la;
        const uint32_t keep_x = (fresh[0] ? 0u : 0x0000ffffu) | (fresh[1] ? 0u : 0xffff0000u);
        const uint32_t keep_y = (fresh[2] ? 0u : 0x0000ffffu) | (fresh[3] ? 0u : 0xffff0000u);
        char* vblk = reinterpret_cast<char*>(latv);
#pragma unroll
        for (int q = 0; q < (NB + 3) / 4; ++q) {
          uint2 w = make_uint2(0u, 0u);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int nb = 4 * q + j;
            if (nb < NB) {
              w.x |= (q4_code(q4v[nb][0], qv[0]) << (4 * j)) | (q4_code(q4v[nb][1], qv[1]) << (16 + 4 * j));
              w.y |= (q4_code(q4v[nb][2], qv[2]) << (4 * j)) | (q4_code(q4v[nb][3], qv[3]) << (16 + 4 * j));
            }
          }
          uint2* dst = reinterpret_cast<uint2*>(vblk + (q * 64 + l) * 8);
          if (!all4) {
            const uint2 old = *dst;
            w.x = (w.x & ~keep_x) | (old.x & keep_x);
            w.y = (w.y & ~keep_y) | (old.y & keep_y);
          }
          if (fresh[0] || fresh[1] || fresh[2] || fresh[3]) *dst = w;
        }
        if (ln == 0) {
          uint16_t* sz = reinterpret_cast<uint16_t*>(vblk + 8 * R + lg * 16);
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (fresh[i]) { sz[i] = (uint16_t)qv[i].scale_bits; sz[4 + i] = (uint16_t)qv[i].zero_bits; }
        }
      }
    }
    if (tok_ok && lg == 0) {
      int32_t* ip = P.idx + (int64_t)page * P.idx_page_stride + (int64_t)h * P.idx_head_stride + ln;
      ip[0] = ord;
      if constexpr (KS > 1) {
#pragma unroll
        for (int i = 1; i < KS; ++i)
          if (i < P.top_k) ip[i * P.idx_slot_stride] = ords[i];
      }
    }
  }
  }
}

// ------------------------------------------------------------------------------------------------
// Non-linear compressor (section 4.1: z = f_c(kv) - f_c(kv_ref) with a two-layer f_c; section 5.3: the gated
// variant).  One latent over K||V per (token, kv-head): JOINT layout, stream 0.
//   mlp_prep     transposes and zero-pads the weights into the workspace: W1^T (and Wg^T) [hidden_pad][kMlpXPad],
//                W2^T by chunks of kMlpChunk hidden columns (each chunk padded to whole KB), b1 padded.  Padded hidden columns have zero weights
//                and bias on both sides, so they contribute act(0) * 0 = 0.
//   project_mlp  grid (pages, B, ceil(Hkv / 4)), 256 threads; wave w takes kv-head 4 z + w of the block's page (the
//                four waves share the staged weights).  Both GEMMs run
//                transposed so that the first one's result is already the second one's operand:
//                  H^T[j][tok]  = sum_f W1^T[j][f] x[tok][f]      A = W1^T rows from LDS, B = the token's raw row
//                  z^T[c][tok] += sum_j W2^T[c][j] d[j][tok]      B = d = act(H_token) - act(H_reference), in the
//                                                                  lane that computed it, split into bf16 hi + lo
//                (the second GEMM is linear, so the difference is formed BEFORE it: one GEMM instead of two, and
//                the cancellation happens in fp32 rather than after a rounding to bf16).
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_mlp_prep(CompressParams P) {
  const int hp = P.mlp_hidden_pad, hd = P.mlp_hidden;
  const int64_t n1 = (int64_t)hp * kMlpXPad, n2 = (int64_t)(hp / kMlpChunk) * mlp_w2_chunk_elems(P.R);
  const int64_t total = n1 + n2 + hp;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    if (i < n1) {
      const int j = (int)(i / kMlpXPad), f = (int)(i % kMlpXPad);
      const bool in = j < hd && f < 2 * kHeadDim;
      P.mlp_w1t[i] = in ? P.mlp_w1[(int64_t)f * hd + j] : (uint16_t)0;
      if (P.mlp_kind == 1) P.mlp_wgt[i] = in ? P.mlp_wg[(int64_t)f * hd + j] : (uint16_t)0;
    } else if (i < n1 + n2) {
      const int64_t k = i - n1;
      const int ce = mlp_w2_chunk_elems(P.R);                 // (a chunk's rows, then padding up to whole KB)
      const int c = (int)(k / ce), rem = (int)(k % ce), rc = rem / kMlpW2Pad, jj = rem % kMlpW2Pad;
      const int j = c * kMlpChunk + jj;
      P.mlp_w2t[k] = (rc < P.R && jj < kMlpChunk && j < hd) ? P.mlp_w2[(int64_t)j * P.R + rc] : (uint16_t)0;
    } else {
      const int j = (int)(i - n1 - n2);
      P.mlp_b1p[j] = j < hd ? P.mlp_b1[j] : 0.f;
    }
  }
}

// erf with one code path: sign(x) (1 - 2^(t P(t))), t = min(|x|, 4), where t P(t) approximates log2(erfc(t)) on
// [0, 4] (beyond, erfc < 2e-8).  Absolute error <= 1e-7 (dominated by the rounding of 1 - 2^q), which is all the GeLU
// below needs: the factor 1 + erf is of order one wherever its error matters.  The coefficients come from the
// weighted least-squares fit in fit_erf_coefficients.py beside this file.  About a third of the instructions of the
// two-branch library routine, and no divergence.
__device__ inline float erf_1b(float x) {
  const float t = fminf(fabsf(x), 4.0f);
  float p = 1.160530155e-05f;
  p = fmaf(p, t, -1.529687725e-04f);
  p = fmaf(p, t, 8.482503472e-04f);
  p = fmaf(p, t, -2.274815692e-03f);
  p = fmaf(p, t, 8.483727288e-05f);
  p = fmaf(p, t, 2.772445790e-02f);
  p = fmaf(p, t, -1.483079046e-01f);
  p = fmaf(p, t, -9.184429049e-01f);
  p = fmaf(p, t, -1.627907276e+00f);
  return copysignf(1.0f - __builtin_amdgcn_exp2f(p * t), x);
}
__device__ inline float gelu_erf(float u) { return 0.5f * u * (1.0f + erf_1b(u * 0.70710678118654752f)); }
__device__ inline float silu(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * g)); }

template <int R, bool GATED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(R <= 64 ? 4 : 3))) void k_project_mlp(CompressParams P) {
  constexpr int NB = R / 16;
  extern __shared__ uint16_t mlds[];
  uint16_t* w1s = mlds;                                        // [kMlpChunk][kMlpXPad]
  uint16_t* wgs = w1s + kMlpChunk * kMlpXPad;                  // (GATED)
  uint16_t* w2s = wgs + (GATED ? kMlpChunk * kMlpXPad : 0);    // [R][kMlpW2Pad]
  const int b = blockIdx.y;
  const int lb = P.len_before[b];
  const int n_new = P.cu_new[b + 1] - P.cu_new[b];
  const int la = lb + n_new;
  const int lp = lb / kPage + blockIdx.x;
  if (n_new <= 0 || lp * kPage >= la) return;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 15, lg = l >> 4;
  const int pos = lp * kPage + ln;
  const bool tok_ok = pos >= lb && pos < la;
  const int64_t n = P.cu_new[b] + (tok_ok ? pos - lb : 0);
  const bool is_ref = (pos % P.stride) == 0;
  int page = P.block_tables[(int64_t)b * P.bt_stride + min(lp, P.bt_stride - 1)];
  page = clampi(page, 0, (int)P.n_pages_pool - 1);
  const int32_t* rtab = P.ref_tables + (int64_t)b * P.rt_stride;
  const int n_chunks = P.mlp_hidden_pad / kMlpChunk;
  {
    const int h0 = blockIdx.z * 4;
    const bool head_ok = h0 + w < P.Hkv;
    const int h = min(h0 + w, P.Hkv - 1);
    const int o = P.ord_all[n * P.Hkv + h];
    const int oe = kKeyIdxMask - (int)(P.exact_key_all[n * P.Hkv + h] & kKeyIdxMask);
    const int ord = clampi(o < 0 ? oe : o, 0, P.rt_stride - 1);
    const int slot = clampi(rtab[ord], 0, (int)P.n_ref_slots - 1);
    const uint16_t* kr = P.k_new + (n * P.Hkv + h) * kHeadDim;
    const uint16_t* vr = P.v_new + (n * P.Hkv + h) * kHeadDim;
    const uint16_t* rk = P.ref + (int64_t)h * P.ref_head_stride + (int64_t)slot * kHeadDim;
    const uint16_t* rv = rk + P.ref_kv_stride;
    // operand rows: contraction step kk covers features 32 kk .. 32 kk + 31 of K||V, the lane its 8-wide chunk lg
    bf16x8 xt[8], xr[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int off = (4 * (kk & 3) + lg) * 8;
      xt[kk] = *reinterpret_cast<const bf16x8*>((kk < 4 ? kr : vr) + off);
      xr[kk] = *reinterpret_cast<const bf16x8*>((kk < 4 ? rk : rv) + off);
    }
    float4v zacc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) zacc[nb] = float4v{0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < n_chunks; ++c) {
      __syncthreads();                       // the previous chunk has been consumed
      // The chunk's weights are contiguous in the packed buffers, in the LDS layout: direct-to-LDS copies of 1 KB per
      // wave instruction (lane l brings 16 bytes to base + 16 l), all issued before any is waited for.
      {
        constexpr int kW1Kb = kMlpChunk * kMlpXPad * 2 / 1024, kW2Kb = mlp_w2_chunk_elems(R) * 2 / 1024;
        static_assert(kMlpChunk * kMlpXPad * 2 % 1024 == 0, "whole wave copies");
        const uint16_t* s1 = P.mlp_w1t + (int64_t)c * kMlpChunk * kMlpXPad;
        const uint16_t* sg = P.mlp_wgt + (int64_t)c * kMlpChunk * kMlpXPad;
        const uint16_t* s2 = P.mlp_w2t + (int64_t)c * mlp_w2_chunk_elems(R);
        const int wu = __builtin_amdgcn_readfirstlane(w);
#pragma unroll
        for (int k = 0; k < (kW1Kb + 3) / 4; ++k) {
          const int kb = 4 * k + wu;
          if (kb < kW1Kb) {
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(s1 + kb * 512 + l * 8),
                                             (void __attribute__((address_space(3)))*)(w1s + kb * 512), 16, 0, 0);
            if constexpr (GATED)
              __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(sg + kb * 512 + l * 8),
                                               (void __attribute__((address_space(3)))*)(wgs + kb * 512), 16, 0, 0);
          }
        }
#pragma unroll
        for (int k = 0; k < (kW2Kb + 3) / 4; ++k) {
          const int kb = 4 * k + wu;
          if (kb < kW2Kb)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(s2 + kb * 512 + l * 8),
                                             (void __attribute__((address_space(3)))*)(w2s + kb * 512), 16, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0);       // this wave's copies have landed before it signals the barrier
      }
      __syncthreads();
#pragma unroll 1
      for (int jb = 0; jb < kMlpChunk / 16; ++jb) {
        float4v ht = {0.f, 0.f, 0.f, 0.f}, hr = ht, gt = ht, gr = ht;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(w1s + (jb * 16 + ln) * kMlpXPad + (4 * kk + lg) * 8);
          ht = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, xt[kk], ht, 0, 0, 0);
          hr = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, xr[kk], hr, 0, 0, 0);
          if constexpr (GATED) {
            const bf16x8 ag = *reinterpret_cast<const bf16x8*>(wgs + (jb * 16 + ln) * kMlpXPad + (4 * kk + lg) * 8);
            gt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag, xt[kk], gt, 0, 0, 0);
            gr = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag, xr[kk], gr, 0, 0, 0);
          }
        }
        // the lane holds hidden columns 16 jb + 4 lg + i (i = 0..3) of token ln: bias, activation, difference
        const float4 bias = *reinterpret_cast<const float4*>(P.mlp_b1p + c * kMlpChunk + jb * 16 + 4 * lg);
        const float bi[4] = {bias.x, bias.y, bias.z, bias.w};
        float d[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float ut = ht[i] + bi[i], ur = hr[i] + bi[i];
          d[i] = GATED ? silu(gt[i]) * ut - silu(gr[i]) * ur : gelu_erf(ut) - gelu_erf(ur);
        }
        const uint32_t hi0 = pack_bf16(d[0], d[1]), hi1 = pack_bf16(d[2], d[3]);
        const uint32_t lo0 = pack_bf16(d[0] - bf16lo(hi0), d[1] - bf16hi(hi0));
        const uint32_t lo1 = pack_bf16(d[2] - bf16lo(hi1), d[3] - bf16hi(hi1));
        const short4v dhi = __builtin_bit_cast(short4v, make_uint2(hi0, hi1));
        const short4v dlo = __builtin_bit_cast(short4v, make_uint2(lo0, lo1));
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const short4v a2 = *reinterpret_cast<const short4v*>(w2s + (nb * 16 + ln) * kMlpW2Pad + jb * 16 + 4 * lg);
          zacc[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a2, dhi, zacc[nb], 0, 0, 0);
          zacc[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a2, dlo, zacc[nb], 0, 0, 0);
        }
      }
    }
    if (head_ok && tok_ok) {
      uint16_t* lat = P.latent + (int64_t)page * P.latent_page_stride + (int64_t)h * P.latent_head_stride;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int cc = nb * 16 + 4 * lg;
        uint2 ov;
        ov.x = is_ref ? 0u : pack_bf16(zacc[nb][0], zacc[nb][1]);
        ov.y = is_ref ? 0u : pack_bf16(zacc[nb][2], zacc[nb][3]);
        *reinterpret_cast<uint2*>(lat + ((cc >> 3) * kPage + ln) * 8 + (cc & 7)) = ov;
      }
      if (lg == 0) P.idx[(int64_t)page * P.idx_page_stride + (int64_t)h * P.idx_head_stride + ln] = ord;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Decode append: every sequence of the call brings exactly one new token.  Two kernels instead of five (the
// step is bound by launch latency: a few microseconds of work per kernel).
//   append_scan   grid (NS, Hkv, B), 256 threads: block (s, h, b) scores its share of the token's candidate
//                 references in fp32 (16 lanes per reference, 16 references per block step) and writes its
//                 (best, second, arg best, |token|^2); if the token is itself a reference, block s = 0 admits it.
//   append_finish grid (Hkv, B), 256 threads: merges the NS partial results; re-scores every candidate in fp64 if
//                 the two best are too close to call (same band as resolve); forms the residual against the chosen
//                 raw reference, projects it (fp32 FMAs) and writes latent + ordinal.
// ------------------------------------------------------------------------------------------------
__device__ inline float group16_sum(float v) {   // sum over the 16 lanes that share lane/16
  v += __shfl_xor(v, 1);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 8);
  return v;
}
__device__ inline double group16_sum(double v) {
  v += __shfl_xor(v, 1);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 8);
  return v;
}
__device__ inline void unpack8(const uint4& c, float (&o)[8]) {
  o[0] = bf16lo(c.x); o[1] = bf16hi(c.x); o[2] = bf16lo(c.y); o[3] = bf16hi(c.y);
  o[4] = bf16lo(c.z); o[5] = bf16hi(c.z); o[6] = bf16lo(c.w); o[7] = bf16hi(c.w);
}

__global__ __launch_bounds__(256) void k_append_scan(CompressParams P) {
  const int s = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, sub = l & 15, lg = l >> 4;
  const int pos = P.len_before[b];
  const int64_t n = P.cu_new[b];
  const uint16_t* kr = P.k_new + (n * P.Hkv + h) * kHeadDim;
  const uint16_t* vr = P.v_new + (n * P.Hkv + h) * kHeadDim;
  const int32_t* rtab = P.ref_tables + (int64_t)b * P.rt_stride;
  if (pos % P.stride == 0) {          // the new token is a reference: raw copy + inverse norm (first wave of split 0)
    if (s != 0 || w != 0) return;
    const int ord = pos / P.stride;
    if (ord >= P.rt_stride) return;
    const int slot = clampi(rtab[ord], 0, (int)P.n_ref_slots - 1);
    const uint32_t kx = reinterpret_cast<const uint32_t*>(kr)[l], vx = reinterpret_cast<const uint32_t*>(vr)[l];
    uint16_t* rk = P.ref + (int64_t)h * P.ref_head_stride + (int64_t)slot * kHeadDim;
    reinterpret_cast<uint32_t*>(rk)[l] = kx;
    reinterpret_cast<uint32_t*>(rk + P.ref_kv_stride)[l] = vx;
    const float ss = bf16lo(kx) * bf16lo(kx) + bf16hi(kx) * bf16hi(kx) + bf16lo(vx) * bf16lo(vx) + bf16hi(vx) * bf16hi(vx);
    const double dd = (double)bf16lo(kx) * bf16lo(kx) + (double)bf16hi(kx) * bf16hi(kx) + (double)bf16lo(vx) * bf16lo(vx) +
                      (double)bf16hi(vx) * bf16hi(vx);
    const float term = ref_term(ss, dd, P.metric);
    if (l == 0) P.ref_inv_norm[(int64_t)h * P.ref_norm_head_stride + slot] = term;
    return;
  }
  // the token's K||V chunk of this lane: dims 8*sub..8*sub+7 of K and of V
  float ak[8], av[8];
  unpack8(*reinterpret_cast<const uint4*>(kr + sub * 8), ak);
  unpack8(*reinterpret_cast<const uint4*>(vr + sub * 8), av);
  float na2 = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) na2 += ak[e] * ak[e] + av[e] * av[e];
  na2 = group16_sum(na2);
  const int n_cand = min(refs_below(pos, P.stride), P.rt_stride);
  const int per = ceil_div(ceil_div(n_cand, P.NS), 16) * 16;       // candidates per split, whole block steps
  const int j0 = s * per, j1 = min(n_cand, j0 + per);
  const uint16_t* kbase = P.ref + (int64_t)h * P.ref_head_stride;
  const float* inorm = P.ref_inv_norm + (int64_t)h * P.ref_norm_head_stride;
  Top2 t2 = {-INFINITY, -INFINITY, -1};
  constexpr int UN = 4;                                              // block steps of 16 references in flight
  for (int jb = j0; jb < j1; jb += 16 * UN) {
    int slot[UN];
    uint4 ck[UN], cv[UN];
    float inv[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = jb + u * 16 + w * 4 + lg;
      slot[u] = rtab[min(j, n_cand - 1)];
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int sl = clampi(slot[u], 0, (int)P.n_ref_slots - 1);
      ck[u] = *reinterpret_cast<const uint4*>(kbase + (int64_t)sl * kHeadDim + sub * 8);
      cv[u] = *reinterpret_cast<const uint4*>(kbase + P.ref_kv_stride + (int64_t)sl * kHeadDim + sub * 8);
      inv[u] = inorm[sl];
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int j = jb + u * 16 + w * 4 + lg;
      float bk[8], bv[8];
      unpack8(ck[u], bk);
      unpack8(cv[u], bv);
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d += ak[e] * bk[e];
#pragma unroll
      for (int e = 0; e < 8; ++e) d += av[e] * bv[e];
      d = P.metric ? group16_sum(d) - inv[u] : group16_sum(d) * inv[u];
      if (j < j1) top2_push(t2, d, j);          // ascending j within a lane group: strict '>' keeps the lowest
    }
  }
  // merge the four lane groups of the wave, then the four waves
#pragma unroll
  for (int o = 16; o < 64; o <<= 1) {
    const float ob = __shfl_xor(t2.best, o), os = __shfl_xor(t2.second, o);
    const int oi = __shfl_xor(t2.idx, o);
    top2_merge(t2, ob, os, oi);
  }
  __shared__ float sb[4], ss2[4];
  __shared__ int si[4];
  if (l == 0) { sb[w] = t2.best; ss2[w] = t2.second; si[w] = t2.idx; }
  __syncthreads();
  if (tid == 0) {
    for (int ww = 1; ww < 4; ++ww) top2_merge(t2, sb[ww], ss2[ww], si[ww]);
    reinterpret_cast<float4*>(P.part)[(n * P.Hkv + h) * P.NS + s] =
        make_float4(t2.best, t2.second, __int_as_float(t2.idx), na2);
  }
}

template <int R>
__global__ __launch_bounds__(256) void k_append_finish(CompressParams P) {
  const int h = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, sub = l & 15, lg = l >> 4;
  const int pos = P.len_before[b];
  const int64_t n = P.cu_new[b];
  const uint16_t* kr = P.k_new + (n * P.Hkv + h) * kHeadDim;
  const uint16_t* vr = P.v_new + (n * P.Hkv + h) * kHeadDim;
  const int32_t* rtab = P.ref_tables + (int64_t)b * P.rt_stride;
  const bool is_ref = pos % P.stride == 0;
  __shared__ int ord_s;
  __shared__ double ebest[4];
  __shared__ int eidx[4];
  __shared__ float resid[2][kHeadDim];
  __shared__ float zpart[2][256];
  __shared__ float zfin[256];           // 4-bit latents: the token's final latent(s)
  __shared__ uint32_t qcode[256];
  // projection: thread (stream, part, c) sums its share of the 128 dims; R <= 128, 256 threads.  Its W_down column
  // does not depend on the retrieval, so all of its loads are issued here, under the latency of everything below.
  constexpr int PARTS = 128 / R >= 1 ? 128 / R : 1;        // threads per (stream, c): 128 / R, at least 1
  constexpr int DP = kHeadDim / PARTS;
  const int pst = tid / 128, prem = tid % 128, pc = prem % R, ppart = prem / R;
  uint16_t wcol[DP];
  {
    const uint16_t* wd = (pst ? P.w_down_v : P.w_down_k) + pc;
#pragma unroll
    for (int i = 0; i < DP; ++i) wcol[i] = wd[(int64_t)(min(ppart, PARTS - 1) * DP + i) * R];
  }
  if (is_ref) {
    if (tid == 0) ord_s = pos / P.stride;
  } else {
    // merge the partial results (ascending ranges; every thread does the same few loads)
    float bb = -INFINITY, b2 = -INFINITY, na2 = 0.f;
    int bi = -1;
    const float4* pp = reinterpret_cast<const float4*>(P.part) + (n * P.Hkv + h) * P.NS;
    for (int s = 0; s < P.NS; ++s) {
      const float4 o = pp[s];
      na2 = o.w;
      const int oi = __float_as_int(o.z);
      if (oi < 0) continue;
      if (o.x > bb) { b2 = fmaxf(bb, o.y); bb = o.x; bi = oi; }
      else b2 = fmaxf(b2, o.x);
    }
    if (bi >= 0 && gap_is_safe(bb, b2, na2, P.metric)) {
      if (tid == 0) ord_s = bi;
    } else {
      // too close to call in fp32: every candidate again in fp64, cos = a.b / (|a| |b|) or -|a - b|^2, lowest
      // ordinal on ties
      float akf[8], avf[8];
      unpack8(*reinterpret_cast<const uint4*>(kr + sub * 8), akf);
      unpack8(*reinterpret_cast<const uint4*>(vr + sub * 8), avf);
      double na = 0.0;
#pragma unroll
      for (int e = 0; e < 8; ++e) na += (double)akf[e] * akf[e] + (double)avf[e] * avf[e];
      const double na2d = group16_sum(na);
      na = sqrt(na2d);
      const int n_cand = min(refs_below(pos, P.stride), P.rt_stride);
      const uint16_t* kbase = P.ref + (int64_t)h * P.ref_head_stride;
      double best = -INFINITY;
      int besti = 0x7fffffff;
      for (int jb = 0; jb < n_cand; jb += 16) {
        const int j = jb + w * 4 + lg;
        const int sl = clampi(rtab[min(j, n_cand - 1)], 0, (int)P.n_ref_slots - 1);
        float bk[8], bv[8];
        unpack8(*reinterpret_cast<const uint4*>(kbase + (int64_t)sl * kHeadDim + sub * 8), bk);
        unpack8(*reinterpret_cast<const uint4*>(kbase + P.ref_kv_stride + (int64_t)sl * kHeadDim + sub * 8), bv);
        double d = 0.0, nb = 0.0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          d += (double)akf[e] * bk[e] + (double)avf[e] * bv[e];
          nb += (double)bk[e] * bk[e] + (double)bv[e] * bv[e];
        }
        d = group16_sum(d);
        const double nb2 = group16_sum(nb);
        nb = sqrt(nb2);
        const double den = na * nb;
        const double c = P.metric ? -fmax(na2d - 2.0 * d + nb2, 0.0) : (den > 0.0 ? d / den : 0.0);
        if (j < n_cand && (c > best || (c == best && j < besti))) { best = c; besti = j; }
      }
#pragma unroll
      for (int o = 16; o < 64; o <<= 1) {
        const double ob = __shfl_xor(best, o);
        const int oi = __shfl_xor(besti, o);
        if (ob > best || (ob == best && oi < besti)) { best = ob; besti = oi; }
      }
      if (l == 0) { ebest[w] = best; eidx[w] = besti; }
      __syncthreads();
      if (tid == 0) {
        for (int ww = 1; ww < 4; ++ww)
          if (ebest[ww] > best || (ebest[ww] == best && eidx[ww] < besti)) { best = ebest[ww]; besti = eidx[ww]; }
        ord_s = besti == 0x7fffffff ? 0 : besti;
      }
    }
  }
  __syncthreads();
  const int ord = clampi(ord_s, 0, P.rt_stride - 1);
  // residual against the chosen raw reference (fp32: exact for bf16 inputs); zero for a reference token
  if (tid < kHeadDim) {
    const int slot = clampi(rtab[ord], 0, (int)P.n_ref_slots - 1);
    const uint16_t* rk = P.ref + (int64_t)h * P.ref_head_stride + (int64_t)slot * kHeadDim;
    const float rkv = __uint_as_float((uint32_t)rk[tid] << 16), rvv = __uint_as_float((uint32_t)rk[P.ref_kv_stride + tid] << 16);
    const float kx = __uint_as_float((uint32_t)kr[tid] << 16), vx = __uint_as_float((uint32_t)vr[tid] << 16);
    resid[0][tid] = is_ref ? 0.f : kx - rkv;
    resid[1][tid] = is_ref ? 0.f : vx - rvv;
  }
  __syncthreads();
  {
    float z = 0.f;
    if (ppart < PARTS) {
#pragma unroll
      for (int i = 0; i < DP; ++i) z += resid[pst][ppart * DP + i] * __uint_as_float((uint32_t)wcol[i] << 16);
    }
    zpart[pst][prem] = z;
  }
  __syncthreads();
  const int tok = pos % kPage;
  const int lp = pos / kPage;
  const int page = clampi(P.block_tables[(int64_t)b * P.bt_stride + min(lp, P.bt_stride - 1)], 0, (int)P.n_pages_pool - 1);
  uint16_t* lat = P.latent + (int64_t)page * P.latent_page_stride + (int64_t)h * P.latent_head_stride;
  if (tid < 2 * R) {
    const int st = tid / R, c = tid % R;
    float z = 0.f;
#pragma unroll
    for (int pt = 0; pt < PARTS; ++pt) z += zpart[st][pt * R + c];
    if (P.joint) {
      if (st == 0) {
        float zv = 0.f;
#pragma unroll
        for (int pt = 0; pt < PARTS; ++pt) zv += zpart[1][pt * R + c];
        if (P.q4) zfin[c] = z + zv;
        else lat[((c >> 3) * kPage + tok) * 8 + (c & 7)] = (uint16_t)f32_to_bf16_bits(z + zv);
      }
    } else if (P.q4) {
      zfin[st * 128 + c] = z;
    } else if (st == 0) {
      lat[((c >> 3) * kPage + tok) * 8 + (c & 7)] = (uint16_t)f32_to_bf16_bits(z);
    } else {
      lat[P.latent_stream_stride + ((c >> 4) * 64 + (tok >> 2) * 16 + (c & 15)) * 4 + (tok & 3)] = (uint16_t)f32_to_bf16_bits(z);
    }
  }
  if (P.q4) {                 // 4-bit record of the token (single stream): codes of value c by thread c
    __syncthreads();
    float mn = INFINITY, mx = -INFINITY;
    for (int c = 0; c < R; ++c) { mn = fminf(mn, zfin[c]); mx = fmaxf(mx, zfin[c]); }
    const Q4Params qp = q4_params(mn, mx);
    if (tid < R) qcode[tid] = q4_code(zfin[tid], qp);
    __syncthreads();
    char* blk = reinterpret_cast<char*>(lat);
    if (tid < R / 8) {
      uint32_t wd = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) wd |= qcode[tid * 8 + e] << (4 * (e >> 1) + 16 * (e & 1));
      *reinterpret_cast<uint32_t*>(blk + 4 * (tid * kPage + tok)) = wd;
    }
    if (tid == 0) {
      uint16_t* sz = reinterpret_cast<uint16_t*>(blk + 8 * R + (tok >> 2) * 16 + (tok & 3) * 2);
      sz[0] = (uint16_t)qp.scale_bits;
      sz[4] = (uint16_t)qp.zero_bits;
    }
    if (!P.joint) {           // value stream: columns c, c+16, c+32, c+48 of the token share a dword with one neighbour token
      float mnv = INFINITY, mxv = -INFINITY;
      for (int c = 0; c < R; ++c) { mnv = fminf(mnv, zfin[128 + c]); mxv = fmaxf(mxv, zfin[128 + c]); }
      const Q4Params qv = q4_params(mnv, mxv);
      if (tid < R) qcode[128 + tid] = q4_code(zfin[128 + tid], qv);
      __syncthreads();
      char* vblk = blk + P.latent_stream_stride * 2;
      if (tid < R / 4) {
        const int q = tid >> 4, c15 = tid & 15;
        uint32_t nib = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) nib |= qcode[128 + 64 * q + 16 * j + c15] << (4 * j);
        uint32_t* dst = reinterpret_cast<uint32_t*>(vblk + (q * 64 + (tok >> 2) * 16 + c15) * 8) + ((tok & 3) >> 1);
        const int sh = 16 * (tok & 1);
        *dst = (*dst & ~(0xffffu << sh)) | (nib << sh);
      }
      if (tid == 0) {
        uint16_t* sz = reinterpret_cast<uint16_t*>(vblk + 8 * R + (tok >> 2) * 16 + (tok & 3) * 2);
        sz[0] = (uint16_t)qv.scale_bits;
        sz[4] = (uint16_t)qv.zero_bits;
      }
    }
  }
  if (tid == 0) P.idx[(int64_t)page * P.idx_page_stride + (int64_t)h * P.idx_head_stride + tok] = ord;
}

// ------------------------------------------------------------------------------------------------
// host launcher
// ------------------------------------------------------------------------------------------------
template <int TB, bool L2M, int NW, bool EXC = false>
static hipError_t launch_sim_m(const CompressParams& P, dim3 grid, hipStream_t st) {
  if constexpr (!EXC) {
    if (P.round > 0) return launch_sim_m<TB, L2M, NW, true>(P, grid, st);
  }
  const size_t lds = 3 * kNT * 256 * 2 + 3 * kNT * 4;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_sim_top2<TB, L2M, NW, EXC>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return note_hip_error(e, "hipFuncSetAttribute(similarity kernel LDS)");
    attr_set = true;
  }
  hipLaunchKernelGGL((k_sim_top2<TB, L2M, NW, EXC>), grid, dim3(NW * 64), lds, st, P);
  return note_hip_error(hipGetLastError(), "launch of sim_top2");
}
template <int TB>
static hipError_t launch_sim(const CompressParams& P, int nw, dim3 grid, hipStream_t st) {
  if constexpr (TB <= 3) {
    if (nw == 8) return P.metric ? launch_sim_m<TB, true, 8>(P, grid, st) : launch_sim_m<TB, false, 8>(P, grid, st);
  }
  return P.metric ? launch_sim_m<TB, true, 4>(P, grid, st) : launch_sim_m<TB, false, 4>(P, grid, st);
}

template <int R, int KS = 1>
static hipError_t launch_project(const CompressParams& P, dim3 grid, hipStream_t st) {
  if constexpr (KS == 1) {
    if (P.top_k > 1) return launch_project<R, 4>(P, grid, st);
  }
  const size_t lds = 2 * R * kWPad * 2;
  static bool attr_set = false;
  if (!attr_set && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_project<R, KS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return note_hip_error(e, "hipFuncSetAttribute(projection kernel LDS)");
    attr_set = true;
  }
  hipLaunchKernelGGL((k_project<R, KS>), grid, dim3(256), lds, st, P);
  return note_hip_error(hipGetLastError(), "launch of project");
}

template <int R, bool GATED>
static hipError_t launch_project_mlp_g(const CompressParams& P, dim3 grid, hipStream_t st) {
  const size_t lds = ((GATED ? 2 : 1) * kMlpChunk * kMlpXPad + mlp_w2_chunk_elems(R)) * 2;
  static bool attr_set = false;
  if (!attr_set && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_project_mlp<R, GATED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return note_hip_error(e, "hipFuncSetAttribute(non-linear projection kernel LDS)");
    attr_set = true;
  }
  hipLaunchKernelGGL((k_project_mlp<R, GATED>), grid, dim3(256), lds, st, P);
  return note_hip_error(hipGetLastError(), "launch of project_mlp");
}
template <int R>
static hipError_t launch_project_mlp(const CompressParams& P, dim3 grid, hipStream_t st) {
  return P.mlp_kind == 1 ? launch_project_mlp_g<R, true>(P, grid, st) : launch_project_mlp_g<R, false>(P, grid, st);
}

int sim_tile_rows(int rb, int nw) { return (nw == 8 && rb <= 3 ? 8 : 4) * 16 * rb; }

hipError_t launch_compress(const CompressParams& P0, const CompressWs& cw, char* ws, int rb, int nw, int tiles_max,
                           int page_tiles_max, int max_new_refs, hipStream_t st) {
  hipError_t e;
  CompressParams P = P0;
  const int items = P.n_new_total * P.Hkv;
  timing_mark(-1, st);
  hipLaunchKernelGGL(k_admit_refs, dim3(ceil_div(max_new_refs * P.Hkv, 4) > 0 ? ceil_div(max_new_refs * P.Hkv, 4) : 1, P.batch),
                     dim3(256), 0, st, P);
  if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of admit_refs");
  timing_mark(K_ADMIT, st);
  dim3 gs(P.batch * P.Hkv, P.NS, tiles_max);
  // one retrieval round per reference rank (a single round unless top_k > 1): similarity search that leaves out
  // what earlier rounds took, merge of the reference-range splits, exact pass for the near-ties of the round
  for (int round = 0; round < P.top_k; ++round) {
    P.round = round;
    P.ord = reinterpret_cast<int32_t*>(ws + cw.ord + round * cw.ord_round);
    P.flag_count = reinterpret_cast<int32_t*>(ws + cw.flag_count + round * cw.flag_count_round);
    P.flag_list = reinterpret_cast<int32_t*>(ws + cw.flag_list + round * cw.flag_list_round);
    P.exact_key = reinterpret_cast<uint64_t*>(ws + cw.exact_key + round * cw.exact_key_round);
    switch (rb) {
      case 1: e = launch_sim<1>(P, nw, gs, st); break;
      case 2: e = launch_sim<2>(P, nw, gs, st); break;
      case 3: e = launch_sim<3>(P, nw, gs, st); break;
      case 4: e = launch_sim<4>(P, nw, gs, st); break;
      default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    timing_mark(K_SIM, st);
    if (P.NS > 1) {           // with one reference-range split the similarity kernel has decided already
      hipLaunchKernelGGL(k_resolve, dim3(ceil_div(items, 256)), dim3(256), 0, st, P);
      if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of resolve");
      timing_mark(K_RESOLVE, st);
    }
    hipLaunchKernelGGL(k_exact, dim3(kExactX, kExactSplits, P.batch * P.Hkv), dim3(256), 0, st, P);
    if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of exact");
    timing_mark(K_EXACT, st);
  }
  if (P.mlp_kind >= 0) {
    hipLaunchKernelGGL(k_mlp_prep, dim3(256), dim3(256), 0, st, P);
    if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of mlp_prep");
    dim3 gm(page_tiles_max, P.batch, ceil_div(P.Hkv, 4));
    e = hipErrorInvalidValue;
    switch (P.R) {
      case 16: e = launch_project_mlp<16>(P, gm, st); break;
      case 32: e = launch_project_mlp<32>(P, gm, st); break;
      case 48: e = launch_project_mlp<48>(P, gm, st); break;
      case 64: e = launch_project_mlp<64>(P, gm, st); break;
      case 80: e = launch_project_mlp<80>(P, gm, st); break;
      case 96: e = launch_project_mlp<96>(P, gm, st); break;
      case 112: e = launch_project_mlp<112>(P, gm, st); break;
      case 128: e = launch_project_mlp<128>(P, gm, st); break;
    }
    timing_mark(K_PROJECT, st);
    return e;
  }
  dim3 gp(ceil_div(page_tiles_max, P.proj_ppb), P.batch);
  e = hipErrorInvalidValue;
  switch (P.R) {
    case 16: e = launch_project<16>(P, gp, st); break;
    case 32: e = launch_project<32>(P, gp, st); break;
    case 48: e = launch_project<48>(P, gp, st); break;
    case 64: e = launch_project<64>(P, gp, st); break;
    case 80: e = launch_project<80>(P, gp, st); break;
    case 96: e = launch_project<96>(P, gp, st); break;
    case 112: e = launch_project<112>(P, gp, st); break;
    case 128: e = launch_project<128>(P, gp, st); break;
  }
  timing_mark(K_PROJECT, st);
  return e;
}

template <int R>
static void launch_append_finish(const CompressParams& P, hipStream_t st) {
  hipLaunchKernelGGL((k_append_finish<R>), dim3(P.Hkv, P.batch), dim3(256), 0, st, P);
}

hipError_t launch_append(const CompressParams& P, hipStream_t st) {
  hipError_t e;
  timing_mark(-1, st);
  hipLaunchKernelGGL(k_append_scan, dim3(P.NS, P.Hkv, P.batch), dim3(256), 0, st, P);
  if ((e = hipGetLastError()) != hipSuccess) return note_hip_error(e, "launch of append_scan");
  timing_mark(K_SIM, st);
  switch (P.R) {
    case 16: launch_append_finish<16>(P, st); break;
    case 32: launch_append_finish<32>(P, st); break;
    case 48: launch_append_finish<48>(P, st); break;
    case 64: launch_append_finish<64>(P, st); break;
    case 80: launch_append_finish<80>(P, st); break;
    case 96: launch_append_finish<96>(P, st); break;
    case 112: launch_append_finish<112>(P, st); break;
    case 128: launch_append_finish<128>(P, st); break;
    default: return hipErrorInvalidValue;
  }
  e = note_hip_error(hipGetLastError(), "launch of append_finish");
  timing_mark(K_PROJECT, st);
  return e;
}

}  // namespace dkv
