// Shared device/host declarations of the DeltaKV gfx950 kernels (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "deltakv.h"

namespace dkv {

constexpr int kWave = 64;
constexpr int kHeadDim = 128;
constexpr int kPage = 16;          // tokens per page
constexpr int kRefChunk = 256;     // reference ordinals handled by one block of the per-reference kernels
constexpr int kMaxSplits = 32;     // upper bound on token-range splits of one (sequence, kv-head)
constexpr int kWPad = 136;         // bf16 elements per staged W_down^T row (128 + 8: shifts LDS banks)
constexpr int kRawChunk = 256;     // raw-segment tokens handled by one block
constexpr int kRawMaxChunks = 16;  // a raw segment holds at most kRawChunk * kRawMaxChunks tokens per sequence
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// Softmax weights are 2^(x - m_ref - bias) with m_ref the largest per-reference score.  Attention over the whole
// cache: every reference token is itself attended with a zero latent, so the true maximum is >= m_ref, the weight
// sum is >= 2^-64 and only the room above m_ref matters: 124 log2 units (86 nats) before a sum reaches 2^60.
// Attention over a selection: the selected tokens may lie anywhere below m_ref, so the frame is centred: 80 log2
// units (55 nats) either way before the sum leaves [2^-100, 2^60).  Rows outside go to the rescue kernel.
constexpr float kExpBias = 64.0f;
constexpr float kExpBiasSubset = 20.0f;
__host__ __device__ inline float exp_bias(bool subset) { return subset ? kExpBiasSubset : kExpBias; }
constexpr float kSumLo = 0x1p-100f, kSumHi = 0x1p60f;      // sums of weights a streaming result is accepted with

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
// Query heads per kv-head padded to a power of two (4, 8 or 16): row width of the per-reference tables.
__host__ __device__ inline int padded_group(int g) { return g <= 4 ? 4 : (g <= 8 ? 8 : 16); }
__host__ __device__ inline int group_shift(int gp) { return gp == 4 ? 2 : (gp == 8 ? 3 : 4); }

// Token-range split s of a sequence with n_pages pages: pages [p0, p1).  The same arithmetic is used
// by the streaming kernel (which owns the range) and by the kernels that consume its partial results.
struct SplitPlan {
  int n_splits;   // splits actually used by this sequence (<= grid's split count)
  int per;        // pages per split
};
__host__ __device__ inline SplitPlan plan_splits(int n_pages, int max_splits, int pages_per_split) {
  SplitPlan sp;
  int want = ceil_div(n_pages, pages_per_split);
  sp.n_splits = want < 1 ? 1 : (want > max_splits ? max_splits : want);
  sp.per = ceil_div(n_pages, sp.n_splits);
  return sp;
}
// Splits of a sequence that hold at least one page (split s covers pages [s*per, (s+1)*per)).
__host__ __device__ inline int used_splits(int n_pages, int max_splits, int pages_per_split) {
  if (n_pages <= 0) return 0;
  const SplitPlan sp = plan_splits(n_pages, max_splits, pages_per_split);
  return ceil_div(n_pages, sp.per);
}
// Number of reference ordinals that tokens [0, end_tok) can point at.
__host__ __device__ inline int refs_below(int end_tok, int stride) { return ceil_div(end_tok, stride); }

// ---- decode workspace carving (host computes, kernels receive pointers) -------------------------
struct DecodeWs {
  int64_t status;   // int32[4]   bit 0: a logit left the range the biased exponent can hold
  int64_t rescue;   // int32 [B][Hq]  rows to be recomputed by the rescue kernel
  int64_t qlat;     // bf16 [2][B][Hq][R]         (W_uK q) * scale * log2(e), split into bf16 hi + lo parts
  int64_t sref;     // fp32 [B][Hkv][n_ref_max][Gp]  per-reference scores, log2 units
  int64_t cmax;     // fp32 [B][Hkv][n_chunk_max][Gp] per-chunk maxima of sref
  int64_t lpart;    // fp32 [B][Hkv][S][Gp]
  int64_t wflag;    // int32 [B][Hkv][S]             1: this split's weight table is already in plain units
  int64_t items;    // int32 [1 + B*kMaxSplits]      number of non-empty (sequence, split) items, then the items
  int64_t accpart;  // fp32 [B][Hkv][S][Gp][R]
  int64_t opart;    // fp32 [B][Hkv][n_chunk_max][Gp][128]
  int64_t wpart;    // fp32 [B][Hkv][S][tab_cap][Gp]     per-split weight tables (LDS windows)
  int64_t spill;    // fp32 [B][Hkv][n_ref_max][Gp]      weights of ordinals older than the windows (long sequences)
  int64_t rawo;     // fp32 [B][Hkv][kRawMaxChunks][Gp][128]  raw-segment partial outputs
  int64_t rawml;    // fp32 [B][Hkv][kRawMaxChunks][Gp][2]    their (largest logit, weight sum)
  int64_t total;
};
// Rows of the streaming kernel's LDS weight table on a compute unit with 160 KiB of LDS (the largest any call
// uses; the host lowers it to what the device and the variant's other buffers leave).
inline int64_t table_rows_max(int Gp) { return (160 * 1024) / (Gp * 4); }
inline DecodeWs plan_decode_ws(const deltakv_dims& d, int64_t batch, int64_t n_ref_max, int splits, int64_t tab_cap) {
  const int64_t G = d.n_q_heads / d.n_kv_heads, Gp = padded_group((int)G), R = d.rank;
  const int64_t BH = batch * d.n_kv_heads, nch = ceil_div64(n_ref_max, kRefChunk);
  DecodeWs w;
  int64_t o = 0;
  auto take = [&](int64_t bytes) { int64_t at = o; o = align_up(o + bytes, 256); return at; };
  w.status = take(16);
  w.rescue = take(batch * d.n_q_heads * 4);
  w.qlat = take(2 * batch * d.n_q_heads * R * 2);
  w.sref = take(BH * n_ref_max * Gp * 4);
  w.cmax = take(BH * nch * Gp * 4);
  w.lpart = take(BH * splits * Gp * 4);
  w.wflag = take(BH * splits * 4);
  w.items = take((1 + batch * kMaxSplits) * 4);
  w.accpart = take(BH * splits * Gp * R * 4);
  w.opart = take(BH * nch * Gp * kHeadDim * 4);
  w.wpart = take(BH * splits * tab_cap * Gp * 4);
  w.spill = take(BH * n_ref_max * Gp * 4);
  w.rawo = take(BH * kRawMaxChunks * Gp * kHeadDim * 4);
  w.rawml = take(BH * kRawMaxChunks * Gp * 2 * 4);
  w.total = o;
  return w;
}

// ---- workspace of the rotary-embedding decode call
struct RopeWs {
  int64_t tab;      // float2 [n_pages_max][64]   (cos, sin) of each page's first position
  int64_t ml;       // fp32 [B][Hkv][S][Gp][2]    running maximum (log2 units) and weight sum of a split
  int64_t acc;      // fp32 [B][Hkv][S][Gp][128 + R]  sum p V_ref, sum p z_V of a split
  int64_t total;
};
inline RopeWs plan_rope_ws(const deltakv_dims& d, int64_t batch, int64_t n_pages_max, int splits) {
  const int64_t Gp = padded_group(d.n_q_heads / d.n_kv_heads), BH = batch * d.n_kv_heads;
  RopeWs w;
  int64_t o = 0;
  auto take = [&](int64_t bytes) { int64_t at = o; o = align_up(o + bytes, 256); return at; };
  w.tab = take(n_pages_max * 64 * 8);
  w.ml = take(BH * splits * Gp * 2 * 4);
  w.acc = take(BH * splits * Gp * (kHeadDim + d.rank) * 4);
  w.total = o;
  return w;
}

// Records which HIP call failed (shown by deltakv_last_error_detail) and passes the code through.
hipError_t note_hip_error(hipError_t e, const char* what);
// Largest dynamic LDS a block may ask for on the current device, bytes.
size_t device_lds_limit();

#ifdef __HIPCC__
__device__ inline float bf16lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN stays NaN).
__device__ inline uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
// two fp32 -> packed bf16 pair (low half = lo), hardware round-to-nearest-even conversion
__device__ inline uint32_t pack_bf16(float lo, float hi) {
  const float2v v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ inline int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }
#endif

}  // namespace dkv
