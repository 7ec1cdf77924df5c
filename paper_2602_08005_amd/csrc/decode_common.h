// Device helpers shared by the decode kernels: sequence / selection arithmetic and the fixed-point units of the
// per-reference weight table (the streaming kernel writes the table, ref_values reads it back).
#pragma once
#include "common.h"
#include "launch.h"

#include <type_traits>

namespace dkv {

typedef uint32_t uint4v __attribute__((ext_vector_type(4)));   // operand types of the non-temporal load builtin
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

__device__ inline int seq_len_of(const DecodeParams& P, int b) {
  return clampi(P.seq_lens[b], 0, P.max_seq_len);
}
// Entries of the page list the blocks of sequence b iterate over: all pages of the sequence, or (subset attention:
// section 4.2, only the tokens the sparse attention mask asks for are reconstructed) its selected pages.
__device__ inline int work_pages_of(const DecodeParams& P, int b, int L) {
  const int n_pages = ceil_div(L, kPage);
  if (!P.sel_pages) return n_pages;
  return clampi(P.n_sel[b], 0, min(P.sel_stride, n_pages));
}
// Logical page of list entry `pos` of sequence b (L > 0), clamped into the sequence.
__device__ inline int work_page(const DecodeParams& P, int b, int L, int pos) {
  if (!P.sel_pages) return pos;
  return clampi(P.sel_pages[(int64_t)b * P.sel_stride + pos], 0, ceil_div(L, kPage) - 1);
}
// Ordinals that list entries [0, p1) of the sequence can point at (p1 >= 1).
__device__ inline int refs_covered(const DecodeParams& P, int b, int L, int p1) {
  return refs_below(min(L, (work_page(P, b, L, p1 - 1) + 1) * kPage), P.stride);
}

// The per-reference weight table is kept in 32-bit fixed point, because the LDS executes integer atomics at
// full rate while a float atomic add costs about three cycles per active lane on this chip.  A token that
// points at reference j with latent logit part delta has weight p = 2^(delta + s_j), s_j = S_ref[j] - m_ref - bias
// being a constant of the reference (and query head).  Entry (j, g) accumulates p * 2^k_j with the integer
// k_j = table_shift(...) within one of kFixQ - s_j, i.e. values near 2^(delta + kFixQ): the reference's own token
// (delta = 0) contributes about 2^kFixQ, so each addend is rounded to 2^-kFixQ of that token's weight whatever
// the dynamic range of the softmax.  ref_values multiplies the sums back by 2^-k_j.  An entry that wraps, or a
// weight too large for an entry (2^11 times its reference token's), is rare: such amounts go, as plain weights,
// to a small per-block list; a block whose list is not empty converts its whole table to plain weights before
// it flushes and marks the split, so that ref_values does not scale it again.
constexpr int kFixQ = 20;
constexpr int kOvfCap = 256;
// Entry (j, g) is kept in units of 2^-table_shift(S_ref[j][g], base(m_ref[g])): an integer within one of
// kFixQ - s_j.  Both kernels evaluate exactly these two expressions, so they agree bit for bit.
__device__ inline float table_shift_base(float mref, float bias) { return mref + (bias + (float)kFixQ); }
// (base - sref >= bias + kFixQ; the conversion saturates and the scaling by a power of two takes any exponent, so
// no clamp is needed: an absurdly distant score just turns its weights into overflow-list records or zeros)
__device__ inline int table_shift(float sref, float base) { return (int)(base - sref); }

__device__ inline float wave16_max(float v) {   // max over the 16 lanes that share lane/16
  v = fmaxf(v, __shfl_xor(v, 1));
  v = fmaxf(v, __shfl_xor(v, 2));
  v = fmaxf(v, __shfl_xor(v, 4));
  v = fmaxf(v, __shfl_xor(v, 8));
  return v;
}

}  // namespace dkv
