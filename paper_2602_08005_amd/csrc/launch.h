// Kernel parameter blocks and host launchers shared by the C ABI file and the kernel files.
#pragma once
#include "common.h"

namespace dkv {

struct DecodeParams {
  // cache
  const uint16_t* latent;
  const int32_t* idx;
  const uint16_t* ref;
  const int32_t* block_tables;
  const int32_t* ref_tables;
  const int32_t* seq_lens;
  // subset attention (all null for the whole cache): per sequence an ascending list of logical pages that hold a
  // selected token, and per listed page the 16-bit mask of its selected tokens
  const int32_t* sel_pages;
  const int32_t* sel_masks;
  const int32_t* n_sel;
  int sel_stride;
  // raw segment (null for none): tokens kept uncompressed beside the cache (sink / recent tokens), attended
  // together with the cached ones; bf16 [batch][raw_cap][Hkv][128] each, raw_lens[b] <= raw_cap of them valid
  const uint16_t* raw_k;
  const uint16_t* raw_v;
  const int32_t* raw_lens;
  int raw_cap;
  int bt_stride, rt_stride;
  int64_t latent_page_stride, latent_head_stride, latent_stream_stride;
  int64_t idx_page_stride, idx_head_stride;
  int64_t ref_head_stride, ref_kv_stride;
  int64_t n_pages_pool, n_ref_slots;
  // weights / query / outputs
  const uint16_t* w_up_k;
  const uint16_t* w_up_v;
  const uint16_t* q;
  uint16_t* out;
  float* lse;
  // shape
  int batch, Hkv, Hq, G, Gp, R, stride, joint;
  int q4;                   // 4-bit token-wise latents
  int top_k;                // ordinal slots per token in the index pool (1, 2 or 4)
  int nt;                   // the call streams more than the last-level cache holds: non-temporal latent loads
  int ref_cpb;              // reference chunks scored per block of ref_scores (1 or 4)
  int max_seq_len;          // host's bound on seq_lens (device values are clamped to it)
  int n_ref_max, n_chunk_max;
  int S, pages_per_split;   // split grid
  int tab_cap;              // ordinals a block's LDS weight table holds (rows of a split's table in the workspace)
  int spill_on;             // some sequence has more ordinals than that: older ordinals go to the spill table
  float qk_scale_log2;      // scale * log2(e)
  // workspace
  int32_t* status;
  int32_t* rescue;          // int32 [B][Hq]: 1 = this output row is recomputed by the rescue kernel
  uint16_t* qlat;
  int64_t qlat_lo_offset;   // elements from the hi part to the lo part of qlat
  float* sref;
  float* cmax;
  float* lpart;
  int32_t* wflag;
  int32_t* items;           // [0] = number of (sequence, split) items, then item = sequence * kMaxSplits + split
  float* accpart;
  float* opart;
  float* wpart;             // fp32 [B][Hkv][S][tab_cap][Gp]
  float* spill;             // fp32 [B][Hkv][n_ref_max][Gp]: plain weights of ordinals older than a block's window
  float* rawo;              // fp32 [B][Hkv][kRawMaxChunks][Gp][128]: sum_t 2^(x_t - m) V_t of one raw chunk
  float* rawml;             // fp32 [B][Hkv][kRawMaxChunks][Gp][2]: the chunk's m (largest logit, log2 units) and sum of weights
};

struct CompressParams {
  uint16_t* latent;
  int32_t* idx;
  uint16_t* ref;
  float* ref_inv_norm;
  const int32_t* block_tables;
  const int32_t* ref_tables;
  int bt_stride, rt_stride;
  int64_t latent_page_stride, latent_head_stride, latent_stream_stride;
  int64_t idx_page_stride, idx_head_stride;
  int64_t ref_head_stride, ref_kv_stride, ref_norm_head_stride;
  int64_t n_pages_pool, n_ref_slots;
  const uint16_t* w_down_k;
  const uint16_t* w_down_v;
  const uint16_t* k_new;
  const uint16_t* v_new;
  const int32_t* cu_new;
  const int32_t* len_before;
  int batch, n_new_total;
  int Hkv, R, stride, joint;
  int q4;                           // 4-bit token-wise latents (single stream)
  int metric;                       // 0: cosine, 1: squared L2 distance (section 4.1)
  int top_k;                        // references retrieved per (token, kv-head): 1, 2 or 4 (section 4.1, arg top-k)
  int round;                        // retrieval round of this launch: finds each token's (round+1)-th nearest reference
  int64_t idx_slot_stride;          // elements between the ordinal slots of a token in the index pool
  int64_t round_stride;             // elements between the rounds' copies of ord / exact_key
  const int32_t* ord_all;           // [top_k][n_new_total][Hkv]: ord of every round (round r at r * round_stride)
  const uint64_t* exact_key_all;    // [top_k][n_new_total][Hkv]
  int32_t* flag_count_all;          // [top_k][batch][Hkv] (cleared by admit_refs)
  int proj_ppb;                     // consecutive pages a block of the projection kernel takes
  int NS;            // reference-range splits of the similarity search
  float* part;       // fp32x4 [n_new_total][Hkv][NS]: best, second best, arg best (int bits), |token|^2
  int32_t* ord;        // [n_new_total][Hkv] chosen reference ordinal
  int32_t* flag_count; // [batch][Hkv] tokens queued for exact re-scoring
  int32_t* flag_list;  // [Hkv][n_new_total] queued token indices, sequence b's segment starts at cu_new[b]
  uint64_t* exact_key; // [n_new_total][Hkv] result keys of the exact pass (valid for queued tokens)
  uint16_t* wt;        // bf16 [2][R][kWPad]: W_dK^T and W_dV^T, rows padded, written by admit_refs for project
  // non-linear compressor (section 4.1): mlp_kind < 0 means the linear projection above is used
  int mlp_kind;                     // 0: GeLU(x W1 + b1) W2; 1: (SiLU(x Wg) * (x W1 + b1)) W2
  int mlp_hidden, mlp_hidden_pad;   // hidden width, and the same rounded up to a multiple of kMlpChunk
  const uint16_t* mlp_w1;           // bf16 [2 * head_dim][hidden]
  const uint16_t* mlp_wg;           // bf16 [2 * head_dim][hidden] (kind 1)
  const uint16_t* mlp_w2;           // bf16 [hidden][R]
  const float* mlp_b1;              // fp32 [hidden]
  uint16_t* mlp_w1t;                // bf16 [hidden_pad][kMlpXPad]: W1^T, zero padded (written by mlp_prep)
  uint16_t* mlp_wgt;                // the same for Wg
  uint16_t* mlp_w2t;                // bf16 [hidden_pad / kMlpChunk][mlp_w2_chunk_elems(R)]: W2^T by chunks of hidden
                                    // columns, each chunk [R][kMlpW2Pad] and padding
  float* mlp_b1p;                   // fp32 [hidden_pad]
};
constexpr int kMlpChunk = 64;       // hidden columns staged in LDS per step of the non-linear projection kernel
constexpr int kMlpXPad = 2 * kHeadDim + 8;   // bf16 elements per staged W1^T row
constexpr int kMlpW2Pad = kMlpChunk + 4;     // bf16 elements per staged W2^T row
constexpr int kMlpHiddenMax = 1024;
// bf16 elements of one chunk of the packed W2^T: [R][kMlpW2Pad], rounded up to whole KB (the unit of a wave's
// direct-to-LDS copy)
__host__ __device__ constexpr int mlp_w2_chunk_elems(int R) { return (R * kMlpW2Pad * 2 + 1023) / 1024 * 512; }
constexpr int64_t kMlpWsBytes = 2ll * kMlpHiddenMax * kMlpXPad * 2 + (int64_t)kMlpHiddenMax / kMlpChunk * 128 * kMlpW2Pad * 2 +
                                kMlpHiddenMax * 4 + 4 * 256;

struct CompressWs {
  int64_t ord, flag_count, flag_list, exact_key, wt, mlp, part;   // byte offsets; `part` takes everything from its offset on
  int64_t ord_round, flag_count_round, flag_list_round, exact_key_round;   // bytes between the rounds of a top-k call
  int64_t total;
};
// Offsets for a call with n_new tokens in total; `total` leaves room for 8 reference-range splits of a large
// call and up to 64 of a small one.
inline CompressWs plan_compress_ws(const deltakv_dims& d, int64_t batch, int64_t n_new, int64_t) {
  CompressWs w;
  int64_t o = 0;
  auto take = [&](int64_t bytes) { int64_t at = o; o = align_up(o + bytes, 256); return at; };
  const int64_t K = d.top_k > 1 ? d.top_k : 1;              // one set of retrieval state per round
  w.ord_round = n_new * d.n_kv_heads * 4;
  w.flag_count_round = batch * d.n_kv_heads * 4;
  w.flag_list_round = n_new * d.n_kv_heads * 4;
  w.exact_key_round = n_new * d.n_kv_heads * 8;
  w.ord = take(K * w.ord_round);
  w.flag_count = take(K * w.flag_count_round);
  w.wt = take(2 * (int64_t)d.rank * kWPad * 2);
  w.mlp = take(kMlpWsBytes);                                // transposed weights of the non-linear compressor
  w.flag_list = take(K * w.flag_list_round);
  w.exact_key = take(K * w.exact_key_round);
  w.part = o;
  const int64_t slots = 8 * n_new > n_new + 64 * batch ? 8 * n_new : n_new + 64 * batch;
  w.total = o + align_up(slots * d.n_kv_heads * 16, 256);
  return w;
}

// Token rows per block of the similarity kernel for row-block factor rb (1, 2 or 4).
int sim_tile_rows(int rb, int nw);
// Enqueues the three compress kernels on `st`.
hipError_t launch_compress(const CompressParams& P, const CompressWs& cw, char* ws, int rb, int nw, int tiles_max,
                           int page_tiles_max, int max_new_refs, hipStream_t st);

// Enqueues the two kernels of the decode-append path (every sequence brings exactly one new token; P.NS = blocks
// per (sequence, kv-head) of the candidate scan).
hipError_t launch_append(const CompressParams& P, hipStream_t st);

// Optional per-kernel timing (deltakv_timing_begin / deltakv_timing_end): when enabled, launchers call
// timing_mark(kernel_id, stream) before the first kernel (id -1) and after every kernel.
enum KernelId { K_REF_SCORES = 0, K_STREAM, K_REF_VALUES, K_FINALIZE, K_ADMIT, K_SIM, K_RESOLVE, K_EXACT, K_PROJECT, K_RAW, K_COUNT };
void timing_mark(int kernel_id, hipStream_t st);

// LDS bytes of the streaming kernel with a weight table of n_rows reference ordinals.
size_t stream_lds_bytes(int n_rows, int Gp, int R, int nw, bool joint);
// The streaming kernel, one function per family of template variants (stream_*.hip); each picks the rank.
hipError_t stream_split_full(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st);
hipError_t stream_split_subset(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st);
hipError_t stream_joint_full(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st);
hipError_t stream_joint_subset(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st);
hipError_t stream_q4_joint(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st);
hipError_t stream_q4_split(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st);
// Decode attention with rotary position embedding on the reconstructed keys (rope_attn.hip): table of the pages'
// rotations, attention over every token's rebuilt and rotated key, merge of the splits.
size_t rope_lds_bytes(int R, int Gp);
hipError_t launch_rope(const DecodeParams& P, float2* tab, int n_pages_max, float base, int batch, hipStream_t st);
// Enqueues the four decode kernels on `st`.
hipError_t launch_decode(const DecodeParams& P, int batch, int n_items, int nw, size_t lds, hipStream_t st);

}  // namespace dkv
