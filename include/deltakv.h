/*
 * deltakv.h -- C ABI of the MI355X (gfx950) DeltaKV hot path.
 *
 * Paper: "DeltaKV: Residual-Based KV Cache Compression via Long-Range
 * Similarity".  The library implements two operations and the layout
 * arithmetic they share:
 *
 *   deltakv_compress     section 4.1 (strided reference set, nearest-reference
 *                        retrieval, residual, compressor) and appendix B.2
 *                        "lifecycle management" steps 1-3 (residual against the
 *                        assigned reference -> down-projection -> write to the
 *                        latent pool), with the retrieval of appendix B.3
 *                        ("batch distance" search as a dense matrix product).
 *   deltakv_decode_attn  section 4.1 "Reconstruction" (KV_hat = f_d(z) + KV_ref)
 *                        with the bias-free linear decoder of section 5.3,
 *                        fused into grouped-query softmax attention for one new
 *                        query token per sequence (the fused
 *                        reconstruction-attention kernel that section 5.3 and
 *                        appendix B.5 name as future work).
 *   deltakv_paged_layout appendix B.1 (separate pools for raw reference tokens
 *                        and for latents, addressed through per-sequence maps).
 *
 * Variants of the two operations (each documented at its declaration):
 *   deltakv_decode_attn_subset / _raw   section 4.2 (attention over the selected
 *                        tokens only) and appendix B.2 (raw sink / recent segment);
 *   deltakv_decode_attn_rope            section 4.1 (pre-RoPE cache): keys rotated
 *                        at their positions after reconstruction;
 *   deltakv_decode_attn_static          the same as deltakv_decode_attn for
 *                        callers that may not allocate or pass a workspace;
 *   deltakv_compress_mlp                section 4.1's non-linear compressor
 *                        (GeLU MLP; the gated variant of section 5.3).
 *
 * Readings fixed by this build (the paper is silent or differs):
 *   - by default one reference per (token, kv-head), chosen by cosine similarity
 *     over the 256-value vector K||V of that head, lowest ordinal wins ties; the
 *     paper's retrieval (top-k by squared L2, k = 4, mean of the references) is
 *     selected with the dims' `metric` and `top_k` fields;
 *   - positions are 0-indexed; token t is a reference iff t % ref_stride == 0,
 *     its ordinal is t / ref_stride; candidates of token i are ordinals j with
 *     j * ref_stride < i;
 *   - a reference token is kept raw in the reference pool AND owns a latent
 *     record (index = its own ordinal, latent = 0), so every cached token is
 *     read the same way;
 *   - SPLIT mode: z_K = (K - K_ref) W_dK, z_V = (V - V_ref) W_dV, two streams;
 *     JOINT mode: z = (K - K_ref) W_dK + (V - V_ref) W_dV, one stream (the
 *     paper's single latent over Concat(K, V));
 *   - latents are bf16 (round to nearest even), accumulation is fp32.
 *
 * General conventions
 *   - every function returns 0 on success or a negative DELTAKV_E_* code; no
 *     function throws, allocates device memory, synchronises the device or uses
 *     the default stream (kernels go to the stream passed in);
 *   - "device" pointers are HIP device memory owned by the caller and must stay
 *     valid until the stream has run the enqueued work; "host" pointers are
 *     ordinary host memory read before the call returns;
 *   - only host-visible arguments are validated.  Device contents (page ids,
 *     slots, stored reference ordinals) are clamped into range before use, so a
 *     corrupt cache gives wrong numbers, not a fault;
 *   - bf16 buffers are raw 16-bit patterns (uint16_t).
 */
#ifndef DELTAKV_H
#define DELTAKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DELTAKV_OK             0
#define DELTAKV_E_INVALID_ARG (-1)  /* null pointer, negative size, inconsistent argument      */
#define DELTAKV_E_UNSUPPORTED (-2)  /* shape outside what the kernels implement                */
#define DELTAKV_E_WORKSPACE   (-3)  /* workspace missing, misaligned or too small              */
#define DELTAKV_E_HIP         (-4)  /* a HIP runtime call failed (launch, attribute)           */

#define DELTAKV_SPLIT 0
#define DELTAKV_JOINT 1

/* Retrieval metric of the reference search (section 4.1): the nearest earlier
 * reference of a token over the per-head vector K||V, by cosine similarity or by
 * squared L2 distance (the section's own choice); lowest ordinal on ties.  One
 * cache uses one metric for its whole life: the per-reference float written at
 * admission depends on it. */
#define DELTAKV_METRIC_COSINE 0
#define DELTAKV_METRIC_L2     1

/* Problem dimensions.  v1 kernels need head_dim == 128, page_tokens == 16,
 * rank a multiple of 16 in [16, 128], 1 <= n_q_heads / n_kv_heads <= 16 and
 * n_q_heads % n_kv_heads == 0; anything else returns DELTAKV_E_UNSUPPORTED.
 * latent_bits = 4 stores the latents as 4-bit codes with a bf16 scale and zero
 * point per (token, kv-head) (section 5.3; format with the pool layout below);
 * compress writes such records and every decode entry point reads them. */
typedef struct {
  int32_t n_kv_heads;
  int32_t n_q_heads;
  int32_t head_dim;
  int32_t rank;         /* r: latent width per stream                              */
  int32_t latent_mode;  /* DELTAKV_SPLIT or DELTAKV_JOINT                          */
  int32_t ref_stride;   /* s >= 1: every s-th token is a reference                 */
  int32_t page_tokens;  /* P: tokens per page                                      */
  int32_t metric;       /* DELTAKV_METRIC_COSINE or DELTAKV_METRIC_L2              */
  int64_t n_pages;      /* capacity of the latent / index pools, in pages          */
  int64_t n_ref_slots;  /* capacity of the reference pool, in reference tokens     */
  int32_t latent_bits;  /* 16 (or 0): bf16 latents; 4: 4-bit token-wise latents    */
  int32_t top_k;        /* 1 (or 0), 2 or 4: references retrieved per (token, kv-head) */
} deltakv_dims;

/* Filled by deltakv_paged_layout; the only source of sizes and strides.
 *
 * Pools (all device memory, base addresses aligned to `alignment` bytes):
 *   latent pool  bf16   [n_pages][n_kv_heads][n_streams] blocks of P*r values.
 *                Inside a block the P x r latents of one (page, head, stream)
 *                are stored in the order the matrix units consume them:
 *                  stream 0 (scores operand; the only stream in JOINT mode):
 *                    value (tok, c) at ((c/8)*P + tok)*8 + c%8
 *                  stream 1 (value operand, SPLIT mode only):
 *                    value (tok, c) at ((c/16)*64 + (tok/4)*16 + c%16)*4 + tok%4
 *                deltakv_latent_block_offsets returns these as a table.
 *                With latent_bits = 4 (section 5.3: token-wise 4-bit quantisation
 *                of the compressed residuals) a (page, head, stream) block is
 *                8*r + 64 bytes: 8*r bytes of codes, then, for each group of
 *                four tokens, 4 bf16 scales followed by 4 bf16 zero points (16
 *                bytes per group).  A value reads back as scale * code + zero.
 *                  stream 0: the dword of (chunk c/8, tok) at byte 4*((c/8)*P + tok),
 *                    the code of value c in bits [s, s+3], s = 4*((c%8)/2) + 16*(c%2)
 *                  stream 1 (SPLIT mode; needs rank 64 or 128, other ranks return
 *                    DELTAKV_E_UNSUPPORTED): an 8-byte pair of dwords per (c/64,
 *                    tok/4, c%16) at byte 8*((c/64)*64 + (tok/4)*16 + c%16); tokens
 *                    tok%4 = 0, 1 in the first dword and 2, 3 in the second; the
 *                    code of value c in bits [s, s+3], s = 4*((c/16)%4) + 16*(tok%2)
 *                Strides stay in 2-byte elements.
 *   index pool   int32  [n_pages][n_kv_heads][top_k][P]   reference ordinals per token: slot i holds the token's
 *                i-th nearest reference (section 4.1, arg top-k), -1 where a token has fewer candidates than
 *                top_k; a reference token holds its own ordinal in slot 0 and -1 elsewhere.  The token's reference
 *                is the MEAN of the raw rows of the slots in use (section 4.1), in compress and in decode alike.
 *                top_k > 1 needs bf16 latents, and decode then needs every sequence's weight table on chip
 *                (roughly seq_len / ref_stride * g <= 39000): otherwise DELTAKV_E_UNSUPPORTED.
 *   reference pool bf16 [n_kv_heads][2][n_ref_slots][head_dim]   (0 = K, 1 = V)
 *   reference inverse norms fp32 [n_kv_heads][n_ref_slots]: 1/||K||V|| of the
 *                slot's raw vector (0 for a zero vector), written at admission;
 *                with DELTAKV_METRIC_L2 the same array holds ||K||V||^2 / 2.
 * Strides are in elements of the pool's type. */
typedef struct {
  int64_t latent_pool_bytes, idx_pool_bytes, ref_pool_bytes, ref_norm_pool_bytes;
  int64_t latent_page_stride, latent_head_stride, latent_stream_stride;
  int64_t idx_page_stride, idx_head_stride, idx_slot_stride;
  int64_t ref_head_stride, ref_kv_stride, ref_slot_stride;
  int64_t ref_norm_head_stride;
  int64_t compress_ws_bytes; /* workspace for deltakv_compress at the sizes asked  */
  int64_t decode_ws_bytes;   /* workspace for deltakv_decode_attn at the sizes asked */
  int32_t n_streams;         /* 2 in SPLIT mode, 1 in JOINT mode                   */
  int32_t alignment;         /* required alignment of pools and workspaces, bytes  */
} deltakv_layout;

/* Host-only, pure.  Computes pool sizes / strides for `dims`, and workspace
 * sizes good for any call with batch <= max_batch, at most max_new_tokens new
 * tokens in total per compress call, and sequences of at most max_seq_len
 * tokens (after appending).  Errors: INVALID_ARG (null, non-positive sizes),
 * UNSUPPORTED (see deltakv_dims). */
int deltakv_paged_layout(const deltakv_dims* dims, int32_t max_batch, int64_t max_new_tokens,
                         int64_t max_seq_len, deltakv_layout* out);

/* Host-only, pure.  out[tok * rank + c] = element offset of latent value
 * (tok, c) inside one (page, head, stream) block; `out` holds P*rank int32. */
int deltakv_latent_block_offsets(const deltakv_dims* dims, int32_t stream, int32_t* out);

/* Host-only, pure; latent_bits = 4 only (UNSUPPORTED otherwise).  Where the 4-bit
 * record of token slot `tok` lives inside one (page, head, stream) block, in
 * 2-byte elements from the block's start:
 *   code of column c : bits code_shift[tok*rank+c] .. +3 of element code_elem[tok*rank+c]
 *   scale, zero point: elements scale_elem[tok], zero_elem[tok] (bf16 bits)
 * code_elem and code_shift hold P*rank int32, scale_elem and zero_elem P int32. */
int deltakv_q4_block_offsets(const deltakv_dims* dims, int32_t stream, int32_t* code_elem,
                             int32_t* code_shift, int32_t* scale_elem, int32_t* zero_elem);

/* Host-only, pure.  Bytes this layout keeps per cached token (latent record +
 * index + the amortised raw reference and its norm) over the bytes of the dense
 * bf16 K and V it replaces: the per-layer bracket of the paper's keep-ratio
 * accounting (appendix D, equation (5)) evaluated for the real record sizes. */
double deltakv_keep_ratio(const deltakv_dims* dims);

/* Residual compression of new tokens (prefill chunk or decode append).
 *
 * For sequence b, tokens cu_new[b] .. cu_new[b+1]-1 of k_new / v_new are its
 * next tokens, at positions len_before[b], len_before[b]+1, ...  For each new
 * token t and kv-head h:
 *   t % s == 0: raw K,V copied to reference slot ref_tables[b][t/s], inverse
 *               norm stored, index := t/s, latent := 0;
 *   otherwise : index := argmax_j cos(K||V of t, K||V of reference ordinal j)
 *               over j*s < t (lowest j on ties; references older than this call
 *               are read from the reference pool), latent := the projected
 *               residual against that reference, rounded to bf16.
 * Results go to page block_tables[b][t / P], token slot t % P.
 *
 *   latent_pool, idx_pool, ref_pool, ref_inv_norm  device, read+written
 *   block_tables  device int32 [batch][bt_stride]: logical page -> pool page
 *   ref_tables    device int32 [batch][rt_stride]: reference ordinal -> slot
 *   w_down_k/v    device bf16 [head_dim][rank]
 *   k_new, v_new  device bf16 [n_new_total][n_kv_heads][head_dim]
 *   cu_new        device int32 [batch+1]; cu_new_host: the same values on the host
 *   len_before    device int32 [batch];   len_before_host: the same on the host
 *   workspace     device, >= layout->compress_ws_bytes, aligned
 *   stream        hipStream_t (as void*); must not be the null stream object of
 *                 another device
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE (too small for this call), HIP. */
int deltakv_compress(const deltakv_dims* dims, const deltakv_layout* layout,
                     void* latent_pool, int32_t* idx_pool, void* ref_pool, float* ref_inv_norm,
                     const int32_t* block_tables, int32_t bt_stride,
                     const int32_t* ref_tables, int32_t rt_stride,
                     const void* w_down_k, const void* w_down_v,
                     const void* k_new, const void* v_new,
                     const int32_t* cu_new, const int32_t* cu_new_host,
                     const int32_t* len_before, const int32_t* len_before_host,
                     int32_t batch, void* workspace, int64_t ws_bytes, void* stream);

/* The non-linear compressor f_c of section 4.1 over the per-head vector
 * x = K||V (2 * head_dim values):
 *   DELTAKV_MLP_GELU    f_c(x) = GeLU(x W1 + b1) W2      (GeLU with the exact erf)
 *   DELTAKV_MLP_SWIGLU  f_c(x) = (SiLU(x Wg) * (x W1 + b1)) W2   (section 5.3, the
 *                       gated variant)
 * The output bias of the section's formula is not taken: the latent is a
 * difference of two f_c values, in which it cancels.  All pointers are device
 * memory owned by the caller; row-major. */
#define DELTAKV_MLP_GELU 0
#define DELTAKV_MLP_SWIGLU 1
typedef struct deltakv_mlp {
  int32_t kind;      /* DELTAKV_MLP_*                                          */
  int32_t hidden;    /* hidden width d_h, 1 .. 1024                            */
  const void* w1;    /* bf16 [2 * head_dim][hidden]                            */
  const void* wg;    /* bf16 [2 * head_dim][hidden] (SWIGLU), else NULL        */
  const float* b1;   /* fp32 [hidden]                                          */
  const void* w2;    /* bf16 [hidden][rank]                                    */
} deltakv_mlp;

/* deltakv_compress with the non-linear compressor (section 4.1): references,
 * retrieval, indices and layout as there, but the latent of a non-reference token
 * is  f_c(K||V of the token) - f_c(K||V of its reference)  rounded to bf16 (the
 * compressor is applied to both sides separately; the decoder stays the linear
 * W_up of deltakv_decode_attn).  Needs latent_mode JOINT (one latent over K||V),
 * 16-bit latents and top_k <= 1: anything else is UNSUPPORTED.  The weights are
 * re-packed into the workspace by every call (a few microseconds).
 * Other arguments and errors: as deltakv_compress. */
int deltakv_compress_mlp(const deltakv_dims* dims, const deltakv_layout* layout,
                         void* latent_pool, int32_t* idx_pool, void* ref_pool, float* ref_inv_norm,
                         const int32_t* block_tables, int32_t bt_stride,
                         const int32_t* ref_tables, int32_t rt_stride,
                         const deltakv_mlp* mlp,
                         const void* k_new, const void* v_new,
                         const int32_t* cu_new, const int32_t* cu_new_host,
                         const int32_t* len_before, const int32_t* len_before_host,
                         int32_t batch, void* workspace, int64_t ws_bytes, void* stream);

/* Grouped-query softmax attention of one query token per sequence over the
 * compressed cache: for q-head g (kv-head h = g / (n_q_heads/n_kv_heads)) and
 * every cached token t < seq_lens[b],
 *   K_hat = K_ref[idx] + z_K W_uK,  V_hat = V_ref[idx] + z_V W_uV  (JOINT: z_V = z_K)
 *   out[g] = sum_t softmax_t(scale * q_g . K_hat_t) V_hat_t .
 * The result equals reconstruct-then-attend; the kernels use the linearity of
 * the decoder to score latents against W_uK q and to up-project the weighted
 * latent sum once.
 *
 *   w_up_k/v      device bf16 [rank][head_dim]
 *   q             device bf16 [batch][n_q_heads][head_dim]
 *   seq_lens      device int32 [batch]; seq_lens_host: same values on the host
 *                 (used to size the launch).  A sequence of length 0 gets out = 0
 *                 and lse = -inf.
 *   out           device bf16 [batch][n_q_heads][head_dim]
 *   lse           device fp32 [batch][n_q_heads] natural-log sum of exp of the
 *                 scaled logits, or NULL
 *   workspace     device, >= layout->decode_ws_bytes, aligned.  Its first int32 is
 *                 a status word written by the call (read it after the stream has
 *                 run the work).  It is diagnostic only -- out and lse are the attention
 *                 defined above whatever it says: the main kernels keep every softmax
 *                 weight in one fixed exponent frame per (sequence, q-head) around the
 *                 largest reference score, and an output row that leaves the frame is
 *                 recomputed inside the same call by a slow kernel that takes the row's
 *                 own largest logit as its offset.  The word says that this happened:
 *                   bit 0  a row left the frame: a logit 86 nats or more above every
 *                          reference token's logit (55 nats in a call with a selection),
 *                          or a selection whose tokens all lie 55 nats or more below the
 *                          largest reference score of the sequence;
 *                   bit 1  more than 256 softmax weights in one block were at least 2^11
 *                          times the weight of the token's own reference, or accumulated
 *                          past the 32-bit range of an on-chip table entry.
 *                 Neither happens with residuals that are small next to the references
 *                 they refine; a set bit means the call took milliseconds instead of
 *                 microseconds for the rows concerned.
 * Sequences may be as long as the pools hold (up to 2^30 tokens and 2^29 / g reference ordinals, g = queries per
 * kv-head rounded up to 4, 8 or 16).  Up to roughly seq_len / ref_stride * g = 39000 (34000 in JOINT mode) a
 * sequence's per-reference weight table lives on chip; beyond, older ordinals are accumulated in global memory,
 * which costs time, not accuracy.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
int deltakv_decode_attn(const deltakv_dims* dims, const deltakv_layout* layout,
                        const void* latent_pool, const int32_t* idx_pool, const void* ref_pool,
                        const int32_t* block_tables, int32_t bt_stride,
                        const int32_t* ref_tables, int32_t rt_stride,
                        const void* w_up_k, const void* w_up_v, const void* q,
                        const int32_t* seq_lens, const int32_t* seq_lens_host,
                        int32_t batch, float scale, void* out, float* lse,
                        void* workspace, int64_t ws_bytes, void* stream);

/* deltakv_decode_attn restricted to selected tokens: the attention of section 4.2
 * ("Inference with Sparse Attention"), where only the tokens a sparse attention
 * mask asks for are reconstructed (appendix B.2, view construction: index
 * resolution and batch reconstruction).  For sequence b the selection is an
 * ascending list of logical pages (token position / page_tokens) that hold at
 * least one selected token, and for each listed page a bit mask of its selected
 * tokens:
 *   sel_pages   device int32 [batch][sel_stride]  logical pages, ascending, distinct
 *   sel_masks   device int32 [batch][sel_stride]  bit t set: token page*P + t selected
 *   n_sel       device int32 [batch] entries used per sequence; n_sel_host: the
 *               same values on the host (each in [0, sel_stride])
 * Positions at or past seq_lens[b] are ignored; a sequence with nothing selected
 * gets out = 0 and lse = -inf.  out / lse are the softmax over the selected tokens
 * only.  Whole pages are streamed, so a selection costs the traffic of the pages it
 * touches: it is cheapest when selected tokens share pages.  Every raw reference
 * is still scored once per call.  The exponent frame of the softmax hangs on the largest
 * reference score of the sequence, selected or not; rows whose selected tokens all lie far
 * below it are recomputed by the slow kernel (bit 0 of the status word).
 * Other arguments, workspace, status word and errors as deltakv_decode_attn. */
int deltakv_decode_attn_subset(const deltakv_dims* dims, const deltakv_layout* layout,
                               const void* latent_pool, const int32_t* idx_pool, const void* ref_pool,
                               const int32_t* block_tables, int32_t bt_stride,
                               const int32_t* ref_tables, int32_t rt_stride,
                               const void* w_up_k, const void* w_up_v, const void* q,
                               const int32_t* seq_lens, const int32_t* seq_lens_host,
                               const int32_t* sel_pages, const int32_t* sel_masks, int32_t sel_stride,
                               const int32_t* n_sel, const int32_t* n_sel_host,
                               int32_t batch, float scale, void* out, float* lse,
                               void* workspace, int64_t ws_bytes, void* stream);

/* Decode attention over the compressed cache TOGETHER WITH a segment of tokens held raw: appendix B.2 keeps
 * sink and recent tokens at full precision in a pool of their own, and the attention view puts those static
 * slots beside the reconstructed tokens.  The result is the softmax attention over the union of
 *   - the cached tokens (all tokens below seq_lens[b], or, if sel_pages is not NULL, the selected ones exactly as
 *     in deltakv_decode_attn_subset; with sel_pages NULL the other four selection arguments are ignored), and
 *   - raw_lens[b] raw tokens of sequence b, which must not also be in the cache (a token in both counts twice).
 *   raw_k, raw_v  device bf16 [batch][raw_cap][n_kv_heads][head_dim], 16-byte aligned; rows at or past
 *                 raw_lens[b] are never read.  Not modified; the caller owns them.
 *   raw_lens      device int32 [batch]; values are clamped to [0, raw_cap]
 *   raw_cap       host, 0 <= raw_cap <= 4096 (larger: DELTAKV_E_UNSUPPORTED); 0 makes this call
 *                 deltakv_decode_attn / deltakv_decode_attn_subset and raw_k, raw_v, raw_lens may be NULL
 * A sequence with neither cached (selected) tokens nor raw tokens gets out = 0 and lse = -inf.  Raw tokens take no
 * part in the exponent offset of the cached part, so their logits may lie anywhere relative to it: the two parts
 * are merged at the larger of their offsets.  Everything else (arguments, workspace, status word, errors) as for
 * deltakv_decode_attn_subset. */
int deltakv_decode_attn_raw(const deltakv_dims* dims, const deltakv_layout* layout,
                            const void* latent_pool, const int32_t* idx_pool, const void* ref_pool,
                            const int32_t* block_tables, int32_t bt_stride,
                            const int32_t* ref_tables, int32_t rt_stride,
                            const void* w_up_k, const void* w_up_v, const void* q,
                            const int32_t* seq_lens, const int32_t* seq_lens_host,
                            const int32_t* sel_pages, const int32_t* sel_masks, int32_t sel_stride,
                            const int32_t* n_sel, const int32_t* n_sel_host,
                            const void* raw_k, const void* raw_v, const int32_t* raw_lens, int32_t raw_cap,
                            int32_t batch, float scale, void* out, float* lse,
                            void* workspace, int64_t ws_bytes, void* stream);

/* Decode attention for models that apply rotary position embedding to keys.  Section 4.1: the method works on
 * pre-RoPE key-value states, so the cache holds un-rotated keys; a key is reconstructed, K_hat = K_ref[idx] + z_K W_uK,
 * and then rotated at its token's position (cached token t has position t) before it meets the query -- the fused
 * re-rotation that appendix B.5 names as future work.  Values carry no rotation.
 *   q_rot      device bf16 [batch][n_q_heads][head_dim]: the query ALREADY rotated at its own position
 *   rope_base  > 1: dimension pair (i, i + head_dim/2) turns by position * rope_base^(-2i/head_dim) (the pairing of
 *              the Llama / Qwen families); no frequency scaling
 * out / lse as deltakv_decode_attn: the softmax attention over K_rot, V_hat of every cached token below seq_lens[b].
 * The per-reference factorisation of the plain call does not exist under a per-token rotation: every token's key is
 * rebuilt (matrix unit) and the raw K and V rows of its reference are gathered, so this call moves about three times
 * the bytes of deltakv_decode_attn.  Softmax is online (running maximum): no exponent frame, no status word.
 * Supported: bf16 latents (both latent modes), top_k = 1, at most 8 queries per kv-head; otherwise
 * DELTAKV_E_UNSUPPORTED.  workspace >= layout->decode_ws_bytes.  Errors as deltakv_decode_attn. */
int deltakv_decode_attn_rope(const deltakv_dims* dims, const deltakv_layout* layout,
                             const void* latent_pool, const int32_t* idx_pool, const void* ref_pool,
                             const int32_t* block_tables, int32_t bt_stride,
                             const int32_t* ref_tables, int32_t rt_stride,
                             const void* w_up_k, const void* w_up_v, const void* q_rot,
                             const int32_t* seq_lens, const int32_t* seq_lens_host,
                             int32_t batch, float scale, float rope_base, void* out, float* lse,
                             void* workspace, int64_t ws_bytes, void* stream);

/* deltakv_decode_attn for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments and result as
 * deltakv_decode_attn without `workspace` / `ws_bytes`: the workspace is a DELTAKV_STATIC_WS_BYTES array inside the
 * library's device image (each GPU the library runs on holds one copy until the process ends).  The call allocates
 * nothing, on the device or through any library.  A call whose batch and sequence lengths need more workspace than
 * that even with a single token-range split returns DELTAKV_E_WORKSPACE (deltakv_last_error_detail says so);
 * deltakv_paged_layout(...).decode_ws_bytes <= DELTAKV_STATIC_WS_BYTES is a sufficient condition for acceptance
 * (8 sequences of 131072 tokens with 8 kv-heads and 4 queries per kv-head fit).  Every call on one GPU uses the
 * same array and overwrites what the last call left there (nothing needs clearing: the kernels write whatever they
 * later read), so calls that overlap in time on one GPU -- from different streams or threads -- race; serialise them.
 * The status word of the call is not readable by the caller.  Errors otherwise as deltakv_decode_attn, plus
 * UNSUPPORTED for a device ordinal above 63. */
#define DELTAKV_STATIC_WS_BYTES (64ll << 20)
int deltakv_decode_attn_static(const deltakv_dims* dims, const deltakv_layout* layout,
                               const void* latent_pool, const int32_t* idx_pool, const void* ref_pool,
                               const int32_t* block_tables, int32_t bt_stride,
                               const int32_t* ref_tables, int32_t rt_stride,
                               const void* w_up_k, const void* w_up_v, const void* q,
                               const int32_t* seq_lens, const int32_t* seq_lens_host,
                               int32_t batch, float scale, void* out, float* lse, void* stream);

const char* deltakv_strerror(int code);
/* For DELTAKV_E_HIP: which runtime call failed and the runtime's message (calling thread's last failure;
 * empty string if none).  The pointer stays valid until the thread's next failing call. */
const char* deltakv_last_error_detail(void);
int deltakv_version(void);

/* The library keeps process-wide state without locks (the launch-shape overrides below, the timing marks, the
 * first-call kernel attributes): call it from one thread at a time.
 *
 * Launch-shape overrides for benchmark sweeps (process-wide; value 0 restores the automatic choice):
 *   "stream_waves"  waves per block of the decode streaming kernel (8)
 *   "splits"        token-range splits per (sequence, kv-head) in decode (1..16)
 *   "sim_tb"        16-token blocks per wave of the similarity kernel (1..4)
 *   "sim_waves"     waves per block of the similarity kernel (4 or 8; 8 needs sim_tb <= 2)
 *   "sim_ns"        reference-range splits of the similarity search (1..64)
 *   "project_pages" consecutive pages per block of the projection kernel (1..16)
 *   "table_rows"    cap on the reference ordinals a block of the streaming kernel keeps in its on-chip weight table
 *                   (>= 16; the default is what the LDS holds); ordinals older than the window go to a table in
 *                   global memory, as they do for sequences beyond about 160 000 tokens
 *   "ref_chunks"    reference chunks scored per block of the decode call's first kernel (1 or 4)
 *   "timing_period" timed regions record events for every value-th call only (0 or 1 = every call): an event costs
 *                   a few microseconds of stream time, which a benchmark may not want in front of every kernel
 * Results do not depend on these beyond floating-point summation order.  Errors: INVALID_ARG. */
int deltakv_tune(const char* name, int32_t value);

/* Per-kernel timing for benchmarks.  Between deltakv_timing_begin() and deltakv_timing_end() every
 * compress / decode call records a HIP event on its stream before its first kernel and after each
 * kernel (use one stream, call from one thread).  deltakv_timing_end waits for the last event and
 * returns, per kernel, the summed time between the surrounding events in milliseconds (this includes
 * the launch gap in front of the kernel) and the number of launches (with "timing_period" p set through
 * deltakv_tune, of the calls 0, p, 2p, ... of the region).  Kernel order:
 *   0 ref_scores, 1 stream, 2 ref_values, 3 finalize + rescue   (deltakv_decode_attn)
 *   4 admit_refs, 5 sim_top2, 6 resolve, 7 exact, 8 project   (deltakv_compress; a call that appends exactly
 *     one token to every sequence runs two kernels, reported as 5 (candidate scan) and 8 (finish))
 *   9 raw_attn   (deltakv_decode_attn_raw with a raw segment)
 * Arrays are host memory with n >= DELTAKV_N_KERNELS entries.  Errors: INVALID_ARG, HIP. */
#define DELTAKV_N_KERNELS 10
int deltakv_timing_begin(void);
int deltakv_timing_end(float* ms_by_kernel, int32_t* launches_by_kernel, int32_t n);

#ifdef __cplusplus
}
#endif
#endif /* DELTAKV_H */
