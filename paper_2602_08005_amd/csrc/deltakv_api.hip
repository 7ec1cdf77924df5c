// C ABI of libdeltakv: argument validation, layout arithmetic, workspace carving, launches.
// See include/deltakv.h for the contract of every entry point.
#include <stdio.h>

#include <vector>
#include <string.h>

#include "common.h"
#include "launch.h"

using namespace dkv;

namespace {

int check_dims(const deltakv_dims* d) {
  if (!d) return DELTAKV_E_INVALID_ARG;
  if (d->n_kv_heads <= 0 || d->n_q_heads <= 0 || d->head_dim <= 0 || d->rank <= 0 || d->ref_stride <= 0 ||
      d->page_tokens <= 0 || d->n_pages <= 0 || d->n_ref_slots <= 0)
    return DELTAKV_E_INVALID_ARG;
  if (d->latent_mode != DELTAKV_SPLIT && d->latent_mode != DELTAKV_JOINT) return DELTAKV_E_INVALID_ARG;
  if (d->n_q_heads % d->n_kv_heads != 0) return DELTAKV_E_UNSUPPORTED;
  if (d->n_q_heads / d->n_kv_heads > 16) return DELTAKV_E_UNSUPPORTED;
  if (d->head_dim != kHeadDim || d->page_tokens != kPage) return DELTAKV_E_UNSUPPORTED;
  if (d->rank % 16 != 0 || d->rank < 16 || d->rank > 128) return DELTAKV_E_UNSUPPORTED;
  if (d->metric != DELTAKV_METRIC_COSINE && d->metric != DELTAKV_METRIC_L2) return DELTAKV_E_INVALID_ARG;
  if (d->n_pages > (1ll << 31) - 1 || d->n_ref_slots > (1ll << 31) - 1) return DELTAKV_E_UNSUPPORTED;
  if (d->top_k != 0 && d->top_k != 1 && d->top_k != 2 && d->top_k != 4) return DELTAKV_E_INVALID_ARG;
  if (d->latent_bits != 0 && d->latent_bits != 16 && d->latent_bits != 4) return DELTAKV_E_INVALID_ARG;
  if (d->latent_bits == 4 && d->latent_mode != DELTAKV_JOINT && d->rank % 64 != 0) return DELTAKV_E_UNSUPPORTED;
  if (d->top_k > 1 && d->latent_bits == 4) return DELTAKV_E_UNSUPPORTED;
  return DELTAKV_OK;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int device_cu_count() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

thread_local char g_detail[256] = "";

// launch-shape overrides for sweeps (0 = automatic)
int g_tune_stream_waves = 0;
int g_tune_splits = 0;
int g_tune_sim_tb = 0;
int g_tune_sim_ns = 0;
int g_tune_sim_waves = 0;
int g_tune_ref_chunks = 0;
int g_tune_project_pages = 0;
int g_tune_table_rows = 0;

// per-kernel timing state (one timed region at a time, one stream)
struct Mark { hipEvent_t ev; int id; };
bool g_timing = false;
int g_timing_period = 1;       // events are recorded for calls 0, p, 2p, ... of a timed region
int g_timing_calls = 0;
bool g_timing_this_call = true;
std::vector<Mark> g_marks;
std::vector<hipEvent_t> g_event_pool;

}  // namespace

namespace dkv {
hipError_t note_hip_error(hipError_t e, const char* what) {
  if (e != hipSuccess) snprintf(g_detail, sizeof(g_detail), "%s: %s", what, hipGetErrorString(e));
  return e;
}
void timing_mark(int kernel_id, hipStream_t st) {
  if (!g_timing) return;
  if (kernel_id < 0) g_timing_this_call = g_timing_calls++ % g_timing_period == 0;   // the mark that opens a call
  if (!g_timing_this_call) return;
  if (g_event_pool.empty()) return;      // pool exhausted: the rest of the region goes unmarked
  hipEvent_t ev = g_event_pool.back();
  g_event_pool.pop_back();
  if (hipEventRecord(ev, st) != hipSuccess) {
    g_event_pool.push_back(ev);
    return;
  }
  g_marks.push_back(Mark{ev, kernel_id});
}
size_t device_lds_limit() {
  static size_t lim = 0;
  if (lim == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && n > 0)
      lim = (size_t)n;
    else
      lim = 64 * 1024;
  }
  return lim;
}
}  // namespace dkv

extern "C" {

int deltakv_version(void) { return 1; }

const char* deltakv_last_error_detail(void) { return g_detail; }

int deltakv_tune(const char* name, int32_t value) {
  if (!name || value < 0) return DELTAKV_E_INVALID_ARG;
  if (!strcmp(name, "stream_waves")) {
    if (value != 0 && value != 8) return DELTAKV_E_INVALID_ARG;
    g_tune_stream_waves = value;
  } else if (!strcmp(name, "splits")) {
    if (value > kMaxSplits) return DELTAKV_E_INVALID_ARG;
    g_tune_splits = value;
  } else if (!strcmp(name, "sim_ns")) {
    if (value > 64) return DELTAKV_E_INVALID_ARG;
    g_tune_sim_ns = value;
  } else if (!strcmp(name, "sim_waves")) {
    if (value != 0 && value != 4 && value != 8) return DELTAKV_E_INVALID_ARG;
    g_tune_sim_waves = value;
  } else if (!strcmp(name, "project_pages")) {
    if (value > 16) return DELTAKV_E_INVALID_ARG;
    g_tune_project_pages = value;
  } else if (!strcmp(name, "table_rows")) {
    if (value != 0 && value < 16) return DELTAKV_E_INVALID_ARG;
    g_tune_table_rows = value;
  } else if (!strcmp(name, "ref_chunks")) {
    if (value != 0 && value != 1 && value != 4) return DELTAKV_E_INVALID_ARG;
    g_tune_ref_chunks = value;
  } else if (!strcmp(name, "timing_period")) {
    g_timing_period = value > 1 ? value : 1;
  } else if (!strcmp(name, "sim_tb")) {
    if (value < 0 || value > 4) return DELTAKV_E_INVALID_ARG;
    g_tune_sim_tb = value;
  } else {
    return DELTAKV_E_INVALID_ARG;
  }
  return DELTAKV_OK;
}

int deltakv_timing_begin(void) {
  for (auto& m : g_marks) g_event_pool.push_back(m.ev);
  g_marks.clear();
  // events are created here, not inside a compress / decode call (which never allocates and may be under capture);
  // a region that needs more than this many marks records the first ones only
  while (g_event_pool.size() < 4096) {
    hipEvent_t ev;
    if (hipEventCreate(&ev) != hipSuccess) break;
    g_event_pool.push_back(ev);
  }
  g_timing_calls = 0;
  g_timing_this_call = true;
  g_timing = true;
  return DELTAKV_OK;
}

int deltakv_timing_end(float* ms_by_kernel, int32_t* launches_by_kernel, int32_t n) {
  g_timing = false;
  if (!ms_by_kernel || !launches_by_kernel || n < DELTAKV_N_KERNELS) return DELTAKV_E_INVALID_ARG;
  for (int i = 0; i < n; ++i) { ms_by_kernel[i] = 0.f; launches_by_kernel[i] = 0; }
  int rc = DELTAKV_OK;
  if (!g_marks.empty() && hipEventSynchronize(g_marks.back().ev) != hipSuccess) rc = DELTAKV_E_HIP;
  for (size_t i = 1; i < g_marks.size() && rc == DELTAKV_OK; ++i) {
    const int id = g_marks[i].id;
    if (id < 0 || id >= DELTAKV_N_KERNELS) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_marks[i - 1].ev, g_marks[i].ev) != hipSuccess) { rc = DELTAKV_E_HIP; break; }
    ms_by_kernel[id] += ms;
    launches_by_kernel[id] += 1;
  }
  for (auto& m : g_marks) g_event_pool.push_back(m.ev);
  g_marks.clear();
  return rc;
}

const char* deltakv_strerror(int code) {
  switch (code) {
    case DELTAKV_OK: return "ok";
    case DELTAKV_E_INVALID_ARG: return "invalid argument";
    case DELTAKV_E_UNSUPPORTED: return "unsupported shape";
    case DELTAKV_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case DELTAKV_E_HIP: return "HIP runtime error";
  }
  return "unknown error code";
}

int deltakv_paged_layout(const deltakv_dims* dims, int32_t max_batch, int64_t max_new_tokens,
                         int64_t max_seq_len, deltakv_layout* out) {
  int rc = check_dims(dims);
  if (rc != DELTAKV_OK) return rc;
  if (!out || max_batch <= 0 || max_new_tokens < 0 || max_seq_len <= 0) return DELTAKV_E_INVALID_ARG;
  if (max_seq_len > (1ll << 30)) return DELTAKV_E_UNSUPPORTED;
  memset(out, 0, sizeof(*out));
  const int64_t H = dims->n_kv_heads, P = dims->page_tokens, R = dims->rank, D = dims->head_dim;
  out->n_streams = dims->latent_mode == DELTAKV_JOINT ? 1 : 2;
  out->alignment = 256;
  out->latent_stream_stride = dims->latent_bits == 4 ? 4 * R + 32 : P * R;   // 2-byte elements
  out->latent_head_stride = out->n_streams * out->latent_stream_stride;
  out->latent_page_stride = H * out->latent_head_stride;
  out->latent_pool_bytes = dims->n_pages * out->latent_page_stride * 2;
  const int64_t KS = dims->top_k > 1 ? dims->top_k : 1;
  out->idx_slot_stride = P;
  out->idx_head_stride = KS * P;
  out->idx_page_stride = H * KS * P;
  out->idx_pool_bytes = dims->n_pages * out->idx_page_stride * 4;
  out->ref_slot_stride = D;
  out->ref_kv_stride = dims->n_ref_slots * D;
  out->ref_head_stride = 2 * out->ref_kv_stride;
  out->ref_pool_bytes = H * out->ref_head_stride * 2;
  out->ref_norm_head_stride = dims->n_ref_slots;
  out->ref_norm_pool_bytes = H * dims->n_ref_slots * 4;
  const int64_t n_ref_max = ceil_div64(max_seq_len, dims->ref_stride);
  {
    const int64_t rows = table_rows_max(padded_group(dims->n_q_heads / dims->n_kv_heads));
    out->decode_ws_bytes = plan_decode_ws(*dims, max_batch, n_ref_max, kMaxSplits, n_ref_max < rows ? n_ref_max : rows).total;
    const int64_t rope = plan_rope_ws(*dims, max_batch, ceil_div64(max_seq_len, P), kMaxSplits).total;
    if (rope > out->decode_ws_bytes) out->decode_ws_bytes = rope;
  }
  out->compress_ws_bytes = plan_compress_ws(*dims, max_batch, max_new_tokens, n_ref_max).total;
  return DELTAKV_OK;
}

int deltakv_latent_block_offsets(const deltakv_dims* dims, int32_t stream, int32_t* out) {
  int rc = check_dims(dims);
  if (rc != DELTAKV_OK) return rc;
  if (!out || stream < 0 || stream > 1) return DELTAKV_E_INVALID_ARG;
  if (stream == 1 && dims->latent_mode == DELTAKV_JOINT) return DELTAKV_E_INVALID_ARG;
  if (dims->latent_bits == 4) return DELTAKV_E_UNSUPPORTED;     // codes are not 2-byte elements
  const int P = dims->page_tokens, R = dims->rank;
  for (int tok = 0; tok < P; ++tok)
    for (int c = 0; c < R; ++c)
      out[tok * R + c] = stream == 0 ? ((c / 8) * P + tok) * 8 + c % 8
                                     : ((c / 16) * 64 + (tok / 4) * 16 + c % 16) * 4 + tok % 4;
  return DELTAKV_OK;
}

int deltakv_q4_block_offsets(const deltakv_dims* dims, int32_t stream, int32_t* code_elem, int32_t* code_shift,
                             int32_t* scale_elem, int32_t* zero_elem) {
  int rc = check_dims(dims);
  if (rc != DELTAKV_OK) return rc;
  if (!code_elem || !code_shift || !scale_elem || !zero_elem || stream < 0 || stream > 1) return DELTAKV_E_INVALID_ARG;
  if (stream == 1 && dims->latent_mode == DELTAKV_JOINT) return DELTAKV_E_INVALID_ARG;
  if (dims->latent_bits != 4) return DELTAKV_E_UNSUPPORTED;
  const int P = dims->page_tokens, R = dims->rank;
  for (int tok = 0; tok < P; ++tok) {
    for (int c = 0; c < R; ++c) {
      // stream 0: one dword per (8-column chunk, token), nibble (c % 8) / 2 of half-word c % 2;
      // stream 1: one dword pair per (64-column group, four tokens, column % 16), nibble (c / 16) % 4 of the token's half-word
      code_elem[tok * R + c] = stream == 0 ? 2 * ((c / 8) * P + tok) + c % 2
                                           : 4 * ((c / 64) * 64 + (tok / 4) * 16 + c % 16) + tok % 4;
      code_shift[tok * R + c] = stream == 0 ? 4 * ((c % 8) / 2) : 4 * ((c / 16) % 4);
    }
    scale_elem[tok] = 4 * R + (tok / 4) * 8 + tok % 4;       // after the codes: per four tokens, four scales then four zero points
    zero_elem[tok] = scale_elem[tok] + 4;
  }
  return DELTAKV_OK;
}

double deltakv_keep_ratio(const deltakv_dims* dims) {
  if (check_dims(dims) != DELTAKV_OK) return -1.0;
  const double streams = dims->latent_mode == DELTAKV_JOINT ? 1.0 : 2.0;
  const double raw = 2.0 * dims->head_dim * 2.0;
  const double rec = streams * (dims->latent_bits == 4 ? dims->rank / 2.0 + 4.0 : dims->rank * 2.0) +
                     4.0 * (dims->top_k > 1 ? dims->top_k : 1);
  return (rec + (raw + 4.0) / dims->ref_stride) / raw;
}

// Selection arguments of the subset entry point (all null / 0 for attention over the whole cache).
struct Selection {
  const int32_t* pages = nullptr;
  const int32_t* masks = nullptr;
  const int32_t* n_sel = nullptr;
  const int32_t* n_sel_host = nullptr;
  int32_t stride = 0;
};

// Raw segment of the third entry point (all null / 0 for none).
struct RawSegment {
  const void* k = nullptr;
  const void* v = nullptr;
  const int32_t* lens = nullptr;
  int32_t cap = 0;
};

static int decode_impl(const deltakv_dims* dims, const deltakv_layout* lay, const void* latent_pool,
                       const int32_t* idx_pool, const void* ref_pool, const int32_t* block_tables,
                       int32_t bt_stride, const int32_t* ref_tables, int32_t rt_stride, const void* w_up_k,
                       const void* w_up_v, const void* q, const int32_t* seq_lens,
                       const int32_t* seq_lens_host, const Selection& sel, const RawSegment& raw, int32_t batch,
                       float scale, void* out, float* lse, void* workspace, int64_t ws_bytes, void* stream) {
  int rc = check_dims(dims);
  if (rc != DELTAKV_OK) return rc;
  if (!lay || !latent_pool || !idx_pool || !ref_pool || !block_tables || !ref_tables || !w_up_k || !w_up_v ||
      !q || !seq_lens || !seq_lens_host || !out || batch < 0 || bt_stride <= 0 || rt_stride <= 0 ||
      !(scale == scale))
    return DELTAKV_E_INVALID_ARG;
  if (raw.cap < 0 || (raw.cap > 0 && (!raw.k || !raw.v || !raw.lens))) return DELTAKV_E_INVALID_ARG;
  if (raw.cap > 0 && (!aligned(raw.k, 16) || !aligned(raw.v, 16))) return DELTAKV_E_INVALID_ARG;
  if (raw.cap > kRawChunk * kRawMaxChunks) return DELTAKV_E_UNSUPPORTED;
  if (batch == 0) return DELTAKV_OK;
  if (batch > 65535) return DELTAKV_E_UNSUPPORTED;
  if (!workspace || !aligned(workspace, 256) || ws_bytes <= 0) return DELTAKV_E_WORKSPACE;
  if (!aligned(latent_pool, 16) || !aligned(idx_pool, 16) || !aligned(ref_pool, 16) || !aligned(q, 16) ||
      !aligned(w_up_k, 16) || !aligned(w_up_v, 16))
    return DELTAKV_E_INVALID_ARG;
  int max_len = 0;
  for (int b = 0; b < batch; ++b) {
    if (seq_lens_host[b] < 0) return DELTAKV_E_INVALID_ARG;
    if (seq_lens_host[b] > max_len) max_len = seq_lens_host[b];
  }
  const int P = dims->page_tokens, S = dims->ref_stride;
  const int max_pages = ceil_div(max_len > 0 ? max_len : 1, P);
  const int n_ref_max = ceil_div(max_len > 0 ? max_len : 1, S);
  if (max_pages > bt_stride || n_ref_max > rt_stride) return DELTAKV_E_INVALID_ARG;
  if ((int64_t)max_pages > dims->n_pages * 1ll || (int64_t)n_ref_max > dims->n_ref_slots * 1ll)
    return DELTAKV_E_INVALID_ARG;

  const int G = dims->n_q_heads / dims->n_kv_heads, Gp = padded_group(G), R = dims->rank;
  const int nw = g_tune_stream_waves ? g_tune_stream_waves : 8;
  // The streaming kernel keeps a (sequence, kv-head)'s per-reference weight table in LDS.  Longer sequences than
  // one compute unit's LDS holds keep a window of the most recent ordinals there and send the rest to a table in
  // global memory (the SPILL variants).
  const bool joint = dims->latent_mode == DELTAKV_JOINT;
  const size_t kLdsLimit = device_lds_limit();
  const size_t lds_other = stream_lds_bytes(0, Gp, R, nw, joint);
  if (lds_other + 4096 > kLdsLimit) return DELTAKV_E_UNSUPPORTED;
  int64_t tab_cap = (int64_t)((kLdsLimit - lds_other) / (Gp * 4)) & ~3ll;
  if (tab_cap > table_rows_max(Gp)) tab_cap = table_rows_max(Gp);
  if (tab_cap > 65535) tab_cap = 65535 & ~3;           // the kernel keeps table rows in 16 bits
  if (g_tune_table_rows > 0 && g_tune_table_rows < tab_cap) tab_cap = g_tune_table_rows & ~3;
  const bool spill_on = n_ref_max > tab_cap;
  if (spill_on && dims->top_k > 1) return DELTAKV_E_UNSUPPORTED;
  if (!spill_on) tab_cap = n_ref_max;
  if ((int64_t)n_ref_max * Gp * 4 >= (1ll << 31)) return DELTAKV_E_UNSUPPORTED;   // 32-bit byte offsets into a pair's tables
  const size_t lds = stream_lds_bytes((int)tab_cap, Gp, R, nw, joint);
  // Blocks of at most pages_per_split pages: about one per COMPUTE UNIT when all sequences have the same length
  // (blocks are handed out longest first as slots free up; each block costs several microseconds of set-up and
  // flush, which nothing overlaps).  Short
  // sequences would let several blocks share a compute unit, but more blocks than compute units only add set-up
  // time: at 8 sequences x 8 kv-heads, 256 blocks beat 512 and 1024 at every length from 2048 to 131072 tokens
  // (2048 tokens: 18 us against 28 and 48; 32768: 95 against 99 and 108).
  const int64_t slots = (int64_t)device_cu_count();
  // pages a sequence's blocks iterate over: all of its pages, or the selected ones
  auto work_pages = [&](int b) {
    const int n_pages = ceil_div(seq_lens_host[b], P);
    if (!sel.pages) return n_pages;
    const int n = sel.n_sel_host[b] < sel.stride ? sel.n_sel_host[b] : sel.stride;
    return n < 0 ? 0 : (n < n_pages ? n : n_pages);
  };
  int64_t total_pages = 0;
  int max_work = 1;
  bool uniform = true;
  for (int b = 0; b < batch; ++b) {
    const int wp = work_pages(b);
    total_pages += wp;
    if (wp > max_work) max_work = wp;
    uniform = uniform && wp == work_pages(0);
  }
  total_pages *= dims->n_kv_heads;
  // mixed lengths: half as many blocks again, so that the long sequences' blocks even out (the ragged batch of 64
  // sequences: 199, 210, 201, 195 k tokens/s with 3, 4, 6, 8 splits of the longest sequence; this rule picks 4)
  const int64_t pages_target = ceil_div64(2 * total_pages, (uniform ? 2 : 3) * slots);
  int splits = (int)ceil_div64(max_work, pages_target > 0 ? pages_target : 1);
  const int split_cap = max_work / 8 > 1 ? max_work / 8 : 1;    // at least 8 pages per split
  if (splits > split_cap) splits = split_cap;
  if (splits > kMaxSplits) splits = kMaxSplits;
  if (splits < 1) splits = 1;
  if (g_tune_splits) splits = g_tune_splits < split_cap ? g_tune_splits : split_cap;
  DecodeWs ws = plan_decode_ws(*dims, batch, n_ref_max, splits, tab_cap);
  while (ws.total > ws_bytes && splits > 1) {
    --splits;
    ws = plan_decode_ws(*dims, batch, n_ref_max, splits, tab_cap);
  }
  if (ws.total > ws_bytes) return DELTAKV_E_WORKSPACE;

  DecodeParams Pm;
  memset(&Pm, 0, sizeof(Pm));
  Pm.latent = static_cast<const uint16_t*>(latent_pool);
  Pm.idx = idx_pool;
  Pm.ref = static_cast<const uint16_t*>(ref_pool);
  Pm.block_tables = block_tables;
  Pm.ref_tables = ref_tables;
  Pm.seq_lens = seq_lens;
  Pm.bt_stride = bt_stride;
  Pm.rt_stride = rt_stride;
  Pm.latent_page_stride = lay->latent_page_stride;
  Pm.latent_head_stride = lay->latent_head_stride;
  Pm.latent_stream_stride = lay->latent_stream_stride;
  Pm.idx_page_stride = lay->idx_page_stride;
  Pm.idx_head_stride = lay->idx_head_stride;
  Pm.ref_head_stride = lay->ref_head_stride;
  Pm.ref_kv_stride = lay->ref_kv_stride;
  Pm.n_pages_pool = dims->n_pages;
  Pm.n_ref_slots = dims->n_ref_slots;
  Pm.w_up_k = static_cast<const uint16_t*>(w_up_k);
  Pm.w_up_v = static_cast<const uint16_t*>(w_up_v);
  Pm.q = static_cast<const uint16_t*>(q);
  Pm.out = static_cast<uint16_t*>(out);
  Pm.lse = lse;
  Pm.batch = batch;
  Pm.Hkv = dims->n_kv_heads;
  Pm.Hq = dims->n_q_heads;
  Pm.G = G;
  Pm.Gp = Gp;
  Pm.R = R;
  Pm.stride = S;
  Pm.joint = dims->latent_mode == DELTAKV_JOINT;
  Pm.q4 = dims->latent_bits == 4;
  Pm.top_k = dims->top_k > 1 ? dims->top_k : 1;
  Pm.max_seq_len = max_len;
  Pm.n_ref_max = n_ref_max;
  Pm.n_chunk_max = ceil_div(n_ref_max, kRefChunk);
  Pm.S = splits;
  Pm.pages_per_split = ceil_div(max_work, splits);
  Pm.sel_pages = sel.pages;
  Pm.sel_masks = sel.masks;
  Pm.n_sel = sel.n_sel;
  Pm.sel_stride = sel.stride;
  Pm.qk_scale_log2 = scale * kLog2e;
  char* wsb = static_cast<char*>(workspace);
  Pm.status = reinterpret_cast<int32_t*>(wsb + ws.status);
  Pm.rescue = reinterpret_cast<int32_t*>(wsb + ws.rescue);
  Pm.qlat = reinterpret_cast<uint16_t*>(wsb + ws.qlat);
  Pm.qlat_lo_offset = (int64_t)batch * dims->n_q_heads * R;
  Pm.sref = reinterpret_cast<float*>(wsb + ws.sref);
  Pm.cmax = reinterpret_cast<float*>(wsb + ws.cmax);
  Pm.lpart = reinterpret_cast<float*>(wsb + ws.lpart);
  Pm.wflag = reinterpret_cast<int32_t*>(wsb + ws.wflag);
  Pm.items = reinterpret_cast<int32_t*>(wsb + ws.items);
  Pm.accpart = reinterpret_cast<float*>(wsb + ws.accpart);
  Pm.opart = reinterpret_cast<float*>(wsb + ws.opart);
  Pm.wpart = reinterpret_cast<float*>(wsb + ws.wpart);
  Pm.spill = reinterpret_cast<float*>(wsb + ws.spill);
  Pm.tab_cap = (int)tab_cap;
  Pm.spill_on = spill_on;
  Pm.rawo = reinterpret_cast<float*>(wsb + ws.rawo);
  Pm.rawml = reinterpret_cast<float*>(wsb + ws.rawml);
  if (raw.cap > 0) {
    Pm.raw_k = static_cast<const uint16_t*>(raw.k);
    Pm.raw_v = static_cast<const uint16_t*>(raw.v);
    Pm.raw_lens = raw.lens;
    Pm.raw_cap = raw.cap;
  }
  // latent bytes the call streams (pages x heads x page block); beyond what the last-level cache (256 MB) can keep
  // for the next call, the records go through the caches as non-temporal loads
  Pm.nt = total_pages * lay->latent_head_stride * 2 > (192ll << 20);
  // ref_scores: four reference chunks per block when that still leaves two blocks per compute unit and the sequences
  // are about equally long (blocks of four chunks balance badly over a ragged batch)
  {
    int64_t chunks = 0;
    for (int b = 0; b < batch; ++b) chunks += ceil_div(ceil_div(seq_lens_host[b], S), kRefChunk);
    const int64_t grid1 = (int64_t)Pm.n_chunk_max * batch;
    Pm.ref_cpb = grid1 * dims->n_kv_heads >= 2048 && Pm.n_chunk_max >= 4 && chunks * 10 >= grid1 * 9 ? 4 : 1;
    if (g_tune_ref_chunks) Pm.ref_cpb = g_tune_ref_chunks;
  }
  // the streaming kernel runs one block per non-empty (sequence, split, kv-head); the kernels derive the same list
  // from the device copy of the lengths
  int64_t n_items = 0;
  for (int b = 0; b < batch; ++b) n_items += used_splits(work_pages(b), Pm.S, Pm.pages_per_split);
  hipError_t e = launch_decode(Pm, batch, (int)n_items, nw, lds, static_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue && g_detail[0] == 0) return DELTAKV_E_UNSUPPORTED;   // no kernel variant for this shape
  return e == hipSuccess ? DELTAKV_OK : DELTAKV_E_HIP;
}

int deltakv_decode_attn(const deltakv_dims* dims, const deltakv_layout* lay, const void* latent_pool,
                        const int32_t* idx_pool, const void* ref_pool, const int32_t* block_tables,
                        int32_t bt_stride, const int32_t* ref_tables, int32_t rt_stride, const void* w_up_k,
                        const void* w_up_v, const void* q, const int32_t* seq_lens,
                        const int32_t* seq_lens_host, int32_t batch, float scale, void* out, float* lse,
                        void* workspace, int64_t ws_bytes, void* stream) {
  return decode_impl(dims, lay, latent_pool, idx_pool, ref_pool, block_tables, bt_stride, ref_tables, rt_stride,
                     w_up_k, w_up_v, q, seq_lens, seq_lens_host, Selection{}, RawSegment{}, batch, scale, out, lse, workspace,
                     ws_bytes, stream);
}

int deltakv_decode_attn_subset(const deltakv_dims* dims, const deltakv_layout* lay, const void* latent_pool,
                               const int32_t* idx_pool, const void* ref_pool, const int32_t* block_tables,
                               int32_t bt_stride, const int32_t* ref_tables, int32_t rt_stride,
                               const void* w_up_k, const void* w_up_v, const void* q, const int32_t* seq_lens,
                               const int32_t* seq_lens_host, const int32_t* sel_pages, const int32_t* sel_masks,
                               int32_t sel_stride, const int32_t* n_sel, const int32_t* n_sel_host, int32_t batch,
                               float scale, void* out, float* lse, void* workspace, int64_t ws_bytes,
                               void* stream) {
  if (!sel_pages || !sel_masks || !n_sel || !n_sel_host || sel_stride <= 0) return DELTAKV_E_INVALID_ARG;
  for (int b = 0; b < batch; ++b)
    if (n_sel_host[b] < 0 || n_sel_host[b] > sel_stride) return DELTAKV_E_INVALID_ARG;
  Selection sel;
  sel.pages = sel_pages;
  sel.masks = sel_masks;
  sel.n_sel = n_sel;
  sel.n_sel_host = n_sel_host;
  sel.stride = sel_stride;
  return decode_impl(dims, lay, latent_pool, idx_pool, ref_pool, block_tables, bt_stride, ref_tables, rt_stride,
                     w_up_k, w_up_v, q, seq_lens, seq_lens_host, sel, RawSegment{}, batch, scale, out, lse, workspace,
                     ws_bytes, stream);
}

int deltakv_decode_attn_raw(const deltakv_dims* dims, const deltakv_layout* lay, const void* latent_pool,
                            const int32_t* idx_pool, const void* ref_pool, const int32_t* block_tables,
                            int32_t bt_stride, const int32_t* ref_tables, int32_t rt_stride, const void* w_up_k,
                            const void* w_up_v, const void* q, const int32_t* seq_lens,
                            const int32_t* seq_lens_host, const int32_t* sel_pages, const int32_t* sel_masks,
                            int32_t sel_stride, const int32_t* n_sel, const int32_t* n_sel_host, const void* raw_k,
                            const void* raw_v, const int32_t* raw_lens, int32_t raw_cap, int32_t batch, float scale,
                            void* out, float* lse, void* workspace, int64_t ws_bytes, void* stream) {
  Selection sel;
  if (sel_pages) {
    if (!sel_masks || !n_sel || !n_sel_host || sel_stride <= 0) return DELTAKV_E_INVALID_ARG;
    for (int b = 0; b < batch; ++b)
      if (n_sel_host[b] < 0 || n_sel_host[b] > sel_stride) return DELTAKV_E_INVALID_ARG;
    sel.pages = sel_pages;
    sel.masks = sel_masks;
    sel.n_sel = n_sel;
    sel.n_sel_host = n_sel_host;
    sel.stride = sel_stride;
  }
  RawSegment raw;
  raw.k = raw_k;
  raw.v = raw_v;
  raw.lens = raw_lens;
  raw.cap = raw_cap;
  return decode_impl(dims, lay, latent_pool, idx_pool, ref_pool, block_tables, bt_stride, ref_tables, rt_stride,
                     w_up_k, w_up_v, q, seq_lens, seq_lens_host, sel, raw, batch, scale, out, lse, workspace,
                     ws_bytes, stream);
}

// ---- decode attention for callers that cannot allocate ------------------------------------------------------
// The workspace of this entry point is an array in the library's own device image: every GPU the library runs on
// holds one copy from the moment the image is loaded until the process ends.  Host code never uses the array's
// name as an address (on the host it is only a handle for the runtime's symbol table): the device address is asked
// for once per device, with that device current, and kept.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[DELTAKV_STATIC_WS_BYTES];
namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

int deltakv_decode_attn_static(const deltakv_dims* dims, const deltakv_layout* lay, const void* latent_pool,
                               const int32_t* idx_pool, const void* ref_pool, const int32_t* block_tables,
                               int32_t bt_stride, const int32_t* ref_tables, int32_t rt_stride, const void* w_up_k,
                               const void* w_up_v, const void* q, const int32_t* seq_lens,
                               const int32_t* seq_lens_host, int32_t batch, float scale, void* out, float* lse,
                               void* stream) {
  int dev = -1;
  if (note_hip_error(hipGetDevice(&dev), "hipGetDevice") != hipSuccess) return DELTAKV_E_HIP;
  if (dev < 0 || dev >= kMaxDevices) return DELTAKV_E_UNSUPPORTED;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (note_hip_error(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(static workspace)") !=
            hipSuccess || !ptr)
      return DELTAKV_E_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  const int rc = decode_impl(dims, lay, latent_pool, idx_pool, ref_pool, block_tables, bt_stride, ref_tables, rt_stride,
                             w_up_k, w_up_v, q, seq_lens, seq_lens_host, Selection{}, RawSegment{}, batch, scale, out,
                             lse, g_scratch_ptr[dev], DELTAKV_STATIC_WS_BYTES, stream);
  if (rc == DELTAKV_E_WORKSPACE)
    snprintf(g_detail, sizeof(g_detail),
             "this batch and these sequence lengths need more than the %lld bytes of the static workspace; use "
             "deltakv_decode_attn with a caller-provided workspace", (long long)DELTAKV_STATIC_WS_BYTES);
  return rc;
}

int deltakv_decode_attn_rope(const deltakv_dims* dims, const deltakv_layout* lay, const void* latent_pool,
                             const int32_t* idx_pool, const void* ref_pool, const int32_t* block_tables,
                             int32_t bt_stride, const int32_t* ref_tables, int32_t rt_stride, const void* w_up_k,
                             const void* w_up_v, const void* q_rot, const int32_t* seq_lens,
                             const int32_t* seq_lens_host, int32_t batch, float scale, float rope_base, void* out,
                             float* lse, void* workspace, int64_t ws_bytes, void* stream) {
  int rc = check_dims(dims);
  if (rc != DELTAKV_OK) return rc;
  if (!lay || !latent_pool || !idx_pool || !ref_pool || !block_tables || !ref_tables || !w_up_k || !w_up_v ||
      !q_rot || !seq_lens || !seq_lens_host || !out || batch < 0 || bt_stride <= 0 || rt_stride <= 0 ||
      !(scale == scale) || !(rope_base > 1.0f))
    return DELTAKV_E_INVALID_ARG;
  const int G = dims->n_q_heads / dims->n_kv_heads, Gp = padded_group(G);
  if (dims->latent_bits == 4 || dims->top_k > 1 || Gp > 8) return DELTAKV_E_UNSUPPORTED;
  if (batch == 0) return DELTAKV_OK;
  if (batch > 65535) return DELTAKV_E_UNSUPPORTED;
  if (!workspace || !aligned(workspace, 256) || ws_bytes <= 0) return DELTAKV_E_WORKSPACE;
  if (!aligned(latent_pool, 16) || !aligned(idx_pool, 16) || !aligned(ref_pool, 16) || !aligned(q_rot, 16) ||
      !aligned(w_up_k, 16) || !aligned(w_up_v, 16))
    return DELTAKV_E_INVALID_ARG;
  int max_len = 0;
  int64_t total_pages = 0;
  for (int b = 0; b < batch; ++b) {
    if (seq_lens_host[b] < 0) return DELTAKV_E_INVALID_ARG;
    if (seq_lens_host[b] > max_len) max_len = seq_lens_host[b];
    total_pages += ceil_div(seq_lens_host[b], dims->page_tokens);
  }
  const int max_pages = ceil_div(max_len > 0 ? max_len : 1, dims->page_tokens);
  const int n_ref_max = ceil_div(max_len > 0 ? max_len : 1, dims->ref_stride);
  if (max_pages > bt_stride || n_ref_max > rt_stride) return DELTAKV_E_INVALID_ARG;
  if ((int64_t)max_pages > dims->n_pages || (int64_t)n_ref_max > dims->n_ref_slots) return DELTAKV_E_INVALID_ARG;
  if (rope_lds_bytes(dims->rank, Gp) > device_lds_limit()) return DELTAKV_E_UNSUPPORTED;
  // token-range splits: about two blocks' worth of work per compute unit over the whole batch (measured at 8 x 131072
  // tokens: 1.056 ms with 8 splits, 1.077 with 12, 1.095 with 16, 1.171 with 32), at least 32 pages each
  int64_t want = ceil_div64(2ll * device_cu_count(), (int64_t)batch * dims->n_kv_heads);
  int splits = (int)(want < 1 ? 1 : (want > kMaxSplits ? kMaxSplits : want));
  const int split_cap = max_pages / 32 > 1 ? max_pages / 32 : 1;
  if (splits > split_cap) splits = split_cap;
  if (g_tune_splits) splits = g_tune_splits < split_cap ? g_tune_splits : split_cap;
  RopeWs ws = plan_rope_ws(*dims, batch, max_pages, splits);
  while (ws.total > ws_bytes && splits > 1) ws = plan_rope_ws(*dims, batch, max_pages, --splits);
  if (ws.total > ws_bytes) return DELTAKV_E_WORKSPACE;
  DecodeParams Pm;
  memset(&Pm, 0, sizeof(Pm));
  Pm.latent = static_cast<const uint16_t*>(latent_pool);
  Pm.idx = idx_pool;
  Pm.ref = static_cast<const uint16_t*>(ref_pool);
  Pm.block_tables = block_tables;
  Pm.ref_tables = ref_tables;
  Pm.seq_lens = seq_lens;
  Pm.bt_stride = bt_stride;
  Pm.rt_stride = rt_stride;
  Pm.latent_page_stride = lay->latent_page_stride;
  Pm.latent_head_stride = lay->latent_head_stride;
  Pm.latent_stream_stride = lay->latent_stream_stride;
  Pm.idx_page_stride = lay->idx_page_stride;
  Pm.idx_head_stride = lay->idx_head_stride;
  Pm.ref_head_stride = lay->ref_head_stride;
  Pm.ref_kv_stride = lay->ref_kv_stride;
  Pm.n_pages_pool = dims->n_pages;
  Pm.n_ref_slots = dims->n_ref_slots;
  Pm.w_up_k = static_cast<const uint16_t*>(w_up_k);
  Pm.w_up_v = static_cast<const uint16_t*>(w_up_v);
  Pm.q = static_cast<const uint16_t*>(q_rot);
  Pm.out = static_cast<uint16_t*>(out);
  Pm.lse = lse;
  Pm.batch = batch;
  Pm.Hkv = dims->n_kv_heads;
  Pm.Hq = dims->n_q_heads;
  Pm.G = G;
  Pm.Gp = Gp;
  Pm.R = dims->rank;
  Pm.stride = dims->ref_stride;
  Pm.joint = dims->latent_mode == DELTAKV_JOINT;
  Pm.top_k = 1;
  Pm.max_seq_len = max_len;
  Pm.n_ref_max = n_ref_max;
  Pm.S = splits;
  Pm.pages_per_split = ceil_div(max_pages, splits);
  Pm.qk_scale_log2 = scale * kLog2e;
  char* wsb = static_cast<char*>(workspace);
  Pm.lpart = reinterpret_cast<float*>(wsb + ws.ml);
  Pm.accpart = reinterpret_cast<float*>(wsb + ws.acc);
  hipError_t e = launch_rope(Pm, reinterpret_cast<float2*>(wsb + ws.tab), max_pages, rope_base, batch,
                             static_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue && g_detail[0] == 0) return DELTAKV_E_UNSUPPORTED;
  return e == hipSuccess ? DELTAKV_OK : DELTAKV_E_HIP;
}

static int compress_impl(const deltakv_dims* dims, const deltakv_layout* lay, void* latent_pool, int32_t* idx_pool,
                         void* ref_pool, float* ref_inv_norm, const int32_t* block_tables, int32_t bt_stride,
                         const int32_t* ref_tables, int32_t rt_stride, const void* w_down_k, const void* w_down_v,
                         const deltakv_mlp* mlp,
                         const void* k_new, const void* v_new, const int32_t* cu_new, const int32_t* cu_new_host,
                         const int32_t* len_before, const int32_t* len_before_host, int32_t batch, void* workspace,
                         int64_t ws_bytes, void* stream) {
  int rc = check_dims(dims);
  if (rc != DELTAKV_OK) return rc;
  if (!lay || !latent_pool || !idx_pool || !ref_pool || !ref_inv_norm || !block_tables || !ref_tables ||
      !k_new || !v_new || !cu_new || !cu_new_host || !len_before ||
      !len_before_host || batch < 0 || bt_stride <= 0 || rt_stride <= 0)
    return DELTAKV_E_INVALID_ARG;
  if (mlp) {
    if (mlp->kind != DELTAKV_MLP_GELU && mlp->kind != DELTAKV_MLP_SWIGLU) return DELTAKV_E_INVALID_ARG;
    if (!mlp->w1 || !mlp->b1 || !mlp->w2 || (mlp->kind == DELTAKV_MLP_SWIGLU && !mlp->wg)) return DELTAKV_E_INVALID_ARG;
    if (mlp->hidden < 1) return DELTAKV_E_INVALID_ARG;
    if (!aligned(mlp->w1, 2) || !aligned(mlp->w2, 2) || !aligned(mlp->b1, 4) || (mlp->wg && !aligned(mlp->wg, 2)))
      return DELTAKV_E_INVALID_ARG;
    // one latent over K||V, stored as bf16, against one reference
    if (mlp->hidden > kMlpHiddenMax || dims->latent_mode != DELTAKV_JOINT || dims->latent_bits == 4 || dims->top_k > 1)
      return DELTAKV_E_UNSUPPORTED;
  } else if (!w_down_k || !w_down_v || !aligned(w_down_k, 2) || !aligned(w_down_v, 2)) {
    return DELTAKV_E_INVALID_ARG;
  }
  if (batch == 0) return DELTAKV_OK;
  if (batch > 65535 / dims->n_kv_heads) return DELTAKV_E_UNSUPPORTED;
  if (rt_stride > (1 << 24)) return DELTAKV_E_UNSUPPORTED;   // exact-pass keys carry 24-bit ordinals
  if (!aligned(latent_pool, 16) || !aligned(idx_pool, 16) || !aligned(ref_pool, 16) || !aligned(k_new, 16) ||
      !aligned(v_new, 16))
    return DELTAKV_E_INVALID_ARG;
  if (cu_new_host[0] != 0) return DELTAKV_E_INVALID_ARG;
  const int P = dims->page_tokens, S = dims->ref_stride;
  int max_new = 0, page_tiles_max = 0, max_new_refs = 0;
  int64_t tiles_total_rows = 0;
  for (int b = 0; b < batch; ++b) {
    const int64_t nb = (int64_t)cu_new_host[b + 1] - cu_new_host[b];
    const int64_t lb = len_before_host[b];
    if (nb < 0 || lb < 0 || lb + nb > (1ll << 30)) return DELTAKV_E_INVALID_ARG;
    if (nb == 0) continue;
    const int64_t la = lb + nb;
    if (ceil_div64(la, P) > bt_stride || ceil_div64(la, S) > rt_stride) return DELTAKV_E_INVALID_ARG;
    if (ceil_div64(la, P) > dims->n_pages || ceil_div64(la, S) > dims->n_ref_slots) return DELTAKV_E_INVALID_ARG;
    if (nb > max_new) max_new = (int)nb;
    const int pt = (int)(ceil_div64(la, P) - lb / P);
    if (pt > page_tiles_max) page_tiles_max = pt;
    const int nr = (int)(ceil_div64(la, S) - ceil_div64(lb, S));
    if (nr > max_new_refs) max_new_refs = nr;
    tiles_total_rows += nb;
  }
  const int n_new_total = cu_new_host[batch];
  if (n_new_total == 0) return DELTAKV_OK;
  if (!workspace || !aligned(workspace, 256) || ws_bytes <= 0) return DELTAKV_E_WORKSPACE;
  // long calls: eight waves (two per SIMD, so one wave's top-2 arithmetic runs under the other's matrix
  // instructions) of two 16-token blocks each; short calls: four waves, smaller tiles
  const int rb = g_tune_sim_tb ? g_tune_sim_tb : (max_new >= 128 ? 2 : 1);
  const int sim_nw = g_tune_sim_waves ? g_tune_sim_waves : (max_new >= 1024 ? 8 : 4);
  const int mt = sim_tile_rows(rb, sim_nw);
  const int tiles_max = ceil_div(max_new, mt);
  int64_t tiles_total = 0;
  int64_t max_len_after = 0;
  for (int b = 0; b < batch; ++b) {
    const int64_t nb = (int64_t)cu_new_host[b + 1] - cu_new_host[b];
    tiles_total += ceil_div64(nb, mt);
    if (nb > 0 && len_before_host[b] + nb > max_len_after) max_len_after = len_before_host[b] + nb;
  }
  // spread the reference scan of small calls (decode append) over enough blocks to fill the chip
  int64_t ns = ceil_div64(4ll * device_cu_count(), tiles_total * dims->n_kv_heads);
  const int64_t ref_tiles = ceil_div64(ceil_div64(max_len_after, S), 64);
  if (g_tune_sim_ns) ns = g_tune_sim_ns;
  if (ns > ref_tiles) ns = ref_tiles;
  if (ns > 64) ns = 64;
  const CompressWs cw = plan_compress_ws(*dims, batch, n_new_total, 0);
  const int64_t per_split = (int64_t)n_new_total * dims->n_kv_heads * 16;
  if (ws_bytes < cw.part + per_split) return DELTAKV_E_WORKSPACE;
  if (ns > (ws_bytes - cw.part) / per_split) ns = (ws_bytes - cw.part) / per_split;
  if (ns < 1) return DELTAKV_E_WORKSPACE;
  if (tiles_max > 65535 || page_tiles_max <= 0) return DELTAKV_E_UNSUPPORTED;   // grid z of the similarity kernel

  CompressParams Pm;
  memset(&Pm, 0, sizeof(Pm));
  Pm.latent = static_cast<uint16_t*>(latent_pool);
  Pm.idx = idx_pool;
  Pm.ref = static_cast<uint16_t*>(ref_pool);
  Pm.ref_inv_norm = ref_inv_norm;
  Pm.block_tables = block_tables;
  Pm.ref_tables = ref_tables;
  Pm.bt_stride = bt_stride;
  Pm.rt_stride = rt_stride;
  Pm.latent_page_stride = lay->latent_page_stride;
  Pm.latent_head_stride = lay->latent_head_stride;
  Pm.latent_stream_stride = lay->latent_stream_stride;
  Pm.idx_page_stride = lay->idx_page_stride;
  Pm.idx_head_stride = lay->idx_head_stride;
  Pm.ref_head_stride = lay->ref_head_stride;
  Pm.ref_kv_stride = lay->ref_kv_stride;
  Pm.ref_norm_head_stride = lay->ref_norm_head_stride;
  Pm.n_pages_pool = dims->n_pages;
  Pm.n_ref_slots = dims->n_ref_slots;
  Pm.w_down_k = static_cast<const uint16_t*>(w_down_k);
  Pm.w_down_v = static_cast<const uint16_t*>(w_down_v);
  Pm.k_new = static_cast<const uint16_t*>(k_new);
  Pm.v_new = static_cast<const uint16_t*>(v_new);
  Pm.cu_new = cu_new;
  Pm.len_before = len_before;
  Pm.batch = batch;
  Pm.n_new_total = n_new_total;
  Pm.Hkv = dims->n_kv_heads;
  Pm.R = dims->rank;
  Pm.stride = S;
  Pm.joint = dims->latent_mode == DELTAKV_JOINT;
  Pm.q4 = dims->latent_bits == 4;
  Pm.metric = dims->metric;
  Pm.top_k = dims->top_k > 1 ? dims->top_k : 1;
  Pm.idx_slot_stride = lay->idx_slot_stride;
  Pm.NS = (int)ns;
  char* wsb = static_cast<char*>(workspace);
  Pm.ord = reinterpret_cast<int32_t*>(wsb + cw.ord);
  Pm.flag_count = reinterpret_cast<int32_t*>(wsb + cw.flag_count);
  Pm.flag_list = reinterpret_cast<int32_t*>(wsb + cw.flag_list);
  Pm.exact_key = reinterpret_cast<uint64_t*>(wsb + cw.exact_key);
  Pm.part = reinterpret_cast<float*>(wsb + cw.part);
  Pm.wt = reinterpret_cast<uint16_t*>(wsb + cw.wt);
  Pm.ord_all = Pm.ord;
  Pm.exact_key_all = Pm.exact_key;
  Pm.flag_count_all = Pm.flag_count;
  Pm.round_stride = (int64_t)n_new_total * dims->n_kv_heads;
  Pm.mlp_kind = -1;
  if (mlp) {
    Pm.mlp_kind = mlp->kind;
    Pm.mlp_hidden = mlp->hidden;
    Pm.mlp_hidden_pad = (int)align_up(mlp->hidden, kMlpChunk);
    Pm.mlp_w1 = static_cast<const uint16_t*>(mlp->w1);
    Pm.mlp_wg = static_cast<const uint16_t*>(mlp->wg);
    Pm.mlp_w2 = static_cast<const uint16_t*>(mlp->w2);
    Pm.mlp_b1 = mlp->b1;
    char* mb = wsb + cw.mlp;
    const int64_t w1_bytes = align_up((int64_t)Pm.mlp_hidden_pad * kMlpXPad * 2, 256);
    Pm.mlp_w1t = reinterpret_cast<uint16_t*>(mb);
    Pm.mlp_wgt = reinterpret_cast<uint16_t*>(mb + w1_bytes);
    Pm.mlp_w2t = reinterpret_cast<uint16_t*>(mb + 2 * w1_bytes);
    Pm.mlp_b1p = reinterpret_cast<float*>(mb + 2 * w1_bytes +
                                          align_up((int64_t)(Pm.mlp_hidden_pad / kMlpChunk) * mlp_w2_chunk_elems(dims->rank) * 2, 256));
  }
  // decode append (one new token for every sequence): two small kernels instead of five
  bool one_each = n_new_total == batch && Pm.top_k == 1 && !mlp;   // (top-k and the non-linear compressor: general path)
  for (int b = 0; b < batch && one_each; ++b) one_each = cu_new_host[b + 1] - cu_new_host[b] == 1;
  hipError_t e;
  if (one_each) {
    int64_t nsa = ceil_div64(ceil_div64(max_len_after, S), 64);      // about 64 candidates per block
    const int64_t cap = (ws_bytes - cw.part) / per_split;
    if (nsa > 64) nsa = 64;
    if (nsa > cap) nsa = cap;
    Pm.NS = nsa < 1 ? 1 : (int)nsa;
    e = launch_append(Pm, static_cast<hipStream_t>(stream));
  } else {
    // pages per block of the projection kernel: up to four while that leaves two blocks per compute unit (measured
    // on a 32768-token prompt, 2048 pages: 69, 64, 60, 74 us with 1, 2, 4, 8 pages per block)
    {
      const int64_t q = (int64_t)page_tiles_max * batch / 512;
      Pm.proj_ppb = q >= 4 ? 4 : (q >= 2 ? 2 : 1);
    }
    if (g_tune_project_pages) Pm.proj_ppb = g_tune_project_pages;
    e = launch_compress(Pm, cw, wsb, rb, sim_nw, tiles_max, page_tiles_max, max_new_refs, static_cast<hipStream_t>(stream));
  }
  return e == hipSuccess ? DELTAKV_OK : DELTAKV_E_HIP;
}

int deltakv_compress(const deltakv_dims* dims, const deltakv_layout* lay, void* latent_pool, int32_t* idx_pool,
                     void* ref_pool, float* ref_inv_norm, const int32_t* block_tables, int32_t bt_stride,
                     const int32_t* ref_tables, int32_t rt_stride, const void* w_down_k, const void* w_down_v,
                     const void* k_new, const void* v_new, const int32_t* cu_new, const int32_t* cu_new_host,
                     const int32_t* len_before, const int32_t* len_before_host, int32_t batch, void* workspace,
                     int64_t ws_bytes, void* stream) {
  return compress_impl(dims, lay, latent_pool, idx_pool, ref_pool, ref_inv_norm, block_tables, bt_stride, ref_tables,
                       rt_stride, w_down_k, w_down_v, nullptr, k_new, v_new, cu_new, cu_new_host, len_before,
                       len_before_host, batch, workspace, ws_bytes, stream);
}

int deltakv_compress_mlp(const deltakv_dims* dims, const deltakv_layout* lay, void* latent_pool, int32_t* idx_pool,
                         void* ref_pool, float* ref_inv_norm, const int32_t* block_tables, int32_t bt_stride,
                         const int32_t* ref_tables, int32_t rt_stride, const deltakv_mlp* mlp,
                         const void* k_new, const void* v_new, const int32_t* cu_new, const int32_t* cu_new_host,
                         const int32_t* len_before, const int32_t* len_before_host, int32_t batch, void* workspace,
                         int64_t ws_bytes, void* stream) {
  if (!mlp) return DELTAKV_E_INVALID_ARG;
  return compress_impl(dims, lay, latent_pool, idx_pool, ref_pool, ref_inv_norm, block_tables, bt_stride, ref_tables,
                       rt_stride, nullptr, nullptr, mlp, k_new, v_new, cu_new, cu_new_host, len_before,
                       len_before_host, batch, workspace, ws_bytes, stream);
}

}  // extern "C"
