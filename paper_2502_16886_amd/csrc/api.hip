// C-ABI layer of librfkv: host-side validation, launch geometry, workspace carving and the
// kernel launch sequences.  The contract of every entry point is documented in include/rfkv.h.
#include "../../include/rfkv.h"
#include "../../include/rfkv_bench.h"

#include <cmath>
#include <cstring>

#include "kernels.h"

#include <mutex>

// Scratch of rfkv_compress_layer_static.  In host code this name is only a handle for
// hipGetSymbolAddress: the device address (one per GPU) is looked up once per device and used from
// then on wherever the array's memory is meant.
static __device__ __align__(256) unsigned char scratch[RFKV_STATIC_SCRATCH_BYTES];

namespace rfkv {

static thread_local int32_t g_last_device_error = 0;

// Device address of `scratch` on the current device, looked up on the first call on that device.
static hipError_t static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Workspace carve_workspace(const Geometry& g, void* base) {
  Workspace w{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* p = base ? static_cast<unsigned char*>(base) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  w.partials = static_cast<float2*>(take((size_t)g.units * g.nspans * g.rows_pad * sizeof(float2)));
  w.bvec = static_cast<float*>(take((size_t)g.units * g.rows_pad * sizeof(float)));
  w.desc = static_cast<int4*>(take((size_t)g.units * sizeof(int4)));
  w.idx_pad = static_cast<int32_t*>(take((size_t)g.total_tokens * g.n_kv_heads * sizeof(int32_t)));
  w.scores = static_cast<float*>(take((size_t)g.total_tokens * g.n_kv_heads * sizeof(float)));
  w.tile_sq = static_cast<double*>(take((size_t)g.tiles_total * g.n_kv_heads * sizeof(double)));
  if (g.spill) w.logits = static_cast<float*>(take((size_t)g.tiles_total * 32 * kSpillRows * g.n_kv_heads * sizeof(float)));
  w.counters = static_cast<int32_t*>(take((size_t)2 * g.units * sizeof(int32_t)));
  if (g.score_slices > 0) {
    w.sel_block = static_cast<uint32_t*>(take((size_t)g.units * kSelWords * sizeof(uint32_t)));
  }
  if (g.per_layer) {
    w.sort_keys = static_cast<uint32_t*>(take((size_t)2 * g.total_tokens * g.n_kv_heads * sizeof(uint32_t)));
    w.sorted_scores = static_cast<float*>(take((size_t)g.total_tokens * g.n_kv_heads * sizeof(float)));
  }
  w.bytes = off;
  return w;
}

namespace {

// Score rows per KV head as the kernels lay them out: a multiple of 32, and up to 256 one of the
// sizes the streaming kernels are instantiated for (1, 2, 4 or 8 row tiles), so that a kernel's
// row tiles and the per-row tables in the workspace always coincide.
int64_t padded_rows(int64_t rows) {
  const int64_t r32 = (rows + 31) / 32 * 32;
  if (r32 > 64 && r32 <= 128) return 128;
  if (r32 > 128 && r32 <= 256) return 256;
  return r32;
}

// keys one score workgroup covers: enough workgroups to fill 256 CUs a few times over, but long
// enough that staging the window queries (once per workgroup) stays a small part of its traffic
int32_t choose_span(int64_t total_tokens, int32_t n_kv_heads, int max_iters) {
  const int64_t work = total_tokens * n_kv_heads;      // keys to score in the layer
  int64_t span = (work / 1024 + kKeysPerIter - 1) / kKeysPerIter * kKeysPerIter;
  if (span < 2 * kKeysPerIter) span = 2 * kKeysPerIter;
  if (span > (int64_t)max_iters * kKeysPerIter) span = (int64_t)max_iters * kKeysPerIter;
  return (int32_t)span;
}

// The wide-window kernels (row-blocked statistics, key-resident column sums) take every window the
// streaming kernels cannot hold, and, where their 256-byte row limit allows, every window of more
// than 128 score rows: from 5 to 8 row tiles they already beat the streaming kernels, which would
// have to re-read part of the queries from LDS for every key tile.
constexpr int kWideAbove = 128;
bool wide_window(const rfkv_params* p) {
  const int64_t rows = (int64_t)p->window * (p->n_q_heads / p->n_kv_heads);
  const int64_t rows32 = (rows + 31) / 32 * 32;
  const int eb = p->dtype == RFKV_DTYPE_BF16 ? 2 : 4;
  if (rows32 > RFKV_MAX_SCORE_ROWS) return true;
  return rows32 > kWideAbove && p->head_dim * eb <= 256;
}

rfkv_status check_params(const rfkv_params* p) {
  if (!p) return RFKV_INVALID_ARG;
  if (p->batch < 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->window < 1 || p->n_sink < 0 ||
      p->min_keep < 0)
    return RFKV_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return RFKV_INVALID_ARG;
  if (!(p->softmax_scale >= 0.f) || !std::isfinite(p->softmax_scale)) return RFKV_INVALID_ARG;
  if (std::isnan(p->threshold)) return RFKV_INVALID_ARG;
  if (p->rank_mode != RFKV_RANK_POSITION && p->rank_mode != RFKV_RANK_SCORE) return RFKV_INVALID_ARG;
  if (p->granularity != RFKV_PER_HEAD && p->granularity != RFKV_PER_LAYER) return RFKV_INVALID_ARG;
  if (p->out_pad_rows < 0) return RFKV_INVALID_ARG;
  if (p->dtype != RFKV_DTYPE_FP32 && p->dtype != RFKV_DTYPE_BF16) return RFKV_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return RFKV_UNSUPPORTED;
  const int64_t rows = (int64_t)p->window * (p->n_q_heads / p->n_kv_heads);
  if ((int64_t)p->batch * p->n_kv_heads > RFKV_MAX_UNITS) return RFKV_UNSUPPORTED;
  const int eb = p->dtype == RFKV_DTYPE_BF16 ? 2 : 4;
  if (wide_window(p)) {
    // row-blocked statistics keep 128 rows of queries in registers: 256-byte rows at most
    if (rows > RFKV_MAX_WIDE_ROWS || p->head_dim * eb > 256) return RFKV_UNSUPPORTED;
    return RFKV_OK;
  }
  // the window queries of one unit must fit in LDS next to the per-row tables
  const int64_t rows_pad = padded_rows(rows);
  if (rows_pad * (p->head_dim * eb + 16 + 8) > 156 * 1024) return RFKV_UNSUPPORTED;
  return RFKV_OK;
}

rfkv_status check_strides(const rfkv_params* p, bool need_q, bool need_k, bool need_v) {
  const int per16 = p->dtype == RFKV_DTYPE_BF16 ? 8 : 4;      // elements per 16 bytes
  auto ok = [&](int64_t tok, int64_t head) {
    return tok >= p->head_dim && head >= p->head_dim && tok % per16 == 0 && head % per16 == 0;
  };
  if (need_q && !ok(p->q_stride_row, p->q_stride_head)) return RFKV_INVALID_ARG;
  if (need_k && !ok(p->k_stride_tok, p->k_stride_head)) return RFKV_INVALID_ARG;
  if (need_v && !ok(p->v_stride_tok, p->v_stride_head)) return RFKV_INVALID_ARG;
  // the tile loaders add up to 127 token strides in 32-bit arithmetic
  if (need_k && p->k_stride_tok > RFKV_MAX_STRIDE_TOK) return RFKV_UNSUPPORTED;
  if (need_v && p->v_stride_tok > RFKV_MAX_STRIDE_TOK) return RFKV_UNSUPPORTED;
  return RFKV_OK;
}

bool aligned16(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

rfkv_status check_cu(const rfkv_params* p, const int32_t* cu_host, const int32_t* cu_dev, int64_t* total,
                     int32_t* max_len) {
  if (!cu_host || !cu_dev) return RFKV_INVALID_ARG;
  if (cu_host[0] != 0) return RFKV_INVALID_ARG;
  int32_t mx = 0;
  for (int b = 0; b < p->batch; ++b) {
    const int64_t len = (int64_t)cu_host[b + 1] - cu_host[b];
    if (len < 0) return RFKV_INVALID_ARG;
    if (len > mx) mx = (int32_t)len;
  }
  *total = cu_host[p->batch];
  *max_len = mx;
  if (*total * p->n_kv_heads >= (int64_t)1 << 31) return RFKV_UNSUPPORTED;   // int32 index lists
  return RFKV_OK;
}

Geometry make_geometry(const rfkv_params* p, int64_t total, int32_t max_len, const int32_t* cu_host = nullptr) {
  Geometry g{};
  g.batch = p->batch;
  g.n_q_heads = p->n_q_heads;
  g.n_kv_heads = p->n_kv_heads;
  g.group = p->n_q_heads / p->n_kv_heads;
  g.head_dim = p->head_dim;
  g.window = p->window;
  g.units = p->batch * p->n_kv_heads;
  g.rows_pad = (int32_t)padded_rows((int64_t)p->window * g.group);
  g.wide = wide_window(p) ? 1 : 0;
  if (g.wide) g.rows_pad = (g.rows_pad + 127) / 128 * 128;      // whole blocks of 128 rows (4 row tiles)
  // few score rows (the paper's k = 1): the first scoring pass keeps its logits, no second pass over K
  g.spill = (int64_t)p->window * g.group <= kSpillRows ? 1 : 0;
  // a wide window multiplies the statistics pass's workgroups by its row blocks: longer spans
  g.span = choose_span(g.wide ? total * (g.rows_pad / 128) / 2 : total, p->n_kv_heads, g.wide ? 64 : 16);
  g.nspans = (max_len + g.span - 1) / g.span;
  g.max_seqlen = max_len;
  g.score_slices = score_slices(max_len, g.units);      // whatever the ranking: a workspace serves both
  g.per_layer = p->granularity == RFKV_PER_LAYER ? 1 : 0;
  g.total_tokens = total;
  g.elem_bytes = p->dtype == RFKV_DTYPE_BF16 ? 2 : 4;
  // 32-position tiles per sequence; without the lengths, the bound every batch of this size obeys
  g.tiles_total = (total + 31) / 32 + p->batch;
  if (cu_host) {
    g.tiles_total = 0;
    for (int b = 0; b < p->batch; ++b) g.tiles_total += (cu_host[b + 1] - cu_host[b] + 31) / 32;
  }
  return g;
}

// The wide-window kernels index their work items (row block, span, unit) / (key block, unit) with 32-bit
// integers on a one-dimensional grid.
rfkv_status check_wide_grid(const Geometry& g) {
  if (!g.wide) return RFKV_OK;
  const int64_t stats_items = (int64_t)(g.rows_pad / 128) * g.nspans * g.units;
  const int64_t colsum_items = ((int64_t)g.max_seqlen + 511) / 512 * g.units;
  return stats_items > ((int64_t)1 << 30) || colsum_items > ((int64_t)1 << 30) ? RFKV_UNSUPPORTED : RFKV_OK;
}

rfkv_status device_status(hipError_t e) {
  if (e == hipSuccess) return RFKV_OK;
  g_last_device_error = (int32_t)e;
  return RFKV_DEVICE_ERROR;
}

float scale_times_log2e(const rfkv_params* p) {
  const double s = p->softmax_scale > 0.f ? (double)p->softmax_scale : 1.0 / std::sqrt((double)p->head_dim);
  return (float)(s * 1.4426950408889634);
}

// Can the scoring pass take the position-ranking cut itself (its streaming kernels can, unit by unit, in
// the workgroup that finishes a unit last)?  The layer pipeline needs that.
bool select_fuses(const rfkv_params* p, const Geometry& g) {
  return p->rank_mode == RFKV_RANK_POSITION && p->granularity == RFKV_PER_HEAD && !g.wide &&
         score_streams(g, p->dtype == RFKV_DTYPE_BF16);
}

ScoreArgs score_args(const rfkv_params* p, const Geometry& g, const Workspace& w, const void* q, const float* lse,
                     const void* k, const int32_t* cu_dev, float* scores, int32_t* kept_fused) {
  ScoreArgs a{};
  a.counters = w.counters;
  a.fuse_merge = kept_fused ? 1 : 0;                   // the layer pipeline: both hand-overs inside the launch
  a.fuse_select = kept_fused ? 1 : 0;
  a.n_sink = p->n_sink;
  a.min_keep = p->min_keep;
  a.threshold = p->threshold;
  a.kept = kept_fused;
  a.desc = w.desc;
  a.sel_block = p->rank_mode == RFKV_RANK_SCORE && g.score_slices > 0 ? w.sel_block : nullptr;
  a.q = q;
  a.lse = lse;
  a.n_q_heads = g.n_q_heads;
  a.k = k;
  a.scores = scores;
  a.cu = cu_dev;
  a.partials = w.partials;
  a.bvec = w.bvec;
  a.tile_sq = w.tile_sq;
  a.logits = g.spill ? w.logits : nullptr;
  a.tiles_total = g.tiles_total;
  a.k_stride_tok = p->k_stride_tok;
  a.k_stride_head = p->k_stride_head;
  a.q_stride_row = p->q_stride_row;
  a.q_stride_head = p->q_stride_head;
  a.total_tokens = g.total_tokens;
  a.n_kv_heads = g.n_kv_heads;
  a.group = g.group;
  a.window = g.window;
  a.rows_pad = g.rows_pad;
  a.span = g.span;
  a.nspans = g.nspans;
  a.units = g.units;
  a.wide_items = g.wide ? (g.rows_pad / 128) * g.nspans * g.units : 0;
  a.span_colsum = g.max_seqlen;
  a.c = scale_times_log2e(p);
  return a;
}

hipError_t run_score(const rfkv_params* p, const Geometry& g, const Workspace& w, const void* q, const float* lse,
                     const void* k, const int32_t* cu_dev, float* scores, hipStream_t stream,
                     const Marks* marks = nullptr, int32_t* kept_fused = nullptr) {
  return launch_score(g, score_args(p, g, w, q, lse, k, cu_dev, scores, kept_fused), p->dtype == RFKV_DTYPE_BF16,
                      stream, marks);
}

hipError_t run_select(const rfkv_params* p, const Geometry& g, const Workspace& w, const float* scores,
                      const int32_t* cu_dev, int32_t* kept, bool from_scores, hipStream_t stream) {
  SelectArgs a{};
  a.scores = scores;
  a.cu = cu_dev;
  a.kept = kept;
  a.desc = w.desc;
  a.idx_pad = p->rank_mode == RFKV_RANK_SCORE ? w.idx_pad : nullptr;
  a.tile_sq = w.tile_sq;
  a.tiles_total = g.tiles_total;
  a.from_scores = from_scores ? 1 : 0;
  a.total_tokens = g.total_tokens;
  a.n_kv_heads = g.n_kv_heads;
  a.n_sink = p->n_sink;
  a.min_keep = p->min_keep;
  a.rank_mode = p->rank_mode;
  a.threshold = p->threshold;
  a.per_layer = p->granularity == RFKV_PER_LAYER ? 1 : 0;
  a.sel_block = w.sel_block;
  a.units = g.units;
  a.sort_keys = w.sort_keys;
  a.sorted_scores = w.sorted_scores;
  return launch_select(g, a, stream);
}

CompactArgs compact_base(const rfkv_params* p, const Geometry& g, const int32_t* cu_dev, const int32_t* kept) {
  CompactArgs a{};
  a.cu = cu_dev;
  a.kept = kept;
  a.k_stride_tok = p->k_stride_tok * g.elem_bytes;
  a.k_stride_head = p->k_stride_head * g.elem_bytes;
  a.v_stride_tok = p->v_stride_tok * g.elem_bytes;
  a.v_stride_head = p->v_stride_head * g.elem_bytes;
  a.n_kv_heads = g.n_kv_heads;
  a.units = g.units;
  a.row_bytes = g.head_dim * g.elem_bytes;
  a.pad_rows = p->out_pad_rows;
  return a;
}

}  // namespace
}  // namespace rfkv

using namespace rfkv;

extern "C" {

int32_t rfkv_version(void) { return 200; }

const char* rfkv_status_string(rfkv_status status) {
  switch (status) {
    case RFKV_OK: return "ok";
    case RFKV_INVALID_ARG: return "invalid argument";
    case RFKV_UNSUPPORTED: return "unsupported problem";
    case RFKV_WORKSPACE_TOO_SMALL: return "workspace too small";
    case RFKV_OUTPUT_TOO_SMALL: return "output too small";
    case RFKV_DEVICE_ERROR: return "device error";
  }
  return "unknown status";
}

int32_t rfkv_last_device_error(void) { return g_last_device_error; }

size_t rfkv_workspace_bytes(const rfkv_params* params, int64_t total_tokens, int32_t max_seqlen) {
  if (check_params(params) != RFKV_OK || total_tokens < 0 || max_seqlen < 0 || max_seqlen > total_tokens) return 0;
  if (total_tokens * params->n_kv_heads >= (int64_t)1 << 31) return 0;
  const Geometry g = make_geometry(params, total_tokens, max_seqlen);
  return carve_workspace(g, nullptr).bytes + 256;
}

static rfkv_status score_impl(const rfkv_params* params, const void* q_win, const float* lse_win, bool with_lse,
                              const void* k, const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                              float* scores, void* ws, size_t ws_bytes, void* stream) {
  rfkv_status st = check_params(params);
  if (st != RFKV_OK) return st;
  if ((st = check_strides(params, true, true, false)) != RFKV_OK) return st;
  int64_t total;
  int32_t max_len;
  if ((st = check_cu(params, cu_seqlens_host, cu_seqlens_dev, &total, &max_len)) != RFKV_OK) return st;
  if (total == 0) return RFKV_OK;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(scores) || !aligned16(ws)) return RFKV_INVALID_ARG;
  if (with_lse && (!lse_win || (reinterpret_cast<uintptr_t>(lse_win) & 3u))) return RFKV_INVALID_ARG;
  const Geometry g = make_geometry(params, total, max_len, cu_seqlens_host);
  if ((st = check_wide_grid(g)) != RFKV_OK) return st;
  const Workspace w = carve_workspace(g, ws);
  if (ws_bytes < w.bytes) return RFKV_WORKSPACE_TOO_SMALL;
  return device_status(run_score(params, g, w, q_win, with_lse ? lse_win : nullptr, k, cu_seqlens_dev, scores,
                                 static_cast<hipStream_t>(stream)));
}

rfkv_status rfkv_score(const rfkv_params* params, const void* q_win, const void* k,
                       const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev, float* scores, void* ws,
                       size_t ws_bytes, void* stream) {
  return score_impl(params, q_win, nullptr, false, k, cu_seqlens_host, cu_seqlens_dev, scores, ws, ws_bytes, stream);
}

rfkv_status rfkv_score_lse(const rfkv_params* params, const void* q_win, const float* lse_win, const void* k,
                           const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev, float* scores, void* ws,
                           size_t ws_bytes, void* stream) {
  return score_impl(params, q_win, lse_win, true, k, cu_seqlens_host, cu_seqlens_dev, scores, ws, ws_bytes, stream);
}

rfkv_status rfkv_select(const rfkv_params* params, const float* scores, const int32_t* cu_seqlens_host,
                        const int32_t* cu_seqlens_dev, int32_t* kept, int64_t* out_offsets, int32_t* idx,
                        void* ws, size_t ws_bytes, void* stream) {
  rfkv_status st = check_params(params);
  if (st != RFKV_OK) return st;
  int64_t total;
  int32_t max_len;
  if ((st = check_cu(params, cu_seqlens_host, cu_seqlens_dev, &total, &max_len)) != RFKV_OK) return st;
  if (!kept || !out_offsets) return RFKV_INVALID_ARG;
  if (params->out_pad_rows > 0 && params->out_pad_rows < max_len) return RFKV_OUTPUT_TOO_SMALL;
  if (params->batch == 0) return RFKV_OK;
  if (!aligned16(ws)) return RFKV_INVALID_ARG;
  if (total > 0 && (!aligned16(scores) || !idx)) return RFKV_INVALID_ARG;
  const Geometry g = make_geometry(params, total, max_len, cu_seqlens_host);
  const Workspace w = carve_workspace(g, ws);
  if (ws_bytes < w.bytes) return RFKV_WORKSPACE_TOO_SMALL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = run_select(params, g, w, scores, cu_seqlens_dev, kept, true, s);
  if (e != hipSuccess) return device_status(e);
  CompactArgs c = compact_base(params, g, cu_seqlens_dev, kept);
  c.source = params->rank_mode == RFKV_RANK_SCORE ? kSrcPaddedIdx : kSrcPositionDesc;
  c.desc = w.desc;
  c.idx_pad = w.idx_pad;
  c.offsets_out = out_offsets;
  c.idx_out = idx;
  // the documented capacity of idx: every position of every head, or every slot of the padded layout
  c.idx_capacity = params->out_pad_rows > 0 ? (int64_t)g.units * params->out_pad_rows : total * params->n_kv_heads;
  return device_status(launch_compact(g, c, s));
}

rfkv_status rfkv_compact(const rfkv_params* params, const void* k, const void* v, const int32_t* cu_seqlens_host,
                         const int32_t* cu_seqlens_dev, const int32_t* kept, const int64_t* out_offsets,
                         const int32_t* idx, void* k_out, void* v_out, int64_t out_capacity_rows, void* stream) {
  rfkv_status st = check_params(params);
  if (st != RFKV_OK) return st;
  if ((st = check_strides(params, false, true, true)) != RFKV_OK) return st;
  int64_t total;
  int32_t max_len;
  if ((st = check_cu(params, cu_seqlens_host, cu_seqlens_dev, &total, &max_len)) != RFKV_OK) return st;
  if (out_capacity_rows < 0) return RFKV_INVALID_ARG;
  if (total == 0) return RFKV_OK;
  if (!kept || !out_offsets || !idx) return RFKV_INVALID_ARG;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out)) return RFKV_INVALID_ARG;
  const Geometry g = make_geometry(params, total, max_len, cu_seqlens_host);
  CompactArgs c = compact_base(params, g, cu_seqlens_dev, kept);
  c.k = k;
  c.v = v;
  c.k_out = k_out;
  c.v_out = v_out;
  c.source = kSrcPackedIdx;
  c.idx_packed = idx;
  c.offsets_in = out_offsets;
  c.capacity_rows = out_capacity_rows;
  return device_status(launch_compact(g, c, static_cast<hipStream_t>(stream)));
}

// Launch geometry of the decode attention: one work item per workgroup the chip holds at once
// (256 CUs, one workgroup each), plus one spare slot per unit for the planner's rounding.
static void decode_geometry(const rfkv_params* p, int32_t n_new, DecodeArgs* a) {
  const int units = p->batch * p->n_kv_heads;
  a->n_q_heads = p->n_q_heads;
  a->n_kv_heads = p->n_kv_heads;
  a->group = p->n_q_heads / p->n_kv_heads;
  a->n_new = n_new;
  a->rows = n_new * a->group;
  a->units = units;
  a->rows_pad = a->rows <= 128 ? 128 : 256;
  a->head_dim = p->head_dim;
  a->target_items = a->rows_pad <= 128 ? 512 : 256;
  a->max_items = a->target_items + units;
  a->c = scale_times_log2e(p);
}

struct DecodeWs {
  size_t part_o, part_ml, item_begin, bytes;
};
static DecodeWs decode_ws(const rfkv_params* p, const DecodeArgs& a) {
  const size_t units = (size_t)p->batch * p->n_kv_heads;
  const size_t slots = (size_t)a.max_items * a.rows_pad;
  DecodeWs w;
  w.part_o = 0;
  w.part_ml = w.part_o + slots * a.head_dim * sizeof(float);
  w.item_begin = w.part_ml + slots * sizeof(float2);
  w.bytes = (w.item_begin + (units + 1) * sizeof(int32_t) + 255) / 256 * 256;
  return w;
}

static rfkv_status decode_check(const rfkv_params* p, int32_t n_new) {
  const rfkv_status st = check_params(p);
  if (st != RFKV_OK) return st;
  if (n_new < 0) return RFKV_INVALID_ARG;
  if (p->dtype != RFKV_DTYPE_BF16) return RFKV_UNSUPPORTED;
  if ((int64_t)n_new * (p->n_q_heads / p->n_kv_heads) > RFKV_MAX_DECODE_ROWS) return RFKV_UNSUPPORTED;
  return RFKV_OK;
}

static rfkv_status decode_impl(const rfkv_params* params, const void* q_new, int32_t n_new, const void* k,
                               const void* v, const int32_t* cu_host, const int32_t* cu_dev,
                               const int64_t* out_offsets, const int32_t* kept, const uint8_t* keep_mask, bool masked,
                               float* out, void* ws, size_t ws_bytes, void* stream) {
  rfkv_status st = decode_check(params, n_new);
  if (st != RFKV_OK) return st;
  if (!cu_host || cu_host[0] != 0) return RFKV_INVALID_ARG;
  int32_t max_len = 0;
  for (int b = 0; b < params->batch; ++b) {
    const int64_t len = (int64_t)cu_host[b + 1] - cu_host[b];
    if (len < 0) return RFKV_INVALID_ARG;
    if (len > max_len) max_len = (int32_t)len;
  }
  if (params->batch == 0 || n_new == 0) return RFKV_OK;
  if (!out || !aligned16(out) || !aligned16(q_new) || !aligned16(ws)) return RFKV_INVALID_ARG;
  if (masked) {
    if (!cu_dev || !keep_mask) return RFKV_INVALID_ARG;
    if ((st = check_strides(params, false, true, true)) != RFKV_OK) return st;
  } else if (!out_offsets || (params->out_pad_rows > 0 && !kept)) {
    return RFKV_INVALID_ARG;       // a padded cache is only described by its kept counts
  }
  if (max_len > 0 && (!aligned16(k) || !aligned16(v))) return RFKV_INVALID_ARG;
  DecodeArgs a{};
  decode_geometry(params, n_new, &a);
  const DecodeWs w = decode_ws(params, a);
  if (ws_bytes < w.bytes) return RFKV_WORKSPACE_TOO_SMALL;
  a.q = q_new;
  a.k = k;
  a.v = v;
  a.out = out;
  a.total_tokens = cu_host[params->batch];
  unsigned char* base = static_cast<unsigned char*>(ws);
  a.part_o = reinterpret_cast<float*>(base + w.part_o);
  a.part_ml = reinterpret_cast<float2*>(base + w.part_ml);
  a.item_begin = reinterpret_cast<int32_t*>(base + w.item_begin);
  if (masked) {
    a.cu = cu_dev;
    a.mask = keep_mask;
    a.k_stride_tok = params->k_stride_tok;
    a.k_stride_head = params->k_stride_head;
    a.v_stride_tok = params->v_stride_tok;
    a.v_stride_head = params->v_stride_head;
  } else {
    a.offsets = out_offsets;
    a.kept = kept;
    a.k_stride_tok = a.v_stride_tok = params->head_dim;
    a.k_stride_head = a.v_stride_head = 0;
  }
  return device_status(launch_decode_attention(a, params->batch * params->n_kv_heads, masked,
                                               static_cast<hipStream_t>(stream)));
}

size_t rfkv_decode_workspace_bytes(const rfkv_params* params, int32_t n_new, int32_t max_seqlen) {
  if (decode_check(params, n_new) != RFKV_OK || max_seqlen < 0) return 0;
  DecodeArgs a{};
  decode_geometry(params, n_new, &a);
  return decode_ws(params, a).bytes;
}

rfkv_status rfkv_decode_attention(const rfkv_params* params, const void* q_new, int32_t n_new, const void* k_c,
                                  const void* v_c, const int32_t* cu_seqlens_host, const int64_t* out_offsets,
                                  const int32_t* kept_opt, float* out, void* ws, size_t ws_bytes, void* stream) {
  return decode_impl(params, q_new, n_new, k_c, v_c, cu_seqlens_host, nullptr, out_offsets, kept_opt, nullptr, false,
                     out, ws, ws_bytes, stream);
}

rfkv_status rfkv_masked_attention(const rfkv_params* params, const void* q_new, int32_t n_new, const void* k,
                                  const void* v, const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                                  const uint8_t* keep_mask, float* out, void* ws, size_t ws_bytes, void* stream) {
  return decode_impl(params, q_new, n_new, k, v, cu_seqlens_host, cu_seqlens_dev, nullptr, nullptr, keep_mask, true,
                     out, ws, ws_bytes, stream);
}

static rfkv_status compress_layer_impl(const rfkv_params* params, const void* q_win, const float* lse_win,
                                bool with_lse, const void* k, const void* v, const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev, float* scores_opt,
                                int32_t* kept, int64_t* out_offsets, int32_t* idx_opt, void* k_out, void* v_out,
                                int64_t out_capacity_rows, void* ws, size_t ws_bytes, void* stream, const Marks* marks) {
  rfkv_status st = check_params(params);
  if (st != RFKV_OK) return st;
  if ((st = check_strides(params, true, true, true)) != RFKV_OK) return st;
  int64_t total;
  int32_t max_len;
  if ((st = check_cu(params, cu_seqlens_host, cu_seqlens_dev, &total, &max_len)) != RFKV_OK) return st;
  if (!kept || !out_offsets || out_capacity_rows < 0) return RFKV_INVALID_ARG;
  if (params->out_pad_rows > 0 &&
      (params->out_pad_rows < max_len ||
       params->out_pad_rows * params->batch * params->n_kv_heads > out_capacity_rows))
    return RFKV_OUTPUT_TOO_SMALL;
  if (params->batch == 0) return RFKV_OK;
  if (!aligned16(ws)) return RFKV_INVALID_ARG;
  // A layer that keeps its whole cache (T <= 0 keeps everything, Sec. 3.3 "Retaining Bottom Layers") and
  // whose scores nobody asked for needs no scoring pass: the call is the re-layout copy alone.
  const bool keep_whole = !(params->threshold > 0.f) && !scores_opt;
  if (total > 0 && (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))) return RFKV_INVALID_ARG;
  if (total > 0 && !keep_whole && !aligned16(q_win)) return RFKV_INVALID_ARG;
  if (scores_opt && !aligned16(scores_opt)) return RFKV_INVALID_ARG;
  if (with_lse && !keep_whole && total > 0 && (!lse_win || (reinterpret_cast<uintptr_t>(lse_win) & 3u)))
    return RFKV_INVALID_ARG;
  const Geometry g = make_geometry(params, total, max_len, cu_seqlens_host);
  if ((st = check_wide_grid(g)) != RFKV_OK) return st;
  const Workspace w = carve_workspace(g, ws);
  if (ws_bytes < w.bytes) return RFKV_WORKSPACE_TOO_SMALL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* scores = scores_opt ? scores_opt : w.scores;
  hipError_t e = hipSuccess;
  if (total > 0 && !keep_whole)
    e = run_score(params, g, w, q_win, with_lse ? lse_win : nullptr, k, cu_seqlens_dev, scores, s, marks);
  if (e != hipSuccess) return device_status(e);
  e = run_select(params, g, w, scores, cu_seqlens_dev, kept, false, s);
  if (e != hipSuccess) return device_status(e);
  if (marks) marks->after(kKernelSelect);
  CompactArgs c = compact_base(params, g, cu_seqlens_dev, kept);
  c.k = k;
  c.v = v;
  c.k_out = total > 0 ? k_out : nullptr;
  c.v_out = v_out;
  c.source = params->rank_mode == RFKV_RANK_SCORE ? kSrcPaddedIdx : kSrcPositionDesc;
  c.desc = w.desc;
  c.idx_pad = w.idx_pad;
  c.offsets_out = out_offsets;
  c.idx_out = idx_opt;
  c.capacity_rows = out_capacity_rows;
  c.idx_capacity = out_capacity_rows;
  e = launch_compact(g, c, s);
  if (marks && e == hipSuccess) marks->after(kKernelCompact);
  return device_status(e);
}

rfkv_status rfkv_compress_layer(const rfkv_params* params, const void* q_win, const void* k, const void* v,
                                const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev, float* scores_opt,
                                int32_t* kept, int64_t* out_offsets, int32_t* idx_opt, void* k_out, void* v_out,
                                int64_t out_capacity_rows, void* ws, size_t ws_bytes, void* stream) {
  return compress_layer_impl(params, q_win, nullptr, false, k, v, cu_seqlens_host, cu_seqlens_dev, scores_opt, kept,
                             out_offsets, idx_opt, k_out, v_out, out_capacity_rows, ws, ws_bytes, stream, nullptr);
}

// ---- all layers of a model in one call ---------------------------------------------------------------
namespace rfkv {
namespace {

// Keys one scoring work item of the layer pipeline covers: about 128 items per pass and layer, so that
// the statistics pass of one layer and the reduction pass of another fill kPipelineScoreWgs workgroups
// with one long span each (a span's fixed costs, query fragments and the first tiles, are paid once).
int32_t pipeline_span(int64_t total_tokens, int32_t n_kv_heads) {
  const int64_t keys = total_tokens * n_kv_heads;
  int64_t span = (keys / (kPipelineScoreWgs / 2) + 127) / 128 * 128;
  if (span < 512) span = 512;
  if (span > 16384) span = 16384;
  return (int32_t)span;
}

Geometry pipeline_geometry(const Geometry& g) {
  Geometry p = g;
  p.span = pipeline_span(g.total_tokens, g.n_kv_heads);
  p.nspans = (g.max_seqlen + p.span - 1) / p.span;
  return p;
}

// Does this problem run as the layer pipeline?  Position ranking with one cut per unit (the scoring pass
// takes the cut itself), the streaming kernels' shapes with two passes over K, ragged output.
bool pipeline_covers(const rfkv_params* p, const Geometry& g, int32_t n_layers) {
  return n_layers >= 2 && g.total_tokens > 0 && p->threshold > 0.f && p->out_pad_rows == 0 && !g.spill &&
         g.units <= kPipelineMaxUnits && select_fuses(p, g);
}

struct LayersWorkspace {
  int32_t* queues;        // [n_layers]              chunk counters of the copies
  int32_t* counters;      // [n_layers][2][units]    arrival counters of the scoring passes
  size_t zero_words;      // int32 words from `queues` on that must be zero when the pipeline starts
  size_t layer_offset;    // first layer's scratch
  size_t layer_bytes;     // scratch per layer
  size_t bytes;
};

LayersWorkspace carve_layers(const Geometry& g, int32_t n_layers, void* base) {
  LayersWorkspace w{};
  unsigned char* b = static_cast<unsigned char*>(base);
  const size_t head = align_up(((size_t)n_layers + (size_t)n_layers * 2 * g.units) * sizeof(int32_t), 256);
  w.queues = reinterpret_cast<int32_t*>(b);
  w.counters = w.queues ? w.queues + n_layers : nullptr;
  w.zero_words = (size_t)n_layers + (size_t)n_layers * 2 * g.units;
  w.layer_offset = head;
  const size_t a = carve_workspace(g, nullptr).bytes, p = carve_workspace(pipeline_geometry(g), nullptr).bytes;
  w.layer_bytes = align_up(a > p ? a : p, 256);
  w.bytes = head + (size_t)n_layers * w.layer_bytes;
  return w;
}

}  // namespace
}  // namespace rfkv

size_t rfkv_layers_workspace_bytes(const rfkv_params* params, int32_t n_layers, int64_t total_tokens,
                                   int32_t max_seqlen) {
  if (n_layers < 0 || rfkv_workspace_bytes(params, total_tokens, max_seqlen) == 0) return 0;
  const Geometry g = make_geometry(params, total_tokens, max_seqlen);
  return carve_layers(g, n_layers, nullptr).bytes + 256;
}

rfkv_status rfkv_compress_layers(const rfkv_params* params, int32_t n_layers, const void* const* q_win,
                                 const void* const* k, const void* const* v, const int32_t* cu_seqlens_host,
                                 const int32_t* cu_seqlens_dev, float* const* scores_opt, int32_t* const* kept,
                                 int64_t* const* out_offsets, int32_t* const* idx_opt, void* const* k_out,
                                 void* const* v_out, int64_t out_capacity_rows, void* ws, size_t ws_bytes,
                                 void* stream) {
  rfkv_status st = check_params(params);
  if (st != RFKV_OK) return st;
  if (n_layers < 0) return RFKV_INVALID_ARG;
  if ((st = check_strides(params, true, true, true)) != RFKV_OK) return st;
  int64_t total;
  int32_t max_len;
  if ((st = check_cu(params, cu_seqlens_host, cu_seqlens_dev, &total, &max_len)) != RFKV_OK) return st;
  if (n_layers == 0) return RFKV_OK;
  if (!q_win || !k || !v || !kept || !out_offsets || !k_out || !v_out || out_capacity_rows < 0) return RFKV_INVALID_ARG;
  if (params->batch > 0 && !aligned16(ws)) return RFKV_INVALID_ARG;
  const Geometry g = make_geometry(params, total, max_len, cu_seqlens_host);
  const LayersWorkspace lw = carve_layers(g, n_layers, ws);
  if (params->batch > 0 && ws_bytes < lw.bytes) return RFKV_WORKSPACE_TOO_SMALL;
  auto layer_ws = [&](int l) { return static_cast<unsigned char*>(ws) + lw.layer_offset + (size_t)l * lw.layer_bytes; };
  hipStream_t s = static_cast<hipStream_t>(stream);

  if (!pipeline_covers(params, g, n_layers)) {
    // layer after layer, each exactly as rfkv_compress_layer (which also validates the layer's pointers)
    for (int l = 0; l < n_layers; ++l) {
      st = compress_layer_impl(params, q_win[l], nullptr, false, k[l], v[l], cu_seqlens_host, cu_seqlens_dev,
                               scores_opt ? scores_opt[l] : nullptr, kept[l], out_offsets[l],
                               idx_opt ? idx_opt[l] : nullptr, k_out[l], v_out[l], out_capacity_rows, layer_ws(l),
                               lw.layer_bytes, stream, nullptr);
      if (st != RFKV_OK) return st;
    }
    return RFKV_OK;
  }

  for (int l = 0; l < n_layers; ++l) {
    if (!kept[l] || !out_offsets[l]) return RFKV_INVALID_ARG;
    if (!aligned16(q_win[l]) || !aligned16(k[l]) || !aligned16(v[l]) || !aligned16(k_out[l]) || !aligned16(v_out[l]))
      return RFKV_INVALID_ARG;
    if (scores_opt && !aligned16(scores_opt[l])) return RFKV_INVALID_ARG;
  }
  const Geometry gp = pipeline_geometry(g);
  const bool bf16 = params->dtype == RFKV_DTYPE_BF16;
  hipError_t e = launch_pipeline_prepare(lw.queues, (int64_t)lw.zero_words, s);
  if (e != hipSuccess) return device_status(e);
  auto score_of = [&](int l) {
    const Workspace w = carve_workspace(gp, layer_ws(l));
    ScoreArgs a = score_args(params, gp, w, q_win[l], nullptr, k[l], cu_seqlens_dev,
                             scores_opt ? scores_opt[l] : w.scores, kept[l]);
    a.counters = lw.counters + (size_t)l * 2 * g.units;
    return a;
  };
  const int items = gp.nspans * g.units;
  // launch j: statistics of layer j, reduction + cut of layer j - 1, compaction of layer j - 2
  for (int j = 0; j < n_layers + 2; ++j) {
    PipelineArgs p{};
    if (j < n_layers) {
      p.stats = score_of(j);
      p.stats_items = items;
    }
    if (j >= 1 && j - 1 < n_layers) {
      p.reduce = score_of(j - 1);
      p.reduce_items = items;
    }
    if (j >= 2) {
      const int l = j - 2;
      const Workspace w = carve_workspace(gp, layer_ws(l));
      CompactArgs c = compact_base(params, g, cu_seqlens_dev, kept[l]);
      c.k = k[l];
      c.v = v[l];
      c.k_out = k_out[l];
      c.v_out = v_out[l];
      c.source = kSrcPositionDesc;
      c.desc = w.desc;
      c.offsets_out = out_offsets[l];
      c.idx_out = idx_opt ? idx_opt[l] : nullptr;
      c.capacity_rows = out_capacity_rows;
      c.idx_capacity = out_capacity_rows;
      p.copy = c;
      p.copy_units = g.units;
      p.queue = lw.queues + l;
    }
    e = launch_pipeline_step(gp, p, bf16, s);
    if (e != hipSuccess) return device_status(e);
  }
  return RFKV_OK;
}

rfkv_status rfkv_compress_layer_static(const rfkv_params* params, const void* q_win, const void* k, const void* v,
                                       const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                                       float* scores_opt, int32_t* kept, int64_t* out_offsets, int32_t* idx_opt,
                                       void* k_out, void* v_out, int64_t out_capacity_rows, void* stream) {
  // the size check comes first: it needs no device, and a problem that does not fit must not get as far
  // as looking the array up
  rfkv_status st = check_params(params);
  if (st != RFKV_OK) return st;
  int64_t total;
  int32_t max_len;
  if ((st = check_cu(params, cu_seqlens_host, cu_seqlens_dev, &total, &max_len)) != RFKV_OK) return st;
  if (params->batch == 0) return RFKV_OK;
  const Geometry g = make_geometry(params, total, max_len, cu_seqlens_host);
  if (carve_workspace(g, nullptr).bytes > (size_t)RFKV_STATIC_SCRATCH_BYTES) return RFKV_WORKSPACE_TOO_SMALL;
  void* ws = nullptr;
  const hipError_t e = static_scratch(&ws);
  if (e != hipSuccess) return device_status(e);
  return compress_layer_impl(params, q_win, nullptr, false, k, v, cu_seqlens_host, cu_seqlens_dev, scores_opt, kept,
                             out_offsets, idx_opt, k_out, v_out, out_capacity_rows, ws, RFKV_STATIC_SCRATCH_BYTES,
                             stream, nullptr);
}

rfkv_status rfkv_compress_layer_lse(const rfkv_params* params, const void* q_win, const float* lse_win, const void* k,
                                    const void* v, const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                                    float* scores_opt, int32_t* kept, int64_t* out_offsets, int32_t* idx_opt,
                                    void* k_out, void* v_out, int64_t out_capacity_rows, void* ws, size_t ws_bytes,
                                    void* stream) {
  return compress_layer_impl(params, q_win, lse_win, true, k, v, cu_seqlens_host, cu_seqlens_dev, scores_opt, kept,
                             out_offsets, idx_opt, k_out, v_out, out_capacity_rows, ws, ws_bytes, stream, nullptr);
}

rfkv_status rfkv_compress_layer_timed(const rfkv_params* params, const void* q_win, const void* k, const void* v,
                                      const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                                      float* scores_opt, int32_t* kept, int64_t* out_offsets, int32_t* idx_opt,
                                      void* k_out, void* v_out, int64_t out_capacity_rows, void* ws,
                                      size_t ws_bytes, void* stream, float* kernel_ms_host) {
  if (!kernel_ms_host) return RFKV_INVALID_ARG;
  for (int i = 0; i < kNumKernels; ++i) kernel_ms_host[i] = 0.f;
  Marks m{};
  m.stream = static_cast<hipStream_t>(stream);
  int made = 0;
  hipError_t e = hipSuccess;
  for (; made <= kNumKernels && e == hipSuccess; ++made) e = hipEventCreate(&m.ev[made]);
  if (e != hipSuccess) --made;
  rfkv_status st = RFKV_OK;
  if (e != hipSuccess) {
    st = device_status(e);
  } else {
    // every slot gets a record first so that kernels this problem skips read as zero time
    for (int i = kNumKernels; i >= 0; --i) (void)hipEventRecord(m.ev[i], m.stream);      // start event last
    st = compress_layer_impl(params, q_win, nullptr, false, k, v, cu_seqlens_host, cu_seqlens_dev, scores_opt, kept,
                             out_offsets, idx_opt, k_out, v_out, out_capacity_rows, ws, ws_bytes, stream, &m);
    e = hipStreamSynchronize(m.stream);
    if (st == RFKV_OK && e != hipSuccess) st = device_status(e);
    if (st == RFKV_OK) {
      for (int i = 0; i < kNumKernels; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, m.ev[i], m.ev[i + 1]) == hipSuccess && ms > 0.f) kernel_ms_host[i] = ms;
      }
    }
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(m.ev[i]);
  return st;
}

}  // extern "C"
