// Internal launch interface between the C-ABI layer (api.hip) and the gfx950 kernels.
// Everything here is device-pointer based; validation happens in api.hip.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace rfkv {

constexpr int kBlockThreads = 256;     // 4 wavefronts per workgroup in the score / compact kernels
constexpr int kKeyTilesPerWave = 2;    // 32-key MFMA tiles a wavefront processes per iteration
constexpr int kKeysPerIter = 4 * kKeyTilesPerWave * 32;   // keys a workgroup consumes per iteration
constexpr int kSelectThreads = 1024;
constexpr int kSpillRows = 8;          // up to this many score rows the first scoring pass keeps its logits

// Geometry shared by the host (workspace sizing, grids) and the kernels.
struct Geometry {
  int32_t batch, n_q_heads, n_kv_heads, group, head_dim, window;
  int32_t units;          // batch * n_kv_heads
  int32_t rows_pad;       // window * group rounded up to a multiple of 32
  int32_t span;           // keys one score workgroup covers (multiple of kKeysPerIter)
  int32_t nspans;         // ceil(max_seqlen / span)
  int32_t max_seqlen;
  int64_t total_tokens;   // N
  int32_t elem_bytes;     // 2 (bf16) or 4 (fp32)
  int64_t tiles_total;    // sum over sequences of ceil(n_b / 32) (an upper bound when sizing)
  int32_t spill;          // window * group <= kSpillRows: scoring keeps its logits instead of re-reading K
  int32_t wide;           // window * group > RFKV_MAX_SCORE_ROWS: row-blocked statistics, key-resident column sums
  int32_t score_slices;   // score ranking: workgroups a unit is split over (0: one workgroup per unit)
  int32_t per_layer;      // one cut per (layer, sequence): the score ranking then needs room to sort
};

// Score ranking of long units: a unit is split over several workgroups when the longest sequence has more
// than kSingleWorkgroupMax positions and the batch is small enough for the split to put idle CUs to work
// (a batch of many units fills the chip with one workgroup per unit; each sliced unit has a 24 KB histogram
// in the workspace).
constexpr int kSingleWorkgroupMax = 8192;
constexpr int kSliceMin = 2048;             // positions per slice at least (two per thread)
constexpr int kMaxSlices = 32;
constexpr int kSliceWorkgroups = 256;       // workgroups of all units together, about one per CU
// A unit's block in the workspace: 2048 counts (uint32), 2048 integer masses (uint64), the arrival counter
// of its workgroups and a pad word.  Every word is zero when the histogram kernel starts: the kernel that
// runs just before it in the same call (the last scoring kernel, or the tile-sum kernel of a separate
// rfkv_select) clears it, one workgroup per unit.
constexpr int kSelCntWords = 2048, kSelMassWords = 4096;
constexpr int kSelWords = kSelCntWords + kSelMassWords + 2;
__device__ __forceinline__ void clear_select_block(uint32_t* sel_block, int unit) {
  uint2* p2 = reinterpret_cast<uint2*>(sel_block + (int64_t)unit * kSelWords);      // 24584 bytes, 8-byte aligned
  for (int i = threadIdx.x; i < kSelWords / 2; i += blockDim.x) p2[i] = make_uint2(0u, 0u);
}
inline int score_slices(int max_seqlen, int units) {
  if (max_seqlen <= kSingleWorkgroupMax || units <= 0) return 0;
  int w = (max_seqlen + kSliceMin - 1) / kSliceMin;
  if (w > kMaxSlices) w = kMaxSlices;
  if (w > kSliceWorkgroups / units) w = kSliceWorkgroups / units;
  return w >= 2 ? w : 0;
}

struct Workspace {
  float2*  partials;      // [units][nspans][rows_pad]  (reference exponent, sum) per span
  float*   bvec;          // [units][rows_pad]          per-row exponent offset for the second pass
  int4*    desc;          // [units]                    {kept, sinks kept, -, -}
  int32_t* idx_pad;       // [N * Hkv]                  per-unit padded index lists (score ranking)
  float*   scores;        // [Hkv][N]                   used when the caller does not want scores
  double*  tile_sq;       // [Hkv][tiles_total]         sum of squared scores per 32-position tile
  float*   logits;        // [Hkv][kSpillRows][tiles_total * 32]  scaled logits, only when window * G <= kSpillRows
  int32_t* counters;      // [2][units]  workgroups of a unit that have finished the statistics / the reduction pass;
                          //             zeroed by the call's first kernel, put back to zero by each last arriver
  uint32_t* sel_block;    // [units][kSelWords]  score ranking of long units, see kSelWords
  uint32_t* sort_keys;    // [2 * N * Hkv]  per-layer cut with the score ranking: every unit's keys, padded to a power of two
  float*   sorted_scores; // [Hkv][N]       ... and its scores in ascending order
  size_t   bytes;
};

Workspace carve_workspace(const Geometry& g, void* base);

struct ScoreArgs {
  const void* q;
  const void* k;
  float* scores;
  const int32_t* cu;
  float2* partials;
  float* bvec;
  double* tile_sq;
  float* logits;          // null unless the first pass keeps its logits (window * G <= kSpillRows)
  const float* lse;       // optional [window rows][Hq]: the rows' log-sum-exp from the prefill; no statistics pass then
  int64_t tiles_total;
  int64_t k_stride_tok, k_stride_head, q_stride_row, q_stride_head;
  int64_t total_tokens;
  int32_t n_q_heads, n_kv_heads, group, window, rows_pad, span, nspans;
  int32_t wide_items;     // wide window: work items of the statistics pass (row blocks * spans * units)
  int32_t units;
  int32_t span_colsum;    // wide window: the longest sequence (keys the column-sum grid covers per unit)
  float c;                // softmax scale * log2(e)
  // The streaming kernels can hand over between workgroups inside a launch: with `fuse_merge` the last
  // workgroup of a unit to finish the statistics pass folds the unit's per-span statistics (no merge
  // kernel), with `fuse_select` the last one to finish the reduction pass takes the unit's position-ranking
  // cut (no selection kernel).  Each hand-over costs a few memory round trips (acknowledged stores, a
  // device-scope atomic, coherent loads), about what a small dependent kernel costs, so it pays only
  // where other work runs beside it: the layer pipeline sets both, the per-layer calls neither.
  // counters: [2][units], zero before the launch, see Workspace.
  int32_t* counters;
  int32_t fuse_merge;
  int32_t fuse_select;
  int32_t n_sink, min_keep;
  float threshold;
  int32_t* kept;          // fuse_select: [units]
  int4* desc;             // fuse_select: [units] {kept, sinks kept, -, -}
  uint32_t* sel_block;    // not null: the last scoring kernel clears every unit's block for the score ranking
};

struct SelectArgs {
  const float* scores;
  const int32_t* cu;
  int32_t* kept;
  int4* desc;
  int32_t* idx_pad;
  double* tile_sq;        // per-tile squared-score sums: read; written first when from_scores is set
  int64_t tiles_total;
  int64_t total_tokens;
  int32_t from_scores;    // the tile sums are not there yet: form them from the scores first
  int32_t n_kv_heads, n_sink, min_keep, rank_mode;
  float threshold;
  int32_t per_layer;      // one cut per (layer, sequence) over all heads instead of one per unit
  int32_t lds_floats;     // set by launch_select: floats of dynamic LDS the select kernel may use
  // score ranking of long units (several workgroups per unit): per unit kSelWords words (first-digit
  // histogram, arrival counter), zero when the histogram kernel starts
  uint32_t* sel_block;
  int32_t units;
  // one cut per (layer, sequence) with the score ranking: see Workspace
  uint32_t* sort_keys;
  float* sorted_scores;
};

enum CompactSource { kSrcPositionDesc = 0, kSrcPaddedIdx = 1, kSrcPackedIdx = 2 };

struct CompactArgs {
  const void* k;
  const void* v;
  void* k_out;            // may be null together with v_out: indices / offsets only
  void* v_out;
  const int32_t* cu;
  const int32_t* kept;
  const int4* desc;             // kSrcPositionDesc
  const int32_t* idx_pad;       // kSrcPaddedIdx
  const int32_t* idx_packed;    // kSrcPackedIdx (with offsets_in)
  const int64_t* offsets_in;    // kSrcPackedIdx
  int64_t* offsets_out;         // other sources: exclusive scan of kept, written here (may be null)
  int32_t* idx_out;             // other sources: packed indices written here (may be null)
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
  int64_t capacity_rows;
  int64_t idx_capacity;         // entries of idx_out; indices at or beyond it are not written
  int64_t pad_rows;             // > 0: padded layout, unit u's rows start at u * pad_rows (not kSrcPackedIdx)
  int32_t n_kv_heads, units, row_bytes, source;
  int32_t offsets_ready;        // set by launch_compact: offsets_out already holds the exclusive scan (many units)
};

// One launch of the layer pipeline (pipeline.hip): the statistics pass of one layer, the reduction
// pass (with the position-ranking cut) of the layer before it and the gather-compaction of the layer
// before that, any of which may be absent at the ends of the pipeline.
constexpr int kPipelineGrid = 512;          // two workgroups on each of 256 CUs
constexpr int kPipelineScoreWgs = 256;      // of which about this many start with a scoring work item
constexpr int kPipelineMaxUnits = 512;      // units of a layer (a table of them lives in LDS)
struct PipelineArgs {
  ScoreArgs stats, reduce;
  CompactArgs copy;
  int32_t* queue;           // chunk counter of this launch's copy, zero before the launch
  int32_t stats_items;      // spans x units of the statistics pass, 0 if absent
  int32_t reduce_items;     // spans x units of the reduction pass, 0 if absent
  int32_t copy_units;       // units of the layer to compact, 0 if absent
};

// Attention of new queries over the compacted cache (offsets != null) or over the full cache
// with a keep mask (cu, mask != null).
struct DecodeArgs {
  const void* q;            // [B, n_new, Hq, d] bf16
  const void* k;
  const void* v;
  const int64_t* offsets;   // compacted: first row of every unit, [units + 1]
  const int32_t* kept;      // compacted, optional: rows of every unit (padded layout: fewer than its slot)
  const int32_t* cu;        // masked: cu_seqlens
  const uint8_t* mask;      // masked: [Hkv][N], non-zero = retained
  float* out;               // [B, n_new, Hq, d]
  float* part_o;            // [max_items][rows_pad][d]  unnormalised partial outputs, one slot per work item
  float2* part_ml;          // [max_items][rows_pad]     (reference exponent, sum)
  int32_t* item_begin;      // [units + 1]  first item of every unit (written by the attention kernel's first workgroup)
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;   // elements
  int64_t total_tokens;
  int32_t n_q_heads, n_kv_heads, group, n_new, rows, rows_pad, head_dim, units;
  int32_t target_items;     // items the planner aims for (workgroups that fit the chip at once)
  int32_t max_items;        // target_items + units: the grid and the number of partial slots
  float c;                  // softmax scale * log2(e)
};

// Optional per-kernel timing: events recorded on the launch stream between kernels.
enum KernelId { kKernelStats = 0, kKernelMerge, kKernelReduce, kKernelSelect, kKernelCompact, kNumKernels };
struct Marks {
  hipEvent_t ev[kNumKernels + 1];
  hipStream_t stream;
  void after(int kernel) const { (void)hipEventRecord(ev[kernel + 1], stream); }
};

// Raises a kernel's limit on dynamic LDS, once per device, to the most any launch of it may ask for.
// (Setting it per launch to that launch's own size would let two host threads with different
// problem sizes lower the limit under each other between the call and the launch.)
template <auto Kernel>
hipError_t allow_lds(size_t max_bytes) {
  static std::atomic<uint64_t> done{0};                // bit d: raised on device d
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)max_bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}
// the most dynamic LDS the argument checks admit for the kernels that keep the window queries in LDS
constexpr size_t kMaxQueryLds = 156 * 1024;

hipError_t launch_score(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream,
                        const Marks* marks = nullptr);
// does launch_score run the streaming kernels (score_qreg.hip) for this shape?
bool score_streams(const Geometry& g, bool bf16);
hipError_t launch_select(const Geometry& g, const SelectArgs& a, hipStream_t stream);
hipError_t launch_compact(const Geometry& g, const CompactArgs& a, hipStream_t stream);
hipError_t launch_pipeline_prepare(int32_t* words, int64_t n, hipStream_t stream);
hipError_t launch_pipeline_step(const Geometry& g, const PipelineArgs& p, bool bf16, hipStream_t stream);
hipError_t launch_decode_attention(const DecodeArgs& a, int units, bool masked, hipStream_t stream);

}  // namespace rfkv
