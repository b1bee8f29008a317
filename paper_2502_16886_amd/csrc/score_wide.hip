// Scoring with a wide observation window: more score rows (window * G) than one workgroup can keep
// in registers or LDS.  The paper's ablation of the window size ("Attention Matrix Reduction":
// k = 1 %, 5 %, 10 % of n) runs Eq. 2 with thousands of rows, where the contraction Q_win K^T is a
// real GEMM and the matrix cores, not HBM, set the pace.
//
// Same two passes as the narrow kernels (row statistics, merge, column sums of the normalised
// probabilities), with the operands the other way round in the second pass:
//
//   pass 1  score_stream_kernel<.., WIDE> (score_qreg.hip): a workgroup keeps one block of 128 score
//           rows in registers and streams its span of keys; grid.z walks the row blocks.
//   merge   score_merge_kernel: b_r = reference + log2(sum * G) per row.
//   pass 2  score_colsum_wide_kernel (here): a workgroup keeps 512 KEYS in registers (each
//           wavefront the MFMA fragments of four 32-key tiles) and streams the window queries, four
//           row tiles per stage, through a double-buffered LDS ring filled by direct-to-LDS
//           loads, together with the rows' exponent offsets b_r.  A lane owns one key column, so
//           the sum over rows is a chain of register adds and the scores leave the kernel once.
//           Rows that cannot see a key block (the causal part of the window) are skipped by
//           whole stages; partly visible stages mask per element with one comparison.
//
// Per 32 x 32 tile of logits a wavefront spends 8 MFMAs (d = 128: 256 cycles) and, per lane, 16 x
// (fma, exp2, add): the quarter-rate exponential makes the vector ALU the longer pole (about
// 1.5 x the matrix time), so two workgroups share a CU and overlap one's MFMAs with the other's
// arithmetic.
#include "kernels.h"
#include "score_common.h"
#include "tile_sum.h"

#include <type_traits>

namespace rfkv {
namespace {

constexpr int kWideKT = 4;             // key tiles a wavefront keeps
constexpr int kWideStage = 4;          // row tiles per stage, one brought in by each wavefront
constexpr int kWideKeys = 4 * kWideKT * 32;    // keys per workgroup

template <typename T, int D>
constexpr size_t wide_lds_bytes() {
  return 2 * kWideStage * 32 * Shape<T, D>::kRowBytes + 2 * kWideStage * 64 * sizeof(float);
}

// 4 x 16 bytes at consecutive 32-byte steps: the exponent offsets of the 16 rows a lane's accumulators hold
__device__ __forceinline__ void read_row_offsets(float* bv, const float* tile, int hi) {
  uint32_t addr[4];
  const uint32_t base = lds_offset(tile) + hi * 16;
#pragma unroll
  for (int j = 0; j < 4; ++j) addr[j] = base + j * 32;
  uint4 raw[4];
  lds_read_b128_x4(raw, addr);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    bv[4 * j + 0] = __uint_as_float(raw[j].x);
    bv[4 * j + 1] = __uint_as_float(raw[j].y);
    bv[4 * j + 2] = __uint_as_float(raw[j].z);
    bv[4 * j + 3] = __uint_as_float(raw[j].w);
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256, 2) void score_colsum_wide_kernel(ScoreArgs a) {
  using S = Shape<T, D>;
  constexpr int kTileBytes = 32 * S::kRowBytes;
  extern __shared__ __attribute__((aligned(1024))) unsigned char wsm[];
  unsigned char* qs = wsm;                                               // [2][kWideStage] query row tiles
  float* bs = reinterpret_cast<float*>(wsm + 2 * kWideStage * kTileBytes);   // [2][kWideStage][64] offsets
  // One-dimensional grid, work item w = key block + blocks * unit.  Workgroups go to the 8 XCDs in
  // turn, so workgroup g takes item (g % 8) * chunk + g / 8: the workgroups resident on one XCD are
  // neighbouring key blocks of one unit and stream the same window queries, which then come from
  // that XCD's L2 rather than from memory once per workgroup.
  const int kblocks = (a.span_colsum + kWideKeys - 1) / kWideKeys;
  const int items = kblocks * a.units;
  const int chunk = (items + 7) >> 3;
  const int w = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= chunk || w >= items) return;
  const int by = w / kblocks;
  const Unit u = load_unit(a, by);
  // the key blocks of a unit back to front: the last ones, whose stages are masked per element and take
  // longest, are dispatched first
  const int kb0 = (kblocks - 1 - (w - by * kblocks)) * kWideKeys;
  if (kb0 >= u.n) return;                              // uniform for the whole workgroup
  if (kb0 == 0 && a.sel_block) clear_select_block(a.sel_block, by);     // for the score ranking of long units

  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 31, hi = lane >> 5;
  const float c = a.c;
  const unsigned char* kunit = static_cast<const unsigned char*>(a.k) +
                               ((int64_t)u.s0 * a.k_stride_tok + (int64_t)u.h * a.k_stride_head) * T::kBytes;
  const TileLoader<T, D> tiles(kunit, a.k_stride_tok * T::kBytes, u.n, lane);

  // this wavefront's keys, staged two tiles at a time through its two slots of the (still unused) query ring
  uint4 kf[kWideKT][S::kChunks];
  int t0[kWideKT];
  static_assert(kWideKT % 2 == 0 && 2 * kWideStage == 2 * 4, "two private ring slots per wavefront");
#pragma unroll
  for (int kt = 0; kt < kWideKT; ++kt) t0[kt] = kb0 + (wave * kWideKT + kt) * 32;   // tiles past the end re-read the last key; never stored
#pragma unroll
  for (int half = 0; half < kWideKT / 2; ++half) {
#pragma unroll
    for (int e = 0; e < 2; ++e) tiles.issue(t0[half * 2 + e], qs + (wave * 2 + e) * kTileBytes);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int e = 0; e < 2; ++e) read_tile_frags<T, D>(kf[half * 2 + e], qs + (wave * 2 + e) * kTileBytes, col, hi);
  }
  __syncthreads();                                     // the ring is free for the queries

  // Row r = t * G + g sees key i iff i <= n - wp + t, i.e. iff r >= G * (i - (n - wp)).
  const int base_pos = u.n - u.wp;
  int rmin[kWideKT];
#pragma unroll
  for (int kt = 0; kt < kWideKT; ++kt) rmin[kt] = a.group * (t0[kt] + col - base_pos);
  const int rows_blind = max(0, a.group * (kb0 - base_pos));                  // rows below see none of the block's keys
  const int wave_rmax = a.group * (t0[kWideKT - 1] + 31 - base_pos);          // rows from here on see all of the wavefront's keys
  const int wave_blind = a.group * (t0[0] - base_pos);                        // rows below see none of the wavefront's keys
  const int stage_begin = rows_blind / (kWideStage * 32);
  const int stage_end = (u.row_tiles + kWideStage - 1) / kWideStage;          // <= rows_pad / 128

  auto issue_stage = [&](int s) {
    const int buf = s & 1;
    const int rt = s * kWideStage + wave;
    issue_q_tile_load<T, D>(a, u, rt, qs + (buf * kWideStage + wave) * kTileBytes, lane);
    const float* src = a.bvec + (int64_t)by * a.rows_pad + min(rt * 32 + lane, a.rows_pad - 1);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(bs + (buf * kWideStage + wave) * 64), 4, 0, 0);
  };

  auto logits = [&](const uint4* q, const uint4* k) {
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int ch = 0; ch < S::kChunks; ++ch) acc = mma_chunk<T>(q[ch], k[ch], acc);     // rows x keys: a lane owns one key
    return acc;
  };

  float colsum[kWideKT];
#pragma unroll
  for (int kt = 0; kt < kWideKT; ++kt) colsum[kt] = 0.f;

  // One stage: kWideStage row tiles against the wavefront's kWideKT key tiles, item by item
  // (row tile j, key tile kt), j-major.  A wavefront issues in order, and a dependent MFMA waits
  // at the issue stage for the one before it, so a chain issued back to back holds up every
  // instruction behind it.  The chain of item it + 1 is therefore issued one MFMA at a time
  // between slices of item it's softmax arithmetic (fma, exp2, add per element), with scheduling
  // barriers so that the compiler keeps that order: the matrix pipe works in the shadow of the
  // vector ALU.
  auto stage_compute = [&](int s, auto masked_tag) {
    constexpr bool kMasked = decltype(masked_tag)::value;
    constexpr int kItems = kWideStage * kWideKT;
    constexpr int kSlice = 16 / S::kChunks;            // elements of this item per chunk of the next chain
    static_assert(kSlice * S::kChunks == 16, "the chain divides the 16 accumulators evenly");
    const int buf = s & 1;
    uint4 qf[2][S::kChunks];
    float bv[16];
    read_tile_frags<T, D>(qf[0], qs + (buf * kWideStage) * kTileBytes, col, hi);
    f32x16 acc = logits(qf[0], kf[0]);
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
      const int j = it / kWideKT, kt = it % kWideKT;
      const bool more = it + 1 < kItems;
      const int j2 = (it + 1) / kWideKT, kt2 = (it + 1) % kWideKT;
      if (more && kt2 == 0) read_tile_frags<T, D>(qf[j2 & 1], qs + (buf * kWideStage + j2) * kTileBytes, col, hi);
      if (kt == 0) read_row_offsets(bv, bs + (buf * kWideStage + j) * 64, hi);
      // accumulator i of this lane: row (s * kWideStage + j) * 32 + (i / 4) * 8 + hi * 4 + i % 4, key t0[kt] + col;
      // visible iff (i / 4) * 8 + i % 4 >= rel
      const int rel = rmin[kt] - (s * kWideStage + j) * 32 - hi * 4;
      f32x16 nxt;
#pragma unroll
      for (int i = 0; i < 16; ++i) nxt[i] = 0.f;
      float sum = colsum[kt];
#pragma unroll
      for (int ch = 0; ch < S::kChunks; ++ch) {
        if (more) nxt = mma_chunk<T>(qf[j2 & 1][ch], kf[kt2][ch], nxt);     // rows x keys: a lane owns one key
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < kSlice; ++e) {
          const int i = ch * kSlice + e;
          const float p = fast_exp2(__builtin_fmaf(acc[i], c, -bv[i]));
          sum += (!kMasked || (i / 4) * 8 + i % 4 >= rel) ? p : 0.f;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      colsum[kt] = sum;
      acc = nxt;
    }
  };

  if (stage_begin < stage_end) issue_stage(stage_begin);
  for (int s = stage_begin; s < stage_end; ++s) {
    // stage s has landed (every wavefront waits for its own loads, then all meet); the other half
    // of the ring was last read in stage s - 1, which every wavefront has left
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (s + 1 < stage_end) issue_stage(s + 1);
    if ((s + 1) * (kWideStage * 32) <= wave_blind) continue;       // no row of this stage sees any of the wavefront's keys
    if (s * (kWideStage * 32) < wave_rmax) stage_compute(s, std::true_type{});
    else stage_compute(s, std::false_type{});
  }

  float* out = a.scores + (int64_t)u.h * a.total_tokens + u.s0;
#pragma unroll
  for (int kt = 0; kt < kWideKT; ++kt) {
    const float tot = colsum[kt] + other_half(colsum[kt]);
    const int key = t0[kt] + col;
    const float score = key < u.n ? tot / (float)min(u.wp, u.n - key) : 0.f;
    if (hi == 0 && key < u.n) out[key] = score;
    const double tsq = tile_sum_sq(score, lane);
    if (lane == 0 && t0[kt] < u.n) a.tile_sq[(int64_t)u.h * a.tiles_total + u.tile_base + (t0[kt] >> 5)] = tsq;
  }
}

template <typename T, int D>
hipError_t launch_colsum_typed(const Geometry& g, const ScoreArgs& a, hipStream_t stream) {
  constexpr size_t lds = wide_lds_bytes<T, D>();
  hipError_t e = allow_lds<&score_colsum_wide_kernel<T, D>>(lds);
  if (e != hipSuccess) return e;
  const int items = (g.max_seqlen + kWideKeys - 1) / kWideKeys * g.units;
  hipLaunchKernelGGL((score_colsum_wide_kernel<T, D>), dim3((items + 7) / 8 * 8), dim3(256), lds, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_wide(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream, const Marks* marks) {
  hipError_t e = launch_score_offsets(g, a, stream, marks);    // from the caller's log-sum-exp, if given
  if (e != hipSuccess) return e;
  if (!a.lse) {
    e = launch_score_wide_stats(g, a, bf16, stream);
    if (e != hipSuccess) return e;
    if (marks) marks->after(kKernelStats);
    e = launch_score_merge(g, a, stream);
    if (e != hipSuccess) return e;
    if (marks) marks->after(kKernelMerge);
  }
  if (bf16) e = g.head_dim == 64 ? launch_colsum_typed<Bf16, 64>(g, a, stream) : launch_colsum_typed<Bf16, 128>(g, a, stream);
  else e = g.head_dim == 64 ? launch_colsum_typed<Fp32, 64>(g, a, stream) : hipErrorInvalidValue;
  if (marks && e == hipSuccess) marks->after(kKernelReduce);
  return e;
}

}  // namespace rfkv
