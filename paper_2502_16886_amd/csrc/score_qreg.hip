// Streaming scoring kernels for up to 128 score rows per KV head (window * G <= 128: the Llama /
// Mistral shapes with a 32-row window and the paper's own k = 1), Sec. 3.2 "Reducing Overhead",
// Eq. 2; the statistics kernel also serves the wide-window path (score_wide.hip) block by block.
//
// Same two-pass scheme as score.hip (row statistics, merge, column reduction); what differs is
// where the operands live:
//
//   Q   every wavefront keeps the MFMA fragments of ALL its (up to 4) row tiles in registers for
//       the whole kernel (4 row tiles x 8 chunks x 16 bytes per lane for bf16, d = 128).  One
//       wavefront per row tile brings the tile in by direct-to-LDS loads, in the layout of a key
//       tile, into the LDS that afterwards serves as the second set of key-tile buffers.
//   K   streamed through wavefront-private LDS buffers of one 32-key tile each by direct-to-LDS
//       loads (global_load_lds_dwordx4): each instruction moves 1 KB of consecutive key bytes, so
//       HBM/L2 requests are whole cache lines, and no VGPRs are held while the data is in flight.
//       A tile lands XOR-swizzled (16-byte slot s of row r holds chunk s ^ (r & 15)) so the
//       MFMA-layout read-back (lane = row, 8 x ds_read_b128) is bank-conflict free.  While tile i
//       is being multiplied, tiles i+1 and i+2 are in flight.
//
// The kernels count their own loads and stores (s_waitcnt vmcnt(N)) and read LDS through inline
// assembly wherever a direct-to-LDS load may be in flight; see score_common.h for why.
//
// A wavefront therefore touches LDS only for 16 KB per 8 KB key tile (DMA write + fragment
// read); its 32 MFMAs per tile reuse the K fragments 4x and the Q fragments for ever.
#include "kernels.h"
#include "score_common.h"
#include "score_stream.h"
#include "select_position.h"
#include "tile_sum.h"

namespace rfkv {
namespace {

template <typename T, int D, int RT_T, int PASS, bool WIDE = false>
__global__ __launch_bounds__(256, 2) void score_stream_kernel(ScoreArgs a) {
  RFKV_STREAM_LDS(T, D, RT_T, lds);
  score_stream_body<T, D, RT_T, PASS, WIDE>(a, blockIdx.x, blockIdx.y, lds);
}

// Scores from kept logits (PASS 3): one thread per key.  x_r = q_r . k (unscaled), c = scale * log2 e,
// b_r = reference + log2(sum * G) from the merge: score = sum_r 2^(x_r c - b_r) / (rows that see the key).
__global__ __launch_bounds__(256) void score_spill_reduce_kernel(ScoreArgs a) {
  const Unit u = load_unit(a, blockIdx.y);
  const int key0 = blockIdx.x * 256;
  if (key0 >= u.n) return;                             // uniform for the whole workgroup
  const int key = key0 + threadIdx.x;
  float sum = 0.f;
  if (key < u.n) {
    const float* lbase = a.logits + ((int64_t)(u.h * kSpillRows) * a.tiles_total + u.tile_base) * 32 + key;
    for (int r = 0; r < u.rows; ++r) {
      const float x = lbase[(int64_t)r * a.tiles_total * 32];
      const float b = a.bvec[(int64_t)blockIdx.y * a.rows_pad + r];
      const int rowlast = u.n - u.wp + r / a.group;
      if (key <= rowlast) sum += fast_exp2(__builtin_fmaf(x, a.c, -b));     // one rounding, as in pass 2
    }
  }
  const float score = key < u.n ? sum / (float)min(u.wp, u.n - key) : 0.f;
  float* score_out = a.scores + (int64_t)u.h * a.total_tokens + u.s0 + key;
  if (key < u.n) *score_out = score;
  // per-tile squared sums: the butterfly of tile_sum_sq, in both halves of the wavefront at once
  double v = (double)score * (double)score;
#pragma unroll
  for (int d = 16; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  if ((threadIdx.x & 31) == 0 && key < u.n) {
    double* tsq_out = a.tile_sq + (int64_t)u.h * a.tiles_total + u.tile_base + (key >> 5);
    *tsq_out = v;
  }
  if (a.sel_block && blockIdx.x == 0) clear_select_block(a.sel_block, blockIdx.y);
}

template <typename T, int D>
hipError_t launch_stream_spill(const Geometry& g, const ScoreArgs& a, hipStream_t stream, const Marks* marks) {
  const dim3 grid(g.nspans, g.units);
  hipLaunchKernelGGL((score_stream_kernel<T, D, 1, 3>), grid, dim3(256), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (marks) marks->after(kKernelStats);
  e = launch_score_merge(g, a, stream);
  if (e != hipSuccess) return e;
  if (marks) marks->after(kKernelMerge);
  hipLaunchKernelGGL(score_spill_reduce_kernel, dim3((g.max_seqlen + 255) / 256, g.units), dim3(256), 0, stream, a);
  e = hipGetLastError();
  if (marks && e == hipSuccess) marks->after(kKernelReduce);
  return e;
}

template <typename T, int D, int RT_T>
hipError_t launch_stream_typed(const Geometry& g, const ScoreArgs& a, hipStream_t stream, const Marks* marks) {
  const dim3 grid(g.nspans, g.units);
  const dim3 block(256);
  // with the caller's log-sum-exp there is no statistics pass, and pass 2 converts it in its prologue
  hipError_t e = hipSuccess;
  if (!a.lse) {
    hipLaunchKernelGGL((score_stream_kernel<T, D, RT_T, 1>), grid, block, 0, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (marks) marks->after(kKernelStats);
    e = launch_score_merge(g, a, stream);
    if (e != hipSuccess) return e;
    if (marks) marks->after(kKernelMerge);
  }
  hipLaunchKernelGGL((score_stream_kernel<T, D, RT_T, 2>), grid, block, 0, stream, a);
  e = hipGetLastError();
  if (marks && e == hipSuccess) marks->after(kKernelReduce);
  return e;
}

template <typename T, int D>
hipError_t launch_stream_rt(const Geometry& g, const ScoreArgs& a, hipStream_t stream, const Marks* marks) {
  const int rt = g.rows_pad / 32;
  // window * G <= kSpillRows: one pass that keeps its logits, unless the row offsets are given anyway
  if (a.logits && !a.lse) return launch_stream_spill<T, D>(g, a, stream, marks);
  if (rt <= 1) return launch_stream_typed<T, D, 1>(g, a, stream, marks);
  if (rt <= 2) return launch_stream_typed<T, D, 2>(g, a, stream, marks);
  if constexpr (Shape<T, D>::kChunks * 4 <= 32) {
    if (rt <= 4) return launch_stream_typed<T, D, 4>(g, a, stream, marks);
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool score_qreg_covers(const Geometry& g, bool bf16) {
  const int rt = g.rows_pad / 32;
  const int chunks = g.head_dim * g.elem_bytes / 32;    // 16-byte chunks of half a row
  (void)bf16;
  if (rt <= 2) return true;
  return rt <= 4 && chunks * 4 <= 32;                   // 4 row tiles of fragments: 256-byte rows only
}

hipError_t launch_score_qreg(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream,
                             const Marks* marks) {
  if (bf16) {
    if (g.head_dim == 64) return launch_stream_rt<Bf16, 64>(g, a, stream, marks);
    return launch_stream_rt<Bf16, 128>(g, a, stream, marks);
  }
  if (g.head_dim == 64) return launch_stream_rt<Fp32, 64>(g, a, stream, marks);
  return launch_stream_rt<Fp32, 128>(g, a, stream, marks);
}

// Row statistics of a wide window: the pass-1 kernel over blocks of 128 score rows.
template <typename T, int D>
hipError_t launch_wide_stats_typed(const Geometry& g, const ScoreArgs& a, hipStream_t stream) {
  if constexpr (Shape<T, D>::kChunks * 4 <= 32) {
    const dim3 grid((a.wide_items + 7) / 8 * 8);
    hipLaunchKernelGGL((score_stream_kernel<T, D, 4, 1, true>), grid, dim3(256), 0, stream, a);
    return hipGetLastError();
  }
  return hipErrorInvalidValue;
}

hipError_t launch_score_wide_stats(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream) {
  if (g.rows_pad % 128 != 0) return hipErrorInvalidValue;
  if (bf16) {
    if (g.head_dim == 64) return launch_wide_stats_typed<Bf16, 64>(g, a, stream);
    return launch_wide_stats_typed<Bf16, 128>(g, a, stream);
  }
  if (g.head_dim == 64) return launch_wide_stats_typed<Fp32, 64>(g, a, stream);
  return hipErrorInvalidValue;
}

}  // namespace rfkv
