// Scoring kernels for gfx950 (Sec. 3.2 "Reducing Overhead", Eq. 2 of the paper).
//
// A'[i] = (1/G) sum_g (1/cnt_i) sum_t softmax_row(t, g)[i] needs every row's softmax
// normaliser before any column can be finished, so the keys are streamed twice:
//
//   score_stats_kernel   logits = K . Q^T on the matrix cores (keys along M, window rows
//                        along N, so one lane owns one row and 16 keys per tile) and a
//                        running (reference exponent, sum of 2^x) per row; one partial per
//                        workgroup span.
//   score_merge_kernel   folds the per-span partials into one offset per row,
//                        b_r = ref_r + log2(sum_r * G).
//   score_reduce_kernel  logits again with the operands swapped (rows along M, keys along
//                        N, so one lane owns one key and the row reduction is in-lane),
//                        p = 2^(logit * c - b_r), column sum, divide by the causal count.
//
// Operand layout.  A 32x32 MFMA wants, per lane, 16 bytes of the contraction axis of row
// (lane % 32); which elements those are is free as long as both operands agree.  Each lane
// therefore owns one contiguous half of its row (lane / 32 picks the half) and feeds
// 16-byte chunk c of it at step c: global loads of K are eight consecutive 16-byte loads
// per lane, and Q is staged in LDS with a 16-byte row pad so the same chunk reads are
// bank-conflict free.  fp32 inputs use the 32x32x2 fp32 MFMA with the same scheme.
#include "kernels.h"
#include "score_common.h"
#include "tile_sum.h"

namespace rfkv {
namespace {

template <typename T, int D>
__device__ __forceinline__ void load_k_half(uint4* f, const unsigned char* kunit,
                                            int64_t tok_bytes, int key, int hi) {
  const uint4* p = reinterpret_cast<const uint4*>(kunit + (int64_t)key * tok_bytes + hi * Shape<T, D>::kHalfBytes);
#pragma unroll
  for (int c = 0; c < Shape<T, D>::kChunks; ++c) f[c] = p[c];
}

// ---------------------------------------------------------------------------------------------
// pass 1: per-row (reference exponent, sum) over this workgroup's span of keys
// ---------------------------------------------------------------------------------------------
template <typename T, int D, int RT_T>
__global__ __launch_bounds__(kBlockThreads, 2) void score_stats_kernel(ScoreArgs a) {
  using S = Shape<T, D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const Unit u = load_unit(a, blockIdx.y);
  const int span_begin = blockIdx.x * a.span;
  if (span_begin >= u.n) return;                       // uniform for the whole workgroup
  const int span_end = min(u.n, span_begin + a.span);

  stage_q<T, D>(a, u, smem);
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hi = lane >> 5;
  const float c = a.c;
  const float kNegInf = -__builtin_inff();

  float mc[RT_T], l[RT_T];
  int rowlast[RT_T];                                   // last key this lane's row may see
#pragma unroll
  for (int rt = 0; rt < RT_T; ++rt) {
    mc[rt] = -1e30f;
    l[rt] = 0.f;
    const int r = rt * 32 + col;
    rowlast[rt] = r < u.rows ? u.n - u.wp + r / a.group : -1;
  }
  const int first_masked_key = u.n - u.wp + 1;         // keys below are visible to every row
  const unsigned char* kunit = static_cast<const unsigned char*>(a.k) +
                               ((int64_t)u.s0 * a.k_stride_tok + (int64_t)u.h * a.k_stride_head) * T::kBytes;
  const int64_t tok_bytes = a.k_stride_tok * T::kBytes;

  for (int tile0 = span_begin + wave * (KT * 32); tile0 < span_end; tile0 += 4 * KT * 32) {
    uint4 kf[KT][S::kChunks];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
      load_k_half<T, D>(kf[kt], kunit, tok_bytes, min(tile0 + kt * 32 + col, u.n - 1), hi);
    const bool masked = tile0 + KT * 32 > first_masked_key;

#pragma unroll
    for (int rt = 0; rt < RT_T; ++rt) {
      if (rt < u.row_tiles) {
        f32x16 acc[KT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[kt][i] = 0.f;
        const unsigned char* qrow = smem + (rt * 32 + col) * S::kLdsRowBytes + hi * S::kHalfBytes;
#pragma unroll
        for (int ch = 0; ch < S::kChunks; ++ch) {
          const uint4 qf = *reinterpret_cast<const uint4*>(qrow + ch * 16);
#pragma unroll
          for (int kt = 0; kt < KT; ++kt) acc[kt] = mma_chunk<T>(kf[kt][ch], qf, acc[kt]);   // keys x rows
        }
        if (masked) {
#pragma unroll
          for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = tile0 + kt * 32 + (i >> 2) * 8 + hi * 4 + (i & 3);
              if (key > rowlast[rt]) acc[kt][i] = kNegInf;
            }
        }
        float tmax = kNegInf;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, acc[kt][i]);
        const float mnew = fmaxf(mc[rt], tmax * c);
        float sum = 0.f;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) sum += fast_exp2(__builtin_fmaf(acc[kt][i], c, -mnew));
        l[rt] = l[rt] * fast_exp2(mc[rt] - mnew) + sum;
        mc[rt] = mnew;
      }
    }
  }

  // the two half-waves hold disjoint keys of the same rows
#pragma unroll
  for (int rt = 0; rt < RT_T; ++rt) {
    const float om = other_half(mc[rt]), ol = other_half(l[rt]);
    const float nm = fmaxf(mc[rt], om);
    l[rt] = l[rt] * fast_exp2(mc[rt] - nm) + ol * fast_exp2(om - nm);
    mc[rt] = nm;
  }
  __syncthreads();                                     // everyone is done reading Q from LDS
  const int rows32 = u.row_tiles * 32;
  float2* red = reinterpret_cast<float2*>(smem);       // [4 waves][rows32]
  if (hi == 0) {
#pragma unroll
    for (int rt = 0; rt < RT_T; ++rt)
      if (rt < u.row_tiles) red[wave * rows32 + rt * 32 + col] = make_float2(mc[rt], l[rt]);
  }
  __syncthreads();
  for (int r = threadIdx.x; r < rows32; r += kBlockThreads) {
    float m = red[r].x, s = red[r].y;
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float2 o = red[w * rows32 + r];
      const float nm = fmaxf(m, o.x);
      s = s * fast_exp2(m - nm) + o.y * fast_exp2(o.x - nm);
      m = nm;
    }
    a.partials[((int64_t)blockIdx.y * a.nspans + blockIdx.x) * a.rows_pad + r] = make_float2(m, s);
  }
}

// ---------------------------------------------------------------------------------------------
// merge: b_r = ref_r + log2(sum_r * G); rows that do not exist get +inf (weight zero).
// Workgroup = 8 rows x 32 lanes; the 32 lanes of a row split the spans and combine by shuffles.
// ---------------------------------------------------------------------------------------------
constexpr int kMergeRows = 8;

__global__ __launch_bounds__(kBlockThreads) void score_merge_kernel(ScoreArgs a) {
  const Unit u = load_unit(a, blockIdx.y);
  const int r = blockIdx.x * kMergeRows + (threadIdx.x >> 5);
  const int sub = threadIdx.x & 31;
  if (r >= a.rows_pad) return;
  const int nsp = (u.n + a.span - 1) / a.span;
  const float2* p = a.partials + (int64_t)blockIdx.y * a.nspans * a.rows_pad + r;
  float m = -1e30f, sum = 0.f;
  if (r < u.rows) {
    for (int s = sub; s < nsp; s += 32) {
      const float2 v = p[(int64_t)s * a.rows_pad];
      const float nm = fmaxf(m, v.x);
      sum = sum * fast_exp2(m - nm) + v.y * fast_exp2(v.x - nm);
      m = nm;
    }
  }
#pragma unroll
  for (int d = 16; d >= 1; d >>= 1) {
    const float om = __shfl_xor(m, d), os = __shfl_xor(sum, d);
    const float nm = fmaxf(m, om);
    sum = sum * fast_exp2(m - nm) + os * fast_exp2(om - nm);
    m = nm;
  }
  if (sub == 0)
    a.bvec[(int64_t)blockIdx.y * a.rows_pad + r] =
        r < u.rows ? m + __log2f(sum * (float)a.group) : __builtin_inff();
}

// Row offsets from a log-sum-exp the caller already has (the causal attention forward of the prefill
// returns ln sum_i exp(scale q.k_i) per query row): b_r = lse_r * log2(e) + log2(G), the value the
// statistics pass and the merge would have produced.  Rows that do not exist get +inf.
__global__ __launch_bounds__(kBlockThreads) void score_lse_offsets_kernel(ScoreArgs a) {
  const Unit u = load_unit(a, blockIdx.y);
  const int r = blockIdx.x * kBlockThreads + threadIdx.x;
  if (r >= a.rows_pad) return;
  float b = __builtin_inff();
  if (r < u.rows) {
    const int t = r / a.group, g = r - t * a.group;
    const double lse = (double)a.lse[(int64_t)(u.q0 + t) * a.n_q_heads + u.h * a.group + g];
    b = (float)(lse * 1.4426950408889634 + log2((double)a.group));
  }
  a.bvec[(int64_t)blockIdx.y * a.rows_pad + r] = b;
}

// ---------------------------------------------------------------------------------------------
// pass 2: column sums of the normalised probabilities
// ---------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(kBlockThreads, 2) void score_reduce_kernel(ScoreArgs a) {
  using S = Shape<T, D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const Unit u = load_unit(a, blockIdx.y);
  const int span_begin = blockIdx.x * a.span;
  if (span_begin >= u.n) return;
  const int span_end = min(u.n, span_begin + a.span);
  const int rows32 = u.row_tiles * 32;

  if (blockIdx.x == 0 && a.sel_block) clear_select_block(a.sel_block, blockIdx.y);   // for the score ranking of long units
  stage_q<T, D>(a, u, smem);
  float* bsm = reinterpret_cast<float*>(smem + rows32 * S::kLdsRowBytes);   // [rows32] exponent offsets
  int* rlast = reinterpret_cast<int*>(bsm + rows32);                        // [rows32] last visible key
  for (int r = threadIdx.x; r < rows32; r += kBlockThreads) {
    bsm[r] = a.bvec[(int64_t)blockIdx.y * a.rows_pad + r];
    rlast[r] = r < u.rows ? u.n - u.wp + r / a.group : -1;
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hi = lane >> 5;
  const float c = a.c;
  const int first_masked_key = u.n - u.wp + 1;
  const unsigned char* kunit = static_cast<const unsigned char*>(a.k) +
                               ((int64_t)u.s0 * a.k_stride_tok + (int64_t)u.h * a.k_stride_head) * T::kBytes;
  const int64_t tok_bytes = a.k_stride_tok * T::kBytes;
  float* out = a.scores + (int64_t)u.h * a.total_tokens + u.s0;

  for (int tile0 = span_begin + wave * (KT * 32); tile0 < span_end; tile0 += 4 * KT * 32) {
    uint4 kf[KT][S::kChunks];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
      load_k_half<T, D>(kf[kt], kunit, tok_bytes, min(tile0 + kt * 32 + col, u.n - 1), hi);
    const bool masked = tile0 + KT * 32 > first_masked_key;

    float colsum[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) colsum[kt] = 0.f;

    for (int rt = 0; rt < u.row_tiles; ++rt) {
      f32x16 acc[KT];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[kt][i] = 0.f;
      const unsigned char* qrow = smem + (rt * 32 + col) * S::kLdsRowBytes + hi * S::kHalfBytes;
#pragma unroll
      for (int ch = 0; ch < S::kChunks; ++ch) {
        const uint4 qf = *reinterpret_cast<const uint4*>(qrow + ch * 16);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) acc[kt] = mma_chunk<T>(qf, kf[kt][ch], acc[kt]);     // rows x keys
      }
      // accumulator i of this lane is row rt*32 + (i/4)*8 + hi*4 + i%4, key tile0 + kt*32 + col
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int rbase = rt * 32 + j * 8 + hi * 4;
        const float4 bv = *reinterpret_cast<const float4*>(bsm + rbase);
        const float bb[4] = {bv.x, bv.y, bv.z, bv.w};
        if (!masked) {
#pragma unroll
          for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int e = 0; e < 4; ++e) colsum[kt] += fast_exp2(__builtin_fmaf(acc[kt][j * 4 + e], c, -bb[e]));
        } else {
          const int4 rv = *reinterpret_cast<const int4*>(rlast + rbase);
          const int rl[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
          for (int kt = 0; kt < KT; ++kt) {
            const int key = tile0 + kt * 32 + col;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float p = fast_exp2(__builtin_fmaf(acc[kt][j * 4 + e], c, -bb[e]));
              colsum[kt] += key <= rl[e] ? p : 0.f;
            }
          }
        }
      }
    }
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const float tot = colsum[kt] + other_half(colsum[kt]);
      const int key = tile0 + kt * 32 + col;
      const float score = key < u.n ? tot / (float)min(u.wp, u.n - key) : 0.f;
      if (hi == 0 && key < u.n) out[key] = score;
      const double tsq = tile_sum_sq(score, lane);
      if (lane == 0 && tile0 + kt * 32 < u.n)
        a.tile_sq[(int64_t)u.h * a.tiles_total + u.tile_base + (tile0 >> 5) + kt] = tsq;
    }
  }
}

template <typename T, int D, int RT_T>
hipError_t launch_stats(const Geometry& g, const ScoreArgs& a, dim3 grid, hipStream_t stream) {
  const size_t lds = (size_t)g.rows_pad * Shape<T, D>::kLdsRowBytes;
  hipError_t e = allow_lds<&score_stats_kernel<T, D, RT_T>>(kMaxQueryLds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_stats_kernel<T, D, RT_T>), grid, dim3(kBlockThreads), lds, stream, a);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_typed(const Geometry& g, const ScoreArgs& a, hipStream_t stream, const Marks* marks) {
  const dim3 grid(g.nspans, g.units);
  const int rt = g.rows_pad / 32;
  hipError_t e = launch_score_offsets(g, a, stream, marks);    // from the caller's log-sum-exp, if given
  if (e != hipSuccess) return e;
  if (!a.lse) {
    if (rt <= 1) e = launch_stats<T, D, 1>(g, a, grid, stream);
    else if (rt <= 2) e = launch_stats<T, D, 2>(g, a, grid, stream);
    else if (rt <= 4) e = launch_stats<T, D, 4>(g, a, grid, stream);
    else if (rt <= 8) e = launch_stats<T, D, 8>(g, a, grid, stream);
    else e = launch_stats<T, D, 16>(g, a, grid, stream);
    if (e != hipSuccess) return e;
    if (marks) marks->after(kKernelStats);

    e = launch_score_merge(g, a, stream);
    if (e != hipSuccess) return e;
    if (marks) marks->after(kKernelMerge);
  }

  const size_t lds = (size_t)g.rows_pad * (Shape<T, D>::kLdsRowBytes + 8);
  e = allow_lds<&score_reduce_kernel<T, D>>(kMaxQueryLds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_reduce_kernel<T, D>), grid, dim3(kBlockThreads), lds, stream, a);
  e = hipGetLastError();
  if (marks && e == hipSuccess) marks->after(kKernelReduce);
  return e;
}

}  // namespace

hipError_t launch_score_merge(const Geometry& g, const ScoreArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(score_merge_kernel, dim3((g.rows_pad + kMergeRows - 1) / kMergeRows, g.units),
                     dim3(kBlockThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_score_offsets(const Geometry& g, const ScoreArgs& a, hipStream_t stream, const Marks* marks) {
  if (!a.lse) return hipSuccess;
  hipLaunchKernelGGL(score_lse_offsets_kernel, dim3((g.rows_pad + kBlockThreads - 1) / kBlockThreads, g.units),
                     dim3(kBlockThreads), 0, stream, a);
  const hipError_t e = hipGetLastError();
  if (marks && e == hipSuccess) {
    marks->after(kKernelStats);       // no statistics pass: zero time
    marks->after(kKernelMerge);       // the offsets kernel stands in for the merge
  }
  return e;
}

bool score_streams(const Geometry& g, bool bf16) { return !g.wide && score_qreg_covers(g, bf16); }

hipError_t launch_score(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream, const Marks* marks) {
  if (g.units == 0 || g.nspans == 0) return hipSuccess;
  if (g.wide) return launch_score_wide(g, a, bf16, stream, marks);
  if (score_qreg_covers(g, bf16)) return launch_score_qreg(g, a, bf16, stream, marks);
  if (bf16) {
    if (g.head_dim == 64) return launch_typed<Bf16, 64>(g, a, stream, marks);
    return launch_typed<Bf16, 128>(g, a, stream, marks);
  }
  if (g.head_dim == 64) return launch_typed<Fp32, 64>(g, a, stream, marks);
  return launch_typed<Fp32, 128>(g, a, stream, marks);
}

}  // namespace rfkv
