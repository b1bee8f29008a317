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
#include "tile_sum.h"

namespace rfkv {
namespace {

// PASS 1: per-row (reference exponent, sum) partials of this workgroup's span.
// PASS 2: scores (and per-tile squared sums) of this workgroup's span.
// PASS 3: pass 1 that also writes the logits of up to kSpillRows rows (the paper's k = 1: the
//         G rows of the last query position), so that the scores follow from 4 * rows bytes per key
//         instead of a second pass over the keys (score_spill_reduce_kernel).
// WIDE:   pass 1 over one block of RT_T row tiles out of many (blockIdx.z picks the block): the
//         statistics of windows with more rows than a workgroup can hold (the large windows of the
//         paper's ablation of k, "Attention Matrix Reduction": k = 1 %, 5 %, 10 % of n).
template <typename T, int D, int RT_T, int PASS, bool WIDE = false>
__global__ __launch_bounds__(256, 2) void score_stream_kernel(ScoreArgs a) {
  using S = Shape<T, D>;
  constexpr bool kStats = PASS != 2;                   // pass 1 (and 3: pass 1 that also keeps its logits)
  constexpr bool kSpill = PASS == 3;
  static_assert(!kSpill || RT_T == 1, "logits are kept for a single row tile only");
  static_assert(!WIDE || PASS == 1, "row blocks exist for the statistics pass only");
  constexpr int kWaves = 4;
  constexpr int kThreads = kWaves * 64;
  constexpr int kTileBytes = 32 * S::kRowBytes;
  constexpr int kLoads = kTileBytes / 1024;            // direct-to-LDS instructions per tile
  // distinct LDS objects, so that reads of one are known not to touch a buffer with loads in flight
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kWaves * kTileBytes];   // tile buffers
  // the window queries on their way to registers, then the odd tiles
  __shared__ __attribute__((aligned(1024))) unsigned char smem_b[kWaves * kTileBytes];
  __shared__ __attribute__((aligned(256))) float bsm[RT_T * 32 < 64 ? 64 : RT_T * 32];   // pass 2: exponent offset per row
  __shared__ __attribute__((aligned(16))) int rlast_s[RT_T * 32];    // pass 2: last visible key per row
  int bx = blockIdx.x, by = blockIdx.y, rblock = 0;
  if (WIDE) {
    // One-dimensional grid, work item w = row block + blocks * (span + spans * unit).  Workgroups go
    // to the 8 XCDs in turn, so workgroup g takes item (g % 8) * chunk + g / 8: the workgroups
    // resident on one XCD are consecutive items, i.e. the row blocks of one span of keys, and
    // share that span in their L2 instead of each streaming it from memory.
    const int chunk = (a.wide_items + 7) >> 3;
    const int w = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= chunk || w >= a.wide_items) return;
    const int blocks = a.rows_pad / (RT_T * 32);
    rblock = w % blocks;
    const int rest = w / blocks;
    bx = rest % a.nspans;
    by = rest / a.nspans;
  }
  const Unit u = load_unit(a, by);
  const int span_begin = bx * a.span;
  if (span_begin >= u.n) return;                       // uniform for the whole workgroup
  const int span_end = min(u.n, span_begin + a.span);
  const int row0 = WIDE ? rblock * (RT_T * 32) : 0;    // first score row of this workgroup
  if (WIDE && row0 >= u.row_tiles * 32) return;        // a short sequence has fewer window rows

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hi = lane >> 5;
  const float c = a.c;
  const float kNegInf = -__builtin_inff();
  unsigned char* kbuf0 = smem + wave * kTileBytes;     // this wavefront's tile buffer(s)
  unsigned char* kbuf1 = smem_b + wave * kTileBytes;
  const unsigned char* kunit = static_cast<const unsigned char*>(a.k) +
                               ((int64_t)u.s0 * a.k_stride_tok + (int64_t)u.h * a.k_stride_head) * T::kBytes;
  const int64_t tok_bytes = a.k_stride_tok * T::kBytes;
  const int first_masked_key = u.n - u.wp + 1;         // keys below are visible to every row
  constexpr int kStep = kWaves * 32;                   // keys the workgroup consumes per iteration

  int tile0 = span_begin + wave * 32;
  const TileLoader<T, D> tiles(kunit, tok_bytes, u.n, lane);
  uint4 qf[RT_T][S::kChunks];                          // query fragments of every row tile, for the whole kernel
  float mc[RT_T], l[RT_T];
  int rowlast[WIDE ? 1 : RT_T];                         // last key a lane's row sees (WIDE: worked out where it is needed)
  auto last_visible = [&](int rt) {
    const int r = row0 + rt * 32 + col;
    return r < u.rows ? u.n - u.wp + r / a.group : -1;
  };
  if (kStats) {
#pragma unroll
    for (int rt = 0; rt < RT_T; ++rt) {
      mc[rt] = -1e30f;
      l[rt] = 0.f;
      if (!WIDE) rowlast[rt] = last_visible(rt);
    }
  }
  {
    // Everything the loop needs arrives by direct-to-LDS loads, issued at once: the first key tile
    // (the bulk: memory is busy from the start), pass 2's per-row exponent offsets (64 per
    // wavefront) and one row tile of window queries per wavefront into the second buffer set.
    // No register depends on a load (the caller's log-sum-exp, if given, aside), so the compiler
    // adds no wait of its own.  (Folding pass 1's per-span statistics here instead of in the merge
    // kernel measured slower: every one of the 512 workgroups then starts 3-4 us later.)
    static_assert(RT_T <= kWaves && RT_T * 32 <= kWaves * 64, "one query tile and 64 offsets per wavefront");
    if (tile0 < span_end) tiles.issue(tile0, kbuf0);
    if (PASS == 2) {
      if (threadIdx.x < RT_T * 32)
        lds_write_b32(rlast_s + threadIdx.x,
                      (uint32_t)((int)threadIdx.x < u.rows ? u.n - u.wp + (int)threadIdx.x / a.group : -1));
    }
    if (wave < RT_T) issue_q_tile_load<T, D>(a, u, (row0 >> 5) + wave, smem_b + wave * kTileBytes, lane);
    if (PASS == 2 && !a.lse && wave * 64 < RT_T * 32) {
      // the rows' exponent offsets from the merge kernel, 64 per wavefront
      const float* src = a.bvec + (int64_t)by * a.rows_pad + min(wave * 64 + lane, a.rows_pad - 1);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(bsm + wave * 64), 4, 0, 0);
    }
    float b_lse = __builtin_inff();
    if (PASS == 2 && a.lse && (int)threadIdx.x < u.rows) {
      // ... or from the caller's log-sum-exp (natural logarithm, scaled logits) of row (t, g):
      // b_r = lse_r * log2(e) + log2(G), formed here rather than by a kernel of its own
      const int r = threadIdx.x, t = r / a.group, g = r - t * a.group;
      const double lse = (double)a.lse[(int64_t)(u.q0 + t) * a.n_q_heads + u.h * a.group + g];
      b_lse = (float)(lse * 1.4426950408889634 + log2((double)a.group));
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_writes_done();
    __syncthreads();
    if (PASS == 2 && a.lse && threadIdx.x < RT_T * 32) bsm[threadIdx.x] = b_lse;      // +inf for rows that do not exist
#pragma unroll
    for (int rt = 0; rt < RT_T; ++rt) read_tile_frags<T, D>(qf[rt], smem_b + rt * kTileBytes, col, hi);
    __syncthreads();                                   // the query tiles become the second buffer set
    if (tile0 + kStep < span_end) tiles.issue(tile0 + kStep, kbuf1);
  }
  float* out = a.scores + (int64_t)u.h * a.total_tokens + u.s0;

  // From here on the loop counts the loads and stores in flight itself.  Per iteration a wavefront
  // issues the kLoads loads of one tile and, in pass 2, kStores stores (scores, tile sum).
  constexpr int kStores = PASS == 2 ? 2 : (kSpill ? 4 : 0);
  for (int it = 0; tile0 < span_end; tile0 += kStep, ++it) {
    uint4 kf[S::kChunks];
    unsigned char* kbuf = (it & 1) ? kbuf1 : kbuf0;
    // Loads and stores complete in issue order.  Behind this tile's loads there are at most the next
    // tile's loads and (from the second iteration on) the stores of the iteration before.
    if (tile0 + kStep < span_end) {
      if (it == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads + kStores) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    read_tile_frags<T, D>(kf, kbuf, col, hi);          // complete on return: the buffer is free
    constexpr int kAhead = 2 * kStep;
    if (tile0 + kAhead < span_end) tiles.issue(tile0 + kAhead, kbuf);
    const bool masked = tile0 + 32 > first_masked_key;

    float colsum = 0.f;
    // Logits of one row tile against this key tile.  Row tiles past the unit's rows hold zero
    // queries: they are computed like the others and their results are never used.
    auto logits = [&](int rt) {
      f32x16 acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
      for (int ch = 0; ch < S::kChunks; ++ch) {
        const uint4 q = qf[rt][ch];
        acc = kStats ? mma_chunk<T>(kf[ch], q, acc)      // keys x rows: a lane owns one row
                        : mma_chunk<T>(q, kf[ch], acc);     // rows x keys: a lane owns one key
      }
      return acc;
    };
    // The MFMA chain of row tile rt + 1 is issued before the softmax arithmetic of row tile rt: its
    // last MFMAs run under that arithmetic, and the other wavefront of the SIMD fills the rest of
    // the chain (a wavefront issues in order, so a dependent chain holds up what follows it).
    // Issuing the chain one MFMA at a time between slices of the arithmetic measured no faster here.
    f32x16 acc = logits(0);
#pragma unroll
    for (int rt = 0; rt < RT_T; ++rt) {
      f32x16 nxt = acc;
      if (rt + 1 < RT_T) nxt = logits(rt + 1);
      if (kStats) {
        if (masked) {
          const int rlast = WIDE ? last_visible(rt) : rowlast[WIDE ? 0 : rt];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = tile0 + (i >> 2) * 8 + hi * 4 + (i & 3);
            if (key > rlast) acc[i] = kNegInf;
          }
        }
        if (kSpill) {
          // raw logits (q . k, unscaled), row `col`, keys tile0 + 8 q + 4 hi + 0..3 per 16-byte store; the
          // buffer holds whole tiles, so the last tile's surplus keys are written and never read
          float* lrow = a.logits + ((int64_t)(u.h * kSpillRows + (col & (kSpillRows - 1))) * a.tiles_total + u.tile_base) * 32 +
                        tile0 + hi * 4;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float4 v = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
            if (col < kSpillRows) *reinterpret_cast<float4*>(lrow + q * 8) = v;
          }
        }
        // The reference exponent only has to keep 2^x in range, not to be the maximum: once every row of
        // the wavefront has one, a tile is summed against it as it stands, and only a tile that would
        // push a sum towards overflow (a logit more than 60 binary orders above the reference) or a row
        // that has seen no key yet takes the path that looks for the tile's maximum first.
        float sum = 0.f;
        bool plain = __all(mc[rt] > -1e29f);                // uniform over the wavefront
        if (plain) {
#pragma unroll
          for (int i = 0; i < 16; ++i) sum += fast_exp2(__builtin_fmaf(acc[i], c, -mc[rt]));
          plain = __all(sum < 0x1p60f);                      // false for inf and NaN as well
          if (plain) l[rt] += sum;
        }
        if (!plain) {
          float tmax = kNegInf;
#pragma unroll
          for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, acc[i]);
          const float mnew = fmaxf(mc[rt], tmax * c);
          sum = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) sum += fast_exp2(__builtin_fmaf(acc[i], c, -mnew));
          l[rt] = l[rt] * fast_exp2(mc[rt] - mnew) + sum;
          mc[rt] = mnew;
        }
      } else {
        // accumulator i of this lane: row rt*32 + (i/4)*8 + hi*4 + i%4, key tile0 + col
        float4 bv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = *reinterpret_cast<const float4*>(bsm + rt * 32 + j * 8 + hi * 4);
        if (!masked) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            colsum += fast_exp2(__builtin_fmaf(acc[j * 4 + 0], c, -bv[j].x));
            colsum += fast_exp2(__builtin_fmaf(acc[j * 4 + 1], c, -bv[j].y));
            colsum += fast_exp2(__builtin_fmaf(acc[j * 4 + 2], c, -bv[j].z));
            colsum += fast_exp2(__builtin_fmaf(acc[j * 4 + 3], c, -bv[j].w));
          }
        } else {
          const int key = tile0 + col;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int4 rv = *reinterpret_cast<const int4*>(rlast_s + rt * 32 + j * 8 + hi * 4);
            const float p0 = fast_exp2(__builtin_fmaf(acc[j * 4 + 0], c, -bv[j].x));
            const float p1 = fast_exp2(__builtin_fmaf(acc[j * 4 + 1], c, -bv[j].y));
            const float p2 = fast_exp2(__builtin_fmaf(acc[j * 4 + 2], c, -bv[j].z));
            const float p3 = fast_exp2(__builtin_fmaf(acc[j * 4 + 3], c, -bv[j].w));
            colsum += (key <= rv.x ? p0 : 0.f) + (key <= rv.y ? p1 : 0.f) + (key <= rv.z ? p2 : 0.f) +
                      (key <= rv.w ? p3 : 0.f);
          }
        }
      }
      acc = nxt;
    }
    if (PASS == 2) {
      const float tot = colsum + other_half(colsum);
      const int key = tile0 + col;
      const float score = key < u.n ? tot / (float)min(u.wp, u.n - key) : 0.f;
      if (hi == 0 && key < u.n) out[key] = score;
      const double tsq = tile_sum_sq(score, lane);
      if (lane == 0) a.tile_sq[(int64_t)u.h * a.tiles_total + u.tile_base + (tile0 >> 5)] = tsq;
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // no load may still be writing LDS from here on
  if (kStats) {
    // the two half-waves hold disjoint keys of the same rows; then the four wavefronts
#pragma unroll
    for (int rt = 0; rt < RT_T; ++rt) {
      const float om = other_half(mc[rt]), ol = other_half(l[rt]);
      const float nm = fmaxf(mc[rt], om);
      l[rt] = l[rt] * fast_exp2(mc[rt] - nm) + ol * fast_exp2(om - nm);
      mc[rt] = nm;
    }
    __syncthreads();                                   // every wavefront is done with its tile buffer
    constexpr int kRows32 = RT_T * 32;
    float2* red = reinterpret_cast<float2*>(smem);     // [kWaves][kRows32]
    if (hi == 0) {
#pragma unroll
      for (int rt = 0; rt < RT_T; ++rt) red[wave * kRows32 + rt * 32 + col] = make_float2(mc[rt], l[rt]);
    }
    __syncthreads();
    for (int r = threadIdx.x; r < (WIDE ? RT_T * 32 : u.row_tiles * 32); r += kThreads) {
      float m = red[r].x, s = red[r].y;
#pragma unroll
      for (int w = 1; w < kWaves; ++w) {
        const float2 o = red[w * kRows32 + r];
        const float nm = fmaxf(m, o.x);
        s = s * fast_exp2(m - nm) + o.y * fast_exp2(o.x - nm);
        m = nm;
      }
      a.partials[((int64_t)by * a.nspans + bx) * a.rows_pad + row0 + r] = make_float2(m, s);
    }
  }
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
  if (key < u.n) a.scores[(int64_t)u.h * a.total_tokens + u.s0 + key] = score;
  // per-tile squared sums: the butterfly of tile_sum_sq, in both halves of the wavefront at once
  double v = (double)score * (double)score;
#pragma unroll
  for (int d = 16; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  if ((threadIdx.x & 31) == 0 && key < u.n) a.tile_sq[(int64_t)u.h * a.tiles_total + u.tile_base + (key >> 5)] = v;
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
