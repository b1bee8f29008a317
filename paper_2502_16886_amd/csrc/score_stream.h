// The streaming scoring pass (Sec. 3.2 "Reducing Overhead", Eq. 2) as a device function: one
// workgroup's share of the statistics pass or of the reduction pass, with the hand-overs between the
// workgroups of a unit (statistics merge, position-ranking cut) done by the last one to finish.
// Used by the per-layer kernels (score_qreg.hip) and by the kernel that runs the passes of several
// layers side by side (pipeline.hip).
#pragma once

#include "kernels.h"
#include "score_common.h"
#include "select_position.h"
#include "tile_sum.h"

namespace rfkv {
namespace {

constexpr int kStreamThreads = 256;

// Folds the per-span statistics of a unit into one exponent offset per row, b_r = ref_r + log2(sum_r * G)
// (+inf for rows that do not exist), by the workgroup that finished the unit's statistics pass last.
// Thread (row group rr, lane sub): rows j * 8 + rr, spans sub, sub + 32, ... in order, then a butterfly
// over the 32 lanes of a row: the arithmetic, operation for operation, of score_merge_kernel.
template <int RT_T>
__device__ __forceinline__ void merge_unit_statistics(const ScoreArgs& a, const Unit& u, int unit) {
  constexpr int J = RT_T * 4;                          // groups of 8 rows
  const int sub = threadIdx.x & 31, rr = threadIdx.x >> 5;
  const int nsp = (u.n + a.span - 1) / a.span;
  const float2* p = a.partials + (int64_t)unit * a.nspans * a.rows_pad;
  float m[J], sum[J];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    m[j] = -1e30f;
    sum[j] = 0.f;
  }
  for (int s = sub; s < nsp; s += 32) {
    // all J loads in flight, no branch between them (a load behind a branch is waited for on the spot); rows
    // that do not exist read an existing row's word and are replaced
    float2 v[J];
#pragma unroll
    for (int j = 0; j < J; ++j) v[j] = coherent_load(p + (int64_t)s * a.rows_pad + min(j * 8 + rr, u.rows - 1));
#pragma unroll
    for (int j = 0; j < J; ++j)
      if (j * 8 + rr >= u.rows) v[j] = make_float2(-1e30f, 0.f);
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const float nm = fmaxf(m[j], v[j].x);
      sum[j] = sum[j] * fast_exp2(m[j] - nm) + v[j].y * fast_exp2(v[j].x - nm);
      m[j] = nm;
    }
  }
#pragma unroll
  for (int j = 0; j < J; ++j) {
#pragma unroll
    for (int d = 16; d >= 1; d >>= 1) {
      const float om = __shfl_xor(m[j], d), os = __shfl_xor(sum[j], d);
      const float nm = fmaxf(m[j], om);
      sum[j] = sum[j] * fast_exp2(m[j] - nm) + os * fast_exp2(om - nm);
      m[j] = nm;
    }
    const int r = j * 8 + rr;
    if (sub == 0)
      coherent_store(a.bvec + (int64_t)unit * a.rows_pad + r,
                     r < u.rows ? m[j] + __log2f(sum[j] * (float)a.group) : __builtin_inff());
  }
}

// The unit's position-ranking cut (Sec. 3.2 "Initial Ranking", Eq. 1) by the workgroup that finished the
// unit's scores last: every score and tile sum of the unit has been written with coherent stores.
__device__ __forceinline__ void cut_unit(const ScoreArgs& a, const Unit& u, int unit, PositionShared<kStreamThreads>* sh) {
  const int m_eff = min(max(a.n_sink, 0), u.n);
  const HeadMass mass{a.scores + (int64_t)u.h * a.total_tokens + u.s0, a.tile_sq + (int64_t)u.h * a.tiles_total + u.tile_base};
  const int kept = position_cut<kStreamThreads>(mass, u.n, m_eff, a.threshold, a.min_keep, sh);
  if (threadIdx.x == 0) {
    coherent_store(a.kept + unit, kept);
    a.desc[unit] = make_int4(kept, min(kept, m_eff), 0, 0);
  }
}

// PASS 1: per-row (reference exponent, sum) partials of this workgroup's span.
// PASS 2: scores (and per-tile squared sums) of this workgroup's span.
// PASS 3: pass 1 that also writes the logits of up to kSpillRows rows (the paper's k = 1: the
//         G rows of the last query position), so that the scores follow from 4 * rows bytes per key
//         instead of a second pass over the keys (score_spill_reduce_kernel).
// WIDE:   pass 1 over one block of RT_T row tiles out of many (blockIdx.z picks the block): the
//         statistics of windows with more rows than a workgroup can hold (the large windows of the
//         paper's ablation of k, "Attention Matrix Reduction": k = 1 %, 5 %, 10 % of n).
// LDS of one streaming workgroup.  Distinct objects, so that reads of one are known not to touch a
// buffer with loads in flight.
template <typename T, int D, int RT_T>
struct StreamLds {
  static constexpr int kWaves = 4;
  static constexpr int kTileBytes = 32 * Shape<T, D>::kRowBytes;
  unsigned char* smem;      // [kWaves * kTileBytes], 1 KB aligned: tile buffers
  unsigned char* smem_b;    // [kWaves * kTileBytes], 1 KB aligned: the window queries on their way to registers, then the odd tiles
  float* bsm;               // [max(64, RT_T * 32)], 256 B aligned: pass 2, exponent offset per row
  int* rlast_s;             // [RT_T * 32], 16 B aligned: pass 2, last visible key per row
};
#define RFKV_STREAM_LDS(T, D, RT_T, name)                                                                   \
  __shared__ __attribute__((aligned(1024))) unsigned char name##_a[4 * 32 * Shape<T, D>::kRowBytes];        \
  __shared__ __attribute__((aligned(1024))) unsigned char name##_b[4 * 32 * Shape<T, D>::kRowBytes];        \
  __shared__ __attribute__((aligned(256))) float name##_c[(RT_T) * 32 < 64 ? 64 : (RT_T) * 32];             \
  __shared__ __attribute__((aligned(16))) int name##_d[(RT_T) * 32];                                        \
  const StreamLds<T, D, RT_T> name{name##_a, name##_b, name##_c, name##_d}

// One workgroup's share of a scoring pass: work item (block_x, block_y) = (span, unit), or for WIDE
// block_x = the one-dimensional item number.  Every thread of the workgroup calls it; all of them
// have left LDS alone when it returns.
template <typename T, int D, int RT_T, int PASS, bool WIDE = false>
__device__ __forceinline__ void score_stream_body(const ScoreArgs& a, int block_x, int block_y,
                                                  const StreamLds<T, D, RT_T>& lds) {
  using S = Shape<T, D>;
  constexpr bool kStats = PASS != 2;                   // pass 1 (and 3: pass 1 that also keeps its logits)
  constexpr bool kSpill = PASS == 3;
  static_assert(!kSpill || RT_T == 1, "logits are kept for a single row tile only");
  static_assert(!WIDE || PASS == 1, "row blocks exist for the statistics pass only");
  constexpr int kWaves = 4;
  constexpr int kThreads = kWaves * 64;
  constexpr int kTileBytes = 32 * S::kRowBytes;
  constexpr int kLoads = kTileBytes / 1024;            // direct-to-LDS instructions per tile
  unsigned char* const smem = lds.smem;
  unsigned char* const smem_b = lds.smem_b;
  float* const bsm = lds.bsm;
  int* const rlast_s = lds.rlast_s;
  int bx = block_x, by = block_y, rblock = 0;
  if (WIDE) {
    // One-dimensional grid, work item w = row block + blocks * (span + spans * unit).  Workgroups go
    // to the 8 XCDs in turn, so workgroup g takes item (g % 8) * chunk + g / 8: the workgroups
    // resident on one XCD are consecutive items, i.e. the row blocks of one span of keys, and
    // share that span in their L2 instead of each streaming it from memory.
    const int chunk = (a.wide_items + 7) >> 3;
    const int w = (block_x & 7) * chunk + (block_x >> 3);
    if ((block_x >> 3) >= chunk || w >= a.wide_items) return;
    const int blocks = a.rows_pad / (RT_T * 32);
    rblock = w % blocks;
    const int rest = w / blocks;
    bx = rest % a.nspans;
    by = rest / a.nspans;
  }
  const Unit u = load_unit(a, by);
  const int span_begin = bx * a.span;
  if (span_begin >= u.n) {                             // uniform for the whole workgroup
    if (PASS == 2 && a.fuse_select && u.n == 0 && bx == 0 && threadIdx.x == 0) {
      a.kept[by] = 0;                                  // an empty sequence has no workgroup that could be its last
      a.desc[by] = make_int4(0, 0, 0, 0);
    }
    return;
  }
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
      const double tsq = tile_sum_sq(score, lane);
      double* tsq_out = a.tile_sq + (int64_t)u.h * a.tiles_total + u.tile_base + (tile0 >> 5);
      if (a.fuse_select) {
        // coherent stores: the unit's last workgroup reads scores and tile sums of all the others
        if (hi == 0 && key < u.n) coherent_store(out + key, score);
        if (lane == 0) coherent_store(tsq_out, tsq);
      } else {
        if (hi == 0 && key < u.n) out[key] = score;
        if (lane == 0) *tsq_out = tsq;
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // no load may still be writing LDS from here on
  if (PASS == 2 && a.sel_block && bx == 0) clear_select_block(a.sel_block, by);
  if (PASS == 2 && a.fuse_select) {
    __syncthreads();                                   // every wavefront is done with its tile buffers
    PositionShared<kStreamThreads>* sh = reinterpret_cast<PositionShared<kStreamThreads>*>(smem);
    int* flag = reinterpret_cast<int*>(smem_b);
    const int nsp = (u.n + a.span - 1) / a.span;
    if (last_arrival(a.counters + a.units + by, nsp, flag)) cut_unit(a, u, by, sh);
  }
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
      if (WIDE || !a.fuse_merge) a.partials[((int64_t)by * a.nspans + bx) * a.rows_pad + row0 + r] = make_float2(m, s);
      else coherent_store(a.partials + ((int64_t)by * a.nspans + bx) * a.rows_pad + row0 + r, make_float2(m, s));
    }
    if (!WIDE && a.fuse_merge) {
      // the last workgroup of the unit folds the spans' statistics: no merge kernel
      int* flag = reinterpret_cast<int*>(smem_b);
      const int nsp = (u.n + a.span - 1) / a.span;
      if (last_arrival(a.counters + by, nsp, flag)) merge_unit_statistics<RT_T>(a, u, by);
    }
  }
}

}  // namespace
}  // namespace rfkv
