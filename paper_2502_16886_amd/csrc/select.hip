// Ranking + Uni-Metric budget rule for gfx950 (Sec. 3.2 "Initial Ranking", Eq. 1; Sec. 3.3, Eq. 3).
//
// One workgroup of 1024 threads per unit (sequence, KV head).  The squared scores are turned
// into integers q_i = round(s_i^2 * 2^60 / F^2), so every prefix mass P_i is an exact integer
// sum: any reduction order (tree, atomics) gives the same value and two runs are bit-identical.
// The stopping test is the paper's, evaluated in fp64 on the exact ratio:
//     1 - sqrt(P_i / P_n) < T.
//
// Position ranking (first m positions, then the rest from the end backwards): a block-wide
// exclusive scan of per-thread chunk masses in rank order locates the thread whose chunk holds
// the crossing; that thread walks its chunk.
//
// Score ranking (descending score, ties by ascending position): most-significant-digit radix
// select over the order-preserving bit pattern of the score (11 + 11 + 10 bits) with per-bucket
// counts and masses; the crossing bucket is found from a suffix scan over buckets, and the number
// of elements taken from the final all-equal bucket by bisection.  The retained positions are
// then emitted in ascending order with a block-wide scan (ties: the lowest positions win).
#include "kernels.h"
#include "select_position.h"
#include "tile_sum.h"

namespace rfkv {
namespace {

constexpr int kT = kSelectThreads;
constexpr int kPosThreads = 256;                   // the position ranking's workgroup, here and in the scoring pass
constexpr int kWaves = kT / 64;
constexpr int kBuckets = 2048;
constexpr int kMaxLdsFloats = 32768 + 4;           // scores of one unit held in LDS by the score ranking
constexpr int kMaxCandidates = 8192;               // scores of a unit's crossing bucket held in LDS (sliced units)
constexpr int kRankDirect = 128;                   // up to this many candidates are ranked pair by pair

struct Pred {
  double total;     // P_n as a double
  double T;
  int min_keep;
  double lo = 0.0, hi = -1.0;   // set_total: masses below lo certainly fail the rule, above hi certainly meet it
  // Away from the boundary the squared form P > (1 - T)^2 P_n decides (the margin of 1e-9 covers the
  // rounding of both forms many times over); only next to it is the paper's form evaluated.
  __device__ void set_total(double t) {
    total = t;
    if (T < 1.0) {
      const double thr = (1.0 - T) * (1.0 - T) * t;
      lo = thr * (1.0 - 1e-9);
      hi = thr * (1.0 + 1e-9);
    }
  }
  // Q(i, P): has the ranked prefix of i elements and mass P reached the stopping condition?
  __device__ bool operator()(int64_t count, uint64_t mass) const {
    if (count <= 0 || count < min_keep) return false;      // a prefix has at least one element
    const double m = (double)mass;
    if (hi >= lo) {
      if (m > hi) return true;
      if (m < lo) return false;
    }
    return 1.0 - sqrt(m / total) < T;
  }
};

__device__ __forceinline__ uint32_t order_key(float s) {
  const uint32_t b = __float_as_uint(s);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ uint64_t quantise(float s, double inv) {
  const double v = (double)s * (double)s * inv;
  return (uint64_t)__double2ll_rn(v);
}

template <typename V>
__device__ __forceinline__ V wave_inclusive_scan(V v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const V o = __shfl_up(v, d);
    if (lane >= d) v += o;
  }
  return v;
}

// Exclusive scan of two values over the 1024 threads (thread order) behind one pair of barriers;
// x and y become the exclusive prefixes, *tot_x and *tot_y the totals.
__device__ __forceinline__ void block_exclusive_scan2(uint64_t& x, uint64_t& y, uint64_t (*wave_tot)[2] /*[kWaves] LDS*/,
                                                      uint64_t* tot_x, uint64_t* tot_y) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t ix = wave_inclusive_scan(x, lane), iy = wave_inclusive_scan(y, lane);
  __syncthreads();
  if (lane == 63) {
    wave_tot[wave][0] = ix;
    wave_tot[wave][1] = iy;
  }
  __syncthreads();
  uint64_t ox = 0, oy = 0, tx = 0, ty = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint64_t wx = wave_tot[w][0], wy = wave_tot[w][1];
    if (w < wave) {
      ox += wx;
      oy += wy;
    }
    tx += wx;
    ty += wy;
  }
  x = ox + ix - x;
  y = oy + iy - y;
  *tot_x = tx;
  *tot_y = ty;
}

// Four consecutive scores from one 16-byte load.  `al` is the unit's score pointer moved back to
// a 16-byte boundary (by `mis` floats), q the first of the four as an index from `al`; the
// unit's scores are al[mis .. span).  A vector that is not wholly inside falls back to guarded
// scalar loads (never touching memory outside the unit); entries outside read as 0.
__device__ __forceinline__ float4 load_scores4(const float* al, int q, int mis, int span) {
  if (q >= mis && q + 4 <= span) return *reinterpret_cast<const float4*>(al + q);
  float4 v;
  v.x = (q + 0 >= mis && q + 0 < span) ? al[q + 0] : 0.f;
  v.y = (q + 1 >= mis && q + 1 < span) ? al[q + 1] : 0.f;
  v.z = (q + 2 >= mis && q + 2 < span) ? al[q + 2] : 0.f;
  v.w = (q + 3 >= mis && q + 3 < span) ? al[q + 3] : 0.f;
  return v;
}

// kBatch 4-vectors of scores, q[j] = qb + (j * kT + tid) * 4, all loads in flight at once: the vectors
// that lie wholly inside the unit (all but its two ends) are loaded without a branch between them.
template <int kBatch>
__device__ __forceinline__ void load_scores_batch(float4* v, const float* al, int qb, int mis, int span) {
  const int tid = threadIdx.x;
  const int q_first = qb + tid * 4, q_last = qb + ((kBatch - 1) * kT + tid) * 4;
  if (q_first >= mis && q_last + 4 <= span) {
#pragma unroll
    for (int j = 0; j < kBatch; ++j) v[j] = *reinterpret_cast<const float4*>(al + qb + (j * kT + tid) * 4);
  } else {
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int q = qb + (j * kT + tid) * 4;
      v[j] = q < span ? load_scores4(al, q, mis, span) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
}

// Per-tile squared-score sums straight from a score array (used when scoring did not run in
// the same call).  One wavefront per tile, same butterfly as the scoring kernel.
__global__ __launch_bounds__(kBlockThreads) void tile_sums_kernel(SelectArgs a) {
  const int unit = blockIdx.y;
  const int b = unit / a.n_kv_heads, h = unit - b * a.n_kv_heads;
  int tile_base = 0;
  for (int bb = 0; bb < b; ++bb) tile_base += (a.cu[bb + 1] - a.cu[bb] + kTileKeys - 1) / kTileKeys;
  const int s0 = a.cu[b];
  const int n = a.cu[b + 1] - s0;
  const int nt = (n + kTileKeys - 1) / kTileKeys;
  const int lane = threadIdx.x & 63;
  const int tile = blockIdx.x * (kBlockThreads / 64) + (threadIdx.x >> 6);
  if (blockIdx.x == 0 && a.sel_block) clear_select_block(a.sel_block, unit);   // for the score ranking of long units
  if (tile >= nt) return;                                  // uniform per wavefront
  const float* s = a.scores + (int64_t)h * a.total_tokens + s0;
  const int pos = tile * kTileKeys + lane;
  const float v = (lane < kTileKeys && pos < n) ? s[pos] : 0.f;
  const double t = tile_sum_sq(v, lane);
  if (lane == 0) a.tile_sq[(int64_t)h * a.tiles_total + tile_base + tile] = t;
}

struct SelectShared {
  uint64_t (*scan)[2];    // [kWaves][2]
  uint32_t* cnt;          // [kBuckets]
  uint64_t* mass;         // [kBuckets]
  int* i;                 // [8]
  uint64_t* u64;          // [2]
};

// Score ranking of one unit by the whole workgroup; returns the kept count and writes the retained
// positions (ascending) to idx_pad.  Positions are dealt out in 256-position chunks (one aligned
// 4-vector per lane), each wavefront owning a contiguous run of chunks.  A unit that fits the
// `lds_floats` floats at `lds` is copied there once and every pass reads it from LDS; a longer
// one is read from memory again in every pass.
__device__ __forceinline__ int score_rank(const float* s, int n, double inv, float threshold, int min_keep,
                                          int32_t* idx_pad, float* lds, int lds_floats, const SelectShared& sh) {
  constexpr int kChunkBatch = 4;                   // loads in flight per lane
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int mis = (int)((reinterpret_cast<uintptr_t>(s) >> 2) & 3);
  const float* al = s - mis;
  const int span = n + mis;
  const int nchunks = (span + 255) / 256;
  const int cpw = (nchunks + kWaves - 1) / kWaves;
  const int c0 = min(nchunks, wave * cpw), c1 = min(nchunks, c0 + cpw);
  const bool resident = span <= lds_floats;        // uniform over the workgroup

  if (resident) {
    constexpr int kFill = 8;
    for (int base = 0; base < span; base += kT * 4 * kFill) {
      float4 v[kFill];
#pragma unroll
      for (int j = 0; j < kFill; ++j) {
        const int q = base + (j * kT + tid) * 4;
        v[j] = q < span ? load_scores4(al, q, mis, span) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int j = 0; j < kFill; ++j) {
        const int q = base + (j * kT + tid) * 4;
        if (q < span) *reinterpret_cast<float4*>(lds + q) = v[j];
      }
    }
    __syncthreads();
  }
  auto load_chunk = [&](int c) -> float4 {
    const int q = c * 256 + lane * 4;
    if (c >= c1 || q >= span) return make_float4(0.f, 0.f, 0.f, 0.f);
    return resident ? *reinterpret_cast<const float4*>(lds + q) : load_scores4(al, q, mis, span);
  };
  // f(c, v): once per chunk c of this wavefront's run with the lane's vector v (uniform per wavefront)
  auto for_each_chunk = [&](auto f) {
    for (int c = c0; c < c1; c += kChunkBatch) {
      float4 v[kChunkBatch];
#pragma unroll
      for (int j = 0; j < kChunkBatch; ++j) v[j] = load_chunk(c + j);
#pragma unroll
      for (int j = 0; j < kChunkBatch; ++j)
        if (c + j < c1) f(c + j, v[j]);
    }
  };

  Pred pred{0.0, (double)threshold, min_keep};
  uint32_t prefix = 0;                             // decided high bits of the cut key
  int64_t cnt_above = 0;
  uint64_t mass_above = 0;
  const int shifts[3] = {21, 10, 0};
  const int widths[3] = {11, 11, 10};
  int done_bits = 0;
  uint32_t cut_cnt = 0;
  uint64_t cut_mass = 0;
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = shifts[pass], width = widths[pass];
    const int nb = 1 << width;
    for (int d = tid; d < kBuckets; d += kT) {
      sh.cnt[d] = 0;
      sh.mass[d] = 0;
    }
    if (tid == 0) sh.i[1] = 0;
    __syncthreads();
    for_each_chunk([&](int c, const float4& v) {
      const float f[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = c * 256 + lane * 4 + e - mis;
        const uint32_t key = order_key(f[e]);
        if (i >= 0 && i < n && (done_bits == 0 || (key >> (32 - done_bits)) == prefix)) {
          const uint32_t d = (key >> shift) & (nb - 1);
          atomicAdd(&sh.cnt[d], 1u);
          atomicAdd(reinterpret_cast<unsigned long long*>(&sh.mass[d]), (unsigned long long)quantise(f[e], inv));
        }
      }
    });
    __syncthreads();
    // suffix sums over buckets in descending digit order: thread t owns digits nb-1-2t, nb-2-2t
    const int d_hi = nb - 1 - 2 * tid, d_lo = d_hi - 1;
    const uint32_t c_hi = d_hi >= 0 ? sh.cnt[d_hi] : 0, c_lo = d_lo >= 0 ? sh.cnt[d_lo] : 0;
    const uint64_t m_hi = d_hi >= 0 ? sh.mass[d_hi] : 0, m_lo = d_lo >= 0 ? sh.mass[d_lo] : 0;
    uint64_t tot_c, tot_m, ex_c = (uint64_t)c_hi + c_lo, ex_m = m_hi + m_lo;
    block_exclusive_scan2(ex_c, ex_m, sh.scan, &tot_c, &tot_m);
    if (pass == 0) {
      // the first histogram holds every position: its mass is P_n exactly
      pred.set_total((double)tot_m);
      if (!pred(n, tot_m)) {                       // min_keep >= n (or no mass): keep everything
        if (idx_pad)
          for (int i = tid; i < n; i += kT) idx_pad[i] = i;
        return n;
      }
    }
    // crossing bucket: predicate false before it, true once it is included
    if (d_hi >= 0) {
      const int64_t n0 = cnt_above + (int64_t)ex_c;
      const uint64_t m0 = mass_above + ex_m;
      const bool p0 = pred(n0, m0);
      const bool p1 = pred(n0 + c_hi, m0 + m_hi);
      if (!p0 && p1 && c_hi > 0) {
        sh.i[1] = d_hi;
        sh.u64[0] = (uint64_t)n0;
        sh.u64[1] = m0;
      } else if (d_lo >= 0 && !p1) {
        const bool p2 = pred(n0 + c_hi + c_lo, m0 + m_hi + m_lo);
        if (p2 && c_lo > 0) {
          sh.i[1] = d_lo;
          sh.u64[0] = (uint64_t)(n0 + c_hi);
          sh.u64[1] = m0 + m_hi;
        }
      }
    }
    __syncthreads();
    const int d_cut = sh.i[1];
    cnt_above = (int64_t)sh.u64[0];
    mass_above = sh.u64[1];
    cut_cnt = sh.cnt[d_cut];
    cut_mass = sh.mass[d_cut];
    prefix = (prefix << width) | (uint32_t)d_cut;
    done_bits += width;
    __syncthreads();
  }
  // all cut_cnt elements of the final bucket share one value: take the fewest that cross
  const uint64_t q_each = cut_mass / (cut_cnt ? cut_cnt : 1u);
  if (tid == 0) {
    int lo = 1, hi = (int)cut_cnt;                 // pred is true at hi
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (pred(cnt_above + mid, mass_above + (uint64_t)mid * q_each)) hi = mid;
      else lo = mid + 1;
    }
    sh.i[2] = lo;
  }
  __syncthreads();
  const uint32_t ties = (uint32_t)sh.i[2];
  const int kept = (int)cnt_above + (int)ties;
  if (!idx_pad) return kept;

  // Emit the retained positions in ascending order: every wavefront counts what its run of chunks
  // retains, the counts of the wavefronts before it give its starting offset, then it writes
  // chunk by chunk with a prefix over lanes.  Of the positions tying the cut score the lowest
  // `ties` are kept.  Bit e of gt / eq: the lane's e-th position is above / at the cut key.
  auto classify = [&](int c, const float4& v, uint32_t& gt, uint32_t& eq) {
    const float f[4] = {v.x, v.y, v.z, v.w};
    gt = eq = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = c * 256 + lane * 4 + e - mis;
      const bool valid = i >= 0 && i < n;
      const uint32_t key = order_key(f[e]);
      gt |= (uint32_t)(valid && key > prefix) << e;
      eq |= (uint32_t)(valid && key == prefix) << e;
    }
  };
  uint32_t n_gt = 0, n_eq = 0;
  for_each_chunk([&](int c, const float4& v) {
    uint32_t gt, eq;
    classify(c, v, gt, eq);
    n_gt += __popc(gt);
    n_eq += __popc(eq);
  });
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    n_gt += __shfl_xor(n_gt, d);
    n_eq += __shfl_xor(n_eq, d);
  }
  if (lane == 0) {
    sh.cnt[2 * wave] = n_gt;
    sh.cnt[2 * wave + 1] = n_eq;
  }
  __syncthreads();
  uint32_t g_run = 0, e_run = 0;
  for (int w = 0; w < wave; ++w) {
    g_run += sh.cnt[2 * w];
    e_run += sh.cnt[2 * w + 1];
  }
  for_each_chunk([&](int c, const float4& v) {
    uint32_t gt, eq;
    classify(c, v, gt, eq);
    const uint32_t packed = ((uint32_t)__popc(gt) << 16) | (uint32_t)__popc(eq);
    const uint32_t inc = wave_inclusive_scan(packed, lane);
    const uint32_t tot = __shfl(inc, 63);
    uint32_t g = g_run + ((inc - packed) >> 16), e = e_run + ((inc - packed) & 0xffffu);
    const int i0 = c * 256 + lane * 4 - mis;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (gt & (1u << k)) {
        idx_pad[g + min(e, ties)] = i0 + k;
        ++g;
      } else if (eq & (1u << k)) {
        if (e < ties) idx_pad[g + e] = i0 + k;
        ++e;
      }
    }
    g_run += tot >> 16;
    e_run += tot & 0xffffu;
  });
  return kept;
}

// Score ranking: one workgroup of 1024 threads per unit.
__global__ __launch_bounds__(kT) void select_kernel(SelectArgs a) {
  __shared__ uint64_t sh_scan[kWaves][2];
  __shared__ double sh_dbl[kWaves];
  __shared__ uint32_t sh_cnt[kBuckets];
  __shared__ uint64_t sh_mass[kBuckets];
  extern __shared__ __attribute__((aligned(16))) float sh_scores[];        // a unit's scores
  __shared__ int sh_i[8];
  __shared__ uint64_t sh_u64[2];

  const int unit = blockIdx.x;
  const int b = unit / a.n_kv_heads, h = unit - b * a.n_kv_heads;
  int tile_base = 0;
  for (int bb = 0; bb < b; ++bb) tile_base += (a.cu[bb + 1] - a.cu[bb] + kTileKeys - 1) / kTileKeys;
  const int s0 = a.cu[b];
  const int n = a.cu[b + 1] - s0;
  const int tid = threadIdx.x;
  if (n == 0) {
    if (tid == 0) {
      a.kept[unit] = 0;
      a.desc[unit] = make_int4(0, 0, 0, 0);
    }
    return;
  }
  const float* s = a.scores + (int64_t)h * a.total_tokens + s0;
  const double* tiles = a.tile_sq + (int64_t)h * a.tiles_total + tile_base;
  const int nt = (n + kTileKeys - 1) / kTileKeys;
  int32_t* idx_pad = a.idx_pad ? a.idx_pad + ((int64_t)s0 * a.n_kv_heads + (int64_t)h * n) : nullptr;
  const bool keep_all = !(a.threshold > 0.f);              // T <= 0: no prefix short of everything qualifies

  int kept = n;
  double f2 = 0.0;
  if (!keep_all) {
    for (int j = tid; j < nt; j += kT) f2 += tiles[j];
    f2 = block_sum_double<kT>(f2, sh_dbl);
  }
  const bool degenerate = !(f2 > 0.0) || !(f2 < 1e300);
  if (degenerate || keep_all) {
    if (idx_pad)
      for (int i = tid; i < n; i += kT) idx_pad[i] = i;
  } else {
    // radix select of the cut value; masses are integers in units of F^2 / 2^60
    SelectShared sh{sh_scan, sh_cnt, sh_mass, sh_i, sh_u64};
    kept = score_rank(s, n, 1152921504606846976.0 / f2, a.threshold, a.min_keep, idx_pad, sh_scores, a.lds_floats, sh);
  }
  if (tid == 0) {
    a.kept[unit] = kept;
    a.desc[unit] = make_int4(kept, 0, 0, 0);
  }
}

// ---------------------------------------------------------------------------------------------
// Score ranking of long units, a unit split over several workgroups.
//
// select_score_hist_kernel, grid (slices, units): every workgroup forms the histogram of the first
// radix digit (count and integer mass per bucket) over its slice of the unit in LDS and adds its
// non-empty buckets to the unit's histogram in the workspace (integer atomics: exact, so the order
// of arrival does not matter).  The workgroup that arrives last finds the crossing bucket, collects
// the unit's positions in that bucket (usually a small part of the unit) into LDS and finishes
// the two remaining digits and the tie count on them alone; it leaves the cut (key, ties, kept count).
// select_score_emit_kernel, grid (slices, units): every workgroup counts the retained positions before
// its slice (above the cut key, and equal to it) and writes the retained positions of its slice in
// ascending order; of the positions that tie the cut key the lowest `ties` are kept.
// ---------------------------------------------------------------------------------------------

// positions [p0, p1) of slice `slice` of `slices`: whole 1024-position blocks, so that the emit
// kernel's chunks and the aligned 16-byte loads of both kernels coincide for every slice
__device__ __forceinline__ void slice_range(int n, int mis, int slice, int slices, int* q0, int* q1) {
  const int span = n + mis;                                 // floats from the aligned base
  const int blocks = (span + kT - 1) / kT;
  const int per = (blocks + slices - 1) / slices;
  *q0 = min(span, slice * per * kT);
  *q1 = min(span, (slice + 1) * per * kT);
}
// slices of a unit that hold positions (a short unit of a ragged batch fills only the first ones)
__device__ __forceinline__ int slices_used(int n, int mis, int slices) {
  const int blocks = (n + mis + kT - 1) / kT;
  const int per = (blocks + slices - 1) / slices;
  return (blocks + per - 1) / per;
}

__global__ __launch_bounds__(kT) void select_score_hist_kernel(SelectArgs a) {
  __shared__ uint64_t sh_scan[kWaves][2];
  __shared__ double sh_dbl[kWaves];
  __shared__ uint32_t sh_cnt[kBuckets];
  __shared__ uint64_t sh_mass[kBuckets];
  extern __shared__ __attribute__((aligned(16))) float sh_cand[];           // the crossing bucket's scores
  __shared__ int sh_i[8];
  __shared__ uint64_t sh_u64[3];
  __shared__ int sh_flag;

  const int unit = blockIdx.y, slice = blockIdx.x;
  const int b = unit / a.n_kv_heads, h = unit - b * a.n_kv_heads;
  int tile_base = 0;
  for (int bb = 0; bb < b; ++bb) tile_base += (a.cu[bb + 1] - a.cu[bb] + kTileKeys - 1) / kTileKeys;
  const int s0 = a.cu[b];
  const int n = a.cu[b + 1] - s0;
  const int tid = threadIdx.x;
  auto publish = [&](int kept, int ties, uint32_t key) {
    if (tid == 0) {
      a.kept[unit] = kept;
      a.desc[unit] = make_int4(kept, 0, ties, (int)key);
    }
  };
  if (n == 0) {
    if (slice == 0) publish(0, -1, 0u);
    return;
  }
  const float* s = a.scores + (int64_t)h * a.total_tokens + s0;
  const int mis = (int)((reinterpret_cast<uintptr_t>(s) >> 2) & 3);
  const float* al = s - mis;
  const int span = n + mis;
  const int slices = slices_used(n, mis, gridDim.x);
  if (slice >= slices) return;                             // nothing of the unit falls to this workgroup
  const double* tiles = a.tile_sq + (int64_t)h * a.tiles_total + tile_base;
  const int nt = (n + kTileKeys - 1) / kTileKeys;
  // F^2: every workgroup of the unit adds the tile sums in the same order and gets the same bits
  double f2 = 0.0;
  const bool keep_all = !(a.threshold > 0.f);
  if (!keep_all) {
    for (int j = tid; j < nt; j += kT) f2 += tiles[j];
    f2 = block_sum_double<kT>(f2, sh_dbl);
  }
  if (keep_all || !(f2 > 0.0) || !(f2 < 1e300)) {          // uniform over the unit's workgroups: keep everything
    if (slice == 0) publish(n, -1, 0u);                    // ties < 0: the emit kernel writes the identity
    return;
  }
  const double inv = 1152921504606846976.0 / f2;            // masses are integers in units of F^2 / 2^60

  // ---- first digit over this workgroup's slice
  for (int d = tid; d < kBuckets; d += kT) {
    sh_cnt[d] = 0;
    sh_mass[d] = 0;
  }
  __syncthreads();
  int q0, q1;
  slice_range(n, mis, slice, gridDim.x, &q0, &q1);
  for (int q = q0 + tid * 4; q < q1; q += kT * 4) {
    const float4 v = load_scores4(al, q, mis, span);
    const float f[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = q + e - mis;
      if (i >= 0 && i < n) {
        const uint32_t d = order_key(f[e]) >> 21;
        atomicAdd(&sh_cnt[d], 1u);
        atomicAdd(reinterpret_cast<unsigned long long*>(&sh_mass[d]), (unsigned long long)quantise(f[e], inv));
      }
    }
  }
  __syncthreads();
  uint32_t* g_cnt = a.sel_block + (int64_t)unit * kSelWords;
  unsigned long long* g_mass = reinterpret_cast<unsigned long long*>(g_cnt + kSelCntWords);
  int32_t* g_arrivals = reinterpret_cast<int32_t*>(g_cnt + kSelCntWords + kSelMassWords);
  if (slices > 1) {
    for (int d = tid; d < kBuckets; d += kT) {
      const uint32_t c = sh_cnt[d];
      if (c) {
        atomicAdd(&g_cnt[d], c);
        atomicAdd(&g_mass[d], (unsigned long long)sh_mass[d]);
      }
    }
    if (!last_arrival(g_arrivals, slices, &sh_flag)) return;
  }
  // ---- the last workgroup of the unit: the whole unit's first-digit histogram
  if (slices > 1) {
    for (int d = tid; d < kBuckets; d += kT) {
      sh_cnt[d] = __hip_atomic_load(&g_cnt[d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sh_mass[d] = __hip_atomic_load(&g_mass[d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
  }
  Pred pred{0.0, (double)a.threshold, a.min_keep};
  uint32_t prefix = 0;
  int64_t cnt_above = 0;
  uint64_t mass_above = 0;
  uint32_t cut_cnt = 0;
  uint64_t cut_mass = 0;
  int done_bits = 0;
  // crossing bucket of the histogram in sh_cnt / sh_mass (nb buckets of `width` bits); false: keep everything
  auto resolve = [&](int width, bool first) -> bool {
    const int nb = 1 << width;
    if (tid == 0) sh_i[1] = 0;
    __syncthreads();
    const int d_hi = nb - 1 - 2 * tid, d_lo = d_hi - 1;
    const uint32_t c_hi = d_hi >= 0 ? sh_cnt[d_hi] : 0, c_lo = d_lo >= 0 ? sh_cnt[d_lo] : 0;
    const uint64_t m_hi = d_hi >= 0 ? sh_mass[d_hi] : 0, m_lo = d_lo >= 0 ? sh_mass[d_lo] : 0;
    uint64_t tot_c, tot_m, ex_c = (uint64_t)c_hi + c_lo, ex_m = m_hi + m_lo;
    block_exclusive_scan2(ex_c, ex_m, sh_scan, &tot_c, &tot_m);
    if (first) {
      pred.set_total((double)tot_m);                       // the first histogram holds every position: P_n exactly
      if (!pred(n, tot_m)) return false;                   // min_keep >= n (or no mass)
    }
    if (d_hi >= 0) {
      const int64_t n0 = cnt_above + (int64_t)ex_c;
      const uint64_t m0 = mass_above + ex_m;
      const bool p0 = pred(n0, m0);
      const bool p1 = pred(n0 + c_hi, m0 + m_hi);
      if (!p0 && p1 && c_hi > 0) {
        sh_i[1] = d_hi;
        sh_u64[0] = (uint64_t)n0;
        sh_u64[1] = m0;
      } else if (d_lo >= 0 && !p1) {
        const bool p2 = pred(n0 + c_hi + c_lo, m0 + m_hi + m_lo);
        if (p2 && c_lo > 0) {
          sh_i[1] = d_lo;
          sh_u64[0] = (uint64_t)(n0 + c_hi);
          sh_u64[1] = m0 + m_hi;
        }
      }
    }
    __syncthreads();
    const int d_cut = sh_i[1];
    cnt_above = (int64_t)sh_u64[0];
    mass_above = sh_u64[1];
    cut_cnt = sh_cnt[d_cut];
    cut_mass = sh_mass[d_cut];
    prefix = (prefix << width) | (uint32_t)d_cut;
    done_bits += width;
    __syncthreads();
    return true;
  };
  if (!resolve(11, true)) {
    publish(n, -1, 0u);
    return;
  }
  // ---- the crossing bucket's scores: into LDS if they fit, else every later digit reads the unit again
  const bool resident = (int)cut_cnt <= a.lds_floats;
  if (tid == 0) sh_i[2] = 0;
  __syncthreads();
  if (resident) {
    // every thread looks at eight 4-vectors at a time; a wavefront reserves places for all its hits with
    // one LDS atomic (prefix over lanes), so a bucket that holds most of the unit costs no more than an
    // almost empty one
    constexpr int kBatch = 8;
    const int lane = tid & 63;
    auto collect = [&](const float4* v, int qb) {
      uint32_t hits = 0;                                   // bit 4 j + e: element e of vector j is in the bucket
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int q = qb + (j * kT + tid) * 4;
        const float f[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = q + e - mis;
          hits |= (uint32_t)(q < span && i >= 0 && i < n && (order_key(f[e]) >> 21) == prefix) << (4 * j + e);
        }
      }
      const int mine = __popc(hits);
      if (__ballot(mine > 0)) {
        const int inc = wave_inclusive_scan(mine, lane);
        int base = 0;
        if (lane == 63) base = atomicAdd(&sh_i[2], inc);
        base = __shfl(base, 63) + inc - mine;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
          const float f[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (hits & (1u << (4 * j + e))) sh_cand[base++] = f[e];
        }
      }
    };
    for (int qb = 0; qb < span; qb += kT * 4 * kBatch) {
      float4 v[kBatch];
      load_scores_batch<kBatch>(v, al, qb, mis, span);
      collect(v, qb);
    }
    __syncthreads();
  }
  const int ncand = resident ? (int)cut_cnt : 0;
  // f(score) for every position of the unit whose key starts with the digits decided so far
  auto for_each_candidate = [&](auto f) {
    if (resident) {
      for (int j = tid; j < ncand; j += kT) {
        const float x = sh_cand[j];
        if ((order_key(x) >> (32 - done_bits)) == prefix) f(x);
      }
    } else {
      for (int q = tid * 4; q < span; q += kT * 4) {
        const float4 v = load_scores4(al, q, mis, span);
        const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = q + e - mis;
          if (i >= 0 && i < n && (order_key(x[e]) >> (32 - done_bits)) == prefix) f(x[e]);
        }
      }
    }
  };
  if (resident && ncand <= kRankDirect) {
    // Few candidates (the cut often lies among the large scores, whose buckets are thin): every candidate
    // is ranked among the others directly, count and integer mass of the larger ones and the number of
    // equal ones, and the one score value at which the rule flips is the final bucket.  (All pairs: beyond
    // a hundred or so candidates the two digit passes below are cheaper.)
    uint32_t key_t = 0;
    uint64_t q_t = 0;
    if (tid < ncand) {
      const float x = sh_cand[tid];
      key_t = order_key(x);
      q_t = quantise(x, inv);
      sh_cnt[tid] = key_t;
      sh_mass[tid] = q_t;
    }
    __syncthreads();
    if (tid < ncand) {
      uint32_t c = 0, e = 0;
      uint64_t m = 0;
#pragma unroll 8
      for (int j = 0; j < ncand; ++j) {
        const uint32_t key_j = sh_cnt[j];
        const uint64_t q_j = sh_mass[j];
        c += key_j > key_t;
        m += key_j > key_t ? q_j : 0;
        e += key_j == key_t;
      }
      const int64_t n0 = cnt_above + c;
      const uint64_t m0 = mass_above + m;
      if (!pred(n0, m0) && pred(n0 + e, m0 + (uint64_t)e * q_t)) {   // the same values from every equal candidate
        sh_u64[0] = (uint64_t)n0;
        sh_u64[1] = m0;
        sh_u64[2] = q_t;
        sh_i[1] = (int)key_t;
        sh_i[3] = (int)e;
      }
    }
    __syncthreads();
    if (tid == 0) {
      const int64_t above = (int64_t)sh_u64[0];
      const uint64_t m_above = sh_u64[1], q_each = sh_u64[2];
      int lo = 1, hi = sh_i[3];                              // pred is true at hi
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (pred(above + mid, m_above + (uint64_t)mid * q_each)) hi = mid;
        else lo = mid + 1;
      }
      publish((int)above + lo, lo, (uint32_t)sh_i[1]);
    }
    return;
  }
  const int shifts[2] = {10, 0}, widths[2] = {11, 10};
  for (int lvl = 0; lvl < 2; ++lvl) {
    const int shift = shifts[lvl], nb = 1 << widths[lvl];
    for (int d = tid; d < kBuckets; d += kT) {
      sh_cnt[d] = 0;
      sh_mass[d] = 0;
    }
    __syncthreads();
    for_each_candidate([&](float x) {
      const uint32_t d = (order_key(x) >> shift) & (nb - 1);
      atomicAdd(&sh_cnt[d], 1u);
      atomicAdd(reinterpret_cast<unsigned long long*>(&sh_mass[d]), (unsigned long long)quantise(x, inv));
    });
    __syncthreads();
    resolve(widths[lvl], false);
  }
  // all cut_cnt positions of the final bucket share one value: take the fewest that cross
  const uint64_t q_each = cut_mass / (cut_cnt ? cut_cnt : 1u);
  if (tid == 0) {
    int lo = 1, hi = (int)cut_cnt;                         // pred is true at hi
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (pred(cnt_above + mid, mass_above + (uint64_t)mid * q_each)) hi = mid;
      else lo = mid + 1;
    }
    publish((int)cnt_above + lo, lo, prefix);
  }
}

__global__ __launch_bounds__(kT) void select_score_emit_kernel(SelectArgs a) {
  __shared__ uint32_t sh_w[kWaves][2];
  const int unit = blockIdx.y, slice = blockIdx.x, slices = gridDim.x;
  const int b = unit / a.n_kv_heads, h = unit - b * a.n_kv_heads;
  const int s0 = a.cu[b];
  const int n = a.cu[b + 1] - s0;
  if (n == 0 || !a.idx_pad) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* s = a.scores + (int64_t)h * a.total_tokens + s0;
  int32_t* idx_pad = a.idx_pad + ((int64_t)s0 * a.n_kv_heads + (int64_t)h * n);
  const int4 cut = a.desc[unit];
  const int ties = cut.z;
  const uint32_t key_cut = (uint32_t)cut.w;
  const int mis = (int)((reinterpret_cast<uintptr_t>(s) >> 2) & 3);
  const float* al = s - mis;
  int q0, q1;
  slice_range(n, mis, slice, slices, &q0, &q1);
  if (q0 >= q1) return;                                    // a short unit: nothing falls to this workgroup
  if (ties < 0) {                                          // everything is kept
    for (int q = q0 + tid; q < q1; q += kT)
      if (q >= mis) idx_pad[q - mis] = q - mis;
    return;
  }
  // retained positions before the slice: above the cut key, and equal to it
  uint32_t g_before = 0, e_before = 0;
  constexpr int kBatch = 8;
  for (int qb = 0; qb < q0; qb += kT * 4 * kBatch) {
    float4 v[kBatch];
    load_scores_batch<kBatch>(v, al, qb, mis, q0);         // q0 <= span; positions from q0 on read as 0 and are skipped
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int q = qb + (j * kT + tid) * 4;
      const float f[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool valid = q + e >= mis && q + e < q0;
        const uint32_t key = order_key(f[e]);
        g_before += valid && key > key_cut;
        e_before += valid && key == key_cut;
      }
    }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    g_before += __shfl_xor(g_before, d);
    e_before += __shfl_xor(e_before, d);
  }
  if (lane == 0) {
    sh_w[wave][0] = g_before;
    sh_w[wave][1] = e_before;
  }
  __syncthreads();
  uint32_t g_run = 0, e_run = 0;
  for (int w = 0; w < kWaves; ++w) {
    g_run += sh_w[w][0];
    e_run += sh_w[w][1];
  }
  // the slice, 1024 positions at a time in ascending order: thread t takes position q0 + c * 1024 + t
  for (int c0 = q0; c0 < q1; c0 += kT) {
    const int q = c0 + tid;
    const bool valid = q < q1 && q >= mis;
    const uint32_t key = valid ? order_key(al[q]) : 0u;
    const uint32_t gt = valid && key > key_cut, eq = valid && key == key_cut;
    const uint32_t packed = (gt << 16) | eq;
    const uint32_t inc = wave_inclusive_scan(packed, lane);
    __syncthreads();                                       // sh_w of the round before has been read
    if (lane == 63) sh_w[wave][0] = inc;
    __syncthreads();
    uint32_t before = 0, total = 0;
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t t = sh_w[w][0];
      if (w < wave) before += t;
      total += t;
    }
    const uint32_t ex = before + inc - packed;
    const uint32_t g = g_run + (ex >> 16), e = e_run + (ex & 0xffffu);
    if (gt) idx_pad[g + min(e, (uint32_t)ties)] = q - mis;
    else if (eq && e < (uint32_t)ties) idx_pad[g + e] = q - mis;
    g_run += total >> 16;
    e_run += total & 0xffffu;
  }
}

// Position ranking, one cut per unit (sequence, KV head) or, with a.per_layer, one cut per (layer,
// sequence): the norm of Eq. 1 then runs over the reduced attention matrix of all KV heads of the
// layer (Fig. 1: eviction "per layer"; Sec. 3.3: "the stopping positions of all layers") and every
// head keeps the same positions.  One workgroup per unit / per sequence.
__global__ __launch_bounds__(kPosThreads) void select_position_kernel(SelectArgs a) {
  __shared__ PositionShared<kPosThreads> sh;
  const int H = a.n_kv_heads;
  const int b = a.per_layer ? blockIdx.x : blockIdx.x / H;
  const int h = a.per_layer ? 0 : blockIdx.x - b * H;
  int tile_base = 0;
  for (int bb = 0; bb < b; ++bb) tile_base += (a.cu[bb + 1] - a.cu[bb] + kTileKeys - 1) / kTileKeys;
  const int s0 = a.cu[b];
  const int n = a.cu[b + 1] - s0;
  const int m_eff = min(max(a.n_sink, 0), n);
  const float* s = a.scores + (int64_t)h * a.total_tokens + s0;
  const double* tiles = a.tile_sq + (int64_t)h * a.tiles_total + tile_base;
  int kept = 0;
  if (n > 0) {
    if (a.per_layer)
      kept = position_cut<kPosThreads>(LayerMass{s, tiles, a.total_tokens, a.tiles_total, H}, n, m_eff, a.threshold,
                                       a.min_keep, &sh);
    else
      kept = position_cut<kPosThreads>(HeadMass{s, tiles}, n, m_eff, a.threshold, a.min_keep, &sh);
  }
  const int4 d = make_int4(kept, min(kept, m_eff), 0, 0);
  if (a.per_layer) {
    for (int hh = threadIdx.x; hh < H; hh += kPosThreads) {
      a.kept[b * H + hh] = kept;
      a.desc[b * H + hh] = d;
    }
  } else if (threadIdx.x == 0) {
    a.kept[blockIdx.x] = kept;
    a.desc[blockIdx.x] = d;
  }
}

// ---------------------------------------------------------------------------------------------
// One cut per (layer, sequence) with the score ranking (Fig. 1 "per layer", Sec. 3.3 "the stopping
// positions of all layers", with the ranking of Sec. 4.4): every head's row is ranked on its own and the
// matrix masked at rank i keeps the i largest scores of EVERY head, so the mass of a ranked prefix is
// sum_h (mass of head h's i largest).  That is a function of the rank, not of a score value shared by
// the heads, so each head's scores are sorted (bitonic network on their order-preserving keys: chunks
// of kSortChunk in LDS, the strides beyond a chunk in global memory), written back in ascending order,
// and the cut is then the position ranking's search with no sinks over the sorted rows (from the end
// backwards = descending score) with masses summed over the heads.  A head keeps its `kept` largest;
// of the scores that tie the kept-th largest, the lowest positions.
// ---------------------------------------------------------------------------------------------
constexpr int kSortChunk = 8192;                   // keys one workgroup sorts or merges in LDS (32 KB)

__device__ __forceinline__ int sort_size(int n) {    // next power of two >= n
  int p = 1;
  while (p < n) p <<= 1;
  return p;
}
__device__ __forceinline__ float key_to_score(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

struct SortUnit {
  int unit, h, s0, n, n2;
  uint32_t* keys;       // [n2] the unit's keys being sorted; pads (key 0) sort first
};
__device__ __forceinline__ SortUnit sort_unit(const SelectArgs& a, int unit) {
  SortUnit u;
  u.unit = unit;
  const int b = unit / a.n_kv_heads;
  u.h = unit - b * a.n_kv_heads;
  u.s0 = a.cu[b];
  u.n = a.cu[b + 1] - u.s0;
  u.n2 = sort_size(u.n);
  u.keys = a.sort_keys + 2 * ((int64_t)u.s0 * a.n_kv_heads + (int64_t)u.h * u.n);     // n2 <= 2 n
  return u;
}

// compare-exchange steps (size k, strides j_hi .. 1, each below kSortChunk) on one chunk in LDS
__device__ __forceinline__ void bitonic_lds_steps(uint32_t* sh, int chunk_base, int len, int k, int j_hi) {
  for (int j = j_hi; j > 0; j >>= 1) {
    __syncthreads();
    for (int t = threadIdx.x; t < len / 2; t += kT) {
      const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));          // the lower index of pair t
      const int l = i | j;
      const bool asc = ((chunk_base + i) & k) == 0;
      const uint32_t x = sh[i], y = sh[l];
      if ((x > y) == asc) {
        sh[i] = y;
        sh[l] = x;
      }
    }
  }
  __syncthreads();
}

// mode 0: load a chunk of keys from the scores (pads first), sort it completely (sizes 2 .. chunk);
// mode 1: for size k (> chunk), the strides below a chunk.  Grid (chunks, units).
__global__ __launch_bounds__(kT) void sort_lds_kernel(SelectArgs a, int mode, int k) {
  __shared__ uint32_t sh[kSortChunk];
  const SortUnit u = sort_unit(a, blockIdx.y);
  if (u.n == 0) return;
  const int len = min(u.n2, kSortChunk);
  const int base = blockIdx.x * kSortChunk;
  if (base >= u.n2 || (mode == 1 && k > u.n2)) return;
  if (mode == 0) {
    const float* s = a.scores + (int64_t)u.h * a.total_tokens + u.s0;
    const int pad = u.n2 - u.n;
    for (int i = threadIdx.x; i < len; i += kT) sh[i] = base + i < pad ? 0u : order_key(s[base + i - pad]);
    for (int kk = 2; kk <= len; kk <<= 1) bitonic_lds_steps(sh, base, len, kk, kk >> 1);
  } else {
    for (int i = threadIdx.x; i < len; i += kT) sh[i] = u.keys[base + i];
    bitonic_lds_steps(sh, base, len, k, len >> 1);
  }
  for (int i = threadIdx.x; i < len; i += kT) u.keys[base + i] = sh[i];
}

// one compare-exchange step (size k, stride j >= kSortChunk) in global memory.  Grid (pairs / kT, units).
__global__ __launch_bounds__(kT) void sort_global_kernel(SelectArgs a, int k, int j) {
  const SortUnit u = sort_unit(a, blockIdx.y);
  if (k > u.n2) return;
  const int t = blockIdx.x * kT + threadIdx.x;
  if (t >= u.n2 / 2) return;
  const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
  const int l = i | j;
  const bool asc = (i & k) == 0;
  const uint32_t x = u.keys[i], y = u.keys[l];
  if ((x > y) == asc) {
    u.keys[i] = y;
    u.keys[l] = x;
  }
}

// the sorted scores of every unit, ascending, in the layout of the scores.  Grid (n / kT, units).
__global__ __launch_bounds__(kT) void sort_store_kernel(SelectArgs a) {
  const SortUnit u = sort_unit(a, blockIdx.y);
  const int r = blockIdx.x * kT + threadIdx.x;
  if (r >= u.n) return;
  a.sorted_scores[(int64_t)u.h * a.total_tokens + u.s0 + r] = key_to_score(u.keys[u.n2 - u.n + r]);
}

// after the cut: every head's cut key (its kept-th largest score) and how many of the scores equal to
// it are kept.  One thread per unit: bisection of the ascending row.
__global__ __launch_bounds__(64) void layer_score_cut_keys_kernel(SelectArgs a) {
  const SortUnit u = sort_unit(a, blockIdx.x);
  if (threadIdx.x != 0) return;
  const int kept = a.kept[u.unit];
  if (u.n == 0 || kept >= u.n) {
    a.desc[u.unit] = make_int4(kept, 0, -1, 0);            // ties < 0: the emit kernel writes the identity
    return;
  }
  const uint32_t* row = u.keys + (u.n2 - u.n);
  const uint32_t key = row[u.n - kept];                    // kept >= 1
  int lo = u.n - kept, hi = u.n;                           // first index whose key is greater than the cut key
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (row[mid] > key) hi = mid;
    else lo = mid + 1;
  }
  a.desc[u.unit] = make_int4(kept, 0, kept - (u.n - lo), (int)key);
}

}  // namespace

hipError_t launch_select(const Geometry& g, const SelectArgs& a, hipStream_t stream) {
  if (g.units == 0) return hipSuccess;
  if (a.from_scores && g.max_seqlen > 0) {
    const int tiles = (g.max_seqlen + kTileKeys - 1) / kTileKeys;
    const int per_block = kBlockThreads / 64;
    hipLaunchKernelGGL(tile_sums_kernel, dim3((tiles + per_block - 1) / per_block, g.units), dim3(kBlockThreads), 0,
                       stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (a.per_layer && a.rank_mode == 1 && g.max_seqlen > 0) {
    // sort every head's scores, cut over the ranks with masses summed over the heads, then each head's keys
    int n2 = 1;
    while (n2 < g.max_seqlen) n2 <<= 1;
    const int chunks = (n2 + kSortChunk - 1) / kSortChunk;
    hipLaunchKernelGGL(sort_lds_kernel, dim3(chunks, g.units), dim3(kT), 0, stream, a, 0, 0);
    for (int k = 2 * kSortChunk; k <= n2; k <<= 1) {
      for (int j = k >> 1; j >= kSortChunk; j >>= 1)
        hipLaunchKernelGGL(sort_global_kernel, dim3((n2 / 2 + kT - 1) / kT, g.units), dim3(kT), 0, stream, a, k, j);
      hipLaunchKernelGGL(sort_lds_kernel, dim3(chunks, g.units), dim3(kT), 0, stream, a, 1, k);
    }
    hipLaunchKernelGGL(sort_store_kernel, dim3((g.max_seqlen + kT - 1) / kT, g.units), dim3(kT), 0, stream, a);
    SelectArgs cut = a;                            // the position search over the sorted rows: no sinks, ranks from the end
    cut.scores = a.sorted_scores;
    cut.n_sink = 0;
    cut.sel_block = nullptr;
    const int tiles = (g.max_seqlen + kTileKeys - 1) / kTileKeys;
    const int per_block = kBlockThreads / 64;
    hipLaunchKernelGGL(tile_sums_kernel, dim3((tiles + per_block - 1) / per_block, g.units), dim3(kBlockThreads), 0,
                       stream, cut);
    hipLaunchKernelGGL(select_position_kernel, dim3(g.batch), dim3(kPosThreads), 0, stream, cut);
    hipLaunchKernelGGL(layer_score_cut_keys_kernel, dim3(g.units), dim3(64), 0, stream, a);
    if (a.idx_pad) {
      const int slices = g.score_slices > 0 ? g.score_slices : 1;
      hipLaunchKernelGGL(select_score_emit_kernel, dim3(slices, g.units), dim3(kT), 0, stream, a);
    }
    return hipGetLastError();
  }
  if (a.rank_mode == 0) {                          // position ranking: one cut per unit, or per sequence over all heads
    hipLaunchKernelGGL(select_position_kernel, dim3(a.per_layer ? g.batch : g.units), dim3(kPosThreads), 0, stream, a);
    return hipGetLastError();
  }
  if (g.score_slices > 0) {
    // long units: a unit split over several workgroups, then the ordered emit
    SelectArgs args = a;
    const int slices = g.score_slices;
    args.lds_floats = kMaxCandidates;              // every workgroup reserves it, only a unit's last one uses it
    const size_t dyn = (size_t)args.lds_floats * sizeof(float);
    hipLaunchKernelGGL(select_score_hist_kernel, dim3(slices, g.units), dim3(kT), dyn, stream, args);
    if (a.idx_pad) hipLaunchKernelGGL(select_score_emit_kernel, dim3(slices, g.units), dim3(kT), 0, stream, args);
    return hipGetLastError();
  }
  // Short units: one workgroup per unit.  It keeps the unit's scores in LDS (with up to three floats of
  // alignment slack).
  SelectArgs args = a;
  args.lds_floats = 0;
  if (a.rank_mode == 1 && a.threshold > 0.f) {
    const int64_t want = ((int64_t)g.max_seqlen + 3 + 3) / 4 * 4;
    args.lds_floats = (int32_t)(want < kMaxLdsFloats ? want : kMaxLdsFloats);
  }
  const size_t dyn = (size_t)args.lds_floats * sizeof(float);
  if (dyn > 0) {
    const hipError_t e = allow_lds<&select_kernel>((size_t)kMaxLdsFloats * sizeof(float));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(select_kernel, dim3(g.units), dim3(kT), dyn, stream, args);
  return hipGetLastError();
}

}  // namespace rfkv
