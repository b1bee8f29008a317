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
#include "tile_sum.h"

namespace rfkv {
namespace {

constexpr int kT = kSelectThreads;
constexpr int kWaves = kT / 64;
constexpr int kBuckets = 2048;

struct Pred {
  double total;     // P_n as a double
  double T;
  int min_keep;
  // Q(i, P): has the ranked prefix of i elements and mass P reached the stopping condition?
  __device__ bool operator()(int64_t count, uint64_t mass) const {
    if (count <= 0 || count < min_keep) return false;      // a prefix has at least one element
    return 1.0 - sqrt((double)mass / total) < T;
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

// Exclusive scan over the 1024 threads (thread order); returns the exclusive prefix and the total.
template <typename V>
__device__ __forceinline__ V block_exclusive_scan(V v, V* wave_tot /*[kWaves+1] LDS*/, V* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const V inc = wave_inclusive_scan(v, lane);
  __syncthreads();
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    V run = 0;
    for (int w = 0; w < kWaves; ++w) {
      const V t = wave_tot[w];
      wave_tot[w] = run;
      run += t;
    }
    wave_tot[kWaves] = run;
  }
  __syncthreads();
  *total = wave_tot[kWaves];
  return wave_tot[wave] + inc - v;
}

__device__ __forceinline__ double block_sum_double(double v, double* wave_tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  __syncthreads();
  if (lane == 0) wave_tot[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < kWaves; ++w) t += wave_tot[w];      // same order in every thread
  return t;
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
  if (tile >= nt) return;                                  // uniform per wavefront
  const float* s = a.scores + (int64_t)h * a.total_tokens + s0;
  const int pos = tile * kTileKeys + lane;
  const float v = (lane < kTileKeys && pos < n) ? s[pos] : 0.f;
  const double t = tile_sum_sq(v, lane);
  if (lane == 0) a.tile_sq[(int64_t)h * a.tiles_total + tile_base + tile] = t;
}

// The stopping test 1 - sqrt(P / F^2) < T on fp64 masses.  Away from the boundary the cheap
// squared form P > (1 - T)^2 F^2 decides; only within 1e-9 relative of it is the paper's form
// (an fp64 divide and square root) evaluated, so sequential walks stay short.
struct PredF {
  double total;     // F^2
  double T;
  int min_keep;
  double lo, hi;    // (1 - T)^2 F^2 shrunk / grown by 1e-9: below lo certainly false, above hi certainly true
  __device__ PredF(double f2, double t, int mk) : total(f2), T(t), min_keep(mk) {
    const double thr = t < 1.0 ? (1.0 - t) * (1.0 - t) * f2 : -1.0;     // T >= 1: any positive mass qualifies
    lo = thr * (1.0 - 1e-9);
    hi = thr * (1.0 + 1e-9);
    if (t >= 1.0) { lo = -1.0; hi = -2.0; }                             // always take the exact path
  }
  __device__ bool operator()(int64_t count, double mass) const {
    if (count <= 0 || count < min_keep) return false;
    if (hi >= lo) {
      if (mass > hi) return true;
      if (mass < lo) return false;
    }
    return 1.0 - sqrt(mass / total) < T;
  }
};

__global__ __launch_bounds__(kT) void select_kernel(SelectArgs a) {
  __shared__ uint64_t sh_scan[kWaves + 1];
  __shared__ double sh_dbl[kWaves];
  __shared__ double sh_incl[kT];
  __shared__ uint32_t sh_cnt[kBuckets];
  __shared__ uint64_t sh_mass[kBuckets];
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
  const int m_eff = min(max(a.n_sink, 0), n);
  const bool by_score = a.rank_mode == 1;
  const bool keep_all = !(a.threshold > 0.f);              // T <= 0: no prefix short of everything qualifies

  int kept = n;
  bool degenerate = false;
  double f2 = 0.0;

  if (!by_score && !keep_all) {
    // ---------------- position ranking: first the sinks [0, m), then the rest from the end backwards.
    // Sink mass directly; tail mass per 32-position tile (from the scoring kernel), reversed.
    double sink = 0.0;
    if (m_eff <= 32) {                                     // the usual case (m = 4): every thread sums them itself
      for (int p = 0; p < m_eff; ++p) sink += (double)s[p] * (double)s[p];
    } else {
      for (int p = tid; p < m_eff; p += kT) sink += (double)s[p] * (double)s[p];
      sink = block_sum_double(sink, sh_dbl);
    }
    const int jm = m_eff / kTileKeys;                      // first tile holding a tail position
    const int ntail = m_eff < n ? nt - jm : 0;
    const int C = (ntail + kT - 1) / kT;                   // tail tiles per thread, in rank order
    const int k0 = min(ntail, tid * C), k1 = min(ntail, k0 + C);
    auto tile_mass = [&](int j) -> double {                // tail mass of tile j
      if (j > jm || m_eff % kTileKeys == 0) return tiles[j];
      double v = 0.0;                                      // the tile shared with the sinks
      for (int p = min(n, (j + 1) * kTileKeys) - 1; p >= m_eff; --p) v += (double)s[p] * (double)s[p];
      return v;
    };
    double mine = 0.0;
    for (int k = k0; k < k1; ++k) mine += tile_mass(nt - 1 - k);
    // inclusive scan over threads, fixed order
    const int lane = tid & 63, wave = tid >> 6;
    double inc = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const double o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    __syncthreads();
    if (lane == 63) sh_dbl[wave] = inc;
    __syncthreads();
    double wave_off = 0.0;
    for (int w = 0; w < wave; ++w) wave_off += sh_dbl[w];
    double tail_total = 0.0;
    for (int w = 0; w < kWaves; ++w) tail_total += sh_dbl[w];
    inc += wave_off;
    sh_incl[tid] = inc;
    f2 = sink + tail_total;
    degenerate = !(f2 > 0.0) || !(f2 < 1e300);
    if (tid == 0) {
      sh_i[0] = n;          // result: no crossing keeps everything
      sh_i[3] = kT;         // first thread whose chunk end satisfies the rule
    }
    __syncthreads();
    if (!degenerate) {
      const PredF pred(f2, (double)a.threshold, a.min_keep);
      // ranks covered up to and including tail-rank tile k: sinks + positions from the end down to tile start
      auto count_through = [&](int k) -> int { return m_eff + n - max((nt - 1 - k) * kTileKeys, m_eff); };
      // Search one run of consecutive ranks with a wavefront: lane l takes the l-th rank of the
      // run (position first + l * step), an inclusive fp64 prefix over lanes gives the mass through
      // each rank, and the first lane whose prefix satisfies the rule is the cut.
      auto wave_search = [&](int first, int step, int len, int ranks_before, double mass_before, int fallback) {
        const int p = first + lane * step;
        double v = 0.0;
        if (lane < len) v = (double)s[p] * (double)s[p];
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const double o = __shfl_up(v, d);
          if (lane >= d) v += o;
        }
        const bool ok = lane < len && pred(ranks_before + lane + 1, mass_before + v);
        const unsigned long long mask = __ballot(ok);
        if (lane == 0) sh_i[0] = mask ? ranks_before + __ffsll((long long)mask) : fallback;
      };
      if (pred(m_eff, sink)) {
        // the cut falls inside the sinks
        if (m_eff <= 64) {
          if (wave == 0) wave_search(0, 1, m_eff, 0, 0.0, m_eff);
        } else if (tid == 0) {
          double run = 0.0;
          int res = m_eff;
          for (int p = 0; p < m_eff; ++p) {
            run += (double)s[p] * (double)s[p];
            if (pred(p + 1, run)) {
              res = p + 1;
              break;
            }
          }
          sh_i[0] = res;
        }
      } else {
        if (k1 > k0 && pred(count_through(k1 - 1), sink + inc)) atomicMin(&sh_i[3], tid);
        __syncthreads();
        if (sh_i[3] == tid) {
          // the tile of this thread's chunk in which the rule is first met (the last one if rounding hides it)
          double run = sink + (tid > 0 ? sh_incl[tid - 1] : 0.0);
          int jstar = nt - k1;
          for (int k = k0; k + 1 < k1; ++k) {
            const double tm = tile_mass(nt - 1 - k);
            if (pred(count_through(k), run + tm)) {
              jstar = nt - 1 - k;
              break;
            }
            run += tm;
          }
          sh_i[4] = jstar;
          sh_dbl[0] = run;
        }
        __syncthreads();
        if (sh_i[3] < kT && wave == 0) {
          const int jt = sh_i[4];
          const int hi_p = min(n, (jt + 1) * kTileKeys) - 1, lo_p = max(jt * kTileKeys, m_eff);
          wave_search(hi_p, -1, hi_p - lo_p + 1, m_eff + (n - 1 - hi_p), sh_dbl[0], m_eff + (n - lo_p));
        }
      }
    }
    __syncthreads();
    kept = degenerate ? n : sh_i[0];
  } else if (by_score && !keep_all) {
    for (int j = tid; j < nt; j += kT) f2 += tiles[j];
    f2 = block_sum_double(f2, sh_dbl);
    degenerate = !(f2 > 0.0) || !(f2 < 1e300);
  }
  const double inv = (degenerate || keep_all || !by_score) ? 0.0 : 1152921504606846976.0 / f2;      // 2^60 / F^2

  if (by_score && (degenerate || keep_all)) {
    if (idx_pad)
      for (int i = tid; i < n; i += kT) idx_pad[i] = i;
  } else if (by_score) {
    // ---------------- score ranking: radix select of the cut value
    uint64_t mine = 0;
    for (int i = tid; i < n; i += kT) mine += quantise(s[i], inv);
    uint64_t total;
    block_exclusive_scan<uint64_t>(mine, sh_scan, &total);
    const Pred pred{(double)total, (double)a.threshold, a.min_keep};
    if (!pred(n, total)) {
      kept = n;                                    // T <= 0 (or min_keep >= n): keep everything
      if (idx_pad)
        for (int i = tid; i < n; i += kT) idx_pad[i] = i;
    } else {
      uint32_t prefix = 0;                         // decided high bits of the cut key
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
          sh_cnt[d] = 0;
          sh_mass[d] = 0;
        }
        if (tid == 0) sh_i[1] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += kT) {
          const float v = s[i];
          const uint32_t key = order_key(v);
          if (done_bits == 0 || (key >> (32 - done_bits)) == prefix) {
            const uint32_t d = (key >> shift) & (nb - 1);
            atomicAdd(&sh_cnt[d], 1u);
            atomicAdd(reinterpret_cast<unsigned long long*>(&sh_mass[d]), (unsigned long long)quantise(v, inv));
          }
        }
        __syncthreads();
        // suffix sums over buckets in descending digit order: thread t owns digits nb-1-2t, nb-2-2t
        const int d_hi = nb - 1 - 2 * tid, d_lo = d_hi - 1;
        const uint32_t c_hi = d_hi >= 0 ? sh_cnt[d_hi] : 0, c_lo = d_lo >= 0 ? sh_cnt[d_lo] : 0;
        const uint64_t m_hi = d_hi >= 0 ? sh_mass[d_hi] : 0, m_lo = d_lo >= 0 ? sh_mass[d_lo] : 0;
        uint64_t tot_c, tot_m;
        const uint64_t ex_c = block_exclusive_scan<uint64_t>((uint64_t)c_hi + c_lo, sh_scan, &tot_c);
        const uint64_t ex_m = block_exclusive_scan<uint64_t>(m_hi + m_lo, sh_scan, &tot_m);
        // crossing bucket: predicate false before it, true once it is included
        if (d_hi >= 0) {
          const int64_t c0 = cnt_above + (int64_t)ex_c;
          const uint64_t m0 = mass_above + ex_m;
          const bool p0 = pred(c0, m0);
          const bool p1 = pred(c0 + c_hi, m0 + m_hi);
          if (!p0 && p1 && c_hi > 0) {
            sh_i[1] = d_hi;
            sh_u64[0] = (uint64_t)c0;
            sh_u64[1] = m0;
          } else if (d_lo >= 0 && !p1) {
            const bool p2 = pred(c0 + c_hi + c_lo, m0 + m_hi + m_lo);
            if (p2 && c_lo > 0) {
              sh_i[1] = d_lo;
              sh_u64[0] = (uint64_t)(c0 + c_hi);
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
      }
      // all cut_cnt elements of the final bucket share one value: take the fewest that cross
      const uint64_t q_each = cut_mass / (cut_cnt ? cut_cnt : 1u);
      if (tid == 0) {
        int lo = 1, hi = (int)cut_cnt;             // pred is true at hi
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (pred(cnt_above + mid, mass_above + (uint64_t)mid * q_each)) hi = mid;
          else lo = mid + 1;
        }
        sh_i[2] = lo;
      }
      __syncthreads();
      const int ties = sh_i[2];
      kept = (int)cnt_above + ties;

      // emit retained positions in ascending order
      if (idx_pad) {
        constexpr int kItems = 8;
        uint32_t carry_gt = 0, carry_eq = 0;
        for (int base = 0; base < n; base += kT * kItems) {
          const int p0 = base + tid * kItems;
          uint32_t gt = 0, eq = 0;
          uint32_t keys[kItems];
#pragma unroll
          for (int j = 0; j < kItems; ++j) {
            const int p = p0 + j;
            keys[j] = p < n ? order_key(s[p]) : 0u;
            gt += (p < n && keys[j] > prefix);
            eq += (p < n && keys[j] == prefix);
          }
          uint64_t tot;
          const uint64_t ex = block_exclusive_scan<uint64_t>(((uint64_t)gt << 32) | eq, sh_scan, &tot);
          uint32_t g_run = carry_gt + (uint32_t)(ex >> 32), e_run = carry_eq + (uint32_t)ex;
#pragma unroll
          for (int j = 0; j < kItems; ++j) {
            const int p = p0 + j;
            if (p < n) {
              if (keys[j] > prefix) {
                idx_pad[g_run + min(e_run, (uint32_t)ties)] = p;
                ++g_run;
              } else if (keys[j] == prefix) {
                if (e_run < (uint32_t)ties) idx_pad[g_run + e_run] = p;
                ++e_run;
              }
            }
          }
          carry_gt += (uint32_t)(tot >> 32);
          carry_eq += (uint32_t)tot;
        }
      }
    }
  }

  if (tid == 0) {
    a.kept[unit] = kept;
    a.desc[unit] = make_int4(kept, by_score ? 0 : min(kept, m_eff), 0, 0);
  }
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
  hipLaunchKernelGGL(select_kernel, dim3(g.units), dim3(kT), 0, stream, a);
  return hipGetLastError();
}

}  // namespace rfkv
