// Position ranking + Uni-Metric budget rule (Sec. 3.2 "Initial Ranking", Eq. 1; Sec. 3.3, Eq. 3)
// as one device function, shared by the selection kernels (one cut per unit, one cut per layer and
// sequence) and by the scoring pass, whose last workgroup of a unit takes the cut itself.
//
// Ranking: the first m positions, then the rest from the end backwards.  The squared-score mass of a
// ranked prefix is the sinks' mass plus a suffix of the sequence; suffix masses come from per-tile
// sums (32 positions, written by the scoring pass in a fixed order), added up in rank order in
// fp64 with a fixed tree, so two runs give the same bits.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tile_sum.h"

namespace rfkv {

// ---- Words that workgroups of one launch hand to each other (per-span statistics, tile sums,
// scores the cut looks at, kept counts).  Device-scope atomic loads and stores go to the point of
// coherence between the XCDs' L2 caches, so a hand-over needs no cache write-back or invalidate:
// the writer waits until its stores are acknowledged (stores_acknowledged), then bumps a counter;
// the workgroup that sees the last count reads with coherent loads.
__device__ __forceinline__ void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(int32_t* p, int32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t coherent_load(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(double* p, double v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double coherent_load(const double* p) {
  return __builtin_bit_cast(double, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void coherent_store(float2* p, float2 v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 coherent_load(const float2* p) {
  return __builtin_bit_cast(float2, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p),
                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Counts one arrival at `counter` (which starts at zero) and tells the whole workgroup whether it
// was the last of `expected`.  Every thread's stores have been acknowledged before the count, so
// the last arriver may read, with coherent loads, what all the others wrote.  The last arriver puts
// the counter back to zero: the same word serves the next launch.  `flag` is one int of LDS.
__device__ __forceinline__ bool last_arrival(int32_t* counter, int expected, int* flag) {
  stores_acknowledged();
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = old == expected - 1;
    if (last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag = last ? 1 : 0;
  }
  __syncthreads();
  return *flag != 0;
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

// LDS the search needs, for a workgroup of kThreads threads.
template <int kThreads>
struct PositionShared {
  double dbl[kThreads / 64];
  double incl[kThreads];
  int i[8];
};

template <int kThreads>
__device__ __forceinline__ double block_sum_double(double v, double* wave_tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  __syncthreads();
  if (lane == 0) wave_tot[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < kThreads / 64; ++w) t += wave_tot[w];      // same order in every thread
  return t;
}

// Masses of one unit: squared score of a position, squared-score sum of a 32-position tile.
struct HeadMass {
  const float* s;          // the unit's scores
  const double* tiles;     // its tile sums
  __device__ double pos(int p) const {
    const double x = (double)coherent_load(s + p);
    return x * x;
  }
  __device__ double tile(int j) const { return coherent_load(tiles + j); }
};

// Masses of a sequence over all KV heads (one cut per layer and sequence): heads added in index order.
struct LayerMass {
  const float* s;          // head h: s + h * total_tokens
  const double* tiles;     // head h: tiles + h * tiles_total
  int64_t total_tokens, tiles_total;
  int heads;
  // Eight heads' loads are issued together and without a branch between them (a load behind a branch is
  // waited for on the spot: a trip to memory per head), a head past the last reads the last head's word
  // and counts as zero; then they are added in index order.
  __device__ double pos(int p) const {
    double v = 0.0;
    for (int h0 = 0; h0 < heads; h0 += 8) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = coherent_load(s + (int64_t)min(h0 + j, heads - 1) * total_tokens + p);
#pragma unroll
      for (int j = 0; j < 8; ++j) v += h0 + j < heads ? (double)x[j] * (double)x[j] : 0.0;
    }
    return v;
  }
  __device__ double tile(int j) const {
    double v = 0.0;
    for (int h0 = 0; h0 < heads; h0 += 8) {
      double x[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) x[i] = coherent_load(tiles + (int64_t)min(h0 + i, heads - 1) * tiles_total + j);
#pragma unroll
      for (int i = 0; i < 8; ++i) v += h0 + i < heads ? x[i] : 0.0;
    }
    return v;
  }
};

// Kept count of the position ranking for n > 0 positions with m_eff = min(m, n) sinks, by all
// kThreads threads of the workgroup (every thread returns the same value).  T <= 0 keeps everything.
template <int kThreads, typename Mass>
__device__ __forceinline__ int position_cut(const Mass& mass, int n, int m_eff, float threshold, int min_keep,
                                            PositionShared<kThreads>* sh) {
  constexpr int kWaves = kThreads / 64;
  if (!(threshold > 0.f)) return n;                        // no prefix short of everything qualifies
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nt = (n + kTileKeys - 1) / kTileKeys;
  // Sink mass directly; tail mass per 32-position tile (from the scoring kernel), reversed.
  double sink = 0.0;
  if (m_eff <= 32) {                                       // the usual case (m = 4): every thread sums them itself
    for (int p0 = 0; p0 < m_eff; p0 += 4) {                // four positions' loads in flight, added in order
      double x[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) x[j] = mass.pos(min(p0 + j, m_eff - 1));
#pragma unroll
      for (int j = 0; j < 4; ++j) sink += p0 + j < m_eff ? x[j] : 0.0;
    }
  } else {
    for (int p = tid; p < m_eff; p += kThreads) sink += mass.pos(p);
    sink = block_sum_double<kThreads>(sink, sh->dbl);
    __syncthreads();
  }
  const int jm = m_eff / kTileKeys;                        // first tile holding a tail position
  const int ntail = m_eff < n ? nt - jm : 0;
  const int C = (ntail + kThreads - 1) / kThreads;         // tail tiles per thread, in rank order
  const int k0 = min(ntail, tid * C), k1 = min(ntail, k0 + C);
  auto tile_mass = [&](int j) -> double {                  // tail mass of tile j
    if (j > jm || m_eff % kTileKeys == 0) return mass.tile(j);
    double v = 0.0;                                        // the tile shared with the sinks
    for (int p = min(n, (j + 1) * kTileKeys) - 1; p >= m_eff; --p) v += mass.pos(p);
    return v;
  };
  // Tail masses of the tiles of ranks k .. k + 7 of this thread's chunk: eight loads in flight with no branch
  // between them (ranks past the chunk read a tile of the chunk and count as zero); the one tile of the unit
  // that the sinks share is put right afterwards.
  auto tile_masses = [&](double* v, int k) {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = mass.tile(nt - 1 - min(k + j, max(k1 - 1, 0)));
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int jt = nt - 1 - (k + j);
      if (k + j >= k1) v[j] = 0.0;
      else if (jt == jm && m_eff % kTileKeys != 0) v[j] = tile_mass(jt);
    }
  };
  double mine = 0.0;
  double head[8];                                          // the chunk's first eight tile masses, kept for the walk below
#pragma unroll
  for (int j = 0; j < 8; ++j) head[j] = 0.0;
  if (k0 < k1) tile_masses(head, k0);
#pragma unroll
  for (int j = 0; j < 8; ++j) mine += head[j];
  for (int k = k0 + 8; k < k1; k += 8) {                   // added in rank order
    double v[8];
    tile_masses(v, k);
#pragma unroll
    for (int j = 0; j < 8; ++j) mine += v[j];
  }
  // inclusive scan over threads, fixed order
  double inc = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const double o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  __syncthreads();
  if (lane == 63) sh->dbl[wave] = inc;
  __syncthreads();
  double wave_off = 0.0, tail_total = 0.0;
  for (int w = 0; w < kWaves; ++w) {
    if (w < wave) wave_off += sh->dbl[w];
    tail_total += sh->dbl[w];
  }
  inc += wave_off;
  sh->incl[tid] = inc;
  const double f2 = sink + tail_total;
  const bool degenerate = !(f2 > 0.0) || !(f2 < 1e300);
  if (tid == 0) {
    sh->i[0] = n;           // result: no crossing keeps everything
    sh->i[3] = kThreads;    // first thread whose chunk end satisfies the rule
  }
  __syncthreads();
  if (!degenerate) {
    const PredF pred(f2, (double)threshold, min_keep);
    // ranks covered up to and including tail-rank tile k: sinks + positions from the end down to tile start
    auto count_through = [&](int k) -> int { return m_eff + n - max((nt - 1 - k) * kTileKeys, m_eff); };
    // Search one run of consecutive ranks with a wavefront: lane l takes the l-th rank of the
    // run (position first + l * step), an inclusive fp64 prefix over lanes gives the mass through
    // each rank, and the first lane whose prefix satisfies the rule is the cut.
    auto wave_search = [&](int first, int step, int len, int ranks_before, double mass_before, int fallback) {
      const int p = first + lane * step;
      double v = lane < len ? mass.pos(p) : 0.0;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const double o = __shfl_up(v, d);
        if (lane >= d) v += o;
      }
      const bool ok = lane < len && pred(ranks_before + lane + 1, mass_before + v);
      const unsigned long long mask = __ballot(ok);
      if (lane == 0) sh->i[0] = mask ? ranks_before + __ffsll((long long)mask) : fallback;
    };
    if (pred(m_eff, sink)) {
      // the cut falls inside the sinks
      if (m_eff <= 64) {
        if (wave == 0) wave_search(0, 1, m_eff, 0, 0.0, m_eff);
      } else if (tid == 0) {
        double run = 0.0;
        int res = m_eff;
        for (int p = 0; p < m_eff; ++p) {
          run += mass.pos(p);
          if (pred(p + 1, run)) {
            res = p + 1;
            break;
          }
        }
        sh->i[0] = res;
      }
    } else {
      if (k1 > k0 && pred(count_through(k1 - 1), sink + inc)) atomicMin(&sh->i[3], tid);
      __syncthreads();
      if (sh->i[3] == tid) {
        // the tile of this thread's chunk in which the rule is first met (the last one if rounding hides it)
        // (the first eight masses are still in registers: up to 8 * kThreads tiles, 65536 positions at 256
        // threads, the walk costs no further trip to memory)
        double run = sink + (tid > 0 ? sh->incl[tid - 1] : 0.0);
        int jstar = nt - k1;
        bool found = false;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int k = k0 + j;
          if (!found && k + 1 < k1) {
            if (pred(count_through(k), run + head[j])) {
              jstar = nt - 1 - k;
              found = true;
            } else {
              run += head[j];
            }
          }
        }
        for (int k = k0 + 8; !found && k + 1 < k1; ++k) {
          const double tm = tile_mass(nt - 1 - k);
          if (pred(count_through(k), run + tm)) {
            jstar = nt - 1 - k;
            found = true;
          } else {
            run += tm;
          }
        }
        sh->i[4] = jstar;
        sh->dbl[0] = run;
      }
      __syncthreads();
      if (sh->i[3] < kThreads && wave == 0) {
        const int jt = sh->i[4];
        const int hi_p = min(n, (jt + 1) * kTileKeys) - 1, lo_p = max(jt * kTileKeys, m_eff);
        wave_search(hi_p, -1, hi_p - lo_p + 1, m_eff + (n - 1 - hi_p), sh->dbl[0], m_eff + (n - lo_p));
      }
    }
  }
  __syncthreads();
  const int kept = degenerate ? n : sh->i[0];
  __syncthreads();                                         // sh may be reused by the caller right away
  return kept;
}

}  // namespace rfkv
