// Gather-compaction of the retained K/V rows (Alg. 1, "Compress K / V by R") for gfx950.
//
// Grid (row blocks, units).  Workgroup (x, u) moves output rows [x * ROWS, ...) of unit u;
// workgroups past the unit's kept count leave at once.  ROWS = 16 with one row per thread step for
// a handful of units (the most workgroups in flight); with many units (a ragged batch, all layers
// of a model in one call) a workgroup moves 32 rows, two independent loads per thread in flight
// (measured on the ragged 8-sequence batch: 81 us with 16 rows, 73 us with 32, 76 us with 64).
// A row of d elements is moved as 16-byte pieces by row_bytes / 16 neighbouring lanes, so loads and
// stores of a row are fully coalesced, and every thread keeps several independent 16-byte loads in
// flight.
//
// Where the source position of output row t comes from:
//   kSrcPositionDesc  position ranking keeps two slabs, [0, sinks) and [n - (kept - sinks), n):
//                     pos = t < sinks ? t : n - kept + t           (no index list is read)
//   kSrcPaddedIdx     the per-unit padded list the select kernel wrote
//   kSrcPackedIdx     a packed list plus offsets supplied by the caller
// In the first two cases the unit's output offset is the sum of the kept counts of the units
// before it (ragged layout) or unit * pad_rows (padded layout, Sec. 3.3 "Running at Scale").  With
// up to 16 units every workgroup adds the counts up itself and workgroup x == 0 of each unit
// publishes the offset (and the grand total); with more, a one-workgroup scan kernel writes the
// offsets first.
#include "kernels.h"

namespace rfkv {
namespace {

constexpr int kRowsFew = 16, kUnrollFew = 1;      // a handful of units
constexpr int kRowsMany = 32, kUnrollMany = 2;    // many units
// The rows are read once and written once: non-temporal accesses keep them from displacing what the
// other kernels of the pass (and of the layers running beside it) re-use from the L2 and the
// Infinity Cache.  The copy itself runs at the same rate; the scoring pass next to it gets faster
// (headline step 71.5 -> 68.5 us).
typedef unsigned int cu32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 nt_load(const uint4* p) {
  const cu32x4 v = __builtin_nontemporal_load(reinterpret_cast<const cu32x4*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void nt_store(uint4* p, const uint4& v) {
  cu32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<cu32x4*>(p));
}
constexpr int kUniformPrefixUnits = 16;    // up to here every workgroup sums the earlier kept counts itself

template <int kRowsPerBlock, int kUnroll>
__global__ __launch_bounds__(kBlockThreads) void compact_kernel(CompactArgs a) {
  const int unit = blockIdx.y;
  const int b = unit / a.n_kv_heads, h = unit - b * a.n_kv_heads;
  const int s0 = a.cu[b];
  const int n = a.cu[b + 1] - s0;
  const int kept = min(max(a.kept[unit], 0), n);         // never trust a count past the sequence
  const int row0 = blockIdx.x * kRowsPerBlock;
  if (blockIdx.x > 0 && row0 >= kept) return;            // uniform

  int64_t off;
  if (a.source == kSrcPackedIdx) {
    off = a.offsets_in[unit];
  } else if (a.pad_rows > 0) {
    // padded layout: a fixed slot per unit, rows past the kept count are left untouched
    off = (int64_t)unit * a.pad_rows;
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.offsets_out) {
      a.offsets_out[unit] = off;
      if (unit == a.units - 1) a.offsets_out[a.units] = (int64_t)a.units * a.pad_rows;
    }
  } else if (a.offsets_ready) {
    off = a.offsets_out[unit];                           // written by compact_offsets_kernel just before
  } else {
    // a handful of units (launch_compact guarantees it): every workgroup adds up the kept counts of
    // the units before it in a uniform loop (scalar loads, no LDS, no barrier)
    off = 0;
    for (int u = 0; u < unit; ++u) {
      const int bu = u / a.n_kv_heads;
      off += min(max(a.kept[u], 0), a.cu[bu + 1] - a.cu[bu]);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && a.offsets_out) {
      a.offsets_out[unit] = off;
      if (unit == a.units - 1) a.offsets_out[a.units] = off + kept;
    }
  }
  if (row0 >= kept) return;

  int sinks = 0;
  const int32_t* idx = nullptr;
  if (a.source == kSrcPositionDesc) sinks = a.desc[unit].y;
  else if (a.source == kSrcPaddedIdx) idx = a.idx_pad + ((int64_t)s0 * a.n_kv_heads + (int64_t)h * n);
  else idx = a.idx_packed + off;

  const int row1 = min(kept, row0 + kRowsPerBlock);
  if (a.idx_out) {
    for (int t = row0 + threadIdx.x; t < row1; t += kBlockThreads)
      if (off + t < a.idx_capacity) a.idx_out[off + t] = idx ? idx[t] : (t < sinks ? t : n - kept + t);
  }
  if (!a.k_out) return;

  const int lanes_per_row = a.row_bytes >> 4;
  const int rows_per_step = kBlockThreads / lanes_per_row;
  const int sub = threadIdx.x / lanes_per_row;
  const int piece = threadIdx.x - sub * lanes_per_row;
  const unsigned char* kb = static_cast<const unsigned char*>(a.k);
  const unsigned char* vb = static_cast<const unsigned char*>(a.v);
  unsigned char* ko = static_cast<unsigned char*>(a.k_out);
  unsigned char* vo = static_cast<unsigned char*>(a.v_out);

  for (int t0 = row0 + sub; t0 < row1; t0 += rows_per_step * kUnroll) {
    uint4 kv[kUnroll], vv[kUnroll];
    int64_t dst[kUnroll];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const int t = t0 + j * rows_per_step;
      dst[j] = -1;
      if (t < row1) {
        int pos = idx ? idx[t] : (t < sinks ? t : n - kept + t);
        pos = min(max(pos, 0), n - 1);                   // a bad caller-supplied index cannot leave the sequence
        const int64_t tok = (int64_t)s0 + pos;
        kv[j] = nt_load(reinterpret_cast<const uint4*>(kb + a.k_stride_tok * tok + a.k_stride_head * h + piece * 16));
        vv[j] = nt_load(reinterpret_cast<const uint4*>(vb + a.v_stride_tok * tok + a.v_stride_head * h + piece * 16));
        if (off + t < a.capacity_rows) dst[j] = (off + t) * a.row_bytes + piece * 16;
      }
    }
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      if (dst[j] >= 0) {
        nt_store(reinterpret_cast<uint4*>(ko + dst[j]), kv[j]);
        nt_store(reinterpret_cast<uint4*>(vo + dst[j]), vv[j]);
      }
    }
  }
}

// Ragged output offsets for many units: the exclusive scan of the kept counts, once, by one
// workgroup, instead of every compaction workgroup adding up the counts of the units before it.
__global__ __launch_bounds__(1024) void compact_offsets_kernel(CompactArgs a) {
  __shared__ int64_t sh_wave[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int64_t carry = 0;
  for (int base = 0; base < a.units; base += 1024) {
    const int u = base + tid;
    int64_t v = 0;
    if (u < a.units) {
      const int bu = u / a.n_kv_heads;
      v = min(max(a.kept[u], 0), a.cu[bu + 1] - a.cu[bu]);
    }
    int64_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int64_t o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    __syncthreads();
    if (lane == 63) sh_wave[wave] = inc;
    __syncthreads();
    int64_t before = carry, total = 0;
    for (int w = 0; w < 16; ++w) {
      if (w < wave) before += sh_wave[w];
      total += sh_wave[w];
    }
    if (u < a.units) a.offsets_out[u] = before + inc - v;
    carry += total;
  }
  if (tid == 0) a.offsets_out[a.units] = carry;
}

}  // namespace

// Strides arrive in bytes here (the C-ABI layer converts from elements).
hipError_t launch_compact(const Geometry& g, const CompactArgs& a_in, hipStream_t stream) {
  if (g.units == 0) return hipSuccess;
  CompactArgs a = a_in;
  a.offsets_ready = 0;
  if (g.units > kUniformPrefixUnits && a.source != kSrcPackedIdx && a.pad_rows == 0) {
    if (!a.offsets_out) return hipErrorInvalidValue;     // the C ABI requires out_offsets
    hipLaunchKernelGGL(compact_offsets_kernel, dim3(1), dim3(1024), 0, stream, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.offsets_ready = 1;
  }
  if (g.units <= kUniformPrefixUnits) {
    const int xblocks = max(1, (g.max_seqlen + kRowsFew - 1) / kRowsFew);
    hipLaunchKernelGGL((compact_kernel<kRowsFew, kUnrollFew>), dim3(xblocks, g.units),
                       dim3(kBlockThreads), 0, stream, a);
  } else {
    const int xblocks = max(1, (g.max_seqlen + kRowsMany - 1) / kRowsMany);
    hipLaunchKernelGGL((compact_kernel<kRowsMany, kUnrollMany>), dim3(xblocks, g.units),
                       dim3(kBlockThreads), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace rfkv
