// Alg. 1's loop over the layers of a prefilled model as a software pipeline: one launch runs the
// statistics pass of layer j, the reduction pass (with the position-ranking cut) of layer j - 1 and the
// gather-compaction of layer j - 2 side by side, in one grid of two workgroups per CU.
//
// Why one kernel.  Run as separate kernels the three steps exclude each other: a scoring kernel holds
// every vector register of the CUs it is on, the compaction kernel every wavefront slot, so kernels
// of different layers on different streams overlap only at their ramps and tails, and each step pays
// its own ramp (first tiles ~5 us after the launch) and hand-over latencies on an otherwise idle
// chip.  Here the steps of three different layers are independent inside a launch (each depends only
// on the launch before), the scoring workgroups take one long span of keys each, the others copy
// rows from the first cycle on, and a workgroup that has finished its span joins the copy.  The memory
// system sees the K stream of one layer and the K / V gather of another at the same time, the matrix
// and vector pipes work under the copy's memory time, and per layer there is one launch instead of five.
//
// Row copy.  The compacted cache of a layer is one packed array of rows (unit after unit); it is cut
// into chunks of kChunkRows output rows that workgroups take from an atomic counter.  For an output
// row the unit follows from a bisection of the layer's offsets (an exclusive scan of the kept counts
// that every workgroup forms for itself in LDS), and the source position from the two slabs the
// position ranking keeps: pos = t < sinks ? t : n - kept + t.
#include "kernels.h"
#include "score_common.h"
#include "score_stream.h"
#include "select_position.h"

namespace rfkv {
namespace {

constexpr int kPipeThreads = 256;
constexpr int kCopyLoads = 8;                            // 1 KB loads of K (and of V) a wavefront keeps in flight

typedef unsigned int pu32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load(const unsigned char* p) {
  const pu32x4 v = __builtin_nontemporal_load(reinterpret_cast<const pu32x4*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void stream_store(unsigned char* p, const uint4& v) {
  pu32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<pu32x4*>(p));
}

// Per-unit table of the copy, in LDS: first output row, first token, length, sinks kept.
struct CopyTable {
  int64_t off[kPipelineMaxUnits + 1];
  int64_t wave_tot[4];
  int32_t s0[kPipelineMaxUnits];
  int32_t n[kPipelineMaxUnits];
  int32_t sinks[kPipelineMaxUnits];
};

// The gather-compaction of one layer (Alg. 1, "Compress K / V by R") by a workgroup that takes chunks
// of output rows until none is left.  `tab`: LDS; `sh_next`: one int of LDS.
__device__ __forceinline__ void copy_role(const CompactArgs& a, int32_t* queue, CopyTable* tab, int* sh_next) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // ---- the layer's units: exclusive scan of the kept counts (fixed order), first token, length, sinks
  __syncthreads();
  {
    const int per = (a.units + kPipeThreads - 1) / kPipeThreads;      // consecutive units per thread
    const int u0 = min(a.units, tid * per), u1 = min(a.units, u0 + per);
    int64_t mine = 0;
    for (int u = u0; u < u1; ++u) {
      const int b = u / a.n_kv_heads;
      const int s0 = a.cu[b], n = a.cu[b + 1] - s0;
      tab->s0[u] = s0;
      tab->n[u] = n;
      tab->sinks[u] = a.desc[u].y;
      mine += min(max(a.kept[u], 0), n);
    }
    int64_t inc = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int64_t o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    if (lane == 63) tab->wave_tot[wave] = inc;
    __syncthreads();
    int64_t run = inc - mine;
    for (int w = 0; w < wave; ++w) run += tab->wave_tot[w];
    for (int u = u0; u < u1; ++u) {
      tab->off[u] = run;
      run += min(max(a.kept[u], 0), tab->n[u]);
    }
    if (tid == kPipeThreads - 1) tab->off[a.units] = run;
    if (tid == 0) *sh_next = atomicAdd(queue, 1);
    __syncthreads();
  }
  const int64_t total = tab->off[a.units];
  if (blockIdx.x == 0 && a.offsets_out)
    for (int u = tid; u <= a.units; u += kPipeThreads) a.offsets_out[u] = tab->off[u];

  const int lanes_per_row = a.row_bytes >> 4;                          // 16-byte pieces of a row
  const int rows_per_load = 64 / lanes_per_row;                        // rows one 1 KB instruction moves
  const int chunk_rows = 4 * kCopyLoads * rows_per_load;               // rows of a chunk (4 wavefronts)
  const int64_t nchunks = (total + chunk_rows - 1) / chunk_rows;
  const int sub = lane / lanes_per_row, piece = lane - sub * lanes_per_row;
  const unsigned char* kb = static_cast<const unsigned char*>(a.k) + piece * 16;
  const unsigned char* vb = static_cast<const unsigned char*>(a.v) + piece * 16;
  unsigned char* ko = static_cast<unsigned char*>(a.k_out) + piece * 16;
  unsigned char* vo = static_cast<unsigned char*>(a.v_out) + piece * 16;
  for (;;) {
    const int64_t c = *sh_next;
    __syncthreads();                                                   // everyone has the chunk number
    if (c >= nchunks) break;
    if (tid == 0) *sh_next = atomicAdd(queue, 1);                      // the next one is fetched under this one's copy
    const int64_t r0 = c * chunk_rows + (int64_t)wave * kCopyLoads * rows_per_load + sub;
    // the unit of the wavefront's first row by bisection (last unit whose offset is <= the row); the rows
    // after it walk on from there
    int u = 0;
    {
      int lo = 0, hi = a.units - 1;
      const int64_t r = r0 < total ? r0 : total - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tab->off[mid] <= r) lo = mid;
        else hi = mid - 1;
      }
      u = lo;
    }
    uint4 kv[kCopyLoads], vv[kCopyLoads];
    int64_t dst[kCopyLoads];
#pragma unroll
    for (int j = 0; j < kCopyLoads; ++j) {
      const int64_t r = r0 + (int64_t)j * rows_per_load;               // output row
      dst[j] = -1;
      if (r < total) {
        while (tab->off[u + 1] <= r) ++u;                              // empty units are stepped over
        const int h = u % a.n_kv_heads;
        const int n = tab->n[u];
        const int kept = (int)(tab->off[u + 1] - tab->off[u]);
        const int t = (int)(r - tab->off[u]);
        int pos = t < tab->sinks[u] ? t : n - kept + t;
        pos = min(max(pos, 0), n - 1);
        const int64_t tok = (int64_t)tab->s0[u] + pos;
        kv[j] = stream_load(kb + a.k_stride_tok * tok + a.k_stride_head * h);
        vv[j] = stream_load(vb + a.v_stride_tok * tok + a.v_stride_head * h);
        if (r < a.capacity_rows) dst[j] = r * a.row_bytes;
        if (a.idx_out && piece == 0 && r < a.idx_capacity) a.idx_out[r] = pos;
      }
    }
#pragma unroll
    for (int j = 0; j < kCopyLoads; ++j) {
      if (dst[j] >= 0) {
        stream_store(ko + dst[j], kv[j]);
        stream_store(vo + dst[j], vv[j]);
      }
    }
    __syncthreads();                                                   // the next chunk number is in LDS
  }
}

// One launch of the pipeline: workgroup w < reduce_items + stats_items takes one scoring work item (those of
// the reduction pass come first), then every workgroup copies rows until none is left.  (One item per
// workgroup, not a loop over items: with the loop the compiler spills ~100 registers of the passes.)
template <typename T, int D, int RT_T>
__global__ __launch_bounds__(kPipeThreads, 2) void pipeline_kernel(PipelineArgs p) {
  RFKV_STREAM_LDS(T, D, RT_T, lds);
  static_assert(sizeof(CopyTable) <= 4 * 32 * Shape<T, D>::kRowBytes, "the copy's table reuses the tile buffers");
  __shared__ int sh_next;
  const int w = blockIdx.x;
  if (w < p.reduce_items) {
    score_stream_body<T, D, RT_T, 2>(p.reduce, w % p.reduce.nspans, w / p.reduce.nspans, lds);
  } else if (w < p.reduce_items + p.stats_items) {
    const int it = w - p.reduce_items;
    score_stream_body<T, D, RT_T, 1>(p.stats, it % p.stats.nspans, it / p.stats.nspans, lds);
  }
  if (p.copy_units > 0) copy_role(p.copy, p.queue, reinterpret_cast<CopyTable*>(lds.smem), &sh_next);
}

__global__ __launch_bounds__(256) void pipeline_prepare_kernel(int32_t* words, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) words[i] = 0;
}

template <typename T, int D>
hipError_t launch_typed(const PipelineArgs& p, int rt, hipStream_t stream) {
  // every scoring item has its workgroup; at least two workgroups per CU, and some that only copy
  const int items = p.reduce_items + p.stats_items;
  const dim3 grid(items + kPipelineGrid / 2 > kPipelineGrid ? items + kPipelineGrid / 2 : kPipelineGrid), block(kPipeThreads);
  if (rt <= 1) hipLaunchKernelGGL((pipeline_kernel<T, D, 1>), grid, block, 0, stream, p);
  else if (rt <= 2) hipLaunchKernelGGL((pipeline_kernel<T, D, 2>), grid, block, 0, stream, p);
  else if constexpr (Shape<T, D>::kChunks * 4 <= 32) {
    if (rt <= 4) hipLaunchKernelGGL((pipeline_kernel<T, D, 4>), grid, block, 0, stream, p);
    else return hipErrorInvalidValue;
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_pipeline_prepare(int32_t* words, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(pipeline_prepare_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, words, n);
  return hipGetLastError();
}

hipError_t launch_pipeline_step(const Geometry& g, const PipelineArgs& p, bool bf16, hipStream_t stream) {
  const int rt = g.rows_pad / 32;
  if (bf16) return g.head_dim == 64 ? launch_typed<Bf16, 64>(p, rt, stream) : launch_typed<Bf16, 128>(p, rt, stream);
  return g.head_dim == 64 ? launch_typed<Fp32, 64>(p, rt, stream) : launch_typed<Fp32, 128>(p, rt, stream);
}

}  // namespace rfkv
