// Pieces shared by the scoring kernels: storage types, MFMA chunk step, per-unit bookkeeping.
#pragma once

#include "kernels.h"
#include "tile_sum.h"

namespace rfkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct Bf16 { static constexpr int kBytes = 2; };
struct Fp32 { static constexpr int kBytes = 4; };

template <typename T, int D>
struct Shape {
  static constexpr int kRowBytes = D * T::kBytes;
  static constexpr int kHalfBytes = kRowBytes / 2;      // owned by one lane
  static constexpr int kChunks = kHalfBytes / 16;
  static constexpr int kLdsRowBytes = kRowBytes + 16;   // pad: consecutive rows shift by 4 banks
};

constexpr int KT = kKeyTilesPerWave;

template <typename T>
__device__ __forceinline__ f32x16 mma_chunk(const uint4& a, const uint4& b, f32x16 acc);

template <>
__device__ __forceinline__ f32x16 mma_chunk<Bf16>(const uint4& a, const uint4& b, f32x16 acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ f32x16 mma_chunk<Fp32>(const uint4& a, const uint4& b, f32x16 acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  return acc;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// The value held by lane (l ^ 32), by the gfx950 half-wave swap (v_permlane32_swap: one vector
// instruction, where a shuffle goes through the LDS crossbar and has to be waited for).  The swap
// exchanges the upper half of its first operand with the lower half of its second; with the same
// value in both, every lane ends up with its own value in one result and its partner's in the other.
__device__ __forceinline__ float other_half(float v) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

struct Unit {
  int b, h;
  int s0, n;        // first packed token and length of the sequence
  int wp;           // window rows in use, min(window, n)
  int q0;           // first packed window row of the sequence
  int rows;         // wp * group
  int row_tiles;    // ceil(rows / 32)
  int tile_base;    // first 32-position tile of the sequence in the per-head tile arrays
};

__device__ __forceinline__ Unit load_unit(const ScoreArgs& a, int unit) {
  Unit u;
  u.b = unit / a.n_kv_heads;
  u.h = unit - u.b * a.n_kv_heads;
  int q0 = 0, tb = 0;
  for (int bb = 0; bb < u.b; ++bb) {
    const int len = a.cu[bb + 1] - a.cu[bb];
    q0 += min(a.window, len);
    tb += (len + kTileKeys - 1) / kTileKeys;
  }
  u.q0 = q0;
  u.tile_base = tb;
  u.s0 = a.cu[u.b];
  u.n = a.cu[u.b + 1] - u.s0;
  u.wp = min(a.window, u.n);
  u.rows = u.wp * a.group;
  u.row_tiles = (u.rows + 31) >> 5;
  return u;
}


// Window queries of the unit -> LDS, row r = t * G + g, rows beyond `rows` zero, row stride
// kLdsRowBytes.  Loads are issued in batches of eight per thread before any of them is stored,
// so the staging costs about one memory round trip instead of one per 16-byte chunk.
template <typename T, int D>
__device__ __forceinline__ void stage_q(const ScoreArgs& a, const Unit& u, unsigned char* smem) {
  using S = Shape<T, D>;
  constexpr int kChunksPerRow = S::kRowBytes / 16;
  constexpr int kBatch = 8;
  const int total = u.row_tiles * 32 * kChunksPerRow;
  const unsigned char* qbase = static_cast<const unsigned char*>(a.q);
  for (int i0 = threadIdx.x; i0 < total; i0 += kBlockThreads * kBatch) {
    uint4 val[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int i = i0 + j * kBlockThreads;
      const int r = i / kChunksPerRow;
      const int c = i - r * kChunksPerRow;
      val[j] = make_uint4(0, 0, 0, 0);
      if (i < total && r < u.rows) {
        const int t = r / a.group;
        const int g = r - t * a.group;
        const int64_t off = (int64_t)(u.q0 + t) * a.q_stride_row + (int64_t)(u.h * a.group + g) * a.q_stride_head;
        val[j] = *reinterpret_cast<const uint4*>(qbase + off * T::kBytes + c * 16);
      }
    }
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int i = i0 + j * kBlockThreads;
      const int r = i / kChunksPerRow;
      const int c = i - r * kChunksPerRow;
      if (i < total) *reinterpret_cast<uint4*>(smem + r * S::kLdsRowBytes + c * 16) = val[j];
    }
  }
}

// Issue the direct-to-LDS loads of the 32-key tile starting at `tile0` (keys past the end of the
// sequence re-read the last key; their logits are masked later).
// A 32-key tile into `buf` by direct-to-LDS loads, 1 KB (64 lanes x 16 bytes) per instruction:
// instruction j brings key rows j * kRowStep .. + kRowStep - 1, lane (rl, cl) 16-byte chunk
// cl ^ (row & kSw) of row j * kRowStep + rl (the XOR makes the MFMA-layout read-back conflict
// free).  Rows past the unit's last key repeat the last key.
template <typename T, int D>
struct TileLoader {
  using S = Shape<T, D>;
  static constexpr int kCpr = S::kRowBytes / 16;        // 16-byte chunks per key row
  static constexpr int kSw = (kCpr < 16 ? kCpr : 16) - 1;
  static constexpr int kLoads = 32 * kCpr / 64;         // instructions per tile
  static constexpr int kRowStep = 64 / kCpr;            // rows per instruction
  static_assert(kRowStep * kCpr == 64 && (kRowStep & (kRowStep - 1)) == 0, "whole rows, a power of two of them");

  const unsigned char* kunit;
  int64_t tok_bytes;
  int n;
  int lane;

  __device__ __forceinline__ TileLoader(const unsigned char* kunit_, int64_t tok_bytes_, int n_, int lane_)
      : kunit(kunit_), tok_bytes(tok_bytes_), n(n_), lane(lane_) {}

  // tile0 must be the same in every lane of the wavefront.
  __device__ __forceinline__ void issue(int tile0, unsigned char* buf) const {
    tile0 = __builtin_amdgcn_readfirstlane(tile0);
    // the per-lane address parts are a few instructions: recomputed per tile (the empty asm hides
    // that they do not change) rather than held in registers across the caller's loop
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int rl = ln / kCpr, cl = ln % kCpr;
    if (tile0 + 32 <= n) {
      const uint32_t lane_off = (uint32_t)rl * (uint32_t)tok_bytes;
      const int c0 = cl ^ (rl & kSw);               // the chunk fetched is c0 ^ ((j * kRowStep) & kSw)
      // interior tile: one scalar base per instruction plus a per-lane 32-bit offset
      // ((j * kRowStep + rl) & kSw == ((j * kRowStep) & kSw) | (rl & kSw), so the XOR splits)
      const unsigned char* base = kunit + (int64_t)tile0 * tok_bytes;
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const uint32_t voff = lane_off + (uint32_t)((c0 ^ ((j * kRowStep) & kSw)) << 4);
        const unsigned char* src = base + (int64_t)(j * kRowStep) * tok_bytes + voff;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(buf + j * 1024), 16, 0, 0);
      }
    } else {
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const int r = j * kRowStep + rl;
        const int chunk = cl ^ (r & kSw);
        const unsigned char* src = kunit + (int64_t)min(tile0 + r, n - 1) * tok_bytes + chunk * 16;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)(buf + j * 1024), 16, 0, 0);
      }
    }
  }
};

// ---- LDS accesses the compiler does not see.
// While a direct-to-LDS load is in flight the compiler makes every LDS access it cannot prove
// disjoint from the load's destination wait for ALL outstanding loads (s_waitcnt vmcnt(0)), which
// would serialise a double-buffered tile pipeline.  The accesses below are issued from inline
// assembly: the kernel orders them against the loads itself (s_waitcnt vmcnt(N) on the tile it is
// about to read, barriers around staging areas).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// Writes; the caller issues lds_writes_done() before the barrier that publishes them.
__device__ __forceinline__ void lds_write_b128(void* dst, const uint4& v) {
  asm volatile("ds_write_b128 %0, %1" ::"v"(lds_offset(dst)), "v"(__builtin_bit_cast(u32x4, v)) : "memory");
}
__device__ __forceinline__ void lds_write_b32(void* dst, uint32_t v) {
  asm volatile("ds_write_b32 %0, %1" ::"v"(lds_offset(dst)), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_writes_done() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// N 16-byte reads at the given LDS offsets, complete on return (the wait is part of the block, so
// no copy of a destination register can be scheduled before its data has arrived).
__device__ __forceinline__ void lds_read_b128_x4(uint4* out, const uint32_t* a) {
  u32x4 r0, r1, r2, r3;
  asm volatile(
      "ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3)
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3])
      : "memory");
  out[0] = __builtin_bit_cast(uint4, r0);
  out[1] = __builtin_bit_cast(uint4, r1);
  out[2] = __builtin_bit_cast(uint4, r2);
  out[3] = __builtin_bit_cast(uint4, r3);
}
__device__ __forceinline__ void lds_read_b128_x8(uint4* out, const uint32_t* a) {
  u32x4 r0, r1, r2, r3, r4, r5, r6, r7;
  asm volatile(
      "ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\tds_read_b128 %3, %11\n\t"
      "ds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\tds_read_b128 %6, %14\n\tds_read_b128 %7, %15\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7])
      : "memory");
  out[0] = __builtin_bit_cast(uint4, r0);
  out[1] = __builtin_bit_cast(uint4, r1);
  out[2] = __builtin_bit_cast(uint4, r2);
  out[3] = __builtin_bit_cast(uint4, r3);
  out[4] = __builtin_bit_cast(uint4, r4);
  out[5] = __builtin_bit_cast(uint4, r5);
  out[6] = __builtin_bit_cast(uint4, r6);
  out[7] = __builtin_bit_cast(uint4, r7);
}
template <int N>
__device__ __forceinline__ void lds_read_b128_n(uint4* out, const uint32_t* a) {
  static_assert(N % 4 == 0, "reads come in blocks of four");
  if constexpr (N == 4) {
    lds_read_b128_x4(out, a);
  } else {
#pragma unroll
    for (int i = 0; i < N; i += 8) lds_read_b128_x8(out + i, a + i);
  }
}

// MFMA fragments of a 32-key tile that TileLoader::issue has brought in (the caller has waited for
// its loads): lane (col, hi) gets the `hi` half of key row `col`, chunk by chunk.  Complete on return.
// One row tile (32 rows) of a unit's window queries into `buf`, in the layout of a key tile
// (row r = t * G + g of the KV head; rows past the unit's last repeat the last row: their
// results are discarded by an infinite exponent offset).
template <typename T, int D>
__device__ __forceinline__ void issue_q_tile_load(const ScoreArgs& a, const Unit& u, int rt, unsigned char* buf, int lane) {
  using S = Shape<T, D>;
  constexpr int kCpr = S::kRowBytes / 16;
  constexpr int kSw = (kCpr < 16 ? kCpr : 16) - 1;
  constexpr int kLoads = 32 * kCpr / 64;
  constexpr int kRowStep = 64 / kCpr;                   // rows one instruction advances
  static_assert(kRowStep * kCpr == 64, "an instruction covers whole rows");
  const unsigned char* qbase = static_cast<const unsigned char*>(a.q);
  const int rl = lane / kCpr, cl = lane % kCpr;         // row within the instruction, chunk
  const int dt = kRowStep / a.group, dg = kRowStep - dt * a.group;
  int row = rt * 32 + rl;
  int t = row / a.group, g = row - t * a.group;
  const int t_last = (u.rows - 1) / a.group, g_last = (u.rows - 1) - t_last * a.group;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const int r = j * kRowStep + rl;                    // row within the tile
    const int chunk = cl ^ (r & kSw);
    const bool in = row < u.rows;
    const int tt = in ? t : t_last, gg = in ? g : g_last;
    const int64_t off = (int64_t)(u.q0 + tt) * a.q_stride_row + (int64_t)(u.h * a.group + gg) * a.q_stride_head;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(qbase + off * T::kBytes + chunk * 16),
                                     (__attribute__((address_space(3))) void*)(buf + j * 1024), 16, 0, 0);
    row += kRowStep;
    t += dt;
    g += dg;
    if (g >= a.group) {
      g -= a.group;
      ++t;
    }
  }
}

template <typename T, int D>
__device__ __forceinline__ void read_tile_frags(uint4* kf, const unsigned char* buf, int col, int hi) {
  using S = Shape<T, D>;
  constexpr int kCpr = S::kRowBytes / 16;
  constexpr int kSw = (kCpr < 16 ? kCpr : 16) - 1;
  const uint32_t base = lds_offset(buf);
  int sw = col & kSw;
  asm volatile("" : "+v"(sw));                          // recompute the addresses per tile: cheaper than
  uint32_t addr[S::kChunks];                            // holding one register per chunk across the loop
#pragma unroll
  for (int ch = 0; ch < S::kChunks; ++ch) {
    const int slot = col * kCpr + ((hi * S::kChunks + ch) ^ sw);
    addr[ch] = base + slot * 16;
  }
  lds_read_b128_n<S::kChunks>(kf, addr);
}

}  // namespace

// defined in score.hip
hipError_t launch_score_merge(const Geometry& g, const ScoreArgs& a, hipStream_t stream);
// row offsets from the caller's log-sum-exp (a.lse) instead of statistics pass + merge; no-op without one
hipError_t launch_score_offsets(const Geometry& g, const ScoreArgs& a, hipStream_t stream, const Marks* marks);
// defined in score_qreg.hip: the streaming kernels and the shapes they cover
bool score_qreg_covers(const Geometry& g, bool bf16);
hipError_t launch_score_qreg(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream, const Marks* marks);
// wide windows (more than RFKV_MAX_SCORE_ROWS score rows): statistics in score_qreg.hip, the whole path in score_wide.hip
hipError_t launch_score_wide_stats(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream);
hipError_t launch_score_wide(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream, const Marks* marks);
}  // namespace rfkv
