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

template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes);
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
template <typename T, int D>
__device__ __forceinline__ void issue_tile_load(const unsigned char* kunit, int64_t tok_bytes, int tile0, int n,
                                                unsigned char* buf, int lane) {
  using S = Shape<T, D>;
  constexpr int kCpr = S::kRowBytes / 16;               // 16-byte chunks per key row
  constexpr int kSw = (kCpr < 16 ? kCpr : 16) - 1;
  constexpr int kLoads = 32 * kCpr / 64;                // instructions per tile, 1 KB each
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const int slot = j * 64 + lane;
    const int r = slot / kCpr;
    const int chunk = (slot % kCpr) ^ (r & kSw);
    const unsigned char* src = kunit + (int64_t)min(tile0 + r, n - 1) * tok_bytes + chunk * 16;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(buf + j * 1024), 16, 0, 0);
  }
}

template <typename T, int D>
__device__ __forceinline__ void read_tile_frags(uint4* kf, const unsigned char* buf, int col, int hi) {
  using S = Shape<T, D>;
  constexpr int kCpr = S::kRowBytes / 16;
  constexpr int kSw = (kCpr < 16 ? kCpr : 16) - 1;
#pragma unroll
  for (int ch = 0; ch < S::kChunks; ++ch) {
    const int slot = col * kCpr + ((hi * S::kChunks + ch) ^ (col & kSw));
    kf[ch] = *reinterpret_cast<const uint4*>(buf + slot * 16);
  }
}

}  // namespace

// defined in score.hip
hipError_t launch_score_merge(const Geometry& g, const ScoreArgs& a, hipStream_t stream);
// defined in score_qreg.hip: the register-resident-Q kernels and the shapes they cover
bool score_qreg_covers(const Geometry& g, bool bf16);
hipError_t launch_score_qreg(const Geometry& g, const ScoreArgs& a, bool bf16, hipStream_t stream, const Marks* marks);
}  // namespace rfkv
