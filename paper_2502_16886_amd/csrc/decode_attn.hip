// Attention of a block of new queries over the compacted ragged cache, and the same over the
// uncompressed cache with the evicted positions masked (the consumer of Alg. 1's compressed K / V;
// Sec. 4.3 compares the two costs).  bf16 storage, fp32 softmax and accumulation, fp32 output.
//
// The kept counts differ from unit to unit and are known on the device only, so every workgroup first
// cuts the units' keys into work items of nearly equal length (about as many items as the launch has
// workgroups to keep every CU busy once; the same arithmetic in every workgroup, no kernel of its own)
// and takes the item of its index -- a contiguous range of keys of one unit (sequence, KV head) --
// and all M = n_new * G query rows of that KV head (row = j * G + g), 32 * RTW rows per wavefront:
//
//   S^T = K Q^T   32x32x16 bf16 MFMA, keys along M, rows along N: a lane owns one query row and
//                 16 of the tile's 32 keys, so the softmax statistics are in-lane (plus one
//                 exchange between the two half-waves).
//   O^T = V^T P^T the probabilities, rounded to bf16, are already in B-operand layout (row =
//                 lane, keys in registers); V^T fragments (one value column, 8 keys) are read
//                 from the row-major LDS tile by the LDS transpose read (ds_read_b64_tr_b16).  The accumulator keeps the
//                 lane <-> row mapping, so the online-softmax rescale is lane-local too.
//
// K and V tiles (32 keys each) arrive by direct-to-LDS loads, kStages tiles deep, every wavefront
// issuing a quarter of each tile; one barrier per tile hands a landed tile to all wavefronts and
// frees the oldest buffer.  Partial results (reference exponent, sum, unnormalised O) per item
// are merged by a last kernel.
#include "kernels.h"
#include "score_common.h"

// Tunables of the 256-row decode workgroup (rows per wavefront / 32, 32-key tiles per stage).
// Measured on config 4 (64 new queries, attention + merge): 4 wavefronts x 64 rows, 1 tile per stage
// 276 us; 8 x 32 rows, 1 tile 208 us; 8 x 32 rows, 2 tiles 193 us; 4 x 64 rows, 2 tiles 254 us.
namespace rfkv {
namespace {

constexpr int kDecodeRtw = 1;          // 32-row tiles per wavefront of the 256-row workgroup
constexpr int kDecodeKt = 2;           // 32-key tiles per stage, 256-row workgroup
constexpr int kDecodeKtSmall = 1;      // 32-key tiles per stage, 128-row workgroup

// Shape of a decode workgroup: W wavefronts of 32 * RTW query rows each; a pipeline stage holds
// KT 32-key tiles of K and of V; kStagesFor stages of them are in flight / in use.
constexpr int stages_for(int kt) { return kt == 1 ? 4 : 3; }
// tiles per stage, raised where a stage would otherwise hold fewer load instructions than wavefronts
constexpr int kt_for(int d, int w, int kt) { return kt * (d / 16) < w ? w / (d / 16) : kt; }

template <int D>
struct DShape {
  static constexpr int kRowBytes = D * 2;
  static constexpr int kCpr = kRowBytes / 16;            // 16-byte chunks per row
  static constexpr int kTileBytes = 32 * kRowBytes;
  static constexpr int kLoads = kTileBytes / 1024;        // direct-to-LDS instructions per tile
  static constexpr int kRowStep = 64 / kCpr;              // rows per instruction
  static constexpr int kChunks = kRowBytes / 32;          // 16-byte chunks of half a row (MFMA steps of S)
  static constexpr int kDT = D / 32;                      // 32-column tiles of the output
};

// V^T fragments for MFMA step S of the O^T product, by the LDS transpose read: element e of lane
// (col, hi) is key 16 S + 8 (e / 4) + 4 hi + e % 4 of the tile (the keys whose probabilities the
// lane's B operand holds in the same order), value column dt * 32 + col.  One ds_read_b64_tr_b16
// hands a group of 16 lanes a transposed 4 keys x 16 columns block: lane j of the group points at
// the 8 bytes (key j / 4, columns 4 (j % 4) ..), lane i receives column i of the four keys.  Two
// reads (keys +0..3 and +8..11) make one fragment.  `addr[dt]` is the lane's pointer for column
// tile dt at key row 4 hi; RB = bytes per key row.  Complete on return.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <int RB, int S>
__device__ __forceinline__ void lds_read_vt_x4(uint4* out, const uint32_t* addr) {
  u32x2 a0, b0, a1, b1, a2, b2, a3, b3;
  asm volatile(
      "ds_read_b64_tr_b16 %0, %8 offset:%12\n\tds_read_b64_tr_b16 %1, %8 offset:%13\n\t"
      "ds_read_b64_tr_b16 %2, %9 offset:%12\n\tds_read_b64_tr_b16 %3, %9 offset:%13\n\t"
      "ds_read_b64_tr_b16 %4, %10 offset:%12\n\tds_read_b64_tr_b16 %5, %10 offset:%13\n\t"
      "ds_read_b64_tr_b16 %6, %11 offset:%12\n\tds_read_b64_tr_b16 %7, %11 offset:%13\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(a0), "=&v"(b0), "=&v"(a1), "=&v"(b1), "=&v"(a2), "=&v"(b2), "=&v"(a3), "=&v"(b3)
      : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "n"((16 * S) * RB), "n"((16 * S + 8) * RB)
      : "memory");
  out[0] = make_uint4(a0[0], a0[1], b0[0], b0[1]);
  out[1] = make_uint4(a1[0], a1[1], b1[0], b1[1]);
  out[2] = make_uint4(a2[0], a2[1], b2[0], b2[1]);
  out[3] = make_uint4(a3[0], a3[1], b3[0], b3[1]);
}
template <int RB, int S>
__device__ __forceinline__ void lds_read_vt_x2(uint4* out, const uint32_t* addr) {
  u32x2 a0, b0, a1, b1;
  asm volatile(
      "ds_read_b64_tr_b16 %0, %4 offset:%6\n\tds_read_b64_tr_b16 %1, %4 offset:%7\n\t"
      "ds_read_b64_tr_b16 %2, %5 offset:%6\n\tds_read_b64_tr_b16 %3, %5 offset:%7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(a0), "=&v"(b0), "=&v"(a1), "=&v"(b1)
      : "v"(addr[0]), "v"(addr[1]), "n"((16 * S) * RB), "n"((16 * S + 8) * RB)
      : "memory");
  out[0] = make_uint4(a0[0], a0[1], b0[0], b0[1]);
  out[1] = make_uint4(a1[0], a1[1], b1[0], b1[1]);
}

__device__ __forceinline__ uint32_t lds_read_b32_now(const void* p) {
  uint32_t r;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(lds_offset(p)) : "memory");
  return r;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

struct DUnit {
  int b, h;
  int64_t row0;      // first key row of the unit in k / v (packed row or token index)
  int len;           // keys of the unit
};

template <bool MASKED>
__device__ __forceinline__ DUnit load_dunit(const DecodeArgs& a, int unit) {
  DUnit u;
  u.b = unit / a.n_kv_heads;
  u.h = unit - u.b * a.n_kv_heads;
  if (MASKED) {
    u.row0 = a.cu[u.b];
    u.len = a.cu[u.b + 1] - (int)u.row0;
  } else {
    u.row0 = a.offsets[unit];
    u.len = (int)(a.offsets[unit + 1] - u.row0);
    if (a.kept) u.len = min(max(a.kept[unit], 0), u.len);    // padded layout: the slot's first kept rows
  }
  return u;
}

// Work items: item_begin[u] .. item_begin[u + 1] are unit u's; item i of unit u covers keys
// [i * C * kChunkKeys, min(len, (i + 1) * C * kChunkKeys)).  Keys are handed out in chunks of kChunkKeys; every
// item gets at most C chunks, C chosen so that the items number about `a.target_items` (never more than
// target_items + units, the launch's grid).  Returns workgroup `bx`'s item {unit, first key, end key, -}
// (unit < 0: the grid has more workgroups than there are items); with `write_table` also writes item_begin
// (for the merge kernel).  Called by all NT threads of the workgroup.
constexpr int kChunkKeys = 256;

template <bool MASKED, int NT>
__device__ __forceinline__ int4 plan_item(const DecodeArgs& a, int bx, bool write_table) {
  constexpr int kW = NT / 64;
  __shared__ long long sh_tot[kW];
  __shared__ int sh_scan[kW];
  __shared__ int4 sh_item;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int units = a.units;
  // total chunks
  long long mine = 0;
  for (int u = tid; u < units; u += NT) mine += (load_dunit<MASKED>(a, u).len + kChunkKeys - 1) / kChunkKeys;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d);
  if (lane == 0) sh_tot[wave] = mine;
  if (tid == 0) sh_item = make_int4(-1, 0, 0, 0);
  __syncthreads();
  long long total = 0;
#pragma unroll
  for (int w = 0; w < kW; ++w) total += sh_tot[w];
  const int C = (int)max(1ll, (total + a.target_items - 1) / a.target_items);
  // items per unit, exclusive prefix over units in batches of NT
  int carry = 0;
  for (int base = 0; base < units; base += NT) {
    const int u = base + tid;
    int len = 0, cnt = 0;
    if (u < units) {
      len = load_dunit<MASKED>(a, u).len;
      const int chunks = (len + kChunkKeys - 1) / kChunkKeys;
      cnt = (chunks + C - 1) / C;
    }
    int inc = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    __syncthreads();
    if (lane == 63) sh_scan[wave] = inc;
    __syncthreads();
    int off = carry, tot = 0;
#pragma unroll
    for (int w = 0; w < kW; ++w) {
      if (w < wave) off += sh_scan[w];
      tot += sh_scan[w];
    }
    const int first = off + inc - cnt;
    if (u < units) {
      if (write_table) a.item_begin[u] = first;
      if (bx >= first && bx < first + cnt) {
        const int i = bx - first;
        sh_item = make_int4(u, i * C * kChunkKeys, min(len, (i + 1) * C * kChunkKeys), 0);
      }
    }
    carry += tot;
  }
  if (write_table && tid == 0) a.item_begin[units] = carry;
  __syncthreads();
  return sh_item;
}

template <int D, int RTW, int W, int KT, bool MASKED>
__global__ __launch_bounds__(W * 64, (W == 4 && RTW == 1) ? 2 : 1) void decode_attn_kernel(DecodeArgs a) {
  using S = DShape<D>;
  using KS = Shape<Bf16, D>;
  constexpr int kStages = stages_for(KT);
  constexpr int kStageBytes = KT * S::kTileBytes;        // K (or V) bytes of one stage
  constexpr int kStageLoads = KT * S::kLoads;            // direct-to-LDS instructions per stage and tensor
  constexpr int kPerWave = kStageLoads / W;              // ... per wavefront
  static_assert(kPerWave >= 1 && kPerWave * W == kStageLoads, "the wavefronts share a stage's loads evenly");
  static_assert(KT <= 2, "one mask byte per lane covers at most 64 keys per stage");
  // dynamic LDS: kStages key stages, kStages value stages, then (MASKED) 64 mask words per stage and wavefront
  extern __shared__ __attribute__((aligned(1024))) unsigned char dsm[];
  unsigned char* ksm = dsm;
  unsigned char* vsm = dsm + kStages * kStageBytes;
  uint32_t* msm = reinterpret_cast<uint32_t*>(dsm + 2 * kStages * kStageBytes);
  const int bx = blockIdx.x;
  const int4 item = plan_item<MASKED, W * 64>(a, bx, bx == 0);
  const int unit = item.x;
  if (unit < 0) return;                                  // uniform for the whole workgroup
  const DUnit u = load_dunit<MASKED>(a, unit);
  const int span_begin = item.y, span_end = item.z;      // 0 <= begin < end <= u.len
  const int ntiles = (span_end - span_begin + 32 * KT - 1) / (32 * KT);      // stages' worth of keys

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hi = lane >> 5;
  const float c = a.c;
  const float kNegInf = -__builtin_inff();

  // ---- query fragments (B operand of S^T): ordinary loads, complete before any tile is requested
  uint4 qf[RTW][S::kChunks];
  {
    const unsigned char* qbase = static_cast<const unsigned char*>(a.q);
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) {
      const int row = (wave * RTW + rt) * 32 + col;
      const int rr = min(row, a.rows - 1);
      const int j = rr / a.group, g = rr - j * a.group;
      const int64_t off = (((int64_t)u.b * a.n_new + j) * a.n_q_heads + (int64_t)u.h * a.group + g) * D;
      const uint4* src = reinterpret_cast<const uint4*>(qbase + off * 2 + hi * KS::kHalfBytes);
#pragma unroll
      for (int ch = 0; ch < S::kChunks; ++ch) qf[rt][ch] = row < a.rows ? src[ch] : make_uint4(0, 0, 0, 0);
    }
  }
  // force the fragments into registers now (the loads must not drift below the first tile request)
#pragma unroll
  for (int rt = 0; rt < RTW; ++rt)
#pragma unroll
    for (int ch = 0; ch < S::kChunks; ++ch) {
      u32x4 t = __builtin_bit_cast(u32x4, qf[rt][ch]);
      asm volatile("" : "+v"(t));
      qf[rt][ch] = __builtin_bit_cast(uint4, t);
    }

  const unsigned char* kunit = static_cast<const unsigned char*>(a.k) +
                               (u.row0 * a.k_stride_tok + (int64_t)u.h * a.k_stride_head) * 2;
  const unsigned char* vunit = static_cast<const unsigned char*>(a.v) +
                               (u.row0 * a.v_stride_tok + (int64_t)u.h * a.v_stride_head) * 2;
  const int64_t k_tok = a.k_stride_tok * 2, v_tok = a.v_stride_tok * 2;
  const unsigned char* munit = MASKED ? a.mask + (int64_t)u.h * a.total_tokens + u.row0 : nullptr;

  // This wavefront's share of stage-load `t` (32 * KT keys from span_begin + t * 32 * KT) into stage
  // t % kStages.  Per-lane parts of the addresses: instruction jj of this wavefront fetches row r_jj
  // of the stage, K chunk cl ^ (r & kSw), V chunk cl ^ (vswz(r) << 2) (the layouts the fragment
  // reads expect; a 32-key tile is kLoads consecutive instructions, so tiles stay contiguous in LDS)
  const int rl = lane / S::kCpr, cl = lane % S::kCpr;
  // 64-byte block b of value row r sits at block b ^ vswz(r): the four key rows a half-wave's
  // transpose read touches then fall into four different quarters of the 64 banks (without it the
  // rows of a read, 256 or 128 bytes apart, met in the same banks: 4-way conflicts on every read)
  auto vswz = [](int r) { return D == 128 ? (r & 3) : ((r >> 1) & 1); };
  uint32_t koff[kPerWave], voff[kPerWave];
#pragma unroll
  for (int jj = 0; jj < kPerWave; ++jj) {
    const int r = (wave * kPerWave + jj) * S::kRowStep + rl;
    koff[jj] = (uint32_t)(r * k_tok) + (uint32_t)((cl ^ (r & ((S::kCpr < 16 ? S::kCpr : 16) - 1))) << 4);
    voff[jj] = (uint32_t)(r * v_tok) + (uint32_t)((cl ^ (vswz(r) << 2)) << 4);
  }
  auto issue_tile = [&](int t) {
    const int tile0 = __builtin_amdgcn_readfirstlane(span_begin + t * 32 * KT);
    const int st = t % kStages;
    if (tile0 + 32 * KT <= u.len) {
      // interior tile: a scalar base per tile plus the per-lane offsets
      const unsigned char* kb = kunit + (int64_t)tile0 * k_tok;
      const unsigned char* vb = vunit + (int64_t)tile0 * v_tok;
#pragma unroll
      for (int jj = 0; jj < kPerWave; ++jj) {
        const int j = wave * kPerWave + jj;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kb + koff[jj]),
                                         (__attribute__((address_space(3))) void*)(ksm + st * kStageBytes + j * 1024),
                                         16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vb + voff[jj]),
                                         (__attribute__((address_space(3))) void*)(vsm + st * kStageBytes + j * 1024),
                                         16, 0, 0);
      }
    } else {
      // the unit's last tile: rows past the end repeat the last key (masked out below)
#pragma unroll
      for (int jj = 0; jj < kPerWave; ++jj) {
        const int j = wave * kPerWave + jj;
        const int r = j * S::kRowStep + rl;
        const int64_t key = min(tile0 + r, u.len - 1);
        const int kchunk = cl ^ (r & ((S::kCpr < 16 ? S::kCpr : 16) - 1));
        const int vchunk = cl ^ (vswz(r) << 2);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kunit + key * k_tok + kchunk * 16),
                                         (__attribute__((address_space(3))) void*)(ksm + st * kStageBytes + j * 1024),
                                         16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vunit + key * v_tok + vchunk * 16),
                                         (__attribute__((address_space(3))) void*)(vsm + st * kStageBytes + j * 1024),
                                         16, 0, 0);
      }
    }
    if (MASKED) {
      // one byte per lane: key tile0 + lane (lanes past the stage's keys repeat); one dword per lane
      const int64_t key = min(tile0 + (lane & (32 * KT - 1)), u.len - 1);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(munit + key),
                                       (__attribute__((address_space(3))) void*)(msm + (st * W + wave) * 64), 1, 0, 0);
    }
  };
  constexpr int kPerTile = 2 * kPerWave + (MASKED ? 1 : 0);        // loads one wavefront issues per stage

  // Per-lane byte offsets of the fragment reads within a 32-key tile.  K: 16-byte chunk
  // (hi * kChunks + ch) of key row `col`, at slot chunk ^ (col & kSw) (the layout TileLoader-style
  // loads leave).  V: lane 16 g + j points at key row 4 hi + j / 4, columns (g % 2) * 16 + 4 (j % 4) ..
  // of column tile dt, whose 64-byte block sits at block dt ^ vswz(row).
  uint32_t klane[S::kChunks], vlane[S::kDT];
  {
    constexpr int kSw = (S::kCpr < 16 ? S::kCpr : 16) - 1;
#pragma unroll
    for (int ch = 0; ch < S::kChunks; ++ch)
      klane[ch] = (uint32_t)(col * S::kCpr + ((hi * S::kChunks + ch) ^ (col & kSw))) * 16u;
    const int j = lane & 15, half = (lane >> 4) & 1;
    const uint32_t vb = (4 * hi + (j >> 2)) * S::kRowBytes + (half * 2 + ((j & 3) >> 1)) * 16 + (j & 1) * 8;
    const int swz = D == 128 ? (j >> 2) : ((j >> 3) & 1);          // vswz of the lane's key row (4 hi + j / 4 + a multiple of 8)
#pragma unroll
    for (int dt = 0; dt < S::kDT; ++dt) vlane[dt] = vb + ((dt ^ swz) << 6);
  }

  float m_run[RTW], l_run[RTW];
  f32x16 o[RTW][S::kDT];
#pragma unroll
  for (int rt = 0; rt < RTW; ++rt) {
    m_run[rt] = kNegInf;
    l_run[rt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < S::kDT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[rt][dt][i] = 0.f;
  }

#pragma unroll
  for (int t = 0; t < kStages - 1; ++t)
    if (t < ntiles) issue_tile(t);

  for (int t = 0; t < ntiles; ++t) {
    // tiles t+1 .. t+kStages-2 (those that exist) are behind tile t in this wavefront's load queue
    const int behind = min(kStages - 2, ntiles - 1 - t);
    if (behind >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kPerTile) : "memory");
    else if (behind == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kPerTile) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // every wavefront's share of tile t has landed and everyone is done with tile t-1.  The bare
    // barrier: the landed data was waited for above, and a fence here would wait for the tiles in flight
    __builtin_amdgcn_s_barrier();
    if (t + kStages - 1 < ntiles) issue_tile(t + kStages - 1);       // into the stage tile t-1 used

    const int st = t % kStages;
    unsigned long long stage_keep = ~0ull;               // bit i: key (stage start + i) takes part
    if (MASKED) {
      const uint32_t mword = lds_read_b32_now(msm + (st * W + wave) * 64 + lane);
      stage_keep = __ballot((mword & 0xffu) != 0);
    }
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
    const int tile0 = span_begin + (t * KT + kt) * 32;
    if (KT > 1 && tile0 >= span_end) break;              // uniform: the span ended inside this stage
    const unsigned char* kbuf = ksm + st * kStageBytes + kt * S::kTileBytes;
    const unsigned char* vbuf = vsm + st * kStageBytes + kt * S::kTileBytes;
    uint4 kf[S::kChunks];
    {
      // the lane's fragment offsets within a tile are kept in registers; per tile one add of the
      // tile's (uniform) LDS base each
      const uint32_t kb = __builtin_amdgcn_readfirstlane(lds_offset(kbuf));
      uint32_t kaddr[S::kChunks];
#pragma unroll
      for (int ch = 0; ch < S::kChunks; ++ch) kaddr[ch] = kb + klane[ch];
      lds_read_b128_n<S::kChunks>(kf, kaddr);
    }

    uint32_t keep_bits = (uint32_t)(stage_keep >> (32 * kt));              // bit i: key tile0 + i takes part
    if (tile0 + 32 > u.len) keep_bits &= (1u << (u.len - tile0)) - 1u;      // 1 <= len - tile0 <= 31 here
    const bool all_in = keep_bits == 0xffffffffu;        // uniform

    uint4 pf[RTW][2];                                    // probabilities, B operand of the two O^T steps
    float alpha[RTW];
    bool rescale = false;
    // the MFMA chains of all row tiles interleaved, so that none waits for its own previous step
    f32x16 sacc[RTW];
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[rt][i] = 0.f;
#pragma unroll
    for (int ch = 0; ch < S::kChunks; ++ch)
#pragma unroll
      for (int rt = 0; rt < RTW; ++rt) sacc[rt] = mma_chunk<Bf16>(kf[ch], qf[rt][ch], sacc[rt]);
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) {
      // value i of this lane: key tile0 + 8 (i / 4) + 4 hi + i % 4, row = lane's row
      float x[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = sacc[rt][i];
      if (!all_in) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kk = (i >> 2) * 8 + hi * 4 + (i & 3);
          if (!((keep_bits >> kk) & 1u)) x[i] = kNegInf;
        }
      }
      // The reference exponent only has to keep 2^x in range: once every row of the wavefront has
      // one, the tile is taken against it as it stands; the tile's maximum is looked for (and the
      // accumulators rescaled) only when a sum nears overflow or a row has seen no key yet.
      float p[16], sum = 0.f;
      alpha[rt] = 1.f;
      bool plain = __all(m_run[rt] > kNegInf);                     // uniform over the wavefront
      if (plain) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          p[i] = fast_exp2(__builtin_fmaf(x[i], c, -m_run[rt]));
          sum += p[i];
        }
        plain = __all(sum < 0x1p60f);                              // false for inf and NaN as well
        if (plain) l_run[rt] += sum;
      }
      if (!plain) {
        float tmax = x[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, x[i]);
        tmax = fmaxf(tmax, other_half(tmax)) * c;               // c > 0: scaling commutes with the maximum
        const float m_new = fmaxf(m_run[rt], tmax);
        const float m_use = m_new == kNegInf ? 0.f : m_new;        // nothing visible yet: every term is 0
        alpha[rt] = fast_exp2(m_run[rt] - m_use);
        sum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          p[i] = fast_exp2(__builtin_fmaf(x[i], c, -m_use));
          sum += p[i];
        }
        l_run[rt] = l_run[rt] * alpha[rt] + sum;
        m_run[rt] = m_new;
      }
      rescale = rescale || alpha[rt] != 1.f;
      pf[rt][0] = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7]));
      pf[rt][1] = make_uint4(pack_bf16(p[8], p[9]), pack_bf16(p[10], p[11]), pack_bf16(p[12], p[13]),
                             pack_bf16(p[14], p[15]));
    }
    if (__any(rescale)) {                                 // rare once the largest logits have been seen
#pragma unroll
      for (int rt = 0; rt < RTW; ++rt)
#pragma unroll
        for (int dt = 0; dt < S::kDT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[rt][dt][i] *= alpha[rt];
    }

    // O^T += V^T P^T.  Lane (col, hi) of the A operand: value column dt * 32 + col, keys as above.
    uint32_t vaddr[S::kDT];
    {
      const uint32_t vb = __builtin_amdgcn_readfirstlane(lds_offset(vbuf));
#pragma unroll
      for (int dt = 0; dt < S::kDT; ++dt) vaddr[dt] = vb + vlane[dt];
    }
    uint4 vf[S::kDT];
    if constexpr (S::kDT == 4) lds_read_vt_x4<S::kRowBytes, 0>(vf, vaddr);
    else lds_read_vt_x2<S::kRowBytes, 0>(vf, vaddr);
#pragma unroll
    for (int dt = 0; dt < S::kDT; ++dt)
#pragma unroll
      for (int rt = 0; rt < RTW; ++rt) o[rt][dt] = mma_chunk<Bf16>(vf[dt], pf[rt][0], o[rt][dt]);
    if constexpr (S::kDT == 4) lds_read_vt_x4<S::kRowBytes, 1>(vf, vaddr);
    else lds_read_vt_x2<S::kRowBytes, 1>(vf, vaddr);
#pragma unroll
    for (int dt = 0; dt < S::kDT; ++dt)
#pragma unroll
      for (int rt = 0; rt < RTW; ++rt) o[rt][dt] = mma_chunk<Bf16>(vf[dt], pf[rt][1], o[rt][dt]);
    }   // kt
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // ---- partial result of this span: (reference exponent, sum) and unnormalised O per row
  const int64_t pbase = (int64_t)bx * a.rows_pad;
#pragma unroll
  for (int rt = 0; rt < RTW; ++rt) {
    const int row = (wave * RTW + rt) * 32 + col;
    const float l_tot = l_run[rt] + other_half(l_run[rt]);
    if (hi == 0) a.part_ml[pbase + row] = make_float2(m_run[rt], l_tot);
    float* orow = a.part_o + (pbase + row) * D;
#pragma unroll
    for (int dt = 0; dt < S::kDT; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        // accumulator values 4 q4 .. 4 q4 + 3: value columns dt * 32 + 8 q4 + 4 hi + 0..3
        const float4 v4 = make_float4(o[rt][dt][4 * q4], o[rt][dt][4 * q4 + 1], o[rt][dt][4 * q4 + 2],
                                      o[rt][dt][4 * q4 + 3]);
        *reinterpret_cast<float4*>(orow + dt * 32 + 8 * q4 + 4 * hi) = v4;
      }
  }
}

// Merge of the per-item partials: out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// One thread per (row, four value columns); grid (ceil(rows * D / 4 / 256), units).
template <bool MASKED>
__global__ __launch_bounds__(256) void decode_merge_kernel(DecodeArgs a) {
  const int unit = blockIdx.y;
  const DUnit u = load_dunit<MASKED>(a, unit);
  const int D = a.head_dim;
  const int quads = D / 4;
  const int item = blockIdx.x * 256 + threadIdx.x;
  const int row = item / quads, qd = item - row * quads;
  if (row >= a.rows) return;
  const int j = row / a.group, g = row - j * a.group;
  float* dst = a.out + ((((int64_t)u.b * a.n_new + j) * a.n_q_heads + (int64_t)u.h * a.group + g) * D + qd * 4);
  const int nsp = a.item_begin[unit + 1] - a.item_begin[unit];
  const int64_t pbase = (int64_t)a.item_begin[unit] * a.rows_pad;
  const float2* ml = a.part_ml + pbase + row;
  const float* po = a.part_o + (pbase + row) * D + qd * 4;
  const int64_t ml_step = a.rows_pad, po_step = (int64_t)a.rows_pad * D;
  // one pass over the items, eight at a time (their loads issued together: a round trip per batch,
  // not per item), with a running reference exponent like the attention kernel's own
  float M = -__builtin_inff();
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
  constexpr int kBatch = 8;
  for (int s0 = 0; s0 < nsp; s0 += kBatch) {
    float2 m8[kBatch];
    float4 o8[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int sj = min(s0 + j, nsp - 1);
      m8[j] = ml[sj * ml_step];
      o8[j] = *reinterpret_cast<const float4*>(po + sj * po_step);
      if (s0 + j >= nsp) m8[j] = make_float2(-__builtin_inff(), 0.f);
    }
    float Mn = M;
#pragma unroll
    for (int j = 0; j < kBatch; ++j) Mn = fmaxf(Mn, m8[j].x);
    if (Mn != -__builtin_inff()) {
      const float keep = fast_exp2(M - Mn);              // 0 while nothing has been seen yet
      acc.x *= keep;
      acc.y *= keep;
      acc.z *= keep;
      acc.w *= keep;
      den *= keep;
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const float w = fast_exp2(m8[j].x - Mn);         // an item without visible keys has m = -inf: weight 0
        acc.x += w * o8[j].x;
        acc.y += w * o8[j].y;
        acc.z += w * o8[j].z;
        acc.w += w * o8[j].w;
        den += w * m8[j].y;
      }
      M = Mn;
    }
  }
  const float inv = den > 0.f ? 1.f / den : 0.f;          // a unit without visible keys gives zeros
  *reinterpret_cast<float4*>(dst) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

template <int D, int RTW, int W, int KT, bool MASKED>
hipError_t launch_attn(const DecodeArgs& a, hipStream_t stream) {
  constexpr int kStages = stages_for(KT);
  const size_t lds = 2 * kStages * KT * DShape<D>::kTileBytes + (MASKED ? kStages * W * 64 * sizeof(uint32_t) : 0);
  const hipError_t e = allow_lds<&decode_attn_kernel<D, RTW, W, KT, MASKED>>(lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((decode_attn_kernel<D, RTW, W, KT, MASKED>), dim3(a.max_items), dim3(W * 64), lds, stream, a);
  return hipGetLastError();
}

template <int D, bool MASKED>
hipError_t launch_typed(const DecodeArgs& a, int units, hipStream_t stream) {
  hipError_t e = hipSuccess;
  // up to 128 rows: 4 wavefronts of 32 rows, two workgroups per CU; up to 256: 8 wavefronts of 32 rows
  constexpr int kWBig = 256 / (32 * kDecodeRtw);
  if (a.rows_pad <= 128) e = launch_attn<D, 1, 4, kt_for(D, 4, kDecodeKtSmall), MASKED>(a, stream);
  else e = launch_attn<D, kDecodeRtw, kWBig, kt_for(D, kWBig, kDecodeKt), MASKED>(a, stream);
  if (e != hipSuccess) return e;
  const int items = a.rows * (D / 4);
  hipLaunchKernelGGL(decode_merge_kernel<MASKED>, dim3((items + 255) / 256, units), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_attention(const DecodeArgs& a, int units, bool masked, hipStream_t stream) {
  if (units == 0 || a.rows == 0) return hipSuccess;
  if (a.head_dim == 128) return masked ? launch_typed<128, true>(a, units, stream) : launch_typed<128, false>(a, units, stream);
  if (a.head_dim == 64) return masked ? launch_typed<64, true>(a, units, stream) : launch_typed<64, false>(a, units, stream);
  return hipErrorInvalidValue;
}

}  // namespace rfkv
