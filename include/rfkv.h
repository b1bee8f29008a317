/*
 * rfkv -- threshold-free KV-cache compression (ReFreeKV) for AMD MI355X (gfx950).
 *
 * C ABI of the post-prefill compression pass: for one transformer layer and a
 * packed ragged batch of prefilled sequences, score every cached position by
 * the causal softmax attention a window of the most recent queries pays to it,
 * rank the positions, apply the paper's norm-ratio budget rule and gather the
 * retained K/V rows into a ragged per-(sequence, KV head) cache.
 *
 * Conventions shared by every entry point
 *   - A *unit* is one (sequence b, KV head h), numbered u = b * n_kv_heads + h.
 *   - B = batch, n_b = tokens of sequence b, N = sum n_b, w'_b = min(window, n_b),
 *     G = n_q_heads / n_kv_heads.
 *   - "device" pointers are HIP device memory owned by the caller and must be
 *     16-byte aligned; "host" pointers are ordinary host memory.  The library
 *     never allocates, frees or retains memory and never synchronises: all work
 *     is enqueued on the HIP stream passed as `stream` (a hipStream_t; NULL is
 *     the default stream).  Buffers must stay alive until that work has run.
 *   - cu_seqlens (int32, B + 1 entries, cu[0] = 0, non-decreasing, cu[B] = N) is
 *     passed twice: a host copy, used for validation and launch geometry, and a
 *     device copy with the same contents, read by the kernels.
 *   - Every call validates its arguments on the host before touching the GPU
 *     and returns a status; nothing is enqueued unless the status is RFKV_OK.
 *     Results that depend on device data (kept counts) are never read back.
 *   - Calls that share a workspace must be ordered on one stream.
 */
#ifndef RFKV_H
#define RFKV_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define RFKV_API __attribute__((visibility("default")))
#else
#define RFKV_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rfkv_status {
  RFKV_OK = 0,
  RFKV_INVALID_ARG = 1,          /* null / misaligned pointer, inconsistent sizes or cu_seqlens   */
  RFKV_UNSUPPORTED = 2,          /* dtype, head_dim or window * G outside what the kernels cover  */
  RFKV_WORKSPACE_TOO_SMALL = 3,  /* ws_bytes < rfkv_workspace_bytes(...)                          */
  RFKV_OUTPUT_TOO_SMALL = 4,     /* a capacity the host can check is too small                    */
  RFKV_DEVICE_ERROR = 5          /* a HIP call failed; see rfkv_last_device_error()               */
} rfkv_status;

enum { RFKV_RANK_POSITION = 0, RFKV_RANK_SCORE = 1 };
enum { RFKV_DTYPE_FP32 = 0, RFKV_DTYPE_BF16 = 1 };
enum { RFKV_PER_HEAD = 0, RFKV_PER_LAYER = 1 };

/* Limits of this build. */
enum {
  RFKV_MAX_SCORE_ROWS = 512,     /* window * G (rounded up to a multiple of 32) of the streaming  */
                                 /* kernels; more rows take the wide-window path below            */
  RFKV_MAX_WIDE_ROWS = 65536,    /* window * G of the wide-window path (the paper's ablation of k */
                                 /* up to 10 % of n): bf16 with head_dim 64 or 128, fp32 with 64; */
                                 /* (window * G / 128) * (longest sequence / 512) * units must    */
                                 /* stay below 2^30, else RFKV_UNSUPPORTED                        */
  RFKV_MAX_UNITS = 65535,        /* B * n_kv_heads                                                */
  RFKV_MAX_STRIDE_TOK = 1 << 22  /* largest k_stride_tok / v_stride_tok (elements), else          */
                                 /* RFKV_UNSUPPORTED: the tile loaders of the scoring and         */
                                 /* attention kernels add up to 127 token strides in 32 bits      */
};

/*
 * Problem description.  Symbols follow the paper: `window` is its k (number of
 * last attention rows averaged into A', Sec. 3.2 "Reducing Overhead", Eq. 2),
 * `n_sink` its m (positions ranked first, Sec. 3.2 "Initial Ranking"),
 * `threshold` its T (Eq. 1; the universal value is 0.01).
 */
typedef struct rfkv_params {
  int32_t batch;            /* B >= 0                                                             */
  int32_t n_q_heads;        /* Hq, a multiple of n_kv_heads                                       */
  int32_t n_kv_heads;       /* Hkv                                                                */
  int32_t head_dim;         /* d: 64 or 128                                                       */
  int32_t window;           /* k >= 1; rows used per sequence = min(window, n_b)                  */
  int32_t n_sink;           /* m >= 0, used by RFKV_RANK_POSITION only                            */
  float   threshold;        /* T; <= 0 keeps everything, >= 1 keeps one position                  */
  int32_t rank_mode;        /* RFKV_RANK_POSITION (the paper's method) or RFKV_RANK_SCORE
                               (descending A', equal scores by ascending position; Sec. 4.4)      */
  int32_t dtype;            /* storage type of Q, K, V: RFKV_DTYPE_FP32 or RFKV_DTYPE_BF16        */
  float   softmax_scale;    /* logit scale; 0 selects 1 / sqrt(head_dim)                          */
  int32_t min_keep;         /* floor on the kept count per unit (0 = the paper's rule alone)      */
  int32_t granularity;      /* RFKV_PER_HEAD: one cut per (sequence, KV head) (Sec. 3.2, "per layer
                               and per attention head"); RFKV_PER_LAYER: one cut per (layer,
                               sequence), the norms of Eq. 1 taken over the reduced attention
                               matrix of all KV heads (Fig. 1 "per layer"; Sec. 3.3 "the stopping
                               positions of all layers"), every head keeping the same number of
                               positions: with the position ranking the same positions, with the
                               score ranking each head its own largest scores.                     */
  /* strides in elements; the head_dim axis is contiguous.  Token index is the packed index
     0..N-1 for K/V and the packed window-row index 0..sum_b w'_b - 1 for Q.                      */
  int64_t k_stride_tok, k_stride_head;
  int64_t v_stride_tok, v_stride_head;
  int64_t q_stride_row, q_stride_head;
  int64_t out_pad_rows;     /* 0: ragged output, unit u at out_offsets[u] = sum of earlier kept counts.
                               > 0: padded output (Sec. 3.3 "Running at Scale": shorter cache segments
                               are padded and masked): unit u owns rows [u * out_pad_rows, (u + 1) *
                               out_pad_rows) of k_out / v_out (and of idx), the first kept[u] of them
                               are written, the rest are left untouched; out_offsets[u] = u *
                               out_pad_rows; the mask is t < kept[u].  Must be >= the longest sequence. */
} rfkv_params;

/* Library version, major * 10000 + minor * 100 + patch. */
RFKV_API int32_t rfkv_version(void);

/* Static, human-readable name of a status code. */
RFKV_API const char* rfkv_status_string(rfkv_status status);

/* hipError_t (as int) of the most recent RFKV_DEVICE_ERROR on the calling thread, 0 if none. */
RFKV_API int32_t rfkv_last_device_error(void);

/*
 * Bytes of device scratch that rfkv_score / rfkv_select / rfkv_compress_layer need for a batch
 * with `total_tokens` = N and longest sequence `max_seqlen`.  Pure host arithmetic; returns 0 if
 * `params` is NULL or describes an unsupported problem.  The workspace contents need no
 * initialisation and carry nothing from one call to the next.
 */
RFKV_API size_t rfkv_workspace_bytes(const rfkv_params* params, int64_t total_tokens, int32_t max_seqlen);

/*
 * Scoring (Sec. 3.2 "Reducing Overhead", Eq. 2; Alg. 1 "Attention(Q[-1], K^T)").
 *   scores[h * N + cu[b] + i] = (1/G) sum_g (1/cnt_i) sum_{t : i <= n_b - w'_b + t} P[t, g, i]
 * where P[t, g, :] is the causal softmax of scale * q_{t,g} . k_i over the keys i the window row
 * t (absolute position n_b - w'_b + t) can see, and cnt_i = min(w'_b, n_b - i) is the number of
 * window rows that see key i.
 *   q_win   device, [sum_b w'_b, Hq, d] through q_stride_*: the (post-RoPE) queries of the last
 *           w'_b positions of each sequence, sequences packed in batch order
 *   k       device, [N, Hkv, d] through k_stride_*
 *   scores  device, float [Hkv, N], written in full
 *   ws      device scratch of at least rfkv_workspace_bytes(...)
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; softmax and the
 * reductions run in fp32.
 */
RFKV_API rfkv_status rfkv_score(const rfkv_params* params, const void* q_win, const void* k,
                       const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                       float* scores, void* ws, size_t ws_bytes, void* stream);

/*
 * Ranking + budget rule (Sec. 3.2 "Initial Ranking", Eq. 1; Sec. 3.3, Eq. 3).  For each unit, with
 * s[r] the score at rank r and P_i = sum_{r <= i} s[r]^2, F^2 = P_n:
 *   i* = min { i : 1 - sqrt(P_i) / F < T }   (n if there is none or F = 0),
 *   kept = min(n, max(i*, min_keep)),
 * and the retained set is ranks 1..kept.  Both rankings are deterministic (two runs give the same
 * bits): the position ranking adds fp64 masses in a fixed order, the score ranking accumulates P
 * exactly (integer fixed point scaled by F^2, resolution 2^-60), so no reduction order enters.
 *   scores       device, float [Hkv, N] as written by rfkv_score
 *   kept         device, int32 [B * Hkv]
 *   out_offsets  device, int64 [B * Hkv + 1], exclusive prefix sum of kept
 *   idx          device, int32: retained positions relative to their sequence start, ascending,
 *                unit u at idx[out_offsets[u] .. out_offsets[u] + kept[u]).  Capacity the caller must
 *                provide: N * Hkv entries with the ragged layout, B * Hkv * out_pad_rows entries with
 *                the padded one (out_pad_rows > 0; never less than N * Hkv, since a slot holds the
 *                longest sequence); nothing is written beyond that
 */
RFKV_API rfkv_status rfkv_select(const rfkv_params* params, const float* scores,
                        const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                        int32_t* kept, int64_t* out_offsets, int32_t* idx,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * Compaction (Alg. 1, "Compress K / V by R"): k_out[out_offsets[u] + t] = K[cu[b] + idx[...], h]
 * and the same for V, rows in ascending original position, moved bit for bit.
 *   kept, out_offsets, idx   device, as produced by rfkv_select
 *   k_out, v_out             device, [out_capacity_rows, d] contiguous.  Rows at or beyond
 *                            out_capacity_rows are not written; N * Hkv rows always suffice.
 */
RFKV_API rfkv_status rfkv_compact(const rfkv_params* params, const void* k, const void* v,
                         const int32_t* cu_seqlens_host, const int32_t* cu_seqlens_dev,
                         const int32_t* kept, const int64_t* out_offsets, const int32_t* idx,
                         void* k_out, void* v_out, int64_t out_capacity_rows, void* stream);

/*
 * One layer of Alg. 1's loop body: score -> rank -> budget rule -> compaction, enqueued
 * back to back with no host synchronisation.  Arguments as above; `scores_opt` may be NULL
 * (scores then live in the workspace only) and `idx_opt` may be NULL (indices not reported);
 * otherwise idx_opt has the capacity rfkv_select asks for, and like the K / V rows its entries at
 * or beyond out_capacity_rows are not written.
 * Layers that keep their whole cache (the paper keeps the first two, Sec. 3.3 "Retaining Bottom
 * Layers") are either not passed to the library at all, or passed with threshold <= 0 and
 * scores_opt NULL: nothing is scored then (q_win may be NULL), every position is kept, and the
 * call only re-lays the cache out into the same ragged per-unit form as the other layers'.
 */
RFKV_API rfkv_status rfkv_compress_layer(const rfkv_params* params, const void* q_win, const void* k,
                                const void* v, const int32_t* cu_seqlens_host,
                                const int32_t* cu_seqlens_dev, float* scores_opt, int32_t* kept,
                                int64_t* out_offsets, int32_t* idx_opt, void* k_out, void* v_out,
                                int64_t out_capacity_rows, void* ws, size_t ws_bytes, void* stream);

/*
 * Alg. 1's loop over the layers of a prefilled model in one call: layer l of n_layers has its own
 * queries, cache and outputs, q_win[l], k[l], v[l], kept[l], ... (host arrays of n_layers device
 * pointers each; scores_opt and idx_opt may be NULL as a whole), and all layers share params, the
 * strides in it, cu_seqlens and out_capacity_rows.  The result for every layer is what
 * rfkv_compress_layer gives for it, up to the rounding of the rows' softmax normalisers (they are
 * folded from longer spans of keys here; scores agree to a few units in the last place).  Layers the
 * caller wants to keep whole (the paper keeps the first two, Sec. 3.3 "Retaining Bottom Layers") are
 * simply not passed.
 * Having all layers at once lets the library run the steps of different layers side by side: with the
 * position ranking, one cut per unit and up to 128 score rows per KV head, one launch works on the
 * statistics pass of layer j, the reduction pass and the cut of layer j - 1 and the compaction of
 * layer j - 2 (they do not depend on each other).  Other problems run layer after layer.
 *   ws   device scratch of at least rfkv_layers_workspace_bytes(params, n_layers, N, longest sequence)
 * Errors as rfkv_compress_layer.
 */
RFKV_API size_t rfkv_layers_workspace_bytes(const rfkv_params* params, int32_t n_layers, int64_t total_tokens,
                                            int32_t max_seqlen);
RFKV_API rfkv_status rfkv_compress_layers(const rfkv_params* params, int32_t n_layers, const void* const* q_win,
                                const void* const* k, const void* const* v, const int32_t* cu_seqlens_host,
                                const int32_t* cu_seqlens_dev, float* const* scores_opt, int32_t* const* kept,
                                int64_t* const* out_offsets, int32_t* const* idx_opt, void* const* k_out,
                                void* const* v_out, int64_t out_capacity_rows, void* ws, size_t ws_bytes,
                                void* stream);

/*
 * rfkv_compress_layer for callers that cannot allocate device memory: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  They have no workspace to hand
 * over, so this entry point takes none: its scratch is a fixed array of RFKV_STATIC_SCRATCH_BYTES
 * that is part of the library's device image (each GPU the library runs on holds its own copy until
 * the process ends).  Nothing is allocated or freed, by the library or by anything it calls.
 *   - The device of `stream` must be the current device.
 *   - RFKV_WORKSPACE_TOO_SMALL if the batch needs more scratch than RFKV_STATIC_SCRATCH_BYTES
 *     (rfkv_workspace_bytes(params, N, longest sequence) bounds the need from above; a 32768-token
 *     Llama3-8B layer needs 2.6 MB, a 131072-token one 8.5 MB).  Nothing is enqueued then.
 *   - All calls on one GPU share that GPU's array: calls that may overlap (different streams,
 *     different host threads) race on it.  Order them on one stream.
 * Arguments, outputs and every other error as rfkv_compress_layer.
 */
enum { RFKV_STATIC_SCRATCH_BYTES = 16 * 1024 * 1024 };
RFKV_API rfkv_status rfkv_compress_layer_static(const rfkv_params* params, const void* q_win, const void* k,
                                const void* v, const int32_t* cu_seqlens_host,
                                const int32_t* cu_seqlens_dev, float* scores_opt, int32_t* kept,
                                int64_t* out_offsets, int32_t* idx_opt, void* k_out, void* v_out,
                                int64_t out_capacity_rows, void* stream);

/*
 * Scoring and the fused pass when the prefill already has the window rows' softmax normalisers.
 * A causal attention forward pass returns, next to its output, the log-sum-exp of every query
 * row: lse[t, hq] = ln sum_{i <= pos(t)} exp(scale * q[t, hq] . k[i]).  For the window rows this is
 * exactly what the first of the two passes over K computes (the denominators of the softmax rows
 * that Eq. 2 averages, Sec. 3.2 "Reducing Overhead"); given it, K is read once.
 *   lse_win  device, float32 [sum_b min(window, n_b)][n_q_heads], contiguous, rows in the order of
 *            q_win (natural logarithm, of the logits scaled by the same softmax_scale; causal).
 * Everything else as in rfkv_score / rfkv_compress_layer, including workspace size and errors;
 * RFKV_INVALID_ARG also when lse_win is null or not 4-byte aligned.  The scores are
 * sum over rows of exp(logit - lse): they are only as good as the lse handed in.
 */
RFKV_API rfkv_status rfkv_score_lse(const rfkv_params* params, const void* q_win, const float* lse_win,
                                    const void* k, const int32_t* cu_seqlens_host,
                                    const int32_t* cu_seqlens_dev, float* scores, void* ws, size_t ws_bytes,
                                    void* stream);
RFKV_API rfkv_status rfkv_compress_layer_lse(const rfkv_params* params, const void* q_win, const float* lse_win,
                                    const void* k, const void* v, const int32_t* cu_seqlens_host,
                                    const int32_t* cu_seqlens_dev, float* scores_opt, int32_t* kept,
                                    int64_t* out_offsets, int32_t* idx_opt, void* k_out, void* v_out,
                                    int64_t out_capacity_rows, void* ws, size_t ws_bytes, void* stream);

/*
 * Decode attention over the compacted cache -- the consumer of Alg. 1's compressed K / V (the
 * paper's efficiency comparison, Sec. 4.3, is between attention over the pruned and over the full
 * cache).  n_new new queries per sequence attend to every retained position of their sequence
 * and to nothing else (no attention among the new positions):
 *   out[b, j, hq, :] = softmax_i(scale * q_new[b, j, hq] . k_c[o_u + i]) . v_c[o_u + i],
 *   u = b * n_kv_heads + hq / G, o_u = out_offsets[u], i in [0, kept_u).
 * bf16 storage only (RFKV_UNSUPPORTED otherwise); n_new * G <= RFKV_MAX_DECODE_ROWS.
 *   q_new        device, bf16 [B, n_new, Hq, d] contiguous
 *   k_c, v_c     device, bf16 [rows, d] contiguous as written by rfkv_compact / rfkv_compress_layer
 *   out_offsets  device, int64 [B * Hkv + 1] as written by rfkv_select / rfkv_compress_layer
 *   kept_opt     device, int32 [B * Hkv] as written by the same call, or NULL.  With the ragged layout
 *                a unit's rows are out_offsets[u] .. out_offsets[u + 1] and kept_opt adds nothing; with
 *                the padded layout (out_pad_rows > 0) only the first kept[u] rows of a unit's slot hold
 *                data, so kept_opt is required (RFKV_INVALID_ARG without it) and bounds every unit
 *   out          device, float [B, n_new, Hq, d]; a unit with no rows gives zeros
 *   ws           device scratch of at least rfkv_decode_workspace_bytes(...)
 * cu_seqlens_host bounds the unit lengths (kept_u <= n_b) for the launch geometry; the kept
 * counts themselves are read on the device only.  Probabilities are rounded to bf16 for the
 * value product (fp32 accumulation), like the stored values themselves.
 */
enum { RFKV_MAX_DECODE_ROWS = 256 };
RFKV_API size_t rfkv_decode_workspace_bytes(const rfkv_params* params, int32_t n_new, int32_t max_seqlen);
RFKV_API rfkv_status rfkv_decode_attention(const rfkv_params* params, const void* q_new, int32_t n_new,
                                  const void* k_c, const void* v_c, const int32_t* cu_seqlens_host,
                                  const int64_t* out_offsets, const int32_t* kept_opt, float* out, void* ws,
                                  size_t ws_bytes, void* stream);

/*
 * The same attention over the uncompressed cache with the evicted positions masked to -inf: the
 * baseline rfkv_decode_attention is timed against, and by the permutation invariance of attention
 * the same result.  k, v through params' k_/v_stride_*; keep_mask device, uint8 [Hkv, N], non-zero
 * = retained.  Other arguments as above.
 */
RFKV_API rfkv_status rfkv_masked_attention(const rfkv_params* params, const void* q_new, int32_t n_new,
                                  const void* k, const void* v, const int32_t* cu_seqlens_host,
                                  const int32_t* cu_seqlens_dev, const uint8_t* keep_mask, float* out,
                                  void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RFKV_H */
