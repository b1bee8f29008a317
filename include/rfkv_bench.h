/*
 * rfkv -- measurement aid, kept apart from the library's interface (rfkv.h): it serves the
 * benchmark's per-kernel roofline figures and nothing else, and unlike every entry point of
 * rfkv.h it synchronises the stream.
 */
#ifndef RFKV_BENCH_H
#define RFKV_BENCH_H

#include "rfkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * rfkv_compress_layer (Alg. 1's loop body, see rfkv.h) with a HIP event recorded
 * on `stream` after each kernel.  Synchronises the stream before returning and fills
 * kernel_ms_host[RFKV_NUM_KERNELS] (host memory) with the elapsed milliseconds between
 * consecutive events, in launch order: score statistics, statistics merge, score reduction,
 * selection, compaction.  Outputs are identical to rfkv_compress_layer's.
 */
enum { RFKV_NUM_KERNELS = 5 };
RFKV_API rfkv_status rfkv_compress_layer_timed(const rfkv_params* params, const void* q_win, const void* k,
                                const void* v, const int32_t* cu_seqlens_host,
                                const int32_t* cu_seqlens_dev, float* scores_opt, int32_t* kept,
                                int64_t* out_offsets, int32_t* idx_opt, void* k_out, void* v_out,
                                int64_t out_capacity_rows, void* ws, size_t ws_bytes, void* stream,
                                float* kernel_ms_host);

#ifdef __cplusplus
}
#endif
#endif /* RFKV_BENCH_H */
