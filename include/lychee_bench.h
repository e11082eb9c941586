/*
 * lychee_bench.h -- measurement aids of liblychee.  NOT part of the decode path and not needed by
 * any caller of lychee.h: a benchmark uses them to time one kernel of a step by itself and to
 * quote what this GPU's memory delivers beside its published peak.  They live in one translation
 * unit of the library (csrc/lc_bench.hip) and keep no state in the index handle.
 */
#ifndef LYCHEE_BENCH_H
#define LYCHEE_BENCH_H

#include "lychee.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Launches only the second kernel of lc_decode_step (selection + attention) for callers who want
 * to time it alone.  It takes the chunk score keys that the previous lc_decode_step with the SAME
 * query, index, budget and workspace left in the workspace: calling it in any other situation
 * gives undefined results (never a fault: every access is range-checked as in lc_decode_step).
 * Arguments, checks and error codes as lc_decode_step without the chunk list outputs;
 * LC_ERR_CAPACITY if the index is too large for lc_decode_step to run as two kernels. */
int lc_bench_select_attend(const lc_index* idx, const void* q, const void* K, const void* V,
                           const int64_t kv_strides[3], int H_q, int budget,
                           float* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/* Reads `bytes` bytes (a multiple of 16, from a 16-byte aligned device pointer) once with plain
 * streaming loads, so that a benchmark can quote the read bandwidth this GPU reaches.  `sink`
 * (device, at least 2048 words; `sink_words` says how many there are) receives one folded word per
 * workgroup.  LC_ERR_INVALID_ARG for a null or misaligned pointer or a size that is 0 or not a
 * multiple of 16, LC_ERR_WORKSPACE_TOO_SMALL for a short sink. */
int lc_bench_read_sweep(const void* src, size_t bytes, uint32_t* sink, size_t sink_words, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LYCHEE_BENCH_H */
