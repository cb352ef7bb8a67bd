/*
 * tsdg_probe.h -- measurement probes of the MI355X library.  NOT part of the method's boundary
 * (include/tsdg_ann.h): two kernels with nothing of the search or the build in them, which the
 * benchmark times to learn what this GPU sustains on the access shape of search step S5 (random
 * whole-row gathers) and on the instruction mix of the k-NN contraction (matrix-core instructions
 * on register operands).  They live in the same shared library and follow its conventions (device
 * pointers, status codes, asynchronous on `stream`).
 */
#ifndef TSDG_PROBE_H
#define TSDG_PROBE_H

#include "tsdg_ann.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement probe, not a step of the method: gathers n rows of row_bytes bytes (a multiple of 16,
 * at most 8192) from base[N rows] (device, 16-byte aligned) at ids[n] (device; an id >= N reads row
 * N-1) with the access shape of search step S5 (Alg. 2's distance step) and writes one xor-folded
 * word per row to out[n] (device).  Asynchronous on `stream`.  Timing it gives the random-row
 * bandwidth this GPU reaches with no search logic around the loads. */
ann_status ann_probe_gather(const void* base, int64_t N, int row_bytes, const uint32_t* ids, int64_t n,
                            uint32_t* out, void* stream);

/* Measurement probe, not a step of the method: `blocks` workgroups of 4 wavefronts each issue
 * 4 * iters matrix-core instructions on constant register fragments, with no memory access in
 * the loop (kind 0: v_mfma_i32_32x32x32_i8, 65,536 operations each; kind 1:
 * v_mfma_f32_32x32x16_bf16, 32,768 each), and write one float per wavefront to out[4 * blocks]
 * (device): 4 * iters * 32 (kind 0) or 4 * iters * 16 (kind 1).  Kinds 2 and 3 are kinds 0 and
 * 1 with pseudo-random fragments instead of ones (the same instructions; more wires toggle, so
 * more power is drawn and the sustained rate falls; out then holds data-dependent sums).  Timing
 * it gives the rate the matrix cores sustain on this GPU with nothing else in the way, against
 * which the k-NN contraction of the build (the exact k-NN graph under Sec. 3's diversification)
 * is read.  1 <= blocks <= 2^20, 1 <= iters <= 100000.  Asynchronous on `stream`. */
ann_status ann_probe_mfma(int kind, int blocks, int iters, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TSDG_PROBE_H */
