/*
 * nimble_probe.h - measurement-only entry points of the library: not part of the method and not
 * needed by a caller of the dynamic-shape path (include/nimble.h).  The benchmark, the tuning
 * script and the tests use them: a dense call pinned to one member of the kernel family (for
 * the tuning procedure and the dispatch ablation of Section 3.5 and Section 5.3), and two
 * calibration probes that show what this GPU sustains next to the nominal peaks.
 * Conventions as in nimble.h.
 */
#ifndef NIMBLE_PROBE_H_
#define NIMBLE_PROBE_H_

#include "nimble.h"

#ifdef __cplusplus
extern "C" {
#endif

/* nimble_dense_dyn with the dispatch decision taken by the caller: `force_variant` as in
 * nimble_dense_plan (NIMBLE_VAR_AUTO = the dispatch function decides, i.e. nimble_dense_dyn).
 * NIMBLE_ERR_ARG when that variant cannot run the shape, NIMBLE_ERR_WORKSPACE when a forced K
 * split does not fit the workspace. */
int nimble_dense_variant_dyn(const void* x, const void* w, const void* bias, void* y, int64_t M,
                             int64_t N, int64_t K, int epilogue, int out_dtype, int force_variant,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Register-only bf16 MFMA loop: 256 workgroups of 4 * waves_per_simd waves (1, 2 or 4), each
 * wave issuing iters * (64 / waves_per_simd) independent MFMAs of 16x16x32 back to back.  seed: device, 64 KiB of bf16 operand data (any
 * finite values); sink: device, 1 MiB, overwritten.  *flops receives the flop count of the
 * launch.  Asynchronous on `stream`; the caller times it. */
int nimble_probe_mfma_bf16(const void* seed, void* sink, int waves_per_simd, int iters,
                           double* flops, void* stream);

/* Plain streaming read of `bytes` (a multiple of 16) from buf (device, 16-byte aligned).
 * sink: device, 16 bytes.  Asynchronous on `stream`; the caller times it. */
int nimble_probe_hbm_read(const void* buf, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NIMBLE_PROBE_H_ */
