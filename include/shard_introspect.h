/*
 * Introspection of libshard's launch decisions, for tests and reports.  Host-only: nothing
 * here touches a GPU.  The library has several tile / pipeline variants of each projection
 * kernel and picks one per launch from the shape; these calls run the very selection code
 * the launchers run, so a test can state which variant a shape lands on and which variants a
 * set of shapes covers.  (The projections are the steps a2, a6, a8, a9 of the decoder layer -
 * QKV, O, gate/up, down - of the prefill and of the autoregressive phase, Sec. 2 "Generative
 * LLM Inference".)
 */
#ifndef SHARD_INTROSPECT_H
#define SHARD_INTROSPECT_H

#include <stdint.h>

#include "shard.h"

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SHARD_FAMILY_PREFILL_GEMM = 0,  /* MFMA GEMMs of shard_prefill */
    SHARD_FAMILY_DECODE_STREAM = 1, /* streaming projections of shard_decode (fp32 activations) */
    SHARD_FAMILY_DECODE_MFMA = 2    /* matrix-core projections of shard_decode (16-bit weights, more than 4 sequences) */
};

/* Name of variant `index` of a family; NULL past the end of the family's table (so a caller
 * enumerates a family by counting up from 0 until NULL) or for an unknown family. */
const char *shard_variant_name(int32_t family, int32_t index);

/* The variant shard_prefill takes for the projection with an [N, K] weight matrix and M = B*T
 * activation rows.  weight_dtype: SHARD_F32 or SHARD_BF16.  residual_epilogue != 0 for the O
 * and down projections (only they may be split along K); *k_slices (may be NULL) receives
 * the number of K slices (1 = not split).  Returns the index into SHARD_FAMILY_PREFILL_GEMM,
 * or -1 on bad arguments. */
int32_t shard_variant_prefill_gemm(int32_t weight_dtype, int32_t M, int32_t N, int32_t K,
                                   int32_t residual_epilogue, int32_t *k_slices);

/* The variant shard_decode takes for the projection with an [N, K] weight matrix in a step of
 * B sequences of the given model.  *family receives SHARD_FAMILY_DECODE_STREAM or
 * SHARD_FAMILY_DECODE_MFMA, *rows_per_pass the activation rows one launch carries (a step of
 * more rows makes several passes over the weights), *rows_per_workgroup the weight rows a
 * workgroup owns (0 when the variant's name states it).  Returns the index into *family, or
 * -1 on bad arguments. */
int32_t shard_variant_decode_linear(const shard_model_cfg *model, int32_t B, int32_t N, int32_t K,
                                    int32_t *family, int32_t *rows_per_pass, int32_t *rows_per_workgroup);

/* For tests of the error path only: on != 0 makes the library behave as if a one-time kernel
 * attribute call (the opt-in to more than 64 KB of LDS) had failed - every following
 * shard_prefill / shard_decode / shard_create then enqueues its work, finds the failure in its
 * final check and returns SHARD_E_HIP with its state rolled back - and on == 0 takes the
 * injected failure away again.  No kernel misbehaves because of it. */
void shard_test_inject_launch_error(int32_t on);

#ifdef __cplusplus
}
#endif
#endif /* SHARD_INTROSPECT_H */
