// n-gram LM on the device: interface between the LM translation unit and the decoder.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/rnnt_beam.h"
#include "lm_device.h"

namespace rb {
int lm_vocab(const rnnt_lm_t *lm);
int lm_order(const rnnt_lm_t *lm);
// a number no other LM created in this process has had (graphs that captured an LM's tables are keyed by it)
uint64_t lm_id(const rnnt_lm_t *lm);
// the tables of an LM as kernel arguments (for launches that carry LM rows as extra blocks)
LmView lm_view(const rnnt_lm_t *lm);
// LM scores (natural log) of every token after each of M hypotheses.
// ctx [M][kCtxMax] most recent token first (-1 = none), len [M] transcript lengths (NULL: derive from ctx),
// out [M][V].  done (nullable): device word; the kernel returns at once when it is non-zero.
void lm_launch_rows(const rnnt_lm_t *lm, const int *ctx, const int *len, float *out, int M, const int *done,
                    hipStream_t s);
}  // namespace rb
