// Device side of the n-gram LM query: the view of the tables and the routine that builds one
// vocabulary-sized row of LM scores in LDS (used by the stand-alone kernel and by the launches
// of the decoder that carry LM rows as extra blocks).
#pragma once
#include "device_utils.h"

namespace rb {

__host__ __device__ inline uint64_t lm_mix(uint64_t x) {
  x ^= x >> 30;
  x *= 0xbf58476d1ce4e5b9ull;
  x ^= x >> 27;
  x *= 0x94d049bb133111ebull;
  x ^= x >> 31;
  return x;
}

// key of a context of j tokens, newest[0] = most recent token
__host__ __device__ inline uint64_t lm_key(const int *newest, int j, int bits) {
  uint64_t key = (uint64_t)j;
  for (int i = 0; i < j; ++i) key |= (uint64_t)(newest[i] + 1) << (4 + bits * i);
  return key;
}

struct LmView {
  const uint64_t *ht_key;
  const int *ht_val;
  const float *ctx_bo;
  const int *ctx_begin, *ctx_count;
  const int *succ_tok;
  const float *succ_p;
  const float *uni;
  uint32_t ht_mask;
  int order, V, bits;
};

// LDS a block needs beside the row itself
struct LmRowScratch {
  int cid[kCtxMax + 1];
  double bo[kCtxMax + 2];
};

// LM scores (natural log) of every token after hypothesis m, by one block of any size >= kCtxMax + 1 threads:
// out[m][v] = ln 10 * q(v | last min(len, order - 1) tokens), ARPA back-off.  row: V floats of LDS.
__device__ __forceinline__ void lm_row_block(const LmView &lm, const int *__restrict__ ctx, const int *__restrict__ len,
                                             float *__restrict__ out, int m, float *row, LmRowScratch &sc) {
  const int tid = threadIdx.x, nthreads = blockDim.x;
  int toks[kCtxMax];
  int have = 0;
#pragma unroll
  for (int i = 0; i < kCtxMax; ++i) {
    toks[i] = ctx[m * kCtxMax + i];
    if (toks[i] >= 0 && have == i) have = i + 1;
  }
  int jmax = lm.order - 1 < have ? lm.order - 1 : have;
  if (len && len[m] < jmax) jmax = len[m];
  if (tid >= 1 && tid <= jmax) {
    const uint64_t key = lm_key(toks, tid, lm.bits);
    uint32_t slot = (uint32_t)lm_mix(key) & lm.ht_mask;
    int cid = -1;
    for (;;) {
      const uint64_t k = lm.ht_key[slot];
      if (k == key) {
        cid = lm.ht_val[slot];
        break;
      }
      if (k == 0) break;
      slot = (slot + 1) & lm.ht_mask;
    }
    sc.cid[tid] = cid;
  }
  __syncthreads();
  if (tid == 0) {
    // bo[j] = sum of back-off weights of the contexts longer than j
    double acc = 0.0;
    sc.bo[jmax] = 0.0;
    for (int j = jmax; j >= 1; --j) {
      acc += sc.cid[j] >= 0 ? (double)lm.ctx_bo[sc.cid[j]] : 0.0;
      sc.bo[j - 1] = acc;
    }
  }
  __syncthreads();
  const float base = (float)sc.bo[0];
  for (int v = tid; v < lm.V; v += nthreads) row[v] = lm.uni[v] + base;
  for (int j = 1; j <= jmax; ++j) {
    __syncthreads();
    const int cid = sc.cid[j];
    if (cid < 0) continue;
    const int beg = lm.ctx_begin[cid], cnt = lm.ctx_count[cid];
    const float add = (float)sc.bo[j];
    for (int i = tid; i < cnt; i += nthreads) row[lm.succ_tok[beg + i]] = lm.succ_p[beg + i] + add;
  }
  __syncthreads();
  const float ln10 = 2.302585092994046f;
  for (int v = tid; v < lm.V; v += nthreads) store_through(out + (size_t)m * lm.V + v, row[v] * ln10);
}

}  // namespace rb
