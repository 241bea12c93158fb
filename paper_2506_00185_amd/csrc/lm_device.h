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

// One slot of the open-addressing table: the context's key (0: empty slot) with everything a query needs of the
// context beside it, so that one round trip to memory both identifies the context and describes it.
struct alignas(32) LmSlot {
  uint64_t key;
  int begin, count;  // its successors: succ_tok / succ_p [begin, begin + count)
  float backoff;     // log10
  int pad[3];
};

struct LmView {
  const LmSlot *slots;
  const int *succ_tok;
  const float *succ_p;
  const float *uni;
  uint32_t ht_mask;
  int order, V, bits;
};

// What a query needs of the context of j tokens: its successors and its back-off weight (count 0, weight 0: the
// context is not in the model, or the hypothesis has fewer than j tokens)
struct alignas(16) LmCtxRec {
  int begin, count;
  float backoff;
  int pad;
};

// LDS a block needs beside the row itself
struct LmRowScratch {
  LmCtxRec rec[kCtxMax + 1];
};

constexpr int kLmProbe = 4;  // slots of a probe sequence read per round trip
constexpr int kLmUni = 4;  // unigram values a thread holds in registers (V <= kLmUni * threads; beyond that: read later)

// The record of the context made of the newest j tokens of a hypothesis (toks[0] = most recent; `have` of them usable)
__device__ __forceinline__ LmCtxRec lm_probe(const LmView &lm, const int *toks, int j, int have) {
  LmCtxRec r{0, 0, 0.f, 0};
  if (j > have) return r;
  const uint64_t key = lm_key(toks, j, lm.bits);
  uint32_t slot = (uint32_t)lm_mix(key) & lm.ht_mask;
  for (;;) {
    // kLmProbe slots of the probe sequence are requested at once ((key, begin, count) and the back-off weight of
    // each): with the table a quarter full at most, a second round trip is rare, also for a context that is not
    // in the model, whose search ends at the first empty slot
    uint4 head[kLmProbe];
    float w[kLmProbe];
#pragma unroll
    for (int q = 0; q < kLmProbe; ++q) {
      const LmSlot *p = lm.slots + ((slot + q) & lm.ht_mask);
      head[q] = *reinterpret_cast<const uint4 *>(p);
      w[q] = p->backoff;
    }
#pragma unroll
    for (int q = 0; q < kLmProbe; ++q) {
      const uint64_t k = (uint64_t)head[q].x | (uint64_t)head[q].y << 32;
      if (k == key) {
        r.begin = (int)head[q].z;
        r.count = (int)head[q].w;
        r.backoff = w[q];
        return r;
      }
      if (k == 0) return r;
    }
    slot = (slot + kLmProbe) & lm.ht_mask;
  }
}

// tokens of hypothesis m's history into toks (newest first); returns how many of them a query may use
__device__ __forceinline__ int lm_history(const LmView &lm, const int *__restrict__ ctx, const int *__restrict__ len,
                                          int m, int *toks) {
  int have = 0;
#pragma unroll
  for (int i = 0; i < kCtxMax; ++i) {
    toks[i] = ctx[m * kCtxMax + i];
    if (toks[i] >= 0 && have == i) have = i + 1;
  }
  int jmax = lm.order - 1 < have ? lm.order - 1 : have;
  if (len && len[m] < jmax) jmax = len[m];
  return jmax;
}

__device__ __forceinline__ void lm_unigrams(const LmView &lm, float *uni) {
#pragma unroll
  for (int q = 0; q < kLmUni; ++q) {
    const int v = threadIdx.x + q * blockDim.x;
    uni[q] = lm.uni[v < lm.V ? v : 0];
  }
}

// The row of hypothesis m from the records of its contexts (r[1 .. order - 1], in every thread's registers) and the
// unigram values requested earlier: out[m][v] = ln 10 * q(v | history).  The first successors of every context are
// requested together; only the writes into the row go context by context, shortest first (a longer context overrides).
__device__ __forceinline__ void lm_row_finish(const LmView &lm, const LmCtxRec *r, const float *uni,
                                              float *__restrict__ out, int m, float *row) {
  const int tid = threadIdx.x, nthreads = blockDim.x, nj = lm.order - 1;
  // bo[j] = sum of back-off weights of the contexts longer than j
  double bo[kCtxMax + 1];
  {
    double acc = 0.0;
#pragma unroll
    for (int j = kCtxMax; j >= 1; --j) {
      bo[j] = acc;
      if (j <= nj) acc += (double)r[j].backoff;
    }
    bo[0] = acc;
  }
  int st[kCtxMax + 1];
  float sp[kCtxMax + 1];
#pragma unroll
  for (int j = 1; j <= kCtxMax; ++j) {
    const bool ok = j <= nj && tid < r[j].count;
    st[j] = ok ? lm.succ_tok[r[j].begin + tid] : -1;
    sp[j] = ok ? lm.succ_p[r[j].begin + tid] : 0.f;
  }
  const float base = (float)bo[0];
#pragma unroll
  for (int q = 0; q < kLmUni; ++q) {
    const int v = tid + q * nthreads;
    if (v < lm.V) row[v] = uni[q] + base;
  }
  for (int v = tid + kLmUni * nthreads; v < lm.V; v += nthreads) row[v] = lm.uni[v] + base;
#pragma unroll
  for (int j = 1; j <= kCtxMax; ++j) {
    if (j > nj) break;
    __syncthreads();
    const float add = (float)bo[j];
    if (st[j] >= 0) row[st[j]] = sp[j] + add;
    const int beg = r[j].begin, cnt = r[j].count;
    for (int i = tid + nthreads; i < cnt; i += nthreads) row[lm.succ_tok[beg + i]] = lm.succ_p[beg + i] + add;
  }
  __syncthreads();
  const float ln10 = 2.302585092994046f;
  for (int v = tid; v < lm.V; v += nthreads) store_through(out + (size_t)m * lm.V + v, row[v] * ln10);
}

// LM scores (natural log) of every token after hypothesis m, by one block of any size >= kCtxMax + 1 threads:
// out[m][v] = ln 10 * q(v | last min(len, order - 1) tokens), ARPA back-off.  row: V floats of LDS.
// The chain of dependent loads is kept short: the unigram row is requested before anything else, and thread j probes
// the hash table for the context of j tokens, whose slot holds all a query needs of it (the contexts in parallel).
__device__ __forceinline__ void lm_row_block(const LmView &lm, const int *__restrict__ ctx, const int *__restrict__ len,
                                             float *__restrict__ out, int m, float *row, LmRowScratch &sc) {
  const int tid = threadIdx.x;
  int toks[kCtxMax];
  const int jmax = lm_history(lm, ctx, len, m, toks);
  float uni[kLmUni];
  lm_unigrams(lm, uni);
  if (tid >= 1 && tid <= kCtxMax) sc.rec[tid] = lm_probe(lm, toks, tid, jmax);
  __syncthreads();
  LmCtxRec r[kCtxMax + 1];
#pragma unroll
  for (int j = 1; j <= kCtxMax; ++j) r[j] = sc.rec[j];
  lm_row_finish(lm, r, uni, out, m, row);
}

}  // namespace rb
