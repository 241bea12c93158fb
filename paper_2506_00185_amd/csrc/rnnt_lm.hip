// n-gram LM for shallow fusion, queried for the whole vocabulary at once (late
// pruning needs LM scores of every token for every hypothesis: Sec. 2.3 of the
// paper, "Early/late pruning").  The paper cites an external GPU n-gram LM and
// does not describe its layout; the structure here is this library's own:
//   * every token sequence that is the history of a stored n-gram, or is itself
//     a stored n-gram of order < max order, is a "context" with a back-off
//     weight and a list of successors (token, log10 p);
//   * contexts are found through an open-addressing hash table keyed by the
//     exact packed token sequence (no false positives), whose 32-byte slots
//     hold the context's back-off weight and successor range beside the key;
//   * a query fills a vocabulary-sized row in LDS with the unigram scores plus
//     all back-off weights, then overwrites it level by level with the stored
//     successors of longer and longer contexts.
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

#include "lm.h"
#include "lm_device.h"

struct rnnt_lm {
  uint64_t id = 0;  // unique per created LM in this process (a later LM may reuse this one's address)
  int order = 0, V = 0, bits = 0;
  uint32_t ht_mask = 0;
  // device
  rb::LmSlot *slots = nullptr;
  int *succ_tok = nullptr;
  float *succ_p = nullptr;
  float *uni = nullptr;
  std::vector<void *> allocs;
};

namespace rb {

__global__ __launch_bounds__(256) void k_lm_rows(LmView lm, const int *__restrict__ ctx, const int *__restrict__ len,
                                                 float *__restrict__ out, int M, const int *done) {
  if (done && *reinterpret_cast<const volatile int *>(done)) return;
  extern __shared__ float row[];
  __shared__ LmRowScratch sc;
  lm_row_block(lm, ctx, len, out, blockIdx.x, row, sc);
}

int lm_vocab(const rnnt_lm_t *lm) { return lm->V; }
int lm_order(const rnnt_lm_t *lm) { return lm->order; }
uint64_t lm_id(const rnnt_lm_t *lm) { return lm->id; }

LmView lm_view(const rnnt_lm_t *lm) {
  return LmView{lm->slots, lm->succ_tok, lm->succ_p, lm->uni, lm->ht_mask, lm->order, lm->V, lm->bits};
}

void lm_launch_rows(const rnnt_lm_t *lm, const int *ctx, const int *len, float *out, int M, const int *done,
                    hipStream_t s) {
  hipLaunchKernelGGL(k_lm_rows, dim3(M), dim3(256), sizeof(float) * lm->V, s, lm_view(lm), ctx, len, out, M, done);
}

}  // namespace rb

namespace {
template <typename T>
bool lm_upload(rnnt_lm *lm, T **p, const std::vector<T> &v) {
  void *q = nullptr;
  if (hipMalloc(&q, (v.size() ? v.size() : 1) * sizeof(T)) != hipSuccess) return false;
  lm->allocs.push_back(q);
  if (v.size() && hipMemcpy(q, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return false;
  *p = static_cast<T *>(q);
  return true;
}
}  // namespace

extern "C" {

// (no exception leaves these functions: host containers that cannot grow report RNNT_E_NOMEM)
int rnnt_lm_create(int32_t order, int64_t n, const int32_t *ngram_tokens, const int8_t *ngram_order,
                   const float *log10_prob, const float *log10_backoff, int32_t V, rnnt_lm_t **out) try {
  if (out) *out = nullptr;
  if (!out || !ngram_tokens || !ngram_order || !log10_prob || !log10_backoff || order < 1 || n < 1 || V < 1)
    return RNNT_E_ARG;
  if (order - 1 > rb::kCtxMax) return RNNT_E_ARG;
  int bits = 1;
  while ((1ll << bits) <= (long long)V) ++bits;  // token + 1 in 1..V fits
  if (4 + bits * (order - 1) > 64) return RNNT_E_ARG;
  if ((size_t)V * sizeof(float) > 60 * 1024) return RNNT_E_ARG;  // the query row lives in LDS

  std::unordered_map<uint64_t, int> ctx_id;
  std::vector<float> ctx_bo;
  std::vector<int> ctx_count;
  auto get_ctx = [&](const int32_t *oldest_first, int j) {
    int newest[rb::kCtxMax];
    for (int i = 0; i < j; ++i) newest[i] = oldest_first[j - 1 - i];
    const uint64_t key = rb::lm_key(newest, j, bits);
    auto it = ctx_id.find(key);
    if (it != ctx_id.end()) return it->second;
    const int id = (int)ctx_bo.size();
    ctx_id.emplace(key, id);
    ctx_bo.push_back(0.f);
    ctx_count.push_back(0);
    return id;
  };
  std::vector<float> uni((size_t)V, -99.f);
  std::vector<int> succ_ctx((size_t)n, -1);
  for (int64_t i = 0; i < n; ++i) {
    const int o = ngram_order[i];
    const int32_t *tk = ngram_tokens + i * order;
    if (o < 1 || o > order) return RNNT_E_ARG;
    for (int j = 0; j < o; ++j)
      if (tk[j] < 0 || tk[j] >= V) return RNNT_E_ARG;
    if (o == 1) uni[tk[0]] = log10_prob[i];
    if (o <= order - 1) ctx_bo[get_ctx(tk, o)] = log10_backoff[i];
    if (o >= 2) {
      const int id = get_ctx(tk, o - 1);
      succ_ctx[i] = id;
      ctx_count[id] += 1;
    }
  }
  const int n_ctx = (int)ctx_bo.size();
  std::vector<int> ctx_begin((size_t)n_ctx + 1, 0);
  for (int i = 0; i < n_ctx; ++i) ctx_begin[i + 1] = ctx_begin[i] + ctx_count[i];
  std::vector<int> fill(ctx_begin.begin(), ctx_begin.end() - 1);
  std::vector<int> succ_tok((size_t)ctx_begin[n_ctx]);
  std::vector<float> succ_p((size_t)ctx_begin[n_ctx]);
  for (int64_t i = 0; i < n; ++i)
    if (succ_ctx[i] >= 0) {
      const int pos = fill[succ_ctx[i]]++;
      succ_tok[pos] = ngram_tokens[i * order + ngram_order[i] - 1];
      succ_p[pos] = log10_prob[i];
    }
  uint32_t size = 64;
  while (size < 4u * (uint32_t)(n_ctx + 1)) size <<= 1;  // at most a quarter full: short probe sequences
  std::vector<rb::LmSlot> slots(size);
  std::memset(slots.data(), 0, slots.size() * sizeof(rb::LmSlot));
  for (auto &kv : ctx_id) {
    uint32_t slot = (uint32_t)rb::lm_mix(kv.first) & (size - 1);
    while (slots[slot].key != 0) slot = (slot + 1) & (size - 1);
    slots[slot].key = kv.first;
    slots[slot].begin = ctx_begin[kv.second];
    slots[slot].count = ctx_count[kv.second];
    slots[slot].backoff = ctx_bo[kv.second];
  }
  rnnt_lm *lm = new (std::nothrow) rnnt_lm();
  if (!lm) return RNNT_E_NOMEM;
  static std::atomic<uint64_t> next_id{1};
  lm->id = next_id.fetch_add(1);
  lm->order = order;
  lm->V = V;
  lm->bits = bits;
  lm->ht_mask = size - 1;
  bool ok = lm_upload(lm, &lm->slots, slots) && lm_upload(lm, &lm->succ_tok, succ_tok) &&
            lm_upload(lm, &lm->succ_p, succ_p) && lm_upload(lm, &lm->uni, uni);
  if (!ok) {
    rnnt_lm_destroy(lm);
    return RNNT_E_NOMEM;
  }
  *out = lm;
  return RNNT_OK;
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_ARG;
}

int rnnt_lm_debug_query(const rnnt_lm_t *lm, const int32_t *ctx_tokens, int32_t n, float *out) try {
  if (!lm || !ctx_tokens || !out || n < 1) return RNNT_E_ARG;
  const int w = lm->order - 1;
  std::vector<int> ctx((size_t)n * rb::kCtxMax, -1);
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < w; ++j) ctx[(size_t)i * rb::kCtxMax + j] = ctx_tokens[(size_t)i * w + j];
  int *d_ctx = nullptr;
  float *d_out = nullptr;
  if (hipMalloc(reinterpret_cast<void **>(&d_ctx), ctx.size() * sizeof(int)) != hipSuccess) return RNNT_E_NOMEM;
  if (hipMalloc(reinterpret_cast<void **>(&d_out), (size_t)n * lm->V * sizeof(float)) != hipSuccess) {
    hipFree(d_ctx);
    return RNNT_E_NOMEM;
  }
  int rc = RNNT_OK;
  if (hipMemcpy(d_ctx, ctx.data(), ctx.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess) rc = RNNT_E_HIP;
  if (!rc) {
    rb::lm_launch_rows(lm, d_ctx, nullptr, d_out, n, nullptr, nullptr);
    if (hipGetLastError() != hipSuccess || hipDeviceSynchronize() != hipSuccess) rc = RNNT_E_HIP;
  }
  if (!rc && hipMemcpy(out, d_out, (size_t)n * lm->V * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
    rc = RNNT_E_HIP;
  hipFree(d_ctx);
  hipFree(d_out);
  return rc;
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_ARG;
}

void rnnt_lm_destroy(rnnt_lm_t *lm) {
  if (!lm) return;
  for (void *p : lm->allocs) hipFree(p);
  delete lm;
}

}  // extern "C"
