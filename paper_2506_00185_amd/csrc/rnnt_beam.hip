// Host side of the rnnt_beam C ABI: weight packing, workspace, the step loop
// (captured as a HIP graph), results.  See include/rnnt_beam.h for the contract.
#include "../../include/rnnt_beam.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <tuple>
#include <type_traits>
#include <vector>

#include "gemm.h"
#include "kernels.h"
#include "kernels_big.h"
#include "kernels_persistent.h"
#include "lm.h"

using namespace rb;

// Workspace of rnnt_beam_decode_static: one array per GPU for the life of the process.  In host code the name
// below is only a handle for the symbol look-up; the device address of each GPU's copy is kept in g_scratch_ptr.
constexpr size_t kScratchBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static char *g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

namespace {

thread_local std::string g_create_error;

inline float host_bf16_round(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return x;
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  memcpy(&x, &u, 4);
  return x;
}

struct KernelTimer {
  const char *name;
  float ms;
  int calls;
};

enum {
  KT_ENCPROJ = 0, KT_INIT, KT_JOINT, KT_SELECT, KT_LM, KT_LSTM, KT_PREDPROJ, KT_BACKTRACE, KT_JOINTBIG, KT_ROWSELECT,
  KT_STATELESS, KT_UTTSELECT, KT_COUNT
};
const char *kKernelNames[KT_COUNT] = {"k_gemm_tiled(enc_proj)", "k_init",      "k_step_main", "k_select",    "k_lm_rows",
                                      "k_lstm_pointwise",    "k_pred_proj", "k_backtrace", "k_joint_big", "k_row_select",
                                      "k_stateless_pre",     "k_utt_select"};

// Device memory a decode works in beyond its inputs and outputs, laid out for given maxima.  The handle owns one
// (a single allocation made at create); the allocation-free entry point lays one out in the static array.
struct Workspace {
  float *f_proj = nullptr, *pre = nullptr, *pre2 = nullptr, *h[2] = {nullptr, nullptr}, *c[2] = {nullptr, nullptr};
  float *lm_rows = nullptr, *Rgates = nullptr;
  int *tile_ctr = nullptr;
  uint16_t *Ab = nullptr;   // materialised-logits path only
  float *Zbig = nullptr;
  uint64_t *cstat = nullptr;  // chunk statistics of the logits, [M][Npad_big / 32]
  double *score = nullptr;
  int *t = nullptr, *sym = nullptr, *len = nullptr, *last = nullptr, *ctx = nullptr, *lengths = nullptr;
  uint32_t *hash = nullptr;
  int *src_row = nullptr, *tok = nullptr;
  float *p_max = nullptr, *p_sum = nullptr, *zs = nullptr;
  uint64_t *p_cand = nullptr;
  int *tree_parent = nullptr, *tree_token = nullptr, *tree_merged = nullptr;
  int *finished = nullptr, *utt_steps = nullptr, *ctrl = nullptr;  // ctrl: n_finished, done, step_base, bad_arg, nonfinite
  int *out_tokens = nullptr, *out_lens = nullptr, *out_steps = nullptr;  // n-best lists; the allocation-free entry
  double *out_scores = nullptr;                                          // point points these at the caller's arrays
  int Mp = 0, S_max = 0, cap = 0, pc_chunks = 0, max_B = 0;
};

// The n-best lists of one decode of the handle's own workspace, packed behind the control words (ctrl is the slot
// before out_tokens in the layout), so that one copy brings flags and results to the host: byte offsets from ctrl.
struct OutPack {
  size_t steps, lens, scores, tokens, bytes;
};
OutPack out_pack(int B, int K, int cap) {
  OutPack o;
  const size_t M = (size_t)B * K;
  o.steps = 256;  // (ctrl's slot)
  o.lens = o.steps + ((size_t)B * 4 + 7) / 8 * 8;
  o.scores = o.lens + (M * 4 + 7) / 8 * 8;
  o.tokens = o.scores + M * 8;
  o.bytes = o.tokens + M * (size_t)cap * 4;
  return o;
}

// Assigns the pointers of `w` inside [base, ..) for a model `c` and the maxima given, every array on a 256-byte
// boundary, and returns the bytes needed.  base == nullptr: only the size is computed.  with_out: room for the
// n-best lists too.  big: the arrays of the materialised-logits path (Npad_big columns, Hb padded k).
size_t layout_workspace(Workspace &w, char *base, const rnnt_config_t &c, int n_chunks, int max_B, int max_T,
                        int max_beam, bool with_out, bool big, int Npad_big, int Hb) {
  size_t off = 0;
  auto take = [&](auto **p, size_t n) {
    typedef typename std::remove_reference<decltype(**p)>::type T;
    *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += (n * sizeof(T) + 255) / 256 * 256;
  };
  const size_t M = (size_t)max_B * max_beam;
  w.max_B = max_B;
  w.Mp = (int)((M + 31) / 32 * 32 + 32);  // a joint tile may start at any multiple of the beam and reads 32 rows
  w.S_max = max_T * (c.max_symbols + 1);
  w.cap = max_T * c.max_symbols + 1;
  w.pc_chunks = n_chunks > 64 ? n_chunks : 64;
  take(&w.f_proj, (size_t)max_B * max_T * c.H);
  take(&w.pre, (size_t)w.Mp * c.H);
  for (int i = 0; i < 2; ++i) {
    take(&w.h[i], (size_t)w.Mp * c.P);
    take(&w.c[i], (size_t)w.Mp * c.P);
  }
  if (big) {
    take(&w.Ab, (size_t)w.Mp * Hb);
    take(&w.Zbig, M * Npad_big);
    take(&w.cstat, M * (Npad_big / 32));
  }
  take(&w.lm_rows, M * c.V);
  take(&w.Rgates, M * 4 * c.P);
  take(&w.tile_ctr, (size_t)max_B);
  take(&w.score, M);
  take(&w.t, M);
  take(&w.sym, M);
  take(&w.len, M);
  take(&w.last, M);
  take(&w.hash, M);
  take(&w.ctx, M * kCtxMax);
  take(&w.lengths, (size_t)max_B);
  take(&w.src_row, M);
  take(&w.tok, M);
  take(&w.p_max, M * w.pc_chunks);
  take(&w.p_sum, M * w.pc_chunks);
  take(&w.p_cand, M * w.pc_chunks * max_beam);
  take(&w.zs, M * (1 + 8));
  const size_t tree = (size_t)max_B * w.S_max * max_beam;
  take(&w.tree_parent, tree);
  take(&w.tree_token, tree);
  take(&w.tree_merged, tree);
  take(&w.finished, (size_t)max_B);
  take(&w.utt_steps, (size_t)max_B);
  take(&w.ctrl, 8);
  if (with_out) {
    take(&w.out_tokens, M * w.cap);
    take(&w.out_lens, M);
    take(&w.out_scores, M);
    take(&w.out_steps, (size_t)max_B);
  }
  take(&w.pre2, (size_t)w.Mp * c.H);  // (the second buffer of the launches that add two halves, see PredProjArgs)
  return off;
}

}  // namespace

struct rnnt_beam {
  rnnt_config_t cfg;
  std::string err;
  int N = 0, n_chunks = 0, M_max = 0;
  std::vector<void *> allocs;
  // packed weights
  float *W_enc = nullptr, *b_enc = nullptr, *W_pred = nullptr, *b_pred = nullptr, *W_out = nullptr,
        *b_out = nullptr, *W_hh = nullptr, *G = nullptr, *tab = nullptr;
  // materialised-logits path (bf16 joint, large shapes)
  bool big = false;
  int Npad_big = 0, Hb = 0;  // padded extents of the bf16 operands: 256 columns, 64 k
  uint16_t *Wb = nullptr;
  float *Wspec = nullptr, *bias_spec = nullptr, *b_big = nullptr;
  Workspace ws;         // the handle's own workspace, laid out for max_B / max_T / max_beam in one allocation
  PersistCtl *pctl = nullptr;  // counters of the single-launch step loop
  int n_cus = 0, spin_limit = kSpinLimit;
  int max_lds = 64 * 1024;  // LDS a block may ask for on this device
  bool last_persistent = false;
  char *h_out = nullptr;          // pinned: the last decode's control words and packed results (see out_pack)
  size_t h_out_bytes = 0;
  OutPack last_out{};
  // pinned host words and their device alias: [0] every utterance has finished, [kProgressWord] the step counter as
  // the device advances it from chunk to chunk
  int *h_done = nullptr, *h_done_dev = nullptr;
  // last decode
  bool have_result = false;
  int last_B = 0, last_K = 0, last_T = 0;
  hipStream_t last_stream = nullptr;
  hipEvent_t ev_begin = nullptr, ev_end = nullptr;
  int pace_misses = 0;          // times the device's report of a chunk did not arrive in time
  bool pace_by_stream = false;  // set at the third: from then on the stream is waited for at once
  bool trace_pacing = false;  // environment RNNT_BEAM_TRACE_PACING: a line on stderr when the pacing falls back
  bool profiling = false;
  bool events_off = false;  // set while the allocation-free entry point enqueues (no event may be created)
  std::vector<hipEvent_t> prof_events;              // pool, two per timed launch
  std::vector<std::pair<int, int>> prof_launches;   // (kernel id, index of its first event)
  size_t prof_used = 0;
  KernelTimer timers[KT_COUNT];
  // graphs of one chunk of steps, keyed by the launch shape
  typedef std::tuple<int, int, int, int, uint64_t, uint32_t> GraphKey;  // B, beam, algo, T, LM id, LM weight
  std::map<GraphKey, std::pair<hipGraphExec_t, uint64_t>> graphs;       // (graph, creation serial)
  uint64_t graph_serial = 0;
};

namespace {

#define RB_HIP(h, call)                                                                              \
  do {                                                                                               \
    hipError_t e_ = (call);                                                                          \
    if (e_ != hipSuccess) {                                                                          \
      (h)->err = std::string(#call) + ": " + hipGetErrorString(e_);                                  \
      return e_ == hipErrorOutOfMemory ? RNNT_E_NOMEM : RNNT_E_HIP;                                  \
    }                                                                                                \
  } while (0)

template <typename T>
int dev_alloc(rnnt_beam *h, T **p, size_t n) {
  void *q = nullptr;
  RB_HIP(h, hipMalloc(&q, (n ? n : 1) * sizeof(T)));
  h->allocs.push_back(q);
  *p = static_cast<T *>(q);
  return RNNT_OK;
}

template <typename T>
int upload(rnnt_beam *h, T **p, const std::vector<T> &v) {
  int rc = dev_alloc(h, p, v.size());
  if (rc) return rc;
  RB_HIP(h, hipMemcpy(*p, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return RNNT_OK;
}

int download(rnnt_beam *h, std::vector<float> &v, const float *dev, size_t n) {
  v.resize(n);
  RB_HIP(h, hipMemcpy(v.data(), dev, n * sizeof(float), hipMemcpyDeviceToHost));
  return RNNT_OK;
}

int fail(rnnt_beam *h, int code, const std::string &msg) {
  h->err = msg;
  return code;
}

int beam_template(int K) { return K <= 4 ? 4 : (K <= 8 ? 8 : 16); }

// The projection of the prediction step split in two along k (k_pred_proj_half): taken when whole tiles would leave
// half of the compute units idle.  Needs P % 128 == 0 (each half of k is divided among 8 waves in steps of 8).
// (With fewer than 8 hypotheses the main launch is so short that the recurrent tiles moved into it would set its
// duration: 508 instead of 739 audio-s/s at batch 1, beam 1.  Up to 200 half tiles: at 240 (B * beam = 192) whole tiles
// with gate tiles beside them are as fast or faster: 22.1 vs 23.2 ms at batch 48, beam 4.)
bool proj_split(const rnnt_config_t &c, int M) {
  return c.P % 128 == 0 && M >= 8 && (c.H / 32) * ((M + 31) / 32) * 2 <= 200;
}

// Gate tiles of the recurrent product computed in the prediction-projection launch (the rest ride in the
// main launch): as many as fit beside the projection's own blocks, one block per compute unit, on every XCD
// (32 compute units each).
// Slot tiles per block of the recurrent product in the main launch.  From 256 slots up that launch has several
// rounds of blocks per compute unit, and a block that keeps its 32 gate rows in registers for 2 or 4 slot tiles and
// requests the next tile's slots while it multiplies takes 3.3 us per further tile instead of 5 to 7 us for a tile
// of its own.  Measured per shape (us per step, blocks of 1 / 2 / 4 tiles): 224 slots 36.6 / 38.7 / 38.2, 256 slots
// 41.4 / 41.7 / 40.6 (4 tiles: two blocks per gate tile, all resident at once), 288 slots 44.3 / 41.2 / 44.6, 320 slots
// 46.6 / 44.3 / 48.3, 512 slots 73.3 / 66.8 / 69.7; at 128 slots single tiles are better (26.0 / 27.0 / 26.9): the
// recurrent blocks run beside the joint blocks there, off the critical path.  Blocks of 3 tiles at 256 slots (216 blocks,
// which need 27 free compute units per XCD): 3 to 7 % slower at six shapes tried, 2.5 % faster with LM rows in the
// projection launch only (beam 8, batch 32).  (The kernels' fully unrolled form only.)
int recurrent_group(const rnnt_config_t &c, int M) {
  const int m_tiles = (M + 31) / 32;
  if (c.pred != RNNT_PRED_LSTM || c.P != 640 || c.H != 640 || m_tiles < 8) return 1;
  return m_tiles == 8 ? 4 : 2;
}
int recurrent_items(const rnnt_config_t &c, int M) {
  const int g = recurrent_group(c, M);
  return ((M + 31) / 32 + g - 1) / g;
}

int recurrent_split(const rnnt_config_t &c, int M) {
  if (proj_split(c, M)) return 0;  // no recurrent tiles beside the half tiles: they would set that launch's duration
  XcdMap m;
  m.a_tiles = c.H / 32;
  m.a_m = m.b_m = (M + 31) / 32;
  m.b_begin = 0;
  for (m.b_end = 4 * c.P / 32; m.b_end > 0; --m.b_end)
    if (xcd_grid(m) <= 256) break;
  return m.b_end;
}

// C = A B^T + bias through the LDS-tiled kernel; round_ops: bf16 operands on the bf16 matrix instructions
int launch_gemm(rnnt_beam *h, hipStream_t s, const float *A, const float *B, const float *bias, float *C, int M, int N,
                int K, int round_ops, int *nonfinite, const int *lengths = nullptr, int T = 0) {
  GemmArgs a{A, B, bias, C, M, N, K, 0, 0, nonfinite, lengths, T};
  auto go = [&](auto kernel, int bm, int bn, size_t lds) {
    a.n_mt = (M + bm - 1) / bm;
    a.n_nt = (N + bn - 1) / bn;
    hipLaunchKernelGGL(kernel, dim3(gemm_grid(a.n_mt, a.n_nt)), dim3(256), lds, s, a);
  };
  // float32: 64 x 64 tiles (a chunk is 16 slow matrix instructions per wave; many blocks balance the chip);
  // bf16: 128 x 128 tiles from 2048 rows up (the traffic from L2 per multiply-add halves), else 64 x 64
  if (!round_ops) go(k_gemm_tiled<false, 1, 1, true>, 64, 64, GemmTile<false, 1, 1>::kLdsBytes);
  else if (M >= 2048) go(k_gemm_tiled<true, 2, 2, false>, 128, 128, GemmTile<true, 2, 2>::kLdsBytes);
  else go(k_gemm_tiled<true, 1, 1, true>, 64, 64, GemmTile<true, 1, 1>::kLdsBytes);
  RB_HIP(h, hipGetLastError());
  return RNNT_OK;
}

// row-major [rows, K] -> k4-major [K][rows_padded] (rows beyond `rows` are zero)
std::vector<float> to_k4(const std::vector<float> &src, int rows, int K, int rows_padded) {
  std::vector<float> out((size_t)K * rows_padded, 0.f);
  for (int r = 0; r < rows; ++r)
    for (int k = 0; k < K; ++k) out[k4_index(k, r, rows_padded)] = src[(size_t)r * K + k];
  return out;
}

int pack_weights(rnnt_beam *h, const rnnt_weights_t *w) {
  const rnnt_config_t &c = h->cfg;
  const int H = c.H, P = c.P, D = c.D, E = c.E, V = c.V, N = h->N;
  const bool bf = c.prec == RNNT_BF16_JOINT;
  std::vector<float> tmp, out;
  std::vector<void *> staging;  // device buffers needed only until the folded tables have been computed
  int rc;
  // encoder projection
  if ((rc = download(h, tmp, w->W_enc, (size_t)H * D))) return rc;
  if (bf)
    for (auto &x : tmp) x = host_bf16_round(x);
  if ((rc = upload(h, &h->W_enc, tmp))) return rc;
  if ((rc = download(h, tmp, w->b_enc, H))) return rc;
  if ((rc = upload(h, &h->b_enc, tmp))) return rc;
  // prediction projection (row-major copy for the table folding, k4-major for the per-step kernel)
  std::vector<float> wpred, bpred;
  if ((rc = download(h, wpred, w->W_pred, (size_t)H * P))) return rc;
  if (bf)
    for (auto &x : wpred) x = host_bf16_round(x);
  float *d_wpred_rm = nullptr;
  if ((rc = upload(h, &d_wpred_rm, wpred))) return rc;
  staging.push_back(d_wpred_rm);
  if ((rc = upload(h, &h->W_pred, to_k4(wpred, H, P, H)))) return rc;
  if ((rc = download(h, bpred, w->b_pred, H))) return rc;
  if ((rc = upload(h, &h->b_pred, bpred))) return rc;
  // output layer, rows padded with zeros to whole 32-column chunks
  if ((rc = download(h, tmp, w->W_out, (size_t)N * H))) return rc;
  if (bf)
    for (auto &x : tmp) x = host_bf16_round(x);
  if ((rc = upload(h, &h->W_out, to_k4(tmp, N, H, h->n_chunks * 32)))) return rc;
  if ((rc = download(h, tmp, w->b_out, N))) return rc;
  out.assign((size_t)h->n_chunks * 32, 0.f);
  for (int i = 0; i < N; ++i) out[i] = tmp[i];
  if ((rc = upload(h, &h->b_out, out))) return rc;
  if (h->big) {
    // token rows as bf16, k8-major, padded to whole blocks of 256 columns; blank / duration rows apart
    std::vector<float> wout;
    if ((rc = download(h, wout, w->W_out, (size_t)N * H))) return rc;
    const int Np = h->Npad_big;
    std::vector<uint16_t> wb((size_t)h->Hb * Np, 0);  // k beyond H stays zero
    for (int r = 0; r < V; ++r)
      for (int k = 0; k < H; ++k) {
        const float x = host_bf16_round(wout[(size_t)r * H + k]);
        uint32_t u;
        memcpy(&u, &x, 4);
        wb[k8_index(k, r, Np)] = (uint16_t)(u >> 16);
      }
    if ((rc = upload(h, &h->Wb, wb))) return rc;
    std::vector<float> spec((size_t)(N - V) * H), bs(N - V), bb((size_t)Np, -INFINITY);  // padded columns: logit -inf
    for (int r = V; r < N; ++r)
      for (int k = 0; k < H; ++k) spec[(size_t)(r - V) * H + k] = host_bf16_round(wout[(size_t)r * H + k]);
    for (int r = V; r < N; ++r) bs[r - V] = tmp[r];
    for (int r = 0; r < V; ++r) bb[r] = tmp[r];
    if ((rc = upload(h, &h->Wspec, spec))) return rc;
    if ((rc = upload(h, &h->bias_spec, bs))) return rc;
    if ((rc = upload(h, &h->b_big, bb))) return rc;
  }

  if (c.pred == RNNT_PRED_LSTM) {
    // gate rows re-ordered so that rows 4u..4u+3 of a 32-row tile hold gates (i, f, g, o) of unit 8*tile + u
    auto packed_row = [&](int r) {  // r = packed row -> original row
      const int tile = r / 32, ul = (r % 32) / 4, gate = r % 4;
      return gate * P + tile * 8 + ul;
    };
    std::vector<float> whh, wih, bih, bhh, emb;
    if ((rc = download(h, whh, w->W_hh, (size_t)4 * P * P))) return rc;
    if ((rc = download(h, wih, w->W_ih, (size_t)4 * P * E))) return rc;
    if ((rc = download(h, bih, w->b_ih, (size_t)4 * P))) return rc;
    if ((rc = download(h, bhh, w->b_hh, (size_t)4 * P))) return rc;
    std::vector<float> whh_p((size_t)4 * P * P), wih_p((size_t)4 * P * E), b_p((size_t)4 * P);
    for (int r = 0; r < 4 * P; ++r) {
      const int o = packed_row(r);
      memcpy(&whh_p[(size_t)r * P], &whh[(size_t)o * P], sizeof(float) * P);
      memcpy(&wih_p[(size_t)r * E], &wih[(size_t)o * E], sizeof(float) * E);
      b_p[r] = bih[o] + bhh[o];
    }
    if ((rc = upload(h, &h->W_hh, to_k4(whh_p, 4 * P, P, 4 * P)))) return rc;
    // G[v] = W_ih emb[v] + b_ih + b_hh for every token (and the start symbol): one GEMM at create
    float *d_wih = nullptr, *d_b = nullptr, *d_emb = nullptr;
    if ((rc = upload(h, &d_wih, wih_p))) return rc;
    staging.push_back(d_wih);
    if ((rc = upload(h, &d_b, b_p))) return rc;
    staging.push_back(d_b);
    if ((rc = download(h, emb, w->emb, (size_t)(V + 1) * E))) return rc;
    if ((rc = upload(h, &d_emb, emb))) return rc;
    staging.push_back(d_emb);
    if ((rc = dev_alloc(h, &h->G, (size_t)(V + 1) * 4 * P))) return rc;
    if ((rc = launch_gemm(h, nullptr, d_emb, d_wih, d_b, h->G, V + 1, 4 * P, E, 0, nullptr))) return rc;
  } else {
    // stateless: tab[i][v] = W_pred emb_i[v] (+ b_pred for i = 0), so that the per-step
    // prediction network is a gather-add inside the joint kernel
    const int ctx = c.stateless_context;
    std::vector<float> emb;
    if ((rc = download(h, emb, w->emb, (size_t)ctx * (V + 1) * P))) return rc;
    float *d_emb = nullptr;
    if ((rc = upload(h, &d_emb, emb))) return rc;
    staging.push_back(d_emb);
    if ((rc = dev_alloc(h, &h->tab, (size_t)ctx * (V + 1) * H))) return rc;
    for (int i = 0; i < ctx; ++i)
      if ((rc = launch_gemm(h, nullptr, d_emb + (size_t)i * (V + 1) * P, d_wpred_rm, i == 0 ? h->b_pred : nullptr,
                            h->tab + (size_t)i * (V + 1) * H, V + 1, H, P, bf ? 1 : 0, nullptr)))
        return rc;
  }
  RB_HIP(h, hipDeviceSynchronize());
  // the row-major copies were only the operands of the folding products above
  for (void *q : staging) {
    hipFree(q);
    for (size_t i = 0; i < h->allocs.size(); ++i)
      if (h->allocs[i] == q) {
        h->allocs.erase(h->allocs.begin() + i);
        break;
      }
  }
  return RNNT_OK;
}

struct StepPlan {
  int B, K, T, algo, M;
  const rnnt_lm_t *lm;
  float lambda;
  const float *inj_tok, *inj_dur;
  int C;
  bool big = false;  // logits through HBM (k_joint_big + k_row_select) instead of the fused main kernel
  const Workspace *ws = nullptr;  // where the decode works
  bool ahead = false;             // enqueue the upper bound of steps at once instead of following the device
  bool plain = false;             // no graph and no profiling events (nothing that could allocate)
  int out_cap = 0;                // row length of ws->out_tokens
};

// Timing wrapper used in profiling mode: an event before and after the launch, nothing waits.
// The pairs are read back once the decode has finished, so the kernels run as densely as in an
// untimed decode (plain launches, no graph).
struct ScopedKernelTime {
  rnnt_beam *h;
  hipStream_t s;
  int which;
  size_t first = 0;
  bool on = false;
  ScopedKernelTime(rnnt_beam *h_, hipStream_t s_, int w) : h(h_), s(s_), which(w) {
    if (!h->profiling || h->events_off) return;
    while (h->prof_events.size() < h->prof_used + 2) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return;
      h->prof_events.push_back(e);
    }
    first = h->prof_used;
    h->prof_used += 2;
    on = hipEventRecord(h->prof_events[first], s) == hipSuccess;
  }
  ~ScopedKernelTime() {
    if (!on) return;
    if (hipEventRecord(h->prof_events[first + 1], s) == hipSuccess) h->prof_launches.push_back({which, (int)first});
  }
};

// steps per graph launch (even: the state parity flips every step)
constexpr int kChunkSteps = 16;
// the next chunk of steps is enqueued at least this long before the running one ends (a graph launch takes some 20 us)
constexpr int kEnqueueMarginUs = 150;
// the word of the pinned pair that carries the step counter (a cache line away from the "done" word)
constexpr int kProgressWord = 16;
// the enqueueing thread waits this long for the device to report the next chunk before it waits for the stream itself
constexpr int kPaceLimitMs = 200;

// Materialised-logits path: selection and next activations in the tail of the row kernel (two launches per step)
// unless a candidate rule needs a selection kernel of its own.
bool big_tail(const rnnt_beam *h, const StepPlan &p) { return p.big && !h->cfg.tdt_all_pairs; }

void fill_stateless_pre_big(rnnt_beam *h, const StepPlan &p, int bump, StatelessPreBigArgs &a) {
  const Workspace &w = *p.ws;
  const rnnt_config_t &c = h->cfg;
  a.f_proj = w.f_proj; a.tab = h->tab; a.ctx_tok = w.ctx; a.t = w.t; a.lengths = w.lengths;
  a.Ab = w.Ab;
  a.M = p.M; a.Mp = w.Mp; a.K = p.K; a.T = p.T; a.H = c.H; a.V = c.V; a.n_ctx = c.stateless_context;
  a.done = w.ctrl + 1; a.step_base = w.ctrl + 2; a.bump = bump;
  a.h_progress = h->h_done_dev + kProgressWord;
}

// One-list selection forms: 16 / 12 for ALSD++ / AES++ (without prune margin and prefix search) on a plain RNN-T
// (no durations, no LM), else the general 4.
int plain_forms(const rnnt_beam *h, const StepPlan &p) {
  const rnnt_config_t &c = h->cfg;
  if (c.n_durations != 0 || p.lm) return 4;
  if (p.algo == RNNT_ALSD) return 16;
  return (!std::isfinite(c.prune_margin) && !c.aes_prefix_search) ? 12 : 4;
}

// fuse_lm: the LM rows of the new hypotheses ride in the projection launch, or in the cell-update launch when
// the row is too large to sit in LDS beside the projection's tiles (LSTM models only; the caller then skips the
// stand-alone LM launch)
constexpr size_t kLmRowBesideTiles = 16 * 1024;
int launch_pred(rnnt_beam *h, hipStream_t s, const StepPlan &p, int cur, int bump, bool fuse_lm = false) {
  const Workspace &w = *p.ws;
  const rnnt_config_t &c = h->cfg;
  int *done = w.ctrl + 1, *step_base = w.ctrl + 2;
  const int m_tiles = (p.M + 31) / 32;
  if (p.inj_tok) {
    if (bump)
      hipLaunchKernelGGL(k_bump, dim3(1), dim3(64), 0, s, step_base, bump, done, h->h_done_dev + kProgressWord);
  } else if (c.pred == RNNT_PRED_LSTM) {
    LmRowsArgs lm_rows{};
    const size_t lm_row_bytes = sizeof(float) * (size_t)c.V;
    if (fuse_lm && p.lm) {
      lm_rows.view = lm_view(p.lm);
      lm_rows.ctx = w.ctx; lm_rows.len = w.len; lm_rows.out = w.lm_rows;
      lm_rows.M = p.M;
    }
    {
      ScopedKernelTime tm(h, s, KT_LSTM);
      const int n = p.M * c.P, n_blocks = (n + 255) / 256;
      LmRowsArgs lmr{};
      size_t lds = 0;
      if (lm_rows.M && lm_row_bytes > kLmRowBesideTiles) {
        lmr = lm_rows;
        lmr.first_block = n_blocks;
        lds = lm_row_bytes;
      }
      const bool split = proj_split(c, p.M);
      auto k_cell = lmr.M ? k_lstm_pointwise<true> : k_lstm_pointwise<false>;
      hipLaunchKernelGGL(k_cell, dim3(n_blocks + lmr.M), dim3(256), lds, s, w.Rgates, h->G, w.h[cur],
                         w.c[cur], w.h[cur ^ 1], w.c[cur ^ 1], w.src_row, w.tok, p.M, w.Mp, c.P, done, lmr,
                         nullptr, 0);
    }
    {
      PredProjArgs a;
      a.Wp = h->W_pred; a.bias = h->b_pred; a.h = w.h[cur ^ 1]; a.f_proj = w.f_proj;
      a.t = w.t; a.lengths = w.lengths;
      a.pre = w.pre;
      if (proj_split(c, p.M)) {  // (the step at parity cur read buffer cur; this launch writes the next step's)
        a.pre = cur ? w.pre : w.pre2;
        a.pre_clear = cur ? w.pre2 : w.pre;
        a.n_pre_clear = c.H * w.Mp;
      }
      a.M = p.M; a.Mp = w.Mp; a.K = p.K; a.T = p.T; a.P = c.P; a.H = c.H;
      a.round_ops = c.prec == RNNT_BF16_JOINT ? 1 : 0;
      a.done = done; a.step_base = step_base; a.bump = bump; a.h_progress = h->h_done_dev + kProgressWord;
      a.rec.Whh = h->W_hh; a.rec.h = w.h[cur ^ 1]; a.rec.R = w.Rgates;
      a.rec.P = c.P; a.rec.M = p.M; a.rec.Mp = w.Mp; a.rec.group = 1;
      a.map.a_tiles = c.H / 32; a.map.a_m = m_tiles;
      a.map.b_begin = 0; a.map.b_end = recurrent_split(c, p.M); a.map.b_m = m_tiles;
      ScopedKernelTime tm(h, s, KT_PREDPROJ);
      if (proj_split(c, p.M)) {  // items (32-slot tile, half of k) in place of 32-slot tiles
        a.map.a_m = 2 * m_tiles;
        a.map.b_end = 0;
      }
      const int n_tiles = xcd_grid(a.map);
      a.lmr = LmRowsArgs{};
      size_t lds = 0;
      if (lm_rows.M && lm_row_bytes <= kLmRowBesideTiles) {
        a.lmr = lm_rows;
        a.lmr.first_block = n_tiles;
        lds = lm_row_bytes;
      }
      const dim3 grid(n_tiles + a.lmr.M);
#define RB_PRED(W, I)                                                                                        \
  do {                                                                                                       \
    if (a.lmr.M) hipLaunchKernelGGL((k_pred_proj<W, I, true>), grid, dim3(W * 64), lds, s, a);              \
    else hipLaunchKernelGGL((k_pred_proj<W, I, false>), grid, dim3(W * 64), 0, s, a);                        \
  } while (0)
#define RB_PRED_HALF(I)                                                                                      \
  do {                                                                                                       \
    if (a.lmr.M) hipLaunchKernelGGL((k_pred_proj_half<8, I, true>), grid, dim3(512), lds, s, a);            \
    else hipLaunchKernelGGL((k_pred_proj_half<8, I, false>), grid, dim3(512), 0, s, a);                      \
  } while (0)
      if (proj_split(c, p.M)) {
        if (c.P == 640) RB_PRED_HALF(5);
        else RB_PRED_HALF(0);
      }
      else if (c.P == 640) RB_PRED(8, 10);
      else if (c.P % 64 == 0) RB_PRED(8, 0);
      else RB_PRED(4, 0);
#undef RB_PRED_HALF
#undef RB_PRED
    }
  } else if (p.big) {
    StatelessPreBigArgs a;
    fill_stateless_pre_big(h, p, bump, a);
    ScopedKernelTime tm(h, s, KT_STATELESS);
    const int n = p.M * (c.H / 8);
    hipLaunchKernelGGL(k_stateless_pre_big, dim3((n + 255) / 256), dim3(256), 0, s, a);
  } else {
    StatelessPreArgs a;
    a.f_proj = w.f_proj; a.tab = h->tab; a.ctx_tok = w.ctx; a.t = w.t; a.lengths = w.lengths;
    a.pre = w.pre;
    a.M = p.M; a.Mp = w.Mp; a.K = p.K; a.T = p.T; a.H = c.H; a.V = c.V; a.n_ctx = c.stateless_context;
    a.done = done; a.step_base = step_base; a.bump = bump; a.h_progress = h->h_done_dev + kProgressWord;
    ScopedKernelTime tm(h, s, KT_STATELESS);
    const int n = p.M * (c.H / 4);
    hipLaunchKernelGGL(k_stateless_pre, dim3((n + 255) / 256), dim3(256), 0, s, a);
  }
  RB_HIP(h, hipGetLastError());
  return RNNT_OK;
}

int launch_lm(rnnt_beam *h, hipStream_t s, const StepPlan &p) {
  const Workspace &w = *p.ws;
  if (!p.lm) return RNNT_OK;
  ScopedKernelTime tm(h, s, KT_LM);
  lm_launch_rows(p.lm, w.ctx, w.len, w.lm_rows, p.M, w.ctrl + 1, s);
  RB_HIP(h, hipGetLastError());
  return RNNT_OK;
}

void fill_select_args(rnnt_beam *h, const StepPlan &p, int step_off, int n_chunks, SelectArgs &a) {
  const Workspace &w = *p.ws;
  const rnnt_config_t &c = h->cfg;
  a.score = w.score; a.t = w.t; a.sym = w.sym; a.len = w.len; a.last = w.last; a.hash = w.hash;
  a.ctx = w.ctx;
  a.lengths = w.lengths;
  a.p_max = w.p_max; a.p_sum = w.p_sum; a.p_cand = w.p_cand; a.zs = w.zs;
  a.n_chunks = n_chunks;
  a.normalized = p.inj_tok ? 1 : 0;
  a.use_ctx = (c.pred == RNNT_PRED_STATELESS || p.lm) ? 1 : 0;
  a.B = p.B; a.K = p.K; a.V = c.V; a.ND = c.n_durations;
  a.dur_bytes = 0;
  for (int i = 0; i < 8; ++i) {
    a.dur[i] = c.durations[i];
    a.dur_bytes |= (uint64_t)(c.durations[i] & 0xff) << (8 * i);
  }
  a.algo = p.algo;
  a.max_sym = c.max_symbols;
  a.gamma = c.prune_margin;
  a.has_lm = p.lm ? 1 : 0;
  a.lm_rule3 = c.lm_rule == 3 ? 1 : 0;
  a.lm_early = (p.lm && c.lm_early_pruning) ? 1 : 0;
  a.prefix = c.aes_prefix_search;
  a.lm_rows = w.lm_rows;
  a.lambda = p.lambda;
  a.src_row = w.src_row; a.tok = w.tok;
  a.tree_parent = w.tree_parent; a.tree_token = w.tree_token; a.tree_merged = w.tree_merged;
  a.S_max = w.S_max;
  a.step_base = w.ctrl + 2;
  a.step_off = step_off;
  a.finished = w.finished; a.utt_steps = w.utt_steps; a.n_finished = w.ctrl; a.done = w.ctrl + 1;
  a.h_done = h->h_done_dev;
}

// stand-alone selection: which kernel takes this beam, list count and candidate rule
void launch_select(rnnt_beam *h, hipStream_t s, const StepPlan &p, const SelectArgs &sa, int n_chunks) {
  if (h->cfg.tdt_all_pairs) hipLaunchKernelGGL(k_select_pairs, dim3((p.B + 1) / 2), dim3(128), 0, s, sa);
  else if (select_needs_wide_forms(p.K, n_chunks) && n_chunks <= 64 * kMergeHeads) {
    MergeSelectArgs ma;  // a block per utterance, a wave per hypothesis: lists merged first, then the one-list selection
    ma.sel = sa;
    ma.sel.n_chunks = 1;
    ma.n_lists = n_chunks;
    const int forms = plain_forms(h, p);
    auto k_sel = forms == 16 ? k_utt_merge_select<16> : forms == 12 ? k_utt_merge_select<12> : k_utt_merge_select<4>;
    hipLaunchKernelGGL(k_sel, dim3(p.B), dim3(64 * p.K), 0, s, ma);
  } else if (select_needs_wide_forms(p.K, n_chunks)) hipLaunchKernelGGL(k_select_wide, dim3((p.B + 3) / 4), dim3(256), 0, s, sa);
  else hipLaunchKernelGGL(k_select, dim3((p.B + 3) / 4), dim3(256), 0, s, sa);
}

// one beam-search step; cur = parity of the prediction-network state it reads
int launch_step(rnnt_beam *h, hipStream_t s, const StepPlan &p, int step_off, int cur, int bump) {
  const Workspace &w = *p.ws;
  const rnnt_config_t &c = h->cfg;
  int *done = w.ctrl + 1;
  const int kt = beam_template(p.K);
  if (p.inj_tok) {
    InjectArgs a;
    a.tok_logp = p.inj_tok;
    a.dur_logp = p.inj_dur;
    a.C = p.C;
    a.t = w.t;
    a.hash = w.hash;
    a.lengths = w.lengths;
    a.M = p.M; a.K = p.K; a.T = p.T; a.V = c.V; a.ND = c.n_durations;
    a.p_cand = w.p_cand;
    a.zs = w.zs;
    a.done = done;
    {
      ScopedKernelTime tm(h, s, KT_JOINT);
      if (kt == 4) hipLaunchKernelGGL(k_inject<4>, dim3(p.M), dim3(64), 0, s, a);
      else if (kt == 8) hipLaunchKernelGGL(k_inject<8>, dim3(p.M), dim3(64), 0, s, a);
      else hipLaunchKernelGGL(k_inject<16>, dim3(p.M), dim3(64), 0, s, a);
    }
    RB_HIP(h, hipGetLastError());
    SelectArgs sa;
    fill_select_args(h, p, step_off, 64, sa);
    ScopedKernelTime tm(h, s, KT_SELECT);
    launch_select(h, s, p, sa, 64);
  } else if (p.big) {
    constexpr int MS = 5;  // 160 hypotheses per block
    {
      BigJointArgs a;
      a.Wb = h->Wb; a.Ab = w.Ab; a.bias = h->b_big; a.Z = w.Zbig; a.cstat = w.cstat;
      a.M = p.M; a.Mp = w.Mp; a.H = h->Hb; a.Npad = h->Npad_big;
      constexpr int WV = 4;  // waves per block; the block covers 32 * WV columns
      a.map.a_tiles = h->Npad_big / (32 * WV); a.map.a_m = (p.M + 32 * MS - 1) / (32 * MS);
      a.map.b_begin = a.map.b_end = 0; a.map.b_m = 0;
      a.done = done;
      a.step_base = w.ctrl + 2;
      a.bump = (big_tail(h, p) && step_off == 0) ? kChunkSteps : 0;
      a.h_progress = h->h_done_dev + kProgressWord;
      ScopedKernelTime tm(h, s, KT_JOINTBIG);
      const dim3 grid(xcd_grid(a.map));
      // the kernel's loop runs in whole groups of D stages of k = 32; the operands are padded to k % 64 == 0
      if (h->Hb % 128 == 0) hipLaunchKernelGGL((k_joint_big<WV, 4>), grid, dim3(64 * WV), 0, s, a);
      else hipLaunchKernelGGL((k_joint_big<WV, 2>), grid, dim3(64 * WV), 0, s, a);
    }
    RB_HIP(h, hipGetLastError());
    {
      RowSelectArgs a;
      a.Z = w.Zbig; a.cstat = w.cstat; a.Npad = h->Npad_big; a.Ab = w.Ab; a.M = p.M; a.Mp = w.Mp; a.H = c.H;
      a.K = p.K; a.V = c.V; a.ND = c.n_durations;
      a.Wspec = h->Wspec; a.bias_spec = h->bias_spec;
      a.lm = (p.lm && !c.lm_early_pruning) ? w.lm_rows : nullptr;  // early pruning ranks without the LM term
      a.lambda = p.lambda;
      a.p_max = w.p_max; a.p_sum = w.p_sum; a.p_cand = w.p_cand; a.zs = w.zs;
      a.finished = w.finished; a.done = done;
      a.utt_ctr = w.tile_ctr;
      fill_select_args(h, p, step_off, 1, a.sel);
      fill_stateless_pre_big(h, p, 0, a.pre);
      ScopedKernelTime tm(h, s, (big_tail(h, p) && !a.lm) ? KT_UTTSELECT : KT_ROWSELECT);
      // without an LM term in the keys the chunk statistics of the contraction say which chunks to read
      const dim3 grid(p.M), block(64 * kRowWaves);
      if (big_tail(h, p)) {
        if (a.lm) hipLaunchKernelGGL((k_row_select<true, false>), grid, block, 0, s, a);
        else {  // one block per utterance
          const int forms = plain_forms(h, p);
          auto k_sel = forms == 16 ? k_utt_select<16> : forms == 12 ? k_utt_select<12> : k_utt_select<4>;
          hipLaunchKernelGGL(k_sel, dim3(p.B), dim3(64 * p.K), 0, s, a);
        }
      } else {
        if (a.lm) hipLaunchKernelGGL((k_row_select<false, false>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_row_select<false, true>), grid, block, 0, s, a);
      }
    }
    RB_HIP(h, hipGetLastError());
    if (big_tail(h, p)) {
      // selection and next activations ran in the row kernel's tail; only the LM rows of the new hypotheses remain
      return launch_lm(h, s, p);
    }
    {
      SelectArgs sa;
      fill_select_args(h, p, step_off, 1, sa);
      ScopedKernelTime tm(h, s, KT_SELECT);
      launch_select(h, s, p, sa, 1);
    }
  } else {
    MainArgs a;
    a.pre = w.pre;
    a.W = h->W_out;
    a.bias = h->b_out;
    a.lm = (p.lm && !c.lm_early_pruning) ? w.lm_rows : nullptr;  // early pruning ranks without the LM term
    a.lambda = p.lambda;
    a.M = p.M; a.Mp = w.Mp; a.K = p.K; a.H = c.H; a.V = c.V; a.ND = c.n_durations;
    a.n_chunks = h->n_chunks;
    a.round_ops = c.prec == RNNT_BF16_JOINT ? 1 : 0;
    a.upt = 32 / p.K < 8 ? 32 / p.K : 8;  // one wave of the completing block per utterance
    a.rpt = a.upt * p.K;
    a.n_jtiles = (p.B + a.upt - 1) / a.upt;
    a.p_max = w.p_max; a.p_sum = w.p_sum; a.p_cand = w.p_cand; a.zs = w.zs;
    a.tile_ctr = w.tile_ctr;
    const bool lstm = c.pred == RNNT_PRED_LSTM;
    if (lstm && proj_split(c, p.M) && cur) a.pre = w.pre2;  // (see launch_pred: the buffers alternate with the steps)
    a.rec.Whh = h->W_hh; a.rec.h = w.h[cur]; a.rec.R = w.Rgates;
    a.rec.P = c.P; a.rec.M = p.M; a.rec.Mp = w.Mp; a.rec.group = recurrent_group(c, p.M);
    // More joint blocks than compute units, and the blank / duration columns alone in the last chunk: its blocks
    // would start when the first ones end, and the selection would wait for them.  The token chunks' blocks take
    // those columns instead (one each), as dot products on the operands that they hold in registers.
    const bool fold = c.V % 32 == 0 && c.H == 640 && (!lstm || c.P == 640) && a.n_chunks - 1 >= 1 + c.n_durations &&
                      a.n_chunks * a.n_jtiles > 256;
    a.n_jchunks = fold ? a.n_chunks - 1 : a.n_chunks;
    a.map.a_tiles = a.n_jchunks; a.map.a_m = a.n_jtiles;
    a.map.b_begin = lstm ? recurrent_split(c, p.M) : 0;
    a.map.b_end = lstm ? 4 * c.P / 32 : 0;
    a.map.b_m = recurrent_items(c, p.M);
    fill_select_args(h, p, step_off, h->n_chunks, a.sel);
    const dim3 grid(xcd_grid(a.map));
    // The selection runs in the tail of this kernel for the beams its in-kernel forms take.  (Building the kernel
    // without it lets two blocks share a compute unit, but they also share its operand path: measured slower at
    // every shape, 11.3 vs 10.6 ms at B * beam = 256, beam 4.)
    const bool tail = p.K <= 8 && !c.tdt_all_pairs;
#define RB_MAIN(W, I)                                                                              \
  do {                                                                                             \
    if (tail) hipLaunchKernelGGL((k_step_main<W, I, true>), grid, dim3(W * 64), 0, s, a);         \
    else hipLaunchKernelGGL((k_step_main<W, I, false>), grid, dim3(W * 64), 0, s, a);             \
  } while (0)
    const bool wide = fold || a.rec.group > 1;  // (both only with the fully unrolled form below)
    {
      ScopedKernelTime tm(h, s, KT_JOINT);
      const bool full = c.H == 640 && (!lstm || c.P == 640);  // the fully unrolled form
      // one selection form in the kernel where the shape is one of the two common ones (a third of the code)
      // (11: form 5 for ALSD++ on a plain RNN-T, i.e. without durations and LM)
      const bool plain = c.n_durations == 0 && !p.lm && p.algo == RNNT_ALSD;
      const bool plain_aes = c.n_durations == 0 && !p.lm && p.algo == RNNT_AES && !std::isfinite(c.prune_margin) &&
                             !c.aes_prefix_search;
      const int sel_any = !tail ? 0 : (p.K <= 2 && a.n_chunks <= 48 && plain) ? 13
                                    : (p.K > 2 && p.K <= 4 && a.n_chunks <= 48) ? (plain ? 11 : plain_aes ? 15 : 5)
                                    : (p.K > 4 && p.K <= 8 && a.n_chunks <= 40) ? (plain ? 14 : 6) : 0;
      const int sel = full ? sel_any : 0;
      // (the kernels for other widths: the ALSD++ forms for a plain RNN-T only)
      const int sel_gen = (sel_any == 11 || sel_any == 13 || sel_any == 14) ? sel_any : 0;
#define RB_MAIN_SEL(WIDE)                                                                                   \
  do {                                                                                                      \
    if (sel == 11) hipLaunchKernelGGL((k_step_main<8, 10, true, WIDE, 11>), grid, dim3(512), 0, s, a);      \
    else if (sel == 13) hipLaunchKernelGGL((k_step_main<8, 10, true, WIDE, 13>), grid, dim3(512), 0, s, a); \
    else if (sel == 14) hipLaunchKernelGGL((k_step_main<8, 10, true, WIDE, 14>), grid, dim3(512), 0, s, a); \
    else if (sel == 15) hipLaunchKernelGGL((k_step_main<8, 10, true, WIDE, 15>), grid, dim3(512), 0, s, a); \
    else if (sel == 5) hipLaunchKernelGGL((k_step_main<8, 10, true, WIDE, 5>), grid, dim3(512), 0, s, a);   \
    else if (sel == 6) hipLaunchKernelGGL((k_step_main<8, 10, true, WIDE, 6>), grid, dim3(512), 0, s, a);   \
    else hipLaunchKernelGGL((k_step_main<8, 10, true, WIDE, 0>), grid, dim3(512), 0, s, a);                 \
  } while (0)
      if (wide && tail) RB_MAIN_SEL(true);
      else if (wide) hipLaunchKernelGGL((k_step_main<8, 10, false, true>), grid, dim3(512), 0, s, a);
      else if (full && tail) RB_MAIN_SEL(false);
      else if (full) RB_MAIN(8, 10);
#undef RB_MAIN_SEL
#define RB_MAIN_GEN(W)                                                                                       \
  do {                                                                                                       \
    if (sel_gen == 11) hipLaunchKernelGGL((k_step_main<W, 0, true, false, 11>), grid, dim3(W * 64), 0, s, a); \
    else if (sel_gen == 13) hipLaunchKernelGGL((k_step_main<W, 0, true, false, 13>), grid, dim3(W * 64), 0, s, a); \
    else if (sel_gen == 14) hipLaunchKernelGGL((k_step_main<W, 0, true, false, 14>), grid, dim3(W * 64), 0, s, a); \
    else RB_MAIN(W, 0);                                                                                      \
  } while (0)
      else if (c.H % 64 == 0 && (!lstm || c.P % 64 == 0)) RB_MAIN_GEN(8);
      else RB_MAIN_GEN(4);
#undef RB_MAIN_GEN
    }
#undef RB_MAIN
    if (!tail) {
      RB_HIP(h, hipGetLastError());
      ScopedKernelTime tm(h, s, KT_SELECT);
      launch_select(h, s, p, a.sel, h->n_chunks);
    }
  }
  RB_HIP(h, hipGetLastError());
  const bool fuse_lm = p.lm && !p.inj_tok && c.pred == RNNT_PRED_LSTM;
  if (!fuse_lm) {
    int rc = launch_lm(h, s, p);
    if (rc) return rc;
  }
  return launch_pred(h, s, p, cur, bump, fuse_lm);
}

// instantiated graphs kept per handle (one per launch shape, LM and LM weight); the oldest is dropped beyond that
constexpr size_t kMaxGraphs = 8;

// The single-launch step loop (k_decode_persistent) takes LSTM decoders without an LM at beams up to 8 whose
// utterances, dealt out over the eight XCDs, leave at most 32 slots per XCD; everything else replays per-step launches.
bool use_persistent(const rnnt_beam *h, const StepPlan &p) {
  const rnnt_config_t &c = h->cfg;
  if (!c.persistent_kernel || p.inj_tok || p.lm || p.plain || p.big || h->profiling) return false;
  if (c.pred != RNNT_PRED_LSTM || c.tdt_all_pairs || p.K > 8) return false;
  if (c.H % 64 || c.P % 64) return false;
  if ((p.B + kXccs - 1) / kXccs * p.K > 32) return false;
  return h->n_cus >= 2 * kXccs;
}

int launch_persistent(rnnt_beam *h, hipStream_t s, const StepPlan &p, int max_steps) {
  const Workspace &w = *p.ws;
  const rnnt_config_t &c = h->cfg;
  PersistArgs a{};
  MainArgs &m = a.main;
  m.pre = w.pre; m.W = h->W_out; m.bias = h->b_out; m.lm = nullptr; m.lambda = 0.f;
  m.M = p.M; m.Mp = w.Mp; m.K = p.K; m.H = c.H; m.V = c.V; m.ND = c.n_durations;
  m.n_chunks = m.n_jchunks = h->n_chunks;
  m.round_ops = c.prec == RNNT_BF16_JOINT ? 1 : 0;
  m.p_max = w.p_max; m.p_sum = w.p_sum; m.p_cand = w.p_cand; m.zs = w.zs;
  m.tile_ctr = w.tile_ctr;
  m.rec.Whh = h->W_hh; m.rec.h = nullptr; m.rec.R = w.Rgates; m.rec.P = c.P; m.rec.M = p.M; m.rec.Mp = w.Mp; m.rec.group = 1;
  fill_select_args(h, p, 0, h->n_chunks, m.sel);  // (the step counter word stays 0: the kernel passes the step itself)
  PredProjArgs &q = a.pp;
  q.Wp = h->W_pred; q.bias = h->b_pred; q.h = nullptr; q.f_proj = w.f_proj; q.t = w.t; q.lengths = w.lengths;
  q.pre = w.pre;
  q.M = p.M; q.Mp = w.Mp; q.K = p.K; q.T = p.T; q.P = c.P; q.H = c.H; q.round_ops = m.round_ops;
  q.done = w.ctrl + 1; q.step_base = w.ctrl + 2; q.bump = 0;
  a.G = h->G;
  for (int i = 0; i < 2; ++i) {
    a.h[i] = w.h[i];
    a.c[i] = w.c[i];
  }
  a.R = w.Rgates;
  a.ctl = h->pctl;
  a.B = p.B;
  a.max_steps = max_steps;
  a.spin_limit = h->spin_limit;
  hipLaunchKernelGGL(k_fill_int, dim3(1), dim3(256), 0, s, reinterpret_cast<int *>(h->pctl), 0,
                     (int)(sizeof(PersistCtl) / sizeof(int)));
  const dim3 grid(h->n_cus / kXccs * kXccs);
  ScopedKernelTime tm(h, s, KT_JOINT);
  if (c.H == 640 && c.P == 640) hipLaunchKernelGGL((k_decode_persistent<8, 10>), grid, dim3(512), 0, s, a);
  else hipLaunchKernelGGL((k_decode_persistent<8, 0>), grid, dim3(512), 0, s, a);
  RB_HIP(h, hipGetLastError());
  return RNNT_OK;
}

int run_decode(rnnt_beam *h, const float *enc, const int32_t *lengths, const StepPlan &p, hipStream_t s) {
  const Workspace &w = *p.ws;
  const rnnt_config_t &c = h->cfg;
  int *n_finished = w.ctrl, *done = w.ctrl + 1, *step_base = w.ctrl + 2, *bad_arg = w.ctrl + 3,
      *nonfinite = w.ctrl + 4;
  h->have_result = false;
  // the previous decode may still be writing the pinned completion word
  if (h->last_stream) RB_HIP(h, hipStreamSynchronize(h->last_stream));
  for (int i = 0; i < KT_COUNT; ++i) h->timers[i] = KernelTimer{kKernelNames[i], 0.f, 0};
  h->prof_used = 0;
  h->prof_launches.clear();
  RB_HIP(h, hipEventRecord(h->ev_begin, s));
  {
    InitArgs a;
    a.score = w.score; a.t = w.t; a.sym = w.sym; a.len = w.len; a.last = w.last; a.hash = w.hash;
    a.ctx = w.ctx;
    a.lengths_in = lengths;
    a.lengths = w.lengths;
    a.src_row = w.src_row; a.tok = w.tok;
    const bool lstm = c.pred == RNNT_PRED_LSTM && !p.inj_tok;
    a.h0 = lstm ? w.h[1] : nullptr;
    a.c0 = lstm ? w.c[1] : nullptr;
    a.n_state = (size_t)c.P * w.Mp;
    a.R = lstm ? w.Rgates : nullptr;
    a.n_R = (size_t)p.M * 4 * c.P;
    const bool halves = lstm && proj_split(c, p.M);
    a.pre0 = halves ? w.pre : nullptr;
    a.pre1 = halves ? w.pre2 : nullptr;
    a.n_pre = (size_t)c.H * w.Mp;
    a.tile_ctr = w.tile_ctr;
    a.n_tiles = w.max_B;
    a.B = p.B; a.K = p.K; a.T = p.T; a.V = c.V;
    a.lstm = lstm ? 1 : 0;
    a.step_base_init = big_tail(h, p) ? -kChunkSteps : 0;
    a.finished = w.finished; a.utt_steps = w.utt_steps; a.n_finished = n_finished; a.done = done;
    a.step_base = step_base; a.bad_arg = bad_arg;
    a.h_done = h->h_done_dev;
    *reinterpret_cast<volatile int *>(h->h_done) = 0;
    *reinterpret_cast<volatile int *>(h->h_done + kProgressWord) = 0;
    ScopedKernelTime tm(h, s, KT_INIT);
    hipLaunchKernelGGL(k_fill_int, dim3(1), dim3(64), 0, s, bad_arg, 0, 2);  // bad_arg, nonfinite
    hipLaunchKernelGGL(k_init, dim3(256), dim3(256), 0, s, a);
  }
  RB_HIP(h, hipGetLastError());
  if (!p.inj_tok) {
    ScopedKernelTime tm(h, s, KT_ENCPROJ);
    // (the frames behind an utterance's last one are never read: tiles that hold nothing else are left out)
    int rc = launch_gemm(h, s, enc, h->W_enc, h->b_enc, w.f_proj, p.B * p.T, c.H, c.D,
                         c.prec == RNNT_BF16_JOINT ? 1 : 0, nonfinite, lengths, p.T);
    if (rc) return rc;
  }
  // every utterance has finished after at most T (s + 1) steps (the selection enforces it)
  const int max_steps = p.T * (c.max_symbols + 1) < w.S_max ? p.T * (c.max_symbols + 1) : w.S_max;
  int rc = RNNT_OK;
  h->last_persistent = use_persistent(h, p);
  if (h->last_persistent) {
    // one launch walks all steps (it starts with the prediction network on the start symbol itself)
    if ((rc = launch_persistent(h, s, p, max_steps))) return rc;
  } else {
  // prediction network on the start symbol (reads parity 1, writes parity 0), LM on the empty context
  if ((rc = launch_pred(h, s, p, 1, 0))) return rc;
  if ((rc = launch_lm(h, s, p))) return rc;
  const bool use_graph = c.use_graph && !h->profiling && !p.inj_tok && !p.plain;
  hipGraphExec_t exec = nullptr;
  if (use_graph) {
    // The captured kernel arguments hold the LM's device tables: the key carries the LM's unique id, not its
    // address, which a later LM may be given again.
    uint32_t lbits;
    memcpy(&lbits, &p.lambda, 4);
    rnnt_beam::GraphKey key(p.B, p.K, p.algo, p.T, p.lm ? lm_id(p.lm) : 0, lbits);
    auto it = h->graphs.find(key);
    if (it == h->graphs.end()) {
      hipStream_t cs;
      RB_HIP(h, hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
      hipGraph_t graph = nullptr;
      hipError_t e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
      if (e == hipSuccess) {
        for (int i = 0; i < kChunkSteps; ++i) {
          rc = launch_step(h, cs, p, i, i & 1, i == kChunkSteps - 1 ? kChunkSteps : 0);
          if (rc) break;
        }
        e = hipStreamEndCapture(cs, &graph);  // always ended, also after a failed launch
      }
      if (e == hipSuccess && !rc) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
      if (graph) hipGraphDestroy(graph);
      hipStreamDestroy(cs);
      if (rc) return rc;
      RB_HIP(h, e);
      if (h->graphs.size() >= kMaxGraphs) {  // drop the graph that was created first
        auto oldest = h->graphs.begin();
        for (auto g = h->graphs.begin(); g != h->graphs.end(); ++g)
          if (g->second.second < oldest->second.second) oldest = g;
        hipGraphExecDestroy(oldest->second.first);
        h->graphs.erase(oldest);
      }
      h->graphs[key] = std::make_pair(exec, h->graph_serial++);
    } else {
      exec = it->second.first;
    }
  }
  // The number of steps depends on the data.  Chunks of steps are enqueued ahead of the device; a pinned word
  // written by the selection tells the host when every utterance has finished, and kernels of steps enqueued
  // after that point return at once (the rest of the chunk that was running, and the one enqueued behind it).
  // `ahead`: the upper bound of steps is enqueued without looking at that word, so the call returns without waiting
  // for the device.
  // One chunk ahead of the device: the next chunk goes in while this one runs (a chunk takes 250 us and up, a graph
  // launch some 20 us of this thread); a step enqueued after the end costs about 7 us, a second chunk ahead 16 of
  // them.  The device reports the begin of a chunk through the second pinned word (bump_step): an event recorded
  // between two chunks would cost the stream 4-5 us each time.
  // The chunk behind the running one is held back until the running one is well under way (what the chunk before it
  // took says how long): a decode that ends in that first part is not followed by a chunk of steps that only find
  // out that there is nothing left to do.
  using HostClock = std::chrono::steady_clock;
  volatile int *host_done = h->h_done, *host_progress = h->h_done + kProgressWord;
  HostClock::time_point chunk_began{}, hold_until{};
  bool have_began = false, hold = false;
  int enq = 0, chunk_i = 0;
  while (enq < max_steps) {
    if (!p.ahead && hold)
      while (!*host_done && HostClock::now() < hold_until) {
      }
    if (!p.ahead && *host_done) break;
    if (use_graph) {
      RB_HIP(h, hipGraphLaunch(exec, s));
    } else {
      for (int i = 0; i < kChunkSteps; ++i)
        if ((rc = launch_step(h, s, p, i, i & 1, i == kChunkSteps - 1 ? kChunkSteps : 0))) return rc;
    }
    enq += kChunkSteps;
    if (!p.ahead && chunk_i >= 1) {
      // until the chunk enqueued just now begins, i.e. the one before it is over
      const int target = kChunkSteps * chunk_i;
      bool waited = false;
      const HostClock::time_point limit = HostClock::now() + std::chrono::milliseconds(kPaceLimitMs);
      while (!*host_done && *host_progress < target) {
        waited = true;
        // (no report in time: whatever is enqueued is waited for instead; from the third time on at once)
        if (h->pace_by_stream || HostClock::now() > limit) {
          RB_HIP(h, hipStreamSynchronize(s));
          if (h->trace_pacing) fprintf(stderr, "rnnt_beam: pacing fell back to the stream at chunk %d\n", chunk_i);
          if (++h->pace_misses >= 3) h->pace_by_stream = true;  // (a stall or two of the device changes nothing)
          break;
        }
      }
      // (a wait that found the chunk begun already: this thread is behind the device, and nothing is held back)
      const HostClock::time_point now = HostClock::now();
      hold = false;
      if (waited && have_began) {
        const auto took = now - chunk_began;
        const auto margin = std::max<HostClock::duration>(took * 2 / 5, std::chrono::microseconds(kEnqueueMarginUs));
        if (took > margin) {
          hold = true;
          hold_until = now + (took - margin);
        }
      }
      have_began = waited;
      chunk_began = now;
    }
    ++chunk_i;
  }
  }  // per-step launches
  {
    BacktraceArgs a;
    a.score = w.score;
    a.len = w.len;
    a.tree_parent = w.tree_parent;
    a.tree_token = w.tree_token;
    a.utt_steps = w.utt_steps;
    a.step_base = step_base;
    a.K = p.K;
    a.S_max = w.S_max;
    a.cap = p.out_cap ? p.out_cap : w.cap;
    const size_t lds = (size_t)w.S_max * p.K * 2 * sizeof(int);
    a.out_tokens = w.out_tokens; a.out_lens = w.out_lens; a.out_scores = w.out_scores; a.out_steps = w.out_steps;
    const bool own = p.ws == &h->ws;  // (the allocation-free entry point writes to the caller's arrays)
    if (own) {
      h->last_out = out_pack(p.B, p.K, a.cap);
      char *base = reinterpret_cast<char *>(w.ctrl);
      a.out_steps = reinterpret_cast<int *>(base + h->last_out.steps);
      a.out_lens = reinterpret_cast<int *>(base + h->last_out.lens);
      a.out_scores = reinterpret_cast<double *>(base + h->last_out.scores);
      a.out_tokens = reinterpret_cast<int *>(base + h->last_out.tokens);
    }
    ScopedKernelTime tm(h, s, KT_BACKTRACE);
    // (beside the tree the kernel holds 16.1 KB of tables in LDS)
    if (lds + 17 * 1024 <= (size_t)h->max_lds)
      hipLaunchKernelGGL(k_backtrace<true>, dim3(p.B), dim3(kBacktraceThreads), lds, s, a);
    else hipLaunchKernelGGL(k_backtrace<false>, dim3(p.B), dim3(kBacktraceThreads), 0, s, a);
    // flags and results to pinned host memory in one copy behind the back-trace: rnnt_beam_results then only waits
    if (own) RB_HIP(h, hipMemcpyAsync(h->h_out, w.ctrl, h->last_out.bytes, hipMemcpyDeviceToHost, s));
  }
  RB_HIP(h, hipGetLastError());
  RB_HIP(h, hipEventRecord(h->ev_end, s));
  h->have_result = true;
  h->last_B = p.B;
  h->last_K = p.K;
  h->last_T = p.T;
  h->last_stream = s;
  return RNNT_OK;
}

int check_shapes(rnnt_beam *h, int B, int T, int beam, int algo) {
  const rnnt_config_t &c = h->cfg;
  if (B < 1 || B > c.max_B) return fail(h, RNNT_E_ARG, "B outside 1..max_B");
  if (T < 1 || T > c.max_T) return fail(h, RNNT_E_ARG, "T outside 1..max_T");
  if (beam < 1 || beam > c.max_beam) return fail(h, RNNT_E_ARG, "beam outside 1..max_beam");
  if (algo != RNNT_ALSD && algo != RNNT_AES) return fail(h, RNNT_E_ARG, "unknown algo");
  return RNNT_OK;
}

int check_lm(rnnt_beam *h, const rnnt_lm_t *lm, int algo) {
  if (lm && lm_vocab(lm) != h->cfg.V) return fail(h, RNNT_E_ARG, "LM vocabulary differs from the model's");
  if (lm && algo == RNNT_AES && std::isfinite(h->cfg.prune_margin))
    return fail(h, RNNT_E_ARG, "an LM together with a finite prune margin is not supported");
  return RNNT_OK;
}

__global__ void k_copy_int(int *dst, const int *src, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) dst[i] = src[i];
}

}  // namespace

extern "C" {

int rnnt_beam_create(const rnnt_config_t *cfg, const rnnt_weights_t *w, rnnt_beam_t **out) try {
  if (out) *out = nullptr;
  if (!cfg || !w || !out || cfg->struct_size != sizeof(rnnt_config_t)) {
    g_create_error = "NULL argument or struct_size mismatch";
    return RNNT_E_ARG;
  }
  rnnt_beam *h = new (std::nothrow) rnnt_beam();
  if (!h) return RNNT_E_NOMEM;
  h->cfg = *cfg;
  const rnnt_config_t &c = h->cfg;
  auto bad = [&](const char *msg) {
    g_create_error = msg;
    delete h;
    return RNNT_E_ARG;
  };
  if (c.D < 32 || c.H < 32 || c.P < 32 || c.D % 32 || c.H % 32 || c.P % 32) return bad("D, H, P must be multiples of 32");
  if (c.V < 1 || c.V >= (1 << kFlatShift) - 1) return bad("V outside 1 .. 2^20 - 2");
  if (c.model != RNNT_MODEL_RNNT && c.model != RNNT_MODEL_TDT) return bad("unknown model");
  if (c.model == RNNT_MODEL_TDT && (c.n_durations < 1 || c.n_durations > 8)) return bad("TDT needs 1..8 durations");
  if (c.model == RNNT_MODEL_RNNT && c.n_durations != 0) return bad("n_durations must be 0 for RNN-T");
  if (c.model == RNNT_MODEL_TDT) {
    bool adv = false;
    for (int i = 0; i < c.n_durations; ++i) {
      if (c.durations[i] < 0) return bad("negative duration");
      if (c.durations[i] > 255) return bad("duration above 255 frames");
      adv |= c.durations[i] >= 1;
    }
    if (!adv) return bad("TDT needs a duration >= 1");
  }
  if (c.pred == RNNT_PRED_LSTM) {
    if (c.E < 32 || c.E % 32) return bad("E must be a multiple of 32");
    if (!w->emb || !w->W_ih || !w->W_hh || !w->b_ih || !w->b_hh) return bad("LSTM weights missing");
  } else if (c.pred == RNNT_PRED_STATELESS) {
    if (c.stateless_context < 1 || c.stateless_context > 4) return bad("stateless_context outside 1..4");
    if (!w->emb) return bad("embedding tables missing");
  } else {
    return bad("unknown prediction network");
  }
  if (!w->W_enc || !w->b_enc || !w->W_pred || !w->b_pred || !w->W_out || !w->b_out) return bad("joint weights missing");
  if (c.max_B < 1 || c.max_T < 1 || c.max_beam < 1 || c.max_beam > kMaxBeam) return bad("max_B/max_T/max_beam");
  if (c.max_symbols < 1) return bad("max_symbols < 1");
  if (c.lm_rule != 0 && c.lm_rule != 3 && c.lm_rule != 4) return bad("lm_rule must be 0, 3 or 4");
  if (c.tdt_all_pairs != 0 && c.tdt_all_pairs != 1) return bad("tdt_all_pairs must be 0 or 1");
  if (c.tdt_all_pairs && (c.model != RNNT_MODEL_TDT || c.max_beam > kPairsMaxBeam))
    return bad("tdt_all_pairs needs a TDT model and max_beam <= 8");
  if (c.lm_early_pruning != 0 && c.lm_early_pruning != 1) return bad("lm_early_pruning must be 0 or 1");
  if (!(c.prune_margin >= 0.f)) return bad("prune_margin must be >= 0 (INFINITY = off)");

  if (c.async_enqueue != 0 && c.async_enqueue != 1) return bad("async_enqueue must be 0 or 1");
  if (c.persistent_kernel != 0 && c.persistent_kernel != 1) return bad("persistent_kernel must be 0 or 1");
  if (c.aes_prefix_search != 0 && c.aes_prefix_search != 1) return bad("aes_prefix_search must be 0 or 1");
  if (c.aes_prefix_search && (c.tdt_all_pairs || c.lm_early_pruning))
    return bad("aes_prefix_search cannot be combined with tdt_all_pairs or lm_early_pruning");

  h->N = c.V + 1 + c.n_durations;
  h->n_chunks = (h->N + 31) / 32;
  h->M_max = c.max_B * c.max_beam;
  {
    const bool can = c.prec == RNNT_BF16_JOINT && c.pred == RNNT_PRED_STATELESS && c.V <= kRowWaves * 64 * 4 * kRowRegs &&
                     c.H % 16 == 0;
    if (c.joint_path == RNNT_JOINT_MATERIALIZED && !can)
      return bad("joint_path MATERIALIZED needs the bf16 joint, a stateless prediction network, V <= 8192, H % 16 == 0");
    if (c.joint_path < RNNT_JOINT_AUTO || c.joint_path > RNNT_JOINT_MATERIALIZED) return bad("unknown joint_path");
    h->big = can && (c.joint_path == RNNT_JOINT_MATERIALIZED ||
                     (c.joint_path == RNNT_JOINT_AUTO && c.V >= 2048 && c.max_B * c.max_beam >= 128));
    h->Npad_big = (c.V + 255) / 256 * 256;
    h->Hb = (c.H + 63) / 64 * 64;
  }
  int rc = RNNT_OK;
  auto A = [&](int r) {
    if (!rc) rc = r;
  };
  try {
    A(pack_weights(h, w));
    if (!rc) {
      const size_t bytes = layout_workspace(h->ws, nullptr, c, h->n_chunks, c.max_B, c.max_T, c.max_beam, true, h->big,
                                            h->Npad_big, h->Hb);
      char *base = nullptr;
      A(dev_alloc(h, &base, bytes));
      if (!rc) {
        layout_workspace(h->ws, base, c, h->n_chunks, c.max_B, c.max_T, c.max_beam, true, h->big, h->Npad_big, h->Hb);
        // (the padded k of the bf16 activations must read as zero; the control words start at zero)
        if (hipMemset(base, 0, bytes) != hipSuccess) rc = RNNT_E_HIP;
      }
    }
  } catch (const std::bad_alloc &) {
    h->err = "out of host memory";
    rc = RNNT_E_NOMEM;
  }
  if (!rc) {
    hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&h->h_done), 128, hipHostMallocMapped);
    if (e == hipSuccess) e = hipHostGetDevicePointer(reinterpret_cast<void **>(&h->h_done_dev), h->h_done, 0);
    h->h_out_bytes = out_pack(c.max_B, c.max_beam, h->ws.cap).bytes;
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&h->h_out), h->h_out_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreate(&h->ev_begin);
    if (e == hipSuccess) e = hipEventCreate(&h->ev_end);
    h->trace_pacing = getenv("RNNT_BEAM_TRACE_PACING") != nullptr;
    {
      int dev = 0, lds = 0;
      if (hipGetDevice(&dev) == hipSuccess &&
          hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && lds >= 64 * 1024)
        h->max_lds = lds;
    }
    if (e == hipSuccess && c.persistent_kernel) {
      // the single-launch loop needs every one of its blocks resident at once: one block per compute unit
      int dev = 0, n_cu = 0, per_cu = 0;
      e = hipGetDevice(&dev);
      if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
      if (e == hipSuccess && c.H == 640 && c.P == 640)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_decode_persistent<8, 10>, 512, 0);
      else if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_decode_persistent<8, 0>, 512, 0);
      h->n_cus = (e == hipSuccess && per_cu >= 1) ? n_cu : 0;
      void *q = nullptr;
      if (e == hipSuccess) e = hipMalloc(&q, sizeof(PersistCtl));
      if (e == hipSuccess) {
        h->allocs.push_back(q);
        h->pctl = static_cast<PersistCtl *>(q);
      }
    }
    if (e != hipSuccess) {
      h->err = std::string("create: ") + hipGetErrorString(e);
      rc = RNNT_E_HIP;
    }
  }
  if (rc) {
    g_create_error = h->err;
    rnnt_beam_destroy(h);
    return rc;
  }
  *out = h;
  return RNNT_OK;
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_HIP;
}

int rnnt_beam_decode(rnnt_beam_t *h, const float *enc, const int32_t *lengths, int32_t B, int32_t T, int32_t beam,
                     int32_t algo, const rnnt_lm_t *lm, float lm_weight, void *hip_stream) try {
  if (!h) return RNNT_E_ARG;
  if (!enc || !lengths) return fail(h, RNNT_E_ARG, "NULL enc or lengths");
  int rc = check_shapes(h, B, T, beam, algo);
  if (rc) return rc;
  if ((rc = check_lm(h, lm, algo))) return rc;
  StepPlan p{B, beam, T, algo, B * beam, lm, lm ? lm_weight : 0.f, nullptr, nullptr, 1};
  p.big = h->big && (h->cfg.joint_path == RNNT_JOINT_MATERIALIZED || B * beam >= 128);
  p.ws = &h->ws;
  p.ahead = h->cfg.async_enqueue != 0;
  return run_decode(h, enc, lengths, p, static_cast<hipStream_t>(hip_stream));
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_HIP;
}

int rnnt_beam_decode_static(rnnt_beam_t *h, const float *enc, const int32_t *lengths, int32_t B, int32_t T,
                            int32_t beam, int32_t algo, const rnnt_lm_t *lm, float lm_weight, int32_t *tokens,
                            int32_t cap, int32_t *lens, double *scores, int32_t *n_steps, int32_t *flags,
                            void *hip_stream) try {
  if (!h) return RNNT_E_ARG;
  if (!enc || !lengths || !tokens || !lens || !scores || !n_steps || cap < 1)
    return fail(h, RNNT_E_ARG, "NULL array or cap < 1");
  int rc = check_shapes(h, B, T, beam, algo);
  if (rc) return rc;
  if ((rc = check_lm(h, lm, algo))) return rc;
  // the static array of the current device (its address is looked up once per device)
  int dev = -1;
  RB_HIP(h, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(h, RNNT_E_ARG, "device index beyond the library's table");
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void *q = nullptr;
      RB_HIP(h, hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
      g_scratch_ptr[dev] = static_cast<char *>(q);
    }
  }
  Workspace ws;
  const size_t need = layout_workspace(ws, g_scratch_ptr[dev], h->cfg, h->n_chunks, B, T, beam, false, false, 0, 0);
  if (need > kScratchBytes)
    return fail(h, RNNT_E_ARG, "rnnt_beam_decode_static: B, T and beam need more than the 64 MiB static workspace");
  ws.out_tokens = tokens;
  ws.out_lens = lens;
  ws.out_scores = scores;
  ws.out_steps = n_steps;
  StepPlan p{B, beam, T, algo, B * beam, lm, lm ? lm_weight : 0.f, nullptr, nullptr, 1};
  p.big = false;  // the fused path only: the logits of the other path would not fit
  p.ws = &ws;
  p.ahead = true;
  p.plain = true;
  p.out_cap = cap;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  h->events_off = true;
  rc = run_decode(h, enc, lengths, p, s);
  h->events_off = false;
  h->have_result = false;  // the n-best lists went to the caller's arrays, not to the handle
  if (rc) return rc;
  if (flags) {
    hipLaunchKernelGGL(k_copy_int, dim3(1), dim3(64), 0, s, flags, ws.ctrl + 3, 2);
    RB_HIP(h, hipGetLastError());
  }
  return RNNT_OK;
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_HIP;
}

int rnnt_beam_decode_injected(rnnt_beam_t *h, const float *tok_logp, const float *dur_logp, int32_t C,
                              const int32_t *lengths, int32_t B, int32_t T, int32_t beam, int32_t algo,
                              void *hip_stream) try {
  if (!h) return RNNT_E_ARG;
  if (!tok_logp || !lengths || C < 1) return fail(h, RNNT_E_ARG, "NULL table or lengths, or C < 1");
  if (h->cfg.n_durations > 0 && !dur_logp) return fail(h, RNNT_E_ARG, "TDT needs dur_logp");
  int rc = check_shapes(h, B, T, beam, algo);
  if (rc) return rc;
  StepPlan p{B, beam, T, algo, B * beam, nullptr, 0.f, tok_logp, dur_logp, C};
  p.ws = &h->ws;
  return run_decode(h, nullptr, lengths, p, static_cast<hipStream_t>(hip_stream));
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_HIP;
}

int rnnt_beam_results(rnnt_beam_t *h, int32_t *tokens, int32_t cap, int32_t *lens, double *scores,
                      int32_t *n_steps) try {
  if (!h) return RNNT_E_ARG;
  if (!h->have_result) return fail(h, RNNT_E_NORESULT, "no decode has been run");
  RB_HIP(h, hipStreamSynchronize(h->last_stream));
  const Workspace &w = h->ws;
  const int B = h->last_B, K = h->last_K;
  // (the decode left flags and results in pinned memory, see run_decode)
  const OutPack &o = h->last_out;
  const int *flags = reinterpret_cast<const int *>(h->h_out) + 3;
  const int *p_lens = reinterpret_cast<const int *>(h->h_out + o.lens);
  if (lens) memcpy(lens, p_lens, sizeof(int) * B * K);
  if (scores) memcpy(scores, h->h_out + o.scores, sizeof(double) * B * K);
  if (n_steps) memcpy(n_steps, h->h_out + o.steps, sizeof(int) * B);
  if (tokens && cap > 0) {
    const int *buf = reinterpret_cast<const int *>(h->h_out + o.tokens);
    for (size_t i = 0; i < (size_t)B * K; ++i) {
      const int n = p_lens[i] < cap ? p_lens[i] : cap;
      if (n > 0) memcpy(tokens + i * cap, buf + i * w.cap, sizeof(int) * n);
    }
  }
  if (h->last_persistent) {
    int ab = 0;
    RB_HIP(h, hipMemcpy(&ab, &h->pctl->abort, sizeof(int), hipMemcpyDeviceToHost));
    if (ab == 1) return fail(h, RNNT_E_HIP, "single-launch step loop: a wait between blocks ran into its limit (results invalid)");
    if (ab == 2) return fail(h, RNNT_E_HIP, "single-launch step loop: blocks not spread evenly over the XCDs (results invalid)");
  }
  if (flags[1]) return fail(h, RNNT_E_NONFINITE, "NaN or Inf in the encoder projection");
  if (flags[0]) return fail(h, RNNT_E_ARG, "an utterance length was outside 0..T (clamped)");
  return RNNT_OK;
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_HIP;
}

int rnnt_beam_dump_tree(rnnt_beam_t *h, int32_t *parent, int32_t *token, int32_t *merged_into, int32_t s_cap) try {
  if (!h) return RNNT_E_ARG;
  if (!h->have_result) return fail(h, RNNT_E_NORESULT, "no decode has been run");
  RB_HIP(h, hipStreamSynchronize(h->last_stream));
  const Workspace &w = h->ws;
  const int B = h->last_B, K = h->last_K;
  std::vector<int> steps(B);
  memcpy(steps.data(), h->h_out + h->last_out.steps, sizeof(int) * B);
  const int *src[3] = {w.tree_parent, w.tree_token, w.tree_merged};
  int32_t *dst[3] = {parent, token, merged_into};
  std::vector<int> buf((size_t)w.S_max * K);
  for (int a = 0; a < 3; ++a) {
    if (!dst[a]) continue;
    for (size_t i = 0; i < (size_t)s_cap * B * K; ++i) dst[a][i] = -9;
    for (int b = 0; b < B; ++b) {
      RB_HIP(h, hipMemcpy(buf.data(), src[a] + (size_t)b * w.S_max * K, sizeof(int) * buf.size(),
                          hipMemcpyDeviceToHost));
      for (int st = 0; st < steps[b] && st < s_cap; ++st)
        for (int k = 0; k < K; ++k) dst[a][((size_t)st * B + b) * K + k] = buf[(size_t)st * K + k];
    }
  }
  return RNNT_OK;
} catch (const std::bad_alloc &) {
  return RNNT_E_NOMEM;
} catch (...) {
  return RNNT_E_HIP;
}

int rnnt_beam_debug_encproj(rnnt_beam_t *h, float *out, int64_t n_floats) {
  if (!h || !out) return RNNT_E_ARG;
  if (!h->have_result) return fail(h, RNNT_E_NORESULT, "no decode has been run");
  RB_HIP(h, hipStreamSynchronize(h->last_stream));
  const int64_t n = (int64_t)h->last_B * h->last_T * h->cfg.H;
  if (n_floats < n) return fail(h, RNNT_E_ARG, "buffer too small");
  RB_HIP(h, hipMemcpy(out, h->ws.f_proj, sizeof(float) * n, hipMemcpyDeviceToHost));
  return RNNT_OK;
}

int rnnt_beam_debug_block_map(int32_t a_tiles, int32_t a_m, int32_t b_begin, int32_t b_end, int32_t b_m, int32_t *role,
                              int32_t *ntile, int32_t *mtile, int32_t cap) {
  if (a_tiles < 0 || a_m < 0 || b_begin < 0 || b_end < b_begin || b_m < 0) return RNNT_E_ARG;
  XcdMap m;
  m.a_tiles = a_tiles; m.a_m = a_m; m.b_begin = b_begin; m.b_end = b_end; m.b_m = b_m;
  const int grid = xcd_grid(m);
  for (int bid = 0; bid < grid && bid < cap; ++bid) {
    int n = -1, mt = -1;
    const int r = xcd_item(m, bid, n, mt);
    if (role) role[bid] = r;
    if (ntile) ntile[bid] = r < 0 ? -1 : n;
    if (mtile) mtile[bid] = r < 0 ? -1 : mt;
  }
  return grid;
}

float rnnt_beam_last_decode_ms(rnnt_beam_t *h) {
  if (!h || !h->have_result) return -1.f;
  if (hipEventSynchronize(h->ev_end) != hipSuccess) return -1.f;
  float ms = -1.f;
  if (hipEventElapsedTime(&ms, h->ev_begin, h->ev_end) != hipSuccess) return -1.f;
  return ms;
}

int rnnt_beam_debug_set_spin_limit(rnnt_beam_t *h, int32_t polls) {
  if (!h || polls < 1) return RNNT_E_ARG;
  h->spin_limit = polls;
  return RNNT_OK;
}

int rnnt_beam_set_profiling(rnnt_beam_t *h, int32_t on) {
  if (!h) return RNNT_E_ARG;
  h->profiling = on != 0;
  return RNNT_OK;
}

int rnnt_beam_kernel_times(rnnt_beam_t *h, const char **names, float *ms, int32_t *calls, int32_t n_cap) {
  if (!h) return RNNT_E_ARG;
  if (!h->prof_launches.empty()) {
    if (h->last_stream || h->have_result) RB_HIP(h, hipStreamSynchronize(h->last_stream));
    for (const auto &l : h->prof_launches) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, h->prof_events[l.second], h->prof_events[l.second + 1]) == hipSuccess) {
        h->timers[l.first].ms += t;
        h->timers[l.first].calls += 1;
      }
    }
    h->prof_launches.clear();
  }
  int n = 0;
  for (int i = 0; i < KT_COUNT && n < n_cap; ++i) {
    if (names) names[n] = h->timers[i].name ? h->timers[i].name : kKernelNames[i];
    if (ms) ms[n] = h->timers[i].ms;
    if (calls) calls[n] = h->timers[i].calls;
    ++n;
  }
  return n;
}

const char *rnnt_beam_last_error(const rnnt_beam_t *h) { return h ? h->err.c_str() : g_create_error.c_str(); }

void rnnt_beam_destroy(rnnt_beam_t *h) {
  if (!h) return;
  hipDeviceSynchronize();
  for (auto &kv : h->graphs) hipGraphExecDestroy(kv.second.first);
  for (void *p : h->allocs) hipFree(p);
  if (h->h_done) hipHostFree(h->h_done);
  if (h->h_out) hipHostFree(h->h_out);
  hipEvent_t evs[] = {h->ev_begin, h->ev_end};
  for (hipEvent_t e : h->prof_events) hipEventDestroy(e);
  for (hipEvent_t e : evs)
    if (e) hipEventDestroy(e);
  delete h;
}

}  // extern "C"
