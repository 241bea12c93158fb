// Kernels of the per-step beam expansion (gfx950).  One step of the loop is
//   k_step_main (joint + selection in its tail + part of W_hh h) -> k_lstm_pointwise -> k_pred_proj (+ LM rows)
// for LSTM models (k_stateless_pre instead of the last two for stateless ones; k_inject -> k_select when the
// log-probabilities are injected; a stand-alone k_select / k_select_wide / k_select_pairs where the tail cannot
// take the selection), and k_gemm_tiled (gemm.h) / k_init / k_backtrace run once per decode call.
#pragma once
#include <type_traits>

#include "device_utils.h"
#include "lm_device.h"

namespace rb {

// ---------------------------------------------------------------------------
// Split-K 32 x 32 tile shared by the three per-step contractions.  The WAVES
// waves of a block each take a slice of K and leave their partial tile in LDS;
// tile_value() then sums the partials of one output element, so that the
// epilogues can spread over every thread of the block instead of one wave
// (these kernels are bound by the instruction latency of their longest wave).
// a_at(k) / b_at(k) return 4 consecutive k of this lane's row of the "output
// row" / "hypothesis" operand.
// ITERS > 0: K == WAVES * ITERS * 8 and every load is issued before the first
// matrix instruction; ITERS == 0: any K with K % (8 * WAVES) == 0, plain loop.
// red: WAVES * 64 * 17 floats of LDS (lane-major, padded: conflict-free both ways).
// ---------------------------------------------------------------------------
constexpr int kRedStride = 17;

// Operand registers of one wave: ITERS > 0 keeps every 16-byte load of the wave's K slice in flight at once.
template <int ITERS>
struct SplitKOperands {
  float4 a[ITERS > 0 ? ITERS : 1], b[ITERS > 0 ? ITERS : 1];
};

// issue the loads (ITERS > 0 only; the plain loop of ITERS == 0 loads as it goes)
template <int WAVES, int ITERS, class AL, class BL>
__device__ __forceinline__ void splitk_load(SplitKOperands<ITERS> &op, AL a_at, BL b_at, int K) {
  if constexpr (ITERS > 0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
    const int kbeg = wave * (K / WAVES) + 4 * half;
    // pairwise, in the order the matrix instructions consume them: loads complete in order, so the first
    // instructions can start after the first pair instead of after all of one operand
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
      op.a[i] = a_at(kbeg + 8 * i);
      op.b[i] = b_at(kbeg + 8 * i);
    }
  }
}

// matrix instructions of the wave's K slice, partial tile to LDS, block barrier.
// fb: applied to each hypothesis-side operand just before use (ReLU).
// bf16 (uniform over the block): both operands are rounded to bfloat16 (weights handed in are bf16 values already)
// and two 8-k rounds at a time go through one bf16 matrix instruction, an eighth of the matrix-core time of the
// eight float32 ones; the accumulation stays float32.
// xw (ITERS > 0 only): this lane's k values of one more output row; the lane's part of that row's product with its
// hypothesis goes into the spare float of its slot in red (extra_value() sums the parts).
template <int WAVES, int ITERS, class AL, class BL, class FB>
__device__ __forceinline__ void splitk_mma(SplitKOperands<ITERS> &op, AL a_at, BL b_at, FB fb, int K, float *red,
                                           int bf16 = 0, const float4 *xw = nullptr) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int kw = K / WAVES;
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if constexpr (ITERS > 0) {
    if (bf16) {
#pragma unroll
      for (int i = 0; i < ITERS; i += 2) {
        const bool two = i + 1 < ITERS;
        acc = mfma32_bf16_from_f32(op.a[i], two ? op.a[i + 1 < ITERS ? i + 1 : i] : zero4, fb(op.b[i]),
                                   two ? fb(op.b[i + 1 < ITERS ? i + 1 : i]) : zero4, acc);
      }
    } else {
#pragma unroll
      for (int i = 0; i < ITERS; ++i) {
        const float4 b = fb(op.b[i]);
        acc = mfma32(op.a[i].x, b.x, acc);
        acc = mfma32(op.a[i].y, b.y, acc);
        acc = mfma32(op.a[i].z, b.z, acc);
        acc = mfma32(op.a[i].w, b.w, acc);
      }
    }
  } else {
    const int kbeg = wave * kw + 4 * half, kend = (wave + 1) * kw;
    if (bf16) {
      for (int k = kbeg; k < kend; k += 16) {
        const bool two = k + 8 < kend;
        const int k2 = two ? k + 8 : k;
        const float4 a0 = a_at(k), a1 = a_at(k2), b0 = fb(b_at(k)), b1 = fb(b_at(k2));
        acc = mfma32_bf16_from_f32(a0, two ? a1 : zero4, b0, two ? b1 : zero4, acc);
      }
    } else {
      for (int k = kbeg; k < kend; k += 8) {
        const float4 a = a_at(k);
        const float4 b = fb(b_at(k));
        acc = mfma32(a.x, b.x, acc);
        acc = mfma32(a.y, b.y, acc);
        acc = mfma32(a.z, b.z, acc);
        acc = mfma32(a.w, b.w, acc);
      }
    }
  }
  float *mine = red + (wave * 64 + lane) * kRedStride;
#pragma unroll
  for (int r = 0; r < 16; ++r) mine[r] = acc[r];
  if constexpr (ITERS > 0) {
    if (xw) {
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < ITERS; ++i) {
        float4 b = fb(op.b[i]);
        if (bf16) {  // (the weights are bf16 values already)
          b.x = __uint_as_float(pack_bf16_rne(b.x, 0.f) << 16);
          b.y = __uint_as_float(pack_bf16_rne(b.y, 0.f) << 16);
          b.z = __uint_as_float(pack_bf16_rne(b.z, 0.f) << 16);
          b.w = __uint_as_float(pack_bf16_rne(b.w, 0.f) << 16);
        }
        part = fmaf(xw[i].x, b.x, part);
        part = fmaf(xw[i].y, b.y, part);
        part = fmaf(xw[i].z, b.z, part);
        part = fmaf(xw[i].w, b.w, part);
      }
      mine[16] = part;
    }
  }
  __syncthreads();
}

// the extra row's product with hypothesis j (see splitk_mma)
template <int WAVES>
__device__ __forceinline__ float extra_value(const float *red, int j) {
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) s += red[(w * 64 + j) * kRedStride + 16] + red[(w * 64 + 32 + j) * kRedStride + 16];
  return s;
}

// element (output row i, hypothesis j) of the finished 32 x 32 tile
template <int WAVES>
__device__ __forceinline__ float tile_value(const float *red, int i, int j) {
  const int r = 4 * (i >> 3) + (i & 3), src = ((i >> 2) & 1) * 32 + j;
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) s += red[(w * 64 + src) * kRedStride + r];
  return s;
}

// Sorted list of the KT best (key, index) pairs seen by one lane.
template <int KT>
struct TopList {
  float v[KT];
  int i[KT];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      v[j] = -INFINITY;
      i[j] = 0x7fffffff;
    }
  }
  __device__ __forceinline__ void insert(float key, int idx) {
    if (!comes_before(key, idx, v[KT - 1], i[KT - 1])) return;
    v[KT - 1] = key;
    i[KT - 1] = idx;
#pragma unroll
    for (int j = KT - 1; j > 0; --j) {
      if (comes_before(v[j], i[j], v[j - 1], i[j - 1])) {
        const float tv = v[j];
        v[j] = v[j - 1];
        v[j - 1] = tv;
        const int ti = i[j];
        i[j] = i[j - 1];
        i[j - 1] = ti;
      }
    }
  }
};

// Operand layout of the per-step contractions ("k4-major"): element (row, k) of a
// matrix with R rows sits at ((k / 4) * R + row) * 4 + k % 4.  A wave's 16-byte
// loads of 32 consecutive rows at one k then cover whole cache lines (512 B
// contiguous per half-wave), for weights and activations alike.
__host__ __device__ inline size_t k4_index(int k, int row, int rows) {
  return ((size_t)(k >> 2) * rows + row) * 4 + (k & 3);
}

// Injected mode: the candidate lists come from a table of log-probabilities
// instead of the joint network.  One wave per hypothesis; lane l fills "chunk" l.
struct InjectArgs {
  const float *tok_logp;  // [B, T, C, V + 1]
  const float *dur_logp;  // [B, T, C, ND] or NULL
  int C;
  const int *t;
  const uint32_t *hash;
  const int *lengths;
  int M, K, T, V, ND;
  uint64_t *p_cand;
  float *zs;
  const int *done;
};

template <int KT>
__global__ __launch_bounds__(64) void k_inject(InjectArgs a) {
  if (*reinterpret_cast<const volatile int *>(a.done)) return;
  const int m = blockIdx.x, lane = threadIdx.x;
  const int b = m / a.K;
  const int T_b = a.lengths[b];
  int tt = a.t[m];
  tt = tt < T_b ? tt : T_b - 1;
  tt = tt < 0 ? 0 : tt;
  const int cls = (int)(a.hash[m] % (uint32_t)a.C);
  const float *row = a.tok_logp + (((size_t)b * a.T + tt) * a.C + cls) * (a.V + 1);
  TopList<KT> top;
  top.init();
  for (int v = lane; v < a.V; v += 64) top.insert(row[v], v);
#pragma unroll
  for (int j = 0; j < KT; ++j)
    if (j < a.K) a.p_cand[((size_t)m * a.K + j) * 64 + lane] = pack_cand(top.v[j], top.i[j]);
  const int nz = 1 + a.ND;
  if (lane == 0) a.zs[(size_t)m * nz] = row[a.V];
  if (lane >= 1 && lane <= a.ND)
    a.zs[(size_t)m * nz + lane] = a.dur_logp[(((size_t)b * a.T + tt) * a.C + cls) * a.ND + lane - 1];
}

// ---------------------------------------------------------------------------
// Selection, tree write, state update and recombination: one block per utterance.
// ---------------------------------------------------------------------------
struct SelectArgs {
  // hypothesis state, [M] each (ctx: [M][kCtxMax])
  double *score;
  int *t, *sym, *len, *last;
  uint32_t *hash;
  int *ctx;
  const int *lengths;
  // candidate lists from the joint (k_step_main, k_row_select) or k_inject
  const float *p_max, *p_sum;
  const uint64_t *p_cand;  // [M, K, n_chunks] packed (key, token): entry j of every chunk's list (best first) side by
                           // side, so that lanes that take neighbouring chunks read neighbouring words
  const float *zs;
  int n_chunks;
  int use_ctx;     // 1: the token history of each hypothesis is kept (stateless prediction network, LM)
  int normalized;  // 1: keys are log-probabilities already (injected mode)
  // configuration
  int B, K, V, ND;
  int dur[8];
  uint64_t dur_bytes;   // the same, one byte each (durations are at most 255): one scalar register pair instead of eight
  int algo, max_sym;
  float gamma;
  int has_lm;
  int lm_rule3;         // 1: Eq. (3) (LM on tokens only, blank as it is); 0: Eq. (4)
  int lm_early;         // 1: early pruning: keys carry no LM term; the kept candidates are charged it here
  int prefix;           // 1: AES++ maximum-length prefix search (ranking credit, see select_utterance)
  const float *lm_rows; // [M, V] natural-log LM scores (read for the kept candidates under early pruning)
  float lambda;
  // what the prediction step has to do for each new slot
  int *src_row, *tok;
  // tree [B][S_max][K]
  int *tree_parent, *tree_token, *tree_merged;
  int S_max;
  // loop control
  const int *step_base;
  int step_off;
  int *finished, *utt_steps, *n_finished, *done;
  volatile int *h_done;  // pinned host word, set when every utterance has finished
};

// Where the selection finds the candidate lists of its utterance: the arrays of SelectArgs (rows indexed by
// hypothesis), or arrays in LDS that hold the rows of this utterance only (row0 = its first hypothesis).
struct CandView {
  const uint64_t *cand;
  const float *pmax, *psum, *zs;
  int row0;
};
__device__ __forceinline__ CandView cand_view(const SelectArgs &a) { return CandView{a.p_cand, a.p_max, a.p_sum, a.zs, 0}; }

__device__ __forceinline__ float logaddexp_f(float a, float b) {
  const float m = fmaxf(a, b), d = fminf(a, b) - m;  // d <= 0
  return d > -INFINITY ? m + log1pf(expf(d)) : m;
}

// LDS scratch of one wave while it handles one utterance
template <int CAND, int STAIR = 64>
struct SelectScratchT {
  static constexpr int kStair = STAIR;  // candidates the staircase form of the ranking can hold (64 per lane pass)
  double score[kMaxBeam];
  double rc_val[CAND];
  double rc_key[CAND];  // early pruning only: what the candidates are ranked by
  double sel_val[kMaxBeam];
  double n_score[kMaxBeam];
  double delta[kMaxBeam];  // prefix search: what the ranking adds to every candidate of the hypothesis
  int t[kMaxBeam], sym[kMaxBeam], len[kMaxBeam], last[kMaxBeam], kind[kMaxBeam];
  uint32_t hash[kMaxBeam];
  int ctx[kMaxBeam][kCtxMax];
  int advt[kMaxBeam], advb[kMaxBeam];
  int rc_flat[CAND];
  int sel_flat[kMaxBeam];
  // staircase form of the ranking (beams 8 .. 10): per hypothesis the place of blank in its sorted list, its head,
  // the order of the lists by their heads; then the K (K + 1) / 2 candidates that can still be among the Beam best
  double head_val[kMaxBeam], st_key[STAIR + 8];
  int head_flat[kMaxBeam], pos_blank[kMaxBeam], ord[kMaxBeam], st_flat[STAIR + 8], st_src[STAIR];
  int n_t[kMaxBeam], n_sym[kMaxBeam], n_len[kMaxBeam], n_last[kMaxBeam], n_live[kMaxBeam];
  uint32_t n_hash[kMaxBeam];
};
// K (K + 1) candidates per utterance: K tokens and blank / stay of every hypothesis
typedef SelectScratchT<kMaxBeam * (kMaxBeam + 1)> SelectScratch;
// the same with room for the staircase of beams up to 16 (16 * 17 / 2 = 136 candidates, three per lane)
typedef SelectScratchT<kMaxBeam * (kMaxBeam + 1), 192> SelectScratchWide;
// TDT with every (symbol, duration) pair as a candidate: K (K + 1) ND of them, for beams up to 8
constexpr int kPairsMaxBeam = 8;
typedef SelectScratchT<kPairsMaxBeam * (kPairsMaxBeam + 1) * 8> SelectScratchPairs;

// the lanes of one wave see each other's LDS writes after this (they run in lockstep; this
// only stops the compiler and the memory pipeline from re-ordering)
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// candidate order inside an utterance: (hypothesis k, token v) -> k * 2^20 + v, the same order as
// k * (V + 1) + v for V < 2^20, without a division on the way back
constexpr int kFlatShift = 20;

// x mod (2^31 - 1) for x < 2^62
__device__ __forceinline__ uint32_t mod_mersenne31(uint64_t x) {
  uint64_t y = (x & kHashMod) + (x >> 31);
  y = (y & kHashMod) + (y >> 31);
  return (uint32_t)(y >= kHashMod ? y - kHashMod : y);
}

// Rank of the calling lane's candidate (value mv, index mf) among the cnt candidates in LDS: the number of those that
// come before it.  Every lane reads all candidates (the same address in all lanes: broadcasts, many in flight), eight
// at a time; the arrays hold eight entries beyond cnt that come before nothing.  First on the values alone (one
// comparison per candidate): when no two finite values are equal, which the sum of the counts tells, that is the
// rank; otherwise once more in the full order (value, then index).
__device__ __forceinline__ int rank_by_counting(const double *keys, const int *flats, int cnt, double mv, int mf) {
  int ge = 0;  // candidates not below mine, myself included
  for (int c0 = 0; c0 < cnt; c0 += 8) {
    double cv[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) cv[q] = keys[c0 + q];
#pragma unroll
    for (int q = 0; q < 8; ++q) ge += (int)(cv[q] >= mv);
  }
  const bool finite = mv > -INFINITY;
  const int F = __popcll(__ballot(finite));
  if (wave_sum_i(finite ? ge : 0) == F * (F + 1) / 2) return ge - 1;
  int rank = 0;
  for (int c0 = 0; c0 < cnt; c0 += 8) {
    double cv[8];
    int cf[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      cv[q] = keys[c0 + q];
      cf[q] = flats[c0 + q];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) rank += comes_before_count(cv[q], cf[q], mv, mf);
  }
  return rank;
}

// The same for OWN candidates per lane (lane, lane + 64, ..): one pass over the candidates serves them all.
template <int OWN>
__device__ __forceinline__ void rank_by_counting_n(const double *keys, const int *flats, int cnt, const double (&mv)[OWN],
                                                   const int (&mf)[OWN], int (&rank)[OWN]) {
  int ge[OWN];
#pragma unroll
  for (int o = 0; o < OWN; ++o) ge[o] = 0;
  for (int c0 = 0; c0 < cnt; c0 += 8) {
    double cv[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) cv[q] = keys[c0 + q];
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int o = 0; o < OWN; ++o) ge[o] += (int)(cv[q] >= mv[o]);
  }
  int F = 0, tot = 0;
#pragma unroll
  for (int o = 0; o < OWN; ++o) {
    const bool finite = mv[o] > -INFINITY;
    F += __popcll(__ballot(finite));
    tot += finite ? ge[o] : 0;
  }
  if (wave_sum_i(tot) == F * (F + 1) / 2) {
#pragma unroll
    for (int o = 0; o < OWN; ++o) rank[o] = ge[o] - 1;
    return;
  }
#pragma unroll
  for (int o = 0; o < OWN; ++o) rank[o] = 0;
  for (int c0 = 0; c0 < cnt; c0 += 8) {
    double cv[8];
    int cf[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      cv[q] = keys[c0 + q];
      cf[q] = flats[c0 + q];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int o = 0; o < OWN; ++o) rank[o] += comes_before_count(cv[q], cf[q], mv[o], mf[o]);
  }
}

// One beam-search step of utterance b by one wave: the K best tokens and blank of every
// hypothesis (LPR lanes per hypothesis, all hypotheses at once), the Beam best of those,
// expansion, tree write, recombination, end-of-utterance detection.
// NCH > 0: a lane keeps the lists of NCH chunks in registers (n_chunks <= LPR * NCH, K <= KMAX) and
// the K best of the hypothesis come out of a K-way merge of list heads; NCH == 0: the lists are
// scanned in memory at every round instead (any size).
// MULTI: the beam may be wider than the 64 / LPR hypotheses handled at once; the per-hypothesis part then
// runs in several passes.
// PAIRS (TDT): every (symbol, duration) pair of a hypothesis is a candidate of its own (blank only with
// durations >= 1) instead of one duration per symbol; candidate (k, j, d) sits at ((k (K + 1) + j) ND + d.
// ONE: every hypothesis comes with exactly one list (n_chunks == 1, NCH == 1), known at compile time: the merge
// of list heads and its registers drop out.
template <int LPR, int NCH, int KMAX, bool MULTI = false, bool PAIRS = false, class Scratch = SelectScratch,
          bool ONE = false, int PLAIN = 0, bool DYNDUR = false>
__device__ __forceinline__ void select_utterance(const SelectArgs &a, int b, Scratch &s, const CandView cv) {
  const int K = a.K, V = a.V, lane = threadIdx.x & 63;
  // PLAIN (the caller has checked): 1 = ALSD++, 2 = AES++ without prune margin and prefix search, both without
  // durations and LM: the code of the other cases drops out
  const int a_ND = PLAIN ? 0 : a.ND;
  const int a_has_lm = PLAIN ? 0 : a.has_lm, a_lm_early = PLAIN ? 0 : a.lm_early, a_lm_rule3 = PLAIN ? 0 : a.lm_rule3;
  const int a_prefix = PLAIN ? 0 : a.prefix;
  const float a_gamma = PLAIN ? INFINITY : a.gamma;
  const int a_algo = PLAIN ? PLAIN - 1 : a.algo;
  const int m_base = b * K;
  const int nz = 1 + a_ND;
  // ---- every load of the prologue is requested before anything waits on one of them
  const int fin = load_agent(a.finished + b);  // (a wave-uniform word that changes: never through the scalar cache)
  const int S = *a.step_base + a.step_off;
  const int T_b = a.lengths[b];
  double my_score = -INFINITY;
  int my_t = 0, my_sym = 0, my_len = 0, my_last = -1;
  uint32_t my_hash = 0;
  if (lane < K) {
    const int m = m_base + lane;
    my_score = a.score[m];
    my_t = a.t[m];
    my_sym = a.sym[m];
    my_len = a.len[m];
    my_last = a.last[m];
    my_hash = a.hash[m];
  }
  // LPR lanes per hypothesis, 64 / LPR hypotheses at once; a beam wider than that takes several passes
  // over the per-hypothesis part (lists -> K best tokens -> candidate scores in LDS)
  constexpr int kRowsPerPass = 64 / LPR;
  const int e = lane % LPR;  // position inside the lane group
  const int ncand = a.n_chunks * K;
  int rk = 0;                // hypothesis of this lane in the current pass
  bool row_ok = false;
  const uint64_t *cands = nullptr;
  const float *pmax = nullptr, *psum = nullptr;
  uint64_t list[NCH > 0 ? NCH : 1][KMAX];
  float pm[NCH > 0 ? NCH : 1], ps[NCH > 0 ? NCH : 1];
  float zb = 0.f;
  float dl[8];
  // a single chunk's list IS the K best of the hypothesis: lane e takes entries e, e + LPR, .. as they are
  constexpr int kMine = (KMAX + LPR - 1) / LPR;
  const bool one_list = ONE || (NCH == 1 && a.n_chunks == 1);
  uint64_t direct[kMine];
  auto load_rows = [&](int r0) {
    rk = r0 + lane / LPR;
    row_ok = rk < K;
    const int krow = row_ok ? rk : 0;
    const int crow = m_base - cv.row0 + krow;
    cands = cv.cand + (size_t)crow * ncand;
    pmax = cv.pmax + (size_t)crow * a.n_chunks;
    psum = cv.psum + (size_t)crow * a.n_chunks;
    const float *zsr = cv.zs + (size_t)crow * nz;
    // (every load is unconditional, from a clamped address, and what does not apply is replaced afterwards: a load
    // under a condition of its own costs a branch each)
    if constexpr (NCH > 0) {
#pragma unroll
      for (int q = 0; q < NCH; ++q) {
        const int ch = e + LPR * q;
        const bool ok = row_ok && ch < a.n_chunks;
        const int chs = min(ch, a.n_chunks - 1);  // (lanes without a chunk repeat their group's last address: no extra line)
        if constexpr (!ONE) {
          if (!one_list) {
#pragma unroll
            for (int j = 0; j < KMAX; ++j) {
              const uint64_t x = load_agent(cands + (j < K ? j : 0) * a.n_chunks + chs);
              list[q][j] = (ok && j < K) ? x : no_cand();
            }
          }
        }
        const float xm = load_agent(pmax + chs), xs = load_agent(psum + chs);
        pm[q] = (ok && !a.normalized) ? xm : -INFINITY;
        ps[q] = (ok && !a.normalized) ? xs : 0.f;
      }
      if (one_list) {
#pragma unroll
        for (int i = 0; i < kMine; ++i) {
          const int j = e + LPR * i;
          const uint64_t x = load_agent(cands + (j < K ? j : 0));
          direct[i] = (row_ok && j < K) ? x : no_cand();
        }
      }
    }
    zb = load_agent(zsr);
    if (a_ND > 0) {
#pragma unroll
      for (int d = 0; d < 8; ++d) dl[d] = load_agent(zsr + 1 + (d < a_ND ? d : 0));
    }
  };
  auto process_rows = [&]() {
    // ---- K rounds of "best remaining candidate" in every lane group at once.
    // Lane e keeps the winners of rounds e, e + LPR, ... (at most KMAX / LPR + 1 of them).
    uint64_t mine[kMine];
#pragma unroll
    for (int i = 0; i < kMine; ++i) mine[i] = no_cand();
    if (one_list) {
#pragma unroll
      for (int i = 0; i < kMine; ++i) mine[i] = direct[i];
    } else if constexpr (ONE) {
    } else if constexpr (NCH > 0) {
#pragma unroll
      for (int j = 0; j < KMAX; ++j) {
        if (j < K) {
          uint64_t best = list[0][0];
#pragma unroll
          for (int q = 1; q < NCH; ++q) best = list[q][0] > best ? list[q][0] : best;
          best = group_max_u64<LPR>(best);
#pragma unroll
          for (int q = 0; q < NCH; ++q)
            if (list[q][0] == best) {  // the winner's list moves up (real candidates are unique)
#pragma unroll
              for (int x = 0; x + 1 < KMAX; ++x) list[q][x] = list[q][x + 1];
              list[q][KMAX - 1] = no_cand();
            }
          if (e == j % LPR) mine[j / LPR] = best;
        }
      }
    } else {
      uint64_t last = ~0ull;
      for (int j = 0; j < K; ++j) {
        uint64_t best = no_cand();
        if (row_ok)
          for (int c = e; c < ncand; c += LPR) {
            const uint64_t v = load_agent(cands + c);
            if (v < last && v > best) best = v;
          }
        best = group_max_u64<LPR>(best);
#pragma unroll
        for (int i = 0; i < kMine; ++i)
          if (e == j % LPR && i == j / LPR) mine[i] = best;
        last = best > no_cand() ? best : no_cand() + 1;  // nothing below "no candidate" is eligible again
      }
    }
    // ---- soft-max statistics of the hypothesis (float transcendental math, scores accumulate in double)
    float lse_all = 0.f, lse_nb = 0.f, max_nb = -INFINITY;
    if (!a.normalized) {
      float st_mx = -INFINITY, st_sum = 0.f;
      if constexpr (NCH > 0) {
#pragma unroll
        for (int q = 0; q < NCH; ++q) st_mx = fmaxf(st_mx, pm[q]);
        st_mx = group_max<LPR>(st_mx);
#pragma unroll
        for (int q = 0; q < NCH; ++q)
          if (pm[q] > -INFINITY) st_sum += ps[q] * __expf(pm[q] - st_mx);
      } else {
        if (row_ok)
          for (int c = e; c < a.n_chunks; c += LPR) st_mx = fmaxf(st_mx, load_agent(pmax + c));
        st_mx = group_max<LPR>(st_mx);
        if (row_ok)
          for (int c = e; c < a.n_chunks; c += LPR) {
            const float p = load_agent(pmax + c);
            if (p > -INFINITY) st_sum += load_agent(psum + c) * __expf(p - st_mx);
          }
      }
      st_sum = group_sum<LPR>(st_sum);
      lse_nb = st_mx + __logf(st_sum);
      const float hi = fmaxf(lse_nb, zb), lo = fminf(lse_nb, zb);
      lse_all = hi + __logf(1.f + __expf(lo - hi));
      max_nb = st_mx;
    } else {
      // keys are log-probabilities already; the best token of the row is round 0's winner, the largest
      // of the winners spread over the group's lanes
      max_nb = cand_key(group_max_u64<LPR>(mine[0]));
    }
    const double logp_b = (double)zb - (double)lse_all;
    const double nb = (double)lse_nb - (double)lse_all;
    const double maxlogp = (double)fmaxf(max_nb, zb) - (double)lse_all;
    // TDT durations
    double x_tok = 0.0, x_blank = 0.0;
    int adv_tok = 0, adv_blank = 1;
    if (a_ND > 0) {
      if constexpr (DYNDUR) {
        // The form with indices computed at run time (every access a dependent load: 2.4 us at five durations).  Kept
        // for the main kernel's instantiation for 256 slots and more, where the selection is not what the launch
        // waits for and the kernel as a whole came out 0.9 us SLOWER with the form below (its joint blocks end 0.8 us
        // later: the compiler's placement of the whole kernel, not this block's own time).
        if (!a.normalized) {
          float dmx = -INFINITY, sm = 0.f;
          for (int d = 0; d < a_ND; ++d) dmx = fmaxf(dmx, dl[d]);
          for (int d = 0; d < a_ND; ++d) sm += __expf(dl[d] - dmx);
          const float l = dmx + __logf(sm);
          for (int d = 0; d < a_ND; ++d) dl[d] -= l;
        }
        int best = -1, best_b = -1;
        for (int d = 0; d < a_ND; ++d) {
          if (best < 0 || dl[d] > dl[best]) best = d;
          if (a.dur[d] >= 1 && (best_b < 0 || dl[d] > dl[best_b])) best_b = d;
        }
        if constexpr (!PAIRS) {
          x_tok = (double)dl[best];
          x_blank = (double)dl[best_b];
          adv_tok = a.dur[best];
          adv_blank = a.dur[best_b];
        }
      } else {
        // (every index into dl and a.dur below is a compile-time constant: an index computed at run time turns each
        // access into a dependent load from memory, 2.4 us for this block at five durations)
        if (!a.normalized) {
          float dmx = -INFINITY, sm = 0.f;
#pragma unroll
          for (int d = 0; d < 8; ++d)
            if (d < a_ND) dmx = fmaxf(dmx, dl[d]);
#pragma unroll
          for (int d = 0; d < 8; ++d)
            if (d < a_ND) sm += __expf(dl[d] - dmx);
          const float l = dmx + __logf(sm);
#pragma unroll
          for (int d = 0; d < 8; ++d)
            if (d < a_ND) dl[d] -= l;
        }
        // the most likely duration (the first of equal ones), and the most likely one that advances
        bool have = false, have_b = false;
        float best_v = 0.f, best_bv = 0.f;
        int best_adv = 0, best_badv = 1;
#pragma unroll
        for (int d = 0; d < 8; ++d)
          if (d < a_ND) {
            const int du = (int)((a.dur_bytes >> (8 * d)) & 0xff);
            if (!have || dl[d] > best_v) {
              have = true;
              best_v = dl[d];
              best_adv = du;
            }
            if (du >= 1 && (!have_b || dl[d] > best_bv)) {
              have_b = true;
              best_bv = dl[d];
              best_badv = du;
            }
          }
        if constexpr (!PAIRS) {  // one duration per candidate: the most likely one (for blank: that advances)
          x_tok = (double)best_v;
          x_blank = (double)best_bv;
          adv_tok = best_adv;
          adv_blank = best_badv;
        }
      }
    }
    wave_sync();  // s.kind / s.score / s.sym are needed per row from here on
    // candidate c of the utterance is rc[k * (K + 1) + j]: j < K tokens, j == K blank / stay
    if (row_ok) {
      const int kind = s.kind[rk];
      const bool forced = s.sym[rk] >= a.max_sym;
      const bool use_gamma = a_algo == 1 && a_gamma < INFINITY;
      const double thr = maxlogp - (double)a_gamma;
      const double sc = s.score[rk];
      const int flat0 = rk << kFlatShift;
      // Eq. (4): tokens get lambda (ln(1 - p_blank) + lm), blank (1 + lambda) ln p_blank; Eq. (3): tokens lambda lm,
      // blank unchanged.  Late pruning: lambda * lm is in the key already; early: added here, after the ranking value.
      const double lm_const = (a_has_lm && !a_lm_rule3) ? (double)a.lambda * nb : 0.0;
      const double tok_base = x_tok - (double)lse_all;
      const bool early = a_lm_early != 0;
      // where candidate (hypothesis rk, j-th symbol[, duration d]) goes and how it is numbered for the tie-break
      const int nd = PAIRS ? a_ND : 1;
      auto put = [&](int j, int token, double key, double val) {
        if constexpr (PAIRS) {
          for (int d = 0; d < nd; ++d) {
            // blank must advance by at least one frame; a waiting hypothesis is the single candidate d = 0
            const bool ok = key > -INFINITY && (kind == 1 ? d == 0 : (token < V || a.dur[d] >= 1));
            const double x = kind == 1 ? 0.0 : (double)dl[d];
            const int c = (rk * (K + 1) + j) * nd + d;
            s.rc_val[c] = ok ? val + x : -INFINITY;
            if (early) s.rc_key[c] = ok ? key + x : -INFINITY;
            s.rc_flat[c] = ((flat0 + token) << 3) | d;
          }
        } else {
          const int c = rk * (K + 1) + j;
          s.rc_val[c] = val;
          if (early) s.rc_key[c] = key;
          s.rc_flat[c] = flat0 + token;
        }
      };
#pragma unroll
      for (int i = 0; i < kMine; ++i) {
        const int j = e + LPR * i;
        if (j < K) {
          const float wk = cand_key(mine[i]);
          const int wi = cand_idx(mine[i]);
          double val = -INFINITY, key = -INFINITY;
          if (kind == 2 && wk > -INFINITY && !forced) {
            const double lp = (double)wk - (double)lse_all;  // pre-LM log-probability when no LM is in the key
            if (!(use_gamma && lp < thr)) {
              key = sc + (double)wk + tok_base;
              val = key + lm_const;
              if (early) val += (double)a.lambda * (double)a.lm_rows[(size_t)(m_base + rk) * V + wi];
            }
          }
          put(j, wi < V ? wi : V - 1, key, val);
        }
      }
      if (e == LPR - 1) {  // blank / stay: the group's last lane (least loaded with winners)
        double val = -INFINITY, key = -INFINITY;
        if (kind == 2) {
          double bl = logp_b;
          if (use_gamma && logp_b < thr && !forced) bl = -INFINITY;
          key = sc + bl + x_blank;
          val = (a_has_lm && !a_lm_rule3 && bl > -INFINITY) ? key + (double)a.lambda * bl : key;
          s.advt[rk] = adv_tok;
          s.advb[rk] = adv_blank;
        } else if (kind == 1) {
          val = key = sc;  // a waiting or finished hypothesis stays as it is
        }
        put(K, V, key, val);
      }
    }
    wave_sync();
  };
  auto per_utterance = [&]() -> bool {  // false: the utterance had finished before this step
    if (a.use_ctx)
      for (int i = lane; i < K * kCtxMax; i += 64) s.ctx[i / kCtxMax][i % kCtxMax] = a.ctx[m_base * kCtxMax + i];
    if (fin) {  // a finished utterance is frozen; its slots tell the prediction step to copy
      if (lane < K) {
        store_through(a.src_row + m_base + lane, m_base + lane);
        store_through(a.tok + m_base + lane, -1);
      }
      return false;
    }
    if (lane < K) {
      s.score[lane] = my_score;
      s.t[lane] = my_t;
      s.sym[lane] = my_sym;
      s.len[lane] = my_len;
      s.last[lane] = my_last;
      s.hash[lane] = my_hash;
      s.sel_val[lane] = -INFINITY;
      s.sel_flat[lane] = -1;
    }
    // frame of the earliest unfinished hypothesis (lanes >= K hold neutral values)
    const bool my_live = my_score > -INFINITY;
    int t_cur = group_min_i<16>((my_live && my_t < T_b) ? my_t : T_b);
    t_cur = __builtin_amdgcn_readlane(t_cur, 0);
    if (lane < K) s.kind[lane] = my_live ? ((my_t < T_b && (a_algo == 0 || my_t == t_cur)) ? 2 : 1) : 0;
    return true;
  };
  if constexpr (MULTI) {
    for (int r0 = 0; r0 < K; r0 += kRowsPerPass) {
      load_rows(r0);
      if (r0 == 0 && !per_utterance()) return;
      process_rows();
    }
  } else {
    load_rows(0);
    if (!per_utterance()) return;
    process_rows();
  }

  const int n = K * (K + 1) * (PAIRS ? a_ND : 1);
  // ---- AES++, maximum-length prefix search (Sec. 2.2, "AES").  Hypotheses i and j expanded at this step in the
  // same frame with transcript(i) = transcript(j) + v: the step's own expansion (j, v), if it is among j's Beam best
  // tokens and stays in the frame, is credited to i for the RANKING of i's candidates; the new scores stay as they
  // are (the expansion competes on its own and meets i in the recombination; adding it to i's score too would count
  // that alignment twice).  Pairs are found through Eq. (1), like equal transcripts in the recombination.
  const bool prefix = !PAIRS && a_prefix && a_algo == 1 && !a_lm_early;
  if constexpr (!PAIRS) {
    if (prefix) {
      if (lane < K) {
        const int i = lane;
        double add = -INFINITY;
        if (s.kind[i] == 2 && s.len[i] >= 1) {
          const uint32_t hi = s.hash[i];
          const int li = s.len[i], la = s.last[i], ti = s.t[i];
          for (int j = 0; j < K; ++j) {
            if (j == i || s.kind[j] != 2 || s.t[j] != ti || s.len[j] + 1 != li) continue;
            if (s.advt[j] != 0) continue;
            if (mod_mersenne31((uint64_t)s.hash[j] * kHashBase + (uint64_t)(la + 1)) != hi) continue;
            for (int c = 0; c < K; ++c) {  // j's Beam best tokens: is v among them, with a finite score?
              const int idx = j * (K + 1) + c;
              if (s.rc_flat[idx] == (j << kFlatShift) + la && s.rc_val[idx] > -INFINITY) add = logaddexp_d(add, s.rc_val[idx]);
            }
          }
        }
        s.delta[i] = add > -INFINITY ? logaddexp_d(s.score[i], add) - s.score[i] : 0.0;
      }
      wave_sync();
      for (int c = lane; c < n; c += 64) s.rc_key[c] = s.rc_val[c] + s.delta[c / (K + 1)];
      wave_sync();
    }
  }
  // ---- the Beam best of all K * (K + 1) candidates, by (ranking value desc, (k, v) asc); the ranking
  // value is the new score itself except under early pruning and with a prefix credit
  double *rank_of = (a_lm_early || prefix) ? s.rc_key : s.rc_val;
  // candidates a lane may own in the counting form below
  constexpr int kOwn = 1;  // (measured: from 65 candidates up the rounds below are faster than two owned candidates)
  if (n <= 64 * kOwn) {
    // Each lane counts, for each candidate it owns (lane, lane + 64, ..), how many candidates come before it; that
    // count is the candidate's new slot.  (Every lane reads all n candidates back from LDS, the same address in all
    // lanes: such reads are broadcasts and, unlike lane reads into scalar registers, can be requested many at a time.)
    double mv[kOwn];
    int mf[kOwn], rank[kOwn];
#pragma unroll
    for (int q = 0; q < kOwn; ++q) {
      const int c = lane + 64 * q;
      mv[q] = c < n ? rank_of[c] : -INFINITY;
      mf[q] = c < n ? s.rc_flat[c] : 0x7fffffff;
      rank[q] = 0;
    }
    // the loop below reads in eights: the (up to seven) places after the last candidate hold one that comes before
    // nothing, so that no comparison needs a bound check (the arrays have room beyond n; nothing else uses it)
    if (lane < 8) {
      rank_of[n + lane] = -INFINITY;
      s.rc_flat[n + lane] = 0x7fffffff;
    }
    wave_sync();
    rank[0] = rank_by_counting(rank_of, s.rc_flat, n, mv[0], mf[0]);
#pragma unroll
    for (int q = 0; q < kOwn; ++q)
      if (mv[q] > -INFINITY && rank[q] < K) {
        s.sel_val[rank[q]] = s.rc_val[lane + 64 * q];
        s.sel_flat[rank[q]] = mf[q];
      }
  } else if (!PAIRS && KMAX > 7 && K * (K + 1) / 2 <= Scratch::kStair) {
    // More than 64 candidates.  The candidates of one hypothesis are a sorted list: its tokens come
    // best first (the ranking value grows with the key) and blank / stay has its place among them.  With the lists
    // ordered by their heads, the entry at place p of the list of order o has at least p + o candidates ahead of it,
    // so only the K (K + 1) / 2 entries with p + o < K can be among the Beam best, and an entry's rank among those
    // is its rank among all whenever that is below K.  One to three per lane, and the counting form applies.
    if (lane < K) {
      const int base = lane * (K + 1);
      const double bv = rank_of[base + K];
      int pos = 0;
#pragma unroll
      for (int j = 0; j < KMAX; ++j) {  // (reads past the K tokens stay inside the array and are not counted)
        const double tv = rank_of[base + j];
        pos += (int)(j < K) & (int)(tv > -INFINITY) & (int)(tv >= bv);  // (equal values: the token comes first)
      }
      s.pos_blank[lane] = pos;
      s.head_val[lane] = pos == 0 ? bv : rank_of[base];
      s.head_flat[lane] = pos == 0 ? s.rc_flat[base + K] : s.rc_flat[base];
    }
    wave_sync();
    if (lane < K) {
      const double hv = s.head_val[lane];
      const int hf = s.head_flat[lane];
      int o = 0;
#pragma unroll
      for (int r = 0; r < KMAX; ++r) o += (int)(r < K) & comes_before_count(s.head_val[r], s.head_flat[r], hv, hf);
      s.ord[lane] = o;
    }
    wave_sync();
    const unsigned inv = 65536u / (unsigned)(K + 1) + 1u;  // c / (K + 1) for c < 272 without a division per lane
    for (int c = lane; c < n; c += 64) {
      const int r = (int)(((unsigned)c * inv) >> 16), j = c - r * (K + 1);
      const int pb = s.pos_blank[r], o = s.ord[r];
      const int p = j == K ? pb : (j < pb ? j : j + 1);
      if (p + o < K) {
        const int slot = o * K - o * (o - 1) / 2 + p;
        s.st_key[slot] = rank_of[c];
        s.st_flat[slot] = s.rc_flat[c];
        s.st_src[slot] = c;
      }
    }
    const int nn = K * (K + 1) / 2;
    if (lane < 8) {  // (as above: the counting loop reads in eights)
      s.st_key[nn + lane] = -INFINITY;
      s.st_flat[nn + lane] = 0x7fffffff;
    }
    wave_sync();
    // (candidates a lane owns: as many as the form's widest beam needs and the scratch holds)
    constexpr int kNeed = (KMAX * (KMAX + 1) / 2 + 63) / 64, kHave = Scratch::kStair / 64;
    constexpr int OWN = kNeed < kHave ? kNeed : kHave;
    double mv[OWN];
    int mf[OWN], rank[OWN];
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      const int slot = lane + 64 * o;
      mv[o] = slot < nn ? s.st_key[slot] : -INFINITY;
      mf[o] = slot < nn ? s.st_flat[slot] : 0x7fffffff;
      rank[o] = K;
    }
    if (OWN == 1 || nn <= 64) rank[0] = rank_by_counting(s.st_key, s.st_flat, nn, mv[0], mf[0]);
    else rank_by_counting_n<OWN>(s.st_key, s.st_flat, nn, mv, mf, rank);
#pragma unroll
    for (int o = 0; o < OWN; ++o)
      if (mv[o] > -INFINITY && rank[o] < K) {
        s.sel_val[rank[o]] = s.rc_val[s.st_src[lane + 64 * o]];
        s.sel_flat[rank[o]] = mf[o];
      }
  } else {
    double last_v = INFINITY;
    int last_i = -1;
    for (int j = 0; j < K; ++j) {
      double bv = -INFINITY;
      int bi = 0x7fffffff;
      for (int c = lane; c < n; c += 64) {
        const double v = rank_of[c];
        const int i = s.rc_flat[c];
        const bool eligible = v > -INFINITY && (v < last_v || (v == last_v && i > last_i));
        if (eligible && comes_before(v, i, bv, bi)) {
          bv = v;
          bi = i;
        }
      }
      wave_best(bv, bi);
      if (!(bv > -INFINITY)) break;
      for (int c = lane; c < n; c += 64)  // the candidate's own lane hands over its score ((k, v) is unique)
        if (s.rc_flat[c] == bi && rank_of[c] == bv) {
          s.sel_val[j] = s.rc_val[c];
          s.sel_flat[j] = bi;
        }
      last_v = bv;
      last_i = bi;
    }
  }
  wave_sync();

  // ---- expansion into the new slots
  int code = -3, parent = -1, appended = -1;
  int ctx_new[kCtxMax];
  if (lane < K) {
    const int j = lane;
    const double val = s.sel_val[j];
#pragma unroll
    for (int i = 0; i < kCtxMax; ++i) ctx_new[i] = -1;
    if (!(val > -INFINITY)) {
      s.n_live[j] = 0;
      s.n_score[j] = -INFINITY;
      s.n_t[j] = 0;
      s.n_sym[j] = 0;
      s.n_len[j] = 0;
      s.n_last[j] = -1;
      s.n_hash[j] = 0;
    } else {
      const int kv = PAIRS ? s.sel_flat[j] >> 3 : s.sel_flat[j];
      const int k = kv >> kFlatShift, v = kv & ((1 << kFlatShift) - 1);
      const int adv_b = PAIRS ? a.dur[s.sel_flat[j] & 7] : s.advb[k];  // frames the step advances: the pair's own
      const int adv_t = PAIRS ? a.dur[s.sel_flat[j] & 7] : s.advt[k];  // duration, or the hypothesis' chosen one
      parent = k;
      int t = s.t[k], sym = s.sym[k], len = s.len[k], last = s.last[k];
      uint32_t hash = s.hash[k];
      if (a.use_ctx) {
#pragma unroll
        for (int i = 0; i < kCtxMax; ++i) ctx_new[i] = s.ctx[k][i];
      }
      if (s.kind[k] == 1) {
        code = -2;
      } else if (v == V) {
        code = -1;
        t += adv_b;
        sym = 0;
      } else {
        code = v;
        appended = v;
        len += 1;
        last = v;
        hash = mod_mersenne31((uint64_t)hash * kHashBase + (uint64_t)(v + 1));
        t += adv_t;
        sym = adv_t == 0 ? sym + 1 : 0;
#pragma unroll
        for (int i = kCtxMax - 1; i > 0; --i) ctx_new[i] = ctx_new[i - 1];
        ctx_new[0] = v;
      }
      if (t > T_b) t = T_b;
      s.n_live[j] = 1;
      s.n_score[j] = val;
      s.n_t[j] = t;
      s.n_sym[j] = sym;
      s.n_len[j] = len;
      s.n_last[j] = last;
      s.n_hash[j] = hash;
    }
  }
  wave_sync();

  // ---- recombination: equal (hash, length, last token, frame, symbols in frame)
  if (lane < K) {
    const int j = lane;
    int merged = -1;
    double score = s.n_score[j];
    bool live = s.n_live[j] != 0;
    if (live) {
      // which slots hold the same (hash, length, last token, frame, symbols in frame): all keys are read without
      // branches in between, so that the LDS reads go out together
      const uint32_t mh = s.n_hash[j];
      const int ml = s.n_len[j], mla = s.n_last[j], mt = s.n_t[j], ms = s.n_sym[j];
      // (the hashes first, read without branches in between; the other fields only of the few slots whose hash is equal)
      uint32_t same_hash = 0;
#pragma unroll
      for (int i = 0; i < KMAX; ++i) {
        const bool e = (i < K) & (s.n_live[i] != 0) & (s.n_hash[i] == mh);
        same_hash |= (uint32_t)e << i;
      }
      uint32_t same = 1u << j;
      for (uint32_t r = same_hash & ~(1u << j); r; r &= r - 1u) {
        const int i = __builtin_ctz(r);
        const bool e = (s.n_len[i] == ml) & (s.n_last[i] == mla) & (s.n_t[i] == mt) & (s.n_sym[i] == ms);
        same |= (uint32_t)e << i;
      }
      const uint32_t lower = same & ((1u << j) - 1u);
      if (lower == 0) {  // the lowest slot of its class keeps the log-sum, added up in slot order
        merged = j;
        for (uint32_t higher = same & ~((2u << j) - 1u); higher; higher &= higher - 1u)
          score = logaddexp_d(score, s.n_score[__builtin_ctz(higher)]);
      } else {
        merged = __builtin_ctz(lower);
        live = false;
        score = -INFINITY;
      }
    }
    const int m = m_base + j;
    // written through (see store_through): nothing of a step's results waits in an L2 for the kernel's end
    store_through(a.score + m, score);
    store_through(a.t + m, s.n_t[j]);
    store_through(a.sym + m, s.n_sym[j]);
    store_through(a.len + m, s.n_len[j]);
    store_through(a.last + m, s.n_last[j]);
    store_through(a.hash + m, s.n_hash[j]);
    if (a.use_ctx) {
#pragma unroll
      for (int i = 0; i < kCtxMax; ++i) {
        store_through(a.ctx + m * kCtxMax + i, ctx_new[i]);
        s.ctx[j][i] = ctx_new[i];  // (every read of the parents' histories lies before the last wave_sync)
      }
    }
    store_through(a.src_row + m, parent >= 0 ? m_base + parent : m);
    store_through(a.tok + m, appended);
    if (S < a.S_max) {
      const size_t ti = ((size_t)b * a.S_max + S) * K + j;
      store_through(a.tree_parent + ti, parent);
      store_through(a.tree_token + ti, code);
      store_through(a.tree_merged + ti, merged);
    }
    // finished when no surviving slot has frames left
    const bool open = live && s.n_t[j] < T_b;
    const unsigned long long any_open = __ballot(open);
    if (j == 0 && (any_open == 0ull || S + 1 >= T_b * (a.max_sym + 1))) {
      store_through(a.finished + b, 1);
      store_through(a.utt_steps + b, S + 1);
      __threadfence();
      const int old = atomicAdd(a.n_finished, 1);
      if (old + 1 == a.B) {
        *reinterpret_cast<volatile int *>(a.done) = 1;
        __threadfence_system();
        *a.h_done = 1;
      }
    }
  }
  wave_sync();
}

// picks the lane-group width and register budget for the beam and list sizes at hand.
// FORMS: 4 = one list per hypothesis, known at compile time (tail of the row kernel of the materialised-logits path);
// 0 = beams up to 8 (what the main kernel of a step runs in its tail); 1 = those plus wider beams
// whose hypotheses come with a single list; 2 = wider beams with many lists (several passes, many
// registers).  The heavy forms are kept out of the kernels that do not need them.
template <int FORMS, class Scratch = SelectScratch>
__device__ __forceinline__ void select_dispatch(const SelectArgs &a, int b, Scratch &s, const CandView cv) {
  if constexpr (FORMS == 12 || FORMS == 16) {  // FORMS == 4 on a plain RNN-T (no durations, no LM): 12 for AES++
    constexpr int P = FORMS == 12 ? 2 : 1;      // without prune margin and prefix search, 16 for ALSD++
    if (a.K <= 4) select_utterance<16, 1, 4, false, false, Scratch, true, P>(a, b, s, cv);
    else if (a.K <= 8) select_utterance<8, 1, 8, false, false, Scratch, true, P>(a, b, s, cv);
    else if (a.K <= 12) select_utterance<4, 1, 12, false, false, Scratch, true, P>(a, b, s, cv);
    else select_utterance<4, 1, 16, false, false, Scratch, true, P>(a, b, s, cv);
  } else if constexpr (FORMS == 4) {  // one list per hypothesis (the materialised-logits path), any beam
    if (a.K <= 4) select_utterance<16, 1, 4, false, false, Scratch, true>(a, b, s, cv);
    else if (a.K <= 8) select_utterance<8, 1, 8, false, false, Scratch, true>(a, b, s, cv);
    else if (a.K <= 12) select_utterance<4, 1, 12, false, false, Scratch, true>(a, b, s, cv);
    else select_utterance<4, 1, 16, false, false, Scratch, true>(a, b, s, cv);
  } else if constexpr (FORMS == 3) {  // TDT, every (symbol, duration) pair a candidate, beams up to 8
    if (a.K <= 4) {
      if (a.n_chunks <= 16 * 3) select_utterance<16, 3, 4, false, true, Scratch>(a, b, s, cv);
      else select_utterance<16, 0, 4, false, true, Scratch>(a, b, s, cv);
    } else {
      if (a.n_chunks <= 8 * 5) select_utterance<8, 5, 8, false, true, Scratch>(a, b, s, cv);
      else select_utterance<8, 0, 8, false, true, Scratch>(a, b, s, cv);
    }
  } else if constexpr (FORMS == 17) {  // forms 5 and 6 with the durations' older code (see select_utterance)
    select_utterance<16, 3, 4, false, false, Scratch, false, 0, true>(a, b, s, cv);
  } else if constexpr (FORMS == 18) {
    select_utterance<8, 5, 8, false, false, Scratch, false, 0, true>(a, b, s, cv);
  } else if constexpr (FORMS == 5) {  // one form alone (the caller has checked 2 < K <= 4, n_chunks <= 48) ...
    select_utterance<16, 3, 4>(a, b, s, cv);
  } else if constexpr (FORMS == 11) {  // ... the same for ALSD++ on a plain RNN-T (no durations, no LM): beams 3, 4,
    select_utterance<16, 3, 4, false, false, Scratch, false, 1>(a, b, s, cv);
  } else if constexpr (FORMS == 13) {  // ... 1, 2 (n_chunks <= 48),
    select_utterance<16, 3, 2, false, false, Scratch, false, 1>(a, b, s, cv);
  } else if constexpr (FORMS == 14) {  // ... 5 to 8 (n_chunks <= 40);
    select_utterance<8, 5, 8, false, false, Scratch, false, 1>(a, b, s, cv);
  } else if constexpr (FORMS == 15) {  // AES++ without prune margin and prefix search on a plain RNN-T, beams 3, 4
    select_utterance<16, 3, 4, false, false, Scratch, false, 2>(a, b, s, cv);
  } else if constexpr (FORMS == 6) {  // ... (4 < K <= 8, n_chunks <= 40): a kernel a third the size
    select_utterance<8, 5, 8>(a, b, s, cv);
  } else if constexpr (FORMS == 2) {
    if (a.n_chunks <= 16 * 3) select_utterance<16, 3, 16, true>(a, b, s, cv);  // four hypotheses per pass
    else select_utterance<4, 0, 16>(a, b, s, cv);
  } else {
    if (a.K <= 2 && a.n_chunks <= 16 * 3) {  // (a form of its own: the lists are loaded and merged KMAX entries wide)
      select_utterance<16, 3, 2>(a, b, s, cv);
    } else if (a.K <= 4) {
      if (a.n_chunks <= 16 * 3) select_utterance<16, 3, 4>(a, b, s, cv);
      else select_utterance<16, 0, 4>(a, b, s, cv);
    } else if (a.K <= 8) {
      if (a.n_chunks <= 8 * 5) select_utterance<8, 5, 8>(a, b, s, cv);
      else select_utterance<8, 0, 8>(a, b, s, cv);
    } else if constexpr (FORMS == 1) {
      select_utterance<4, 1, 16>(a, b, s, cv);
    }
  }
}
template <int FORMS, class Scratch = SelectScratch>
__device__ __forceinline__ void select_dispatch(const SelectArgs &a, int b, Scratch &s) {
  select_dispatch<FORMS, Scratch>(a, b, s, cand_view(a));
}
// which stand-alone selection kernel takes a beam of K with n_chunks lists per hypothesis
__host__ __device__ inline bool select_needs_wide_forms(int K, int n_chunks) { return K > 8 && n_chunks > 4; }

// Block -> work item, aware of the eight XCDs.  Workgroup i of a launch runs on XCD i % 8, and each
// XCD has its own L2.  A launch has up to two roles, each a grid of (n-tile, m-tile) items; every
// item of an n-tile (one 32-row slice of a weight matrix) is given to the XCD  n-tile % 8, so that a
// slice is only ever read through one L2 and stays there from one step to the next.
struct XcdMap {
  int a_tiles, a_m;          // role 0: n-tiles [0, a_tiles) x a_m m-tiles
  int b_begin, b_end, b_m;   // role 1: n-tiles [b_begin, b_end) x b_m m-tiles
};
__host__ __device__ inline int xcd_role_a_tiles(const XcdMap &m, int x) {
  return m.a_tiles > x ? (m.a_tiles - x + 7) / 8 : 0;
}
__host__ __device__ inline int xcd_role_b_first(const XcdMap &m, int x) {
  return m.b_begin + ((x - m.b_begin) % 8 + 8) % 8;
}
__host__ __device__ inline int xcd_role_b_tiles(const XcdMap &m, int x) {
  const int t0 = xcd_role_b_first(m, x);
  return m.b_end > t0 ? (m.b_end - t0 + 7) / 8 : 0;
}
// number of blocks to launch: eight times the largest per-XCD item count
__host__ inline int xcd_grid(const XcdMap &m) {
  int most = 0;
  for (int x = 0; x < 8; ++x) {
    const int n = xcd_role_a_tiles(m, x) * m.a_m + xcd_role_b_tiles(m, x) * m.b_m;
    most = n > most ? n : most;
  }
  return 8 * most;
}
// role of block `bid` (0, 1, or -1 = nothing to do) and its item
__host__ __device__ __forceinline__ int xcd_item(const XcdMap &m, int bid, int &ntile, int &mtile) {
  const int x = bid & 7;
  int s = bid >> 3;
  const int na = xcd_role_a_tiles(m, x) * m.a_m;
  if (s < na) {
    ntile = x + 8 * (s / m.a_m);
    mtile = s % m.a_m;
    return 0;
  }
  s -= na;
  if (s < xcd_role_b_tiles(m, x) * m.b_m) {
    ntile = xcd_role_b_first(m, x) + 8 * (s / m.b_m);
    mtile = s % m.b_m;
    return 1;
  }
  return -1;
}

// R[m] = W_hh h[m] for one tile of 32 gate rows x the 32 current slots from m0 on (it does not depend on the
// selection, so its blocks ride along in the launches that have idle compute units).
struct RecurrentArgs {
  const float *Whh;    // k4-major [P][4P], gate rows re-ordered (NULL: no such blocks)
  const float *h;      // k4-major [P][Mp]
  float *R;            // [M][4P]
  int P, M, Mp;
  int group;           // slot tiles per block (1, or kRecGroup: the map's items are then groups of slot tiles)
};
constexpr int kRecGroup = 4;

template <int WAVES, int ITERS>
__device__ __forceinline__ void recurrent_tile(const RecurrentArgs &a, int tile, int m0, int done, float *red) {
  constexpr int LPH = 2 * WAVES, VPL = 32 / LPH;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31;
  const int R4 = 4 * a.P, Mp = a.Mp;
  const float *wp = a.Whh + (size_t)(tile * 32 + col) * 4;
  const float *hp = a.h + (size_t)(m0 + col) * 4;
  auto a_at = [&](int k) { return *reinterpret_cast<const float4 *>(wp + (size_t)(k >> 2) * R4 * 4); };
  auto b_at = [&](int k) { return *reinterpret_cast<const float4 *>(hp + (size_t)(k >> 2) * Mp * 4); };
  auto fb = [](float4 v) { return v; };
  SplitKOperands<ITERS> op;
  splitk_load<WAVES, ITERS>(op, a_at, b_at, a.P);
  if (done) return;
  splitk_mma<WAVES, ITERS>(op, a_at, b_at, fb, a.P, red);
  // thread -> (slot j, VPL adjacent rows of the tile)
  const int j = tid / LPH, i0 = (tid % LPH) * VPL;
  const int m = m0 + j;
  if (m < a.M) {
#pragma unroll
    for (int q = 0; q < VPL; ++q) store_through(a.R + (size_t)m * R4 + tile * 32 + i0 + q, tile_value<WAVES>(red, i0 + q, j));
  }
}

// The same for up to G slot tiles in a row (item `grp` of the tile's row: slot tiles grp * G ...): the 32 gate rows
// stay in registers, and the slots of the next tile are requested before the matrix instructions of the current one
// start, so that a block streams half as much per tile and streams while it multiplies.
template <int WAVES, int ITERS, int G>
__device__ __forceinline__ void recurrent_tiles(const RecurrentArgs &a, int tile, int grp, int done, float *red) {
  static_assert(ITERS > 0, "every load of a slice in flight at once");
  constexpr int LPH = 2 * WAVES, VPL = 32 / LPH;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, wave = tid >> 6, half = lane >> 5;
  const int R4 = 4 * a.P, Mp = a.Mp;
  const int m_tiles = (a.M + 31) / 32;
  const int t0 = grp * a.group, n_mt = m_tiles - t0 < a.group ? m_tiles - t0 : a.group;
  const int kbeg = wave * (a.P / WAVES) + 4 * half;
  const float *wp = a.Whh + (size_t)(tile * 32 + col) * 4 + (size_t)(kbeg >> 2) * R4 * 4;
  const float *hp = a.h + (size_t)(t0 * 32 + col) * 4 + (size_t)(kbeg >> 2) * Mp * 4;
  float4 wa[ITERS], hb[2][ITERS];
#pragma unroll
  for (int i = 0; i < ITERS; ++i) {
    wa[i] = *reinterpret_cast<const float4 *>(wp + (size_t)(2 * i) * R4 * 4);
    hb[0][i] = *reinterpret_cast<const float4 *>(hp + (size_t)(2 * i) * Mp * 4);
  }
  if (done) return;
  const int j = tid / LPH, i0 = (tid % LPH) * VPL;
  // one slot tile; G copies of this code, each with its register set known at compile time (a loop over g that can
  // end early is kept as a loop by the compiler, with the next tile's loads waited for one by one inside it).
  // (Reading the previous tile's sums back beside this tile's matrix instructions, from a second buffer, was slower:
  // its stores then sit between the loads in the order that the wait counts follow.)
  auto one_tile = [&](auto g_const) {
    constexpr int g = decltype(g_const)::value;
    if (g >= n_mt) return;
    if constexpr (g + 1 < G) {
      if (g + 1 < n_mt) {
#pragma unroll
        for (int i = 0; i < ITERS; ++i)
          hb[(g + 1) & 1][i] = *reinterpret_cast<const float4 *>(hp + (size_t)(g + 1) * 32 * 4 + (size_t)(2 * i) * Mp * 4);
      }
    }
    __builtin_amdgcn_sched_barrier(0);  // the next tile's loads are under way before the first matrix instruction
    floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
      const float4 b = hb[g & 1][i];
      acc = mfma32(wa[i].x, b.x, acc);
      acc = mfma32(wa[i].y, b.y, acc);
      acc = mfma32(wa[i].z, b.z, acc);
      acc = mfma32(wa[i].w, b.w, acc);
    }
    if (g > 0) __syncthreads();  // the previous tile's partial sums have been read
    float *mine = red + (wave * 64 + lane) * kRedStride;
#pragma unroll
    for (int r = 0; r < 16; ++r) mine[r] = acc[r];
    __syncthreads();
    const int m = (t0 + g) * 32 + j;
    if (m < a.M) {
#pragma unroll
      for (int q = 0; q < VPL; ++q)
        store_through(a.R + (size_t)m * R4 + tile * 32 + i0 + q, tile_value<WAVES>(red, i0 + q, j));
    }
  };
  static_assert(G == 4, "four copies below");
  one_tile(std::integral_constant<int, 0>{});
  one_tile(std::integral_constant<int, 1>{});
  one_tile(std::integral_constant<int, 2>{});
  one_tile(std::integral_constant<int, 3>{});
}

struct MainArgs {
  // ---- joint role
  const float *pre;   // k4-major [H][Mp]: f_proj[b, t_m] + prediction projection of hypothesis m
  const float *W;     // k4-major [H][n_chunks * 32] output layer, zero rows beyond V + 1 + ND
  const float *bias;  // [n_chunks * 32]
  const float *lm;    // [M, V] natural-log LM scores or NULL
  float lambda;
  int M, Mp, K, H, V, ND, n_chunks, round_ops;
  int n_jchunks;           // chunks that have joint blocks.  n_chunks - 1: the blank and duration columns, alone in the
                           // last chunk, are folded into the token chunks' blocks (column V + c of tile ty into chunk
                           // (n_jchunks - 1 - c + ty) mod n_jchunks)
  int upt, rpt, n_jtiles;  // utterances and rows per joint tile (rpt = upt * K <= 32), number of such tiles
  float *p_max, *p_sum;    // [M, n_chunks] soft-max statistics of the chunk's token logits
  uint64_t *p_cand;        // [M, K, n_chunks] best (key = z + lambda * lm, token) of the chunk, packed
  float *zs;               // [M, 1 + ND] raw blank and duration logits
  int *tile_ctr;           // [n_jtiles] blocks of the tile that have written their lists
  // ---- recurrent-product role (LSTM)
  RecurrentArgs rec;
  XcdMap map;              // role 0 = joint (chunk, tile), role 1 = recurrent (gate tile, 32-row tile)
  // ---- selection (run by the block that completes a tile)
  SelectArgs sel;
};

// Joint network for 32 output columns (chunk) x the hypotheses [m0, m0 + rows): z[n] = W_out[n] . ReLU(pre_m) + b_out[n]
// with pre_m = f_proj[b, t_m] + g_m, then, in the epilogue, the soft-max statistics and the K best keys of the chunk,
// so that the [M, V + 1] logits never reach memory (LPH = 2 * WAVES lanes share a hypothesis, each holds 32 / LPH
// columns; the best K are found in K rounds of an LPH-lane arg-max).  Lists and statistics are written with
// device-coherent stores.  red: the block's reduction buffer (WAVES * 64 * kRedStride floats).
template <int WAVES, int ITERS, bool WIDE = false>
__device__ __forceinline__ void joint_tile(const MainArgs &a, int chunk, int m0, int rows, int done, float *red) {
  constexpr int LPH = 2 * WAVES, VPL = 32 / LPH;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31;
  const int n0 = chunk * 32;
  // (shifted by the tile's index: the blocks with a folded column finish last, and the one that completes a tile
  // keeps its compute unit for the selection: on a different XCD for every tile this way)
  const int fold_c = (a.n_jchunks - 1 - chunk + m0 / rows) % a.n_jchunks;
  const bool folds = WIDE && ITERS > 0 && a.n_jchunks < a.n_chunks && fold_c <= a.ND;
  {
    const int Np = a.n_chunks * 32;
    const float *wp = a.W + (size_t)(n0 + col) * 4;
    const float *pp = a.pre + (size_t)(m0 + col) * 4;
    const int Mp = a.Mp, round_ops = a.round_ops;
    auto a_at = [&](int k) { return *reinterpret_cast<const float4 *>(wp + (size_t)(k >> 2) * Np * 4); };
    auto b_at = [&](int k) { return *reinterpret_cast<const float4 *>(pp + (size_t)(k >> 2) * Mp * 4); };
    auto fb = [&](float4 f) {
      f.x = fmaxf(f.x, 0.f); f.y = fmaxf(f.y, 0.f); f.z = fmaxf(f.z, 0.f); f.w = fmaxf(f.w, 0.f);
      return f;
    };
    SplitKOperands<ITERS> op;
    splitk_load<WAVES, ITERS>(op, a_at, b_at, a.H);
    if constexpr (WIDE && ITERS > 0) {
      if (folds) {  // (uniform over the block) the folded column's weights, requested behind the operands
        float4 xw[ITERS];
        const int kbeg = (tid >> 6) * (a.H / WAVES) + 4 * (lane >> 5);
        const float *xp = a.W + (size_t)(a.V + fold_c) * 4;
#pragma unroll
        for (int i = 0; i < ITERS; ++i) xw[i] = *reinterpret_cast<const float4 *>(xp + (size_t)((kbeg + 8 * i) >> 2) * Np * 4);
        if (done) return;
        splitk_mma<WAVES, ITERS>(op, a_at, b_at, fb, a.H, red, round_ops, xw);
      } else {
        if (done) return;
        splitk_mma<WAVES, ITERS>(op, a_at, b_at, fb, a.H, red, round_ops);
      }
    } else {
      if (done) return;
      splitk_mma<WAVES, ITERS>(op, a_at, b_at, fb, a.H, red, round_ops);
    }
  }

  // epilogue: thread -> (hypothesis j, columns i0 .. i0 + VPL - 1)
  const int j = tid / LPH, e = tid % LPH, i0 = e * VPL;
  const int m = m0 + j;
  const bool mvalid = j < rows && m < a.M;
  const int nz = 1 + a.ND;
  if (WIDE && folds && mvalid) {
    if (e == 0) store_agent(a.zs + (size_t)m * nz + fold_c, extra_value<WAVES>(red, j) + a.bias[a.V + fold_c]);
    if (fold_c == 0) {  // ... and the empty lists of the chunk that has no block now
      const size_t pl = (size_t)m * a.n_chunks + a.n_chunks - 1;
      if (e == 0) {
        store_agent(a.p_max + pl, -INFINITY);
        store_agent(a.p_sum + pl, 0.f);
      }
      uint64_t *ll = a.p_cand + (size_t)m * a.K * a.n_chunks + a.n_chunks - 1;
      if (e < a.K) store_agent(ll + (size_t)e * a.n_chunks, no_cand());
      if (LPH + e < a.K) store_agent(ll + (size_t)(LPH + e) * a.n_chunks, no_cand());
    }
  }
  uint64_t cand[VPL];
  float mx = -INFINITY;
  float zv[VPL];
#pragma unroll
  for (int q = 0; q < VPL; ++q) {
    const int n = n0 + i0 + q;
    const float z = tile_value<WAVES>(red, i0 + q, j) + a.bias[n];
    zv[q] = z;
    cand[q] = no_cand();
    if (n < a.V) {
      cand[q] = pack_cand((a.lm && mvalid) ? z + a.lambda * a.lm[(size_t)m * a.V + n] : z, n);
      mx = fmaxf(mx, z);
    } else if (n < a.V + nz && mvalid) {
      store_agent(a.zs + (size_t)m * nz + (n - a.V), z);
    }
  }
  mx = group_max<LPH>(mx);
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < VPL; ++q)
    if (n0 + i0 + q < a.V) sum += __expf(zv[q] - mx);
  sum = group_sum<LPH>(sum);
  // local order of this lane's candidates (VPL is 2 or 4: a few compare-exchanges)
#pragma unroll
  for (int x = 0; x < VPL; ++x)
#pragma unroll
    for (int y = 0; y + 1 < VPL - x; ++y)
      if (cand[y + 1] > cand[y]) {
        const uint64_t tc = cand[y];
        cand[y] = cand[y + 1];
        cand[y + 1] = tc;
      }
  // K rounds: the best remaining candidate among the LPH lanes of the hypothesis
  uint64_t mine[2] = {no_cand(), no_cand()};  // lane e keeps the winners of rounds e and e + LPH
  for (int r = 0; r < a.K; ++r) {
    const uint64_t best = group_max_u64<LPH>(cand[0]);
    if (best == cand[0]) {  // mine was taken: move my list up
#pragma unroll
      for (int q = 0; q + 1 < VPL; ++q) cand[q] = cand[q + 1];
      cand[VPL - 1] = no_cand();
    }
    if (e == (r & (LPH - 1))) {
      if (r < LPH) mine[0] = best; else mine[1] = best;
    }
  }
  if (mvalid) {
    const size_t pc = (size_t)m * a.n_chunks + chunk;
    if (e == 0) {
      store_agent(a.p_max + pc, mx);
      store_agent(a.p_sum + pc, sum);
    }
    uint64_t *lists = a.p_cand + (size_t)m * a.K * a.n_chunks + chunk;
    if (e < a.K) store_agent(lists + (size_t)e * a.n_chunks, mine[0]);
    if (LPH + e < a.K) store_agent(lists + (size_t)(LPH + e) * a.n_chunks, mine[1]);
  }

}

// Main kernel of a step.  Blocks [0, n_chunks * n_jtiles): joint network for a tile of up to 32
// hypotheses (whole utterances) x 32 output columns (joint_tile).  The block that completes a
// tile (counted with one atomic per block) then runs the selection for the tile's utterances, one
// wave per utterance.  Remaining blocks: R = W_hh h for the current slots; it does not depend on
// the selection, so it overlaps with it instead of following it.
// TAIL = false: no selection in the kernel (a launch of its own follows): for beams wider than the
// in-kernel forms take.
// WIDE: the forms for 256 slots and more (folded blank / duration columns, recurrent blocks of several slot tiles);
// an instantiation of their own, because their code costs the smaller shapes 0.2 us per launch when it is only there.
// SEL: the selection forms in the tail (0: every in-kernel form; 5, 6: one form, see select_dispatch).
template <int WAVES, int ITERS, bool TAIL = true, bool WIDE = false, int SEL = 0>
__global__ __launch_bounds__(WAVES * 64, TAIL ? 1 : 16 / WAVES) void k_step_main(MainArgs a) {
  constexpr int kRedFloats = WAVES * 64 * kRedStride;
  constexpr int kScratchFloats = TAIL ? (int)((sizeof(SelectScratch) * WAVES + 3) / 4) : 1;
  __shared__ __align__(16) float smem[kRedFloats > kScratchFloats ? kRedFloats : kScratchFloats];
  __shared__ int s_is_last;
  float *red = smem;
  constexpr int LPH = 2 * WAVES, VPL = 32 / LPH;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31;
  const int done = *reinterpret_cast<const volatile int *>(a.sel.done);
  int chunk, ty;
  const int role = xcd_item(a.map, blockIdx.x, chunk, ty);
  if (role < 0) return;
  if (role == 1) {
    if constexpr (WIDE && ITERS > 0) {
      if (a.rec.group > 1) {
        recurrent_tiles<WAVES, ITERS, kRecGroup>(a.rec, chunk, ty, done, red);
        return;
      }
    }
    recurrent_tile<WAVES, ITERS>(a.rec, chunk, ty * 32, done, red);
    return;
  }

  joint_tile<WAVES, ITERS, WIDE>(a, chunk, ty * a.rpt, a.rpt, done, red);
  if (done) return;

  if constexpr (!TAIL) {
    return;
  } else {
  // ---- the block that completes the tile runs the selection for its utterances.
  // The lists were written with device-coherent (write-through) stores.  Every thread first waits until its own
  // stores have been acknowledged by the memory side (a workgroup-scope release alone does not wait for
  // outstanding global stores), then the barrier, then one thread counts the block in: the count can therefore
  // not become visible before any list of the block.  The completing block reads the lists with
  // device-coherent loads issued after it has seen the full count, so no cache is written back or invalidated.
  wait_stores_acknowledged();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (tid == 0) {
    const int old = __hip_atomic_fetch_add(a.tile_ctr + ty, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = old == (WIDE ? a.n_jchunks : a.n_chunks) - 1;
    if (last) store_agent(a.tile_ctr + ty, 0);  // every other block of the tile has been counted
    s_is_last = last;
  }
  __syncthreads();
  if (!s_is_last) {
    return;
  }
  SelectScratch *scratch = reinterpret_cast<SelectScratch *>(smem);
  const int wave = tid >> 6;
  for (int u = wave; u < a.upt; u += WAVES) {
    const int b = ty * a.upt + u;
    constexpr int kForms = WIDE ? (SEL == 5 ? 17 : SEL == 6 ? 18 : SEL) : SEL;
    if (b < a.sel.B) select_dispatch<kForms>(a.sel, b, scratch[wave]);
  }
  }  // TAIL
}

// stand-alone selection kernels: one wave per utterance, four utterances per block
__global__ __launch_bounds__(256) void k_select(SelectArgs a) {
  __shared__ SelectScratchWide scratch[4];
  if (*reinterpret_cast<volatile int *>(a.done)) return;
  const int wave = threadIdx.x >> 6;
  const int b = blockIdx.x * 4 + wave;
  if (b < a.B) select_dispatch<1, SelectScratchWide>(a, b, scratch[wave]);
}
// two utterances per block: the candidate arrays of this form are larger
__global__ __launch_bounds__(128) void k_select_pairs(SelectArgs a) {
  __shared__ SelectScratchPairs scratch[2];
  if (*reinterpret_cast<volatile int *>(a.done)) return;
  const int wave = threadIdx.x >> 6;
  const int b = blockIdx.x * 2 + wave;
  if (b < a.B) select_dispatch<3, SelectScratchPairs>(a, b, scratch[wave]);
}
__global__ __launch_bounds__(256) void k_select_wide(SelectArgs a) {
  __shared__ SelectScratchWide scratch[4];
  if (*reinterpret_cast<volatile int *>(a.done)) return;
  const int wave = threadIdx.x >> 6;
  const int b = blockIdx.x * 4 + wave;
  if (b < a.B) select_dispatch<2, SelectScratchWide>(a, b, scratch[wave]);
}

// Beams too wide for the in-kernel forms (9 to 16) on the fused path, where the selection has a launch of its own:
// one block per utterance, a wave per hypothesis.  A wave first reduces its hypothesis' n_lists chunk lists to the K
// best keys: the K-th largest of the lists' heads is a lower bound of the K-th largest key, the entries at or above
// it (the first few of a few lists) are collected in LDS and ranked by counting; the chunks' soft-max statistics are
// combined into one pair.  Wave 0 then runs the selection on those one-list rows in LDS (the forms of the
// materialised-logits path).  Against a single wave that merges K x n_lists entries per hypothesis in registers, in
// several passes: 27 -> about 10 us at beam 12.
struct MergeSelectArgs {
  SelectArgs sel;  // n_chunks = 1: what the selection proper sees
  int n_lists;     // chunk lists per hypothesis in the global arrays (at most 64 * kMergeHeads)
};
constexpr int kMergeHeads = 8, kMergeCap = 128;

template <int FORMS>  // 4, or 12 / 16 on a plain RNN-T (see select_dispatch)
__global__ __launch_bounds__(64 * kMaxBeam) void k_utt_merge_select(MergeSelectArgs a) {
  __shared__ SelectScratchWide scratch;
  __shared__ uint64_t l_cand[kMaxBeam * kMaxBeam];
  __shared__ float l_max[kMaxBeam], l_sum[kMaxBeam], l_zs[kMaxBeam * 9];
  __shared__ uint64_t surv[kMaxBeam][kMergeCap];
  __shared__ int surv_n[kMaxBeam];
  if (*reinterpret_cast<volatile int *>(a.sel.done)) return;
  const int K = a.sel.K, nl = a.n_lists, nz = 1 + a.sel.ND;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, b = blockIdx.x;  // wave < K
  const int m = b * K + wave;
  const uint64_t *cands = a.sel.p_cand + (size_t)m * K * nl;  // [K][n_lists]
  uint64_t head[kMergeHeads];
  float pm[kMergeHeads], ps[kMergeHeads];
#pragma unroll
  for (int q = 0; q < kMergeHeads; ++q) {
    const int c = lane + 64 * q;
    const bool ok = c < nl;
    const uint64_t x = cands[ok ? c : 0];
    const float xm = a.sel.p_max[(size_t)m * nl + (ok ? c : 0)], xs = a.sel.p_sum[(size_t)m * nl + (ok ? c : 0)];
    head[q] = ok ? x : no_cand();
    pm[q] = (ok && !a.sel.normalized) ? xm : -INFINITY;
    ps[q] = (ok && !a.sel.normalized) ? xs : 0.f;
  }
  if (lane == 0) surv_n[wave] = 0;
  if (lane < nz) l_zs[wave * nz + lane] = a.sel.zs[(size_t)m * nz + lane];
  // soft-max statistics of the row: the largest chunk maximum, the chunks' sums brought to it
  float mx = -INFINITY;
#pragma unroll
  for (int q = 0; q < kMergeHeads; ++q) mx = fmaxf(mx, pm[q]);
  mx = wave_max(mx);
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < kMergeHeads; ++q)
    if (pm[q] > -INFINITY) sum += ps[q] * __expf(pm[q] - mx);
  sum = wave_sum(sum);
  if (lane == 0) {
    l_max[wave] = mx;
    l_sum[wave] = sum;
  }
  // tau: the K-th largest head (packed keys are distinct).  Up to kMergeCap lists: every head counts the heads above
  // it (the heads wait in the survivors' buffer meanwhile), the one with K - 1 above it is tau; more lists: K rounds
  // of "largest remaining head"
  uint64_t tau = no_cand();
  if (nl <= kMergeCap) {
    __shared__ uint64_t s_tau[kMaxBeam];
    if (lane == 0) s_tau[wave] = no_cand();
#pragma unroll
    for (int q = 0; q < 2; ++q)
      if (lane + 64 * q < nl) surv[wave][lane + 64 * q] = head[q];
    wave_sync();
    int above[2] = {0, 0};
    for (int c = 0; c < nl; ++c) {
      const uint64_t x = surv[wave][c];
      above[0] += (int)(x > head[0]);
      above[1] += (int)(x > head[1]);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q)
      if (lane + 64 * q < nl && above[q] == K - 1 && head[q] > no_cand()) s_tau[wave] = head[q];
    wave_sync();
    tau = s_tau[wave];
  } else {
    for (int j = 0; j < K; ++j) {
      uint64_t best = head[0];
#pragma unroll
      for (int q = 1; q < kMergeHeads; ++q) best = head[q] > best ? head[q] : best;
      tau = wave_max_u64(best);
#pragma unroll
      for (int q = 0; q < kMergeHeads; ++q)
        if (head[q] == tau) head[q] = no_cand();
    }
  }
  wave_sync();
  // entries at or above tau (never "no candidate"): every list holds them at its front
  for (int e = lane; e < K * nl; e += 64) {
    const uint64_t x = cands[e];
    if (x >= tau && x > no_cand()) {
      const int pos = atomicAdd(&surv_n[wave], 1);
      if (pos < kMergeCap) surv[wave][pos] = x;
    }
  }
  wave_sync();
  const int total = surv_n[wave];
  uint64_t *out = l_cand + wave * K;
  if (total <= kMergeCap) {
    if (lane < K && lane >= total) out[lane] = no_cand();
    for (int i = lane; i < total; i += 64) {
      const uint64_t mine = surv[wave][i];
      int rank = 0;
      for (int q = 0; q < total; ++q) rank += surv[wave][q] > mine;
      if (rank < K) out[rank] = mine;
    }
  } else {  // (many equal keys) K plain rounds over all entries
    uint64_t last = ~0ull;
    for (int j = 0; j < K; ++j) {
      uint64_t best = no_cand();
      for (int c = lane; c < K * nl; c += 64) {
        const uint64_t x = cands[c];
        if (x < last && x > best) best = x;
      }
      best = wave_max_u64(best);
      if (lane == 0) out[j] = best;
      last = best > no_cand() ? best : no_cand() + 1;
    }
  }
  __syncthreads();
  if (wave == 0) select_dispatch<FORMS, SelectScratchWide>(a.sel, b, scratch, CandView{l_cand, l_max, l_sum, l_zs, b * K});
}

// ---------------------------------------------------------------------------
// LSTM cell for every slot: gates = G[token] + W_hh h_parent (G = emb W_ih^T + b_ih + b_hh
// folded at create), rows packed so that a lane holds the four gates of a unit.
// Slots that did not append a token copy their parent's state.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float sigmoid_f(float x) { return 1.f / (1.f + __expf(-x)); }
__device__ __forceinline__ float tanh_f(float x) {
  const float e = __expf(-2.f * fabsf(x));
  const float r = (1.f - e) / (1.f + e);
  return x < 0.f ? -r : r;
}

// Pointwise part of the LSTM cell for every new slot: gates = R[parent] + G[token] with
// R = W_hh h of the parent (computed for every current slot by the main kernel, before the selection
// was known) and G = W_ih emb + biases per token; slots that did not append a token copy their
// parent's state.  R, G: [.][4P] with the four gates of a unit adjacent; h: k4-major [P][Mp]; c: [M][P].
// LM rows riding in another launch as extra blocks: block first_block + m builds the row of hypothesis m
struct LmRowsArgs {
  LmView view;
  const int *ctx, *len;
  float *out;
  int M;            // 0: no LM rows in this launch
  int first_block;
};

// unit u of slot m: gates = R[src] + G[token] (the four gates of a unit adjacent), or a copy of the parent's state
__device__ __forceinline__ void lstm_cell(const float *__restrict__ R, const float *__restrict__ G,
                                          const float *__restrict__ h_cur, const float *__restrict__ c_cur,
                                          float *__restrict__ h_nxt, float *__restrict__ c_nxt, int src, int token, int m,
                                          int u, int Mp, int P, int done_flag) {
  const float c_old = c_cur[(size_t)src * P + u];
  float c = c_old, h;
  if (token >= 0) {
    const float4 r4 = *reinterpret_cast<const float4 *>(R + (size_t)src * 4 * P + 4 * u);
    const float4 g4 = *reinterpret_cast<const float4 *>(G + (size_t)token * 4 * P + 4 * u);
    if (done_flag) return;
    c = sigmoid_f(r4.y + g4.y) * c_old + sigmoid_f(r4.x + g4.x) * tanh_f(r4.z + g4.z);
    h = sigmoid_f(r4.w + g4.w) * tanh_f(c);
  } else {
    h = h_cur[k4_index(u, src, Mp)];
    if (done_flag) return;
  }
  store_through(c_nxt + (size_t)m * P + u, c);
  store_through(h_nxt + k4_index(u, m, Mp), h);
}

template <bool LM>
__global__ __launch_bounds__(256) void k_lstm_pointwise(const float *__restrict__ R, const float *__restrict__ G,
                                                        const float *__restrict__ h_cur,
                                                        const float *__restrict__ c_cur, float *__restrict__ h_nxt,
                                                        float *__restrict__ c_nxt, const int *__restrict__ src_row,
                                                        const int *__restrict__ tok, int M, int Mp, int P,
                                                        const int *done, LmRowsArgs lmr, float *pre_clear,
                                                        int n_pre_clear) {
  if constexpr (LM) {  // (an instantiation of its own: the plain launch is faster without this code in it)
    if (lmr.M > 0 && (int)blockIdx.x >= lmr.first_block) {
      // (vocabularies whose row would take the projection launch's LDS: the rows ride here instead)
      extern __shared__ float lm_row[];
      __shared__ LmRowScratch lm_sc;
      if (*reinterpret_cast<const volatile int *>(done)) return;
      lm_row_block(lmr.view, lmr.ctx, lmr.len, lmr.out, (int)blockIdx.x - lmr.first_block, lm_row, lm_sc);
      return;
    }
  }
  const int gid = blockIdx.x * 256 + threadIdx.x;
  // (no launch asks for this any more, n_pre_clear = 0: the projection launch clears its buffers itself.  Left in
  // place: without it the same launches measured 0.03 ms slower per decode at batch 32, beam 4)
  for (int i = 4 * gid; i < n_pre_clear; i += 4 * M * P) store16_through(pre_clear + i, floatx4{0.f, 0.f, 0.f, 0.f});
  const int m = gid / P, u = gid % P;
  if (m >= M) return;
  const int done_flag = *reinterpret_cast<const volatile int *>(done);
  lstm_cell(R, G, h_cur, c_cur, h_nxt, c_nxt, src_row[m], tok[m], m, u, Mp, P, done_flag);
}

// Advances the step counter at the boundary of two chunks of steps (one thread of one launch per chunk) and tells
// the enqueueing host thread, through a word of pinned host memory, that the next chunk begins.
__device__ __forceinline__ void bump_step(int *step_base, int bump, volatile int *h_progress) {
  const int next = *step_base + bump;
  *step_base = next;
  if (h_progress) *h_progress = next;
}

// pre[m] = f_proj[b, t_m] + W_pred h[m] + b_pred: the input of the joint's ReLU, written k4-major.
// W_pred: k4-major [P][H]; h: k4-major [P][Mp]; f_proj: row-major [B * T, H].
struct PredProjArgs {
  const float *Wp, *bias, *h, *f_proj;
  const int *t, *lengths;
  float *pre;
  int M, Mp, K, T, P, H, round_ops;
  const int *done;
  int *step_base;
  int bump;
  volatile int *h_progress = nullptr;  // see bump_step
  // k_pred_proj_half adds its two halves into pre, which therefore starts at zero: there are two such buffers, a
  // step's launch adds into the one and clears the other, which the joint has just read (n_pre_clear floats, a
  // multiple of 4; the blocks of the launch share the work)
  float *pre_clear = nullptr;
  int n_pre_clear = 0;
  RecurrentArgs rec;   // recurrent tiles of the new state ride along
  XcdMap map;          // role 0 = projection (tile of H, 32-row tile), role 1 = recurrent
  LmRowsArgs lmr;      // blocks from lmr.first_block on build LM rows (lmr.M = 0: none)
};

// The LM rows of the new hypotheses depend on the selection only, and the next selection is the first to read them:
// their blocks (a chain of memory round trips with next to no arithmetic) share the compute units with the tiles of
// the projection.  Dynamic LDS of the launch: V floats.
__device__ __forceinline__ bool pred_proj_lm_block(const PredProjArgs &a) {
  if (a.lmr.M == 0 || (int)blockIdx.x < a.lmr.first_block) return false;
  extern __shared__ float lm_row[];
  __shared__ LmRowScratch lm_sc;
  if (!*reinterpret_cast<const volatile int *>(a.done))
    lm_row_block(a.lmr.view, a.lmr.ctx, a.lmr.len, a.lmr.out, (int)blockIdx.x - a.lmr.first_block, lm_row, lm_sc);
  return true;
}

// One tile of the projection: 32 outputs of H (tile) x the slots [m0, m0 + 32).
template <int WAVES, int ITERS>
__device__ __forceinline__ void pred_proj_tile(const PredProjArgs &a, int tile, int m0, int done_flag, float *red) {
  constexpr int LPH = 2 * WAVES, VPL = 32 / LPH;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31;
  const float *wp = a.Wp + (size_t)(tile * 32 + col) * 4;
  const float *hp = a.h + (size_t)(m0 + col) * 4;
  const int H = a.H, Mp = a.Mp, round_ops = a.round_ops;
  auto a_at = [&](int k) { return *reinterpret_cast<const float4 *>(wp + (size_t)(k >> 2) * H * 4); };
  auto b_at = [&](int k) { return *reinterpret_cast<const float4 *>(hp + (size_t)(k >> 2) * Mp * 4); };
  auto fb = [](float4 v) { return v; };
  // epilogue role: (hypothesis j, outputs o0 .. o0 + VPL - 1).  Its frame index is loaded BEFORE the operands: the
  // address of the frame's projection depends on it, and a wait for a load that was issued after the operands would
  // wait for all of them too (loads complete in order), i.e. hold the first matrix instruction back until the last
  // operand has arrived.
  const int j = tid / LPH, o0 = tile * 32 + (tid % LPH) * VPL;
  const int me = m0 + j;
  const int me_ok = me < a.M ? me : 0;  // (unconditional loads: a branch here would end in a wait for them)
  const int T_b = a.lengths[me_ok / a.K];
  int tt = a.t[me_ok];
  SplitKOperands<ITERS> op;
  splitk_load<WAVES, ITERS>(op, a_at, b_at, a.P);
  __builtin_amdgcn_sched_barrier(0);  // nothing below may be scheduled (and waited for) ahead of the operand loads
  if (done_flag) return;
  float fv[VPL], bv[VPL];
  if (me < a.M) {
    const int b = me / a.K;
    tt = tt < T_b ? tt : T_b - 1;
    tt = tt < 0 ? 0 : tt;
#pragma unroll
    for (int q = 0; q < VPL; ++q) {
      fv[q] = a.f_proj[((size_t)b * a.T + tt) * a.H + o0 + q];
      bv[q] = a.bias[o0 + q];
    }
  }
  splitk_mma<WAVES, ITERS>(op, a_at, b_at, fb, a.P, red, round_ops);
  if (me >= a.M) return;
#pragma unroll
  for (int q = 0; q < VPL; ++q)
    store_through(a.pre + k4_index(o0 + q, me, a.Mp), tile_value<WAVES>(red, (tid % LPH) * VPL + q, j) + bv[q] + fv[q]);
}

// LM: the launch carries LM rows (an instantiation of its own: the test for them costs the plain launch 0.26 us)
template <int WAVES, int ITERS, bool LM = false>
__global__ __launch_bounds__(WAVES * 64) void k_pred_proj(PredProjArgs a) {
  __shared__ float red[WAVES * 64 * kRedStride];
  if constexpr (LM) {
    if (pred_proj_lm_block(a)) return;
  }
  int tile, mtile;
  const int role = xcd_item(a.map, blockIdx.x, tile, mtile);
  if (role < 0) return;
  const int done_flag = *reinterpret_cast<const volatile int *>(a.done);
  if (role == 1) {
    recurrent_tile<WAVES, ITERS>(a.rec, tile, mtile * 32, done_flag, red);
    return;
  }
  if (!done_flag && a.bump && tile == 0 && mtile == 0 && threadIdx.x == 0) bump_step(a.step_base, a.bump, a.h_progress);
  pred_proj_tile<WAVES, ITERS>(a, tile, mtile * 32, done_flag, red);
}

// The same projection with the contraction split in two across blocks, for launches that would leave half the
// chip idle (B * beam <= 128 at H = 640): block (tile, 32-slot tile, half) takes k in [half * P / 2, (half + 1) * P / 2)
// and ADDS its part to pre, which the cell-update launch has cleared; two addends commute, so the sum does not depend
// on which block comes first.  Half the operands and half the matrix instructions per block: 3.0 instead of 4.8 us.
// No recurrent tiles ride in this launch (they would set its duration); the main launch takes them all.
// ITERS = P / 2 / WAVES / 8.
template <int WAVES, int ITERS, bool LM = false>
__global__ __launch_bounds__(WAVES * 64) void k_pred_proj_half(PredProjArgs a) {
  __shared__ float red[WAVES * 64 * kRedStride];
  constexpr int LPH = 2 * WAVES, VPL = 32 / LPH;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31;
  if constexpr (LM) {
    if (pred_proj_lm_block(a)) return;
  }
  int tile, item;
  if (xcd_item(a.map, blockIdx.x, tile, item) != 0) return;
  const int mtile = item >> 1, half = item & 1;
  const int m0 = mtile * 32, koff = half * (a.P / 2);
  const float *wp = a.Wp + (size_t)(tile * 32 + col) * 4;
  const float *hp = a.h + (size_t)(m0 + col) * 4;
  const int H = a.H, Mp = a.Mp, round_ops = a.round_ops;
  auto a_at = [&](int k) { return *reinterpret_cast<const float4 *>(wp + (size_t)((k + koff) >> 2) * H * 4); };
  auto b_at = [&](int k) { return *reinterpret_cast<const float4 *>(hp + (size_t)((k + koff) >> 2) * Mp * 4); };
  auto fb = [](float4 v) { return v; };
  const int done_flag = *reinterpret_cast<const volatile int *>(a.done);
  const int j = tid / LPH, o0 = tile * 32 + (tid % LPH) * VPL;
  const int me = m0 + j;
  const int me_ok = me < a.M ? me : 0;  // loaded before the operands, without a branch (see k_pred_proj)
  const int T_b = a.lengths[me_ok / a.K];
  int tt = a.t[me_ok];
  SplitKOperands<ITERS> op;
  splitk_load<WAVES, ITERS>(op, a_at, b_at, a.P / 2);
  __builtin_amdgcn_sched_barrier(0);  // nothing below may be scheduled (and waited for) ahead of the operand loads
  if (done_flag) return;
  float fv[VPL], bv[VPL];
#pragma unroll
  for (int q = 0; q < VPL; ++q) fv[q] = bv[q] = 0.f;
  if (me < a.M && half == 0) {  // the frame's projection and the bias come in with the first half
    const int b = me / a.K;
    tt = tt < T_b ? tt : T_b - 1;
    tt = tt < 0 ? 0 : tt;
#pragma unroll
    for (int q = 0; q < VPL; ++q) {
      fv[q] = a.f_proj[((size_t)b * a.T + tt) * a.H + o0 + q];
      bv[q] = a.bias[o0 + q];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // (behind every load of the block, whose waits then do not include these stores; they are on their way while the
  // operands come in and are multiplied)
  for (int i = 4 * ((tile * a.map.a_m + item) * WAVES * 64 + tid); i < a.n_pre_clear;
       i += 4 * WAVES * 64 * a.map.a_tiles * a.map.a_m)
    store16_through(a.pre_clear + i, floatx4{0.f, 0.f, 0.f, 0.f});
  __builtin_amdgcn_sched_barrier(0);
  splitk_mma<WAVES, ITERS>(op, a_at, b_at, fb, a.P / 2, red, round_ops);
  if (a.bump && tile == 0 && item == 0 && tid == 0) bump_step(a.step_base, a.bump, a.h_progress);
  if (me >= a.M) return;
#pragma unroll
  for (int q = 0; q < VPL; ++q)
    __hip_atomic_fetch_add(a.pre + k4_index(o0 + q, me, a.Mp),
                           tile_value<WAVES>(red, (tid % LPH) * VPL + q, j) + bv[q] + fv[q], __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
}

// Stateless prediction network: pre[m] = f_proj[b, t_m] + sum_i tab_i[token_i of m] (tables folded
// with W_pred and b_pred at create).  One thread per (hypothesis, group of 4 outputs).
struct StatelessPreArgs {
  const float *f_proj, *tab;
  const int *ctx_tok, *t, *lengths;
  float *pre;
  int M, Mp, K, T, H, V, n_ctx;
  const int *done;
  int *step_base;
  int bump;
  volatile int *h_progress = nullptr;  // see bump_step
};

__global__ __launch_bounds__(256) void k_stateless_pre(StatelessPreArgs a) {
  if (*reinterpret_cast<const volatile int *>(a.done)) return;
  const int gid = blockIdx.x * 256 + threadIdx.x;
  if (a.bump && gid == 0) bump_step(a.step_base, a.bump, a.h_progress);
  const int H4 = a.H >> 2;
  const int m = gid / H4, o4 = gid % H4;
  if (m >= a.M) return;
  const int b = m / a.K;
  const int T_b = a.lengths[b];
  int tt = a.t[m];
  tt = tt < T_b ? tt : T_b - 1;
  tt = tt < 0 ? 0 : tt;
  float4 v = *reinterpret_cast<const float4 *>(a.f_proj + ((size_t)b * a.T + tt) * a.H + 4 * o4);
  for (int i = 0; i < a.n_ctx; ++i) {
    int tk = a.ctx_tok[m * kCtxMax + i];
    tk = tk < 0 ? a.V : tk;
    const float4 g = *reinterpret_cast<const float4 *>(a.tab + ((size_t)i * (a.V + 1) + tk) * a.H + 4 * o4);
    v.x += g.x; v.y += g.y; v.z += g.z; v.w += g.w;
  }
  *reinterpret_cast<float4 *>(a.pre + ((size_t)o4 * a.Mp + m) * 4) = v;  // (16-byte store: cheaper than two written through)
}

__global__ void k_fill_int(int *p, int value, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = value;
}

// advances the step counter when no prediction projection closes the step (stateless, injected)
__global__ void k_bump(int *step_base, int bump, const int *done, volatile int *h_progress) {
  if (*reinterpret_cast<const volatile int *>(done)) return;
  if (threadIdx.x == 0 && blockIdx.x == 0) bump_step(step_base, bump, h_progress);
}

// ---------------------------------------------------------------------------
// Start of a decode call: one live hypothesis per utterance (the empty
// transcript), everything else empty; lengths clamped into [0, T].
// ---------------------------------------------------------------------------
struct InitArgs {
  double *score;
  int *t, *sym, *len, *last;
  uint32_t *hash;
  int *ctx;
  const int *lengths_in;
  int *lengths;
  int *src_row, *tok;
  float *h0, *c0;  // zeroed state the first LSTM step reads (nullable), n_state floats each
  size_t n_state;
  float *R;        // recurrent product of the zero state (nullable), n_R floats
  size_t n_R;
  float *pre0, *pre1;  // the two buffers that k_pred_proj_half adds into (nullable), n_pre floats each
  size_t n_pre;
  int *tile_ctr;   // per-tile block counters of the main kernel
  int n_tiles;
  int B, K, T, V, lstm;
  int step_base_init;  // 0, or minus one chunk of steps when the step counter is advanced at the START of a chunk
  int *finished, *utt_steps, *n_finished, *done, *step_base, *bad_arg;
  volatile int *h_done;
};

__global__ void k_init(InitArgs a) {
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;
  const int M = a.B * a.K;
  if (blockIdx.x == 0) {  // the utterances, one per thread of the first block (one thread for all took 0.2 us each)
    __shared__ int s_nfin;
    if (threadIdx.x == 0) {
      s_nfin = 0;
      *a.step_base = a.step_base_init;
    }
    __syncthreads();
    int nfin = 0;
    for (int b = threadIdx.x; b < a.B; b += blockDim.x) {
      int L = a.lengths_in[b];
      if (L < 0 || L > a.T) {
        *a.bad_arg = 1;
        L = L < 0 ? 0 : a.T;
      }
      a.lengths[b] = L;
      a.finished[b] = L == 0;
      a.utt_steps[b] = L == 0 ? 0 : -1;
      nfin += L == 0;
    }
    if (nfin) atomicAdd(&s_nfin, nfin);
    __syncthreads();
    if (threadIdx.x == 0) {
      *a.n_finished = s_nfin;
      *a.done = s_nfin == a.B;
      *a.h_done = s_nfin == a.B;
    }
  }
  if (gid < M) {
    const int k = gid % a.K;
    a.score[gid] = k == 0 ? 0.0 : -INFINITY;
    a.t[gid] = 0;
    a.sym[gid] = 0;
    a.len[gid] = 0;
    a.last[gid] = -1;
    a.hash[gid] = 0;
    for (int i = 0; i < kCtxMax; ++i) a.ctx[gid * kCtxMax + i] = -1;
    a.src_row[gid] = gid;
    a.tok[gid] = (a.lstm && k == 0) ? a.V : -1;
  }
  for (int i = gid; i < a.n_tiles; i += gridDim.x * blockDim.x) a.tile_ctr[i] = 0;
  if (a.R)
    for (size_t i = gid; i < a.n_R; i += (size_t)gridDim.x * blockDim.x) a.R[i] = 0.f;
  if (a.pre0)
    for (size_t i = gid; i < a.n_pre; i += (size_t)gridDim.x * blockDim.x) a.pre0[i] = a.pre1[i] = 0.f;
  if (a.h0) {
    const size_t n = a.n_state;
    for (size_t i = gid; i < n; i += (size_t)gridDim.x * blockDim.x) {
      a.h0[i] = 0.f;
      a.c0[i] = 0.f;
    }
  }
}

// ---------------------------------------------------------------------------
// End of a decode call: rank the slots of each utterance and walk the tree
// back from each of them (latest token first, Sec. 2.1 "Efficient hypothesis storing").
// ---------------------------------------------------------------------------
struct BacktraceArgs {
  const double *score;
  const int *len;
  const int *tree_parent, *tree_token;
  const int *utt_steps, *step_base;
  int K, S_max, cap;
  int *out_tokens;     // [B, K, cap]
  int *out_lens;       // [B, K]
  double *out_scores;  // [B, K]
  int *out_steps;      // [B]
};

constexpr int kBacktraceThreads = 256;
constexpr int kBacktraceSegs = 64;  // the steps of an utterance are walked in at most this many segments
// The walk from a final slot back to the first step is a chain of dependent reads, one per step (45 ns each from LDS);
// it is cut into segments that are walked at once: (1) every segment from each of its K end slots, which gives the
// slot the path has before the segment and the tokens on it; (2) per hypothesis, one read per segment chains these
// into the slot and the output position with which its path enters every segment; (3) every (hypothesis, segment)
// pair walks its segment again and writes the tokens.  2 * segment length + segments dependent reads instead of one
// per step (687 steps: 37 segments of 19).
// LDS: the utterance's tree is copied into LDS first (S_max * K * 8 bytes of dynamic LDS).  (A template parameter
// rather than a flag: with one pointer for both cases the reads become flat loads, which also wait for the token
// stores in flight: 185 ns per step instead of 45.)
template <bool LDS>
__global__ __launch_bounds__(kBacktraceThreads) void k_backtrace(BacktraceArgs a) {
  extern __shared__ int tree_lds[];
  __shared__ int seg_from[kBacktraceSegs * kMaxBeam], seg_cnt[kBacktraceSegs * kMaxBeam];  // [segment][end slot]
  __shared__ int hyp_slot[kMaxBeam * kBacktraceSegs], hyp_u[kMaxBeam * kBacktraceSegs];    // [hypothesis][segment]
  __shared__ int hyp_pos[kMaxBeam];
  const int b = blockIdx.x, K = a.K, tid = threadIdx.x;
  int n = a.utt_steps[b];
  if (n < 0) n = min(*a.step_base, a.S_max);
  if (tid == 0) a.out_steps[b] = n;
  const int *gp = a.tree_parent + (size_t)b * a.S_max * K;
  const int *gt = a.tree_token + (size_t)b * a.S_max * K;
  int *sp = tree_lds, *st = tree_lds + n * K;
  if constexpr (LDS) {
    constexpr int U = 8;  // loads of each array in flight per thread
    for (int i0 = tid; i0 < n * K; i0 += U * kBacktraceThreads) {
      int vp[U], vt[U];
#pragma unroll
      for (int q = 0; q < U; ++q) {
        const int i = i0 + q * kBacktraceThreads;
        const int ic = i < n * K ? i : 0;
        vp[q] = gp[ic];
        vt[q] = gt[ic];
      }
#pragma unroll
      for (int q = 0; q < U; ++q) {
        const int i = i0 + q * kBacktraceThreads;
        if (i < n * K) {
          sp[i] = vp[q];
          st[i] = vt[q];
        }
      }
    }
  }
  // segment length: about sqrt(n / 2) (the three phases then take 2 L + n / L reads in a row), at most 64 segments
  int L = 16;
  while (2 * L * L < n) ++L;
  if (L * kBacktraceSegs < n) L = (n + kBacktraceSegs - 1) / kBacktraceSegs;
  const int nseg = (n + L - 1) / L;  // <= kBacktraceSegs
  __syncthreads();
  auto tok_at = [&](int s, int slot) { return LDS ? st[s * K + slot] : gt[s * K + slot]; };
  auto par_at = [&](int s, int slot) { return LDS ? sp[s * K + slot] : gp[s * K + slot]; };
  // (1) every segment from every end slot
  for (int w = tid; w < nseg * K; w += kBacktraceThreads) {
    const int j = w / K, lo = j * L, hi = min(n, lo + L) - 1;
    int cur = w % K, cnt = 0;
    for (int s = hi; s >= lo && cur >= 0; --s) {
      cnt += tok_at(s, cur) >= 0 ? 1 : 0;
      cur = par_at(s, cur);
    }
    seg_from[w] = cur;
    seg_cnt[w] = cnt;
  }
  // ranks of the final slots by score (ties: lower slot first); a dead slot has no path
  if (tid < K) {
    const double my = a.score[b * K + tid];
    int pos = 0;
    for (int i = 0; i < K; ++i) {
      const double o = a.score[b * K + i];
      if (o > my || (o == my && i < tid)) ++pos;
    }
    hyp_pos[tid] = pos;
    const size_t oi = (size_t)b * K + pos;
    const bool live = my > -INFINITY;
    a.out_lens[oi] = live ? a.len[b * K + tid] : -1;
    a.out_scores[oi] = live ? my : -INFINITY;
  }
  __syncthreads();
  // (2) the slot and the output position with which hypothesis tid's path enters each segment (from its last step)
  if (tid < K) {
    int cur = a.score[b * K + tid] > -INFINITY ? tid : -1;
    int u = a.len[b * K + tid];
    for (int j = nseg - 1; j >= 0; --j) {
      hyp_slot[tid * kBacktraceSegs + j] = cur;
      hyp_u[tid * kBacktraceSegs + j] = u;
      if (cur >= 0) {
        u -= seg_cnt[j * K + cur];
        cur = seg_from[j * K + cur];
      }
    }
  }
  __syncthreads();
  // (3) the tokens of every (hypothesis, segment) pair
  for (int w = tid; w < nseg * K; w += kBacktraceThreads) {
    const int j = w / K, hyp = w % K, lo = j * L, hi = min(n, lo + L) - 1;
    int cur = hyp_slot[hyp * kBacktraceSegs + j], u = hyp_u[hyp * kBacktraceSegs + j];
    const size_t oi = (size_t)b * K + hyp_pos[hyp];
    for (int s = hi; s >= lo && cur >= 0; --s) {
      const int tk = tok_at(s, cur);
      const int up = par_at(s, cur);
      if (tk >= 0) {
        --u;
        if (u >= 0 && u < a.cap) a.out_tokens[oi * a.cap + u] = tk;
      }
      cur = up;
    }
  }
}

}  // namespace rb
