// Kernels of the per-step beam expansion (gfx950).  One step of the loop is
//   k_joint (or k_inject) -> k_select -> [k_lm_rows] -> k_lstm -> k_pred_proj
// and k_gemm_nt / k_init / k_backtrace run once per decode call.
#pragma once
#include "device_utils.h"

namespace rb {

// ---------------------------------------------------------------------------
// C[M, N] = A[M, K] B[N, K]^T + bias[N]   (both operands K-contiguous, fp32 matrix cores)
// 256 threads = 2 x 2 waves, each a 32 x 32 tile; K % 8 == 0.
// round_ops: both operands are rounded to bf16 before they are multiplied.
// nonfinite (nullable): set to 1 when an output is NaN or Inf.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_gemm_nt(const float *__restrict__ A, const float *__restrict__ B,
                                                 const float *__restrict__ bias, float *__restrict__ C, int M,
                                                 int N, int K, int round_ops, int *nonfinite) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5, col = lane & 31;
  const int m0 = blockIdx.y * 64 + (wave >> 1) * 32, n0 = blockIdx.x * 64 + (wave & 1) * 32;
  if (m0 >= M || n0 >= N) return;
  const int am = min(m0 + col, M - 1), bn = min(n0 + col, N - 1);
  const float *ap = A + (size_t)am * K + 4 * half, *bp = B + (size_t)bn * K + 4 * half;
  floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 4
  for (int k = 0; k < K; k += 8) {
    float4 a = *reinterpret_cast<const float4 *>(ap + k);
    float4 b = *reinterpret_cast<const float4 *>(bp + k);
    if (round_ops) {
      a = bf16_round4(a);
      b = bf16_round4(b);
    }
    acc = mfma32(a.x, b.x, acc);
    acc = mfma32(a.y, b.y, acc);
    acc = mfma32(a.z, b.z, acc);
    acc = mfma32(a.w, b.w, acc);
  }
  const int n = n0 + col;
  bool bad = false;
  if (n < N) {
    const float bv = bias ? bias[n] : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + 8 * (r >> 2) + 4 * half + (r & 3);
      if (m < M) {
        const float v = acc[r] + bv;
        C[(size_t)m * N + n] = v;
        bad |= !isfinite(v);
      }
    }
  }
  if (nonfinite && bad) *nonfinite = 1;
}

// ---------------------------------------------------------------------------
// Split-K 32 x 32 tile shared by the three per-step contractions: the 4 waves
// of a block each take a quarter of K (K % 32 == 0), partial tiles are summed
// through LDS into wave 0.  a_at(k) / b_at(k) return 4 consecutive k of this
// lane's row of the "vocabulary side" / "hypothesis side" operand.
// ---------------------------------------------------------------------------
template <class AL, class BL>
__device__ __forceinline__ floatx16 splitk_tile(AL a_at, BL b_at, int K, float *red /* [3 * 16 * 64] */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int kw = K >> 2;
  floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  const int kend = (wave + 1) * kw;
#pragma unroll 5
  for (int k = wave * kw + 4 * half; k < kend; k += 8) {
    const float4 a = a_at(k);
    const float4 b = b_at(k);
    acc = mfma32(a.x, b.x, acc);
    acc = mfma32(a.y, b.y, acc);
    acc = mfma32(a.z, b.z, acc);
    acc = mfma32(a.w, b.w, acc);
  }
  if (wave > 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) red[((wave - 1) * 16 + r) * 64 + lane] = acc[r];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int w = 0; w < 3; ++w)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] += red[(w * 16 + r) * 64 + lane];
  }
  return acc;
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

struct JointArgs {
  const float *f_proj;  // [B * T, H]
  const float *g_proj;  // [M, H] prediction projection (LSTM), or NULL
  const float *tab;     // stateless: [ctx][V + 1][H] folded embedding tables
  const int *ctx_tok;   // [M][kCtxMax] most recent token first, -1 = none
  int n_ctx;
  const int *t;         // [M] frame of each hypothesis
  const int *lengths;   // [B]
  const float *W;       // [n_chunks * 32, H] output layer, zero rows beyond V + 1 + ND
  const float *bias;    // [n_chunks * 32]
  const float *lm;      // [M, V] natural-log LM scores or NULL
  float lambda;
  int M, K, T, H, V, ND, n_chunks, round_ops;
  float *p_max, *p_sum;  // [M, n_chunks] soft-max statistics of the chunk's token logits
  float *p_key;          // [M, n_chunks, K] best keys z + lambda * lm of the chunk
  int *p_idx;            // [M, n_chunks, K] their token ids
  float *zs;             // [M, 1 + ND] raw blank and duration logits
  const int *done;
};

// Joint network for a tile of 32 hypotheses x 32 output columns:
//   z[n] = W_out[n] . ReLU(f_proj[b, t_m] + g_m) + b_out[n]
// with the soft-max statistics and the K best keys of the chunk in the epilogue,
// so that the [M, V + 1] logits never reach memory.
template <int KT>
__global__ __launch_bounds__(256) void k_joint(JointArgs a) {
  if (*reinterpret_cast<const volatile int *>(a.done)) return;
  __shared__ float red[3 * 16 * 64];
  const int lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int chunk = blockIdx.x, n0 = chunk * 32, m0 = blockIdx.y * 32;
  const int m = m0 + col;
  const bool mvalid = m < a.M;
  const int mm = mvalid ? m : a.M - 1;
  const int b = mm / a.K;
  const int T_b = a.lengths[b];
  int tt = a.t[mm];
  tt = tt < T_b ? tt : T_b - 1;
  tt = tt < 0 ? 0 : tt;
  const float *fp = a.f_proj + ((size_t)b * a.T + tt) * a.H;
  const float *gp = a.g_proj ? a.g_proj + (size_t)mm * a.H : nullptr;
  const float *tp[4] = {nullptr, nullptr, nullptr, nullptr};
  if (!gp) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (i < a.n_ctx) {
        int tk = a.ctx_tok[mm * kCtxMax + i];
        tk = tk < 0 ? a.V : tk;
        tp[i] = a.tab + ((size_t)i * (a.V + 1) + tk) * a.H;
      }
  }
  const float *wp = a.W + (size_t)(n0 + col) * a.H;
  const int round_ops = a.round_ops;
  auto a_at = [&](int k) { return *reinterpret_cast<const float4 *>(wp + k); };
  auto b_at = [&](int k) {
    float4 f = *reinterpret_cast<const float4 *>(fp + k);
    if (gp) {
      const float4 g = *reinterpret_cast<const float4 *>(gp + k);
      f.x += g.x; f.y += g.y; f.z += g.z; f.w += g.w;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (tp[i]) {
          const float4 g = *reinterpret_cast<const float4 *>(tp[i] + k);
          f.x += g.x; f.y += g.y; f.z += g.z; f.w += g.w;
        }
    }
    f.x = fmaxf(f.x, 0.f); f.y = fmaxf(f.y, 0.f); f.z = fmaxf(f.z, 0.f); f.w = fmaxf(f.w, 0.f);
    if (round_ops) f = bf16_round4(f);
    return f;
  };
  floatx16 acc = splitk_tile(a_at, b_at, a.H, red);
  if (threadIdx.x >= 64) return;

  // epilogue (wave 0): lane holds 16 logits of hypothesis m
  TopList<KT> top;
  top.init();
  float mx = -INFINITY, sum = 0.f;
  const int nz = 1 + a.ND;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int nb = n0 + 8 * q + 4 * half;
    const float4 bias = *reinterpret_cast<const float4 *>(a.bias + nb);
    const float bz[4] = {bias.x, bias.y, bias.z, bias.w};
    float lz[4] = {0.f, 0.f, 0.f, 0.f};
    if (a.lm) {
#pragma unroll
      for (int e = 0; e < 4; ++e) lz[e] = nb + e < a.V ? a.lm[(size_t)mm * a.V + nb + e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = nb + e;
      const float z = acc[4 * q + e] + bz[e];
      if (n < a.V) {
        const float key = a.lm ? z + a.lambda * lz[e] : z;
        if (z > mx) {
          sum = sum * __expf(mx - z) + 1.f;
          mx = z;
        } else {
          sum += __expf(z - mx);
        }
        top.insert(key, n);
      } else if (n < a.V + nz && mvalid) {
        a.zs[(size_t)m * nz + (n - a.V)] = z;
      }
    }
  }
  // the two lanes that share a hypothesis (l and l ^ 32) combine
  {
    const float mx2 = __shfl_xor(mx, 32), sum2 = __shfl_xor(sum, 32);
    const float mm2 = fmaxf(mx, mx2);
    float s = 0.f;
    if (mx > -INFINITY) s += sum * __expf(mx - mm2);
    if (mx2 > -INFINITY) s += sum2 * __expf(mx2 - mm2);
    mx = mm2;
    sum = s;
  }
  {
    // every lane takes a copy of its partner's list, then inserts it; both end with the same merged list
    float pv[KT];
    int pi[KT];
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      pv[j] = __shfl_xor(top.v[j], 32);
      pi[j] = __shfl_xor(top.i[j], 32);
    }
#pragma unroll
    for (int j = 0; j < KT; ++j) top.insert(pv[j], pi[j]);
  }
  if (half == 0 && mvalid) {
    const size_t pc = (size_t)m * a.n_chunks + chunk;
    a.p_max[pc] = mx;
    a.p_sum[pc] = sum;
#pragma unroll
    for (int j = 0; j < KT; ++j)
      if (j < a.K) {
        a.p_key[pc * a.K + j] = top.v[j];
        a.p_idx[pc * a.K + j] = top.i[j];
      }
  }
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
  float *p_key;
  int *p_idx;
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
  const size_t pc = (size_t)m * 64 + lane;
#pragma unroll
  for (int j = 0; j < KT; ++j)
    if (j < a.K) {
      a.p_key[pc * a.K + j] = top.v[j];
      a.p_idx[pc * a.K + j] = top.i[j];
    }
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
  // candidate lists from k_joint / k_inject
  const float *p_max, *p_sum, *p_key;
  const int *p_idx;
  const float *zs;
  int n_chunks;
  int normalized;  // 1: keys are log-probabilities already (injected mode)
  // configuration
  int B, K, V, ND;
  int dur[8];
  int algo, max_sym;
  float gamma;
  int has_lm;
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

__global__ __launch_bounds__(256) void k_select(SelectArgs a) {
  if (*reinterpret_cast<volatile int *>(a.done)) return;
  const int b = blockIdx.x, K = a.K, V = a.V, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m_base = b * K;
  if (a.finished[b]) {
    if (tid < K) {
      a.src_row[m_base + tid] = m_base + tid;
      a.tok[m_base + tid] = -1;
    }
    return;
  }
  const int S = *a.step_base + a.step_off;
  const int T_b = a.lengths[b];
  const int nz = 1 + a.ND;

  __shared__ double s_score[kMaxBeam];
  __shared__ int s_t[kMaxBeam], s_sym[kMaxBeam], s_len[kMaxBeam], s_last[kMaxBeam], s_kind[kMaxBeam];
  __shared__ uint32_t s_hash[kMaxBeam];
  __shared__ int s_ctx[kMaxBeam][kCtxMax];
  __shared__ int s_advt[kMaxBeam], s_advb[kMaxBeam];
  __shared__ double rc_val[kMaxBeam][kMaxBeam + 1];
  __shared__ int rc_tok[kMaxBeam][kMaxBeam + 1];
  __shared__ double sel_val[kMaxBeam];
  __shared__ int sel_k[kMaxBeam], sel_v[kMaxBeam];
  // new state
  __shared__ double n_score[kMaxBeam];
  __shared__ int n_t[kMaxBeam], n_sym[kMaxBeam], n_len[kMaxBeam], n_last[kMaxBeam], n_live[kMaxBeam];
  __shared__ uint32_t n_hash[kMaxBeam];

  if (tid < K) {
    const int m = m_base + tid;
    s_score[tid] = a.score[m];
    s_t[tid] = a.t[m];
    s_sym[tid] = a.sym[m];
    s_len[tid] = a.len[m];
    s_last[tid] = a.last[m];
    s_hash[tid] = a.hash[m];
#pragma unroll
    for (int i = 0; i < kCtxMax; ++i) s_ctx[tid][i] = a.ctx[m * kCtxMax + i];
  }
  __syncthreads();
  int t_cur = T_b;
  for (int k = 0; k < K; ++k)
    if (s_score[k] > -INFINITY && s_t[k] < T_b && s_t[k] < t_cur) t_cur = s_t[k];
  if (tid < K) {
    int kind = 0;
    if (s_score[tid] > -INFINITY) kind = (s_t[tid] < T_b && (a.algo == 0 || s_t[tid] == t_cur)) ? 2 : 1;
    s_kind[tid] = kind;
  }
  __syncthreads();

  // ---- per hypothesis: the K best tokens and blank, as total scores
  for (int k = wave; k < K; k += 4) {
    const int m = m_base + k;
    const int kind = s_kind[k];
    if (kind != 2) {
      if (lane <= K) {
        rc_val[k][lane] = (kind == 1 && lane == K) ? s_score[k] : -INFINITY;
        rc_tok[k][lane] = V;
      }
      continue;
    }
    const int ncand = a.n_chunks * K;
    const float *keys = a.p_key + (size_t)m * ncand;
    const int *idxs = a.p_idx + (size_t)m * ncand;
    // K rounds of "best remaining candidate"
    float my_key = -INFINITY;  // lane j keeps the j-th winner
    int my_idx = 0x7fffffff;
    float last_v = INFINITY;
    int last_i = -1;
    for (int j = 0; j < K; ++j) {
      float bv = -INFINITY;
      int bi = 0x7fffffff;
      for (int c = lane; c < ncand; c += 64) {
        const float v = keys[c];
        const int i = idxs[c];
        const bool eligible = v > -INFINITY && (v < last_v || (v == last_v && i > last_i));
        if (eligible && comes_before(v, i, bv, bi)) {
          bv = v;
          bi = i;
        }
      }
      wave_best(bv, bi);
      if (lane == j) {
        my_key = bv;
        my_idx = bi;
      }
      last_v = bv;
      last_i = bi;
      if (bv == -INFINITY) break;
    }
    // soft-max statistics
    double lse_all = 0.0, lse_nb = 0.0, max_nb;
    const double zb = (double)a.zs[(size_t)m * nz];
    if (!a.normalized) {
      float mx = -INFINITY;
      for (int c = lane; c < a.n_chunks; c += 64) mx = fmaxf(mx, a.p_max[(size_t)m * a.n_chunks + c]);
      mx = wave_max(mx);
      double s = 0.0;
      for (int c = lane; c < a.n_chunks; c += 64) {
        const float pm = a.p_max[(size_t)m * a.n_chunks + c];
        if (pm > -INFINITY) s += (double)a.p_sum[(size_t)m * a.n_chunks + c] * exp((double)pm - (double)mx);
      }
      s = wave_sum(s);
      lse_nb = (double)mx + log(s);
      lse_all = logaddexp_d(lse_nb, zb);
      max_nb = (double)mx;
    } else {
      max_nb = (double)__shfl(my_key, 0);
    }
    const double logp_b = zb - lse_all;
    const double nb = lse_nb - lse_all;
    const double maxlogp = fmax(max_nb, zb) - lse_all;
    // TDT: one duration per candidate
    double x_tok = 0.0, x_blank = 0.0;
    int adv_tok = 0, adv_blank = 1;
    if (a.ND > 0) {
      double dl[8];
      double dmx = -INFINITY;
      for (int d = 0; d < a.ND; ++d) {
        dl[d] = (double)a.zs[(size_t)m * nz + 1 + d];
        dmx = fmax(dmx, dl[d]);
      }
      if (!a.normalized) {
        double s = 0.0;
        for (int d = 0; d < a.ND; ++d) s += exp(dl[d] - dmx);
        const double l = dmx + log(s);
        for (int d = 0; d < a.ND; ++d) dl[d] -= l;
      }
      int best = -1, best_b = -1;
      for (int d = 0; d < a.ND; ++d) {
        if (best < 0 || dl[d] > dl[best]) best = d;
        if (a.dur[d] >= 1 && (best_b < 0 || dl[d] > dl[best_b])) best_b = d;
      }
      x_tok = dl[best];
      x_blank = dl[best_b];
      adv_tok = a.dur[best];
      adv_blank = a.dur[best_b];
    }
    const bool forced = s_sym[k] >= a.max_sym;
    const bool use_gamma = a.algo == 1 && a.gamma < INFINITY;
    const double thr = maxlogp - (double)a.gamma;
    const double sc = s_score[k];
    if (lane < K) {
      double val = -INFINITY;
      if (my_key > -INFINITY && !forced) {
        const double lp = (double)my_key - lse_all;  // pre-LM log-probability when no LM is fused
        if (!(use_gamma && lp < thr)) val = sc + lp + (a.has_lm ? (double)a.lambda * nb : 0.0) + x_tok;
      }
      rc_val[k][lane] = val;
      rc_tok[k][lane] = my_idx;
    }
    if (lane == K) {
      double val = a.has_lm ? (1.0 + (double)a.lambda) * logp_b : logp_b;
      if (use_gamma && logp_b < thr && !forced) val = -INFINITY;
      rc_val[k][K] = sc + val + x_blank;
      rc_tok[k][K] = V;
      s_advt[k] = adv_tok;
      s_advb[k] = adv_blank;
    }
  }
  __syncthreads();

  // ---- the Beam best of all K * (K + 1) candidates, by (value desc, k * (V + 1) + v asc)
  if (wave == 0) {
    const int n = K * (K + 1);
    double last_v = INFINITY;
    long long last_i = -1;
    for (int j = 0; j < K; ++j) {
      double bv = -INFINITY;
      long long bi = 0x7fffffffffffffffll;
      for (int c = lane; c < n; c += 64) {
        const int k = c / (K + 1), e = c % (K + 1);
        const double v = rc_val[k][e];
        const long long i = (long long)k * (V + 1) + rc_tok[k][e];
        const bool eligible = v > -INFINITY && (v < last_v || (v == last_v && i > last_i));
        if (eligible && comes_before(v, i, bv, bi)) {
          bv = v;
          bi = i;
        }
      }
      wave_best(bv, bi);
      if (lane == 0) {
        sel_val[j] = bv;
        sel_k[j] = bv > -INFINITY ? (int)(bi / (V + 1)) : -1;
        sel_v[j] = bv > -INFINITY ? (int)(bi % (V + 1)) : -1;
      }
      last_v = bv;
      last_i = bi;
    }
  }
  __syncthreads();

  // ---- expansion into the new slots
  int code = -3, parent = -1, appended = -1;
  int ctx_new[kCtxMax];
  if (tid < K) {
    const int j = tid;
    const double val = sel_val[j];
    if (!(val > -INFINITY)) {
      n_live[j] = 0;
      n_score[j] = -INFINITY;
      n_t[j] = 0;
      n_sym[j] = 0;
      n_len[j] = 0;
      n_last[j] = -1;
      n_hash[j] = 0;
#pragma unroll
      for (int i = 0; i < kCtxMax; ++i) ctx_new[i] = -1;
    } else {
      const int k = sel_k[j], v = sel_v[j];
      parent = k;
      int t = s_t[k], sym = s_sym[k], len = s_len[k], last = s_last[k];
      uint32_t hash = s_hash[k];
#pragma unroll
      for (int i = 0; i < kCtxMax; ++i) ctx_new[i] = s_ctx[k][i];
      if (s_kind[k] == 1) {
        code = -2;
      } else if (v == V) {
        code = -1;
        t += s_advb[k];
        sym = 0;
      } else {
        code = v;
        appended = v;
        len += 1;
        last = v;
        hash = (uint32_t)(((uint64_t)hash * kHashBase + (uint64_t)(v + 1)) % kHashMod);
        t += s_advt[k];
        sym = s_advt[k] == 0 ? sym + 1 : 0;
#pragma unroll
        for (int i = kCtxMax - 1; i > 0; --i) ctx_new[i] = ctx_new[i - 1];
        ctx_new[0] = v;
      }
      if (t > T_b) t = T_b;
      n_live[j] = 1;
      n_score[j] = val;
      n_t[j] = t;
      n_sym[j] = sym;
      n_len[j] = len;
      n_last[j] = last;
      n_hash[j] = hash;
    }
  }
  __syncthreads();

  // ---- recombination: equal (hash, length, last token, frame, symbols in frame)
  if (tid < K) {
    const int j = tid;
    int merged = -1;
    double score = n_score[j];
    bool live = n_live[j] != 0;
    if (live) {
      merged = j;
      for (int i = 0; i < j; ++i) {
        if (n_live[i] && n_hash[i] == n_hash[j] && n_len[i] == n_len[j] && n_last[i] == n_last[j] &&
            n_t[i] == n_t[j] && n_sym[i] == n_sym[j]) {
          merged = i;
          break;
        }
      }
      if (merged == j) {
        for (int i = j + 1; i < K; ++i)
          if (n_live[i] && n_hash[i] == n_hash[j] && n_len[i] == n_len[j] && n_last[i] == n_last[j] &&
              n_t[i] == n_t[j] && n_sym[i] == n_sym[j])
            score = logaddexp_d(score, n_score[i]);
      } else {
        live = false;
        score = -INFINITY;
      }
    }
    const int m = m_base + j;
    a.score[m] = score;
    a.t[m] = n_t[j];
    a.sym[m] = n_sym[j];
    a.len[m] = n_len[j];
    a.last[m] = n_last[j];
    a.hash[m] = n_hash[j];
#pragma unroll
    for (int i = 0; i < kCtxMax; ++i) a.ctx[m * kCtxMax + i] = ctx_new[i];
    a.src_row[m] = parent >= 0 ? m_base + parent : m;
    a.tok[m] = appended;
    if (S < a.S_max) {
      const size_t ti = ((size_t)b * a.S_max + S) * K + j;
      a.tree_parent[ti] = parent;
      a.tree_token[ti] = code;
      a.tree_merged[ti] = merged;
    }
    // second pass over shared state needs the surviving flags
    s_kind[j] = live ? 1 : 0;
  }
  __syncthreads();
  if (tid == 0) {
    bool unfinished = false;
    for (int j = 0; j < K; ++j)
      if (s_kind[j] && n_t[j] < T_b) unfinished = true;
    if (!unfinished || S + 1 >= T_b * (a.max_sym + 1)) {
      a.finished[b] = 1;
      a.utt_steps[b] = S + 1;
      __threadfence();
      const int old = atomicAdd(a.n_finished, 1);
      if (old + 1 == a.B) {
        *reinterpret_cast<volatile int *>(a.done) = 1;
        __threadfence_system();
        *a.h_done = 1;
      }
    }
  }
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

__global__ __launch_bounds__(256) void k_lstm(const float *__restrict__ Whh, const float *__restrict__ G,
                                              const float *__restrict__ h_cur, const float *__restrict__ c_cur,
                                              float *__restrict__ h_nxt, float *__restrict__ c_nxt,
                                              const int *__restrict__ src_row, const int *__restrict__ tok, int M,
                                              int P, const int *done) {
  if (*reinterpret_cast<const volatile int *>(done)) return;
  __shared__ float red[3 * 16 * 64];
  const int lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int tile = blockIdx.x, m = blockIdx.y * 32 + col;
  const bool mvalid = m < M;
  const int src = mvalid ? src_row[m] : 0;
  const float *wp = Whh + (size_t)(tile * 32 + col) * P;
  const float *hp = h_cur + (size_t)src * P;
  auto a_at = [&](int k) { return *reinterpret_cast<const float4 *>(wp + k); };
  auto b_at = [&](int k) { return *reinterpret_cast<const float4 *>(hp + k); };
  floatx16 acc = splitk_tile(a_at, b_at, P, red);
  if (threadIdx.x >= 64 || !mvalid) return;
  const int token = tok[m];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int ul = 2 * q + half, u = tile * 8 + ul;
    float c, h;
    if (token >= 0) {
      const float4 g4 = *reinterpret_cast<const float4 *>(G + (size_t)token * 4 * P + tile * 32 + 4 * ul);
      const float gi = acc[4 * q + 0] + g4.x, gf = acc[4 * q + 1] + g4.y, gg = acc[4 * q + 2] + g4.z,
                  go = acc[4 * q + 3] + g4.w;
      c = sigmoid_f(gf) * c_cur[(size_t)src * P + u] + sigmoid_f(gi) * tanh_f(gg);
      h = sigmoid_f(go) * tanh_f(c);
    } else {
      c = c_cur[(size_t)src * P + u];
      h = h_cur[(size_t)src * P + u];
    }
    c_nxt[(size_t)m * P + u] = c;
    h_nxt[(size_t)m * P + u] = h;
  }
}

// g_proj[m] = W_pred h[m] + b_pred
__global__ __launch_bounds__(256) void k_pred_proj(const float *__restrict__ Wp, const float *__restrict__ bias,
                                                   const float *__restrict__ h, float *__restrict__ g, int M, int P,
                                                   int H, int round_ops, const int *done, int *step_base,
                                                   int bump) {
  if (*reinterpret_cast<const volatile int *>(done)) return;
  __shared__ float red[3 * 16 * 64];
  const int lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int tile = blockIdx.x, m = blockIdx.y * 32 + col;
  const bool mvalid = m < M;
  const float *wp = Wp + (size_t)(tile * 32 + col) * P;
  const float *hp = h + (size_t)(mvalid ? m : 0) * P;
  auto a_at = [&](int k) { return *reinterpret_cast<const float4 *>(wp + k); };
  auto b_at = [&](int k) {
    float4 v = *reinterpret_cast<const float4 *>(hp + k);
    if (round_ops) v = bf16_round4(v);
    return v;
  };
  floatx16 acc = splitk_tile(a_at, b_at, P, red);
  if (bump && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *step_base += bump;
  if (threadIdx.x >= 64 || !mvalid) return;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int j = tile * 32 + 8 * q + 4 * half;
    const float4 bv = *reinterpret_cast<const float4 *>(bias + j);
    float4 o = make_float4(acc[4 * q] + bv.x, acc[4 * q + 1] + bv.y, acc[4 * q + 2] + bv.z, acc[4 * q + 3] + bv.w);
    *reinterpret_cast<float4 *>(g + (size_t)m * H + j) = o;
  }
}

__global__ void k_fill_int(int *p, int value, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = value;
}

// advances the step counter when no prediction projection closes the step (stateless, injected)
__global__ void k_bump(int *step_base, int bump, const int *done) {
  if (*reinterpret_cast<const volatile int *>(done)) return;
  if (threadIdx.x == 0 && blockIdx.x == 0) *step_base += bump;
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
  float *h0, *c0;  // [M, P] zeroed state the first LSTM step reads (nullable)
  int P;
  int B, K, T, V, lstm;
  int *finished, *utt_steps, *n_finished, *done, *step_base, *bad_arg;
  volatile int *h_done;
};

__global__ void k_init(InitArgs a) {
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;
  const int M = a.B * a.K;
  if (gid == 0) {
    *a.step_base = 0;
    int nfin = 0;
    for (int b = 0; b < a.B; ++b) {
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
    *a.n_finished = nfin;
    *a.done = nfin == a.B;
    *a.h_done = nfin == a.B;
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
  if (a.h0) {
    const size_t n = (size_t)M * a.P;
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
  int K, S_max, cap, use_lds;
  int *out_tokens;     // [B, K, cap]
  int *out_lens;       // [B, K]
  double *out_scores;  // [B, K]
  int *out_steps;      // [B]
};

__global__ __launch_bounds__(64) void k_backtrace(BacktraceArgs a) {
  extern __shared__ int tree_lds[];
  const int b = blockIdx.x, K = a.K, tid = threadIdx.x;
  int n = a.utt_steps[b];
  if (n < 0) n = min(*a.step_base, a.S_max);
  if (tid == 0) a.out_steps[b] = n;
  const int *gp = a.tree_parent + (size_t)b * a.S_max * K;
  const int *gt = a.tree_token + (size_t)b * a.S_max * K;
  const int *lp = gp, *lt = gt;
  if (a.use_lds) {
    int *sp = tree_lds, *st = tree_lds + n * K;
    for (int i = tid; i < n * K; i += 64) {
      sp[i] = gp[i];
      st[i] = gt[i];
    }
    lp = sp;
    lt = st;
  }
  __syncthreads();
  if (tid >= K) return;
  const double my = a.score[b * K + tid];
  int pos = 0;
  for (int i = 0; i < K; ++i) {
    const double o = a.score[b * K + i];
    if (o > my || (o == my && i < tid)) ++pos;
  }
  const size_t oi = (size_t)b * K + pos;
  if (!(my > -INFINITY)) {
    a.out_lens[oi] = -1;
    a.out_scores[oi] = -INFINITY;
    return;
  }
  int u = a.len[b * K + tid];
  a.out_lens[oi] = u;
  a.out_scores[oi] = my;
  int cur = tid;
  for (int st = n - 1; st >= 0 && cur >= 0; --st) {
    const int tk = lt[st * K + cur];
    if (tk >= 0) {
      --u;
      if (u >= 0 && u < a.cap) a.out_tokens[oi * a.cap + u] = tk;
    }
    cur = lp[st * K + cur];
  }
}

}  // namespace rb
