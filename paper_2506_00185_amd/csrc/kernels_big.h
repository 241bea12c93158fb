// Kernels for large (hypotheses x vocabulary) products with a bf16 joint: the joint's output
// layer as a bf16 matrix-core contraction that writes float32 logits, and a row-wise exact
// top-K over them.  A step of this mode is
//   k_joint_big -> k_utt_select (one block per utterance: row scan, selection, next activations), or, with an LM
//   term in the keys, k_joint_big -> k_row_select (one block per hypothesis; the block that completes an utterance
//   runs the selection and writes the next activations in its tail).
// Keeping the per-row top-K in the contraction's epilogue, as the small-shape kernel does, costs
// more vector instructions at K = 10 and V = 8192 than the trip of the logits through HBM.  The epilogue does
// keep the maximum and the sum of exponentials of every (hypothesis, 32-column chunk), so that the row kernel
// reads 8 bytes per chunk and then only the few chunks that can hold one of the K best keys.
#pragma once
#include "kernels.h"

namespace rb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// bf16 operand layout ("k8-major"): element (row, k) of an R-row matrix at ((k / 8) * R + row) * 8 + k % 8,
// so that a lane's 8 consecutive k are one 16-byte load and 32 consecutive rows are 512 contiguous bytes.
__host__ __device__ inline size_t k8_index(int k, int row, int rows) {
  return ((size_t)(k >> 3) * rows + row) * 8 + (k & 7);
}

__device__ __forceinline__ uint16_t bf16_bits(float x) {  // round to nearest even
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// acc[i][j] += sum_{k<16} A[i][k] B[k][j] on the bf16 matrix cores.  Lane l supplies
// A[i = l % 32][k = 8 * (l / 32) .. + 7] and B[k = 8 * (l / 32) .. + 7][j = l % 32] and receives
// acc[i = 8 * (r / 4) + 4 * (l / 32) + r % 4][j = l % 32] in register r.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ floatx16 mfma32_bf16(u32x4 a, u32x4 b, floatx16 acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0,
                                                 0);
}

struct BigJointArgs {
  const uint16_t *Wb;  // bf16 k8-major [H][Npad] output layer (token rows; rows >= V are zero)
  const uint16_t *Ab;  // bf16 k8-major [H][Mp]: ReLU(pre), rounded
  const float *bias;   // [Npad]
  float *Z;            // [M][Npad] logits of the token columns
  uint64_t *cstat;     // [M][Npad / 32] (maximum, sum of exp(z - maximum)) of each 32-column chunk, two floats
  int M, Mp, H, Npad;
  XcdMap map;          // role 0: (block of 256 columns, block of 32 * MS rows)
  const int *done;
  int *step_base;      // advanced by `bump` before anything of this step reads it (first step of a chunk of steps,
  int bump;            // when the selection runs in the tail of the row kernel and no later launch closes the step)
  volatile int *h_progress = nullptr;  // see bump_step
};

// Z[m][n] = W_out[n] . a_m + b_out[n] for a block of 32 * WAVES columns x 160 hypotheses.
// Two waves per SIMD (one block of 8 waves or two of 4): a wave issues in order and nothing of its own
// overlaps with its matrix instructions (measured: 30 vector instructions beside 10 matrix ones cost
// their full 4 cycles each), so the loads, LDS traffic and barriers of one wave have to run while the
// SIMD's other wave multiplies.
// Wave w owns 32 columns x all five hypothesis tiles (80 accumulator registers).  A stage is two k-steps
// of 16: the wave's own output-layer rows come straight from global memory into a ring of D register
// sets, requested D stages ahead; the activation tile (160 x 32, 10 KB) is shared, so it goes
// registers -> LDS one stage ahead of its use, in a ring of three slots with one barrier per stage.
// The stage loop has no branches, so that the compiler's count of outstanding loads stays exact.
// Needs H % (32 * D) == 0 (the caller pads the operands with zeros along k).
// The vocabulary is the row index of the matrix-core product and the hypotheses its columns: a lane ends up with
// 16 logits of ONE hypothesis (four runs of four consecutive columns), so the chunk statistics need no reduction
// across lanes beyond one exchange between the wave's halves.  A tile then goes through LDS (transposed) so that
// eight lanes store the 128 contiguous bytes of a hypothesis' chunk (16-byte stores scattered over 32 rows took
// twice as long as stores of whole 128-byte runs, non-temporal ones four times).
template <int WAVES, int D>
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void k_joint_big(BigJointArgs a) {
  constexpr int MS = 5, NP = 2 * MS;  // pieces (k-step, hypothesis tile) of 1 KB per stage
  constexpr int PW = NP / WAVES;      // pieces a wave loads whole, 16 bytes per lane (pieces wave, wave + WAVES, ..)
  constexpr int FP = PW * WAVES;      // the other NP - FP pieces are loaded 4 bytes per thread
  constexpr int XD = (NP - FP) * 256 / (64 * WAVES);
  static_assert(WAVES == 4 || WAVES == 8, "two waves per SIMD: one block of 8 or two blocks of 4");
  // activation ring of three slots; the epilogue reuses the memory (transposition buffers + chunk statistics)
  constexpr int TS = 36;  // floats per hypothesis in a transposition buffer (32 + 4: 16-byte aligned rows)
  constexpr size_t kRingBytes = sizeof(u32x4) * 3 * NP * 64;
  constexpr size_t kEpiBytes = (size_t)WAVES * 32 * TS * 4 + (size_t)32 * MS * WAVES * 8;
  __shared__ __align__(16) unsigned char lds_raw[kRingBytes > kEpiBytes ? kRingBytes : kEpiBytes];
  u32x4 (*tile)[NP][64] = reinterpret_cast<u32x4 (*)[NP][64]>(lds_raw);
  const int done = *reinterpret_cast<const volatile int *>(a.done);
  if (a.bump && !done && blockIdx.x == 0 && threadIdx.x == 0) bump_step(a.step_base, a.bump, a.h_progress);
  int nb, mb;
  if (xcd_item(a.map, blockIdx.x, nb, mb) != 0) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 31, kg = lane >> 5;
  const int n0 = (nb * WAVES + wave) * 32, m0 = mb * 32 * MS;
  const char *wbase = reinterpret_cast<const char *>(a.Wb), *abase = reinterpret_cast<const char *>(a.Ab);
  const size_t wks = (size_t)2 * a.Npad * 16, aks = (size_t)2 * a.Mp * 16;  // bytes per k-step (two k8 groups)
  const uint32_t woff = (uint32_t)(((size_t)kg * a.Npad + n0 + col) * 16);
  auto act_off = [&](int piece, int l) {  // the 16 bytes that lane l feeds to the matrix cores for a piece
    int row = m0 + 32 * (piece % MS) + (l & 31);
    row = row < a.Mp ? row : a.Mp - 1;
    return (uint32_t)((piece / MS) * aks + ((size_t)(l >> 5) * a.Mp + row) * 16);
  };
  uint32_t aoff[PW], xoff[XD];
#pragma unroll
  for (int i = 0; i < PW; ++i) aoff[i] = act_off(wave + WAVES * i, lane);
#pragma unroll
  for (int d = 0; d < XD; ++d) {
    const int g = tid + 64 * WAVES * d;  // dword g of the pieces FP .. NP - 1
    xoff[d] = act_off(FP + (g >> 8), (g & 255) >> 2) + 4 * (g & 3);
  }
  const int n_st = a.H / 32;
  u32x4 wr[D][2], ar[D][PW];
  uint32_t xr[D][XD];
  auto request = [&](int set, int st) {
    const char *wk = wbase + (size_t)st * 2 * wks, *ak = abase + (size_t)st * 2 * aks;
    wr[set][0] = *reinterpret_cast<const u32x4 *>(wk + woff);
    wr[set][1] = *reinterpret_cast<const u32x4 *>(wk + wks + woff);
#pragma unroll
    for (int i = 0; i < PW; ++i) ar[set][i] = *reinterpret_cast<const u32x4 *>(ak + aoff[i]);
#pragma unroll
    for (int d = 0; d < XD; ++d) xr[set][d] = *reinterpret_cast<const uint32_t *>(ak + xoff[d]);
  };
  auto stage = [&](int set, int slot) {  // activation tile of a stage: registers -> LDS
#pragma unroll
    for (int i = 0; i < PW; ++i) tile[slot][wave + WAVES * i][lane] = ar[set][i];
#pragma unroll
    for (int d = 0; d < XD; ++d) reinterpret_cast<uint32_t *>(&tile[slot][FP][0])[tid + 64 * WAVES * d] = xr[set][d];
  };
  floatx16 acc[MS];
  auto multiply = [&](int set, int slot) {
    u32x4 bf[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) bf[p] = tile[slot][p][lane];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int t = 0; t < MS; ++t) acc[t] = mfma32_bf16(wr[set][kk], bf[kk * MS + t], acc[t]);
  };
#pragma unroll
  for (int j = 0; j < D; ++j) request(j, j);
  if (done) return;
#pragma unroll
  for (int t = 0; t < MS; ++t) acc[t] = floatx16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  // stage st: operands in register set st % D, activation tile in LDS slot st % 3.  The slot written in
  // an iteration was last read two iterations (two barriers) earlier.
  stage(0, 0);
  __syncthreads();
  int s0 = 0, s1 = 1, s2 = 2;  // slots of stages st, st + 1, st + 2
  for (int st0 = 0; st0 < n_st - D; st0 += D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      stage((j + 1) % D, s1);
      multiply(j, s0);
      request(j, st0 + j + D);
      __syncthreads();
      const int r = s0;
      s0 = s1;
      s1 = s2;
      s2 = r;
    }
  }
#pragma unroll
  for (int j = 0; j < D; ++j) {  // last D stages: nothing left to request
    if (j + 1 < D) stage(j + 1, s1);
    multiply(j, s0);
    if (j + 1 < D) __syncthreads();
    const int r = s0;
    s0 = s1;
    s1 = s2;
    s2 = r;
  }
  // epilogue: register r of tile t is column n0 + 8 (r / 4) + 4 kg + r % 4 of hypothesis m0 + 32 t + col
  __syncthreads();  // every wave is through with the activation ring, which the buffers below reuse
  float *tr = reinterpret_cast<float *>(lds_raw) + wave * 32 * TS;
  uint64_t *stat = reinterpret_cast<uint64_t *>(reinterpret_cast<float *>(lds_raw) + WAVES * 32 * TS);
  floatx4 b4[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) b4[g] = *reinterpret_cast<const floatx4 *>(a.bias + n0 + 8 * g + 4 * kg);
  const float kLog2e = 1.4426950408889634f;
#pragma unroll
  for (int t = 0; t < MS; ++t) {
    floatx4 v[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int e = 0; e < 4; ++e) v[g][e] = acc[t][4 * g + e] + b4[g][e];
    float mx = -INFINITY;
#pragma unroll
    for (int g = 0; g < 4; ++g) mx = fmaxf(mx, fmaxf(fmaxf(v[g][0], v[g][1]), fmaxf(v[g][2], v[g][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float off = mx > -INFINITY ? -mx * kLog2e : 0.f;  // (a chunk of padding columns holds -inf only)
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < 4; ++g)
      sum += (exp2f(fmaf(v[g][0], kLog2e, off)) + exp2f(fmaf(v[g][1], kLog2e, off))) +
             (exp2f(fmaf(v[g][2], kLog2e, off)) + exp2f(fmaf(v[g][3], kLog2e, off)));
    sum += __shfl_xor(sum, 32);
    if (kg == 0) stat[(32 * t + col) * WAVES + wave] = ((uint64_t)__float_as_uint(sum) << 32) | __float_as_uint(mx);
#pragma unroll
    for (int g = 0; g < 4; ++g) *reinterpret_cast<floatx4 *>(tr + col * TS + 8 * g + 4 * kg) = v[g];
    wave_sync();  // (the buffer is this wave's own)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int hl = (lane >> 3) + 8 * i, q = lane & 7;
      const floatx4 x = *reinterpret_cast<const floatx4 *>(tr + hl * TS + 4 * q);
      const int m = m0 + 32 * t + hl;
      if (m < a.M) store16_through(a.Z + (size_t)m * a.Npad + n0 + 4 * q, x);
    }
    wave_sync();
  }
  __syncthreads();
  const int n_stat = a.Npad >> 5;
  for (int i = tid; i < 32 * MS * WAVES; i += 64 * WAVES) {
    const int m = m0 + i / WAVES;
    if (m < a.M) store_through(a.cstat + (size_t)m * n_stat + nb * WAVES + i % WAVES, stat[i]);
  }
}

// Stateless prediction network for the large mode: a_m = bf16(ReLU(f_proj[b, t_m] + sum_i tab_i[token_i]))
// written k8-major.  One thread per (hypothesis, group of 8 outputs).
struct StatelessPreBigArgs {
  const float *f_proj, *tab;
  const int *ctx_tok, *t, *lengths;
  uint16_t *Ab;
  int M, Mp, K, T, H, V, n_ctx;
  const int *done;
  int *step_base;
  int bump;
  volatile int *h_progress = nullptr;  // see bump_step
};

// a_m[8 o8 .. + 7] for hypothesis m of utterance b standing at frame tt with token history toks (most recent first)
__device__ __forceinline__ void stateless_pre_big_item(const StatelessPreBigArgs &a, int m, int b, int tt, const int *toks,
                                                       int o8) {
  const float *fp = a.f_proj + ((size_t)b * a.T + tt) * a.H + 8 * o8;
  float v[8];
  {
    const float4 x = *reinterpret_cast<const float4 *>(fp), y = *reinterpret_cast<const float4 *>(fp + 4);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
  }
  for (int i = 0; i < a.n_ctx; ++i) {
    int tk = toks[i];
    tk = tk < 0 ? a.V : tk;
    const float *gp = a.tab + ((size_t)i * (a.V + 1) + tk) * a.H + 8 * o8;
    const float4 x = *reinterpret_cast<const float4 *>(gp), y = *reinterpret_cast<const float4 *>(gp + 4);
    v[0] += x.x; v[1] += x.y; v[2] += x.z; v[3] += x.w; v[4] += y.x; v[5] += y.y; v[6] += y.z; v[7] += y.w;
  }
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = (uint32_t)bf16_bits(fmaxf(v[2 * i], 0.f)) | ((uint32_t)bf16_bits(fmaxf(v[2 * i + 1], 0.f)) << 16);
  *reinterpret_cast<uint4 *>(a.Ab + ((size_t)o8 * a.Mp + m) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
}

// two items at once: every load of both is requested before either is finished (the second may be a repeat of the
// first, `two` false: it is then not stored)
__device__ __forceinline__ void stateless_pre_big_pair(const StatelessPreBigArgs &a, int m1, int tt1, const int *toks1, int o81,
                                                       int m2, int tt2, const int *toks2, int o82, int b, bool two) {
  const float *fp1 = a.f_proj + ((size_t)b * a.T + tt1) * a.H + 8 * o81;
  const float *fp2 = a.f_proj + ((size_t)b * a.T + tt2) * a.H + 8 * o82;
  floatx4 v1[2] = {*reinterpret_cast<const floatx4 *>(fp1), *reinterpret_cast<const floatx4 *>(fp1 + 4)};
  floatx4 v2[2] = {*reinterpret_cast<const floatx4 *>(fp2), *reinterpret_cast<const floatx4 *>(fp2 + 4)};
  floatx4 g1[4][2], g2[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (i < a.n_ctx) {
      int t1 = toks1[i], t2 = toks2[i];
      t1 = t1 < 0 ? a.V : t1;
      t2 = t2 < 0 ? a.V : t2;
      const float *p1 = a.tab + ((size_t)i * (a.V + 1) + t1) * a.H + 8 * o81;
      const float *p2 = a.tab + ((size_t)i * (a.V + 1) + t2) * a.H + 8 * o82;
      g1[i][0] = *reinterpret_cast<const floatx4 *>(p1);
      g1[i][1] = *reinterpret_cast<const floatx4 *>(p1 + 4);
      g2[i][0] = *reinterpret_cast<const floatx4 *>(p2);
      g2[i][1] = *reinterpret_cast<const floatx4 *>(p2 + 4);
    }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (i < a.n_ctx) {
      v1[0] += g1[i][0]; v1[1] += g1[i][1];
      v2[0] += g2[i][0]; v2[1] += g2[i][1];
    }
  auto put = [&](int m, int o8, const floatx4(&v)[2]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float lo = v[i >> 1][2 * (i & 1)], hi = v[i >> 1][2 * (i & 1) + 1];
      w[i] = (uint32_t)bf16_bits(fmaxf(lo, 0.f)) | ((uint32_t)bf16_bits(fmaxf(hi, 0.f)) << 16);
    }
    *reinterpret_cast<uint4 *>(a.Ab + ((size_t)o8 * a.Mp + m) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  };
  put(m1, o81, v1);
  if (two) put(m2, o82, v2);
}

__global__ __launch_bounds__(256) void k_stateless_pre_big(StatelessPreBigArgs a) {
  if (*reinterpret_cast<const volatile int *>(a.done)) return;
  const int gid = blockIdx.x * 256 + threadIdx.x;
  if (a.bump && gid == 0) bump_step(a.step_base, a.bump, a.h_progress);
  const int H8 = a.H >> 3;
  const int m = gid / H8, o8 = gid % H8;
  if (m >= a.M) return;
  const int b = m / a.K;
  const int T_b = a.lengths[b];
  int tt = a.t[m];
  tt = tt < T_b ? tt : T_b - 1;
  tt = tt < 0 ? 0 : tt;
  stateless_pre_big_item(a, m, b, tt, a.ctx_tok + m * kCtxMax, o8);
}

struct RowSelectArgs {
  const float *Z;        // [M][Npad]
  const uint64_t *cstat; // [M][Npad / 32] chunk statistics written with the logits (see BigJointArgs)
  int Npad;
  const uint16_t *Ab;    // bf16 k8-major [H][Mp]
  int M, Mp, H, K, V, ND;
  const float *Wspec;    // [1 + ND][H] rows V .. V + ND of the output layer (bf16-rounded values)
  const float *bias_spec;
  const float *lm;       // [M][V] or NULL
  float lambda;
  float *p_max, *p_sum;  // [M] (one list per row)
  uint64_t *p_cand;      // [M][K]
  float *zs;             // [M][1 + ND]
  const int *finished;   // [B]
  const int *done;
  // TAIL: the block that completes an utterance (counted in utt_ctr) runs its selection and writes the
  // activations of its new hypotheses, so that the step needs no further launch
  int *utt_ctr;          // [B], zero between steps
  SelectArgs sel;
  StatelessPreBigArgs pre;
};

constexpr int kRowWaves = 4;       // waves that share a row
constexpr int kRowRegs = 8;        // float4 registers per lane: V <= kRowWaves * 64 * 4 * kRowRegs = 8192
constexpr int kSurvivorCap = 256;

// One block of four waves per hypothesis: exact K best of the row's keys (as a one-chunk candidate list
// for the selection), soft-max statistics, blank / duration logits.  Columns V .. Npad - 1 of Z
// hold -inf (their bias is -inf), so the row needs no tail masks.
// The K best are found without sorting the row.  A lower bound tau of the K-th largest key comes first; only keys
// at or above it (a few dozen) are collected in LDS, and each of those finds its rank by counting the ones ahead of it.
// STATS (no LM term in the keys): the contraction has left (maximum, sum of exponentials) of every 32-column chunk.
// Thread c takes chunk c; in every wave the K-th largest of its 64 chunk maxima bounds the row's K-th largest key
// from below, so does the largest of the four; only chunks whose maximum reaches tau are read, eight lanes each.
// Otherwise the whole row is read, 32 values per lane, and the lane maxima play the part of the chunk maxima.
// Four waves per row rather than one: 32 instead of 128 registers of logits per lane, five waves per SIMD
// instead of 1.25, so that the arithmetic of one row overlaps with the loads of another.
template <bool TAIL, bool STATS>
__global__ __launch_bounds__(64 * kRowWaves) void k_row_select(RowSelectArgs a) {
  __shared__ uint64_t surv[kSurvivorCap];
  __shared__ int surv_n;
  __shared__ float s_max[kRowWaves], s_sum[kRowWaves], s_tau[kRowWaves];
  const int K = a.K, V = a.V;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (*reinterpret_cast<const volatile int *>(a.done)) return;
  const int m = blockIdx.x;
  if (a.finished[m / K]) return;
  const float *zrow = a.Z + (size_t)m * a.Npad;
  const float *lmrow = a.lm ? a.lm + (size_t)m * V : nullptr;
  float mx;
  if constexpr (STATS) {
    __shared__ int s_chunks[64 * kRowWaves];
    __shared__ int s_nq;
    const int n_stat = a.Npad >> 5;  // <= 256
    float cm = -INFINITY, cs = 0.f;
    if (tid < n_stat) {
      const uint64_t st = a.cstat[(size_t)m * n_stat + tid];
      cm = __uint_as_float((uint32_t)st);
      cs = __uint_as_float((uint32_t)(st >> 32));
    }
    if (tid == 0) {
      surv_n = 0;
      s_nq = 0;
    }
    {
      const float wm = wave_max(cm);
      if (lane == 0) s_max[wave] = wm;
    }
    float tau = -INFINITY, cur = cm;
    for (int j = 0; j < K; ++j) {
      tau = wave_max(cur);
      if (cur == tau) cur = -INFINITY;
    }
    if (lane == 0) s_tau[wave] = tau;
    __syncthreads();
    mx = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
    float sum = cm > -INFINITY ? cs * exp2f((cm - mx) * 1.4426950408889634f) : 0.f;
    sum = wave_sum(sum);
    if (lane == 0) s_sum[wave] = sum;
    tau = fmaxf(fmaxf(s_tau[0], s_tau[1]), fmaxf(s_tau[2], s_tau[3]));
    if (cm >= tau && cm > -INFINITY) s_chunks[atomicAdd(&s_nq, 1)] = tid;
    __syncthreads();
    const int nq = s_nq;
    for (int i = tid >> 3; i < nq; i += 8 * kRowWaves) {
      const int n = 32 * s_chunks[i] + 4 * (tid & 7);
      const floatx4 z = *reinterpret_cast<const floatx4 *>(zrow + n);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (z[e] >= tau && z[e] > -INFINITY) {
          const int pos = atomicAdd(&surv_n, 1);
          if (pos < kSurvivorCap) surv[pos] = pack_cand(z[e], n + e);
        }
    }
  } else {
  // thread tid holds columns 4 (tid + 256 q) .. + 3
  floatx4 z[kRowRegs];
#pragma unroll
  for (int q = 0; q < kRowRegs; ++q) {
    z[q] = floatx4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (1024 * q + 4 * tid < a.Npad) z[q] = *reinterpret_cast<const floatx4 *>(zrow + 4 * (tid + 256 * q));
  }
  if (tid == 0) surv_n = 0;
  // soft-max statistics of the logits: block maximum, then the sum of exponentials against it
  float km = -INFINITY;
#pragma unroll
  for (int q = 0; q < kRowRegs; ++q) km = fmaxf(km, fmaxf(fmaxf(z[q][0], z[q][1]), fmaxf(z[q][2], z[q][3])));
  {
    const float wm = wave_max(km);
    if (lane == 0) s_max[wave] = wm;
  }
  __syncthreads();
  mx = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  float sum = 0.f;
  {
    const float kLog2e = 1.4426950408889634f, off = -mx * kLog2e;
#pragma unroll
    for (int q = 0; q < kRowRegs; ++q)
      sum += (exp2f(fmaf(z[q][0], kLog2e, off)) + exp2f(fmaf(z[q][1], kLog2e, off))) +
             (exp2f(fmaf(z[q][2], kLog2e, off)) + exp2f(fmaf(z[q][3], kLog2e, off)));
  }
  sum = wave_sum(sum);
  // keys = logit + lambda * LM score
  if (lmrow) {
    km = -INFINITY;
#pragma unroll
    for (int q = 0; q < kRowRegs; ++q) {
      const int n = 4 * (tid + 256 * q);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (n + e < V) z[q][e] += a.lambda * lmrow[n + e];
      km = fmaxf(km, fmaxf(fmaxf(z[q][0], z[q][1]), fmaxf(z[q][2], z[q][3])));
    }
  }
  // this wave's lower bound of the row's K-th largest key: K rounds of "largest remaining lane maximum"
  float tau = -INFINITY, cur = km;
  for (int j = 0; j < K; ++j) {
    tau = wave_max(cur);
    if (cur == tau) cur = -INFINITY;
  }
  if (lane == 0) {
    s_sum[wave] = sum;
    s_tau[wave] = tau;
  }
  __syncthreads();
  tau = fmaxf(fmaxf(s_tau[0], s_tau[1]), fmaxf(s_tau[2], s_tau[3]));
  // keys at or above tau (never -inf) are appended to the row's list
#pragma unroll
  for (int q = 0; q < kRowRegs; ++q) {
    const float m4 = fmaxf(fmaxf(z[q][0], z[q][1]), fmaxf(z[q][2], z[q][3]));
    if (m4 >= tau && m4 > -INFINITY) {
      const int n = 4 * (tid + 256 * q);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (z[q][e] >= tau && z[q][e] > -INFINITY) {
          const int pos = atomicAdd(&surv_n, 1);
          if (pos < kSurvivorCap) surv[pos] = pack_cand(z[q][e], n + e);
        }
    }
  }
  }  // !STATS
  __syncthreads();
  const int total = surv_n;
  uint64_t *out = a.p_cand + (size_t)m * K;
  if (total <= kSurvivorCap) {
    // rank of every collected key = number of collected keys ahead of it (packed keys are distinct)
    if (tid < K && tid >= total) store_through(out + tid, no_cand());
    for (int i = tid; i < total; i += 64 * kRowWaves) {
      const uint64_t mine = surv[i];
      int rank = 0;
      for (int j = 0; j < total; ++j) rank += surv[j] > mine;
      if (rank < K) store_through(out + rank, mine);
    }
  } else if (wave == 0) {
    // more than kSurvivorCap keys at or above tau (many equal keys): K plain rounds over the row in memory
    uint64_t last = ~0ull;
    for (int j = 0; j < K; ++j) {
      uint64_t best = no_cand();
      for (int n = lane; n < V; n += 64) {
        float key = zrow[n];
        if (lmrow) key += a.lambda * lmrow[n];
        const uint64_t c = key > -INFINITY ? pack_cand(key, n) : no_cand();
        if (c < last && c > best) best = c;
      }
      best = wave_max_u64(best);
      if (lane == 0) store_through(out + j, best);
      last = best > no_cand() ? best : no_cand() + 1;
    }
  }
  if (tid == 0) {
    store_through(a.p_max + m, mx);
    store_through(a.p_sum + m, (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]));
  }
  // blank and duration logits from the bf16 activations: z[V + d] = Wspec[d] . a_m + bias; wave 3, a lane takes 8 k
  if (wave == kRowWaves - 1) {
    const int nz = 1 + a.ND;
    float acc[9];
#pragma unroll
    for (int d = 0; d < 9; ++d) acc[d] = 0.f;
    for (int g = lane; g < (a.H >> 3); g += 64) {
      const uint4 u = *reinterpret_cast<const uint4 *>(a.Ab + ((size_t)g * a.Mp + m) * 8);
      const uint32_t w[4] = {u.x, u.y, u.z, u.w};
      float x[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(w[i] << 16);
        x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
#pragma unroll
      for (int d = 0; d < 9; ++d)
        if (d < nz) {
          const float4 p = *reinterpret_cast<const float4 *>(a.Wspec + (size_t)d * a.H + 8 * g);
          const float4 q = *reinterpret_cast<const float4 *>(a.Wspec + (size_t)d * a.H + 8 * g + 4);
          acc[d] += (x[0] * p.x + x[1] * p.y) + (x[2] * p.z + x[3] * p.w) + (x[4] * q.x + x[5] * q.y) +
                    (x[6] * q.z + x[7] * q.w);
        }
    }
#pragma unroll
    for (int d = 0; d < 9; ++d)
      if (d < nz) {
        const float v = wave_sum(acc[d]);
        if (lane == 0) store_through(a.zs + (size_t)m * nz + d, v + a.bias_spec[d]);
      }
  }
  if constexpr (TAIL) {
    // Every thread waits until its write-through stores (list, statistics, blank / duration logits) have been
    // acknowledged, then the barrier, then one thread counts the row in: the count cannot become visible before
    // anything of the row.  The block that brings the utterance's count to K owns the rest of its step.
    __shared__ int s_is_last;
    __shared__ SelectScratchWide scratch;
    const int b = m / K;
    wait_stores_acknowledged();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) {
      const int old = __hip_atomic_fetch_add(a.utt_ctr + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int last = old == K - 1;
      if (last) store_agent(a.utt_ctr + b, 0);  // every other row of the utterance has been counted
      s_is_last = last;
    }
    __syncthreads();
    if (!s_is_last) return;
    if (wave == 0) select_dispatch<4, SelectScratchWide>(a.sel, b, scratch);  // (reads the lists with device-coherent loads)
    __syncthreads();
    // activations of the utterance's new hypotheses, from the selection's scratch (frame, token history)
    const int T_b = a.pre.lengths[b];
    const int H8 = a.pre.H >> 3;
    // (two items per thread and round, so that the loads of both are in flight together)
    for (int it = tid; it < K * H8; it += 2 * 64 * kRowWaves) {
      const int it2 = it + 64 * kRowWaves;
      const bool two = it2 < K * H8;
      const int j = it / H8, o8 = it % H8, j2 = two ? it2 / H8 : j, o82 = two ? it2 % H8 : o8;
      int tt = scratch.n_t[j], tt2 = scratch.n_t[j2];
      tt = tt < T_b ? tt : T_b - 1;
      tt = tt < 0 ? 0 : tt;
      tt2 = tt2 < T_b ? tt2 : T_b - 1;
      tt2 = tt2 < 0 ? 0 : tt2;
      stateless_pre_big_pair(a.pre, b * K + j, tt, scratch.ctx[j], o8, b * K + j2, tt2, scratch.ctx[j2], o82, b, two);
    }
  }
}

// The row scan, the selection and the next activations of ONE utterance in one block: wave w takes hypothesis w of
// the utterance (K <= 16 waves).  For keys without an LM term, from the chunk statistics of the contraction.  Nothing
// is handed from block to block: the K lists, the soft-max statistics and the blank / duration logits stay in LDS, a
// barrier replaces the write-through stores, their acknowledgement and the counter of the row-per-block form.
// A wave finds its row's K best keys like a block of the row-per-block form does (threshold from the chunk maxima,
// here the K-th largest of the lanes' maxima over four chunks each, which is a lower bound as well; keys at or above
// it collected and ranked by counting).
constexpr int kUttSurvivorCap = 128;

// FORMS: 4, or 12 / 16 for AES++ / ALSD++ on a plain RNN-T (see select_dispatch)
template <int FORMS>
__global__ __launch_bounds__(64 * kMaxBeam) void k_utt_select(RowSelectArgs a) {
  __shared__ SelectScratchWide scratch;
  __shared__ uint64_t l_cand[kMaxBeam * kMaxBeam];
  __shared__ float l_max[kMaxBeam], l_sum[kMaxBeam], l_zs[kMaxBeam * 9];
  __shared__ uint64_t surv[kMaxBeam][kUttSurvivorCap];
  __shared__ uint16_t qchunk[kMaxBeam][256];
  __shared__ int surv_n[kMaxBeam], q_n[kMaxBeam];
  const int K = a.K, V = a.V;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;  // wave < K
  if (*reinterpret_cast<const volatile int *>(a.done)) return;
  const int b = blockIdx.x;
  if (a.finished[b]) return;
  const int m = b * K + wave;
  const float *zrow = a.Z + (size_t)m * a.Npad;
  const int n_stat = a.Npad >> 5;  // <= 256: four chunks per lane
  const float kLog2e = 1.4426950408889634f;
  float cm[4], cs[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int c = lane + 64 * q;
    const uint64_t st = a.cstat[(size_t)m * n_stat + (c < n_stat ? c : 0)];
    cm[q] = c < n_stat ? __uint_as_float((uint32_t)st) : -INFINITY;
    cs[q] = c < n_stat ? __uint_as_float((uint32_t)(st >> 32)) : 0.f;
  }
  if (lane == 0) {
    surv_n[wave] = 0;
    q_n[wave] = 0;
  }
  const float lmx = fmaxf(fmaxf(cm[0], cm[1]), fmaxf(cm[2], cm[3]));
  const float mx = wave_max(lmx);
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q) sum += cm[q] > -INFINITY ? cs[q] * exp2f((cm[q] - mx) * kLog2e) : 0.f;
  sum = wave_sum(sum);
  float tau = -INFINITY, cur = lmx;
  for (int j = 0; j < K; ++j) {
    tau = wave_max(cur);
    if (cur == tau) cur = -INFINITY;
  }
  wave_sync();
#pragma unroll
  for (int q = 0; q < 4; ++q)
    if (cm[q] >= tau && cm[q] > -INFINITY) qchunk[wave][atomicAdd(&q_n[wave], 1)] = (uint16_t)(lane + 64 * q);
  wave_sync();
  const int nq = q_n[wave];
  for (int i = lane >> 3; i < nq; i += 8) {  // eight lanes read the 128 bytes of a chunk
    const int n = 32 * (int)qchunk[wave][i] + 4 * (lane & 7);
    const floatx4 z = *reinterpret_cast<const floatx4 *>(zrow + n);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (z[e] >= tau && z[e] > -INFINITY) {
        const int pos = atomicAdd(&surv_n[wave], 1);
        if (pos < kUttSurvivorCap) surv[wave][pos] = pack_cand(z[e], n + e);
      }
  }
  wave_sync();
  const int total = surv_n[wave];
  uint64_t *out = l_cand + wave * K;
  if (total <= kUttSurvivorCap) {
    if (lane < K && lane >= total) out[lane] = no_cand();
    for (int i = lane; i < total; i += 64) {
      const uint64_t mine = surv[wave][i];
      int rank = 0;
      for (int j = 0; j < total; ++j) rank += surv[wave][j] > mine;
      if (rank < K) out[rank] = mine;
    }
  } else {
    // more keys at or above tau than the list holds (many equal keys): K plain rounds over the row in memory
    uint64_t last = ~0ull;
    for (int j = 0; j < K; ++j) {
      uint64_t best = no_cand();
      for (int n = lane; n < V; n += 64) {
        const float key = zrow[n];
        const uint64_t c = key > -INFINITY ? pack_cand(key, n) : no_cand();
        if (c < last && c > best) best = c;
      }
      best = wave_max_u64(best);
      if (lane == 0) out[j] = best;
      last = best > no_cand() ? best : no_cand() + 1;
    }
  }
  if (lane == 0) {
    l_max[wave] = mx;
    l_sum[wave] = sum;
  }
  // blank and duration logits from the bf16 activations: z[V + d] = Wspec[d] . a_m + bias; a lane takes 8 k at a time
  {
    const int nz = (FORMS == 12 || FORMS == 16) ? 1 : 1 + a.ND;  // (the plain forms: no durations)
    float acc[9];
#pragma unroll
    for (int d = 0; d < 9; ++d) acc[d] = 0.f;
    for (int g = lane; g < (a.H >> 3); g += 64) {
      const uint4 u = *reinterpret_cast<const uint4 *>(a.Ab + ((size_t)g * a.Mp + m) * 8);
      const uint32_t w[4] = {u.x, u.y, u.z, u.w};
      float x[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(w[i] << 16);
        x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
      }
#pragma unroll
      for (int d = 0; d < 9; ++d)
        if (d < nz) {
          const float4 p = *reinterpret_cast<const float4 *>(a.Wspec + (size_t)d * a.H + 8 * g);
          const float4 q = *reinterpret_cast<const float4 *>(a.Wspec + (size_t)d * a.H + 8 * g + 4);
          acc[d] += (x[0] * p.x + x[1] * p.y) + (x[2] * p.z + x[3] * p.w) + (x[4] * q.x + x[5] * q.y) +
                    (x[6] * q.z + x[7] * q.w);
        }
    }
#pragma unroll
    for (int d = 0; d < 9; ++d)
      if (d < nz) {
        const float v = wave_sum(acc[d]);
        if (lane == 0) l_zs[wave * nz + d] = v + a.bias_spec[d];
      }
  }
  __syncthreads();
  if (wave == 0) select_dispatch<FORMS, SelectScratchWide>(a.sel, b, scratch, CandView{l_cand, l_max, l_sum, l_zs, b * K});
  __syncthreads();
  // activations of the utterance's new hypotheses, from the selection's scratch (frame, token history)
  const int T_b = a.pre.lengths[b];
  const int H8 = a.pre.H >> 3;
  const int nthr = 64 * K;
  // (two items per thread and round, so that the loads of both are in flight together)
  for (int it = tid; it < K * H8; it += 2 * nthr) {
    const int it2 = it + nthr;
    const bool two = it2 < K * H8;
    const int j = it / H8, o8 = it % H8, j2 = two ? it2 / H8 : j, o82 = two ? it2 % H8 : o8;
    int tt = scratch.n_t[j], tt2 = scratch.n_t[j2];
    tt = tt < T_b ? tt : T_b - 1;
    tt = tt < 0 ? 0 : tt;
    tt2 = tt2 < T_b ? tt2 : T_b - 1;
    tt2 = tt2 < 0 ? 0 : tt2;
    stateless_pre_big_pair(a.pre, b * K + j, tt, scratch.ctx[j], o8, b * K + j2, tt2, scratch.ctx[j2], o82, b, two);
  }
}

}  // namespace rb
