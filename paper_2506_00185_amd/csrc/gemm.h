// C[M, N] = A[M, K] B[N, K]^T + bias[N]: the encoder projection of the joint network (f = W_enc enc + b_enc, once
// per decode call; Methods, "Joint network") and the table folding at create.  Row-major float32 in and out.
//
// 256 threads = 2 x 2 waves; a wave owns (32 WM) x (32 WN) of the block's (64 WM) x (64 WN) tile.  Both operands
// are staged through LDS in k-chunks of 32, double buffered with one barrier per chunk (the next two chunks are in
// flight in registers while the current one is multiplied), so every element fetched from L2 feeds 64 WN (resp.
// 64 WM) multiply-adds instead of 32 as with per-wave operand loads.
// BF16 = false: float32 matrix instructions (32x32x2).  BF16 = true: both operands are rounded to bfloat16 (nearest
// even) on their way into LDS and multiplied with the bf16 matrix instructions (32x32x16), float32 accumulation.
// DEEP: two register sets, chunks requested two ahead (hides the load latency of the small tiles, whose chunks hold
// few matrix instructions); otherwise one set, one chunk ahead.
// Block -> tile: all N-tiles of one M-tile run on one XCD (block i runs on XCD i % 8), back to back, so a tile of A
// is fetched into one L2 only; B (the weights) is small and is fetched once per XCD.
#pragma once
#include "device_utils.h"

namespace rb {

constexpr int kGemmChunk = 32;  // k per LDS stage

template <bool BF16, int WM, int WN>
struct GemmTile {
  static constexpr int BM = 64 * WM, BN = 64 * WN;
  // row stride in bytes: 32 floats + 16 B, or 32 bf16 + 16 B (16-byte reads of 16 consecutive rows hit distinct banks)
  static constexpr int kStride = BF16 ? 80 : 144;
  static constexpr int kLdsBytes = 2 * (BM + BN) * kStride;
};

struct GemmArgs {
  const float *A, *B, *bias;
  float *C;
  int M, N, K;
  int n_mt, n_nt;  // tiles along M and N
  int *nonfinite;  // nullable: set to 1 when an output is NaN or Inf
  // nullable: the rows are B utterances of T frames each and lengths[b] of them are in use (values outside 0..T are
  // clamped here as the decode clamps them); a tile all of whose rows lie behind their utterance's last frame is
  // left out (frame 0 of every utterance is always computed).  C keeps whatever it held in those rows.
  const int *lengths;
  int T;
};

__host__ inline int gemm_grid(int n_mt, int n_nt) { return 8 * ((n_mt + 7) / 8) * n_nt; }

template <bool BF16, int WM, int WN, bool DEEP>
__global__ __launch_bounds__(256) void k_gemm_tiled(GemmArgs a) {
  typedef GemmTile<BF16, WM, WN> T;
  constexpr int BM = T::BM, BN = T::BN, ST = T::kStride;
  constexpr int LA = BM / 32, LB = BN / 32;  // 16-byte global loads per thread and chunk
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, col = lane & 31;
  const int x = blockIdx.x & 7, s = blockIdx.x >> 3;
  const int mt = (s / a.n_nt) * 8 + x, nt = s % a.n_nt;
  if (mt >= a.n_mt) return;
  const int m0 = mt * BM, n0 = nt * BN;
  if (a.lengths) {  // (uniform over the block)
    const int last = min(m0 + BM, a.M) - 1;
    bool needed = false;
    for (int b = m0 / a.T; b <= last / a.T; ++b) {
      const int first_t = max(m0 - b * a.T, 0);  // the utterance's first frame inside the tile
      const int len = min(max(a.lengths[b], 1), a.T);
      needed |= first_t < len;
    }
    if (!needed) return;
  }
  const int wm0 = (wave >> 1) * 32 * WM, wn0 = (wave & 1) * 32 * WN;
  // staging: thread -> (row tid / 8 + 32 i, floats 4 (tid % 8) .. + 3) of the chunk
  const int srow = tid >> 3, sc4 = tid & 7;
  const float *ga[LA], *gb[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) ga[i] = a.A + (size_t)min(m0 + srow + 32 * i, a.M - 1) * a.K + 4 * sc4;
#pragma unroll
  for (int i = 0; i < LB; ++i) gb[i] = a.B + (size_t)min(n0 + srow + 32 * i, a.N - 1) * a.K + 4 * sc4;
  // two register sets: chunk c + 2 is requested while chunk c is multiplied, so a load has two chunks' worth of
  // matrix instructions (and the other blocks of the compute unit) to hide behind
  // (vector-typed registers and array references: a struct type or a decayed pointer here sends the sets to scratch)
  floatx4 ra0[LA], rb0[LB], ra1[LA], rb1[LB];
  auto fetch = [&](floatx4(&ra)[LA], floatx4(&rb_)[LB], int k0) {
#pragma unroll
    for (int i = 0; i < LA; ++i) ra[i] = *reinterpret_cast<const floatx4 *>(ga[i] + k0);
#pragma unroll
    for (int i = 0; i < LB; ++i) rb_[i] = *reinterpret_cast<const floatx4 *>(gb[i] + k0);
  };
  auto stash = [&](const floatx4(&ra)[LA], const floatx4(&rb_)[LB], int buf) {
    unsigned char *As = lds + buf * (BM + BN) * ST, *Bs = As + BM * ST;
    if constexpr (BF16) {
#pragma unroll
      for (int i = 0; i < LA; ++i)
        *reinterpret_cast<uintx2_t *>(As + (srow + 32 * i) * ST + 8 * sc4) =
            uintx2_t{pack_bf16_rne(ra[i][0], ra[i][1]), pack_bf16_rne(ra[i][2], ra[i][3])};
#pragma unroll
      for (int i = 0; i < LB; ++i)
        *reinterpret_cast<uintx2_t *>(Bs + (srow + 32 * i) * ST + 8 * sc4) =
            uintx2_t{pack_bf16_rne(rb_[i][0], rb_[i][1]), pack_bf16_rne(rb_[i][2], rb_[i][3])};
    } else {
#pragma unroll
      for (int i = 0; i < LA; ++i) *reinterpret_cast<floatx4 *>(As + (srow + 32 * i) * ST + 16 * sc4) = ra[i];
#pragma unroll
      for (int i = 0; i < LB; ++i) *reinterpret_cast<floatx4 *>(Bs + (srow + 32 * i) * ST + 16 * sc4) = rb_[i];
    }
  };
  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j) acc[i][j] = floatx16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  auto multiply = [&](int buf) {
    const unsigned char *As = lds + buf * (BM + BN) * ST, *Bs = As + BM * ST;
    if constexpr (BF16) {
      // a matrix instruction covers 16 k: the lane supplies 8 consecutive k of its row (half 0: k 0..7, half 1: 8..15)
#pragma unroll
      for (int kk = 0; kk < kGemmChunk / 16; ++kk) {
        uintx4_t fa[WM], fb[WN];
#pragma unroll
        for (int i = 0; i < WM; ++i)
          fa[i] = *reinterpret_cast<const uintx4_t *>(As + (wm0 + 32 * i + col) * ST + 32 * kk + 16 * half);
#pragma unroll
        for (int j = 0; j < WN; ++j)
          fb[j] = *reinterpret_cast<const uintx4_t *>(Bs + (wn0 + 32 * j + col) * ST + 32 * kk + 16 * half);
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int j = 0; j < WN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[i]),
                                                                __builtin_bit_cast(bf16x8_t, fb[j]), acc[i][j], 0, 0, 0);
      }
    } else {
      // 8 k per round: the lane holds 4 consecutive k of its half; instruction q multiplies k = 4 half + q of both
#pragma unroll
      for (int kk = 0; kk < kGemmChunk / 8; ++kk) {
        floatx4 fa[WM], fb[WN];
#pragma unroll
        for (int i = 0; i < WM; ++i)
          fa[i] = *reinterpret_cast<const floatx4 *>(As + (wm0 + 32 * i + col) * ST + 32 * kk + 16 * half);
#pragma unroll
        for (int j = 0; j < WN; ++j)
          fb[j] = *reinterpret_cast<const floatx4 *>(Bs + (wn0 + 32 * j + col) * ST + 32 * kk + 16 * half);
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int j = 0; j < WN; ++j) {
            acc[i][j] = mfma32(fa[i][0], fb[j][0], acc[i][j]);
            acc[i][j] = mfma32(fa[i][1], fb[j][1], acc[i][j]);
            acc[i][j] = mfma32(fa[i][2], fb[j][2], acc[i][j]);
            acc[i][j] = mfma32(fa[i][3], fb[j][3], acc[i][j]);
          }
      }
    }
  };
  const int n_chunks = a.K / kGemmChunk;
  if constexpr (!DEEP) {
    // one register set, one chunk ahead: for the large tiles, whose accumulators leave no room for a second set
    fetch(ra0, rb0, 0);
    stash(ra0, rb0, 0);
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
      if (c + 1 < n_chunks) fetch(ra0, rb0, (c + 1) * kGemmChunk);
      multiply(c & 1);
      if (c + 1 < n_chunks) stash(ra0, rb0, (c + 1) & 1);
      __syncthreads();
    }
  } else {
  fetch(ra0, rb0, 0);
  if (n_chunks > 1) fetch(ra1, rb1, kGemmChunk);
  stash(ra0, rb0, 0);
  __syncthreads();
  // chunk c sits in LDS buffer c % 2 and came through register set c % 2; the buffer written in an iteration was
  // last read two barriers earlier
  for (int c = 0; c < n_chunks; c += 2) {
    if (c + 2 < n_chunks) fetch(ra0, rb0, (c + 2) * kGemmChunk);
    multiply(0);
    if (c + 1 < n_chunks) stash(ra1, rb1, 1);
    __syncthreads();
    if (c + 1 >= n_chunks) break;
    if (c + 3 < n_chunks) fetch(ra1, rb1, (c + 3) * kGemmChunk);
    multiply(1);
    if (c + 2 < n_chunks) stash(ra0, rb0, 0);
    __syncthreads();
  }
  }  // DEEP
  // register r of a tile is row 8 (r / 4) + 4 half + r % 4, column = lane % 32: 32 lanes store 128 contiguous bytes
  bool bad = false;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int n = n0 + wn0 + 32 * j + col;
    if (n >= a.N) continue;
    const float bv = a.bias ? a.bias[n] : 0.f;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
        if (m < a.M) {
          const float v = acc[i][j][r] + bv;
          a.C[(size_t)m * a.N + n] = v;
          bad |= !isfinite(v);
        }
      }
  }
  if (a.nonfinite && bad) *a.nonfinite = 1;
}

}  // namespace rb
