// The whole step loop of a decode in ONE launch, as the alternative to replaying a graph of per-step kernels
// (Sec. 2.1, "CUDA Graphs": the per-step launches and their boundaries are the cost being avoided).
//
// One block per compute unit.  The blocks that run on one XCD form a group that decodes its own share of the
// utterances from the first step to the last, independently of the other groups, so that a barrier spans 32 blocks
// instead of 256 and no group ever waits for another.  Hand-over between blocks is the device-scope protocol of the
// per-step kernels' tail: write-through stores, then a count; the waiting side polls the count with device-coherent
// loads and then invalidates its caches.  Every group streams all weights itself.  A step of a group:
//   C  cell update of the LSTM for the group's slots                                   | group barrier
//   D  prediction projection (H / 32 tiles), the other blocks start on  R' = W_hh h'   | counter: projection tiles done
//   A  joint network (n_chunks tiles, candidate lists), then the rest of R'            | counter: joint tiles done
//   B  selection / tree / recombination of the group's utterances by the group's first block, under the rest of R'
//                                                                                      | group barrier
// LSTM prediction network, beams up to 8, no LM; other decoders take the per-step launches.
// Every wait is bounded: a block that waits too long raises the abort word and returns, every other block sees the
// word at its next wait and returns too, and the host reports the error.
#pragma once
#include "kernels.h"

namespace rb {

constexpr int kXccs = 8;
constexpr int kSpinLimit = 1 << 22;  // polls of one wait (each a device-coherent load and a short sleep): seconds

// per group, one cache line each so that no two groups share one
struct alignas(256) GroupCtl {
  int arrive;      // barrier: blocks that have arrived, counted up for ever
  int pp_done;     // projection tiles finished, counted up for ever
  int joint_done;  // joint tiles finished, counted up for ever
  int stop;        // set by the selecting block when every utterance of the group has finished
};

struct PersistCtl {
  GroupCtl grp[kXccs];
  int xcc_count[kXccs];  // blocks that found themselves on each XCD
  int started;           // blocks that have registered
  int abort;             // != 0: a wait ran into its limit (1), or the blocks are not spread evenly over the XCDs (2)
};

struct PersistArgs {
  MainArgs main;      // joint + selection (sel.step_base must point at a word that stays 0)
  PredProjArgs pp;    // h / pre are set per step inside the kernel
  const float *G;     // [V + 1][4P] token part of the gates
  float *h[2], *c[2]; // state, double buffered (parity 1 holds the zero state at the start)
  float *R;           // [M][4P]
  PersistCtl *ctl;    // zeroed before the launch
  int B, max_steps;
  int spin_limit;     // kSpinLimit (a test may pass a tiny limit together with a grid that cannot be whole)
};

// index of the XCD this wave runs on (hardware register XCC_ID, bits 3:0)
__device__ __forceinline__ int xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | 20) & 7; }

// every thread: my stores have reached the L2
__device__ __forceinline__ void publish_stores() { wait_stores_acknowledged(); }
// every thread, after a wait: device-scope acquire.  What other blocks handed over was written through to the memory
// side (store_through / store_agent) before they counted in; this drops every line of the L1 and every clean line of
// the XCD's L2 that could be older.  (The workgroup-scope form, "buffer_inv sc0", and loads with only sc0 set were
// measured to be no-ops on the L1 in this mode: a poll with them never saw another compute unit's count.)
__device__ __forceinline__ void refresh_caches() { asm volatile("buffer_inv sc1" ::: "memory"); }

// thread 0 of the block polls `word` until it reaches `target` (or the abort word is raised, or the limit is hit);
// returns false to the whole block if the kernel must end.  Ends with the block in step and a fresh L1.
__device__ __forceinline__ bool block_wait(const int *word, int target, PersistCtl *ctl, int limit, int *s_flag) {
  if (threadIdx.x == 0) {
    int ok = 0;
    for (int i = 0; i < limit; ++i) {
      if (load_agent(word) - target >= 0) {
        ok = 1;
        break;
      }
      if (load_agent(&ctl->abort)) break;
      __builtin_amdgcn_s_sleep(2);
    }
    if (!ok && !load_agent(&ctl->abort)) store_agent(&ctl->abort, 1);
    *s_flag = ok;
  }
  __syncthreads();
  const int ok = *s_flag;
  __syncthreads();
  refresh_caches();
  return ok != 0;
}

// all blocks of a group: stores published, count in, wait for the n-th round of arrivals
__device__ __forceinline__ bool group_barrier(GroupCtl *g, int n_blocks, int round, PersistCtl *ctl, int limit, int *s_flag) {
  publish_stores();
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(&g->arrive, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return block_wait(&g->arrive, n_blocks * round, ctl, limit, s_flag);
}

// a finished tile: stores published, one count
__device__ __forceinline__ void tile_done(int *counter) {
  publish_stores();
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int WAVES, int ITERS>
__global__ __launch_bounds__(WAVES * 64, 1) void k_decode_persistent(PersistArgs a) {
  constexpr int kRedFloats = WAVES * 64 * kRedStride;
  constexpr int kScratchFloats = (int)((sizeof(SelectScratch) * WAVES + 3) / 4);
  // (more than half of a compute unit's LDS: two blocks can never share one)
  constexpr int kLdsFloats = 21 * 1024;
  static_assert(kLdsFloats >= kRedFloats && kLdsFloats >= kScratchFloats, "LDS");
  __shared__ __align__(16) float smem[kLdsFloats];
  __shared__ int s_flag;
  float *red = smem;
  const int tid = threadIdx.x, wave = tid >> 6;
  PersistCtl *ctl = a.ctl;
  const int limit = a.spin_limit;

  // ---- which XCD am I on, and which block of it
  __shared__ int s_rank;
  const int g = xcc_id();
  if (tid == 0) {
    s_rank = __hip_atomic_fetch_add(&ctl->xcc_count[g], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_fetch_add(&ctl->started, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  const int rank = s_rank;
  if (!block_wait(&ctl->started, (int)gridDim.x, ctl, limit, &s_flag)) return;  // every block is resident and registered
  const int n_blocks = (int)gridDim.x / kXccs;
  for (int x = 0; x < kXccs; ++x)
    if (load_agent(&ctl->xcc_count[x]) != n_blocks) {  // (every block sees the same counts: all return)
      if (tid == 0 && blockIdx.x == 0) store_agent(&ctl->abort, 2);
      return;
    }
  GroupCtl *grp = &ctl->grp[g];

  // ---- the group's utterances and slots
  const int K = a.main.K;
  const int per = (a.B + kXccs - 1) / kXccs;
  const int b0 = g * per, nb = min(per, a.B - b0);
  if (nb <= 0) return;  // (groups are independent: a group without utterances has nothing to wait for)
  const int m0 = b0 * K, rows = nb * K;  // rows <= 32: one tile of slots
  const int P = a.pp.P, n_pp = a.pp.H / 32, n_rec = 4 * P / 32, n_chunks = a.main.n_chunks;
  // recurrent tiles by block: the blocks without a projection tile take one each during D; the rest go round the
  // blocks 1 .. n_blocks - 1 (block 0 selects) after their joint tiles
  const int rec_early = rank >= n_pp ? rank - n_pp : -1;
  const int n_early = max(n_blocks - n_pp, 0);

  // (the tile routines write every slot below their M: the group's slots end at m0 + rows, the next group's follow)
  SelectArgs sel = a.main.sel;
  RecurrentArgs rec = a.main.rec;
  rec.M = m0 + rows;
  PredProjArgs pp = a.pp;
  pp.M = m0 + rows;
  int cur = 1, bar = 0;
  for (int step = 0; step < a.max_steps; ++step) {
    // ---- C: cell update, state parity cur -> cur ^ 1
    for (int i = rank * (WAVES * 64) + tid; i < rows * P; i += n_blocks * WAVES * 64) {
      const int m = m0 + i / P, u = i % P;
      lstm_cell(a.R, a.G, a.h[cur], a.c[cur], a.h[cur ^ 1], a.c[cur ^ 1], load_agent(sel.src_row + m),
                load_agent(sel.tok + m), m, u, a.main.Mp, P, 0);
    }
    if (!group_barrier(grp, n_blocks, ++bar, ctl, limit, &s_flag)) return;
    cur ^= 1;
    // ---- D: projection tiles; blocks without one start on R' = W_hh h'
    pp.h = a.h[cur];
    rec.h = a.h[cur];
    if (rank < n_pp) {
      for (int tile = rank; tile < n_pp; tile += n_blocks) {
        pred_proj_tile<WAVES, ITERS>(pp, tile, m0, 0, red);
        tile_done(&grp->pp_done);
      }
    } else if (rec_early < n_rec) {
      recurrent_tile<WAVES, ITERS>(rec, rec_early, m0, 0, red);
      __syncthreads();
    }
    // ---- A: joint tiles need every projection tile
    if (!block_wait(&grp->pp_done, n_pp * (step + 1), ctl, limit, &s_flag)) return;
    for (int chunk = rank; chunk < n_chunks; chunk += n_blocks) {
      // (block 0 selects: it takes one tile only, its further ones go to block 1)
      if (rank == 0 && chunk > 0) break;
      joint_tile<WAVES, ITERS>(a.main, chunk, m0, rows, 0, red);
      tile_done(&grp->joint_done);
    }
    if (rank == 1)
      for (int chunk = n_blocks; chunk < n_chunks; chunk += n_blocks) {  // block 0's further tiles
        joint_tile<WAVES, ITERS>(a.main, chunk, m0, rows, 0, red);
        tile_done(&grp->joint_done);
      }
    if (rank == 0) {
      // ---- B: selection, one wave per utterance
      if (!block_wait(&grp->joint_done, n_chunks * (step + 1), ctl, limit, &s_flag)) return;
      SelectScratch *scratch = reinterpret_cast<SelectScratch *>(smem);
      sel.step_off = step;
      for (int u = wave; u < nb; u += WAVES) select_dispatch<0>(sel, b0 + u, scratch[wave]);
      __syncthreads();
      if (tid == 0) {
        int open = 0;
        for (int u = 0; u < nb; ++u) open += load_agent(sel.finished + b0 + u) == 0;
        if (!open) store_agent(&grp->stop, 1);
      }
    } else {
      // the rest of R': tiles n_early .. n_rec - 1 go round the blocks 1 .. n_blocks - 1
      for (int tile = n_early + rank - 1; tile < n_rec; tile += n_blocks - 1) {
        recurrent_tile<WAVES, ITERS>(rec, tile, m0, 0, red);
        __syncthreads();
      }
    }
    if (!group_barrier(grp, n_blocks, ++bar, ctl, limit, &s_flag)) return;
    if (load_agent(&grp->stop)) break;
  }
}

}  // namespace rb
