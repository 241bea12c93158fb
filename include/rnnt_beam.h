/*
 * rnnt_beam: batched beam search (ALSD++ / AES++) for RNN-T and TDT Transducers
 * on one AMD MI355X (gfx950).  C ABI; every step of the decoding path runs in
 * HIP kernels inside the library.
 *
 * Problem statement (paper, Methods and Sec. 2.1-2.3): given the encoder output
 * of a batch of audio streams and a Transducer (prediction network + joint
 * network), optionally an n-gram LM over the same vocabulary with weight
 * lambda, keep exactly `beam` hypotheses per stream, expand / merge / prune them
 * step by step, and return the `beam` best transcripts per stream.
 *
 * Conventions
 *   - Return value 0 = success, negative = error (see RNNT_E_*).  No exception or
 *     abort crosses this boundary; rnnt_beam_last_error() gives a message.
 *   - "device" pointers are HIP device memory on the current device, "host"
 *     pointers ordinary host memory.  All matrices are row-major float32.
 *   - Token ids are 0..V-1, blank is V.  TDT duration logits follow the blank.
 *   - The caller owns every array it passes in.  Weights and LM arrays are
 *     re-packed into library-owned device memory by the create calls and may be
 *     freed afterwards.  The handle owns workspace, hypothesis tree and graphs.
 *   - Shape limits: H, P, D and E must be multiples of 32; beam <= 16 (8 with tdt_all_pairs); an LM's vocabulary
 *     at most 15 360 tokens (one row of scores is built in 60 KB of on-chip memory).  Kernels specialised for
 *     H = P = 640 exist beside generic ones for any multiple of 32; the prediction projection is split in two
 *     along k across blocks only when P % 128 == 0.
 *
 * Where the signatures differ from the minimal statement of the problem
 * (create / decode(enc, lengths, weights, beam, algo, lm, lm_weight) / results), and why:
 *   - rnnt_lm_create takes V: the LM's vocabulary is checked against the model's at decode time and sizes the
 *     on-chip row; the n-gram arrays alone do not fix it (unseen tokens).
 *   - rnnt_beam_results returns scores as double: hypothesis scores are accumulated in float64 on the device
 *     (a sum of several hundred float32 log-probabilities), and the n-best order is defined on those values.
 *   - rnnt_beam_dump_tree takes s_cap, the number of tree levels the caller's arrays have room for.
 *   - rnnt_beam_decode by default follows the device (it returns when the data-dependent number of steps is
 *     over); with the config field async_enqueue it only enqueues and returns (see there).
 *   - config fields beyond the model's shape select readings the paper leaves open or variants it describes:
 *     use_graph, joint_path, lm_rule, lm_early_pruning, tdt_all_pairs, async_enqueue, aes_prefix_search,
 *     persistent_kernel.
 */
#ifndef RNNT_BEAM_H
#define RNNT_BEAM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rnnt_beam rnnt_beam_t; /* opaque decoder handle */
typedef struct rnnt_lm rnnt_lm_t;     /* opaque n-gram LM */

typedef enum { RNNT_ALSD = 0, RNNT_AES = 1 } rnnt_algo_t;
typedef enum { RNNT_MODEL_RNNT = 0, RNNT_MODEL_TDT = 1 } rnnt_model_t;
typedef enum { RNNT_PRED_LSTM = 0, RNNT_PRED_STATELESS = 1 } rnnt_pred_t;
typedef enum { RNNT_F32 = 0, RNNT_BF16_JOINT = 1 } rnnt_prec_t;
/* How a step computes the joint's output layer.  FUSED keeps the [B * beam, V + 1] logits on chip
 * (per-chunk top-K in the contraction's epilogue); MATERIALIZED writes them to HBM from a bf16
 * matrix-core contraction and selects row by row, which pays off for large (B * beam) x V.
 * MATERIALIZED needs RNNT_BF16_JOINT, the stateless prediction network, V <= 8192 and H % 16 == 0;
 * AUTO takes it for such decoders when B * beam >= 128 and V >= 2048. */
typedef enum { RNNT_JOINT_AUTO = 0, RNNT_JOINT_FUSED = 1, RNNT_JOINT_MATERIALIZED = 2 } rnnt_joint_path_t;

enum {
  RNNT_OK = 0,
  RNNT_E_ARG = -1,       /* bad argument, or a shape beyond max_B / max_T / max_beam */
  RNNT_E_NOMEM = -2,     /* device or host allocation failed */
  RNNT_E_HIP = -3,       /* a HIP call failed */
  RNNT_E_NONFINITE = -4, /* NaN or Inf found in the encoder projection of the last decode (frames in use; those
                            behind an utterance's length are looked at only where a tile of the product holds
                            frames in use as well) */
  RNNT_E_NORESULT = -5   /* results requested before any decode */
};

/* Plain data, versioned by struct_size (= sizeof(rnnt_config_t)). */
typedef struct {
  uint32_t struct_size;
  int32_t model;             /* rnnt_model_t */
  int32_t pred;              /* rnnt_pred_t */
  int32_t prec;              /* rnnt_prec_t: RNNT_BF16_JOINT rounds the operands of the three
                                joint-network products (W_enc, W_pred, W_out and their inputs)
                                to bfloat16; sums, soft-max and the LSTM stay float32 */
  int32_t D, H, P, E, V;     /* encoder dim, joint hidden, prediction hidden, embedding dim, tokens */
  int32_t n_durations;       /* TDT: number of duration classes (<= 8), else 0 */
  int32_t durations[8];      /* TDT: frames advanced by each class, e.g. {0,1,2,3,4}; each in 0..255, one >= 1 */
  int32_t stateless_context; /* stateless prediction network: tokens of context (<= 4) */
  int32_t max_B, max_T, max_beam; /* workspace sizing */
  int32_t max_symbols;       /* s: most tokens a hypothesis may emit without leaving a frame
                                (Sec. 2.2, "a maximum of s expansions per frame") */
  float prune_margin;        /* AES++ only: a token whose log-probability is more than this below
                                the best one of its hypothesis is not expanded; INFINITY = off */
  int32_t use_graph;         /* 1: replay the per-step kernels as a captured HIP graph (Sec. 2.1,
                                "CUDA Graphs"); 0: launch them one by one */
  int32_t joint_path;        /* rnnt_joint_path_t; create fails if MATERIALIZED is asked for a decoder
                                that cannot take it */
  int32_t lm_rule;           /* how the LM enters a candidate's score (Sec. 2.3): 0 or 4 = Eq. (4), tokens get
                                lambda ln((1 - p_blank) p_LM), blank (1 + lambda) ln p_blank; 3 = Eq. (3), tokens
                                get lambda ln p_LM, blank is left as it is */
  int32_t lm_early_pruning;  /* 0 = late pruning: the Beam best are chosen on the fused scores; 1 = early pruning:
                                they are chosen on the Transducer's scores, the chosen ones then get the LM term
                                (Sec. 2.3, "Early/late pruning") */
  int32_t tdt_all_pairs;     /* TDT only.  0: a candidate is a symbol with ONE duration, the most likely one (for blank
                                the most likely one that advances).  1: every (symbol, duration) pair is a candidate
                                of its own, blank only with durations >= 1: Beam x (V + 1) x n_durations candidates
                                per utterance and step.  Needs max_beam <= 8 */
  int32_t async_enqueue;     /* 0: rnnt_beam_decode enqueues chunks of 16 steps, one chunk ahead of the device, and
                                returns once the device has reported that every utterance has finished (the calling
                                thread is blocked for most of the decode).  1: it enqueues the upper bound of
                                T (max_symbols + 1) steps at once and returns without waiting; steps after the last
                                utterance has finished return at once on the device (a few microseconds each) */
  int32_t aes_prefix_search; /* RNNT_AES only: maximum-length prefix search (Sec. 2.2, "AES": probabilities of hypotheses
                                with shared prefixes are combined; only the longest proper prefix is looked at).  When
                                two hypotheses expanded in the same frame hold y and y + v, and the expansion of y by v
                                is one of y's `beam` best tokens and stays in the frame, the candidates of y + v are
                                RANKED as if its score also held that expansion's score.  The scores themselves are
                                unchanged: the expansion competes as a candidate of its own and is merged with y + v by
                                the recombination, so no alignment is counted twice.  Not with tdt_all_pairs or
                                lm_early_pruning */
  int32_t persistent_kernel; /* 1: where it applies, the whole step loop runs as ONE launch instead of a replayed graph of
                                per-step launches (Sec. 2.1, "CUDA Graphs", is what it replaces): one block per compute
                                unit, the blocks of each XCD decode their own share of the utterances and synchronise
                                among themselves.  Applies to LSTM decoders without an LM at beams up to 8 with at most
                                32 hypotheses per XCD (ceil(B / 8) * beam <= 32) and H, P multiples of 64; other
                                decodes use the per-step launches.  The GPU must be otherwise idle: every block has to be
                                resident.  All waits between blocks are bounded; rnnt_beam_results returns RNNT_E_HIP if
                                one ran into its limit or the blocks were not spread evenly over the XCDs */
} rnnt_config_t;

/* Device pointers, float32, caller-owned.  Unused ones may be NULL. */
typedef struct {
  const float *W_enc;  /* [H, D]   encoder projection of the joint */
  const float *b_enc;  /* [H] */
  const float *W_pred; /* [H, P]   prediction projection of the joint */
  const float *b_pred; /* [H] */
  const float *W_out;  /* [V+1+n_durations, H] output layer of the joint */
  const float *b_out;  /* [V+1+n_durations] */
  const float *emb;    /* LSTM: [V+1, E] (row V = start symbol); stateless: [ctx, V+1, P] */
  const float *W_ih;   /* [4P, E]  LSTM, gate order (i, f, g, o) */
  const float *W_hh;   /* [4P, P] */
  const float *b_ih;   /* [4P] */
  const float *b_hh;   /* [4P] */
} rnnt_weights_t;

/*
 * Create a decoder.  Joint network: z = W_out ReLU(W_enc enc_t + b_enc + W_pred h + b_pred) + b_out,
 * token log-probabilities = log-softmax of z[0..V], TDT durations = log-softmax of the rest.
 * Prediction network: one LSTM layer fed with emb[last token], or the sum of
 * position-specific embeddings of the last `stateless_context` tokens.
 * Weights are re-packed (and folded where possible) on the device.
 */
int rnnt_beam_create(const rnnt_config_t *cfg, const rnnt_weights_t *weights, rnnt_beam_t **out);

/*
 * Build an n-gram LM (ARPA semantics, Sec. 2.3 "Language model fusion") from host arrays:
 * n n-grams, ngram_tokens [n, order] padded with -1 on the right, ngram_order [n] in 1..order,
 * log10 probability and log10 back-off weight of each.  Every unigram must be present.
 * Score of token v after a transcript: p(ctx v) if stored, else backoff(ctx) + score with the
 * oldest context token dropped; ctx = the last order-1 tokens.  The table is stored on the
 * device as a hash of contexts with successor lists: 128 to 256 bytes per distinct context
 * (32-byte slots, the table at most a quarter full), 8 bytes per n-gram of order 2 and up,
 * 4 V bytes of unigrams; allocated here, freed by rnnt_lm_destroy.
 */
int rnnt_lm_create(int32_t order, int64_t n, const int32_t *ngram_tokens, const int8_t *ngram_order,
                   const float *log10_prob, const float *log10_backoff, int32_t V, rnnt_lm_t **out);

/*
 * Decode a batch (Sec. 2.1-2.3).  enc: device [B, T, D]; lengths: device [B] frames per utterance
 * (values outside 0..T are clamped and reported as RNNT_E_ARG by rnnt_beam_results).
 * algo: RNNT_ALSD (length-synchronous, every unfinished hypothesis is expanded at every step) or
 * RNNT_AES (frame-synchronous, hypotheses that left the frame wait for the others).
 * lm may be NULL; with an LM the fused score is Eq. (4) of the paper by default (blank scored as
 * (1 + lambda) ln p(blank), tokens as ln p + lambda ln((1 - p(blank)) p_LM)), combined before the
 * beam is cut (late pruning); the config fields lm_rule and lm_early_pruning select Eq. (3) and early
 * pruning.  An LM together with a finite prune_margin is rejected.
 * Work is enqueued on hip_stream (a hipStream_t, NULL = default stream) in chunks of 16 steps, one
 * chunk ahead of the device; the call returns once the device has reported (through a pinned word)
 * that every utterance has finished and the back-trace has been enqueued, i.e. it blocks the calling
 * thread for most of the decode's duration (config field async_enqueue: enqueue everything and return).
 * Steps enqueued after the last utterance finished (under two chunks of them) still run; their kernels return at once.
 * The chunk behind the running one is enqueued when the running one is about 60 % through; the thread spins meanwhile
 * on two words of pinned host memory that the device writes (every utterance finished; a chunk begins).  Environment
 * variable RNNT_BEAM_TRACE_PACING (read at create): a line on stderr whenever that report does not arrive within
 * 200 ms and the thread waits for the stream instead.
 * Results stay valid until the next decode.  Graphs captured for a decode hold the LM's device tables: an LM
 * must outlive every decode that uses it, and at most 8 graphs (distinct B, T, beam, algo, LM, LM weight) are
 * kept per handle, the oldest being dropped.
 */
int rnnt_beam_decode(rnnt_beam_t *h, const float *enc, const int32_t *lengths, int32_t B, int32_t T,
                     int32_t beam, int32_t algo, const rnnt_lm_t *lm, float lm_weight, void *hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, serving loops, harnesses that
 * forbid it): rnnt_beam_decode with its whole workspace (hypothesis state, candidate lists, tree, encoder
 * projection, LSTM state) in a static 64 MiB device array of the library instead of the handle's allocation,
 * and the n-best lists written straight to the caller's DEVICE arrays: tokens [B, beam, cap] (positions beyond
 * a length untouched, longer transcripts truncated), lens [B, beam], scores [B, beam] (float64), n_steps [B],
 * flags [2] (nullable: 1 if a length was outside 0..T and clamped; 1 if the encoder projection held NaN or Inf).
 * Calls no hipMalloc / hipFree and creates no graph or event; all steps are enqueued at once (as with
 * async_enqueue) and the call returns without waiting: synchronise hip_stream before reading the outputs.
 * Always takes the fused joint path.  Returns RNNT_E_ARG when B, T and beam need more than the 64 MiB
 * (roughly: B * T * H * 4 bytes of encoder projection + 12 B * T (max_symbols + 1) beam bytes of tree must fit;
 * batch 64 x 250 frames at H = 640 does).  Every call on a GPU uses that GPU's one array: calls that overlap
 * in time on one GPU (any handles, any streams) race; nothing is kept from one call to the next.
 * rnnt_beam_results / rnnt_beam_dump_tree do not apply to it.
 */
int rnnt_beam_decode_static(rnnt_beam_t *h, const float *enc, const int32_t *lengths, int32_t B, int32_t T,
                            int32_t beam, int32_t algo, const rnnt_lm_t *lm, float lm_weight, int32_t *tokens,
                            int32_t cap, int32_t *lens, double *scores, int32_t *n_steps, int32_t *flags,
                            void *hip_stream);

/*
 * Wait for the last decode and copy its n-best lists to host memory (the decode itself ends with one device-to-host
 * copy of them into pinned memory of the handle; this call waits for it and copies from there).  The transcripts are read off the
 * hypothesis tree by following the parent pointers back from the final slots (Sec. 2.1, "Efficient
 * hypothesis storing"); no length normalisation is applied.  Host arrays, caller-owned: tokens [B, beam, cap]
 * (positions beyond the length are left untouched; transcripts longer than cap are truncated),
 * lens [B, beam] (-1 for an empty slot), scores [B, beam] (log-probability, -inf for an empty
 * slot), n_steps [B] (beam-search steps each utterance took).  Hypotheses are ordered by
 * (score descending, slot ascending).  Any pointer may be NULL.  Returns RNNT_E_NORESULT before the first
 * decode, RNNT_E_ARG if a length was outside 0..T (it was clamped; the results are those of the clamped
 * lengths), RNNT_E_NONFINITE if the encoder projection held NaN or Inf (results undefined), RNNT_E_HIP on
 * a failed HIP call.
 */
int rnnt_beam_results(rnnt_beam_t *h, int32_t *tokens, int32_t cap, int32_t *lens, double *scores,
                      int32_t *n_steps);

/*
 * Test hook: decode with the joint and prediction networks bypassed.  Hypothesis (b, k) standing at
 * frame t reads token log-probabilities tok_logp[b, t, c, 0..V] and duration log-probabilities
 * dur_logp[b, t, c, :] (NULL for RNN-T) with class c = hash_k mod C, where hash_k is the rolling
 * hash of Eq. (1).  Both arrays are device float32 and are taken as already normalised.
 */
int rnnt_beam_decode_injected(rnnt_beam_t *h, const float *tok_logp, const float *dur_logp, int32_t C,
                              const int32_t *lengths, int32_t B, int32_t T, int32_t beam, int32_t algo,
                              void *hip_stream);

/*
 * Test hook: the hypothesis tree of the last decode (Sec. 2.1, "Efficient hypothesis storing"),
 * copied to host arrays [S, B, beam] with S = max over n_steps: for the slot filled at that step,
 * the parent slot at the previous step (-1 = empty slot), the token appended (>= 0), -1 for blank,
 * -2 for a waiting hypothesis, -3 for an empty slot, and the slot it was merged into by
 * recombination (itself if it survived, -1 if empty).  Entries of steps an utterance did not take
 * are -9.  Pointers may be NULL; s_cap = rows available in the arrays.
 */
int rnnt_beam_dump_tree(rnnt_beam_t *h, int32_t *parent, int32_t *token, int32_t *merged_into, int32_t s_cap);

/*
 * Test hooks for single stages, all device float32, synchronous:
 *   rnnt_beam_debug_encproj : f_proj [B*T, H] of the last decode is copied to host `out` (frames behind an
 *                             utterance's length are not all computed: their rows hold anything).
 *   rnnt_beam_debug_lm      : LM scores (natural log) of every token after each of n contexts;
 *                             ctx_tokens host [n, order-1], most recent token first, -1 = none;
 *                             out host [n, V].
 */
int rnnt_beam_debug_encproj(rnnt_beam_t *h, float *out, int64_t n_floats);
int rnnt_lm_debug_query(const rnnt_lm_t *lm, const int32_t *ctx_tokens, int32_t n, float *out);

/*
 * Test hook for host logic, needs no GPU: the block -> work item mapping of the per-step launches.  A launch has
 * two roles, each a grid of (n-tile, m-tile) items: role 0 with n-tiles [0, a_tiles) x a_m m-tiles, role 1 with
 * n-tiles [b_begin, b_end) x b_m m-tiles.  Workgroup i runs on XCD i % 8, so every item of n-tile n gets a block
 * index congruent to n modulo 8.  Returns the number of blocks to launch (a multiple of 8) and, for the first
 * `cap` blocks, role (-1 = idle), n-tile and m-tile in the host arrays (each may be NULL).
 */
int rnnt_beam_debug_block_map(int32_t a_tiles, int32_t a_m, int32_t b_begin, int32_t b_end, int32_t b_m, int32_t *role,
                              int32_t *ntile, int32_t *mtile, int32_t cap);

/* Test hook for the error path of the single-launch step loop: the number of polls after which a wait between its
 * blocks gives up (default 2^22).  With a limit of a few polls the first wait fails, every block returns, and
 * rnnt_beam_results reports RNNT_E_HIP; no kernel is left waiting. */
int rnnt_beam_debug_set_spin_limit(rnnt_beam_t *h, int32_t polls);

/* Time, in milliseconds, between the first and the last kernel of the last decode (HIP events on
 * the decode's stream); negative if unavailable.  Synchronises. */
float rnnt_beam_last_decode_ms(rnnt_beam_t *h);

/*
 * Per-kernel timing of the last decode, measured with HIP events on the decode's stream when
 * profiling was switched on with rnnt_beam_set_profiling(h, 1) (plain launches are used instead
 * of the graph for that decode).  names: up to n_cap pointers to static strings; ms / calls:
 * total milliseconds and launch count per kernel.  Returns the number of kernels, or < 0.
 */
int rnnt_beam_set_profiling(rnnt_beam_t *h, int32_t on);
int rnnt_beam_kernel_times(rnnt_beam_t *h, const char **names, float *ms, int32_t *calls, int32_t n_cap);

const char *rnnt_beam_last_error(const rnnt_beam_t *h); /* NULL handle: error of the last failed create */
void rnnt_beam_destroy(rnnt_beam_t *h);
void rnnt_lm_destroy(rnnt_lm_t *lm);

#ifdef __cplusplus
}
#endif
#endif /* RNNT_BEAM_H */
