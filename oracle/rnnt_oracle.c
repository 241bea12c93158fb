/*
 * CPU oracle for batched Transducer beam search (ALSD++ / AES++, RNN-T and TDT).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * decoding path computes.  Only the tests, the smoke check and the CPU-baseline
 * leg of the benchmark may call it; the HIP library never does and shares no
 * code, table or helper with it.
 *
 * Every utterance is decoded on its own with explicit token vectors per
 * hypothesis (no tree), in double precision from the float32 inputs.
 *
 * What follows the paper and where:
 *   - a beam iteration is expansion, merging of hypotheses with identical
 *     transcripts, and pruning to the Beam best (Methods, first paragraph);
 *   - exactly Beam slots are kept per utterance, a deleted hypothesis is a slot
 *     whose score is -inf (Sec. 2.1, "Audio- and beam-level batching" and
 *     "Efficient hypothesis pruning and merging");
 *   - hypotheses are compared through the rolling hash of Eq. (1) together with
 *     length and last token (Sec. 2.1);
 *   - ALSD++ walks the T frames with at most s expansions per frame, all
 *     hypotheses sharing the alignment length; AES++ is frame-synchronous with a
 *     limited number of expansions per frame (Sec. 2.2);
 *   - shallow fusion scores follow Eq. (3) or Eq. (4), combined before the
 *     Beam best are chosen (late pruning, Sec. 2.3).
 * The paper leaves many details to its code.  The readings taken here (hash
 * constants, merge key, log-sum merge, step-wise frame limit, AES++ waiting
 * rule, TDT duration rule, prune margin) are listed in the repository's design
 * notes; the parity of those readings with the authors' code is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_HASH_BASE 1000003ULL
#define ORC_HASH_MOD 2147483647ULL /* 2^31 - 1 */

typedef struct {
  int32_t model;       /* 0 = RNN-T, 1 = TDT */
  int32_t pred;        /* 0 = LSTM, 1 = stateless */
  int32_t prec;        /* 0 = float32 operands, 1 = joint operands rounded to bf16 */
  int32_t D, H, P, E, V;
  int32_t n_dur;
  int32_t durations[8];
  int32_t ctx;         /* stateless context size */
  int32_t max_symbols; /* s */
  int32_t lm_rule;     /* 4 = Eq. (4) blank scoring, 3 = Eq. (3) */
  int32_t lm_prune;    /* 0 = late pruning: the Beam best are chosen on the fused scores;
                          1 = early pruning: they are chosen on the Transducer's scores alone and the
                          chosen ones are then rescored with the LM (Sec. 2.3, "Early/late pruning") */
  int32_t tdt_pairs;   /* TDT: 0 = one duration per candidate (the most likely one; for blank the most likely one
                          that advances); 1 = every (symbol, duration) pair is a candidate of its own, blank only
                          with durations >= 1 */
  int32_t aes_prefix;  /* AES++ only: maximum-length prefix search (Sec. 2.2, "AES"), see decode_utterance */
  double gamma;        /* prune margin on log-probability, INFINITY = off */
} orc_config;

typedef struct {
  const float *W_enc, *b_enc, *W_pred, *b_pred, *W_out, *b_out, *emb, *W_ih, *W_hh, *b_ih, *b_hh;
} orc_weights;

/* ------------------------------------------------------------------ numerics */

/* float32 value rounded to bfloat16 (round to nearest, ties to even). */
static double bf16_round(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

static inline double opnd(const orc_config *c, double x) { return c->prec ? bf16_round(x) : x; }

static double logsumexp(const double *x, int n) {
  double m = -INFINITY;
  for (int i = 0; i < n; ++i)
    if (x[i] > m) m = x[i];
  if (m == -INFINITY) return -INFINITY;
  double s = 0.0;
  for (int i = 0; i < n; ++i) s += exp(x[i] - m);
  return m + log(s);
}

static double logaddexp(double a, double b) {
  if (a == -INFINITY) return b;
  if (b == -INFINITY) return a;
  double m = a > b ? a : b;
  return m + log(exp(a - m) + exp(b - m));
}

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* ------------------------------------------------------------------- model */

/* out[r] = sum_j W[r, j] x[j], W row-major float32 [rows, cols], x already in
 * the operand precision.  round_w: round each weight to bf16 first. */
static void matvec(const float *W, const double *x, int rows, int cols, int round_w, double *out) {
  for (int r = 0; r < rows; ++r) {
    const float *row = W + (size_t)r * cols;
    double acc = 0.0;
    if (round_w) {
      for (int j = 0; j < cols; ++j) acc += bf16_round((double)row[j]) * x[j];
    } else {
#pragma omp simd reduction(+ : acc)
      for (int j = 0; j < cols; ++j) acc += (double)row[j] * x[j];
    }
    out[r] = acc;
  }
}

/* w_ready: the three joint matrices handed in were rounded to bf16 beforehand
 * (only the batch decoder does that, to avoid rounding them again at every call). */
static void enc_proj_impl(const orc_config *c, const orc_weights *w, const float *enc_t, double *f, int w_ready) {
  double *x = (double *)malloc(sizeof(double) * (size_t)c->D);
  for (int d = 0; d < c->D; ++d) x[d] = opnd(c, (double)enc_t[d]);
  matvec(w->W_enc, x, c->H, c->D, c->prec && !w_ready, f);
  for (int j = 0; j < c->H; ++j) f[j] += (double)w->b_enc[j];
  free(x);
}

/* f = W_enc enc_t + b_enc */
void orc_enc_proj(const orc_config *c, const orc_weights *w, const float *enc_t, double *f) {
  enc_proj_impl(c, w, enc_t, f, 0);
}

/* One LSTM cell step, gate order (i, f, g, o); x = emb[token].  Always in full
 * precision: the bf16 variant rounds the joint network's operands only. */
void orc_lstm_step(const orc_config *c, const orc_weights *w, const double *h_in, const double *c_in,
                   int token, double *h_out, double *c_out) {
  const int P = c->P, E = c->E;
  double *x = (double *)malloc(sizeof(double) * (size_t)E);
  double *gi = (double *)malloc(sizeof(double) * 4 * (size_t)P);
  double *gh = (double *)malloc(sizeof(double) * 4 * (size_t)P);
  for (int e = 0; e < E; ++e) x[e] = (double)w->emb[(size_t)token * E + e];
  matvec(w->W_ih, x, 4 * P, E, 0, gi);
  matvec(w->W_hh, h_in, 4 * P, P, 0, gh);
  for (int p = 0; p < P; ++p) {
    double gate[4];
    for (int q = 0; q < 4; ++q) {
      int r = q * P + p;
      gate[q] = gi[r] + (double)w->b_ih[r] + gh[r] + (double)w->b_hh[r];
    }
    double ig = sigmoid(gate[0]);
    double fg = sigmoid(gate[1]);
    double gg = tanh(gate[2]);
    double og = sigmoid(gate[3]);
    double cn = fg * c_in[p] + ig * gg;
    c_out[p] = cn;
    h_out[p] = og * tanh(cn);
  }
  free(x);
  free(gi);
  free(gh);
}

/* Stateless prediction network: sum of position-specific embeddings of the
 * last ctx tokens (position 0 = latest; row V stands for "no token yet").  In
 * the bf16 variant each embedding row is an operand of the joint's prediction
 * projection and is rounded on its own, before the sum. */
void orc_stateless_embed(const orc_config *c, const orc_weights *w, const int *tokens, int len, double *e) {
  for (int p = 0; p < c->P; ++p) e[p] = 0.0;
  for (int i = 0; i < c->ctx; ++i) {
    int tok = (len - 1 - i >= 0) ? tokens[len - 1 - i] : c->V;
    const float *row = w->emb + ((size_t)i * (c->V + 1) + tok) * c->P;
    for (int p = 0; p < c->P; ++p) e[p] += opnd(c, (double)row[p]);
  }
}

static void pred_proj_impl(const orc_config *c, const orc_weights *w, const double *h, double *g, int w_ready,
                           int x_ready) {
  double *x = (double *)malloc(sizeof(double) * (size_t)c->P);
  for (int p = 0; p < c->P; ++p) x[p] = x_ready ? h[p] : opnd(c, h[p]);
  matvec(w->W_pred, x, c->H, c->P, c->prec && !w_ready, g);
  for (int j = 0; j < c->H; ++j) g[j] += (double)w->b_pred[j];
  free(x);
}

/* Stateless prediction network output for a transcript: W_pred (sum of embeddings) + b_pred */
void orc_stateless_pred(const orc_config *c, const orc_weights *w, const int *tokens, int len, double *g) {
  double *e = (double *)malloc(sizeof(double) * (size_t)c->P);
  orc_stateless_embed(c, w, tokens, len, e);
  pred_proj_impl(c, w, e, g, 0, 1);
  free(e);
}

/* g = W_pred h + b_pred */
void orc_pred_proj(const orc_config *c, const orc_weights *w, const double *h, double *g) {
  pred_proj_impl(c, w, h, g, 0, 0);
}

static void joint_impl(const orc_config *c, const orc_weights *w, const double *f, const double *g, double *z,
                       int w_ready) {
  const int H = c->H, N = c->V + 1 + c->n_dur;
  double *a = (double *)malloc(sizeof(double) * (size_t)H);
  for (int j = 0; j < H; ++j) {
    double s = f[j] + g[j];
    a[j] = opnd(c, s > 0.0 ? s : 0.0);
  }
  matvec(w->W_out, a, N, H, c->prec && !w_ready, z);
  for (int n = 0; n < N; ++n) z[n] += (double)w->b_out[n];
  free(a);
}

/* z = W_out ReLU(f + g) + b_out, all V+1+n_dur logits. */
void orc_joint(const orc_config *c, const orc_weights *w, const double *f, const double *g, double *z) {
  joint_impl(c, w, f, g, z, 0);
}

/* The same three joint-network products for callers that hold the weight matrices already rounded to bf16
 * (rounding is idempotent, so the results are those of the functions above; the per-call rounding of every
 * weight is what is saved). */
void orc_enc_proj_rounded(const orc_config *c, const orc_weights *w, const float *enc_t, double *f) {
  enc_proj_impl(c, w, enc_t, f, 1);
}
void orc_pred_proj_rounded(const orc_config *c, const orc_weights *w, const double *h, double *g) {
  pred_proj_impl(c, w, h, g, 1, 0);
}
void orc_stateless_pred_rounded(const orc_config *c, const orc_weights *w, const int *tokens, int len, double *g) {
  double *e = (double *)malloc(sizeof(double) * (size_t)c->P);
  orc_stateless_embed(c, w, tokens, len, e);
  pred_proj_impl(c, w, e, g, 1, 1);
  free(e);
}
void orc_joint_rounded(const orc_config *c, const orc_weights *w, const double *f, const double *g, double *z) {
  joint_impl(c, w, f, g, z, 1);
}

/* ---------------------------------------------------------------- n-gram LM */

typedef struct {
  int order;        /* highest order */
  int64_t n;
  int32_t *tokens;  /* [n, order], -1 padded, sorted by (order, tokens) */
  int8_t *ng_order; /* [n] */
  float *prob, *backoff; /* log10 */
} orc_lm;

static int g_cmp_order; /* qsort has no context argument; oracle creation is single-threaded */
static const int32_t *g_cmp_tokens;
static const int8_t *g_cmp_ng;

static int ngram_cmp_keys(int oa, const int32_t *ta, int ob, const int32_t *tb) {
  if (oa != ob) return oa < ob ? -1 : 1;
  for (int i = 0; i < oa; ++i)
    if (ta[i] != tb[i]) return ta[i] < tb[i] ? -1 : 1;
  return 0;
}

static int cmp_perm(const void *a, const void *b) {
  int64_t ia = *(const int64_t *)a, ib = *(const int64_t *)b;
  return ngram_cmp_keys(g_cmp_ng[ia], g_cmp_tokens + ia * g_cmp_order, g_cmp_ng[ib],
                        g_cmp_tokens + ib * g_cmp_order);
}

orc_lm *orc_lm_create(int order, int64_t n, const int32_t *tokens, const int8_t *ng_order,
                      const float *log10_prob, const float *log10_backoff) {
  orc_lm *lm = (orc_lm *)calloc(1, sizeof(orc_lm));
  lm->order = order;
  lm->n = n;
  lm->tokens = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * order);
  lm->ng_order = (int8_t *)malloc((size_t)n);
  lm->prob = (float *)malloc(sizeof(float) * (size_t)n);
  lm->backoff = (float *)malloc(sizeof(float) * (size_t)n);
  int64_t *perm = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
  for (int64_t i = 0; i < n; ++i) perm[i] = i;
  g_cmp_order = order;
  g_cmp_tokens = tokens;
  g_cmp_ng = ng_order;
  qsort(perm, (size_t)n, sizeof(int64_t), cmp_perm);
  for (int64_t i = 0; i < n; ++i) {
    int64_t s = perm[i];
    memcpy(lm->tokens + i * order, tokens + s * order, sizeof(int32_t) * order);
    lm->ng_order[i] = ng_order[s];
    lm->prob[i] = log10_prob[s];
    lm->backoff[i] = log10_backoff[s];
  }
  free(perm);
  return lm;
}

void orc_lm_destroy(orc_lm *lm) {
  if (!lm) return;
  free(lm->tokens);
  free(lm->ng_order);
  free(lm->prob);
  free(lm->backoff);
  free(lm);
}

/* index of the n-gram with these tokens, or -1 */
static int64_t lm_find(const orc_lm *lm, const int32_t *toks, int n) {
  int64_t lo = 0, hi = lm->n - 1;
  while (lo <= hi) {
    int64_t mid = lo + (hi - lo) / 2;
    int c = ngram_cmp_keys(lm->ng_order[mid], lm->tokens + mid * lm->order, n, toks);
    if (c == 0) return mid;
    if (c < 0) lo = mid + 1; else hi = mid - 1;
  }
  return -1;
}

/* Back-off rule of ARPA models, log10: q(v | ctx) = p(ctx v) if stored, else
 * bo(ctx) + q(v | ctx without its oldest token); bo = 0 for a context that is
 * not stored.  ctx holds n tokens, oldest first. */
static double lm_q10(const orc_lm *lm, const int32_t *ctx, int n, int v) {
  int32_t key[16];
  for (int i = 0; i < n; ++i) key[i] = ctx[i];
  key[n] = v;
  int64_t hit = lm_find(lm, key, n + 1);
  if (hit >= 0) return (double)lm->prob[hit];
  if (n == 0) return -99.0; /* every unigram is stored; an absent one is "impossible" */
  int64_t c = lm_find(lm, ctx, n);
  double bo = c >= 0 ? (double)lm->backoff[c] : 0.0;
  return bo + lm_q10(lm, ctx + 1, n - 1, v);
}

/* Natural-log LM scores of every token after a hypothesis with the given
 * transcript: context = its last min(len, order-1) tokens. */
void orc_lm_query(const orc_lm *lm, const int32_t *tokens, int len, int V, double *out) {
  int n = len < lm->order - 1 ? len : lm->order - 1;
  const int32_t *ctx = tokens + (len - n);
  const double ln10 = log(10.0);
  for (int v = 0; v < V; ++v) out[v] = ln10 * lm_q10(lm, ctx, n, v);
}

/* ------------------------------------------------------- per-row score rule */

/*
 * From the logits of one (utterance, hypothesis) pair to the total score of
 * every candidate of that hypothesis.
 *   logp = log_softmax(z[0..V]) (blank = V); TDT: dlogp = log_softmax(z[V+1..]).
 *   LM, Eq. (4): tot[v] = logp[v] + lambda (ln(1 - p_blank) + lm[v]),
 *                tot[blank] = (1 + lambda) logp[blank];
 *       Eq. (3): tot[v] = logp[v] + lambda lm[v], tot[blank] = logp[blank].
 *   ln(1 - p_blank) = lse(z[0..V-1]) - lse(z[0..V]).
 *   Prune margin (if apply_gamma): tokens with logp < max logp - gamma get -inf.
 *   Frame limit (if forced_blank): every non-blank gets -inf, blank keeps its
 *   unpruned value.
 *   TDT: one duration per candidate: the most likely one for tokens, the most
 *   likely one that advances at least one frame for blank; its log-probability
 *   is added.  adv_tok / adv_blank return the frames advanced.
 * logp_in != NULL: z is ignored and logp_in[0..V] (and dlogp_in) are taken as
 * already normalised log-probabilities (injected mode).
 * gap_out (nullable) is lowered to the smallest margin by which a duration
 * argmax was decided.
 * dl_out (nullable, TDT): the duration log-probabilities are returned there and NOT
 * added to tot (every (symbol, duration) pair is then a candidate of the caller's).
 */
void orc_score_row(const orc_config *c, const double *z, const double *logp_in, const double *dlogp_in,
                   const double *lm, double lambda, int apply_gamma, int forced_blank, double *tot,
                   double *logp_out, int *adv_tok, int *adv_blank, double *gap_out, double *dl_out) {
  const int V = c->V;
  double *logp = logp_out;
  double nb = 0.0;
  if (logp_in) {
    for (int v = 0; v <= V; ++v) logp[v] = logp_in[v];
    if (lm) {
      double l_nb = logsumexp(logp, V), l_all = logsumexp(logp, V + 1);
      nb = l_nb - l_all;
    }
  } else {
    double l_all = logsumexp(z, V + 1);
    double l_nb = logsumexp(z, V);
    for (int v = 0; v <= V; ++v) logp[v] = z[v] - l_all;
    nb = l_nb - l_all;
  }
  for (int v = 0; v < V; ++v) {
    if (!lm) tot[v] = logp[v];
    else if (c->lm_rule == 3) tot[v] = logp[v] + lambda * lm[v];
    else tot[v] = logp[v] + lambda * (nb + lm[v]);
  }
  tot[V] = (lm && c->lm_rule != 3) ? (1.0 + lambda) * logp[V] : logp[V];
  double blank_unpruned = tot[V];
  if (apply_gamma && isfinite(c->gamma)) {
    double mx = -INFINITY;
    for (int v = 0; v <= V; ++v)
      if (logp[v] > mx) mx = logp[v];
    for (int v = 0; v <= V; ++v)
      if (logp[v] < mx - c->gamma) tot[v] = -INFINITY;
  }
  if (forced_blank) {
    for (int v = 0; v < V; ++v) tot[v] = -INFINITY;
    tot[V] = blank_unpruned;
  }
  *adv_tok = 0;
  *adv_blank = 1;
  if (c->model == 1) {
    double dl[8];
    if (dlogp_in) {
      for (int d = 0; d < c->n_dur; ++d) dl[d] = dlogp_in[d];
    } else {
      double l = logsumexp(z + V + 1, c->n_dur);
      for (int d = 0; d < c->n_dur; ++d) dl[d] = z[V + 1 + d] - l;
    }
    if (dl_out) {
      for (int d = 0; d < c->n_dur; ++d) dl_out[d] = dl[d];
      return;
    }
    int best = -1, best_b = -1;
    for (int d = 0; d < c->n_dur; ++d) {
      if (best < 0 || dl[d] > dl[best]) best = d;
      if (c->durations[d] >= 1 && (best_b < 0 || dl[d] > dl[best_b])) best_b = d;
    }
    if (gap_out) {
      for (int d = 0; d < c->n_dur; ++d) {
        if (d != best && dl[best] - dl[d] < *gap_out) *gap_out = dl[best] - dl[d];
        if (d != best_b && c->durations[d] >= 1 && dl[best_b] - dl[d] < *gap_out) *gap_out = dl[best_b] - dl[d];
      }
    }
    for (int v = 0; v < V; ++v) tot[v] += dl[best];
    tot[V] += dl[best_b];
    *adv_tok = c->durations[best];
    *adv_blank = c->durations[best_b];
  }
}

/* --------------------------------------------------------------- selection */

typedef struct {
  double key; /* what the candidates are ranked by */
  double val; /* the score the new hypothesis gets; differs from key under early pruning only */
  int64_t idx;
} cand_t;

static int cand_cmp(const void *a, const void *b) {
  const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
  if (x->key > y->key) return -1;
  if (x->key < y->key) return 1;
  return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
}

/* The K best of n candidates by (value descending, index ascending): a full
 * sort, the definition of top-K.  out_idx[K]. */
void orc_topk(const double *val, int64_t n, int K, int64_t *out_idx) {
  cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)n);
  for (int64_t i = 0; i < n; ++i) {
    c[i].key = val[i];
    c[i].val = val[i];
    c[i].idx = i;
  }
  qsort(c, (size_t)n, sizeof(cand_t), cand_cmp);
  for (int k = 0; k < K; ++k) out_idx[k] = k < n ? c[k].idx : -1;
  free(c);
}

/* --------------------------------------------------------------- hypotheses */

typedef struct {
  int live;
  double score;
  int t, sym, len, last;
  uint32_t hash;
  int32_t *tok; /* explicit transcript */
  double *h, *c; /* LSTM state [P] */
  double *g;     /* prediction-network output after W_pred [H] */
  double *lm;    /* LM scores of every token after this transcript [V] */
} hyp_t;

static void hyp_alloc(hyp_t *h, const orc_config *c, int cap, int with_lm) {
  memset(h, 0, sizeof(*h));
  h->tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)(cap + 1));
  h->h = (double *)calloc((size_t)c->P, sizeof(double));
  h->c = (double *)calloc((size_t)c->P, sizeof(double));
  h->g = (double *)calloc((size_t)c->H, sizeof(double));
  h->lm = with_lm ? (double *)calloc((size_t)c->V, sizeof(double)) : NULL;
}

static void hyp_free(hyp_t *h) {
  free(h->tok);
  free(h->h);
  free(h->c);
  free(h->g);
  free(h->lm);
}

static void hyp_copy(hyp_t *dst, const hyp_t *src, const orc_config *c) {
  dst->live = src->live;
  dst->score = src->score;
  dst->t = src->t;
  dst->sym = src->sym;
  dst->len = src->len;
  dst->last = src->last;
  dst->hash = src->hash;
  memcpy(dst->tok, src->tok, sizeof(int32_t) * (size_t)src->len);
  memcpy(dst->h, src->h, sizeof(double) * (size_t)c->P);
  memcpy(dst->c, src->c, sizeof(double) * (size_t)c->P);
  memcpy(dst->g, src->g, sizeof(double) * (size_t)c->H);
  if (dst->lm && src->lm) memcpy(dst->lm, src->lm, sizeof(double) * (size_t)c->V);
}

/* prediction network output for the transcript held in hyp (after a token was appended,
 * or for the empty transcript when len == 0 and first != 0) */
static void hyp_pred(hyp_t *hy, const orc_config *c, const orc_weights *w, const hyp_t *parent, int token,
                     int w_ready) {
  if (c->pred == 0) {
    double *hn = (double *)malloc(sizeof(double) * (size_t)c->P);
    double *cn = (double *)malloc(sizeof(double) * (size_t)c->P);
    orc_lstm_step(c, w, parent->h, parent->c, token, hn, cn);
    memcpy(hy->h, hn, sizeof(double) * (size_t)c->P);
    memcpy(hy->c, cn, sizeof(double) * (size_t)c->P);
    free(hn);
    free(cn);
    pred_proj_impl(c, w, hy->h, hy->g, w_ready, 0);
  } else {
    double *e = (double *)malloc(sizeof(double) * (size_t)c->P);
    orc_stateless_embed(c, w, hy->tok, hy->len, e);
    pred_proj_impl(c, w, e, hy->g, w_ready, 1);
    free(e);
  }
}

typedef struct {
  /* inputs */
  const orc_config *cfg;
  const orc_weights *w;
  const float *enc;       /* [T_pad, D] of this utterance, or NULL in injected mode */
  int T_b, beam, algo;    /* algo 0 = ALSD, 1 = AES */
  const orc_lm *lm;
  double lambda;
  int w_ready;            /* joint matrices pre-rounded to bf16 */
  const float *inj_tok;   /* [T_pad, C, V+1] or NULL */
  const float *inj_dur;   /* [T_pad, C, n_dur] or NULL */
  int C;
  /* outputs */
  int32_t *tokens; int cap; int32_t *lens; double *scores; /* [beam, cap], [beam], [beam] */
  int32_t *log_parent, *log_token, *log_merged; int S_cap;  /* [S_cap, beam] each, nullable */
  double *log_gap;        /* [S_cap] smallest margin by which a decision of the step was taken, nullable */
  int32_t *snap_tokens, *snap_lens; int snap_every, n_snap; /* [n_snap, beam, cap], [n_snap, beam] */
  int n_steps;
  double min_gap;
  int64_t collisions, n_cut;
  double max_logp; /* largest log-probability / total score seen (must stay <= 0) */
} utt_job;

static void decode_utterance(utt_job *J) {
  const orc_config *c = J->cfg;
  const orc_weights *w = J->w;
  const int V = c->V, K = J->beam, H = c->H, s = c->max_symbols, T_b = J->T_b;
  const int N = V + 1 + c->n_dur;
  const int injected = J->inj_tok != NULL;
  const int cap_tok = T_b * (s > 0 ? s : 1) + 1;

  hyp_t *cur = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)K);
  hyp_t *nxt = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)K);
  for (int k = 0; k < K; ++k) {
    hyp_alloc(&cur[k], c, cap_tok, J->lm != NULL);
    hyp_alloc(&nxt[k], c, cap_tok, J->lm != NULL);
    cur[k].live = 0;
    cur[k].score = -INFINITY;
    cur[k].last = -1;
  }
  /* frames after the encoder projection */
  double *f_proj = NULL;
  if (!injected) {
    f_proj = (double *)malloc(sizeof(double) * (size_t)(T_b > 0 ? T_b : 1) * H);
    for (int t = 0; t < T_b; ++t) enc_proj_impl(c, w, J->enc + (size_t)t * c->D, f_proj + (size_t)t * H, J->w_ready);
  }
  /* slot 0: empty transcript, prediction network fed with the start symbol (row V) */
  cur[0].live = 1;
  cur[0].score = 0.0;
  cur[0].t = 0;
  cur[0].sym = 0;
  cur[0].len = 0;
  cur[0].last = -1;
  cur[0].hash = 0;
  if (!injected) {
    hyp_t zero;
    hyp_alloc(&zero, c, 1, 0);
    hyp_pred(&cur[0], c, w, &zero, V, J->w_ready);
    hyp_free(&zero);
  }
  if (J->lm) orc_lm_query(J->lm, cur[0].tok, 0, V, cur[0].lm);

  /* candidate (k, v[, d]) has index (k (V+1) + v) [* n_dur + d]: the order in which ties are broken */
  const int pairs = c->model == 1 && c->tdt_pairs;
  const int nd = pairs ? c->n_dur : 1;
  const int64_t n_kv = (int64_t)K * (V + 1);
  const int64_t n_cand = n_kv * nd;
  cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)n_cand);
  double *unpruned = (double *)malloc(sizeof(double) * (size_t)n_kv);
  double *rowlogp = (double *)malloc(sizeof(double) * (size_t)n_kv);
  double dl[8], dl2[8];
  double *z = (double *)malloc(sizeof(double) * (size_t)N);
  double *tot = (double *)malloc(sizeof(double) * (size_t)(V + 1));
  double *logp = (double *)malloc(sizeof(double) * (size_t)(V + 1));
  double *tmp_in = (double *)malloc(sizeof(double) * (size_t)(V + 1 + 8));
  int *adv_tok = (int *)malloc(sizeof(int) * (size_t)K);
  int *adv_blank = (int *)malloc(sizeof(int) * (size_t)K);
  int *kind = (int *)malloc(sizeof(int) * (size_t)K); /* 0 dead, 1 stay, 2 active */
  double *rowmax = (double *)malloc(sizeof(double) * (size_t)K);

  J->min_gap = INFINITY;
  J->collisions = 0;
  J->n_cut = 0;
  J->max_logp = -INFINITY;
  int step = 0;
  const int step_cap = T_b * (s + 1);
  int snap_i = 0;

  for (;;) {
    /* stop when every live slot has consumed its frames */
    int unfinished = 0, t_cur = T_b;
    for (int k = 0; k < K; ++k)
      if (cur[k].live && cur[k].t < T_b) {
        unfinished = 1;
        if (cur[k].t < t_cur) t_cur = cur[k].t;
      }
    if (!unfinished || step >= step_cap) break;

    double step_gap = INFINITY;
    for (int64_t i = 0; i < n_cand; ++i) {
      cand[i].key = -INFINITY;
      cand[i].val = -INFINITY;
      cand[i].idx = i;
    }
    for (int64_t i = 0; i < n_kv; ++i) {
      unpruned[i] = -INFINITY;
      rowlogp[i] = -INFINITY;
    }
    for (int k = 0; k < K; ++k) {
      hyp_t *hy = &cur[k];
      rowmax[k] = -INFINITY;
      if (!hy->live) {
        kind[k] = 0;
        continue;
      }
      int active = hy->t < T_b && (J->algo == 0 || hy->t == t_cur);
      if (!active) {
        kind[k] = 1;
        cand[((int64_t)k * (V + 1) + V) * nd].val = hy->score; /* stay */
        cand[((int64_t)k * (V + 1) + V) * nd].key = hy->score;
        continue;
      }
      kind[k] = 2;
      const int forced = hy->sym >= s;
      const int use_gamma = J->algo == 1;
      if (injected) {
        int cls = (int)(hy->hash % (uint32_t)J->C);
        const float *row = J->inj_tok + ((size_t)hy->t * J->C + cls) * (V + 1);
        for (int v = 0; v <= V; ++v) tmp_in[v] = (double)row[v];
        if (c->model == 1) {
          const float *drow = J->inj_dur + ((size_t)hy->t * J->C + cls) * c->n_dur;
          for (int d = 0; d < c->n_dur; ++d) tmp_in[V + 1 + d] = (double)drow[d];
        }
        orc_score_row(c, NULL, tmp_in, c->model == 1 ? tmp_in + V + 1 : NULL, J->lm ? hy->lm : NULL, J->lambda,
                      use_gamma, forced, tot, logp, &adv_tok[k], &adv_blank[k], &step_gap, pairs ? dl : NULL);
      } else {
        joint_impl(c, w, f_proj + (size_t)hy->t * H, hy->g, z, J->w_ready);
        orc_score_row(c, z, NULL, NULL, J->lm ? hy->lm : NULL, J->lambda, use_gamma, forced, tot, logp,
                      &adv_tok[k], &adv_blank[k], &step_gap, pairs ? dl : NULL);
      }
      for (int v = 0; v <= V; ++v) {
        for (int d = 0; d < nd; ++d) {
          /* pairs: symbol v with duration d; blank must advance at least one frame */
          double x = pairs ? ((v == V && c->durations[d] < 1) ? -INFINITY : dl[d]) : 0.0;
          cand[((int64_t)k * (V + 1) + v) * nd + d].val = hy->score + tot[v] + x;
          cand[((int64_t)k * (V + 1) + v) * nd + d].key = hy->score + tot[v] + x;
        }
        rowlogp[(int64_t)k * (V + 1) + v] = logp[v];
        if (logp[v] > rowmax[k]) rowmax[k] = logp[v];
        if (logp[v] > J->max_logp) J->max_logp = logp[v];
        if (tot[v] > J->max_logp) J->max_logp = tot[v];
      }
      if (J->lm && c->lm_prune == 1) {
        /* early pruning: rank by the same rule without the LM term (masks and durations included) */
        int a1, a2;
        double *tot_asr = (double *)malloc(sizeof(double) * (size_t)(V + 1));
        double *lp2 = (double *)malloc(sizeof(double) * (size_t)(V + 1));
        if (injected)
          orc_score_row(c, NULL, tmp_in, c->model == 1 ? tmp_in + V + 1 : NULL, NULL, 0.0, use_gamma, forced, tot_asr,
                        lp2, &a1, &a2, NULL, pairs ? dl2 : NULL);
        else
          orc_score_row(c, z, NULL, NULL, NULL, 0.0, use_gamma, forced, tot_asr, lp2, &a1, &a2, NULL, pairs ? dl2 : NULL);
        for (int v = 0; v <= V; ++v)
          for (int d = 0; d < nd; ++d) {
            double x = pairs ? ((v == V && c->durations[d] < 1) ? -INFINITY : dl2[d]) : 0.0;
            cand[((int64_t)k * (V + 1) + v) * nd + d].key = hy->score + tot_asr[v] + x;
          }
        free(tot_asr);
        free(lp2);
      }
      if (use_gamma && isfinite(c->gamma) && !forced && !pairs) {
        /* what the candidates would have been worth without the margin, for the near-tie report */
        int a1, a2;
        double *tot2 = (double *)malloc(sizeof(double) * (size_t)(V + 1));
        double *lp2 = (double *)malloc(sizeof(double) * (size_t)(V + 1));
        if (injected)
          orc_score_row(c, NULL, tmp_in, c->model == 1 ? tmp_in + V + 1 : NULL, J->lm ? hy->lm : NULL, J->lambda, 0,
                        forced, tot2, lp2, &a1, &a2, NULL, NULL);
        else
          orc_score_row(c, z, NULL, NULL, J->lm ? hy->lm : NULL, J->lambda, 0, forced, tot2, lp2, &a1, &a2, NULL, NULL);
        for (int v = 0; v <= V; ++v) unpruned[(int64_t)k * (V + 1) + v] = hy->score + tot2[v];
        free(tot2);
        free(lp2);
      }
    }

    /* AES++, maximum-length prefix search (Sec. 2.2, "AES": the probabilities of hypotheses with shared prefixes
     * are combined; only the longest proper prefix is looked at).  For hypotheses i and j expanded at this step
     * in the same frame with transcript(i) = transcript(j) + v, the step's own expansion (j, v) reaches the
     * transcript of i.  Its score is credited to i for the RANKING of i's candidates only: the new scores stay
     * what they are, because the expansion (j, v) competes as a candidate of its own and meets i in the
     * recombination once both have left the frame; adding it to i's score as well would count that alignment
     * twice.  The credit exists only if (j, v) is one of j's Beam best token candidates (no other expansion of j
     * can be kept) and stays in the frame (TDT: duration 0).  Pairs are found through Eq. (1), as recombination
     * finds equal transcripts. */
    if (c->aes_prefix && J->algo == 1 && !pairs && !(J->lm && c->lm_prune == 1)) {
      for (int i = 0; i < K; ++i) {
        if (kind[i] != 2 || cur[i].len < 1) continue;
        double add = -INFINITY;
        const int v = cur[i].last;
        for (int j = 0; j < K; ++j) {
          if (j == i || kind[j] != 2 || cur[j].t != cur[i].t || cur[j].len + 1 != cur[i].len) continue;
          if (adv_tok[j] != 0) continue;
          if ((uint32_t)(((uint64_t)cur[j].hash * ORC_HASH_BASE + (uint64_t)(v + 1)) % ORC_HASH_MOD) != cur[i].hash) continue;
          if (memcmp(cur[j].tok, cur[i].tok, sizeof(int32_t) * (size_t)cur[j].len) != 0) J->collisions++;
          const double credit = cand[((int64_t)j * (V + 1) + v) * nd].val;
          if (!isfinite(credit)) continue;
          int better = 0; /* token candidates of j that come before (j, v) */
          for (int u = 0; u < V; ++u) {
            const double x = cand[((int64_t)j * (V + 1) + u) * nd].val;
            if (x > credit || (x == credit && u < v)) ++better;
          }
          if (better < K) add = logaddexp(add, credit);
        }
        if (add > -INFINITY) {
          const double delta = logaddexp(cur[i].score, add) - cur[i].score;
          for (int u = 0; u <= V; ++u) cand[((int64_t)i * (V + 1) + u) * nd].key += delta;
        }
      }
    }

    /* pruning: the Beam best by (value descending, flat index ascending) */
    qsort(cand, (size_t)n_cand, sizeof(cand_t), cand_cmp);
    for (int i = 0; i < K && i + 1 < n_cand; ++i)
      if (isfinite(cand[i].key) && isfinite(cand[i + 1].key)) {
        double gap = cand[i].key - cand[i + 1].key;
        if (gap < step_gap) step_gap = gap;
      }
    for (int64_t i = K; i < n_cand; ++i)
      if (isfinite(cand[i].key)) J->n_cut++; else break;
    if (J->algo == 1 && isfinite(c->gamma) && !pairs) {
      /* a token close to the margin whose candidate could have entered the beam is a near tie too */
      double thr = (K - 1 < n_cand && isfinite(cand[K - 1].val)) ? cand[K - 1].val : -INFINITY;
      for (int k = 0; k < K; ++k) {
        if (kind[k] != 2) continue;
        for (int v = 0; v <= V; ++v) {
          int64_t i = (int64_t)k * (V + 1) + v;
          if (isfinite(unpruned[i]) && unpruned[i] >= thr - 1e-3) {
            double dist = fabs(rowlogp[i] - (rowmax[k] - c->gamma));
            if (dist < step_gap) step_gap = dist;
          }
        }
      }
    }
    if (step_gap < J->min_gap) J->min_gap = step_gap;
    if (J->log_gap && step < J->S_cap) J->log_gap[step] = step_gap;

    /* expansion of the selected candidates into the new slots */
    for (int j = 0; j < K; ++j) {
      hyp_t *nh = &nxt[j];
      int32_t lp = -1, lt = -3;
      if (!isfinite(cand[j].val)) {
        nh->live = 0;
        nh->score = -INFINITY;
        nh->len = 0;
        nh->last = -1;
        nh->t = 0;
        nh->sym = 0;
        nh->hash = 0;
      } else {
        const int64_t kv = cand[j].idx / nd;
        const int dsel = (int)(cand[j].idx % nd);
        int k = (int)(kv / (V + 1)), v = (int)(kv % (V + 1));
        if (pairs) adv_tok[k] = adv_blank[k] = c->durations[dsel]; /* the pair's own duration */
        hyp_copy(nh, &cur[k], c);
        nh->score = cand[j].val;
        lp = k;
        if (kind[k] == 1) {
          lt = -2; /* stay: nothing changes */
        } else if (v == V) {
          lt = -1; /* blank: move on by one frame (TDT: by the blank's duration) */
          nh->t += adv_blank[k];
          nh->sym = 0;
        } else {
          lt = v;
          nh->tok[nh->len] = v;
          nh->len += 1;
          nh->last = v;
          nh->hash = (uint32_t)(((uint64_t)nh->hash * ORC_HASH_BASE + (uint64_t)(v + 1)) % ORC_HASH_MOD);
          nh->t += adv_tok[k];
          nh->sym = adv_tok[k] == 0 ? nh->sym + 1 : 0;
          if (!injected) hyp_pred(nh, c, w, &cur[k], v, J->w_ready);
          if (J->lm) orc_lm_query(J->lm, nh->tok, nh->len, V, nh->lm);
        }
        if (nh->t > T_b) nh->t = T_b;
      }
      if (J->log_parent && step < J->S_cap) {
        J->log_parent[(size_t)step * K + j] = lp;
        J->log_token[(size_t)step * K + j] = lt;
      }
    }

    /* merging: equal (hash, length, last token, frame, symbols in frame) -> the lowest slot keeps the log-sum */
    for (int j = 0; j < K; ++j) {
      int32_t m = -1;
      if (nxt[j].live) {
        m = j;
        for (int i = 0; i < j; ++i) {
          if (!nxt[i].live) continue;
          if (nxt[i].hash == nxt[j].hash && nxt[i].len == nxt[j].len && nxt[i].last == nxt[j].last &&
              nxt[i].t == nxt[j].t && nxt[i].sym == nxt[j].sym) {
            if (memcmp(nxt[i].tok, nxt[j].tok, sizeof(int32_t) * (size_t)nxt[j].len) != 0) J->collisions++;
            nxt[i].score = logaddexp(nxt[i].score, nxt[j].score);
            nxt[j].live = 0;
            nxt[j].score = -INFINITY;
            m = i;
            break;
          }
        }
      }
      if (J->log_merged && step < J->S_cap) J->log_merged[(size_t)step * K + j] = m;
    }
    for (int j = 0; j < K; ++j)
      if (nxt[j].live && nxt[j].score > J->max_logp) J->max_logp = nxt[j].score;

    hyp_t *sw = cur;
    cur = nxt;
    nxt = sw;
    ++step;

    if (J->snap_tokens && J->snap_every > 0 && step % J->snap_every == 0 && snap_i < J->n_snap) {
      for (int k = 0; k < K; ++k) {
        J->snap_lens[(size_t)snap_i * K + k] = cur[k].live ? cur[k].len : -1;
        if (cur[k].live)
          for (int u = 0; u < cur[k].len && u < J->cap; ++u)
            J->snap_tokens[((size_t)snap_i * K + k) * J->cap + u] = cur[k].tok[u];
      }
      ++snap_i;
    }
  }
  J->n_steps = step;

  /* n-best: live slots by (score descending, slot ascending), raw scores */
  {
    cand_t *r = (cand_t *)malloc(sizeof(cand_t) * (size_t)K);
    for (int k = 0; k < K; ++k) {
      r[k].val = cur[k].live ? cur[k].score : -INFINITY;
      r[k].key = r[k].val;
      r[k].idx = k;
    }
    qsort(r, (size_t)K, sizeof(cand_t), cand_cmp);
    for (int j = 0; j < K; ++j) {
      int k = (int)r[j].idx;
      if (!cur[k].live) {
        J->lens[j] = -1;
        J->scores[j] = -INFINITY;
        continue;
      }
      J->lens[j] = cur[k].len;
      J->scores[j] = cur[k].score;
      for (int u = 0; u < cur[k].len && u < J->cap; ++u) J->tokens[(size_t)j * J->cap + u] = cur[k].tok[u];
    }
    free(r);
  }

  for (int k = 0; k < K; ++k) {
    hyp_free(&cur[k]);
    hyp_free(&nxt[k]);
  }
  free(cur); free(nxt); free(f_proj); free(cand); free(unpruned); free(rowlogp); free(z); free(tot); free(logp);
  free(tmp_in); free(adv_tok); free(adv_blank); free(kind); free(rowmax);
}

/*
 * Decode a batch.  Utterances are independent; OpenMP spreads them over the
 * host cores and nothing else is parallel.
 *   enc [B, T, D] float32 (NULL in injected mode), lengths [B].
 *   inj_tok [B, T, C, V+1], inj_dur [B, T, C, n_dur]: when inj_tok != NULL the
 *   networks are bypassed and hypothesis (b, k) reads class hash_k mod C.
 * Outputs (caller-allocated): tokens [B, beam, cap] (untouched beyond lens),
 * lens [B, beam] (-1 = dead), scores [B, beam], n_steps [B]; logs
 * [B, S_cap, beam] (nullable): parent slot, token (>= 0 token, -1 blank,
 * -2 stay, -3 dead), merged_into (-1 dead); log_gap [B, S_cap]; snapshots every snap_every steps
 * (nullable); min_gap [B], collisions [B], n_cut [B], max_logp [B].
 * Returns the number of threads used.
 */
int orc_decode(const orc_config *cfg, const orc_weights *w, const float *enc, const int32_t *lengths, int B, int T,
               int beam, int algo, const orc_lm *lm, double lambda, const float *inj_tok, const float *inj_dur,
               int C, int32_t *tokens, int cap, int32_t *lens, double *scores, int32_t *n_steps,
               int32_t *log_parent, int32_t *log_token, int32_t *log_merged, double *log_gap, int S_cap,
               int32_t *snap_tokens,
               int32_t *snap_lens, int snap_every, int n_snap, double *min_gap, int64_t *collisions,
               int64_t *n_cut, double *max_logp, int n_threads) {
  int used = 1;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
  used = omp_get_max_threads();
  if (used > B) used = B;
#endif
  const int V = cfg->V;
  /* bf16 variant: round the three joint matrices once instead of at every use */
  orc_weights wr = *w;
  float *r_enc = NULL, *r_pred = NULL, *r_out = NULL;
  int w_ready = 0;
  if (cfg->prec && enc) {
    size_t n_enc = (size_t)cfg->H * cfg->D, n_pred = (size_t)cfg->H * cfg->P,
           n_out = (size_t)(V + 1 + cfg->n_dur) * cfg->H;
    r_enc = (float *)malloc(sizeof(float) * n_enc);
    r_pred = (float *)malloc(sizeof(float) * n_pred);
    r_out = (float *)malloc(sizeof(float) * n_out);
    for (size_t i = 0; i < n_enc; ++i) r_enc[i] = (float)bf16_round((double)w->W_enc[i]);
    for (size_t i = 0; i < n_pred; ++i) r_pred[i] = (float)bf16_round((double)w->W_pred[i]);
    for (size_t i = 0; i < n_out; ++i) r_out[i] = (float)bf16_round((double)w->W_out[i]);
    wr.W_enc = r_enc;
    wr.W_pred = r_pred;
    wr.W_out = r_out;
    w_ready = 1;
  }
  w = &wr;
#pragma omp parallel for schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    utt_job J;
    memset(&J, 0, sizeof(J));
    J.cfg = cfg;
    J.w = w;
    J.enc = enc ? enc + (size_t)b * T * cfg->D : NULL;
    J.T_b = lengths[b];
    J.beam = beam;
    J.algo = algo;
    J.lm = lm;
    J.lambda = lambda;
    J.w_ready = w_ready;
    J.inj_tok = inj_tok ? inj_tok + (size_t)b * T * C * (V + 1) : NULL;
    J.inj_dur = inj_dur ? inj_dur + (size_t)b * T * C * cfg->n_dur : NULL;
    J.C = C;
    J.tokens = tokens + (size_t)b * beam * cap;
    J.cap = cap;
    J.lens = lens + (size_t)b * beam;
    J.scores = scores + (size_t)b * beam;
    J.S_cap = S_cap;
    J.log_parent = log_parent ? log_parent + (size_t)b * S_cap * beam : NULL;
    J.log_token = log_token ? log_token + (size_t)b * S_cap * beam : NULL;
    J.log_merged = log_merged ? log_merged + (size_t)b * S_cap * beam : NULL;
    J.log_gap = log_gap ? log_gap + (size_t)b * S_cap : NULL;
    J.snap_every = snap_every;
    J.n_snap = n_snap;
    J.snap_tokens = snap_tokens ? snap_tokens + (size_t)b * n_snap * beam * cap : NULL;
    J.snap_lens = snap_lens ? snap_lens + (size_t)b * n_snap * beam : NULL;
    decode_utterance(&J);
    n_steps[b] = J.n_steps;
    if (min_gap) min_gap[b] = J.min_gap;
    if (collisions) collisions[b] = J.collisions;
    if (n_cut) n_cut[b] = J.n_cut;
    if (max_logp) max_logp[b] = J.max_logp;
  }
  free(r_enc);
  free(r_pred);
  free(r_out);
  return used;
}

/* Eq. (1): rolling hash of a transcript, token fed as v + 1, H_0 = 0. */
uint32_t orc_hash_tokens(const int32_t *tokens, int len) {
  uint32_t h = 0;
  for (int i = 0; i < len; ++i)
    h = (uint32_t)(((uint64_t)h * ORC_HASH_BASE + (uint64_t)(tokens[i] + 1)) % ORC_HASH_MOD);
  return h;
}
