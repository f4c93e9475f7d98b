/*
 * CPU ORACLE for the phrase-boosting tree -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, per-hypothesis / per-token implementation of what the
 * phrase-boosting tree computes, written from the paper's Algorithm 1 and
 * Sec. II-B, in the paper's order.  It exists only so that the HIP path can be
 * checked against it; it shares no code with that path and must never be
 * called from it.  Only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg may use it.
 *
 * Structure (all host memory):
 *   Stage 1 (Alg. 1, Stage 1)  prefix tree by insertion, arc score assigned when
 *                              the arc is created, accumulated node score,
 *                              end-of-phrase marks, failure links in BFS order.
 *   Stage 2 (Alg. 1, Stage 2)  per-node backoff score = acc(fail) - acc(node),
 *                              zero for end-of-phrase nodes (Sec. II-B, the
 *                              paragraph on backoff paths); root is total over
 *                              the vocabulary through self-loops with c_unk.
 *   Stage 3 (Alg. 1, Stage 3)  query one (state, token) by explicit failure-link
 *                              chasing; the whole-vocabulary row is that query
 *                              repeated V times; fusion is Eq. 1 evaluated per
 *                              token, followed by first-max argmax or by a full
 *                              sort of the beam*V candidates.
 *   Sec. II-C                  the two-stage greedy token selection with the CTC rule for
 *                              repeated labels, and the end-of-sentence heuristics of
 *                              encoder-decoder models, each written out as the text states it.
 *
 * Arithmetic: tree scores are accumulated in double and rounded once to fp32;
 * query-time sums and the fusion run in fp32, one rounding per operation, no
 * fused multiply-add (compile with -ffp-contract=off).
 *
 * State ids are canonical: root 0, then breadth-first order with the children
 * of a node visited by ascending token id.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ERANGE (-2)
#define ORC_ENOMEM (-3)

#define ORC_W_UNIFORM 0
#define ORC_W_LOGDEPTH 1
#define ORC_W_UNIFORM_FINAL 2 /* uniform arcs plus, on the arc into an end-of-phrase node, the accumulated
                                 score of all its transitions (the variant the paper compares with, Sec. II-B, III-D) */

typedef struct {
  int parent;      /* creation-order id of the parent, -1 for root           */
  int token;       /* token on the arc parent -> this                         */
  int depth;       /* root 0, first token of a phrase 1                       */
  double arc;      /* score of the arc parent -> this                         */
  double acc;      /* accumulated score root -> this                          */
  int is_final;    /* some phrase ends here                                   */
  int fail;        /* longest proper suffix that is a tree prefix             */
  int first_child; /* sibling list used while inserting                       */
  int next_sibling;
} raw_node;

typedef struct {
  int n;            /* number of states                                       */
  int V, blank;
  float c_unk;
  int eos;          /* end-of-sentence token with heuristic scores (Sec. II-C), or -1      */
  float c_eos;      /* final weight added to the EOS score at end-of-phrase states          */
  /* everything below is indexed by canonical state id */
  int *parent, *token, *depth, *fail, *is_final;
  double *acc, *arc;
  float *arcw;      /* fp32 arc score of the arc leading INTO the state       */
  float *bw;        /* fp32 backoff score of the state                        */
  int *child_begin; /* children of state s: child_tok/child_id[begin..end)    */
  int *child_tok, *child_id;
  int max_depth;
} orc_tree;

/* ---- Stage 1 helpers -------------------------------------------------------------- */

static int raw_child(const raw_node *nd, int s, int tok) {
  for (int c = nd[s].first_child; c >= 0; c = nd[c].next_sibling)
    if (nd[c].token == tok) return c;
  return -1;
}

static int cmp_tok(const void *a, const void *b) {
  const int *x = (const int *)a, *y = (const int *)b;
  return (x[0] > y[0]) - (x[0] < y[0]);
}

void orc_free(orc_tree *t) {
  if (!t) return;
  free(t->parent); free(t->token); free(t->depth); free(t->fail); free(t->is_final);
  free(t->acc); free(t->arc); free(t->arcw); free(t->bw);
  free(t->child_begin); free(t->child_tok); free(t->child_id);
  free(t);
}

orc_tree *orc_build(const int32_t *tokens, const int64_t *offsets, int64_t n_phrases,
                    const float *weights, int32_t V, int32_t blank, int32_t mode, float beta,
                    float c_unk, int32_t final_zero_backoff, int32_t *err) {
  *err = ORC_OK;
  if (V <= 0 || n_phrases < 0 || blank < -1 || blank >= V || (n_phrases > 0 && (!tokens || !offsets)) ||
      (mode != ORC_W_UNIFORM && mode != ORC_W_LOGDEPTH && mode != ORC_W_UNIFORM_FINAL)) {
    *err = ORC_EINVAL;
    return NULL;
  }
  for (int64_t i = 0; i < n_phrases; ++i) {
    if (offsets[i + 1] <= offsets[i] || offsets[i] < 0) { *err = ORC_EINVAL; return NULL; }
    for (int64_t j = offsets[i]; j < offsets[i + 1]; ++j) {
      if (tokens[j] < 0 || tokens[j] >= V) { *err = ORC_ERANGE; return NULL; }
      if (tokens[j] == blank) { *err = ORC_EINVAL; return NULL; }
    }
  }
  int64_t total = n_phrases ? offsets[n_phrases] - offsets[0] : 0;
  raw_node *nd = (raw_node *)malloc(sizeof(raw_node) * (size_t)(total + 1));
  if (!nd) { *err = ORC_ENOMEM; return NULL; }
  int n = 1;
  nd[0].parent = -1; nd[0].token = -1; nd[0].depth = 0; nd[0].arc = 0.0; nd[0].acc = 0.0;
  nd[0].is_final = 0; nd[0].fail = 0; nd[0].first_child = -1; nd[0].next_sibling = -1;

  /* Stage 1: insert every phrase; an arc gets its score when it is created. */
  for (int64_t i = 0; i < n_phrases; ++i) {
    double c0 = weights ? (double)weights[i] : 1.0;
    int cur = 0;
    int depth = 0;
    for (int64_t j = offsets[i]; j < offsets[i + 1]; ++j) {
      int tok = tokens[j];
      depth += 1; /* the first token of a phrase sits at depth 1 */
      int c = raw_child(nd, cur, tok);
      if (c < 0) {
        c = n++;
        nd[c].parent = cur; nd[c].token = tok; nd[c].depth = depth;
        if (mode == ORC_W_UNIFORM || mode == ORC_W_UNIFORM_FINAL) nd[c].arc = c0;
        else nd[c].arc = (depth == 1) ? c0 : c0 * (double)beta + log((double)depth);
        nd[c].acc = nd[cur].acc + nd[c].arc;
        nd[c].is_final = 0; nd[c].fail = 0; nd[c].first_child = -1;
        nd[c].next_sibling = nd[cur].first_child;
        nd[cur].first_child = c;
      }
      cur = c;
    }
    nd[cur].is_final = 1;
  }

  if (mode == ORC_W_UNIFORM_FINAL) {
    /* Which nodes end a phrase is known only now.  The arc into such a node gets, on top of its
       uniform score, the sum of the uniform scores of all transitions from the root to the node;
       accumulated scores are then rebuilt from the root (a parent is created before its children). */
    double *plain = (double *)malloc(sizeof(double) * (size_t)n);
    if (!plain) { free(nd); *err = ORC_ENOMEM; return NULL; }
    plain[0] = 0.0;
    for (int c = 1; c < n; ++c) {
      plain[c] = plain[nd[c].parent] + nd[c].arc;
      if (nd[c].is_final) nd[c].arc += plain[c];
      nd[c].acc = nd[nd[c].parent].acc + nd[c].arc;
    }
    free(plain);
  }

  /* Breadth-first order with children by ascending token: this is the canonical numbering. */
  int *order = (int *)malloc(sizeof(int) * (size_t)n);   /* canonical id -> creation id */
  int *canon = (int *)malloc(sizeof(int) * (size_t)n);   /* creation id -> canonical id */
  int *tmp = (int *)malloc(sizeof(int) * 2 * (size_t)(V > n ? V : n));
  if (!order || !canon || !tmp) { free(nd); free(order); free(canon); free(tmp); *err = ORC_ENOMEM; return NULL; }
  int head = 0, tail = 0;
  order[tail++] = 0;
  while (head < tail) {
    int s = order[head++];
    int k = 0;
    for (int c = nd[s].first_child; c >= 0; c = nd[c].next_sibling) { tmp[2 * k] = nd[c].token; tmp[2 * k + 1] = c; ++k; }
    qsort(tmp, (size_t)k, 2 * sizeof(int), cmp_tok);
    for (int i = 0; i < k; ++i) order[tail++] = tmp[2 * i + 1];
  }
  for (int i = 0; i < n; ++i) canon[order[i]] = i;

  /* Failure links in BFS order: follow the parent's failure chain until a node with an arc
     on this node's token is found; depth-1 nodes fail to the root. */
  for (int i = 1; i < n; ++i) {
    int s = order[i];
    int p = nd[s].parent;
    if (p == 0) { nd[s].fail = 0; continue; }
    int f = nd[p].fail;
    int target = 0;
    for (;;) {
      int c = raw_child(nd, f, nd[s].token);
      if (c >= 0) { target = c; break; }
      if (f == 0) break;
      f = nd[f].fail;
    }
    nd[s].fail = target;
  }

  orc_tree *t = (orc_tree *)calloc(1, sizeof(orc_tree));
  if (!t) { free(nd); free(order); free(canon); free(tmp); *err = ORC_ENOMEM; return NULL; }
  t->n = n; t->V = V; t->blank = blank; t->c_unk = c_unk; t->eos = -1; t->c_eos = 0.0f;
  t->parent = (int *)malloc(sizeof(int) * (size_t)n);
  t->token = (int *)malloc(sizeof(int) * (size_t)n);
  t->depth = (int *)malloc(sizeof(int) * (size_t)n);
  t->fail = (int *)malloc(sizeof(int) * (size_t)n);
  t->is_final = (int *)malloc(sizeof(int) * (size_t)n);
  t->acc = (double *)malloc(sizeof(double) * (size_t)n);
  t->arc = (double *)malloc(sizeof(double) * (size_t)n);
  t->arcw = (float *)malloc(sizeof(float) * (size_t)n);
  t->bw = (float *)malloc(sizeof(float) * (size_t)n);
  t->child_begin = (int *)malloc(sizeof(int) * (size_t)(n + 1));
  t->child_tok = (int *)malloc(sizeof(int) * (size_t)n);
  t->child_id = (int *)malloc(sizeof(int) * (size_t)n);
  if (!t->parent || !t->token || !t->depth || !t->fail || !t->is_final || !t->acc || !t->arc ||
      !t->arcw || !t->bw || !t->child_begin || !t->child_tok || !t->child_id) {
    orc_free(t); free(nd); free(order); free(canon); free(tmp); *err = ORC_ENOMEM; return NULL;
  }
  int pos = 0;
  for (int i = 0; i < n; ++i) {
    const raw_node *r = &nd[order[i]];
    t->parent[i] = r->parent < 0 ? -1 : canon[r->parent];
    t->token[i] = r->token;
    t->depth[i] = r->depth;
    t->fail[i] = canon[r->fail];
    t->is_final[i] = r->is_final;
    t->acc[i] = r->acc;
    t->arc[i] = r->arc;
    t->arcw[i] = (float)r->arc;
    if (r->depth > t->max_depth) t->max_depth = r->depth;
    /* Stage 2: backoff score; zero for end-of-phrase nodes. */
    if (i == 0) t->bw[i] = 0.0f;
    else if (r->is_final && final_zero_backoff) t->bw[i] = 0.0f;
    else t->bw[i] = (float)(nd[r->fail].acc - r->acc);
    /* children sorted by token */
    int k = 0;
    for (int c = r->first_child; c >= 0; c = nd[c].next_sibling) { tmp[2 * k] = nd[c].token; tmp[2 * k + 1] = canon[c]; ++k; }
    qsort(tmp, (size_t)k, 2 * sizeof(int), cmp_tok);
    t->child_begin[i] = pos;
    for (int j = 0; j < k; ++j) { t->child_tok[pos] = tmp[2 * j]; t->child_id[pos] = tmp[2 * j + 1]; ++pos; }
  }
  t->child_begin[n] = pos;
  free(nd); free(order); free(canon); free(tmp);
  return t;
}

/* ---- accessors -------------------------------------------------------------------- */

int32_t orc_num_states(const orc_tree *t) { return t->n; }
int32_t orc_max_depth(const orc_tree *t) { return t->max_depth; }

int32_t orc_node(const orc_tree *t, int32_t s, int32_t *parent, int32_t *token, int32_t *depth,
                 int32_t *fail, int32_t *is_final, double *acc, float *arcw, float *bw) {
  if (s < 0 || s >= t->n) return ORC_ERANGE;
  *parent = t->parent[s]; *token = t->token[s]; *depth = t->depth[s]; *fail = t->fail[s];
  *is_final = t->is_final[s]; *acc = t->acc[s]; *arcw = t->arcw[s]; *bw = t->bw[s];
  return ORC_OK;
}

/* child(s, v) or -1 */
static int child_of(const orc_tree *t, int s, int v) {
  int lo = t->child_begin[s], hi = t->child_begin[s + 1];
  while (lo < hi) {
    int mid = lo + (hi - lo) / 2;
    if (t->child_tok[mid] < v) lo = mid + 1; else hi = mid;
  }
  return (lo < t->child_begin[s + 1] && t->child_tok[lo] == v) ? t->child_id[lo] : -1;
}

int32_t orc_child(const orc_tree *t, int32_t s, int32_t v) {
  if (s < 0 || s >= t->n) return -1;
  return child_of(t, s, v);
}

/* ---- Stage 3: one (state, token) query by explicit failure-link chasing ---------- */

static void tree_query(const orc_tree *t, int s, int v, float *score, int *next) {
  if (v == t->blank) { *score = 0.0f; *next = s; return; }
  float p = 0.0f;
  int x = s;
  int c = child_of(t, x, v);
  while (x != 0 && c < 0) {
    p = p + t->bw[x];
    x = t->fail[x];
    c = child_of(t, x, v);
  }
  if (c >= 0) { *score = p + t->arcw[c]; *next = c; }
  else        { *score = p + t->c_unk;   *next = 0; }
}

/* End-of-sentence heuristics for attention encoder-decoder models (Sec. II-C, the paragraph on the
   EOS symbol).  The tree cannot score the EOS token itself, so that non-EOS boosts would suppress it.
   The EOS score of a state is therefore
     - the largest score the tree gives from this state to any other token (blank aside), and
     - on top of it the final weight c_eos when the state is an end-of-phrase state, i.e. a whole
       phrase has just been matched.
   Taking the EOS ends the hypothesis: the state is left unchanged. */
static void query(const orc_tree *t, int s, int v, float *score, int *next) {
  if (t->eos >= 0 && v == t->eos) {
    float best = 0.0f;
    int have = 0;
    for (int u = 0; u < t->V; ++u) {
      if (u == t->eos || u == t->blank) continue;
      float sc; int nx;
      tree_query(t, s, u, &sc, &nx);
      if (!have || sc > best) { best = sc; have = 1; }
    }
    float fw = t->is_final[s] ? t->c_eos : 0.0f;
    *score = best + fw;
    *next = s;
    return;
  }
  tree_query(t, s, v, score, next);
}

/* Switches the EOS heuristics on (eos_id in [0, V), not the blank, not a token of any phrase) or off (-1). */
int32_t orc_set_eos(orc_tree *t, int32_t eos_id, float final_eos_score) {
  if (eos_id < -1 || eos_id >= t->V || (eos_id >= 0 && eos_id == t->blank)) return ORC_EINVAL;
  if (eos_id >= 0)
    for (int i = 1; i < t->n; ++i) if (t->token[i] == eos_id) return ORC_EINVAL;
  t->eos = eos_id;
  t->c_eos = final_eos_score;
  return ORC_OK;
}

int32_t orc_query(const orc_tree *t, int32_t s, int32_t v, float *score, int32_t *next) {
  if (s < 0 || s >= t->n || v < 0 || v >= t->V) return ORC_ERANGE;
  int nx; query(t, s, v, score, &nx); *next = nx;
  return ORC_OK;
}

/* Whole-vocabulary rows: the single query, V times per hypothesis. */
int32_t orc_score(const orc_tree *t, const int32_t *states, int32_t B, float *scores, int32_t *next) {
  for (int b = 0; b < B; ++b) if (states[b] < 0 || states[b] >= t->n) return ORC_ERANGE;
#pragma omp parallel for schedule(static)
  for (int b = 0; b < B; ++b)
    for (int v = 0; v < t->V; ++v) {
      float sc; int nx;
      query(t, states[b], v, &sc, &nx);
      scores[(size_t)b * t->V + v] = sc;
      if (next) next[(size_t)b * t->V + v] = nx;
    }
  return ORC_OK;
}

/* Eq. 1 per token, then the first maximum (lowest token id on ties). */
int32_t orc_fuse_step(const orc_tree *t, const float *logp, int64_t row_stride, const int32_t *states_in,
                      float alpha, int32_t B, int32_t *tokens, int32_t *states_out, float *scores) {
  for (int b = 0; b < B; ++b) if (states_in[b] < 0 || states_in[b] >= t->n) return ORC_ERANGE;
#pragma omp parallel for schedule(static)
  for (int b = 0; b < B; ++b) {
    const float *row = logp + (size_t)b * row_stride;
    int s = states_in[b];
    int best_v = -1, best_next = s;
    float best = 0.0f;
    for (int v = 0; v < t->V; ++v) {
      float sc; int nx;
      query(t, s, v, &sc, &nx);
      float boost = alpha * sc;
      float fused = row[v] + boost;
      if (best_v < 0 || fused > best) { best = fused; best_v = v; best_next = nx; }
    }
    tokens[b] = best_v; states_out[b] = best_next; scores[b] = best;
  }
  return ORC_OK;
}

/* T greedy frames: the step above applied frame after frame (CTC-like: all frames known). */
int32_t orc_fuse_frames(const orc_tree *t, const float *logp, int64_t frame_stride, int64_t row_stride,
                        const int32_t *states0, float alpha, int32_t T, int32_t B, int32_t *tokens,
                        int32_t *states, float *scores) {
  int32_t *cur = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B > 0 ? B : 1));
  if (!cur) return ORC_ENOMEM;
  memcpy(cur, states0, sizeof(int32_t) * (size_t)B);
  for (int f = 0; f < T; ++f) {
    int rc = orc_fuse_step(t, logp + (size_t)f * frame_stride, row_stride, cur, alpha, B,
                           tokens + (size_t)f * B, states + (size_t)f * B, scores + (size_t)f * B);
    if (rc != ORC_OK) { free(cur); return rc; }
    memcpy(cur, states + (size_t)f * B, sizeof(int32_t) * (size_t)B);
  }
  free(cur);
  return ORC_OK;
}

/* ---- Two-stage greedy token selection (Sec. II-C, adaptation for CTC and transducer models) ----
 *
 * Per hypothesis and decoding step:
 *   stage 1  the best token WITHOUT boosting (first maximum of the acoustic row);
 *            - it is the blank: emit it, go on to the next step (tree not consulted);
 *            - CTC only: it repeats the label emitted on the previous frame: keep it, unboosted,
 *              tree state unchanged (the tree consumed that label when it was first emitted);
 *   stage 2  otherwise the remaining tokens -- non-blank, and for CTC also not the previous
 *            label -- are re-weighted by the tree (Eq. 1) and the best of THAT set is emitted
 *            (first maximum), advancing the tree state.
 * mode: 0 = single-stage (the plain fused argmax above), 1 = two-stage (transducer),
 *       2 = two-stage with the CTC repeat rule.  last_tokens[b] is the label of the previous
 *       frame (any value outside [0, V) means "none"); ignored unless mode == 2.
 */
#define ORC_SELECT_FUSED 0
#define ORC_SELECT_TWO_STAGE 1
#define ORC_SELECT_TWO_STAGE_CTC 2

int32_t orc_fuse_step_select(const orc_tree *t, const float *logp, int64_t row_stride, const int32_t *states_in,
                             const int32_t *last_tokens, float alpha, int32_t B, int32_t mode, int32_t *tokens,
                             int32_t *states_out, float *scores) {
  if (mode == ORC_SELECT_FUSED)
    return orc_fuse_step(t, logp, row_stride, states_in, alpha, B, tokens, states_out, scores);
  if (mode != ORC_SELECT_TWO_STAGE && mode != ORC_SELECT_TWO_STAGE_CTC) return ORC_EINVAL;
  for (int b = 0; b < B; ++b) if (states_in[b] < 0 || states_in[b] >= t->n) return ORC_ERANGE;
#pragma omp parallel for schedule(static)
  for (int b = 0; b < B; ++b) {
    const float *row = logp + (size_t)b * row_stride;
    int s = states_in[b];
    int last = (mode == ORC_SELECT_TWO_STAGE_CTC && last_tokens) ? last_tokens[b] : -1;
    /* stage 1: greedy selection without boosting */
    int v0 = 0;
    for (int v = 1; v < t->V; ++v) if (row[v] > row[v0]) v0 = v;
    if (v0 == t->blank || (mode == ORC_SELECT_TWO_STAGE_CTC && v0 == last)) {
      tokens[b] = v0; states_out[b] = s; scores[b] = row[v0];
      continue;
    }
    /* stage 2: re-weight the rest and reselect from it */
    int best_v = -1, best_next = s;
    float best = 0.0f;
    for (int v = 0; v < t->V; ++v) {
      if (v == t->blank) continue;
      if (mode == ORC_SELECT_TWO_STAGE_CTC && v == last) continue;
      float sc; int nx;
      query(t, s, v, &sc, &nx);
      float boost = alpha * sc;
      float fused = row[v] + boost;
      if (best_v < 0 || fused > best) { best = fused; best_v = v; best_next = nx; }
    }
    tokens[b] = best_v; states_out[b] = best_next; scores[b] = best;
  }
  return ORC_OK;
}

/* T frames of the selection above; the previous label of frame f is the token emitted at frame
   f - 1 (last0, or "none" when last0 is NULL, for the first frame). */
int32_t orc_fuse_frames_select(const orc_tree *t, const float *logp, int64_t frame_stride, int64_t row_stride,
                               const int32_t *states0, const int32_t *last0, float alpha, int32_t T, int32_t B,
                               int32_t mode, int32_t *tokens, int32_t *states, float *scores) {
  int32_t *cur = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B > 0 ? B : 1));
  int32_t *last = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B > 0 ? B : 1));
  if (!cur || !last) { free(cur); free(last); return ORC_ENOMEM; }
  memcpy(cur, states0, sizeof(int32_t) * (size_t)B);
  for (int b = 0; b < B; ++b) last[b] = last0 ? last0[b] : -1;
  for (int f = 0; f < T; ++f) {
    int rc = orc_fuse_step_select(t, logp + (size_t)f * frame_stride, row_stride, cur, last, alpha, B, mode,
                                  tokens + (size_t)f * B, states + (size_t)f * B, scores + (size_t)f * B);
    if (rc != ORC_OK) { free(cur); free(last); return rc; }
    memcpy(cur, states + (size_t)f * B, sizeof(int32_t) * (size_t)B);
    memcpy(last, tokens + (size_t)f * B, sizeof(int32_t) * (size_t)B);
  }
  free(cur); free(last);
  return ORC_OK;
}

typedef struct { float total; int64_t idx; } cand;

static int cmp_cand(const void *a, const void *b) {
  const cand *x = (const cand *)a, *y = (const cand *)b;
  if (x->total > y->total) return -1;
  if (x->total < y->total) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx);
}

/* Beam step: every (beam, token) candidate of an utterance, fully sorted by
   (total descending, flat index ascending); the first K survive. */
int32_t orc_fuse_step_beam(const orc_tree *t, const float *logp, int64_t row_stride, const float *hyp_scores,
                           const int32_t *states_in, float alpha, int32_t U, int32_t K, int32_t *tokens,
                           int32_t *parents, int32_t *states_out, float *scores_out) {
  for (int i = 0; i < U * K; ++i) if (states_in[i] < 0 || states_in[i] >= t->n) return ORC_ERANGE;
  int V = t->V;
  int fail_alloc = 0;
#pragma omp parallel for schedule(static)
  for (int u = 0; u < U; ++u) {
    cand *c = (cand *)malloc(sizeof(cand) * (size_t)K * V);
    int *nx_all = (int *)malloc(sizeof(int) * (size_t)K * V);
    if (!c || !nx_all) { fail_alloc = 1; free(c); free(nx_all); continue; }
    for (int k = 0; k < K; ++k) {
      int h = u * K + k;
      const float *row = logp + (size_t)h * row_stride;
      for (int v = 0; v < V; ++v) {
        float sc; int nx;
        query(t, states_in[h], v, &sc, &nx);
        float boost = alpha * sc;
        float expansion = row[v] + boost;
        float total = hyp_scores[h] + expansion;
        c[(size_t)k * V + v].total = total;
        c[(size_t)k * V + v].idx = (int64_t)k * V + v;
        nx_all[(size_t)k * V + v] = nx;
      }
    }
    qsort(c, (size_t)K * V, sizeof(cand), cmp_cand);
    for (int j = 0; j < K; ++j) {
      int64_t idx = c[j].idx;
      tokens[u * K + j] = (int)(idx % V);
      parents[u * K + j] = (int)(idx / V);
      states_out[u * K + j] = nx_all[idx];
      scores_out[u * K + j] = c[j].total;
    }
    free(c); free(nx_all);
  }
  return fail_alloc ? ORC_ENOMEM : ORC_OK;
}

/* Timing aid: number of threads the OpenMP loops above may use (no effect without OpenMP). */
void orc_set_threads(int32_t n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int32_t orc_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
