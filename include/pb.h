/*
 * pb.h -- C ABI of the MI355X (gfx950) phrase-boosting tree for shallow-fusion context biasing.
 *
 * The library compiles a list of tokenized key phrases into a flattened Aho-Corasick-style
 * boosting tree (goto arcs sorted by token id, failure links, per-state backoff scores,
 * end-of-phrase flags) on the host, uploads it once, and evaluates it on the GPU for whole
 * batches of hypotheses: dense per-vocabulary boost scores and next states, and the fused
 * "acoustic log-prob + lambda * boost" selection step (greedy argmax or per-utterance beam top-k).
 *
 * Conventions for every entry point
 *   - returns a pb_status code; never throws, never aborts; PB_OK == 0;
 *   - "d_" pointers are DEVICE memory owned by the caller, on the device the tree was built for,
 *     which must be the current HIP device of the calling thread; plain pointers are HOST memory;
 *   - step calls (pb_score, pb_fuse_*) are asynchronous on `hip_stream` (a hipStream_t, NULL = the
 *     default stream); they allocate nothing, synchronise nothing and read no host memory besides
 *     their scalar arguments, so they may be captured into a HIP graph;
 *   - state ids: 0 is the root (the initial state of every hypothesis); ids follow breadth-first
 *     order with the children of a state visited by ascending token id, so the arc with index j
 *     of the (from_state, token)-sorted arc table leads to state j + 1;
 *   - a state id outside [0, num_states) in a step call does not fault: the row's outputs are
 *     filled with -1 (ids) and NaN (scores);
 *   - all scores are IEEE fp32; sums run in the order stated below with one rounding per
 *     operation and no fused multiply-add.
 */
#ifndef PB_H_
#define PB_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pb_tree pb_tree; /* opaque; owns its host and device arrays */

enum pb_status {
  PB_OK = 0,
  PB_EINVAL = -1,       /* malformed argument (null pointer, empty phrase, blank inside a phrase, ...) */
  PB_ERANGE = -2,       /* a token or size outside its range                                            */
  PB_ENOMEM = -3,       /* host or device allocation failed                                             */
  PB_EHIP = -4,         /* a HIP runtime call failed (no device, launch error)                          */
  PB_EUNSUPPORTED = -5  /* valid request outside the limits of this build (see each call)               */
};

enum pb_weight_mode {
  PB_W_UNIFORM = 0, /* every arc created by phrase i scores weights[i]                                  */
  PB_W_LOGDEPTH = 1, /* depth 1: weights[i] (= c0); depth d > 1: weights[i] * beta + ln(d)
                        (Sec. II-B, score distribution; Alg. 1 Stage 1, arc.score)                      */
  PB_W_UNIFORM_FINAL = 2 /* uniform arcs, and the arc into a state where a phrase ends additionally
                        carries the sum of the uniform scores of the path root -> state: the uniform
                        distribution with a reward at the final node that Sec. II-B describes and
                        Sec. III-D compares with                                                        */
};

enum pb_select_mode {
  PB_SELECT_FUSED = 0,        /* one stage: arg-max of the fused row over the whole vocabulary          */
  PB_SELECT_TWO_STAGE = 1,    /* two-stage greedy selection of transducer decoding (Sec. II-C)          */
  PB_SELECT_TWO_STAGE_CTC = 2 /* the same with the CTC rule for repeated labels (Sec. II-C)             */
};

typedef struct {
  int32_t vocab_size;         /* V > 0                                                                  */
  int32_t blank_id;           /* in [0, V), or -1 for a blank-free vocabulary                           */
  int32_t weight_mode;        /* enum pb_weight_mode                                                    */
  float beta;                 /* depth scaling of PB_W_LOGDEPTH (paper's example: 2)                    */
  float unk_score;            /* c_unk: score of the root self-loop taken by tokens that start no phrase
                                 (Sec. II-B; Alg. 1 Stage 2); default 0                                 */
  int32_t final_zero_backoff; /* 1: end-of-phrase states back off with score 0 (Sec. II-B, the paper's
                                 rule); 0: every state backs off with acc(fail) - acc(state)            */
  int32_t device;             /* HIP device ordinal to upload to; -1 = host-only tree (no GPU needed,
                                 step calls on it return PB_EINVAL)                                     */
  int32_t eos_id;             /* end-of-sentence token of attention encoder-decoder models, or -1.  With
                                 an EOS token, score(s, eos) = max over v != eos, v != blank of
                                 score(s, v), plus final_eos_score if s is an end-of-phrase state, and
                                 next(s, eos) = s (Sec. II-C, EOS heuristics); in every call               */
  float final_eos_score;      /* the final weight of end-of-phrase states used by that rule             */
} pb_build_opts;

typedef struct {
  int32_t num_states;     /* N, root included                        */
  int32_t num_arcs;       /* N - 1                                   */
  int32_t max_depth;      /* longest phrase                          */
  int32_t max_fail_chain; /* most failure hops from any state to root */
  int32_t root_degree;    /* tokens that start a phrase              */
  int32_t vocab_size;
  int32_t blank_id;
  int32_t eos_id;         /* -1 if the tree has no EOS rule            */
  int64_t device_bytes;   /* size of the uploaded tree, 0 if host-only */
} pb_tree_info;

/* Host view of the flat arrays the kernels read (owned by the tree; valid until pb_free). */
typedef struct {
  const int32_t* arc_begin; /* [N]   first arc of a state in the sorted arc table                       */
  const int32_t* arc_count; /* [N]   number of arcs leaving the state                                   */
  const int32_t* fail;      /* [N]   failure link (longest proper suffix that is a tree prefix)         */
  const float* backoff;     /* [N]   backoff score of the state, fp32                                   */
  const uint8_t* is_final;  /* [N]   1 if a phrase ends at the state                                    */
  const int32_t* depth;     /* [N]                                                                      */
  const int32_t* parent;    /* [N]   -1 for the root                                                    */
  const int32_t* arc_token; /* [N-1] token of arc j (rows sorted strictly ascending); target = j + 1    */
  const float* arc_score;   /* [N-1] score of arc j, fp32                                               */
  const double* acc;        /* [N]   accumulated score root -> state, double                            */
  const float* root_score;  /* [V]   dense root row: arc score or c_unk                                 */
  const int32_t* root_next; /* [V]   dense root row: depth-1 state or 0 (self-loop)                     */
  const float* p_root;      /* [N]   backoff scores summed from the state down to the root, fp32, in the
                                     order a query pays them                                            */
  const float* eos_score;   /* [N]   boost of the EOS token in every state (Sec. II-C): the largest score of
                                     the other tokens, the blank aside, plus the final weight of an
                                     end-of-phrase state; NULL for a tree without an EOS rule            */
} pb_host_view;

/*
 * pb_build -- compile the context list into the tree (Alg. 1, Stages 1 and 2; Sec. II-B).
 *   tokens[offsets[i] .. offsets[i+1]) are the token ids of phrase i; weights[i] is its context
 *   score c0 (NULL: all 1.0).  An arc takes the score of the phrase that creates it; later
 *   phrases sharing the prefix reuse it.  Duplicate phrases, phrases that are prefixes of others
 *   and one-token phrases are legal; n_phrases == 0 gives a root-only tree.
 *   Host-synchronous.  On success *out receives the tree (free with pb_free); on failure *out is
 *   untouched.  PB_EINVAL: null argument, V <= 0, blank_id outside [-1, V), unknown weight_mode,
 *   offsets not strictly increasing (an empty phrase), a phrase containing blank_id or eos_id,
 *   eos_id outside [-1, V) or equal to blank_id, a weight, beta, unk_score or final_eos_score that is not
 *   finite.  PB_ERANGE: a token outside [0, V), or scores that add up to an overflow.
 *   PB_EHIP / PB_ENOMEM: upload failed.
 */
int pb_build(const int32_t* tokens, const int64_t* offsets, int64_t n_phrases, const float* weights,
             const pb_build_opts* opts, pb_tree** out);

/* Releases host and device memory of the tree; NULL is a no-op. */
int pb_free(pb_tree* tree);

int pb_info(const pb_tree* tree, pb_tree_info* out);

/* Host view of the compiled arrays, for inspection and structural tests. */
int pb_host_arrays(const pb_tree* tree, pb_host_view* out);

/* Token string spelled by the path root -> state (host-side).  Writes min(len, cap) tokens to
   out_tokens and the full length to *out_len.  PB_ERANGE for an unknown state. */
int pb_state_prefix(const pb_tree* tree, int32_t state, int32_t* out_tokens, int32_t cap, int32_t* out_len);

/*
 * pb_score -- whole-vocabulary query, the tree's get_scores (Alg. 1 Stage 3; Sec. II-B).
 *   For every hypothesis b and every token v: starting at s = d_states[b] with p = 0, while s is
 *   not the root and has no arc on v, p += backoff(s) and s = fail(s); then
 *     d_scores[b,v] = p + arc_score(s,v), d_next[b,v] = target(s,v)      if s has an arc on v,
 *     d_scores[b,v] = p + c_unk,          d_next[b,v] = 0                 otherwise (root self-loop).
 *   The blank column is 0 with next = d_states[b].
 *   d_states int32[B]; d_scores float[B,V] row-major; d_next int32[B,V] or NULL to skip it.
 *   B == 0 is a no-op.
 */
int pb_score(const pb_tree* tree, const int32_t* d_states, int32_t B, float* d_scores, int32_t* d_next,
             void* hip_stream);

/*
 * pb_fuse_step -- one greedy shallow-fusion step (Eq. 1; Alg. 1 Stage 3) without materialising
 * the [B,V] boost.  For every hypothesis b:
 *     fused[v]        = d_logp[b*row_stride + v] + (alpha * score(d_states_in[b], v))
 *     d_tokens[b]     = argmax_v fused[v], the lowest token id among equal maxima
 *     d_states_out[b] = next(d_states_in[b], d_tokens[b])   (unchanged when the token is the blank)
 *     d_scores[b]     = fused[d_tokens[b]]
 *   row_stride >= V in elements.  d_states_out may alias d_states_in.  NaN log-probs are a
 *   precondition violation (the result is then unspecified but in range); -inf is legal.
 */
int pb_fuse_step(const pb_tree* tree, const float* d_logp, int64_t row_stride, const int32_t* d_states_in,
                 float alpha, int32_t B, int32_t* d_tokens, int32_t* d_states_out, float* d_scores,
                 void* hip_stream);

/*
 * pb_fuse_frames -- T greedy steps in one launch for the case where all frames exist up front
 * (CTC-style decoding, Sec. II-C): frame t uses d_logp[t*frame_stride + b*row_stride + v] and the
 * states produced by frame t-1 (d_states0 for t = 0).  Outputs are [T,B] row-major: the token,
 * the state after the frame and the fused score of every frame; identical to T calls of
 * pb_fuse_step.  T == 0 or B == 0 is a no-op.
 */
int pb_fuse_frames(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                   const int32_t* d_states0, float alpha, int32_t T, int32_t B, int32_t* d_tokens,
                   int32_t* d_states, float* d_scores, void* hip_stream);

/*
 * pb_fuse_step_select / pb_fuse_frames_select -- the greedy step and the multi-frame decoder with the
 * token selection rule of Sec. II-C ("two-stage token selection"), chosen by `mode`:
 *   PB_SELECT_FUSED          exactly pb_fuse_step / pb_fuse_frames (d_last* ignored).
 *   PB_SELECT_TWO_STAGE      stage 1: v0 = argmax_v d_logp[b, v] (lowest id among equal maxima), no
 *                            boosting.  If v0 is the blank: token = blank, state unchanged,
 *                            score = d_logp[b, blank]; the tree is not consulted.
 *                            Stage 2 otherwise: token = argmax over v != blank of
 *                            d_logp[b, v] + (alpha * score(state, v)) (lowest id among equal maxima),
 *                            state = next(state, token), score = that fused value.
 *   PB_SELECT_TWO_STAGE_CTC  additionally, with last = the label emitted for the hypothesis on the
 *                            previous frame: if v0 == last the repeated label is kept as it is
 *                            (token = v0, state unchanged, score = d_logp[b, v0], no boost), and
 *                            stage 2 runs over v != blank and v != last.
 *   Previous labels: pb_fuse_step_select reads d_last_tokens[b] (int32[B]; NULL or any value outside
 *   [0, V) = no previous label; it may alias d_tokens, so a decoding loop can pass the same buffer);
 *   pb_fuse_frames_select uses d_last0[b] for frame 0 (NULL = none) and the token of frame t-1 for
 *   frame t.  With a blank-free tree PB_SELECT_TWO_STAGE equals PB_SELECT_FUSED.
 *   All other arguments, outputs and error codes are those of pb_fuse_step / pb_fuse_frames;
 *   PB_EINVAL also for an unknown mode.
 */
int pb_fuse_step_select(const pb_tree* tree, const float* d_logp, int64_t row_stride, const int32_t* d_states_in,
                        const int32_t* d_last_tokens, float alpha, int32_t B, int32_t mode, int32_t* d_tokens,
                        int32_t* d_states_out, float* d_scores, void* hip_stream);

int pb_fuse_frames_select(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                          const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B,
                          int32_t mode, int32_t* d_tokens, int32_t* d_states, float* d_scores, void* hip_stream);

/*
 * pb_fuse_frames_ws -- pb_fuse_frames_select with a caller-owned workspace, the faster form of the same call
 * (identical outputs).  The decoder cuts the T frames of every hypothesis into segments decoded side by side,
 * each from a guess of the state the frame before it ends in; with the workspace a segment that finds the
 * guess for its right neighbour wrong repairs the neighbour's first frames itself and leaves them there
 * (comparing with the first frames the neighbour has decoded, which every segment leaves there too), and
 * nothing is decoded a second time.
 *   d_workspace: device memory of at least pb_fuse_frames_workspace_bytes(tree, T, B) bytes, 8-byte aligned,
 *   used only during the call (contents before and after mean nothing; two calls that overlap in time need
 *   two workspaces).  pb_fuse_frames_workspace_bytes returns the size (0 when the call needs none: T or B zero,
 *   or rows wider than 1024 tokens, which are repaired without it), or PB_EINVAL for a null tree or negative sizes.
 *   PB_EINVAL also for a workspace that is null, too small or misaligned when one is needed.
 */
int64_t pb_fuse_frames_workspace_bytes(const pb_tree* tree, int32_t T, int32_t B);
int pb_fuse_frames_ws(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                      const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B, int32_t mode,
                      int32_t* d_tokens, int32_t* d_states, float* d_scores, void* d_workspace, int64_t workspace_bytes,
                      void* hip_stream);

/*
 * pb_fuse_frames_plan -- how pb_fuse_frames* would cut the T frames of a call with B hypotheses into segments (host
 * only, nothing is launched; for tests and for sizing).  Writes the number of segments to *n_segments and, if
 * `bounds` is not NULL, n_segments + 1 frame indices to it (host array with room for 65 entries): segment j covers
 * frames bounds[j] .. bounds[j + 1] - 1, bounds[0] = 0, bounds[n_segments] = T; every hypothesis is cut the same way.
 * T == 0 or B == 0 gives zero segments.  PB_EINVAL for a null tree or n_segments, or negative sizes.
 */
int pb_fuse_frames_plan(const pb_tree* tree, int32_t T, int32_t B, int32_t* n_segments, int32_t* bounds);

/*
 * pb_fuse_frames_static -- pb_fuse_frames_ws for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation): the workspace is a fixed array inside
 * the library, 2 MiB per GPU, held from the first pb_build on that GPU until the process ends.  The call
 * allocates and frees nothing.  Outputs are those of pb_fuse_frames_ws.
 *   PB_EUNSUPPORTED when pb_fuse_frames_workspace_bytes(tree, T, B) exceeds 2 MiB (464 bytes per segment
 *   boundary; the library's segment plan keeps a call below 4096 boundaries = 1856 KiB, so only a build with a
 *   larger plan can exceed it).  Nothing in the array has to be cleared between calls (a call reads only what it
 *   has written itself), but every call on a GPU shares that GPU's array: two calls that overlap in time on one
 *   GPU, on any streams, race and may both return wrong results.
 */
int pb_fuse_frames_static(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                          const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B,
                          int32_t mode, int32_t* d_tokens, int32_t* d_states, float* d_scores, void* hip_stream);

/*
 * pb_fuse_step_beam -- one beam-search step: expansion scores, pruning and the state gather by
 * parent (Alg. 1 Stage 3: hyps_expansion_score, prune_expanded, S[t]).  Hypotheses u*K .. u*K+K-1
 * are the beams of utterance u.  For every candidate (k, v) of utterance u
 *     total = d_hyp_scores[u*K+k] + (d_logp[(u*K+k)*row_stride + v] + (alpha * score(state[u*K+k], v)))
 *   the K candidates that come first by (total descending, k*V+v ascending) are written, in that
 *   order, to slots u*K .. u*K+K-1: d_tokens = v, d_parents = k, d_states_out = next(state of the
 *   parent, v), d_scores_out = total.  -inf hypothesis scores (dead beams) are legal.
 *   1 <= K <= 32.  d_states_out must not alias d_states_in.  U == 0 is a no-op.
 */
int pb_fuse_step_beam(const pb_tree* tree, const float* d_logp, int64_t row_stride, const float* d_hyp_scores,
                      const int32_t* d_states_in, float alpha, int32_t U, int32_t K, int32_t* d_tokens,
                      int32_t* d_parents, int32_t* d_states_out, float* d_scores_out, void* hip_stream);

/*
 * Forests -- a different context list per hypothesis (or, in the beam step, per utterance).  Not in the
 * paper, whose decoders use one list per run; serving needs one per request.
 *   pb_forest_build groups n_trees trees built for the same device with the same vocab_size and blank_id
 *   and without an EOS rule (PB_EUNSUPPORTED otherwise; PB_EINVAL for null arguments, n_trees < 1 or a
 *   host-only tree).  The forest refers to the trees' device arrays: free it before them.
 *   The *_forest calls are pb_score, pb_fuse_step_select, pb_fuse_frames_select and pb_fuse_step_beam with one more device
 *   array: d_tree_ids int32[B] (beam: int32[U]) names the member tree of every row; states are states
 *   of that tree.  An id outside [0, n_trees) marks the row's outputs like an invalid state (-1 / NaN).
 */
typedef struct pb_forest pb_forest;
int pb_forest_build(const pb_tree* const* trees, int32_t n_trees, pb_forest** out);
int pb_forest_free(pb_forest* forest);
int pb_score_forest(const pb_forest* forest, const int32_t* d_tree_ids, const int32_t* d_states, int32_t B,
                    float* d_scores, int32_t* d_next, void* hip_stream);
int pb_fuse_step_forest(const pb_forest* forest, const float* d_logp, int64_t row_stride, const int32_t* d_tree_ids,
                        const int32_t* d_states_in, const int32_t* d_last_tokens, float alpha, int32_t B, int32_t mode,
                        int32_t* d_tokens, int32_t* d_states_out, float* d_scores, void* hip_stream);
int pb_fuse_frames_forest(const pb_forest* forest, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                          const int32_t* d_tree_ids, const int32_t* d_states0, const int32_t* d_last0, float alpha,
                          int32_t T, int32_t B, int32_t mode, int32_t* d_tokens, int32_t* d_states, float* d_scores,
                          void* hip_stream);
int pb_fuse_step_beam_forest(const pb_forest* forest, const float* d_logp, int64_t row_stride,
                             const int32_t* d_tree_ids, const float* d_hyp_scores, const int32_t* d_states_in,
                             float alpha, int32_t U, int32_t K, int32_t* d_tokens, int32_t* d_parents,
                             int32_t* d_states_out, float* d_scores_out, void* hip_stream);

/*
 * pb_validate -- debug aid (host-side, O(N + V)): bounds-checks every index the kernels follow in the compiled
 * tree -- arc rows tile the arc table and stay inside it, tokens in [0, V) and strictly ascending per row, arc j
 * leads to state j + 1 one level deeper, failure links lead to strictly shallower states, the root row points at
 * depth-1 states on the right token, the packed records equal the flat arrays.  PB_OK, or PB_ERANGE at the first
 * violation.  pb_build runs it by itself when the environment variable PB_DEBUG is set to anything but "0".
 * pb_validate_states -- the same for a HOST array of n state ids: PB_ERANGE and *first_bad (may be NULL) = the
 * first index whose id is outside [0, num_states).  (On the device an id outside the range never faults: see the
 * conventions above.)
 */
int pb_validate(const pb_tree* tree);
int pb_validate_states(const pb_tree* tree, const int32_t* states, int64_t n, int64_t* first_bad);

const char* pb_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* PB_H_ */
