// Wave kernels for rows wider than 1024 tokens (gfx950, wave64): the multi-frame greedy decoder and the
// single greedy step with their selection rules (Alg. 1 Stage 3, Eq. 1; Sec. II-C).
//
//  * A row is consumed in chunks of 1024 tokens in the 16-tokens-per-lane layout of the narrow kernels.  In
//    the multi-frame decoder one wave owns a hypothesis segment and streams its rows through a ring of four
//    register buffers that runs across frame boundaries: while a frame is being decided the first chunks of
//    the next one are already in flight.  The root scores of the row sit in LDS, shared by the workgroup.
//  * Base candidates.  Every lane keeps a running maximum of logp[v] + alpha * (p_root + root_score[v])
//    over its tokens in ascending order (strictly greater replaces, so the lowest token among equal values
//    stays); one wave reduction per frame yields the row maximum and its lowest token.  The two-stage rules
//    keep a second running maximum of the raw row in the same pass.
//  * Arc candidates.  After the pass the arcs of the failure chain are evaluated one per lane, their
//    log-probs gathered from the row in memory (it has just been read, so the gathers hit in cache); chains
//    with more than one state mark tokens in an LDS bit set so that an arc shadowed by a deeper chain state
//    is skipped.  The frame is decided as in the narrow kernels: the best arc against the base winner.
//    The rare cases that this cannot settle -- the base winner is itself overridden by an arc that does not
//    beat it, the CTC rule bars the winner, or every candidate is -inf -- take a plain second pass over the
//    row with all overridden tokens marked.
//  * The single step spreads one row over a workgroup, one chunk per wave, so that the whole row is
//    requested at once; the waves' partial winners meet in LDS and wave 0 evaluates the arcs and decides.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>
#include <type_traits>

#include "pb_kernels.hpp"
#include "pb_wave.hpp"

namespace pb {

namespace {

using namespace wv;

#ifndef PB_WIDE_RING
#define PB_WIDE_RING 4
#endif
#ifndef PB_WIDE_WAVES_EU
#define PB_WIDE_WAVES_EU 2
#endif
constexpr int kRing = PB_WIDE_RING;  // chunks in flight or in use per wave

// Running arg-max of a lane over its tokens of a row; code = 16 * chunk + slot of the lane's token.
struct LaneBest {
  float m;
  int code;
};
__device__ __forceinline__ LaneBest lane_best_init() { return LaneBest{-INFINITY, 0}; }
__device__ __forceinline__ int code_token(int code, int lane) { return (code >> 4) * kChunk + tok_of(code & 15, lane); }

// Row maximum and its lowest token from the lanes' running maxima.  A row whose candidates are all -inf (or
// excluded) comes back as M == -inf with a token that means nothing: the caller takes the second pass then.
__device__ __forceinline__ void wave_pick(const LaneBest& lb, int lane, float& M, int& tok) {
  M = ukey_val(wave_max_u(ukey(lb.m)));
  tok = wave_min_nn(lb.m == M ? code_token(lb.code, lane) : INT_MAX);
}

// Boosts alpha * (p_root + root_score[v]) of the lane's 16 tokens of chunk `cb`; the blank boosts by 0
// (SEL == 0) or is excluded (NaN), the EOS token by `ce` = alpha * (EOS boost of the state) when `ce_on`.
template <int SEL>
__device__ __forceinline__ void chunk_boosts(const TreeView& t, int cb, int lane, float p_root, float alpha, bool ce_on,
                                             float ce, const float (&rw)[16], float (&bo)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j) bo[j] = __fmul_rn(alpha, __fadd_rn(p_root, rw[j]));
  const bool has_blank = static_cast<unsigned>(t.blank - cb) < static_cast<unsigned>(kChunk);
  const bool has_eos = ce_on && static_cast<unsigned>(t.eos - cb) < static_cast<unsigned>(kChunk);
  if (has_blank || has_eos) {  // uniform, and false for most chunks
    const int ln = opaque(lane);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (has_blank && slot_is(j, ln, t.blank - cb)) bo[j] = SEL == 0 ? __fmul_rn(alpha, 0.0f) : NAN;
      if (has_eos && slot_is(j, ln, t.eos - cb)) bo[j] = ce;
    }
  }
}

// One chunk of a row into the running maxima: `fb` fused under the state's boosts, `rb` the raw row
// (two-stage rules), `gb` fused under root-state boosts (TRACK: what a boundary guess needs).
// `rw` are the root scores of the chunk with NaN in the blank and EOS columns: those two tokens never enter
// the running maxima of the fused values; `special_candidates` adds them to the arc candidates instead.
template <int SEL, bool TRACK>
__device__ __forceinline__ void wide_chunk(const float (&x)[16], const float (&rw)[16], int ch, float p_root,
                                           float alpha, LaneBest& fb, LaneBest& rb, LaneBest& gb) {
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const float f = __fadd_rn(x[j], __fmul_rn(alpha, __fadd_rn(p_root, rw[j])));
    const bool up = f > fb.m;
    fb.m = up ? f : fb.m;
    fb.code = up ? 16 * ch + j : fb.code;
  }
  if constexpr (SEL != 0) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const bool up = x[j] > rb.m;
      rb.m = up ? x[j] : rb.m;
      rb.code = up ? 16 * ch + j : rb.code;
    }
  }
  if constexpr (TRACK) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float f = __fadd_rn(x[j], __fmul_rn(alpha, __fadd_rn(0.0f, rw[j])));
      const bool up = f > gb.m;
      gb.m = up ? f : gb.m;
      gb.code = up ? 16 * ch + j : gb.code;
    }
  }
}

// The blank (single-stage rule: boost 0, state kept) and the EOS token (boost tabulated per state, state kept;
// Sec. II-C) as candidates of their own: lane 63 takes the blank, lane 62 the EOS.  `ce` = alpha * (EOS boost).
// Returns whether the lane holds one, with its token and fused value.
template <int SEL>
__device__ __forceinline__ bool special_candidate(const TreeView& t, const float* __restrict__ rowp, float alpha,
                                                  float ce, bool with_eos, int lane, int& tok, float& val) {
  const bool is_blank = SEL == 0 && t.blank >= 0 && lane == 63;
  const bool is_eos = with_eos && t.eos >= 0 && lane == 62;
  tok = is_blank ? t.blank : t.eos;
  val = 0.0f;
  if (is_blank || is_eos) val = __fadd_rn(rowp[tok], is_blank ? __fmul_rn(alpha, 0.0f) : ce);
  return is_blank || is_eos;
}

__device__ __forceinline__ void read_rs_lds(const float* rs, int cb, int lane, float (&rw)[16]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 q = *reinterpret_cast<const float4*>(rs + cb + 256 * i + 4 * lane);
    rw[4 * i + 0] = q.x; rw[4 * i + 1] = q.y; rw[4 * i + 2] = q.z; rw[4 * i + 3] = q.w;
  }
}

__device__ __forceinline__ void tags_clear_n(unsigned* bits, int words, int lane) {
  for (int i = lane; i < words; i += 64) bits[i] = 0u;
}

struct FrameOut {  // wave-uniform outcome of one frame
  float val;
  int tok;
  bool arc;    // the winner is an arc of the failure chain: the next state is `child`
  int child;
};

// The whole decision of a frame by a plain second pass (any case, no speculation): every token that some
// chain state overrides is marked, the arcs are evaluated deepest state first, and the base arg-max runs
// over the unmarked tokens only.  `excl` (CTC rule): a token barred from the selection, or -1.
template <bool FULL, int SEL>
__device__ __forceinline__ FrameOut slow_frame(const TreeView& t, const Cursor& cur, const float* __restrict__ rowp,
                                               float alpha, int excl, unsigned* tags, int tag_words, int nch, int lane) {
  tags_clear_n(tags, tag_words, lane);
  float bf = 0.0f;
  int btok = INT_MAX, bchild = 0;
  {
    float p = 0.0f;
    for (int xs = cur.s; xs != 0;) {
      const Rec r = load_rec(t, xs);
      for (int j = lane; j < r.count; j += 64) {  // tokens of one state are distinct: no two lanes meet on a mark
        const ArcRec a = t.arc[r.begin + j];
        if (!tag_test(tags, a.token)) {
          tag_set(tags, a.token);
          if (SEL != 2 || a.token != excl) {
            const float fa = __fadd_rn(rowp[a.token], __fmul_rn(alpha, __fadd_rn(p, a.score)));
            if (btok == INT_MAX || fa > bf || (fa == bf && a.token < btok)) {
              bf = fa;
              btok = a.token;
              bchild = r.begin + j + 1;
            }
          }
        }
      }
      p = __fadd_rn(p, r.backoff);
      xs = uniform_i(r.fail);
    }
  }
  bool has = false;
  float m = 0.0f;
  int mtok = INT_MAX;
  const float ce = __fmul_rn(alpha, cur.eos_boost);
  for (int ch = 0; ch < nch; ++ch) {
    const int cb = ch * kChunk;
    float x[16], rw[16], bo[16];
    load16<FULL>(rowp, cb, t.V, lane, -INFINITY, x);
    load16<FULL>(t.root_score, cb, t.V, lane, 0.0f, rw);
    chunk_boosts<SEL>(t, cb, lane, cur.p_root, alpha, t.eos >= 0, ce, rw, bo);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int v = cb + tok_of(j, lane);
      const float f = __fadd_rn(x[j], bo[j]);
      const bool out = v >= t.V || f != f || (SEL == 2 && v == excl) || tag_test(tags, min(v, t.V - 1));
      if (!out && (!has || f > m)) {
        has = true;
        m = f;
        mtok = v;
      }
    }
  }
  FrameOut o{0.0f, 0, false, 0};
  const bool any_base = __ballot(has) != 0;
  float Mb = 0.0f;
  int vbase = INT_MAX;
  if (any_base) {
    Mb = ukey_val(wave_max_u(has ? ukey(m) : 0u));
    vbase = wave_min_nn((has && m == Mb) ? mtok : INT_MAX);
  }
  const bool mine0 = btok != INT_MAX;
  const bool any_arc = __ballot(mine0) != 0;
  float MA = 0.0f;
  int va = INT_MAX, achild = 0;
  if (any_arc) {
    MA = ukey_val(wave_max_u(mine0 ? ukey(bf) : 0u));
    const bool mine = mine0 && bf == MA;
    va = wave_min_nn(mine ? btok : INT_MAX);
    achild = __builtin_amdgcn_readlane(bchild, first_lane(__ballot(mine && btok == va)));
  }
  if (any_arc && (!any_base || MA > Mb || (MA == Mb && va < vbase))) {
    o = FrameOut{MA, va, true, achild};
  } else if (any_base) {
    o = FrameOut{Mb, vbase, false, 0};
  }  // (no candidate at all: only with NaN rows, a precondition violation; token 0 keeps the result in range)
  o.val = uniform_f(o.val);
  o.tok = uniform_i(o.tok);
  o.child = uniform_i(o.child);
  return o;
}

// Decides a frame whose base winner (M, vb) over all tokens is known: the arcs of the failure chain against it.
//   early: arc number `lane` of the state (clamped into its arc range), requested before the row pass, and
//   early_x: the log-prob of that arc's token, gathered during the pass
//   last:  label of the previous frame (SEL == 2; any value outside [0, V) = none)
template <bool FULL, int SEL>
__device__ __forceinline__ FrameOut decide_wide(const TreeView& t, const Cursor& cur, const float* __restrict__ rowp,
                                                float alpha, float M, int vb, const ArcRec& early, float early_x, int last,
                                                unsigned* tags, int tag_words, int nch, int lane) {
  const Rec rec0 = cur.rec;
  const bool chain = cur.s != 0;
  const bool multi = chain && rec0.fail != 0;
  float bf = -INFINITY;
  int btok = INT_MAX, bchild = 0;
  bool hit_vb = false;
  if (chain) {
    if (multi) tags_clear_n(tags, tag_words, lane);
    Rec r = rec0;
    float p = 0.0f;
    for (int level = 0;; ++level) {
      for (int j0 = 0; j0 < r.count; j0 += 64) {
        const int j = j0 + lane;
        const bool valid = j < r.count;
        ArcRec a = early;
        float xv = early_x;
        const bool first = level == 0 && j0 == 0;
        if (!first) a = t.arc[r.begin + min(j, r.count - 1)];
        const int tk = valid ? a.token : 0;  // an unused entry may hold anything: keep the indices in range
        if (!first) xv = rowp[tk];
        bool shadowed = !valid;
        if (multi) {
          if (level > 0) shadowed = shadowed || tag_test(tags, tk);  // a deeper chain state owns this token
          if (valid) tag_set(tags, tk);
        }
        hit_vb = hit_vb || (valid && tk == vb);
        const float fa = __fadd_rn(xv, __fmul_rn(alpha, __fadd_rn(p, a.score)));
        const bool take = !shadowed && (fa > bf || (fa == bf && tk < btok));
        bf = take ? fa : bf;
        btok = take ? tk : btok;
        bchild = take ? r.begin + j + 1 : bchild;
      }
      p = __fadd_rn(p, r.backoff);
      if (r.fail == 0) break;
      r = load_rec(t, r.fail);
    }
  }
  if ((SEL == 0 && t.blank >= 0) || t.eos >= 0) {  // the blank and the EOS token, kept out of the base pass
    int tk;
    float fv;
    if (special_candidate<SEL>(t, rowp, alpha, __fmul_rn(alpha, cur.eos_boost), true, lane, tk, fv)) {
      const bool take = fv > bf || (fv == bf && tk < btok);
      bf = take ? fv : bf;
      btok = take ? tk : btok;
      bchild = take ? -1 : bchild;  // no arc: the state stays
    }
  }
  bool settled = M != -INFINITY;
  FrameOut o{M, vb, false, 0};
  const bool mine0 = btok != INT_MAX;
  if (settled && __ballot(mine0) != 0) {
    const float MA = ukey_val(wave_max_u(mine0 ? ukey(bf) : 0u));
    const bool vb_overridden = __ballot(hit_vb) != 0;
    if (vb_overridden || MA >= M) {
      const bool mine = mine0 && bf == MA;
      const int va = wave_min_nn(mine ? btok : INT_MAX);
      const int achild = __builtin_amdgcn_readlane(bchild, first_lane(__ballot(mine && btok == va)));
      if (MA > M || (!vb_overridden && MA == M && va < vb)) {
        o = FrameOut{MA, va, achild >= 0, achild};
      } else if (vb_overridden) {
        settled = false;  // the base winner is shadowed by an arc that does not beat it
      }
    }
  }
  if (settled && SEL == 2 && o.tok == last) settled = false;  // the CTC rule bars the previous label
  if (!settled) {
    int excl = -1;
    if (SEL == 2) {
      // first without the exclusion (the label may not even win), then, if it does win, without the label
      o = slow_frame<FULL, SEL>(t, cur, rowp, alpha, -1, tags, tag_words, nch, lane);
      if (o.tok != last) return o;
      excl = last;
    }
    o = slow_frame<FULL, SEL>(t, cur, rowp, alpha, excl, tags, tag_words, nch, lane);
    return o;
  }
  o.val = uniform_f(o.val);
  o.tok = uniform_i(o.tok);
  o.child = uniform_i(o.child);
  return o;
}

// The state after a frame decided as `o` (need_record: false when only the id is wanted).
__device__ __forceinline__ void advance(const TreeView& t, Cursor& cur, const FrameOut& o, bool need_record) {
  if (o.arc) {
    if (need_record) {
      cur = cursor_at(t, o.child);
    } else {
      cur.s = o.child;
    }
  } else if (o.tok != t.blank && o.tok != t.eos) {  // the blank and the EOS keep the state
    const v8i rr = t.root_rec[o.tok];
    cur = cursor_from_root_rec(rr);
  }
  cur.s = uniform_i(cur.s);
  cur.rec.begin = uniform_i(cur.rec.begin);
  cur.rec.count = uniform_i(cur.rec.count);
  cur.rec.fail = uniform_i(cur.rec.fail);
  cur.rec.backoff = uniform_f(cur.rec.backoff);
  cur.p_root = uniform_f(cur.p_root);
  cur.eos_boost = uniform_f(cur.eos_boost);
}

// Winner under root-state boosts from the lanes' running maxima `gb`; under the single-stage rule the blank
// (kept out of the pass) competes with boost 0.
template <int SEL>
__device__ __forceinline__ int root_winner(const TreeView& t, const LaneBest& gb, const float* __restrict__ rowp,
                                           float alpha, int lane) {
  float M;
  int w;
  wave_pick(gb, lane, M, w);
  w = uniform_i(w);
  if (SEL == 0 && t.blank >= 0) {
    const float fb = __fadd_rn(uniform_f(rowp[t.blank]), __fmul_rn(alpha, 0.0f));
    if (fb > M || (fb == M && t.blank < w)) w = t.blank;
  }
  return w;
}

// Raw arg-max v0 (two-stage rules) and winner w under root-state boosts of one row, by a plain pass.
template <bool FULL, int SEL>
__device__ __forceinline__ void row_winners(const TreeView& t, const float* __restrict__ rowp, float alpha,
                                            const float* rs, int nch, int lane, int& v0, int& w) {
  LaneBest fb = lane_best_init(), rb = lane_best_init(), gb = lane_best_init();
  float x[2][16];
  load16<FULL>(rowp, 0, t.V, lane, -INFINITY, x[0]);
  for (int ch0 = 0; ch0 < nch; ch0 += 2) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int ch = ch0 + u;
      if (ch < nch) {
        if (ch + 1 < nch) load16<FULL>(rowp, (ch + 1) * kChunk, t.V, lane, -INFINITY, x[(u + 1) % 2]);
        float rw[16];
        read_rs_lds(rs, ch * kChunk, lane, rw);
        wide_chunk<SEL, true>(x[u], rw, ch, 0.0f, alpha, fb, rb, gb);
      }
    }
  }
  w = root_winner<SEL>(t, gb, rowp, alpha, lane);
  v0 = -1;
  if (SEL != 0) {
    float M;
    wave_pick(rb, lane, M, v0);
    v0 = uniform_i(v0);
  }
}

// Boundary guess for wide rows, the scheme of the narrow kernels: (v0, w) are the winners of frame f, the one
// before the boundary; frames that keep the state are skipped going back, up to kLookBack frames or the start
// of the call.  Both neighbours of a boundary compute it from the same rows with the same arithmetic.
template <bool FULL, int SEL>
__device__ __forceinline__ void guess_boundary_wide(const TreeView& t, int v0, int w, const float* __restrict__ rowp,
                                                    int64_t frame_stride, int f, const int32_t* __restrict__ states0,
                                                    int b, float alpha, const float* rs, int nch, int lane, int& state,
                                                    int& label) {
  label = -1;
  for (int k = 0;; ++k) {
    bool keep = false;
    int win = w;
    if (SEL != 0) {
      keep = v0 == t.blank;
      if (keep) win = v0;
    }
    if (!keep) keep = win == t.blank || win == t.eos;
    if (k == 0) label = win;
    if (!keep) {
      state = uniform_i(t.root_next[win]);
      return;
    }
    if (f - k == 0) {  // nothing since the start of the call has moved the state
      const int s0 = uniform_i(states0[b]);
      state = valid_state(t, s0) ? s0 : 0;
      return;
    }
    if (k + 1 >= kLookBack) {
      state = 0;
      return;
    }
    rowp -= frame_stride;
    row_winners<FULL, SEL>(t, rowp, alpha, rs, nch, lane, v0, w);
  }
}

// Decodes frames [f0, f1) of hypothesis b, as run_frames_1k does for narrow rows (same arguments and rules).
//   rs: root scores of the row in LDS, zero-padded to nchp chunks; tags: this wave's token marks (32 * nchp words)
//   nchp: chunks per row rounded up to a whole turn of the ring (chunks past the row load nothing)
template <bool COMPARE, bool FULL, int SEL, bool EDGE>
__device__ __forceinline__ bool run_frames_wide(const TreeView& t, const float* __restrict__ logp, int64_t frame_stride,
                                                int64_t row_stride, float alpha, int B, int b, int f0, int f1, int s_in,
                                                int last_in, int T, const int32_t* __restrict__ states0,
                                                int32_t* __restrict__ tokens, int32_t* __restrict__ states,
                                                float* __restrict__ scores, const float* rs, unsigned* tags, int nchp,
                                                int lane) {
  if (f0 >= f1) return true;
  constexpr bool GUESS = EDGE && !COMPARE;
  const int V = t.V;
  const int nch = (V + kChunk - 1) / kChunk;
  const int tag_words = nchp * kTagWords;
  const float* rp = logp + static_cast<size_t>(b) * row_stride + static_cast<size_t>(f0) * frame_stride;
  // The ring: buffer u holds chunk ch with ch % kRing == u.  A chunk is requested kRing - 1 chunks ahead, into
  // the buffer the chunk before the current one has just left, at the start of a chunk's turn.
  float xb[kRing][16];
#pragma unroll
  for (int u = 0; u + 1 < kRing; ++u) load16<FULL>(rp, u * kChunk, V, lane, -INFINITY, xb[u]);
  StoredLane<SEL == 2> stored;
  if (COMPARE) stored.fetch(lane, f0, f1, B, b, tokens, states);
  int s = uniform_i(s_in);
  int last = -1;
  if (SEL == 2) last = uniform_i(last_in);
  const bool guessable = GUESS && t.num_states < kGuessOk;
  if (guessable && f0 > 0 && s == 0) {  // (an invalid start state, e.g. of an unknown tree, is left as it is)
    int v0, w, label;
    row_winners<FULL, SEL>(t, rp - frame_stride, alpha, rs, nch, lane, v0, w);
    guess_boundary_wide<FULL, SEL>(t, v0, w, rp - frame_stride, frame_stride, f0 - 1, states0, b, alpha, rs, nch, lane,
                                   s, label);
    if (SEL == 2) last = label;
  }
  if (!valid_state(t, s)) {
    fill_invalid(B, b, f0, f1, tokens, states, scores, lane);
    return false;
  }
  Cursor cur = cursor_at(t, s);
  LaneOut out{f0, 0, 0, 0.0f};
  for (int f = f0; f < f1; ++f) {
    if (GUESS) set_wave_priority(min(3, 4 * (f1 - f) / (f1 - f0)));  // (pass 1: the more is left, the higher)
    const bool more = f + 1 < f1;
    const bool track = guessable && !more && f1 < T;  // last frame of the range: also its root-state winner
    // the first arcs of the state, requested before the pass over the row (unconditionally; the index is
    // clamped into the state's arc range, see the narrow kernels)
    const ArcRec early = t.arc[cur.rec.begin + max(0, min(lane, cur.rec.count - 1))];
    LaneBest fb = lane_best_init(), rb = lane_best_init(), gb = lane_best_init();
    const float* rpn = more ? rp + frame_stride : rp;
    float early_x = 0.0f;  // log-prob of the early arc's token: gathered after the first turn of the ring, when the arc is there
    auto pass = [&](auto track_c) {
      constexpr bool TRACK = decltype(track_c)::value;
      auto turn = [&](int g) {  // one turn of the ring: kRing chunks, straight-line code
#pragma unroll
        for (int u = 0; u < kRing; ++u) {
          const int ch = g + u;
          // Request the chunk kRing - 1 ahead, of this row or of the next, without a condition (after the last
          // frame of the range the row in hand is asked for again, from cache): straight-line code lets the
          // compiler wait for exactly the chunk it needs and keep the others in flight.
          const int nx = ch + kRing - 1;
          const bool wrap = nx >= nchp;
          load16<FULL>(wrap ? rpn : rp, (wrap ? nx - nchp : nx) * kChunk, V, lane, -INFINITY, xb[(u + kRing - 1) % kRing]);
          float rw[16];
          read_rs_lds(rs, ch * kChunk, lane, rw);
          wide_chunk<SEL, TRACK>(xb[u], rw, ch, cur.p_root, alpha, fb, rb, gb);
          __builtin_amdgcn_sched_barrier(0);  // (the four turns would otherwise be interleaved and run out of registers)
        }
      };
      turn(0);
      // the early arc is there by now: the log-prob of its token is gathered while the rest of the row streams
      early_x = rp[lane < cur.rec.count ? early.token : 0];
      for (int g = kRing; g < nchp; g += kRing) turn(g);
    };
    if (track) {
      pass(std::integral_constant<bool, true>{});
    } else {
      pass(std::integral_constant<bool, false>{});
    }
    float M;
    int vb;
    wave_pick(fb, lane, M, vb);
    int v0 = -1;
    FrameOut o;
    bool stage1 = false;
    if (SEL != 0) {  // stage 1: selection without boosting; a blank (or a CTC repeat) is emitted as it is
      float M0;
      wave_pick(rb, lane, M0, v0);
      v0 = uniform_i(v0);
      if (v0 == t.blank || (SEL == 2 && v0 == last)) {
        o = FrameOut{uniform_f(M0), v0, false, 0};
        stage1 = true;
      }
    }
    if (!stage1) {
      o = decide_wide<FULL, SEL>(t, cur, rp, alpha, M, uniform_i(vb), early, early_x, last, tags, tag_words, nch, lane);
      advance(t, cur, o, more);
    }
    const int word = cur.s;
    const int slot = f - out.base;
    out.put(lane, f, o.tok, word, o.val);
    if (COMPARE) {
      // met the stored trajectory: this frame is written too (its score may differ), the rest stands
      if (stored.state_at(slot) == word && (SEL != 2 || stored.token_at(slot) == o.tok)) {
        out.template flush<true>(lane, slot + 1, B, b, tokens, states, scores);
        return true;
      }
    }
    if (track) {
      // the guess the next range starts from, made from the same rows; if it is what this range really ends
      // in, the last state word says so
      int g, glabel;
      const int w = root_winner<SEL>(t, gb, rp, alpha, lane);
      guess_boundary_wide<FULL, SEL>(t, v0, w, rp, frame_stride, f, states0, b, alpha, rs, nch, lane, g, glabel);
      if (g == cur.s && (SEL != 2 || glabel == o.tok)) {
        if (lane == slot) out.st |= kGuessOk;
      }
    }
    if (slot == 63 && more) {  // (the last group is written at the end)
      out.template flush<COMPARE>(lane, 64, B, b, tokens, states, scores);
      out.base = f + 1;
      if (COMPARE) stored.fetch(lane, f + 1, f1, B, b, tokens, states);
    }
    if (SEL == 2) last = o.tok;
    rp += frame_stride;
  }
  out.template flush<COMPARE>(lane, f1 - out.base, B, b, tokens, states, scores);
  return false;  // (a re-run: the end of the range was reached without meeting the stored trajectory)
}

// Root scores of a row for the pass over it: zero beyond V, NaN in the blank and EOS columns (those two tokens
// are candidates of their own, see special_candidate).
__device__ __forceinline__ float4 mask_special(const TreeView& t, int i, float4 q) {
  float e[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (i + k == t.blank || i + k == t.eos) e[k] = NAN;
  return make_float4(e[0], e[1], e[2], e[3]);
}
__device__ __forceinline__ float4 staged_root_scores(const TreeView& t, int i) {
  float4 q = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  if (i < t.V) q = *reinterpret_cast<const float4*>(t.root_score + i);  // V % 4 == 0
  return mask_special(t, i, q);
}

// The same into LDS for a whole row, by the whole workgroup; ends with a barrier.
__device__ __forceinline__ void stage_root_scores(const TreeView& t, float* rs, int nchp) {
  const int n = nchp * kChunk;
  for (int i = 4 * static_cast<int>(threadIdx.x); i < n; i += 4 * static_cast<int>(blockDim.x))
    *reinterpret_cast<float4*>(rs + i) = staged_root_scores(t, i);
  __syncthreads();
}

// Pass 1 (see frames_spec_kernel of the narrow rows).  With a table of trees the workgroup's waves may use
// different trees, so each wave then keeps its own copy of the root scores.
template <bool FULL, int SEL, bool FOREST>
__global__ void __launch_bounds__(256, PB_WIDE_WAVES_EU) wide_spec_kernel(DeviceTree dt, TreePick pick, const float* __restrict__ logp,
                                                         int64_t frame_stride, int64_t row_stride,
                                                         const int32_t* __restrict__ states0,
                                                         const int32_t* __restrict__ last0, float alpha, int T, int B,
                                                         int seg_len, int nseg, int nchp, int32_t* __restrict__ tokens,
                                                         int32_t* __restrict__ states, float* __restrict__ scores) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = uniform_i(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
  const int chain = blockIdx.x * nwaves + wave;
  const bool live = chain < B * nseg;
  const int j = live ? chain / B : 0, b = live ? chain - j * B : 0;
  DeviceTree mine = dt;
  bool tree_ok = true;
  if constexpr (FOREST) tree_ok = pick_tree(pick, b, mine);
  const TreeView t = make_view(mine);
  const int row_floats = nchp * kChunk;
  float* rs = lds;
  unsigned* tags;
  if constexpr (FOREST) {
    rs = lds + wave * (row_floats + nchp * kTagWords);
    tags = reinterpret_cast<unsigned*>(rs + row_floats);
    if (tree_ok) {
      for (int i = 4 * lane; i < row_floats; i += 256) *reinterpret_cast<float4*>(rs + i) = staged_root_scores(t, i);
    }
  } else {
    tags = reinterpret_cast<unsigned*>(lds + row_floats) + wave * nchp * kTagWords;
    stage_root_scores(t, rs, nchp);
  }
  if (!live) return;
  const int f0 = seg_begin(j, T, nseg), f1 = seg_begin(j + 1, T, nseg);
  int s = 0, last = -1;
  if (j == 0) {
    s = states0[b];
    if (SEL == 2 && last0 != nullptr) last = last0[b];
  }
  if (!tree_ok) s = -1;  // an unknown tree marks every frame of the hypothesis like an invalid state
  run_frames_wide<false, FULL, SEL, true>(t, logp, frame_stride, row_stride, alpha, B, b, f0, f1, s, last, T, states0,
                                          tokens, states, scores, rs, tags, nchp, lane);
}

// Pass 2: one workgroup per hypothesis (one tree, so the root scores are shared).
template <bool FULL, int SEL, bool FOREST>
__global__ void __launch_bounds__(512) wide_fix_kernel(DeviceTree dt, TreePick pick, const float* __restrict__ logp,
                                                        int64_t frame_stride, int64_t row_stride, float alpha, int T,
                                                        int B, int seg_len, int nseg, int nchp,
                                                        int32_t* __restrict__ tokens, int32_t* __restrict__ states,
                                                        float* __restrict__ scores) {
  extern __shared__ float lds[];
  __shared__ int assumed[64], assumed_tok[64];
  __shared__ unsigned bad_words[2];
  const int lane = threadIdx.x & 63, wave = uniform_i(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
  const int b = blockIdx.x;
  DeviceTree mine = dt;
  if constexpr (FOREST) {
    if (!pick_tree(pick, b, mine)) return;  // pass 1 has marked every frame of this hypothesis (the whole workgroup leaves)
  }
  const TreeView t = make_view(mine);
  float* rs = lds;
  unsigned* tags = reinterpret_cast<unsigned*>(lds + nchp * kChunk) + wave * nchp * kTagWords;
  stage_root_scores(t, rs, nchp);
  fix_segments<SEL == 2>(T, B, b, seg_len, nseg, tokens, states, scores, nullptr, assumed, assumed_tok, bad_words, lane,
                         wave, nwaves,
                         [&](int seg, int s, int last) {
                           const int f0 = seg_begin(seg, T, nseg), f1 = seg_begin(seg + 1, T, nseg);
                           return run_frames_wide<true, FULL, SEL, false>(t, logp, frame_stride, row_stride, alpha, B, b, f0, f1,
                                                                   s, last, T, nullptr, tokens, states, scores, rs, tags,
                                                                   nchp, lane);
                         });
}

// Single step: one workgroup per hypothesis, one chunk per wave, so that the whole row is requested at once.
// The waves' winners meet in LDS; wave 0 evaluates the arcs and decides.
struct StepPart {
  float M, M0;
  int vb, v0;
};

// (The order of the requests is what a single step costs: the root scores, which sit in a cache, and the row go out
// first, with the state id, before anything is waited for.  LEAN: one tree for all rows; the leading arguments,
// the root-score array among them, are then in registers when the wave starts, and an invalid state is decoded as
// the root and marked at the end, so that no early exit stands between the wave start and the requests.)
template <bool FULL, int SEL, bool LEAN>
__global__ void __launch_bounds__(1024) step_wide_kernel(
    const float* __restrict__ logp, int64_t row_stride, const int32_t* __restrict__ states_in,
    const float* __restrict__ root_score, const int32_t* __restrict__ last_in, float alpha, int B,
    int32_t* __restrict__ tokens, int32_t* __restrict__ states_out, float* __restrict__ scores, DeviceTree dt,
    TreePick pick) {
  extern __shared__ float lds[];  // wave 0's token marks
  __shared__ StepPart part[16];
  const int lane = threadIdx.x & 63, wave = uniform_i(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
  const int b = blockIdx.x;
  DeviceTree mine = dt;
  bool tree_ok = true;
  if constexpr (!LEAN) tree_ok = pick_tree(pick, b, mine);
  const TreeView t = make_view(mine);
  const int nch = nwaves;  // launched with one wave per chunk
  const float* rowp = logp + static_cast<size_t>(b) * row_stride;
  const float* rsp = LEAN ? root_score : t.root_score;
  float x[16], rw[16];
  load16<FULL>(rsp, wave * kChunk, t.V, lane, 0.0f, rw);
  load16<FULL>(rowp, wave * kChunk, t.V, lane, -INFINITY, x);
  int s = tree_ok ? states_in[b] : -1;  // an unknown tree marks the hypothesis like an invalid state
  __builtin_amdgcn_sched_barrier(0);
  s = uniform_i(s);
  const bool ok = valid_state(t, s);  // uniform over the workgroup
  if (!LEAN && !ok) {
    if (threadIdx.x == 0) {
      tokens[b] = -1;
      states_out[b] = -1;
      scores[b] = NAN;
    }
    return;
  }
  if (!ok) s = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {  // NaN in the blank and EOS columns: those two are candidates of their own
    const float4 q = mask_special(t, wave * kChunk + 256 * i + 4 * lane,
                                  make_float4(rw[4 * i], rw[4 * i + 1], rw[4 * i + 2], rw[4 * i + 3]));
    rw[4 * i + 0] = q.x; rw[4 * i + 1] = q.y; rw[4 * i + 2] = q.z; rw[4 * i + 3] = q.w;
  }
  Cursor cur;
  ArcRec early = ArcRec{0, 0.0f};
  float p_root;
  if (wave == 0) {
    cur = cursor_at(t, s);
    early = t.arc[cur.rec.begin + max(0, min(lane, cur.rec.count - 1))];
    p_root = cur.p_root;
  } else {
    p_root = t.p_root[s];
  }
  float early_x = 0.0f;  // (wave 0: the log-prob of its early arc's token, requested before the row is looked at)
  if (wave == 0) early_x = rowp[lane < cur.rec.count ? early.token : 0];
  LaneBest fb = lane_best_init(), rb = lane_best_init(), gb = lane_best_init();
  wide_chunk<SEL, false>(x, rw, wave, p_root, alpha, fb, rb, gb);
  StepPart mine_part{0.0f, 0.0f, 0, 0};
  wave_pick(fb, lane, mine_part.M, mine_part.vb);
  if (SEL != 0) wave_pick(rb, lane, mine_part.M0, mine_part.v0);
  if (lane == 0) part[wave] = mine_part;
  __syncthreads();
  if (wave != 0) return;
  // chunks ascend with the wave index, so among equal maxima the lowest wave holds the lowest token
  const bool have = lane < nch;
  const StepPart q = part[have ? lane : 0];
  const float M = ukey_val(wave_max_u(have ? ukey(q.M) : 0u));
  const int vb = __builtin_amdgcn_readlane(q.vb, first_lane(__ballot(have && q.M == M)));
  const int vb_next = t.root_next[vb];  // where the base winner leads, requested before the arcs are evaluated
  int last = -1;
  if (SEL == 2 && last_in != nullptr) last = uniform_i(last_in[b]);
  FrameOut o;
  bool stage1 = false;
  if (SEL != 0) {
    const float M0 = ukey_val(wave_max_u(have ? ukey(q.M0) : 0u));
    const int v0 = __builtin_amdgcn_readlane(q.v0, first_lane(__ballot(have && q.M0 == M0)));
    if (v0 == t.blank || (SEL == 2 && v0 == last)) {
      o = FrameOut{M0, v0, false, 0};
      stage1 = true;
    }
  }
  if (!stage1) {
    unsigned* tags = reinterpret_cast<unsigned*>(lds);
    o = decide_wide<FULL, SEL>(t, cur, rowp, alpha, M, vb, early, early_x, last, tags, nch * kTagWords, nch, lane);
    if (!o.arc && o.tok == vb && vb != t.blank && vb != t.eos) {
      cur.s = uniform_i(vb_next);  // only the state id leaves the kernel
    } else {
      advance(t, cur, o, false);
    }
  }
  if (lane == 0) {
    tokens[b] = ok ? o.tok : -1;
    states_out[b] = ok ? cur.s : -1;
    scores[b] = ok ? o.val : NAN;
  }
}

int g_wide_fix_waves = 8;   // waves per fix-up workgroup the device's LDS allows for the widest row, set once
int g_wide_max_lds = 64 * 1024;

inline int padded_chunks(int V) {
  const int nch = (V + kChunk - 1) / kChunk;
  return (nch + kRing - 1) / kRing * kRing;
}

}  // namespace

// Expands to one launch per (row shape, selection rule) pair; FULL: V a multiple of a whole ring turn of chunks.
#define PB_DISPATCH(full, sel, LAUNCH)   \
  switch ((full ? 0 : 3) + (sel)) {      \
    case 0: LAUNCH(true, 0); break;      \
    case 1: LAUNCH(true, 1); break;      \
    case 2: LAUNCH(true, 2); break;      \
    case 3: LAUNCH(false, 0); break;     \
    case 4: LAUNCH(false, 1); break;     \
    default: LAUNCH(false, 2); break;    \
  }

int launch_step_wide(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t row_stride,
                     const int32_t* d_states_in, const int32_t* d_last, float alpha, int32_t B, int sel,
                     int32_t* d_tokens, int32_t* d_states_out, float* d_scores, hipStream_t stream) {
  const int V = t.vocab_size;
  const int nch = (V + kChunk - 1) / kChunk;  // <= 16 (kWideMaxV)
  const bool full = V % kChunk == 0;
  const size_t lds = static_cast<size_t>(nch) * kTagWords * sizeof(unsigned);
  const dim3 grid(static_cast<unsigned>(B)), block(static_cast<unsigned>(64 * nch));
  const bool lean = pick.table == nullptr;
#define PB_STEP(FULL, SEL, LEAN)                                                                                   \
  hipLaunchKernelGGL((step_wide_kernel<FULL, SEL, LEAN>), grid, block, lds, stream, d_logp, row_stride,            \
                     d_states_in, t.root_score, d_last, alpha, B, d_tokens, d_states_out, d_scores, t, pick)
#define PB_LAUNCH(FULL, SEL)   \
  if (lean) {                  \
    PB_STEP(FULL, SEL, true);  \
  } else {                     \
    PB_STEP(FULL, SEL, false); \
  }
  PB_DISPATCH(full, sel, PB_LAUNCH)
#undef PB_LAUNCH
#undef PB_STEP
  return hipGetLastError() == hipSuccess ? PB_OK : PB_EHIP;
}

int launch_frames_wide(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t frame_stride,
                       int64_t row_stride, const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T,
                       int32_t B, int sel, int32_t* d_tokens, int32_t* d_states, float* d_scores, hipStream_t stream) {
  const int V = t.vocab_size;
  const int nchp = padded_chunks(V);
  const bool full = V % (kRing * kChunk) == 0;
  const bool forest = pick.table != nullptr;
  const size_t row_bytes = static_cast<size_t>(nchp) * kChunk * sizeof(float);
  const size_t tag_bytes = static_cast<size_t>(nchp) * kTagWords * sizeof(unsigned);
  // pass 1: four waves per workgroup share the root scores (a forest: one copy per wave, fewer waves if LDS is short)
  int waves = 4;
  size_t lds = row_bytes + waves * tag_bytes;
  if (forest) {
    while (waves > 1 && waves * (row_bytes + tag_bytes) > static_cast<size_t>(g_wide_max_lds)) waves /= 2;
    lds = waves * (row_bytes + tag_bytes);
  }
  if (lds > static_cast<size_t>(g_wide_max_lds)) return PB_EUNSUPPORTED;
  const SegPlan plan = plan_segments(T, B, kWideTargetChains);
  const int nseg = plan.nseg, seg_len = plan.seg_len;
  const int64_t chains = static_cast<int64_t>(B) * nseg;
  const int64_t blocks = (chains + waves - 1) / waves;
  if (blocks > INT32_MAX) return PB_EUNSUPPORTED;
#define PB_SPEC(FULL, SEL, FOREST)                                                                                 \
  hipLaunchKernelGGL((wide_spec_kernel<FULL, SEL, FOREST>), dim3(static_cast<unsigned>(blocks)), dim3(64 * waves), \
                     lds, stream, t, pick, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B,      \
                     seg_len, nseg, nchp, d_tokens, d_states, d_scores)
#define PB_LAUNCH(FULL, SEL) PB_SPEC(FULL, SEL, false)
#define PB_LAUNCH_F(FULL, SEL) PB_SPEC(FULL, SEL, true)
  if (forest) {
    PB_DISPATCH(full, sel, PB_LAUNCH_F)
  } else {
    PB_DISPATCH(full, sel, PB_LAUNCH)
  }
#undef PB_LAUNCH
#undef PB_LAUNCH_F
#undef PB_SPEC
  if (hipGetLastError() != hipSuccess) return PB_EHIP;
  if (nseg > 1) {
    int fw = nseg - 1 < g_wide_fix_waves ? nseg - 1 : g_wide_fix_waves;
    while (fw > 1 && row_bytes + fw * tag_bytes > static_cast<size_t>(g_wide_max_lds)) --fw;
    const size_t lds2 = row_bytes + fw * tag_bytes;
    if (lds2 > static_cast<size_t>(g_wide_max_lds)) return PB_EUNSUPPORTED;
#define PB_FIX(FULL, SEL, FOREST)                                                                                   \
  hipLaunchKernelGGL((wide_fix_kernel<FULL, SEL, FOREST>), dim3(static_cast<unsigned>(B)), dim3(64 * fw), lds2,     \
                     stream, t, pick, d_logp, frame_stride, row_stride, alpha, T, B, seg_len, nseg, nchp, d_tokens, \
                     d_states, d_scores)
#define PB_LAUNCH(FULL, SEL) PB_FIX(FULL, SEL, false)
#define PB_LAUNCH_F(FULL, SEL) PB_FIX(FULL, SEL, true)
    if (forest) {
      PB_DISPATCH(full, sel, PB_LAUNCH_F)
    } else {
      PB_DISPATCH(full, sel, PB_LAUNCH)
    }
#undef PB_LAUNCH
#undef PB_LAUNCH_F
#undef PB_FIX
    if (hipGetLastError() != hipSuccess) return PB_EHIP;
  }
  return PB_OK;
}

int prepare_wide_kernels(int max_lds_bytes) {
  // The widest row needs 64 KiB of root scores plus the waves' token marks: past 64 KiB of dynamic LDS the
  // limit of each kernel must be raised.
  constexpr int kPlainLimit = 64 * 1024 - 1024;  // static LDS of the kernels included
  const int want = (padded_chunks(kWideMaxV) * kChunk + 8 * padded_chunks(kWideMaxV) * kTagWords) * 4 + 1024;
  int limit = kPlainLimit;
  if (max_lds_bytes > kPlainLimit) {
    const int bytes = (want < max_lds_bytes ? want : max_lds_bytes) - 1024;
    const hipFuncAttribute attr = hipFuncAttributeMaxDynamicSharedMemorySize;
    bool ok = true;
#define PB_SET(FULL, SEL)                                                                                               \
  ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(wide_fix_kernel<FULL, SEL, false>), attr, bytes) == hipSuccess && \
       hipFuncSetAttribute(reinterpret_cast<const void*>(wide_fix_kernel<FULL, SEL, true>), attr, bytes) == hipSuccess &&        \
       hipFuncSetAttribute(reinterpret_cast<const void*>(wide_spec_kernel<FULL, SEL, false>), attr, bytes) == hipSuccess &&      \
       hipFuncSetAttribute(reinterpret_cast<const void*>(wide_spec_kernel<FULL, SEL, true>), attr, bytes) == hipSuccess
    for (int ms = 0; ms < 6; ++ms) PB_DISPATCH(ms < 3, ms % 3, PB_SET)
#undef PB_SET
    if (ok) {
      limit = bytes;
    } else {
      (void)hipGetLastError();
    }
  }
  g_wide_max_lds = limit;
  g_wide_fix_waves = 8;
  return PB_OK;
}

}  // namespace pb
