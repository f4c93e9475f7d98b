// Wave-per-hypothesis kernels (gfx950, wave64): the fused greedy step with its selection rules, the
// multi-frame decoder and the beam step for rows of up to 1024 tokens.
//
// One wavefront owns one hypothesis row; nothing crosses waves, so there is no barrier on the path.
//
//  * Row streaming.  A row is consumed in chunks of 1024 tokens; lane l owns tokens
//    256*i + 4*l + {0..3}, i = 0..3 of a chunk, so each of the four 16-byte loads of a lane is part
//    of one contiguous 1 KiB wave access.  Rows travel through a ring of register buffers, requested
//    one or two frames ahead.  Vector loads retire in order, so the first 64 arcs of the state are
//    requested before the row prefetch of the frame: a wait for them then leaves the prefetch in flight.
//  * Base candidates.  For every token that no chain state overrides the boost is
//    p_root + root_score[v] (all backoffs down to the root, then the root arc or the c_unk
//    self-loop).  alpha * that is cached per lane while p_root does not change, so the common
//    frame costs one add and a max per token.  The row max is reduced with DPP on order-preserving
//    unsigned keys; the winner is the lowest token index holding that value (fp32 compare), found
//    with ballots over the four 256-token groups.
//  * Arc candidates.  The failure chain is walked with scalar loads (the state is wave-uniform);
//    at each chain state the lanes take one arc each, gather its log-prob from the LDS copy of the
//    row and evaluate Eq. 1 for it.  In a chain with more than one state an evaluated arc leaves a NaN
//    in its token's entry of that copy (the CTC rule: a mark in an LDS bit set), so that an arc shadowed
//    by a deeper chain state is skipped.  If the base winner is itself an
//    overridden token and the arcs do not beat it, a second pass recomputes the base winner
//    without the overridden tokens.
//  * The record of the next state (arc range, failure link, backoffs) is fetched with the lookup
//    that yields the state: a dense per-token table holds it for the base winner and is read as
//    soon as that winner is known, before the arcs have been evaluated.
//  * Multi-frame decoding splits the T frames of a hypothesis into segments decoded concurrently.  A
//    segment that does not begin the call starts from a guess: the state the base winner of the frame
//    before it leads to (right in most frames).  The decoder is a finite automaton step, so a re-run
//    from the true start state needs to go only as far as the frame where it meets the stored
//    trajectory.  The segment on the left certifies a right guess with a bit in its last state word;
//    a second kernel re-runs the other segments (in parallel, from the neighbouring segment's end
//    state), then compares the assumed start states with the final ones, re-running stale segments in
//    parallel rounds, and clears the bits.  With a workspace the segment on the left repairs a wrong guess
//    itself (it decodes on until it meets what the segment on the right has left of its first frames) and
//    the second kernel only copies the repaired frames.  The result is identical to T sequential steps.
//  * Selection rules (Sec. II-C).  The two-stage rules first take the arg-max of the raw row; a blank
//    (or, for CTC, a repeat of the previous label) ends the frame there.  Tokens barred from the
//    boosted re-selection are NaN in the candidate registers, which no maximum and no equality test
//    ever selects.
#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <climits>
#include <cmath>
#include <cstdint>
#include <random>
#include <type_traits>

#include "pb_kernels.hpp"
#include "pb_wave.hpp"

namespace pb {

namespace {

using namespace wv;

#ifdef PB_STATS  // development build: counters of the fix-up pass (re-runs, frames re-run, re-runs that reached their end)
__device__ unsigned long long g_stats[8];
#define PB_STAT(i, v) do { if (lane == 0) atomicAdd(&g_stats[i], static_cast<unsigned long long>(v)); } while (0)
#else
#define PB_STAT(i, v) do { } while (0)
#endif

// ------------------------------------------------------------------------------------------------
// Base boosts of a row with V <= 1024 for the lane's 16 tokens; the root scores come from memory
// (cache-resident) because they are needed only when the accumulated backoff of the state changes.
template <bool FULL, int SEL>
__device__ __forceinline__ void rebuild_base_boost(const TreeView& t, int lane, float p_root, float alpha,
                                                   float (&c)[16]) {
  const int ln = opaque(lane);
  float rw[16];
  load16<FULL>(t.root_score, 0, t.V, ln, 0.0f, rw);
  make_base_boost<SEL>(0, ln, t.blank, p_root, alpha, rw, c);
}

// One frame of a row with V <= 1024 (a single chunk).  `cur` is the hypothesis' state with its
// record; on return it is the state after the chosen token.  Returns the token and fused value.
//   x     lane's raw log-probs (registers); `next_row()` requests a later frame's row into other
//         registers
//   c / c_p  cached base boosts and the p_root they are for
//   row / tags  this wave's LDS copy of the row and its token marks
//   last  label of the previous frame (SEL == 2 only; any value outside [0, V) = none)
//   need_record  false when no frame follows: the record of the next state is then not fetched
template <bool FULL, int SEL, int EARLY, int EARLY1, int GROUP, typename NextRow>
__device__ __forceinline__ void frame_1k(const TreeView& t, Cursor& cur, const float (&x)[16], float (&c)[16],
                                         float& c_p, float alpha, float* row, unsigned* tags, int lane, int last,
                                         bool need_record, NextRow&& next_row, float& out_val, int& out_tok,
                                         bool& row_in_lds) {
  const int s = cur.s;
  const Rec rec0 = cur.rec;
  const bool chain = (s != 0);
  const bool multi = chain && rec0.fail != 0;
  // Vector loads retire in order, so a wait for arcs also waits for every row requested before them.
  // The first arcs of the state are therefore requested first and the row prefetch right after:
  // the wait for these arcs leaves the prefetch in flight.
  // (Requested without a condition, so that no merge of control flow forces an early wait: for a state
  // without arcs, or the last state of the table, the clamped index reads the entry at arc_begin, which
  // lies inside the tree's allocation -- the arc table is followed by the dense root row -- and is
  // never used.)
  constexpr int kEarly = EARLY;  // batches of 64 arcs requested up front
  ArcRec early[kEarly];
#pragma unroll
  for (int q = 0; q < kEarly; ++q) early[q] = t.arc[rec0.begin + max(0, min(64 * q + lane, rec0.count - 1))];
  // The cursor also holds the record of the second chain state (often a depth-1 state with hundreds of arcs):
  // its first arcs are requested here as well, when there is such a state.
  constexpr int kEarly1 = EARLY1;
  const Rec rec1 = cur.rec1;
  ArcRec early1[kEarly1 > 0 ? kEarly1 : 1];
  if (multi) {
#pragma unroll
    for (int q = 0; q < kEarly1; ++q) early1[q] = t.arc[rec1.begin + max(0, min(64 * q + lane, rec1.count - 1))];
  }
  next_row();
  if constexpr (SEL != 0) {
    // stage 1: selection without boosting; a blank (or a CTC repeat) is emitted as it is
    float M0;
    int v0;
    plain_argmax(x, lane, M0, v0);
    if (v0 == t.blank || (SEL == 2 && v0 == last)) {
      out_val = uniform_f(M0);
      out_tok = uniform_i(v0);
      row_in_lds = false;
      return;
    }
  }
  if (__float_as_int(c_p) != __float_as_int(cur.p_root)) {
    rebuild_base_boost<FULL, SEL>(t, lane, cur.p_root, alpha, c);
    c_p = cur.p_root;
  }
  float f[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) f[j] = __fadd_rn(x[j], c[j]);
  if (t.eos >= 0) {  // EOS rule (Sec. II-C): the EOS token is boosted by the value tabulated for the state
    const float ce = __fmul_rn(alpha, cur.eos_boost);
    const int ln = opaque(lane);
#pragma unroll
    for (int j = 0; j < 16; ++j) f[j] = slot_is(j, ln, t.eos) ? __fadd_rn(x[j], ce) : f[j];
  }
  if (chain) store_row_lds(row, lane, x);
  constexpr bool MARK_IN_ROW = SEL != 2;  // how an arc finds its token claimed by a deeper chain state, see below
  row_in_lds = chain && !(MARK_IN_ROW && multi);  // (such a chain leaves marks in the copy)
  const Cursor start = cur;
  // The CTC rule bars the previous label from the re-selection.  The frame is first decided with the
  // label still in; only if it wins is the frame decided again with the label excluded (excl >= 0).
  for (int excl = -1;;) {
    // ---- early load: records of the third and fourth chain state -----------------------------------
    Rec2 nn{rec1, rec1};
    if (multi && rec1.fail != 0) nn = load_rec2(t, rec1.fail);

    // ---- base candidates -------------------------------------------------------------------------
    float g[4];
    if (SEL == 2 && excl >= 0) {
#pragma unroll
      for (int j = 0; j < 16; ++j) f[j] = slot_is(j, opaque(lane), excl) ? NAN : f[j];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) g[i] = max4(f[4 * i], f[4 * i + 1], f[4 * i + 2], f[4 * i + 3]);
    const float M = ukey_val(wave_max_u(ukey(max4(g[0], g[1], g[2], g[3]))));
    const int vb = first_token_equal(f, g, M, lane);
    const v8i rr = t.root_rec[vb];  // record of the state the base winner leads to (speculative)

    // ---- arc candidates along the failure chain --------------------------------------------------
    float bf = -INFINITY;
    int btok = INT_MAX, bchild = 0;
    bool hit_vb = false;
    if (chain) {
      // One arc per lane: `a` with its child state, on chain level `level` with accumulated backoff p.  A chain
      // of several states is walked deepest state first, and an arc whose token a deeper state has already
      // claimed must be skipped: every arc that is evaluated replaces its token's entry in the LDS copy of the
      // row by a NaN, so a later arc on the same token computes a NaN, which no comparison selects.  (The
      // tokens of one state are distinct, and LDS accesses of a wave complete in order.)  The CTC rule may decide
      // a frame twice and would need the row again for that, which the registers of its kernels do not hold:
      // it marks the claimed tokens in a bit set beside the row instead (one more LDS round trip per batch).
      if (!MARK_IN_ROW && multi) tags_clear(tags, lane);
      auto eval = [&](const ArcRec& a, bool valid, int child, float p, int level) {
        const int tk = valid ? a.token : 0;  // an unused entry may hold anything: keep the LDS index in range
        bool shadowed = !valid;
        if (SEL == 2) shadowed = shadowed || tk == excl;
        if (!MARK_IN_ROW && multi) {
          if (level > 0) shadowed = shadowed || tag_test(tags, tk);
          if (valid) tag_set(tags, tk);
        }
        const float lp = row[tk];
        if (MARK_IN_ROW && multi && valid) row[tk] = NAN;
        hit_vb = hit_vb || (valid && tk == vb);
        const float fa = __fadd_rn(lp, __fmul_rn(alpha, __fadd_rn(p, a.score)));
        const bool take = !shadowed & ((fa > bf) | ((fa == bf) & (tk < btok)));  // (no short-circuit: no branches)
        bf = take ? fa : bf;
        btok = take ? tk : btok;
        bchild = take ? child : bchild;
      };
      Rec r = rec0;
      float p = 0.0f;
      // The first arcs of the chain head were requested at the start of the frame.  They are used
      // here, outside the loop, so that the wait for them is a wait for them alone: inside the loop
      // the compiler could not tell them from the arcs loaded there and would wait for every load in
      // flight, the prefetched rows included.
#pragma unroll
      for (int q = 0; q < kEarly; ++q) {
        if (q == 0 || 64 * q < r.count)
          eval(early[q], 64 * q + lane < r.count, r.begin + max(0, min(64 * q + lane, r.count - 1)) + 1, p, 0);
      }
      for (int level = 0;; ++level) {
        int first = 0;  // arcs of this level already requested at the start of the frame
        if (level == 0) first = 64 * kEarly;
        if (level == 1) {
          first = 64 * kEarly1;
#pragma unroll
          for (int q = 0; q < kEarly1; ++q) {
            if (q == 0 || 64 * q < r.count)
              eval(early1[q], 64 * q + lane < r.count, r.begin + max(0, min(64 * q + lane, r.count - 1)) + 1, p, 1);
          }
        }
        // Further arcs, up to four batches at a time so that their latencies overlap.  Every lane loads (the
        // index is clamped into the row) so that the load and its use stay in one block; lanes past the
        // end of the row are discarded by `valid`.
        constexpr int kGroup = GROUP;
        for (int j0 = first; j0 < r.count; j0 += 64 * kGroup) {
          ArcRec more[kGroup];
#pragma unroll
          for (int q = 0; q < kGroup; ++q) more[q] = t.arc[r.begin + min(j0 + 64 * q + lane, r.count - 1)];
#pragma unroll
          for (int q = 0; q < kGroup; ++q) {
            if (q == 0 || j0 + 64 * q < r.count)
              eval(more[q], j0 + 64 * q + lane < r.count, r.begin + min(j0 + 64 * q + lane, r.count - 1) + 1, p, level);
          }
        }
        p = __fadd_rn(p, r.backoff);
        if (r.fail == 0) break;
        // one load serves two chain states: the cursor the first two, `nn` the next two, and so on
        if (level == 0) {
          r = rec1;
        } else if ((level & 1) != 0) {
          r = nn.a;
        } else {
          r = nn.b;
          if (r.fail != 0) nn = load_rec2(t, r.fail);
        }
      }
    }

    // ---- decision --------------------------------------------------------------------------------
    bool arc_wins = false;
    int va = INT_MAX, achild = 0;
    float MA = 0.0f;
    float base_val = M;
    int base_tok = vb;
    const bool mine0 = btok != INT_MAX;
    // Most frames end here: the best arc stays below the base winner and does not shadow it.
    bool contest = false;
    bool vb_overridden = false;
    if (__ballot(mine0) != 0) {
      MA = ukey_val(wave_max_u(mine0 ? ukey(bf) : 0u));
      vb_overridden = __ballot(hit_vb) != 0;
      contest = vb_overridden || MA >= M;
    }
    if (contest) {
      const bool mine = mine0 && bf == MA;
      const u64 eq = __ballot(mine);
      if ((eq & (eq - 1)) == 0) {  // one lane holds the maximum
        const int L = first_lane(eq);
        va = __builtin_amdgcn_readlane(btok, L);
        achild = __builtin_amdgcn_readlane(bchild, L);
      } else {
        va = wave_min_nn(mine ? btok : INT_MAX);
        achild = __builtin_amdgcn_readlane(bchild, first_lane(__ballot(mine && btok == va)));
      }
      if (MA > M) {
        arc_wins = true;
      } else if (!vb_overridden) {
        arc_wins = (MA == M) && (va < vb);
      } else {
        // The base winner is shadowed by an arc that does not beat it: mark every overridden token and
        // redo the base arg-max without them (and without the excluded ones, which hold NaN).
        tags_clear(tags, lane);
        for (int xs = s; xs != 0;) {
          const Rec r = load_rec(t, xs);
          for (int j = lane; j < r.count; j += 64) tag_set(tags, t.arc[r.begin + j].token);
          xs = uniform_i(r.fail);
        }
        const int ln = opaque(lane);
        unsigned k[16], mk = 0u;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const bool out = tag_test(tags, tok_of(j, ln)) || (SEL != 0 && f[j] != f[j]);
          k[j] = out ? 0u : ukey(f[j]);
          mk = max(mk, k[j]);
        }
        const unsigned Mk = wave_max_u(mk);
        bool have_base = Mk != 0u;
        if (have_base) {
          base_val = ukey_val(Mk);
          int l2 = INT_MAX;
#pragma unroll
          for (int j = 15; j >= 0; --j) l2 = (k[j] != 0u && f[j] == base_val) ? tok_of(j, ln) : l2;
          base_tok = wave_min_nn(l2);
          have_base = base_tok != INT_MAX;
        }
        arc_wins = !have_base || MA > base_val || (MA == base_val && va < base_tok);
      }
    }
    if (arc_wins) {
      out_val = MA;
      out_tok = va;
      if (need_record) {
        cur = cursor_at(t, achild);
      } else {  // last frame of the call: only the state id leaves the kernel
        cur.s = achild;
      }
    } else {
      out_val = base_val;
      out_tok = base_tok;
      if (base_tok != t.blank && base_tok != t.eos) {  // the blank and the EOS keep the state
        if (base_tok == vb) {
          cur = cursor_from_root_rec(rr);
        } else {
          const v8i r2 = t.root_rec[base_tok];
          cur = cursor_from_root_rec(r2);
        }
      }
    }
    out_tok = uniform_i(out_tok);
    if (SEL != 2 || excl >= 0 || out_tok != last) break;
    excl = last;  // the previous label won the re-selection: decide again without it
    cur = start;
  }
  cur.s = uniform_i(cur.s);
  cur.rec.begin = uniform_i(cur.rec.begin);
  cur.rec.count = uniform_i(cur.rec.count);
  cur.rec.fail = uniform_i(cur.rec.fail);
  cur.rec.backoff = uniform_f(cur.rec.backoff);
  cur.rec1.begin = uniform_i(cur.rec1.begin);
  cur.rec1.count = uniform_i(cur.rec1.count);
  cur.rec1.fail = uniform_i(cur.rec1.fail);
  cur.rec1.backoff = uniform_f(cur.rec1.backoff);
  cur.p_root = uniform_f(cur.p_root);
  cur.eos_boost = uniform_f(cur.eos_boost);
  out_val = uniform_f(out_val);
}

// Boundary guess of the multi-frame decoder for rows of up to 1024 tokens: the state (and label) assumed after
// frame f, from the rows alone.  Going back from frame f, a frame whose winner under root-state boosts keeps the
// state (the blank; under the two-stage rules a blank raw arg-max) is skipped; the first frame that moves the
// state gives root_next[its winner] -- what the true decode does in most frames.  Reaching the first frame of
// the call gives the call's start state, kLookBack skipped frames give the root.  The label is the winner of
// frame f itself.  Both neighbours of a boundary call this with the same rows and get the same answer.
//   x: row of frame f (registers, overwritten), rp: its address, c0: root-state base boosts of the rule.
template <bool FULL, int SEL>
__device__ __forceinline__ void guess_boundary_1k(const TreeView& t, float (&x)[16], const float* rp,
                                                  int64_t frame_stride, int f, const int32_t* __restrict__ states0,
                                                  int b, const float (&c0)[16], int lane, int& state, int& label) {
  label = -1;
  for (int k = 0;; ++k) {
    bool keep = false;
    int w = 0;
    if constexpr (SEL != 0) {
      float M0;
      plain_argmax(x, lane, M0, w);
      w = uniform_i(w);
      keep = w == t.blank;
    }
    if (!keep) {
      float fz[16], g[4];
#pragma unroll
      for (int j = 0; j < 16; ++j) fz[j] = __fadd_rn(x[j], c0[j]);
#pragma unroll
      for (int i = 0; i < 4; ++i) g[i] = max4(fz[4 * i], fz[4 * i + 1], fz[4 * i + 2], fz[4 * i + 3]);
      const float M = ukey_val(wave_max_u(ukey(max4(g[0], g[1], g[2], g[3]))));
      w = uniform_i(first_token_equal(fz, g, M, lane));
      keep = w == t.blank || w == t.eos;
    }
    if (k == 0) label = w;
    if (!keep) {
      state = uniform_i(t.root_next[w]);
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
    rp -= frame_stride;
    load16<FULL>(rp, 0, t.V, lane, -INFINITY, x);
  }
}

// A wrong boundary guess, repaired where it is found.  The range that ends here decodes on from its real outcome
// (state sA, label lastA) over the frames that follow, at most n_max of them, until it agrees on state and label
// with the trajectory the guess has led to -- from there on what the next range wrote is right.  That trajectory
// is read from the start record the next range leaves as it goes (`start_rec`, its tag in tag_lo / tag_hi; see
// kStartInts), so only one track is decoded.  The frames decoded up to the meeting point go to `patch` (entry i
// in lane i) and their number is returned; 0 if the two have not met within n_max frames or a frame of the record
// is not there (looked at twice): the boundary then stays uncertified and pass 2 decodes the next range again.
// rp: row of the first frame after the range.  Uses the caller's cache of base boosts (c for c_p, left in an
// unspecified state; the caller's cursor is not used: after the last frame of a range it holds the state id only).
template <bool FULL, int SEL>
__device__ __forceinline__ int run_on_1k(const TreeView& t, const float* __restrict__ rp, int64_t frame_stride,
                                         float alpha, int sA, float (&c)[16], float& c_p, int lastA, int n_max,
                                         int32_t* __restrict__ patch, float* row, unsigned* tags, int lane,
                                         const int32_t* start_rec, unsigned tag_lo) {
  if (n_max <= 0 || start_rec == nullptr) return 0;
  const unsigned tag_hi = start_tag_hi(tag_lo);
  const int V = t.V;
  float x[16], xn[16];
  load16<FULL>(rp, 0, V, lane, -INFINITY, x);  // (requested before the record is waited for)
  Cursor ca = cursor_at(t, sA);
  int b_st = 0, b_tok = 0;  // lane i: state and token of the guessed trajectory after frame i
  const bool b_mine = read_start_frame(start_rec, min(lane, kPatchMax - 1), tag_lo, tag_hi, b_st, b_tok);
  u64 there = __ballot(b_mine);
  int e_tok = 0, e_st = 0;
  float e_sc = 0.0f;
  for (int i = 0; i < n_max; ++i) {
    float valA;
    int tokA;
    bool in_lds;
    const float* rpn = rp + static_cast<int64_t>(min(i + 1, n_max - 1)) * frame_stride;  // (the last frame asks for its own row again)
    frame_1k<FULL, SEL, 1, 1, 4>(t, ca, x, c, c_p, alpha, row, tags, lane, lastA, true,
                                 [&]() { load16<FULL>(rpn, 0, V, lane, -INFINITY, xn); }, valA, tokA, in_lds);
    if (((there >> i) & 1ull) == 0) {  // not there when first looked at: look once more
      int st1, tok1;
      const bool now = read_start_frame(start_rec, i, tag_lo, tag_hi, st1, tok1);
      st1 = uniform_i(st1);  // (every lane has read the same two words)
      tok1 = uniform_i(tok1);
      if (uniform_i(now ? 1 : 0) == 0) return 0;
      if (lane == i) {
        b_st = st1;
        b_tok = tok1;
      }
    }
    const int stB = plain_state(__builtin_amdgcn_readlane(b_st, i)), tokB = __builtin_amdgcn_readlane(b_tok, i);
    if (lane == i) {
      e_tok = tokA;
      e_st = ca.s;
      e_sc = valA;
    }
    lastA = tokA;
    if (ca.s == stB && (SEL != 2 || tokA == tokB)) {
      if (lane <= i) {
        patch[4 + lane] = e_tok;
        patch[4 + kPatchMax + lane] = e_st;
        patch[4 + 2 * kPatchMax + lane] = __float_as_int(e_sc);
      }
      return i + 1;
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = xn[j];
  }
  return 0;
}

// Decodes frames [f0, f1) of hypothesis b (V <= 1024) starting in state s_in with previous label
// last_in (values that may still be in flight from a load: they are first looked at after the row
// loads have been issued; an invalid state marks the frames).  With COMPARE set, stops after the
// first frame whose outcome equals the one already stored -- the out-state in `states` and, under
// the CTC rule where the label feeds the next frame, the token in `tokens` (the stored trajectory is
// then valid from there on).
//   Rows travel through a ring of three register buffers: the frame in hand and the two after it.
//   EDGE (pass 1 of the multi-frame decoder): the range starts from a guess when it does not begin the call
//   (f0 > 0) and marks its last state word when its own guess for the next range (f1 < T) turns out right -- or,
//   given a patch record (`patch`, with `next_len` the length of the next range), when it has repaired a wrong
//   guess itself.
template <bool COMPARE, bool FULL, int SEL, bool EDGE>
__device__ __forceinline__ bool run_frames_1k(const TreeView& t, const float* __restrict__ logp, int64_t frame_stride,
                                              int64_t row_stride, float alpha, int B, int b, int f0, int f1, int s_in,
                                              int last_in, int T, const int32_t* __restrict__ states0,
                                              int32_t* __restrict__ patch, int next_len,
                                              int32_t* __restrict__ tokens, int32_t* __restrict__ states,
                                              float* __restrict__ scores, float* row, unsigned* tags, int lane,
                                              int32_t* start_rec = nullptr, unsigned tag_lo = 0u) {
  if (f0 >= f1) return true;
  constexpr bool GUESS = EDGE && !COMPARE;
  const int V = t.V;
  const float* rp = logp + static_cast<size_t>(b) * row_stride + static_cast<size_t>(f0) * frame_stride;
#ifndef PB_RING_FUSED
#define PB_RING_FUSED 3
#endif
  constexpr int NB = (COMPARE || SEL != 0) ? 3 : PB_RING_FUSED;  // ring size
  // Batches of 64 arcs requested at the start of a frame: 256 arcs cover all but a few states; the two-stage
  // rules hold more state in registers and take half of that, a re-run (16 waves per workgroup) one batch.
  constexpr int kEarlyBatches = COMPARE ? 1 : (SEL == 0 ? 4 : 2);
  // ... of the second chain state, and batches per round of what remains of a long arc row (a re-run has the
  // registers for eight: its frames are mostly deep states, whose chains end in such rows)
  constexpr int kEarlyBatches1 = COMPARE ? 4 : (SEL == 0 ? 4 : (SEL == 1 ? 2 : 0));
  constexpr int kArcGroup = COMPARE ? 8 : 4;
  float xb[NB][16], c[16];
  load16<FULL>(rp, 0, V, lane, -INFINITY, xb[0]);
  if (f0 + 1 < f1) load16<FULL>(rp + frame_stride, 0, V, lane, -INFINITY, xb[1]);
  if (NB > 3 && f0 + 2 < f1) load16<FULL>(rp + 2 * frame_stride, 0, V, lane, -INFINITY, xb[2]);
  load16<FULL>(t.root_score, 0, V, lane, 0.0f, c);  // needs no state: requested before the state is looked at
  StoredLane<SEL == 2> stored;
  if (COMPARE) stored.fetch(lane, f0, f1, B, b, tokens, states);
  int s = uniform_i(s_in);
  int last = -1;
  if (SEL == 2) last = uniform_i(last_in);
  const bool guessable = GUESS && t.num_states < kGuessOk;
  if (guessable && f0 > 0 && s == 0) {  // (an invalid start state, e.g. of an unknown tree, is left as it is)
    float xw[16], c0[16];
    load16<FULL>(rp - frame_stride, 0, V, lane, -INFINITY, xw);
    make_base_boost<SEL>(0, lane, t.blank, 0.0f, alpha, c, c0);
    int label;
    guess_boundary_1k<FULL, SEL>(t, xw, rp - frame_stride, frame_stride, f0 - 1, states0, b, c0, lane, s, label);
    if (SEL == 2) last = label;
  }
  if (!valid_state(t, s)) {
    fill_invalid(B, b, f0, f1, tokens, states, scores, lane);
    if (GUESS && patch != nullptr && lane == 0) patch[0] = 0;
    return false;
  }
  Cursor cur = cursor_at(t, s);
  float c_p = cur.p_root;
  make_base_boost<SEL>(0, lane, t.blank, c_p, alpha, c, c);  // element-wise, in place
  // Outputs: those of up to 64 consecutive frames are kept in the lanes and written together, so that no store
  // sits in the in-order queue of the loads (measured on the two-stage rules: pass 1 of config 3 109 -> 102 us).
  LaneOut out{f0, 0, 0, 0.0f};
  // (the repair of a boundary looks at up to kPatchMax frames of the range behind it, never at its last one)
  // `start_rec`: the start record of the boundary behind this range (read by its repair); the record of the
  // boundary before it, which this range fills, lies B records earlier.
  const int pub_frame = (GUESS && start_rec != nullptr && f0 > 0 && f1 - f0 >= 2) ? f0 + min(kPatchMax, f1 - f0 - 1) - 1 : -1;
  bool row_in_lds = false;  // the LDS row holds the raw row of the frame decoded last
  // One frame with its row in ring slot U.  STEADY frames request the row NB-1 frames ahead without a
  // condition (the last frames of the range ask for the last row again): only then can the compiler
  // count the loads issued after the arcs and after the current row, and wait for exactly those instead of
  // for everything in flight.  Returns true when a re-run has met the stored trajectory.
  auto do_frame = [&](auto slot_c, auto steady_c, int f) -> bool {
    constexpr int U = decltype(slot_c)::value;
    constexpr bool STEADY = decltype(steady_c)::value;
    const int ahead = min(f + NB - 1, f1 - 1) - f;  // frames between this one and the row requested now
    const float* rpn = rp + static_cast<int64_t>(ahead) * frame_stride;
    const bool more = f + NB - 1 < f1;
    float val;
    int tok;
    frame_1k<FULL, SEL, kEarlyBatches, kEarlyBatches1, kArcGroup>(t, cur, xb[U], c, c_p, alpha, row, tags, lane, last, f + 1 < f1,
                        [&]() {
                          if (STEADY || more) load16<FULL>(rpn, 0, V, lane, -INFINITY, xb[(U + NB - 1) % NB]);
                        },
                        val, tok, row_in_lds);
    const int word = cur.s;
    const int slot = f - out.base;
    out.put(lane, f, tok, word, val);
    // The first frames of the range, for whoever repairs the boundary before it.  A store sits in the in-order
    // queue of the loads, so they go out in two groups: frames 0-5 (a range that is slow there, in deep states,
    // would otherwise have nothing to show when its neighbour asks) and the rest.
    if (GUESS && f <= pub_frame && (slot == 5 || f == pub_frame))
      publish_start_frames(start_rec - static_cast<size_t>(B) * kStartInts, lane, slot <= 5 ? 0 : 6, slot, out.st, out.tok,
                           tag_lo, start_tag_hi(tag_lo));
    if (COMPARE) {
      // met the stored trajectory: this frame is written too (its score may differ), the rest stands
      if (stored.state_at(slot) == word && (SEL != 2 || stored.token_at(slot) == tok)) {
        out.template flush<true>(lane, slot + 1, B, b, tokens, states, scores);
        PB_STAT(0, 1);
        PB_STAT(1, f - f0 + 1);
        return true;
      }
    }
    if (slot == 63 && f + 1 < f1) {  // (the last group is written at the end, after the boundary bit is known)
      out.template flush<COMPARE>(lane, 64, B, b, tokens, states, scores);
      out.base = f + 1;
      if (COMPARE) stored.fetch(lane, f + 1, f1, B, b, tokens, states);
    }
    if (SEL == 2) last = tok;
    rp += frame_stride;
    return false;
  };
  using std::integral_constant;
  int fb = f0;
  for (; fb + NB <= f1; fb += NB) {  // whole turns of the ring: straight-line code
    if (GUESS) set_wave_priority(min(3, 4 * (f1 - fb) / (f1 - f0)));  // (pass 1: the more is left, the higher)
    if (do_frame(integral_constant<int, 0>{}, integral_constant<bool, true>{}, fb)) return true;
    if (do_frame(integral_constant<int, 1>{}, integral_constant<bool, true>{}, fb + 1)) return true;
    if (do_frame(integral_constant<int, 2>{}, integral_constant<bool, true>{}, fb + 2)) return true;
    if constexpr (NB > 3) {
      if (do_frame(integral_constant<int, 3>{}, integral_constant<bool, true>{}, fb + 3)) return true;
    }
  }
  if (fb < f1 && do_frame(integral_constant<int, 0>{}, integral_constant<bool, false>{}, fb)) return true;
  if (fb + 1 < f1 && do_frame(integral_constant<int, 1>{}, integral_constant<bool, false>{}, fb + 1)) return true;
  if constexpr (NB > 3) {
    if (fb + 2 < f1 && do_frame(integral_constant<int, 2>{}, integral_constant<bool, false>{}, fb + 2)) return true;
  }
  if (guessable && f1 < T) {
    // The guess the next range starts from, made here from the same rows; if it is what this range really
    // ends in, the last state word says so.
    float xl[16], c0[16];
    if (row_in_lds) {  // the usual case: the last frame left its raw row in LDS
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 q = *reinterpret_cast<const float4*>(row + 256 * i + 4 * lane);
        xl[4 * i + 0] = q.x; xl[4 * i + 1] = q.y; xl[4 * i + 2] = q.z; xl[4 * i + 3] = q.w;
      }
    } else {
      load16<FULL>(rp - frame_stride, 0, V, lane, -INFINITY, xl);
    }
    rebuild_base_boost<FULL, SEL>(t, opaque(lane), 0.0f, alpha, c0);
    int g, glabel;
    guess_boundary_1k<FULL, SEL>(t, xl, rp - frame_stride, frame_stride, f1 - 1, states0, b, c0, lane, g, glabel);
    bool certified = g == cur.s && (SEL != 2 || glabel == last);
    if (patch != nullptr) {
      int npatch = 0;
      if (!certified) {
        // (at most up to the frame before the last one of the next range, whose state word carries that range's own bit)
        set_wave_priority(3);  // the kernel ends with these waves
        npatch = run_on_1k<FULL, SEL>(t, rp, frame_stride, alpha, cur.s, c, c_p, last, min(kPatchMax, next_len - 1),
                                      patch, row, tags, lane, f1 < T ? start_rec : nullptr, tag_lo);
        certified = npatch > 0;
      }
      if (lane == 0) patch[0] = npatch;
    }
    if (certified && lane == f1 - 1 - out.base) out.st |= kGuessOk;
  } else if (GUESS && patch != nullptr && f1 < T && lane == 0) {
    patch[0] = 0;
  }
  out.template flush<COMPARE>(lane, f1 - out.base, B, b, tokens, states, scores);
  if (COMPARE) {
    PB_STAT(0, 1);
    PB_STAT(1, f1 - f0);
    PB_STAT(2, 1);
  }
  return false;  // (a re-run: the end of the range was reached without meeting the stored trajectory)
}

// LDS of one wave: a copy of the current row and the token marks.
constexpr int kWaveLdsFloats = kChunk + kTagWords;
constexpr size_t kWaveLdsBytes = kWaveLdsFloats * sizeof(float);

// Pass 1: chain (b, j) decodes segment j of hypothesis b; j = 0 starts from states0[b] and the
// caller's previous label (exact), j > 0 from a guess.  One wave per chain.
template <bool FULL, int SEL, bool FOREST>
__global__ void __launch_bounds__(256, 4) frames_spec_kernel(DeviceTree dt, TreePick pick, const float* __restrict__ logp,
                                                          int64_t frame_stride, int64_t row_stride,
                                                          const int32_t* __restrict__ states0,
                                                          const int32_t* __restrict__ last0, float alpha, int T, int B,
                                                          int seg_len, int nseg, int32_t* __restrict__ patches,
                                                          unsigned tag_lo, int32_t* __restrict__ tokens,
                                                          int32_t* __restrict__ states, float* __restrict__ scores) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = uniform_i(threadIdx.x >> 6);
  const int chain = blockIdx.x * (blockDim.x >> 6) + wave;
  if (chain >= B * nseg) return;
  const int j = chain / B, b = chain - j * B;
  float* row = lds + wave * kWaveLdsFloats;
  unsigned* tags = reinterpret_cast<unsigned*>(row + kChunk);
  DeviceTree mine = dt;
  bool tree_ok = true;
  if constexpr (FOREST) tree_ok = pick_tree(pick, b, mine);  // a table of trees: hypothesis b names its own
  const TreeView t = make_view(mine);
  const int f0 = seg_begin(j, T, nseg), f1 = seg_begin(j + 1, T, nseg);
  int s = 0, last = -1;
  if (j == 0) {
    s = states0[b];
    if (SEL == 2 && last0 != nullptr) last = last0[b];
  }
  if (!tree_ok) s = -1;  // an unknown tree marks every frame of the hypothesis like an invalid state
  int32_t* patch = nullptr;  // the record of the boundary after this segment
  if (patches != nullptr && f1 < T) patch = patches + (static_cast<size_t>(j) * B + b) * kPatchInts;
  // start records, behind the patches: that of the boundary behind this segment (the one it fills lies B earlier;
  // for the last segment this address lies behind the records and is only used to find the one B earlier)
  int32_t* start_recs = patches != nullptr ? patches + static_cast<size_t>(nseg - 1) * B * kPatchInts : nullptr;
  int32_t* start_rec = start_recs != nullptr ? start_recs + (static_cast<size_t>(j) * B + b) * kStartInts : nullptr;
  run_frames_1k<false, FULL, SEL, true>(t, logp, frame_stride, row_stride, alpha, B, b, f0, f1, s, last, T, states0,
                                        patch, (j + 2 <= nseg ? seg_begin(j + 2, T, nseg) : f1) - f1, tokens, states, scores,
                                        row, tags, lane, start_rec, tag_lo);
}

// Pass 2: one workgroup per hypothesis; its waves share the segments j = 1 .. nseg-1.
template <bool FULL, int SEL, bool FOREST>
__global__ void __launch_bounds__(512) frames_fix_kernel(DeviceTree dt, TreePick pick, const float* __restrict__ logp,
                                                          int64_t frame_stride, int64_t row_stride, float alpha, int T,
                                                          int B, int seg_len, int nseg,
                                                          const int32_t* __restrict__ patches,
                                                          int32_t* __restrict__ tokens,
                                                          int32_t* __restrict__ states, float* __restrict__ scores) {
  extern __shared__ float lds[];
  __shared__ int assumed[64], assumed_tok[64];
  __shared__ unsigned bad_words[2];
#ifdef PB_STATS
  const long long kernel_c0 = wall_clock64();
#endif
  const int lane = threadIdx.x & 63, wave = uniform_i(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
  const int b = blockIdx.x;
  float* row = lds + wave * kWaveLdsFloats;
  unsigned* tags = reinterpret_cast<unsigned*>(row + kChunk);
  DeviceTree mine = dt;
  if constexpr (FOREST) {
    if (!pick_tree(pick, b, mine)) return;  // pass 1 has marked every frame of this hypothesis (the whole workgroup leaves)
  }
  const TreeView t = make_view(mine);
  fix_segments<SEL == 2>(T, B, b, seg_len, nseg, tokens, states, scores, patches, assumed, assumed_tok, bad_words, lane,
                         wave, nwaves,
                         [&](int seg, int s, int last) {
                           const int f0 = seg_begin(seg, T, nseg), f1 = seg_begin(seg + 1, T, nseg);
#ifdef PB_STATS
                           const long long c0 = wall_clock64();
#endif
                           const bool met = run_frames_1k<true, FULL, SEL, false>(t, logp, frame_stride, row_stride, alpha, B, b, f0, f1, s,
                                                                 last, T, nullptr, nullptr, 0, tokens, states, scores, row, tags, lane);
#ifdef PB_STATS
                           const long long dt = wall_clock64() - c0;
                           PB_STAT(3, dt);
                           if (lane == 0) atomicMax(&g_stats[4], static_cast<unsigned long long>(dt));
#endif
                           return met;
                         });
#ifdef PB_STATS
  if (lane == 0) atomicMax(&g_stats[5], static_cast<unsigned long long>(wall_clock64() - kernel_c0));
#endif
}

// Single step: one wave per hypothesis, no speculation.  A step is a handful of dependent memory accesses long
// (arguments -> state id -> state record -> arcs -> record of the winner's target), so what the kernel costs is
// set by the order of its requests: the row, the root scores and the state id are requested together before
// anything is waited for, then the state's record, accumulated backoff and EOS boost together, then the arcs.
// LEAN: one wave per workgroup and one tree for all rows -- the grid is exactly B, no argument has to arrive
// before the requests go out and nothing but the hypothesis index separates the waves.  Otherwise a table of
// trees, every hypothesis naming its own (launched with one wave per workgroup as well; any number works).
template <bool FULL, int SEL, bool LEAN>
__global__ void __launch_bounds__(LEAN ? 64 : 256) step_wave_kernel(
    const float* __restrict__ logp, int64_t row_stride, const int32_t* __restrict__ states_in,
    const float* __restrict__ root_score, const int32_t* __restrict__ last_in, float alpha, int blank,
    int32_t* __restrict__ tokens, int B, int32_t* __restrict__ states_out, float* __restrict__ scores, DeviceTree dt,
    TreePick pick) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = LEAN ? 0 : uniform_i(threadIdx.x >> 6);
  const int b = LEAN ? static_cast<int>(blockIdx.x) : static_cast<int>(blockIdx.x * (blockDim.x >> 6)) + wave;
  if (!LEAN && b >= B) return;
  float* row = lds + wave * kWaveLdsFloats;
  unsigned* tags = reinterpret_cast<unsigned*>(row + kChunk);
  DeviceTree mine = dt;
  bool tree_ok = true;
  if constexpr (!LEAN) tree_ok = pick_tree(pick, b, mine);
  const TreeView t = make_view(mine);
  // (arc batches requested up front, for the state and for the state its failure link leads to; the lone wave of
  // the small-batch form has registers to spare under every rule)
  // Arc batches requested up front, for the state and for the state its failure link leads to.  The lone wave of the
  // small-batch form pays for every instruction, also for the addresses of batches most states do not have: one
  // batch up front measured fastest there under every rule (3.11 against 3.21 us per step with four and four).
  constexpr int kEarlyBatches = LEAN ? 1 : (SEL == 0 ? 4 : 2);
  constexpr int kEarlyBatches1 = LEAN ? 0 : (SEL == 0 ? 4 : (SEL == 1 ? 2 : 0));
  float x[16], c[16];
  // (loads retire in order: the root scores come from a cache and are worked on while the row is on its way)
  // (`root_score` is the tree's array again, as an argument of its own: the leading arguments are in registers
  // when the wave starts, the tree structure has to be fetched)
  load16<FULL>(LEAN ? root_score : t.root_score, 0, t.V, lane, 0.0f, c);
  load16<FULL>(logp + static_cast<size_t>(b) * row_stride, 0, t.V, lane, -INFINITY, x);
  int s = tree_ok ? states_in[b] : -1;  // an unknown tree marks the hypothesis like an invalid state
  int last = -1;
  if (SEL == 2 && last_in != nullptr) last = last_in[b];
  __builtin_amdgcn_sched_barrier(0);  // (all of the above is in flight before the first wait)
  // A lone wave issues one instruction every few cycles whatever it is, so what comes after the state's record
  // has arrived is kept short: the boost of a token is am * (p_root + root_score) with am = alpha, except in the
  // one slot of the one lane that holds the blank (0: no boost; NaN under the two-stage rules: excluded).  The
  // multipliers depend on nothing that is loaded (`blank` is the tree's, as a leading argument like
  // `root_score`) and are formed while the state id is on its way.
  // (The form with a table of trees learns the blank with the tree and keeps the test per slot.)
  float am[LEAN ? 16 : 1];
  if constexpr (LEAN) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      am[j] = slot_is(j, lane, blank) ? (SEL == 0 ? 0.0f : NAN) : alpha;
      asm volatile("" : "+v"(am[j]));  // (formed here, not where it is used)
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  s = uniform_i(s);
  last = uniform_i(last);
  // An invalid state is decoded as the root and marked at the end: an early exit here would let the compiler
  // move the row requests behind the test, i.e. behind the wait for the state id.
  const bool ok = valid_state(t, s);
  if (!LEAN && !ok) {
    if (lane == 0) {
      tokens[b] = -1;
      states_out[b] = -1;
      scores[b] = NAN;
    }
    return;
  }
  Cursor cur = cursor_at(t, ok ? s : 0);
  __builtin_amdgcn_sched_barrier(0);  // (the three parts of the cursor are requested together)
  float c_p = cur.p_root;
  if constexpr (LEAN) {
#pragma unroll
    for (int j = 0; j < 16; ++j) c[j] = __fmul_rn(am[j], __fadd_rn(c_p, c[j]));  // base boosts, in place
  } else {
    make_base_boost<SEL>(0, lane, t.blank, c_p, alpha, c, c);  // element-wise, in place
  }
  float val;
  int tok;
  bool row_in_lds = false;
  frame_1k<FULL, SEL, kEarlyBatches, kEarlyBatches1, 4>(t, cur, x, c, c_p, alpha, row, tags, lane, last, false, [] {},
                                                        val, tok, row_in_lds);
  if (lane == 0) {
    tokens[b] = ok ? tok : -1;
    states_out[b] = ok ? cur.s : -1;
    scores[b] = ok ? val : NAN;
  }
}

// ------------------------------------------------------------------------------------------------
// Beam step, one wave per hypothesis row (V <= 1024, K <= kBeamWaveMaxK): the workgroup of an utterance
// has K waves.  Every wave forms the fused row of its beam -- base candidates in registers, the arcs
// of the failure chain scattered into an LDS overlay (value and child state per overridden token,
// deepest chain state first, later ones skipped through the token marks) -- adds the hypothesis
// score and extracts its K best totals in order by repeated wave arg-max (a taken entry becomes
// NaN, which no maximum or equality test selects).  The K*K survivors meet in LDS, and wave 0
// picks the utterance's K best by (total descending, flat index k*V+v ascending).
// A step is latency-bound, so the requests go out in the order of the single greedy step: root scores, row,
// states and hypothesis score before the first wait; an utterance with an invalid state is decoded from the
// root and marked at the end, so that no early exit separates the wave start from the requests.  The raw row
// goes into the overlay first: an arc then finds its log-prob in LDS instead of in memory.
constexpr int kBeamWaveMaxK = 8;
constexpr int kBeamWaveLdsFloats = 2 * kChunk + kTagWords;                   // overlay values, overlay children, marks
constexpr size_t kBeamCandBytes = kBeamWaveMaxK * kBeamWaveMaxK * 3 * sizeof(int);  // value, flat index, child

template <bool FULL>
__global__ void __launch_bounds__(64 * kBeamWaveMaxK) beam_wave_kernel(
    const float* __restrict__ logp, int64_t row_stride, const float* __restrict__ hyp,
    const int32_t* __restrict__ states_in, const float* __restrict__ root_score, float alpha, int K,
    int32_t* __restrict__ tokens, int32_t* __restrict__ parents, int32_t* __restrict__ states_out,
    float* __restrict__ scores_out, DeviceTree dt) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = uniform_i(threadIdx.x >> 6);
  const int u = blockIdx.x, h = u * K + wave;
  const TreeView t = make_view(dt);
  const int V = t.V;
  const float* lrow = logp + static_cast<size_t>(h) * row_stride;
  float x[16], c[16];
  load16<FULL>(root_score, 0, V, lane, 0.0f, c);  // (the tree's array, as a leading argument: in registers at the start)
  load16<FULL>(lrow, 0, V, lane, -INFINITY, x);
  const int sk = states_in[u * K + min(lane, K - 1)];  // every wave sees all K states
  const float hs_in = hyp[h];
  __builtin_amdgcn_sched_barrier(0);  // (all of the above is in flight before the first wait)
  // per-slot multiplier of the boost (alpha; 0 in the blank's slot), formed while the states are on their way:
  // what follows the arrival of the state's record is then two instructions per slot (see step_wave_kernel)
  float am[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    am[j] = slot_is(j, lane, t.blank) ? 0.0f : alpha;
    asm volatile("" : "+v"(am[j]));  // (formed here, not where it is used)
  }
  __builtin_amdgcn_sched_barrier(0);
  float* cand_val = lds;  // [K*K], then the flat indices and the children
  int* cand_idx = reinterpret_cast<int*>(lds + kBeamWaveMaxK * kBeamWaveMaxK);
  int* cand_nxt = cand_idx + kBeamWaveMaxK * kBeamWaveMaxK;
  float* ov = lds + 3 * kBeamWaveMaxK * kBeamWaveMaxK + wave * kBeamWaveLdsFloats;
  int* ov_next = reinterpret_cast<int*>(ov + kChunk);
  unsigned* tags = reinterpret_cast<unsigned*>(ov + 2 * kChunk);

  // an utterance with an invalid state is marked as a whole (at the end)
  const bool bad = __ballot(!valid_state(t, sk)) != 0;
  const int s = bad ? 0 : __builtin_amdgcn_readlane(sk, wave);
  const float hs = uniform_f(hs_in);
  const Cursor cur = cursor_at(t, s);
  __builtin_amdgcn_sched_barrier(0);  // (the parts of the cursor are requested together)
#pragma unroll
  for (int j = 0; j < 16; ++j) c[j] = __fmul_rn(am[j], __fadd_rn(cur.p_root, c[j]));  // base boosts, in place
  tags_clear(tags, lane);
  store_row_lds(ov, lane, x);  // the raw row: an arc reads its log-prob here and puts its fused value in its place
  // ---- overlay: arcs of the failure chain, deepest state first ------------------------------------
  {
    float p = 0.0f;
    for (int xs = s; xs != 0;) {
      const Rec r = load_rec(t, xs);
      for (int j = lane; j < r.count; j += 64) {
        const ArcRec a = t.arc[r.begin + j];
        if (!tag_test(tags, a.token)) {  // tokens of one state are distinct: no lane races for an entry
          tag_set(tags, a.token);
          ov[a.token] = __fadd_rn(ov[a.token], __fmul_rn(alpha, __fadd_rn(p, a.score)));
          ov_next[a.token] = r.begin + j + 1;
        }
      }
      p = __fadd_rn(p, r.backoff);
      xs = uniform_i(r.fail);
    }
  }
  // ---- totals of the lane's 16 tokens -------------------------------------------------------------
  float tv[16];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v0 = 256 * i + 4 * lane;
    const unsigned bits = tags[v0 >> 5] >> (v0 & 31);
    const float4 o = *reinterpret_cast<const float4*>(ov + v0);
    const float oa[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float expansion = ((bits >> k) & 1u) ? oa[k] : __fadd_rn(x[4 * i + k], c[4 * i + k]);
      // positions past V hold -inf: with at most V rounds the real tokens, which come first, are taken before them
      tv[4 * i + k] = (FULL || v0 + k < V) ? __fadd_rn(hs, expansion) : -INFINITY;
    }
  }
  if (t.eos >= 0) {  // EOS rule (Sec. II-C): boosted by the value tabulated for the state; no arc carries the token
    const float ce = __fmul_rn(alpha, cur.eos_boost);
    const int ln = opaque(lane);
#pragma unroll
    for (int j = 0; j < 16; ++j) tv[j] = slot_is(j, ln, t.eos) ? __fadd_rn(hs, __fadd_rn(x[j], ce)) : tv[j];
  }
  // ---- the row's best totals, in order ---------------------------------------------------------------
  const int rounds = min(K, V);
  for (int r = 0; r < rounds; ++r) {
    float g[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) g[i] = max4(tv[4 * i], tv[4 * i + 1], tv[4 * i + 2], tv[4 * i + 3]);
    const float M = ukey_val(wave_max_u(ukey(max4(g[0], g[1], g[2], g[3]))));
    const int v = uniform_i(first_token_equal(tv, g, M, lane));
    int nx = s;  // the blank and the EOS keep the state
    if (v != t.blank && v != t.eos) nx = tag_test(tags, v) ? ov_next[v] : t.root_next[v];
    if (lane == 0) {  // `rounds` entries per wave, packed
      cand_val[wave * rounds + r] = M;
      cand_idx[wave * rounds + r] = wave * V + v;
      cand_nxt[wave * rounds + r] = nx;
    }
    const int taken = slot_in_lane(opaque(lane), v);
#pragma unroll
    for (int j = 0; j < 16; ++j) tv[j] = taken == j ? NAN : tv[j];
  }
  __syncthreads();
  if (wave != 0) return;
  // ---- merge: one candidate per lane ------------------------------------------------------------------
  const int n = K * rounds;
  const bool have = lane < n;
  float val = have ? cand_val[lane] : 0.0f;
  const int idx = have ? cand_idx[lane] : INT_MAX;
  const int nxt = have ? cand_nxt[lane] : 0;
  bool live = have;
  for (int j = 0; j < K; ++j) {
    const float M = ukey_val(wave_max_u(live ? ukey(val) : 0u));
    const int best = wave_min_nn((live && val == M) ? idx : INT_MAX);
    if (live && idx == best) {
      tokens[u * K + j] = bad ? -1 : idx % V;
      parents[u * K + j] = bad ? -1 : idx / V;
      states_out[u * K + j] = bad ? -1 : nxt;
      scores_out[u * K + j] = bad ? NAN : val;
      live = false;
    }
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int g_fix_waves = 8;  // waves per fix-up workgroup the device's LDS allows, set once

}  // namespace

bool wave_path_ok(const DeviceTree& t, const float* d_logp, int64_t frame_stride, int64_t row_stride) {
  return t.p_root != nullptr && t.root_rec != nullptr && t.vocab_size % 4 == 0 && t.vocab_size <= kWideMaxV &&
         row_stride % 4 == 0 && frame_stride % 4 == 0 && aligned16(d_logp) && aligned16(t.root_score);
}

SegPlan plan_segments(int32_t T, int32_t B, int target_chains) {
  // Segments: enough concurrent chains to cover the memory latency, at most kMaxSegments per
  // hypothesis, at least kMinSegLen frames long.
  int nseg = (target_chains + B - 1) / B;
  nseg = nseg < 1 ? 1 : (nseg > kMaxSegments ? kMaxSegments : nseg);
  int seg_len = (T + nseg - 1) / nseg;
  if (seg_len < kMinSegLen) seg_len = kMinSegLen;
  nseg = (T + seg_len - 1) / seg_len;
  return SegPlan{nseg, seg_len};
}

// Expands to one launch per (row shape, selection rule) pair; FULL: V == 1024, `sel` a runtime value in 0..2.
#define PB_DISPATCH(full, sel, LAUNCH)   \
  switch ((full ? 0 : 3) + (sel)) {      \
    case 0: LAUNCH(true, 0); break;      \
    case 1: LAUNCH(true, 1); break;      \
    case 2: LAUNCH(true, 2); break;      \
    case 3: LAUNCH(false, 0); break;     \
    case 4: LAUNCH(false, 1); break;     \
    default: LAUNCH(false, 2); break;    \
  }

int launch_step_wave(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t row_stride,
                     const int32_t* d_states_in, const int32_t* d_last, float alpha, int32_t B, int sel, int32_t* d_tokens, int32_t* d_states_out,
                     float* d_scores, hipStream_t stream) {
  if (t.vocab_size > kChunk)
    return launch_step_wide(t, pick, d_logp, row_stride, d_states_in, d_last, alpha, B, sel, d_tokens, d_states_out,
                            d_scores, stream);
  // One wave per workgroup at every batch size (measured against four waves per workgroup from B = 128 to
  // B = 65536: never slower, 12 % faster at B = 65536 on states of all depths -- no wave waits for the slowest of
  // its workgroup, and a small batch spreads over as many CUs as it has rows).  `lean`: one tree for all rows.
  const bool lean = pick.table == nullptr;
  const int waves = 1;  // (also with a table of trees: 68.7 against 73.7 us at B = 65536, 5.8 against 6.4 us at B = 128)
  const dim3 grid(static_cast<unsigned>((B + waves - 1) / waves)), block(static_cast<unsigned>(64 * waves));
  const size_t lds = static_cast<size_t>(waves) * kWaveLdsBytes;
  const bool full = t.vocab_size == kChunk;
#define PB_STEP(FULL, SEL, LEAN)                                                                                   \
  hipLaunchKernelGGL((step_wave_kernel<FULL, SEL, LEAN>), grid, block, lds, stream, d_logp, row_stride,            \
                     d_states_in, t.root_score, d_last, alpha, t.blank_id, d_tokens, B, d_states_out, d_scores, t,  \
                     pick)
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

// A number that no earlier call of this process has used: a counter from a random 64-bit start.
uint64_t next_call_tag() {
  static std::atomic<uint64_t> counter{[] {
    std::random_device rd;
    const uint64_t a = rd(), b = rd();
    return (a << 32) ^ b ^ static_cast<uint64_t>(std::chrono::steady_clock::now().time_since_epoch().count());
  }()};
  return counter.fetch_add(0x9E3779B97F4A7C15ull, std::memory_order_relaxed);  // (odd step: all 2^64 values in turn)
}

int64_t frames_workspace_bytes(const DeviceTree& t, int32_t T, int32_t B) {
  if (t.vocab_size > kChunk) return 0;  // (wide rows repair wrong guesses in pass 2)
  const SegPlan plan = plan_segments(T, B, kTargetChains);
  return static_cast<int64_t>(plan.nseg - 1) * B * (kPatchInts + kStartInts) * static_cast<int64_t>(sizeof(int32_t));
}

int launch_frames_wave(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t frame_stride,
                       int64_t row_stride,
                       const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B, int sel,
                       int32_t* d_tokens, int32_t* d_states, float* d_scores, int32_t* d_patches, hipStream_t stream) {
  if (t.vocab_size > kChunk)
    return launch_frames_wide(t, pick, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B, sel, d_tokens,
                              d_states, d_scores, stream);
  const SegPlan plan = plan_segments(T, B, kTargetChains);
  const int nseg = plan.nseg, seg_len = plan.seg_len;
  const int64_t chains = static_cast<int64_t>(B) * nseg;
  const uint64_t tag = next_call_tag();  // marks the start records of this call (see kStartInts)
  const unsigned tag_lo = static_cast<unsigned>(tag);
  const int waves = 4;
  const int64_t blocks = (chains + waves - 1) / waves;
  if (blocks > INT32_MAX) return PB_EUNSUPPORTED;
  const size_t lds = static_cast<size_t>(waves) * kWaveLdsBytes;
  const bool full = t.vocab_size == kChunk;
  const bool forest = pick.table != nullptr;
#define PB_SPEC(FULL, SEL, FOREST)                                                                                   \
  hipLaunchKernelGGL((frames_spec_kernel<FULL, SEL, FOREST>), dim3(static_cast<unsigned>(blocks)), dim3(64 * waves), \
                     lds, stream, t, pick, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B,        \
                     seg_len, nseg, d_patches, tag_lo, d_tokens, d_states, d_scores)
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
    int fw = nseg - 1 < g_fix_waves ? nseg - 1 : g_fix_waves;
    const size_t lds2 = static_cast<size_t>(fw) * kWaveLdsBytes;
#define PB_FIX(FULL, SEL, FOREST)                                                                                     \
  hipLaunchKernelGGL((frames_fix_kernel<FULL, SEL, FOREST>), dim3(static_cast<unsigned>(B)), dim3(64 * fw), lds2,     \
                     stream, t, pick, d_logp, frame_stride, row_stride, alpha, T, B, seg_len, nseg, d_patches,        \
                     d_tokens, d_states, d_scores)
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

#ifdef PB_STATS
extern "C" int pb_debug_stats(unsigned long long* out8, int reset) {
  if (hipMemcpyFromSymbol(out8, HIP_SYMBOL(g_stats), 8 * sizeof(unsigned long long)) != hipSuccess) return -1;
  if (reset) {
    unsigned long long z[8] = {0};
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_stats), z, sizeof(z)) != hipSuccess) return -1;
  }
  return 0;
}
#endif

int g_beam_wave_max_k = 7;  // widest beam the wave kernel's LDS allows on the device, set once

bool beam_wave_ok(const DeviceTree& t, const float* d_logp, int64_t row_stride, int32_t K) {
  return wave_path_ok(t, d_logp, 0, row_stride) && t.vocab_size <= kChunk && K <= g_beam_wave_max_k;
}

int launch_beam_wave(const DeviceTree& t, const float* d_logp, int64_t row_stride, const float* d_hyp,
                     const int32_t* d_states_in, float alpha, int32_t U, int32_t K, int32_t* d_tokens,
                     int32_t* d_parents, int32_t* d_states_out, float* d_scores_out, hipStream_t stream) {
  const size_t lds = kBeamCandBytes + static_cast<size_t>(K) * kBeamWaveLdsFloats * sizeof(float);
  const dim3 grid(static_cast<unsigned>(U)), block(static_cast<unsigned>(64 * K));
  if (t.vocab_size == kChunk)
    hipLaunchKernelGGL(beam_wave_kernel<true>, grid, block, lds, stream, d_logp, row_stride, d_hyp, d_states_in,
                       t.root_score, alpha, K, d_tokens, d_parents, d_states_out, d_scores_out, t);
  else
    hipLaunchKernelGGL(beam_wave_kernel<false>, grid, block, lds, stream, d_logp, row_stride, d_hyp, d_states_in,
                       t.root_score, alpha, K, d_tokens, d_parents, d_states_out, d_scores_out, t);
  return hipGetLastError() == hipSuccess ? PB_OK : PB_EHIP;
}

int prepare_wave_kernels() {
  // The fix-up workgroup uses kWaveLdsBytes of dynamic LDS per wave; past 64 KiB the limit must be raised.
  int dev = 0, max_lds = 0;
  if (hipGetDevice(&dev) != hipSuccess) return PB_EHIP;
  if (hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return PB_EHIP;
  int waves = (max_lds - 1024) / static_cast<int>(kWaveLdsBytes);
  waves = waves > 8 ? 8 : (waves < 1 ? 1 : waves);  // 8 waves per workgroup leave each wave 256 registers
  constexpr int kPlainLimit = 64 * 1024 - 1024;  // static LDS of the kernel included
  if (waves * static_cast<int>(kWaveLdsBytes) > kPlainLimit) {
    const int bytes = waves * static_cast<int>(kWaveLdsBytes);
    const hipFuncAttribute attr = hipFuncAttributeMaxDynamicSharedMemorySize;
    bool ok = true;
#define PB_SET(FULL, SEL)                                                                                              \
  ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(frames_fix_kernel<FULL, SEL, false>), attr, bytes) == hipSuccess && \
       hipFuncSetAttribute(reinterpret_cast<const void*>(frames_fix_kernel<FULL, SEL, true>), attr, bytes) == hipSuccess
    for (int ms = 0; ms < 6; ++ms) PB_DISPATCH(ms < 3, ms % 3, PB_SET)
#undef PB_SET
    if (!ok) {
      (void)hipGetLastError();
      waves = kPlainLimit / static_cast<int>(kWaveLdsBytes);
    }
  }
  g_fix_waves = waves;
  // The beam kernel with kBeamWaveMaxK waves needs a little more than 64 KiB.
  const int beam_bytes = static_cast<int>(kBeamCandBytes + kBeamWaveMaxK * kBeamWaveLdsFloats * sizeof(float));
  g_beam_wave_max_k = static_cast<int>((kPlainLimit - kBeamCandBytes) / (kBeamWaveLdsFloats * sizeof(float)));
  if (beam_bytes <= max_lds) {
    const hipFuncAttribute attr = hipFuncAttributeMaxDynamicSharedMemorySize;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(beam_wave_kernel<true>), attr, beam_bytes) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(beam_wave_kernel<false>), attr, beam_bytes) == hipSuccess)
      g_beam_wave_max_k = kBeamWaveMaxK;
    else
      (void)hipGetLastError();
  }
  return prepare_wide_kernels(max_lds);
}

}  // namespace pb
