// Device helpers shared by the wave-per-hypothesis kernels (gfx950, wave64): scalar-path views of the tree,
// order-preserving keys and DPP reductions, row loads in the 16-tokens-per-lane layout, per-wave token marks.
#pragma once
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "pb_kernels.hpp"

namespace pb {
namespace wv {

#define PB_AS4 __attribute__((address_space(4)))

constexpr int kChunk = 1024;  // tokens per chunk: 16 per lane

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
using u64 = unsigned long long;

// Scalar-load views: the tree is never written while kernels run, so wave-uniform reads may go
// through the constant address space (scalar cache).
struct TreeView {
  const v8i PB_AS4* state;     // StateRec as eight dwords: arc_begin, arc_count, fail, backoff bits, twice
  const float PB_AS4* p_root;
  const int32_t PB_AS4* root_next;
  const v8i PB_AS4* root_rec;  // RootRec as eight dwords
  const float PB_AS4* eos_score;  // null without an EOS rule
  const ArcRec* arc;
  const float* root_score;
  int num_states, V, blank, eos;
};

__device__ __forceinline__ TreeView make_view(const DeviceTree& t) {
  TreeView v;
  v.state = (const v8i PB_AS4*)t.state;
  v.p_root = (const float PB_AS4*)t.p_root;
  v.root_next = (const int32_t PB_AS4*)t.root_next;
  v.root_rec = (const v8i PB_AS4*)t.root_rec;
  v.eos_score = (const float PB_AS4*)t.eos_score;
  v.arc = t.arc;
  v.root_score = t.root_score;
  v.num_states = t.num_states;
  v.V = t.vocab_size;
  v.blank = t.blank_id;
  v.eos = t.eos_id;
  return v;
}

// Values that are wave-uniform by construction, told to the compiler (keeps them in SGPRs and the
// loads they address on the scalar path).
__device__ __forceinline__ int uniform_i(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uniform_f(float v) {
  return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}

// Order-preserving fp32 <-> uint32 (every real value, -inf included, maps above 0).
__device__ __forceinline__ unsigned ukey(float f) {
  const int b = __float_as_int(f);
  return static_cast<unsigned>(b) ^ (static_cast<unsigned>(b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float ukey_val(unsigned k) {
  const unsigned m = (k & 0x80000000u) ? 0x80000000u : 0xffffffffu;
  return __uint_as_float(k ^ m);
}

template <int CTRL>
__device__ __forceinline__ unsigned dpp0(unsigned v) {  // lanes without a source read 0
  return static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, true));
}
// Wave-wide unsigned max; 0 is the identity.  The result is wave-uniform (read from lane 63).
__device__ __forceinline__ unsigned wave_max_u(unsigned v) {
  v = max(v, dpp0<0x111>(v));  // row_shr:1
  v = max(v, dpp0<0x112>(v));  // row_shr:2
  v = max(v, dpp0<0x114>(v));  // row_shr:4
  v = max(v, dpp0<0x118>(v));  // row_shr:8
  v = max(v, dpp0<0x142>(v));  // row_bcast:15
  v = max(v, dpp0<0x143>(v));  // row_bcast:31
  return static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(v), 63));
}
// Wave-wide min of non-negative ints (INT_MAX = nothing).
__device__ __forceinline__ int wave_min_nn(int v) {
  return INT_MAX - static_cast<int>(wave_max_u(static_cast<unsigned>(INT_MAX - v)));
}
// The lane id again, but opaque to the optimiser: values derived from it inside a rarely taken branch
// are then computed there instead of being hoisted out of the frame loop into long-lived registers.
__device__ __forceinline__ int opaque(int v) {
  asm volatile("" : "+v"(v));
  return v;
}
__device__ __forceinline__ int first_lane(u64 mask) { return __builtin_ctzll(mask); }

__device__ __forceinline__ int tok_of(int j, int lane) { return 256 * (j >> 2) + 4 * lane + (j & 3); }
// Does the lane's slot j hold chunk-relative token `rel` (wave-uniform)?  Written so that the slot
// test stays on the scalar side and no per-slot token ids have to live in vector registers.
__device__ __forceinline__ bool slot_is(int j, int lane, int rel) {
  const int slot = ((rel >> 8) << 2) | (rel & 3);  // uniform
  return (slot == j) && (lane == ((rel >> 2) & 63)) && (static_cast<unsigned>(rel) < static_cast<unsigned>(kChunk));
}

// The slot in which this lane holds chunk-relative token `rel` (wave-uniform), -1 in every other lane: a test of
// all 16 slots against it is one vector compare per slot, where slot_is takes three scalar instructions and a
// vector one -- for a lone wave, which issues one instruction every few cycles whatever it is, the cheaper form.
__device__ __forceinline__ int slot_in_lane(int lane, int rel) {
  const bool here = static_cast<unsigned>(rel) < static_cast<unsigned>(kChunk) && lane == ((rel >> 2) & 63);
  return here ? (((rel >> 8) << 2) | (rel & 3)) : -1;
}

__device__ __forceinline__ bool valid_state(const TreeView& t, int s) {
  return static_cast<unsigned>(s) < static_cast<unsigned>(t.num_states);
}

struct Rec {  // wave-uniform copy of one half of a StateRec
  int begin, count, fail;
  float backoff;
};
struct Rec2 {  // a state and the state its failure link leads to
  Rec a, b;
};
__device__ __forceinline__ Rec load_rec(const TreeView& t, int s) {
  const v4i r = reinterpret_cast<const v4i PB_AS4*>(t.state)[2 * s];
  Rec o;
  o.begin = r.x;
  o.count = r.y;
  o.fail = r.z;
  o.backoff = __int_as_float(r.w);
  return o;
}
__device__ __forceinline__ Rec2 load_rec2(const TreeView& t, int s) {
  const v8i r = t.state[s];
  Rec2 o;
  o.a.begin = r.s0;
  o.a.count = r.s1;
  o.a.fail = r.s2;
  o.a.backoff = __int_as_float(r.s3);
  o.b.begin = r.s4;
  o.b.count = r.s5;
  o.b.fail = r.s6;
  o.b.backoff = __int_as_float(r.s7);
  return o;
}

struct Cursor {  // wave-uniform decoding state of one hypothesis
  int s;
  Rec rec;   // of the state
  Rec rec1;  // of the state its failure link leads to (meaningful when rec.fail != 0)
  float p_root;
  float eos_boost;  // boost of the EOS token in this state (Sec. II-C); 0 without an EOS rule
};
__device__ __forceinline__ Cursor cursor_at(const TreeView& t, int s) {
  Cursor c;
  c.s = s;
  const Rec2 r = load_rec2(t, s);
  c.rec = r.a;
  c.rec1 = r.b;
  c.p_root = t.p_root[s];
  c.eos_boost = 0.0f;
  if (t.eos >= 0) c.eos_boost = t.eos_score[s];
  return c;
}
__device__ __forceinline__ Cursor cursor_from_root_rec(const v8i& r) {
  Cursor c;
  c.s = r.s0;
  c.rec.begin = r.s1;
  c.rec.count = r.s2;
  c.rec.fail = r.s3;
  c.rec.backoff = __int_as_float(r.s4);
  c.rec1 = Rec{0, 0, 0, 0.0f};  // the root row leads to the root or a depth-1 state: the chain ends there
  c.p_root = __int_as_float(r.s5);
  c.eos_boost = __int_as_float(r.s6);
  return c;
}

// Selection rule (enum pb_select_mode): 0 = single-stage fused arg-max, 1 = two-stage, 2 = two-stage
// with the CTC repeat rule (Sec. II-C).  In the two-stage modes the blank is never a candidate of
// the boosted re-selection: its column carries NaN, which neither fmaxf nor an equality test ever
// selects, so an excluded token costs nothing in the reductions.
//
// alpha * (p_root + root_score[v]) for the lane's 16 tokens; the blank column boosts by 0 (SEL == 0)
// or is excluded (SEL != 0).
template <int SEL>
__device__ __forceinline__ void make_base_boost(int cb, int lane, int blank, float p_root, float alpha,
                                                const float (&rw)[16], float (&c)[16]) {
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const float boost = slot_is(j, lane, blank - cb) ? (SEL == 0 ? 0.0f : NAN) : __fadd_rn(p_root, rw[j]);
    c[j] = __fmul_rn(alpha, boost);
  }
}

// Loads the lane's 16 values of chunk `cb` of a V-long fp32 array; positions >= V read as `fill`.
template <bool FULL>
__device__ __forceinline__ void load16(const float* __restrict__ base, int cb, int V, int lane, float fill,
                                       float (&x)[16]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = cb + 256 * i + 4 * lane;
    if (FULL || v < V) {  // V % 4 == 0: a 16-byte group is entirely inside or outside the row
      const float4 q = *reinterpret_cast<const float4*>(base + v);
      x[4 * i + 0] = q.x; x[4 * i + 1] = q.y; x[4 * i + 2] = q.z; x[4 * i + 3] = q.w;
    } else {
      x[4 * i + 0] = x[4 * i + 1] = x[4 * i + 2] = x[4 * i + 3] = fill;
    }
  }
}

__device__ __forceinline__ void store_row_lds(float* row, int lane, const float (&x)[16]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<float4*>(row + 256 * i + 4 * lane) = make_float4(x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]);
}

// Lowest token (chunk-relative) whose fused value equals M; g are the lane's four group maxima.
__device__ __forceinline__ int first_token_equal(const float (&f)[16], const float (&g)[4], float M, int lane) {
  const u64 b0 = __ballot(g[0] == M), b1 = __ballot(g[1] == M), b2 = __ballot(g[2] == M), b3 = __ballot(g[3] == M);
  int gi;
  u64 bm, e0, e1, e2;  // the fourth token of a group needs no ballot: it is the one left
  if (b0) {
    gi = 0; bm = b0;
    e0 = __ballot(f[0] == M); e1 = __ballot(f[1] == M); e2 = __ballot(f[2] == M);
  } else if (b1) {
    gi = 1; bm = b1;
    e0 = __ballot(f[4] == M); e1 = __ballot(f[5] == M); e2 = __ballot(f[6] == M);
  } else if (b2) {
    gi = 2; bm = b2;
    e0 = __ballot(f[8] == M); e1 = __ballot(f[9] == M); e2 = __ballot(f[10] == M);
  } else if (b3) {
    gi = 3; bm = b3;
    e0 = __ballot(f[12] == M); e1 = __ballot(f[13] == M); e2 = __ballot(f[14] == M);
  } else {
    return 0;  // only with NaN inputs (precondition violation): stay in range
  }
  const int L = first_lane(bm);
  const u64 bit = 1ull << L;
  const int k = (e0 & bit) ? 0 : (e1 & bit) ? 1 : (e2 & bit) ? 2 : 3;
  return 256 * gi + 4 * L + k;
}

// Per-wave token marks: one bit per token of the current chunk (32 dwords of LDS).  LDS operations
// of one wave execute in order, so clear -> set -> test needs no barrier inside the wave.
constexpr int kTagWords = kChunk / 32;
__device__ __forceinline__ void tags_clear(unsigned* bits, int lane) {
  if (lane < kTagWords) bits[lane] = 0u;
}
__device__ __forceinline__ void tag_set(unsigned* bits, int tk) { atomicOr(&bits[tk >> 5], 1u << (tk & 31)); }
__device__ __forceinline__ bool tag_test(const unsigned* bits, int tk) { return ((bits[tk >> 5] >> (tk & 31)) & 1u) != 0u; }

// Maximum of four values in two instructions.  Written out because the compiler puts a canonicalising
// max(x, x) in front of every operand of fmaxf whose origin it cannot see, which doubles the count; the
// instructions return the other operand when one is a NaN, as fmaxf does.
__device__ __forceinline__ float max4(float a, float b, float c, float d) {
  float m;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m) : "v"(a), "v"(b), "v"(c));
  asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(m), "v"(d));
  return m;
}

// Stage 1 of the two-stage rule on one chunk: the unboosted row maximum and its lowest token.
__device__ __forceinline__ void plain_argmax(const float (&x)[16], int lane, float& M0, int& v0) {
  float g[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) g[i] = max4(x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]);
  M0 = ukey_val(wave_max_u(ukey(max4(g[0], g[1], g[2], g[3]))));
  v0 = first_token_equal(x, g, M0, lane);
}

// ------------------------------------------------------------------------------------------------
// Multi-frame decoding in speculative segments: what the row layouts (rows of up to 1024 tokens, wider
// rows) share.
//
// The T frames of a hypothesis are cut into segments decoded concurrently, one wave each (pass 1).  A
// segment that does not begin the call starts from a guess of the state (and, under the CTC rule, of
// the label) the frame before it ends in.  The segment on the left computes the same guess from the
// same rows at its end and, when it equals what it really ended in, sets kGuessOk in the state word
// it stores for its last frame.  Pass 2 re-runs the other segments from their neighbour's end state
// until they meet the stored trajectory (a finite automaton: equal (state, label) after a frame means
// an identical future), then compares every assumed start with the final outcome before it and re-runs
// the stale segments in parallel rounds, and clears the bits.  States stay below 2^30 for this.
constexpr int kGuessOk = 1 << 30;
// Frames a boundary guess may look back over.  A frame that keeps the state (a blank, under every rule)
// says nothing about it, so the guess goes back to the last frame that moved it.
constexpr int kLookBack = 8;

// Patches (optional workspace of the multi-frame decoder).  A segment that finds its guess for the next segment
// wrong decodes on from its real outcome until it meets the trajectory the guess has led to -- at most kPatchMax
// frames, usually one to three -- and leaves the frames it has decoded as a patch for the start of the next
// segment.  The boundary then counts as certified, and pass 2 only copies the patch over what the next segment
// wrote; nothing is decoded again.  One record per boundary: count, then tokens, states, scores.
constexpr int kPatchMax = 16;
constexpr int kPatchInts = 4 + 3 * kPatchMax;

// Start records (same workspace, behind the patches).  The repair above needs the trajectory the guess has led
// to, and the segment on the right decodes exactly that: it leaves the states and tokens of its first frames in
// the record of its left boundary (in two groups: a store sits in the in-order queue of the loads).  The segment
// on the left, when it comes to repair that boundary (usually tens of microseconds later), reads them there; a
// frame that is not there (looked at twice) ends the repair, and pass 2 decodes the segment on the right again.
//   No fence orders these accesses (a release at agent scope writes back the whole L2 of the XCD: with one per
//   segment pass 1 took 283 us instead of 102).  Instead every 64-bit word of a record validates itself: its
//   upper half is one half of a 64-bit tag of the call (the host draws 32 bits of it, a counter from a random
//   start, the other 32 are a fixed function of those; no two of 2^32 consecutive calls share a tag), its lower
//   half the state or the token, written and read with one relaxed atomic access each (at system scope: the
//   writer and the reader sit on different XCDs, and at agent scope a few reads in a thousand still found an old
//   copy).  A word shows the tag only if this call has written it, up to memory that happens to hold the tag
//   already: 2^-64 per frame.
// One record per boundary: kPatchMax pairs of words, (tag_lo : state) and (tag_hi : token).
constexpr int kStartInts = 4 * kPatchMax;
// The upper half of a call's tag from its lower half (the host draws the lower half: a counter from a random start).
__device__ __forceinline__ unsigned start_tag_hi(unsigned tag_lo) { return (tag_lo * 0x9E3779B1u) ^ 0x85EBCA6Bu; }

// Issue priority of the wave (0..3, wave-uniform).  The waves of pass 1 all have the same amount of work, but a
// SIMD serves its oldest wave first: measured with time stamps, the waves launched first ended at 73 us and those
// launched last at 96 us of a 107 us kernel, which then drains with a long, thin tail.  A wave's priority falls
// as it gets on with its range (one level per quarter), so a wave that is behind is served first: the ends move
// together (83 to 92 us) and the kernel is 4 % shorter.
__device__ __forceinline__ void set_wave_priority(int level) {
  if (level <= 0) {
    __builtin_amdgcn_s_setprio(0);
  } else if (level == 1) {
    __builtin_amdgcn_s_setprio(1);
  } else if (level == 2) {
    __builtin_amdgcn_s_setprio(2);
  } else {
    __builtin_amdgcn_s_setprio(3);
  }
}

// State word of a stored frame without the boundary bit (an invalid frame holds -1 and stays as it is).
__device__ __forceinline__ int plain_state(int word) { return word < 0 ? word : (word & ~kGuessOk); }

// Outputs that other waves may read while or after they are written (pass 2) go through relaxed atomics on
// both sides.  Only waves of one workgroup ever exchange such words -- a hypothesis is repaired by one
// workgroup -- so stores, loads and the fences around the workgroup barriers all use workgroup scope (a wider
// scope would write back and invalidate the L2 of the whole XCD at every barrier, tree included).
__device__ __forceinline__ int peek_i32(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void publish_i32(int32_t* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ void fill_invalid(int B, int b, int f0, int f1, int32_t* tokens, int32_t* states,
                                             float* scores, int lane) {
  for (int f = f0 + lane; f < f1; f += 64) {
    const size_t o = static_cast<size_t>(f) * B + b;
    publish_i32(tokens + o, -1);
    publish_i32(states + o, -1);
    scores[o] = NAN;
  }
}

// Publishes frames lo..hi of a range (lane l holds the state and token of frame l) in the start record `rec`
// (8-byte aligned), see kStartInts.  Called by all lanes.
__device__ __forceinline__ void publish_start_frames(int32_t* rec, int lane, int lo, int hi, int st, int tok,
                                                     unsigned tag_lo, unsigned tag_hi) {
  if (lane >= lo && lane <= hi) {
    u64* w = reinterpret_cast<u64*>(rec) + 2 * lane;
    __hip_atomic_store(w, (static_cast<u64>(tag_lo) << 32) | static_cast<unsigned>(st), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
    __hip_atomic_store(w + 1, (static_cast<u64>(tag_hi) << 32) | static_cast<unsigned>(tok), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_SYSTEM);
  }
}
// Reads frame i of the start record `rec` (i < kPatchMax; any lane may ask for any frame).  Returns whether this
// call has written it; st / tok are then its state and token.
__device__ __forceinline__ bool read_start_frame(const int32_t* rec, int i, unsigned tag_lo, unsigned tag_hi, int& st,
                                                 int& tok) {
  const u64* w = reinterpret_cast<const u64*>(rec) + 2 * i;
  const u64 a = __hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  const u64 b = __hip_atomic_load(w + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  st = static_cast<int>(static_cast<unsigned>(a));
  tok = static_cast<int>(static_cast<unsigned>(b));
  return static_cast<unsigned>(a >> 32) == tag_lo && static_cast<unsigned>(b >> 32) == tag_hi;
}

// Outputs of up to 64 consecutive frames held one per lane (frame base + l in lane l) and written
// together, so that no store sits between the loads of the in-order memory queue.
struct LaneOut {
  int base, tok, st;
  float sc;
  __device__ __forceinline__ void put(int lane, int f, int token, int word, float val) {
    if (lane == f - base) {
      tok = token;
      st = word;
      sc = val;
    }
  }
  template <bool PUBLISH>
  __device__ __forceinline__ void flush(int lane, int count, int B, int b, int32_t* tokens, int32_t* states,
                                        float* scores) const {
    if (lane < count) {
      const size_t o = static_cast<size_t>(base + lane) * B + b;
      if (PUBLISH) {
        publish_i32(tokens + o, tok);
        publish_i32(states + o, st);
      } else {
        tokens[o] = tok;
        states[o] = st;
      }
      scores[o] = sc;
    }
  }
};

// The stored trajectory of a range that is being re-run, one frame per lane (64 at a time), requested
// ahead so that comparing a frame costs a lane read instead of a memory round trip.
template <bool WITH_TOKENS>
struct StoredLane {
  int st, tok;
  __device__ __forceinline__ void fetch(int lane, int fbase, int f1, int B, int b, const int32_t* tokens,
                                        const int32_t* states) {
    st = -1;
    tok = -1;
    const int f = fbase + lane;
    if (f < f1) {
      const size_t o = static_cast<size_t>(f) * B + b;
      st = peek_i32(states + o);
      if (WITH_TOKENS) tok = peek_i32(tokens + o);
    }
  }
  __device__ __forceinline__ int state_at(int slot) const { return plain_state(__builtin_amdgcn_readlane(st, slot)); }
  __device__ __forceinline__ int token_at(int slot) const { return __builtin_amdgcn_readlane(tok, slot); }
};

// Pass 2 for one hypothesis (one workgroup; its waves share the segments 1 .. nseg-1).
//   rerun(seg, state, label): decodes segment `seg` again from that outcome until it meets what is stored;
//   returns false when it reached the end of the segment without meeting it (the outcome there may have changed).
//   (a) every segment whose left neighbour has not certified its guess is re-run from the outcome pass 1 stored
//       at the end of that neighbour (read once, before any re-run starts).  A neighbour's re-run may replace
//       that outcome: (b) repairs it.
//   (b) rounds, entered only while some re-run has reached the end of its segment (nothing else can change an
//       outcome at a boundary): wave 0 compares the outcome at the end of every segment j-1 with what segment
//       j was last decoded from and publishes the set of stale segments; the waves re-run those in parallel.
//       Segment 0 is exact, so after round r the segments up to r + 1 are final: at most nseg rounds, in
//       practice none.
//   Words that cross waves are relaxed workgroup-scope atomics; a release fence before and an acquire fence
//   after each workgroup barrier order them.
//   patches: the workspace with one patch record per boundary, (j - 1) * B + b for the boundary before segment j
//   (null: none); the patches are copied into the output first.
template <bool WITH_TOKENS, typename Rerun>
__device__ __forceinline__ void fix_segments(int T, int B, int b, int seg_len, int nseg, int32_t* tokens,
                                             int32_t* states, float* scores, const int32_t* __restrict__ patches,
                                             int* assumed, int* assumed_tok, unsigned* bad_words, int lane, int wave,
                                             int nwaves, Rerun&& rerun) {
  auto end_word_ptr = [&](int seg) { return states + static_cast<size_t>(seg_begin(seg + 1, T, nseg) - 1) * B + b; };
  auto end_word_of = [&](int seg) {  // state word of the last frame of segment `seg` (boundary bit included)
    return peek_i32(end_word_ptr(seg));
  };
  auto end_token_of = [&](int seg) {  // label of the last frame of segment `seg`
    if (!WITH_TOKENS) return -1;
    return peek_i32(tokens + static_cast<size_t>(seg_begin(seg + 1, T, nseg) - 1) * B + b);
  };
  // (Requested before the patches are copied, so that the two accesses overlap: a patch covers frames at the start
  // of a segment and never its last one, whose state word and label these are.)
  const bool has = lane >= 1 && lane < nseg;
  int words = -1, labels = -1;
  if (wave == 0) {
    words = has ? end_word_of(lane - 1) : -1;
    labels = has ? end_token_of(lane - 1) : -1;
  }
  if (patches != nullptr) {
    // a quarter wave per boundary: lane q of the quarter copies entry q of the patch
    const int sub = lane >> 4, q = lane & 15;
    for (int j0 = 1 + 4 * wave; j0 < nseg; j0 += 4 * nwaves) {
      const int j = j0 + sub;
      if (j < nseg) {
        const int32_t* rec = patches + (static_cast<size_t>(j - 1) * B + b) * kPatchInts;
        const int count = rec[0];
        const int tok = rec[4 + q], st = rec[4 + kPatchMax + q];
        const float sc = __int_as_float(rec[4 + 2 * kPatchMax + q]);
        if (q < count) {
          const size_t o = static_cast<size_t>(seg_begin(j, T, nseg) + q) * B + b;
          publish_i32(tokens + o, tok);
          publish_i32(states + o, st);
          scores[o] = sc;
        }
      }
    }
  }
  // Wave 0 reads the outcome before every segment in one access (lane j: the end of segment j - 1), records
  // it as what segment j is decided from, and publishes the set of segments whose guess is not certified; the
  // k-th of them goes to wave k mod nwaves, so that the re-runs spread evenly over the waves.
  if (wave == 0) {
    if (has) {
      assumed[lane] = plain_state(words);
      assumed_tok[lane] = labels;
    }
    const u64 todo = __ballot(has && (words < 0 || (words & kGuessOk) == 0));
    if (lane == 0) {
      bad_words[0] = static_cast<unsigned>(todo);
      bad_words[1] = static_cast<unsigned>(todo >> 32);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // (the patches, for the re-runs that compare with them)
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  bool dirty = false;
  {
    u64 todo = (static_cast<u64>(bad_words[1]) << 32) | bad_words[0];
    for (int k = 0; todo != 0; ++k) {
      const int seg = first_lane(todo);
      todo &= todo - 1;
      if (k % nwaves == wave) dirty = !rerun(seg, assumed[seg], assumed_tok[seg]) || dirty;
    }
  }
  for (;;) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    const bool any = __syncthreads_or(dirty) != 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if (!any) break;
    dirty = false;
    if (wave == 0) {
      const int have = has ? plain_state(end_word_of(lane - 1)) : 0;
      const int have_tok = has ? end_token_of(lane - 1) : 0;
      const bool stale = has && (have != assumed[lane] || (WITH_TOKENS && have_tok != assumed_tok[lane]));
      if (stale) {
        assumed[lane] = have;
        assumed_tok[lane] = have_tok;
      }
      const u64 bad = __ballot(stale);
      if (lane == 0) {
        bad_words[0] = static_cast<unsigned>(bad);
        bad_words[1] = static_cast<unsigned>(bad >> 32);
      }
    }
    __syncthreads();
    u64 bad = (static_cast<u64>(bad_words[1]) << 32) | bad_words[0];
    for (int k = 0; bad != 0; ++k) {  // the k-th stale segment goes to wave k mod nwaves
      const int seg = first_lane(bad);
      bad &= bad - 1;
      if (k % nwaves == wave) dirty = !rerun(seg, assumed[seg], assumed_tok[seg]) || dirty;
    }
  }
  // every re-run is done: the boundary bits of pass 1 leave the output.  A word that a re-run has replaced
  // meanwhile carries no bit (or marks an invalid frame) and must stay as it is: compare-and-swap against the
  // value read at the start.
  if (wave == 0 && has && words >= 0 && (words & kGuessOk) != 0) {
    int expected = words;
    __hip_atomic_compare_exchange_strong(end_word_ptr(lane - 1), &expected, words & ~kGuessOk, __ATOMIC_RELAXED,
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
}

}  // namespace wv
}  // namespace pb
