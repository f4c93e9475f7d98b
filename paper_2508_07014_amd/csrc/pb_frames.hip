// Wave-per-hypothesis greedy kernels (gfx950, wave64): the fused step and the multi-frame decoder.
//
// One wavefront owns one hypothesis row; nothing crosses waves, so there is no barrier on the path.
//
//  * Row streaming.  A row is consumed in chunks of 1024 tokens; lane l owns tokens
//    256*i + 4*l + {0..3}, i = 0..3 of a chunk, so each of the four 16-byte loads of a lane is part
//    of one contiguous 1 KiB wave access.  Chunks are prefetched two ahead into registers.
//  * Base candidates.  For every token that no chain state overrides the boost is
//    p_root + root_score[v] (all backoffs down to the root, then the root arc or the c_unk
//    self-loop).  alpha * that is cached per lane while p_root does not change, so the common
//    frame costs one add and a max per token.  The row max is reduced with DPP on order-preserving
//    integer keys; the winner is the lowest token index holding that value (fp32 compare).
//  * Arc candidates.  The failure chain is walked with scalar loads (the state is wave-uniform);
//    at each chain state the lanes take one arc each, gather its log-prob from the LDS copy of the
//    row and evaluate Eq. 1 for it.  A per-token LDS tag written with a per-(frame, chunk) stamp
//    marks overridden tokens: it hides arcs shadowed by a deeper chain state and tells whether the
//    base winner is itself overridden.  Only in that last case (and only if the arcs do not beat it
//    anyway) a second pass recomputes the base winner without the overridden tokens.
//  * Multi-frame decoding splits the T frames of a hypothesis into segments decoded concurrently,
//    every segment but the first speculatively from the root state.  The decoder is a finite
//    automaton step, so a re-run from the true start state needs to go only as far as the frame
//    where its state meets the speculative trajectory; a second kernel does these short re-runs
//    (all segments in parallel, from the neighbouring segment's end state) and then validates the
//    assumed start states in order, repairing where a re-run changed a segment's end state.
//    The result is identical to T sequential steps.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "pb_kernels.hpp"

namespace pb {

namespace {

#define PB_AS4 __attribute__((address_space(4)))

constexpr int kChunk = 1024;  // tokens per chunk: 16 per lane

// Scalar-load views: the tree is never written while kernels run, so wave-uniform reads may go
// through the constant address space (scalar cache).
typedef int v4i __attribute__((ext_vector_type(4)));

struct TreeView {
  const v4i PB_AS4* state;  // StateRec as four dwords: arc_begin, arc_count, fail, backoff bits
  const float PB_AS4* p_root;
  const int32_t PB_AS4* root_next;
  const ArcRec* arc;
  const float* root_score;
  int num_states, V, blank;
};

__device__ __forceinline__ TreeView make_view(const DeviceTree& t) {
  TreeView v;
  v.state = (const v4i PB_AS4*)t.state;
  v.p_root = (const float PB_AS4*)t.p_root;
  v.root_next = (const int32_t PB_AS4*)t.root_next;
  v.arc = t.arc;
  v.root_score = t.root_score;
  v.num_states = t.num_states;
  v.V = t.vocab_size;
  v.blank = t.blank_id;
  return v;
}

__device__ __forceinline__ int key_of(float f) {  // order-preserving fp32 -> int32 (an involution)
  const int b = __float_as_int(f);
  return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float val_of(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }

template <int CTRL>
__device__ __forceinline__ int dpp(int v) {
  return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
// Wave-wide max / min of an int; the result is wave-uniform (read from lane 63).
__device__ __forceinline__ int wave_max_i(int v) {
  v = max(v, dpp<0x111>(v));  // row_shr:1
  v = max(v, dpp<0x112>(v));  // row_shr:2
  v = max(v, dpp<0x114>(v));  // row_shr:4
  v = max(v, dpp<0x118>(v));  // row_shr:8
  v = max(v, dpp<0x142>(v));  // row_bcast:15
  v = max(v, dpp<0x143>(v));  // row_bcast:31
  return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_min_i(int v) {
  v = min(v, dpp<0x111>(v));
  v = min(v, dpp<0x112>(v));
  v = min(v, dpp<0x114>(v));
  v = min(v, dpp<0x118>(v));
  v = min(v, dpp<0x142>(v));
  v = min(v, dpp<0x143>(v));
  return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ int tok_of(int j, int lane) { return 256 * (j >> 2) + 4 * lane + (j & 3); }

struct Win {  // wave-uniform result of one chunk or frame
  float val;
  int tok;
  int next;
};

// Loads the lane's 16 log-probs of chunk `cb` (token base) of a row; tokens >= V read as -inf.
__device__ __forceinline__ void load_chunk(const float* __restrict__ lrow, int cb, int V, int lane, float (&x)[16]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = cb + 256 * i + 4 * lane;
    if (v < V) {  // V % 4 == 0: a 16-byte group is entirely inside or outside the row
      const float4 q = *reinterpret_cast<const float4*>(lrow + v);
      x[4 * i + 0] = q.x; x[4 * i + 1] = q.y; x[4 * i + 2] = q.z; x[4 * i + 3] = q.w;
    } else {
      x[4 * i + 0] = x[4 * i + 1] = x[4 * i + 2] = x[4 * i + 3] = -INFINITY;
    }
  }
}

// alpha * (p_root + root_score[v]) for the lane's tokens of a chunk; the blank column boosts by 0.
__device__ __forceinline__ void make_base_boost(const TreeView& t, int cb, int lane, float p_root, float alpha,
                                                float (&c)[16]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = cb + 256 * i + 4 * lane;
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (v < t.V) r = *reinterpret_cast<const float4*>(t.root_score + v);
    const float rs[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float boost = (v + k == t.blank) ? 0.0f : __fadd_rn(p_root, rs[k]);
      c[4 * i + k] = __fmul_rn(alpha, boost);
    }
  }
}

// One chunk of one row for a valid state s: the best token of the chunk by (fused value descending,
// token ascending), its fused value and the state it leads to.
//   x      lane's raw log-probs of the chunk (registers)
//   c      lane's base boosts for (s, chunk) (registers)
//   row    this wave's LDS copy of the chunk (written here when the state has a chain)
//   tag    this wave's LDS tags; `stamp` must be unique per call
template <typename AfterArcs>
__device__ __forceinline__ Win decide_chunk(const TreeView& t, int s, int cb, const float (&x)[16], const float (&c)[16],
                                            float alpha, float* row, unsigned* tag, unsigned stamp, int lane,
                                            AfterArcs&& after_arcs) {
  // ---- base candidates ---------------------------------------------------------------------------
  float f[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) f[j] = __fadd_rn(x[j], c[j]);
  float m = f[0];
#pragma unroll
  for (int j = 1; j < 16; ++j) m = fmaxf(m, f[j]);
  const float M = val_of(wave_max_i(key_of(m)));
  int loc = INT_MAX;
#pragma unroll
  for (int j = 15; j >= 0; --j) loc = (f[j] == M) ? tok_of(j, lane) : loc;
  int vb = wave_min_i(loc);
  if (vb == INT_MAX) vb = 0;  // only with NaN inputs (precondition violation): stay in range

  // ---- arc candidates along the failure chain ----------------------------------------------------
  bool have_arcs = false;
  float bf = 0.0f;
  int bk = INT_MIN, btok = INT_MAX, bchild = 0;
  if (s != 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<float4*>(row + 256 * i + 4 * lane) = make_float4(x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]);
    float p = 0.0f;
    int xs = s, level = 0;
    while (xs != 0) {
      const v4i raw = t.state[xs];
      StateRec r;
      r.arc_begin = raw.x;
      r.arc_count = raw.y;
      r.fail = raw.z;
      r.backoff = __int_as_float(raw.w);
      for (int j0 = 0; j0 < r.arc_count; j0 += 64) {
        const int j = j0 + lane;
        if (j < r.arc_count) {
          const ArcRec a = t.arc[r.arc_begin + j];
          const unsigned rel = static_cast<unsigned>(a.token - cb);
          if (rel < static_cast<unsigned>(kChunk)) {
            bool shadowed = false;
            if (level > 0) shadowed = (tag[rel] == stamp);  // a deeper chain state owns this token
            tag[rel] = stamp;
            if (!shadowed) {
              const float fa = __fadd_rn(row[rel], __fmul_rn(alpha, __fadd_rn(p, a.score)));
              if (bk == INT_MIN || fa > bf || (fa == bf && static_cast<int>(rel) < btok)) {
                bf = fa;
                bk = key_of(fa);
                btok = static_cast<int>(rel);
                bchild = r.arc_begin + j + 1;
              }
            }
          }
        }
      }
      have_arcs = have_arcs || r.arc_count > 0;
      p = __fadd_rn(p, r.backoff);
      xs = r.fail;
      ++level;
    }
  }
  after_arcs();

  Win w;
  bool arc_wins = false;
  int va = INT_MAX, achild = 0;
  float MA = 0.0f;
  bool have_cand = false;
  if (have_arcs) {
    const int ak = wave_max_i(bk);
    if (ak != INT_MIN) {  // some arc fell into this chunk
      have_cand = true;
      MA = val_of(ak);
      const bool mine = (bk != INT_MIN) && (bf == MA);
      va = wave_min_i(mine ? btok : INT_MAX);
      const unsigned long long who = __ballot(mine && btok == va);
      achild = __builtin_amdgcn_readlane(bchild, __ffsll(static_cast<long long>(who)) - 1);
    }
  }
  float base_val = M;
  int base_tok = vb;
  bool have_base = true;
  if (have_cand) {
    const bool vb_overridden = __builtin_amdgcn_readfirstlane(static_cast<int>(tag[vb] == stamp)) != 0;
    if (MA > M) {
      arc_wins = true;
    } else if (!vb_overridden) {
      arc_wins = (MA == M) && (va < vb);
    } else {
      // The base winner is shadowed by an arc that does not beat it: redo the base arg-max without
      // the overridden tokens.
      int k[16];
      int mk = INT_MIN;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        k[j] = (tag[tok_of(j, lane)] == stamp) ? INT_MIN : key_of(f[j]);
        mk = max(mk, k[j]);
      }
      const int Mk = wave_max_i(mk);
      if (Mk == INT_MIN) {
        have_base = false;
      } else {
        base_val = val_of(Mk);
        int l2 = INT_MAX;
#pragma unroll
        for (int j = 15; j >= 0; --j) l2 = (k[j] != INT_MIN && f[j] == base_val) ? tok_of(j, lane) : l2;
        base_tok = wave_min_i(l2);
        if (base_tok == INT_MAX) have_base = false;
      }
      arc_wins = !have_base || MA > base_val || (MA == base_val && va < base_tok);
    }
  }
  if (arc_wins) {
    w.val = MA;
    w.tok = cb + va;
    w.next = achild;
  } else {
    w.val = base_val;
    w.tok = cb + base_tok;
    w.next = (w.tok == t.blank) ? s : t.root_next[w.tok];
  }
  return w;
}

__device__ __forceinline__ bool valid_state(const TreeView& t, int s) {
  return static_cast<unsigned>(s) < static_cast<unsigned>(t.num_states);
}

// Decodes frames [f0, f1) of hypothesis b starting in state s (valid).  With `compare` set, stops
// after the first frame whose out-state equals the one already stored in `states` (the stored
// trajectory is then valid from there on).  Returns the state after the last decoded frame; *met
// tells whether the stored trajectory was met before f1.
template <bool COMPARE>
__device__ __forceinline__ int run_frames(const TreeView& t, const float* __restrict__ logp, int64_t frame_stride,
                                          int64_t row_stride, float alpha, int B, int b, int f0, int f1, int s,
                                          int32_t* __restrict__ tokens, int32_t* __restrict__ states,
                                          float* __restrict__ scores, float* row, unsigned* tag, unsigned& stamp,
                                          int lane, bool* met) {
  const int V = t.V;
  const int nch = (V + kChunk - 1) / kChunk;
  const int total = (f1 - f0) * nch;
  const float* base_ptr = logp + static_cast<size_t>(b) * row_stride;
  float buf[3][16];
  float c[16];
  float c_p = 0.0f;
  int c_chunk = -1;  // (p_root, chunk) the cached base boosts belong to
  auto issue = [&](int q, float (&dst)[16]) {
    const int f = f0 + q / nch, ch = q - (q / nch) * nch;
    load_chunk(base_ptr + static_cast<size_t>(f) * frame_stride, ch * kChunk, V, lane, dst);
  };
  if (total > 0) issue(0, buf[0]);
  if (total > 1) issue(1, buf[1]);
  Win best{0.0f, -1, s};
  bool stop = false;
  if (met) *met = false;
  for (int q0 = 0; q0 < total && !stop; q0 += 3) {
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      const int q = q0 + u;
      if (q < total && !stop) {
        const int f = f0 + q / nch, ch = q - (q / nch) * nch;
        const float p_root = t.p_root[s];
        if (c_chunk != ch || __float_as_int(c_p) != __float_as_int(p_root)) {
          make_base_boost(t, ch * kChunk, lane, p_root, alpha, c);
          c_chunk = ch;
          c_p = p_root;
        }
        const Win w = decide_chunk(t, s, ch * kChunk, buf[u], c, alpha, row, tag, ++stamp, lane, [&]() {
          if (!COMPARE && q + 2 < total) issue(q + 2, buf[(u + 2) % 3]);
        });
        if (COMPARE && q + 2 < total) issue(q + 2, buf[(u + 2) % 3]);
        if (best.tok < 0 || w.val > best.val) best = w;  // chunks ascend, so ties keep the lower token
        if (ch == nch - 1) {
          const size_t o = static_cast<size_t>(f) * B + b;
          int stored = 0;
          if (COMPARE) stored = states[o];
          if (lane == 0) {
            tokens[o] = best.tok;
            states[o] = best.next;
            scores[o] = best.val;
          }
          s = best.next;
          best.tok = -1;
          if (COMPARE && __builtin_amdgcn_readfirstlane(stored) == s) {
            stop = true;
            if (met) *met = true;
          }
        }
      }
    }
  }
  return s;
}

__device__ __forceinline__ void fill_invalid(int B, int b, int f0, int f1, int32_t* tokens, int32_t* states,
                                             float* scores, int lane) {
  for (int f = f0 + lane; f < f1; f += 64) {
    const size_t o = static_cast<size_t>(f) * B + b;
    tokens[o] = -1;
    states[o] = -1;
    scores[o] = NAN;
  }
}

__device__ __forceinline__ void clear_tags(unsigned* tag, int lane) {
#pragma unroll
  for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(tag + 256 * i + 4 * lane) = make_uint4(0u, 0u, 0u, 0u);
}

// Pass 1: chain (b, j) decodes segment j of hypothesis b; j = 0 starts from states0[b] (exact),
// j > 0 from the root (speculative).  One wave per chain.
__global__ void __launch_bounds__(256) frames_spec_kernel(DeviceTree dt, const float* __restrict__ logp,
                                                          int64_t frame_stride, int64_t row_stride,
                                                          const int32_t* __restrict__ states0, float alpha, int T, int B,
                                                          int seg_len, int nseg, int32_t* __restrict__ tokens,
                                                          int32_t* __restrict__ states, float* __restrict__ scores) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chain = blockIdx.x * (blockDim.x >> 6) + wave;
  if (chain >= B * nseg) return;
  const int j = chain / B, b = chain - j * B;
  float* row = lds + wave * 2 * kChunk;
  unsigned* tag = reinterpret_cast<unsigned*>(row + kChunk);
  clear_tags(tag, lane);
  const TreeView t = make_view(dt);
  const int f0 = j * seg_len, f1 = min(T, f0 + seg_len);
  int s = 0;
  if (j == 0) {
    s = states0[b];
    if (!valid_state(t, s)) {
      fill_invalid(B, b, f0, f1, tokens, states, scores, lane);
      return;
    }
  }
  unsigned stamp = 0;
  run_frames<false>(t, logp, frame_stride, row_stride, alpha, B, b, f0, f1, s, tokens, states, scores, row, tag, stamp,
                    lane, nullptr);
}

// Pass 2: one workgroup per hypothesis, wave j owns segment j.
//   (a) every wave j > 0 re-runs its segment from the end state pass 1 left in segment j-1 until the
//       stored trajectory is met;
//   (b) wave 0 then walks the segments in order: if the end state of segment j-1 is no longer the
//       state wave j started from, segment j is re-run from the true state the same way.
__global__ void __launch_bounds__(1024) frames_fix_kernel(DeviceTree dt, const float* __restrict__ logp,
                                                          int64_t frame_stride, int64_t row_stride, float alpha, int T,
                                                          int B, int seg_len, int nseg, int32_t* __restrict__ tokens,
                                                          int32_t* __restrict__ states, float* __restrict__ scores) {
  extern __shared__ float lds[];
  __shared__ int assumed[16];
  const int lane = threadIdx.x & 63, j = threadIdx.x >> 6;
  const int b = blockIdx.x;
  float* row = lds + j * 2 * kChunk;
  unsigned* tag = reinterpret_cast<unsigned*>(row + kChunk);
  clear_tags(tag, lane);
  const TreeView t = make_view(dt);
  unsigned stamp = 0;
  auto rerun = [&](int seg, int s) {
    const int f0 = seg * seg_len, f1 = min(T, f0 + seg_len);
    if (!valid_state(t, s)) {
      fill_invalid(B, b, f0, f1, tokens, states, scores, lane);
      return;
    }
    run_frames<true>(t, logp, frame_stride, row_stride, alpha, B, b, f0, f1, s, tokens, states, scores, row, tag,
                     stamp, lane, nullptr);
  };
  if (j > 0 && j < nseg) {
    const int s = states[static_cast<size_t>(j * seg_len - 1) * B + b];
    if (lane == 0) assumed[j] = s;
    if (s != 0) rerun(j, s);  // pass 1 assumed the root
  }
  __threadfence_block();
  __syncthreads();
  if (j == 0) {
    for (int seg = 1; seg < nseg; ++seg) {
      const int32_t* p = states + static_cast<size_t>(seg * seg_len - 1) * B + b;
      const int true_start = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (true_start != assumed[seg]) rerun(seg, true_start);
    }
  }
}

// Single step: one wave per hypothesis, no speculation.
__global__ void __launch_bounds__(256) step_wave_kernel(DeviceTree dt, const float* __restrict__ logp, int64_t row_stride,
                                                        const int32_t* __restrict__ states_in, float alpha, int B,
                                                        int32_t* __restrict__ tokens, int32_t* __restrict__ states_out,
                                                        float* __restrict__ scores) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b = blockIdx.x * (blockDim.x >> 6) + wave;
  if (b >= B) return;
  float* row = lds + wave * 2 * kChunk;
  unsigned* tag = reinterpret_cast<unsigned*>(row + kChunk);
  clear_tags(tag, lane);
  const TreeView t = make_view(dt);
  const int s = states_in[b];
  if (!valid_state(t, s)) {
    fill_invalid(B, b, 0, 1, tokens, states_out, scores, lane);
    return;
  }
  unsigned stamp = 0;
  run_frames<false>(t, logp, 0, row_stride, alpha, B, b, 0, 1, s, tokens, states_out, scores, row, tag, stamp, lane,
                    nullptr);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

bool wave_path_ok(const DeviceTree& t, const float* d_logp, int64_t frame_stride, int64_t row_stride) {
  return t.p_root != nullptr && t.vocab_size % 4 == 0 && row_stride % 4 == 0 && frame_stride % 4 == 0 &&
         aligned16(d_logp) && aligned16(t.root_score);
}

int launch_step_wave(const DeviceTree& t, const float* d_logp, int64_t row_stride, const int32_t* d_states_in,
                     float alpha, int32_t B, int32_t* d_tokens, int32_t* d_states_out, float* d_scores,
                     hipStream_t stream) {
  const int waves = B >= 1024 ? 4 : 1;  // few rows: spread them over as many CUs as possible
  const dim3 grid(static_cast<unsigned>((B + waves - 1) / waves)), block(static_cast<unsigned>(64 * waves));
  const size_t lds = static_cast<size_t>(waves) * 2 * kChunk * sizeof(float);
  hipLaunchKernelGGL(step_wave_kernel, grid, block, lds, stream, t, d_logp, row_stride, d_states_in, alpha, B, d_tokens,
                     d_states_out, d_scores);
  return hipGetLastError() == hipSuccess ? PB_OK : PB_EHIP;
}

int launch_frames_wave(const DeviceTree& t, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                       const int32_t* d_states0, float alpha, int32_t T, int32_t B, int32_t* d_tokens,
                       int32_t* d_states, float* d_scores, hipStream_t stream) {
  // Segments: enough concurrent chains to cover the memory latency, at most 16 per hypothesis
  // (one wave each in the fix-up workgroup), at least kMinSegLen frames long.
  int nseg = (kTargetChains + B - 1) / B;
  nseg = nseg < 1 ? 1 : (nseg > 16 ? 16 : nseg);
  int seg_len = (T + nseg - 1) / nseg;
  if (seg_len < kMinSegLen) seg_len = kMinSegLen;
  nseg = (T + seg_len - 1) / seg_len;
  const int64_t chains = static_cast<int64_t>(B) * nseg;
  const int waves = 4;
  const int64_t blocks = (chains + waves - 1) / waves;
  if (blocks > INT32_MAX) return PB_EUNSUPPORTED;
  const size_t lds = static_cast<size_t>(waves) * 2 * kChunk * sizeof(float);
  hipLaunchKernelGGL(frames_spec_kernel, dim3(static_cast<unsigned>(blocks)), dim3(64 * waves), lds, stream, t, d_logp,
                     frame_stride, row_stride, d_states0, alpha, T, B, seg_len, nseg, d_tokens, d_states, d_scores);
  if (hipGetLastError() != hipSuccess) return PB_EHIP;
  if (nseg > 1) {
    const size_t lds2 = static_cast<size_t>(nseg) * 2 * kChunk * sizeof(float);
    hipLaunchKernelGGL(frames_fix_kernel, dim3(static_cast<unsigned>(B)), dim3(64 * nseg), lds2, stream, t, d_logp,
                       frame_stride, row_stride, alpha, T, B, seg_len, nseg, d_tokens, d_states, d_scores);
    if (hipGetLastError() != hipSuccess) return PB_EHIP;
  }
  return PB_OK;
}

int prepare_wave_kernels() {
  // the fix-up workgroup may need more than the default 64 KiB of dynamic LDS (16 waves x 8 KiB)
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(frames_fix_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 16 * 2 * kChunk * 4);
  return e == hipSuccess ? PB_OK : PB_EHIP;
}

}  // namespace pb
