// HIP kernels (gfx950, wave64) of the phrase-boosting tree: whole-vocabulary query, fused greedy
// step, multi-frame greedy decoding and the beam step.
//
// Common scheme ("row build").  The boost row of one hypothesis is assembled in LDS as one 64-bit
// entry per token, (next_state << 32) | fp32 bits of the score.  The failure chain of the state is
// walked once per workgroup; at every chain state the lanes take one outgoing arc each and merge
// (child id, accumulated backoff + arc score) into the token's entry with a 64-bit LDS max.
// Because states are numbered breadth-first, a child of a deeper chain state always has a larger
// id than a child of a shallower one, so the max keeps exactly the arc the per-token failure-link
// walk would have found first (Sec. II-B; Alg. 1 Stage 3 get_scores).  Tokens with no entry fall
// through to the dense root row (real root arc or the c_unk self-loop).  Work per row is
// V + (arcs on the chain), independent of how the arcs are spread over the chain states.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdint>

#include "pb_kernels.hpp"

namespace pb {

namespace {

using u64 = unsigned long long;

__device__ __forceinline__ u64 pack_entry(int next, float score) {
  return (static_cast<u64>(static_cast<unsigned>(next)) << 32) | __float_as_uint(score);
}

// Merges the arcs of the failure chain of `s` whose token lies in [v0, v0 + n) into `row`, and
// returns the backoff accumulated down to the root (fp32, chain order).  `row` must be zeroed and
// the zeroing visible (barrier) before the call; entries are final after the next barrier.
__device__ __forceinline__ float scatter_chain(const DeviceTree& t, int s, int v0, int n, u64* row) {
  float p = 0.0f;
  int x = s;
  while (x != 0) {
    // One record holds the state and the state its failure link leads to: the arcs of both levels are requested
    // in one sweep (two chain levels per pair of dependent accesses instead of one).
    const StateRec r = t.state[x];
    const int c0 = r.arc_count, c1 = r.fail != 0 ? r.f_arc_count : 0;
    const float p1 = __fadd_rn(p, r.backoff);
    for (int j = threadIdx.x; j < c0 + c1; j += blockDim.x) {
      const bool second = j >= c0;
      const int idx = second ? r.f_arc_begin + (j - c0) : r.arc_begin + j;
      const ArcRec a = t.arc[idx];
      const unsigned rel = static_cast<unsigned>(a.token - v0);
      if (rel < static_cast<unsigned>(n)) atomicMax(&row[rel], pack_entry(idx + 1, __fadd_rn(second ? p1 : p, a.score)));
    }
    if (r.fail == 0) return p1;
    p = __fadd_rn(p1, r.f_backoff);
    x = r.f_fail;
  }
  return p;
}

// (score, next) of token v from its LDS entry, the root row and the blank rule.
__device__ __forceinline__ void resolve(const DeviceTree& t, int s, float p_root, u64 e, int v, float root_score,
                                        int root_next, float& score, int& next) {
  const unsigned hi = static_cast<unsigned>(e >> 32);
  if (hi != 0u) {
    next = static_cast<int>(hi);
    score = __uint_as_float(static_cast<unsigned>(e));
  } else {
    next = root_next;
    score = __fadd_rn(p_root, root_score);
  }
  if (v == t.blank_id) {
    score = 0.0f;
    next = s;
  }
  if (v == t.eos_id) {  // EOS rule (Sec. II-C): tabulated per state by the host compiler; the state does not move
    score = t.eos_score[s];
    next = s;
  }
}

__device__ __forceinline__ bool better(float a_val, int a_idx, float b_val, int b_idx) {
  return a_val > b_val || (a_val == b_val && a_idx < b_idx);
}

// Workgroup-wide arg-max of (val, idx) by (val descending, idx ascending); idx < 0 marks "nothing".
// Every thread returns the winning (val, idx).  `sv`/`si` hold one slot per wave.
__device__ __forceinline__ void block_best(float& val, int& idx, float* sv, int* si) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(val, off, 64);
    const int oi = __shfl_xor(idx, off, 64);
    if (oi >= 0 && (idx < 0 || better(ov, oi, val, idx))) {
      val = ov;
      idx = oi;
    }
  }
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();  // previous users of sv/si are done
  if ((threadIdx.x & 63) == 0) {
    sv[wave] = val;
    si[wave] = idx;
  }
  __syncthreads();
  val = sv[0];
  idx = si[0];
  for (int w = 1; w < nw; ++w) {
    const float ov = sv[w];
    const int oi = si[w];
    if (oi >= 0 && (idx < 0 || better(ov, oi, val, idx))) {
      val = ov;
      idx = oi;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// pb_score: one workgroup per (group of `per` consecutive hypotheses, vocabulary tile).  The tile of
// the dense root row is read once per workgroup and kept in registers (VEC == 4: up to 8 tokens per
// thread).  A hypothesis in the root state has no chain: its row is
// the root row itself and skips LDS and barriers.
template <int VEC>
__global__ void __launch_bounds__(256) score_kernel(DeviceTree t0, TreePick pick, const int32_t* __restrict__ states,
                                                    int B, float* __restrict__ scores, int32_t* __restrict__ next,
                                                    int tile, int tiles, int per) {
  extern __shared__ u64 row[];
  const int grp = blockIdx.x / tiles;
  const int v0 = (blockIdx.x - grp * tiles) * tile;
  const int V = t0.vocab_size;
  const int n = min(tile, V - v0);
  DeviceTree t = t0;
  if (!pick_tree(pick, grp, t)) {  // with a table of trees every workgroup has one hypothesis (per == 1)
    const size_t base = static_cast<size_t>(grp) * V + v0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
      scores[base + i] = NAN;
      if (next) next[base + i] = -1;
    }
    return;
  }
  constexpr int kMaxSlots = kScoreTile / (256 * 4);  // float4 groups per thread
  float4 rs[kMaxSlots];
  int4 rn[kMaxSlots];
  if constexpr (VEC == 4) {
#pragma unroll
    for (int q = 0; q < kMaxSlots; ++q) {
      const int i = (q * 256 + static_cast<int>(threadIdx.x)) * 4;
      if (i < n) {
        rs[q] = *reinterpret_cast<const float4*>(t.root_score + v0 + i);
        rn[q] = *reinterpret_cast<const int4*>(t.root_next + v0 + i);
      }
    }
  }
  const int b_end = min(B, (grp + 1) * per);
  for (int b = grp * per; b < b_end; ++b) {
    const int s = states[b];
    const size_t base = static_cast<size_t>(b) * V + v0;
    if (static_cast<unsigned>(s) >= static_cast<unsigned>(t.num_states)) {
      for (int i = threadIdx.x; i < n; i += blockDim.x) {
        scores[base + i] = NAN;
        if (next) next[base + i] = -1;
      }
      continue;
    }
    const bool chain = s != 0;  // uniform over the workgroup
    float p_root = 0.0f;
    if (chain) {
      __syncthreads();  // everyone has read the previous hypothesis' entries
      for (int i = threadIdx.x; i < n; i += blockDim.x) row[i] = 0ull;
      __syncthreads();
      p_root = scatter_chain(t, s, v0, n, row);
      __syncthreads();
    }
    if constexpr (VEC == 4) {
#pragma unroll
      for (int q = 0; q < kMaxSlots; ++q) {
        const int i = (q * 256 + static_cast<int>(threadIdx.x)) * 4;
        if (i < n) {
          const float rsa[4] = {rs[q].x, rs[q].y, rs[q].z, rs[q].w};
          const int rna[4] = {rn[q].x, rn[q].y, rn[q].z, rn[q].w};
          float sc[4];
          int nx[4];
#pragma unroll
          for (int k = 0; k < 4; ++k)
            resolve(t, s, p_root, chain ? row[i + k] : 0ull, v0 + i + k, rsa[k], rna[k], sc[k], nx[k]);
          typedef float vf4 __attribute__((ext_vector_type(4)));
          typedef int vi4 __attribute__((ext_vector_type(4)));
          const vf4 so = {sc[0], sc[1], sc[2], sc[3]};
          const vi4 no = {nx[0], nx[1], nx[2], nx[3]};
          *reinterpret_cast<vf4*>(scores + base + i) = so;
          if (next) *reinterpret_cast<vi4*>(next + base + i) = no;
        }
      }
    } else {
      for (int i = threadIdx.x; i < n; i += blockDim.x) {
        float sc;
        int nx;
        resolve(t, s, p_root, chain ? row[i] : 0ull, v0 + i, t.root_score[v0 + i], t.root_next[v0 + i], sc, nx);
        scores[base + i] = sc;
        if (next) next[base + i] = nx;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Fused row: boost row in LDS, Eq. 1 per token, per-thread running best.  All threads of the
// workgroup must call it (barriers inside).  On return (best, best_v, best_next) is the thread's
// own partial result; best_v < 0 if the thread saw no token.
// Tokens equal to `excl_a` or `excl_b` are not candidates (-1 = none): the two-stage selection rules
// bar the blank, and under the CTC rule the previous label, from the boosted re-selection.
// The EOS column, where the tree has one, comes out of `resolve` like any other token.
template <int VEC>
__device__ __forceinline__ void fused_row(const DeviceTree& t, const float* __restrict__ lrow, int s, float alpha,
                                          u64* row, int chunk, int excl_a, int excl_b, float& best, int& best_v,
                                          int& best_next) {
  const int V = t.vocab_size;
  best = 0.0f;
  best_v = -1;
  best_next = s;
  for (int v0 = 0; v0 < V; v0 += chunk) {
    const int n = min(chunk, V - v0);
    if (v0 > 0) __syncthreads();  // everyone has read the previous chunk
    for (int i = threadIdx.x; i < n; i += blockDim.x) row[i] = 0ull;
    __syncthreads();
    const float p_root = scatter_chain(t, s, v0, n, row);
    __syncthreads();
    if constexpr (VEC == 4) {
      for (int i = threadIdx.x * 4; i < n; i += blockDim.x * 4) {
        const float4 lp = *reinterpret_cast<const float4*>(lrow + v0 + i);
        const float4 rs = *reinterpret_cast<const float4*>(t.root_score + v0 + i);
        const int4 rn = *reinterpret_cast<const int4*>(t.root_next + v0 + i);
        const float lpa[4] = {lp.x, lp.y, lp.z, lp.w};
        const float rsa[4] = {rs.x, rs.y, rs.z, rs.w};
        const int rna[4] = {rn.x, rn.y, rn.z, rn.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float sc;
          int nx;
          resolve(t, s, p_root, row[i + k], v0 + i + k, rsa[k], rna[k], sc, nx);
          const float fused = __fadd_rn(lpa[k], __fmul_rn(alpha, sc));
          const int v = v0 + i + k;
          if (v != excl_a && v != excl_b && (best_v < 0 || fused > best)) {
            best = fused;
            best_v = v;
            best_next = nx;
          }
        }
      }
    } else {
      for (int i = threadIdx.x; i < n; i += blockDim.x) {
        float sc;
        int nx;
        resolve(t, s, p_root, row[i], v0 + i, t.root_score[v0 + i], t.root_next[v0 + i], sc, nx);
        const float fused = __fadd_rn(lrow[v0 + i], __fmul_rn(alpha, sc));
        const int v = v0 + i;
        if (v != excl_a && v != excl_b && (best_v < 0 || fused > best)) {
          best = fused;
          best_v = v;
          best_next = nx;
        }
      }
    }
  }
}

// pb_fuse_step / pb_fuse_frames, any row shape: one workgroup per hypothesis; T frames are walked in
// sequence with the state (and, under the CTC rule, the previous label) carried in registers.
// sel: 0 single-stage, 1 two-stage, 2 two-stage with the CTC repeat rule (Sec. II-C).
template <int VEC>
__global__ void __launch_bounds__(1024) fuse_kernel(DeviceTree t0, TreePick pick, const float* __restrict__ logp,
                                                    int64_t frame_stride, int64_t row_stride,
                                                    const int32_t* __restrict__ states0,
                                                    const int32_t* __restrict__ last0, float alpha, int T, int B, int sel,
                                                    int32_t* __restrict__ tokens, int32_t* __restrict__ states,
                                                    float* __restrict__ scores, int chunk) {
  extern __shared__ u64 row[];
  __shared__ float sv[16];
  __shared__ int si[16];
  __shared__ int s_next;
  const int b = blockIdx.x;
  DeviceTree t = t0;
  const bool tree_ok = pick_tree(pick, b, t);
  const int V = t.vocab_size;
  int s = tree_ok ? states0[b] : -1;  // an unknown tree marks the hypothesis like an invalid state
  int last = (sel == 2 && last0 != nullptr) ? last0[b] : -1;
  for (int f = 0; f < T; ++f) {
    const size_t o = static_cast<size_t>(f) * B + b;
    if (static_cast<unsigned>(s) >= static_cast<unsigned>(t.num_states)) {
      if (threadIdx.x == 0) {
        tokens[o] = -1;
        states[o] = -1;
        scores[o] = NAN;
      }
      s = -1;
      continue;
    }
    const float* lrow = logp + static_cast<size_t>(f) * frame_stride + static_cast<size_t>(b) * row_stride;
    if (sel != 0) {
      // stage 1: arg-max of the acoustic row alone; a blank or a CTC repeat is emitted as it is
      float m = 0.0f;
      int mv = -1;
      for (int v = threadIdx.x; v < V; v += blockDim.x) {
        const float x = lrow[v];
        if (mv < 0 || x > m) {
          m = x;
          mv = v;
        }
      }
      block_best(m, mv, sv, si);
      if (mv == t.blank_id || (sel == 2 && mv == last)) {
        if (threadIdx.x == 0) {
          tokens[o] = mv;
          states[o] = s;
          scores[o] = m;
        }
        last = mv;
        continue;
      }
    }
    float best;
    int best_v, best_next;
    const int excl_a = sel != 0 ? t.blank_id : -1, excl_b = sel == 2 ? last : -1;
    fused_row<VEC>(t, lrow, s, alpha, row, chunk, excl_a, excl_b, best, best_v, best_next);
    float win = best;
    int win_v = best_v;
    block_best(win, win_v, sv, si);
    if (best_v == win_v) {  // exactly one thread owns the winning token
      tokens[o] = win_v;
      states[o] = best_next;
      scores[o] = win;
      s_next = best_next;
    }
    __syncthreads();
    s = s_next;
    last = win_v;
  }
}

// ------------------------------------------------------------------------------------------------
// pb_fuse_step_beam: one workgroup per utterance.  Every thread keeps the KC best candidates it
// has seen (sorted, registers); K rounds of workgroup arg-max over the list heads then emit the
// utterance's K best in order.
template <int KC>
struct TopList {
  float val[KC];
  int idx[KC];
  int nxt[KC];
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int i = 0; i < KC; ++i) {
      val[i] = -INFINITY;
      idx[i] = INT_MAX;
      nxt[i] = -1;
    }
  }
  __device__ __forceinline__ void push(float v, int id, int nx) {
    if (!better(v, id, val[KC - 1], idx[KC - 1])) return;
    val[KC - 1] = v;
    idx[KC - 1] = id;
    nxt[KC - 1] = nx;
#pragma unroll
    for (int i = KC - 1; i >= 1; --i) {
      if (better(val[i], idx[i], val[i - 1], idx[i - 1])) {
        const float tv = val[i]; val[i] = val[i - 1]; val[i - 1] = tv;
        const int ti = idx[i]; idx[i] = idx[i - 1]; idx[i - 1] = ti;
        const int tn = nxt[i]; nxt[i] = nxt[i - 1]; nxt[i - 1] = tn;
      }
    }
  }
  __device__ __forceinline__ void pop() {
#pragma unroll
    for (int i = 0; i + 1 < KC; ++i) {
      val[i] = val[i + 1];
      idx[i] = idx[i + 1];
      nxt[i] = nxt[i + 1];
    }
    val[KC - 1] = -INFINITY;
    idx[KC - 1] = INT_MAX;
    nxt[KC - 1] = -1;
  }
};

template <int KC, int VEC>
__global__ void __launch_bounds__(1024) beam_kernel(DeviceTree t0, TreePick pick, const float* __restrict__ logp,
                                                    int64_t row_stride, const float* __restrict__ hyp,
                                                    const int32_t* __restrict__ states_in,
                                                    float alpha, int K, int32_t* __restrict__ tokens,
                                                    int32_t* __restrict__ parents, int32_t* __restrict__ states_out,
                                                    float* __restrict__ scores_out, int chunk) {
  extern __shared__ u64 row[];
  __shared__ float sv[16];
  __shared__ int si[16];
  const int u = blockIdx.x;
  DeviceTree t = t0;
  bool valid = pick_tree(pick, u, t);  // one tree per utterance
  const int V = t.vocab_size;
  for (int k = 0; k < K; ++k)
    valid = valid && static_cast<unsigned>(states_in[u * K + k]) < static_cast<unsigned>(t.num_states);
  if (!valid) {
    for (int j = threadIdx.x; j < K; j += blockDim.x) {
      tokens[u * K + j] = -1;
      parents[u * K + j] = -1;
      states_out[u * K + j] = -1;
      scores_out[u * K + j] = NAN;
    }
    return;
  }
  TopList<KC> top;
  top.init();
  for (int k = 0; k < K; ++k) {
    const int h = u * K + k;
    const int s = states_in[h];
    const float hs = hyp[h];
    const float* lrow = logp + static_cast<size_t>(h) * row_stride;
    for (int v0 = 0; v0 < V; v0 += chunk) {
      const int n = min(chunk, V - v0);
      __syncthreads();  // everyone has read the previous row
      for (int i = threadIdx.x; i < n; i += blockDim.x) row[i] = 0ull;
      __syncthreads();
      const float p_root = scatter_chain(t, s, v0, n, row);
      __syncthreads();
      for (int i0 = threadIdx.x * VEC; i0 < n; i0 += blockDim.x * VEC) {
        float lpa[VEC];
        if constexpr (VEC == 4) {
          const float4 lp = *reinterpret_cast<const float4*>(lrow + v0 + i0);
          lpa[0] = lp.x; lpa[1] = lp.y; lpa[2] = lp.z; lpa[3] = lp.w;
        } else {
          lpa[0] = lrow[v0 + i0];
        }
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
          const int v = v0 + i0 + q;
          float sc;
          int nx;
          resolve(t, s, p_root, row[i0 + q], v, t.root_score[v], t.root_next[v], sc, nx);
          const float expansion = __fadd_rn(lpa[q], __fmul_rn(alpha, sc));
          const float total = __fadd_rn(hs, expansion);
          top.push(total, k * V + v, nx);
        }
      }
    }
  }
  for (int j = 0; j < K; ++j) {
    float win = top.val[0];
    int win_i = top.idx[0] == INT_MAX ? -1 : top.idx[0];
    block_best(win, win_i, sv, si);
    if (top.idx[0] == win_i) {
      tokens[u * K + j] = win_i % V;
      parents[u * K + j] = win_i / V;
      states_out[u * K + j] = top.nxt[0];
      scores_out[u * K + j] = win;
      top.pop();
    }
  }
}

inline int pick_chunk(int V) { return V < kMaxChunk ? ((V + 3) & ~3) : kMaxChunk; }

inline int pick_threads(int V) {
  int nt = ((V + 3) / 4 + 63) & ~63;
  return nt < 64 ? 64 : (nt > 1024 ? 1024 : nt);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int check_launch() { return hipGetLastError() == hipSuccess ? PB_OK : PB_EHIP; }

}  // namespace

int launch_score(const DeviceTree& t, const TreePick& pick, const int32_t* d_states, int32_t B, float* d_scores,
                 int32_t* d_next, hipStream_t stream) {
  const int V = t.vocab_size;
  const int tile = V < kScoreTile ? ((V + 3) & ~3) : kScoreTile;
  const int tiles = (V + tile - 1) / tile;
  // Hypotheses per workgroup: one up to 16384 workgroups, then as many as keep the launch near that size, at most
  // eight (V = 8192: one hypothesis measured fastest at B = 4096 -- 49 against 55 us with four -- and slowest at
  // B = 16384 -- 253 us against 222 with four and 215 with eight).
  const int64_t wgs = static_cast<int64_t>(B) * tiles;
  const int per = pick.table ? 1 : static_cast<int>(std::min<int64_t>(8, std::max<int64_t>(1, wgs / 16384)));
  const int64_t groups = (static_cast<int64_t>(B) + per - 1) / per;
  if (groups * tiles > INT32_MAX) return PB_EUNSUPPORTED;
  const dim3 grid(static_cast<unsigned>(groups * tiles));
  const size_t lds = static_cast<size_t>(tile) * sizeof(u64);
  const bool vec = (V % 4 == 0) && aligned16(d_scores) && (d_next == nullptr || aligned16(d_next));
  if (vec)
    hipLaunchKernelGGL(score_kernel<4>, grid, dim3(256), lds, stream, t, pick, d_states, B, d_scores, d_next, tile,
                       tiles, per);
  else
    hipLaunchKernelGGL(score_kernel<1>, grid, dim3(256), lds, stream, t, pick, d_states, B, d_scores, d_next, tile,
                       tiles, per);
  return check_launch();
}

int launch_fuse(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B, int sel,
                int32_t* d_tokens, int32_t* d_states, float* d_scores, hipStream_t stream) {
  const int V = t.vocab_size;
  const int chunk = pick_chunk(V);
  const size_t lds = static_cast<size_t>(chunk) * sizeof(u64);
  const bool vec = (V % 4 == 0) && (row_stride % 4 == 0) && (frame_stride % 4 == 0) && aligned16(d_logp);
  const dim3 grid(static_cast<unsigned>(B)), block(static_cast<unsigned>(pick_threads(V)));
  if (vec)
    hipLaunchKernelGGL(fuse_kernel<4>, grid, block, lds, stream, t, pick, d_logp, frame_stride, row_stride, d_states0, d_last0,
                       alpha, T, B, sel, d_tokens, d_states, d_scores, chunk);
  else
    hipLaunchKernelGGL(fuse_kernel<1>, grid, block, lds, stream, t, pick, d_logp, frame_stride, row_stride, d_states0, d_last0,
                       alpha, T, B, sel, d_tokens, d_states, d_scores, chunk);
  return check_launch();
}

template <int KC>
static int launch_beam_kc(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t row_stride, const float* d_hyp,
                          const int32_t* d_states_in, float alpha, int32_t U, int32_t K, int32_t* d_tokens,
                          int32_t* d_parents, int32_t* d_states_out, float* d_scores_out, hipStream_t stream) {
  const int V = t.vocab_size;
  const int chunk = pick_chunk(V);
  const size_t lds = static_cast<size_t>(chunk) * sizeof(u64);
  const bool vec = (V % 4 == 0) && (row_stride % 4 == 0) && aligned16(d_logp);
  const dim3 grid(static_cast<unsigned>(U)), block(static_cast<unsigned>(pick_threads(V)));
  if (vec)
    hipLaunchKernelGGL((beam_kernel<KC, 4>), grid, block, lds, stream, t, pick, d_logp, row_stride, d_hyp, d_states_in, alpha,
                       K, d_tokens, d_parents, d_states_out, d_scores_out, chunk);
  else
    hipLaunchKernelGGL((beam_kernel<KC, 1>), grid, block, lds, stream, t, pick, d_logp, row_stride, d_hyp, d_states_in, alpha,
                       K, d_tokens, d_parents, d_states_out, d_scores_out, chunk);
  return check_launch();
}

int launch_beam(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t row_stride, const float* d_hyp,
                const int32_t* d_states_in, float alpha, int32_t U, int32_t K, int32_t* d_tokens, int32_t* d_parents,
                int32_t* d_states_out, float* d_scores_out, hipStream_t stream) {
#define PB_BEAM(KC)                                                                                            \
  return launch_beam_kc<KC>(t, pick, d_logp, row_stride, d_hyp, d_states_in, alpha, U, K, d_tokens, d_parents, \
                            d_states_out, d_scores_out, stream)
  if (K <= 1) PB_BEAM(1);
  if (K <= 2) PB_BEAM(2);
  if (K <= 4) PB_BEAM(4);
  if (K <= 8) PB_BEAM(8);
  if (K <= 16) PB_BEAM(16);
  PB_BEAM(32);
#undef PB_BEAM
}

}  // namespace pb
