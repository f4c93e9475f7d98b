// Host tree compiler: context list -> flat, GPU-ready boosting tree (Alg. 1, Stages 1 and 2).
//
// Stage 1  prefix tree by insertion; an arc is scored when it is created (uniform: c0; log-depth:
//          c0 at depth 1, c0*beta + ln(depth) below, Sec. II-B); accumulated score per state;
//          end-of-phrase flags; failure link = longest proper suffix that is a tree prefix.
// Stage 2  states renumbered breadth-first with children by ascending token, which makes the
//          (from_state, token)-sorted arc table implicit in the numbering (arc j -> state j+1);
//          backoff score = acc(fail) - acc(state), zero for end-of-phrase states; the root row is
//          made total over the vocabulary with c_unk self-loops.
// Tree scores are accumulated in double and rounded to fp32 once.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <unordered_map>
#include <vector>

#include "pb_tree.hpp"

namespace pb {

namespace {

struct TmpNode {
  int32_t parent, token, depth;
  double arc, acc;
  bool is_final;
};

// child of canonical state s on token v in the canonical CSR, or -1
inline int32_t find_child(const HostTree& t, int32_t s, int32_t v) {
  const int32_t* first = t.arc_token.data() + t.arc_begin[s];
  const int32_t* last = first + t.arc_count[s];
  const int32_t* it = std::lower_bound(first, last, v);
  if (it == last || *it != v) return -1;
  return static_cast<int32_t>(it - t.arc_token.data()) + 1;
}

}  // namespace

int compile_tree(const int32_t* tokens, const int64_t* offsets, int64_t n_phrases, const float* weights,
                 const pb_build_opts& o, HostTree& out) {
  const int32_t V = o.vocab_size;
  if (V <= 0 || o.blank_id < -1 || o.blank_id >= V || n_phrases < 0) return PB_EINVAL;
  if (o.weight_mode != PB_W_UNIFORM && o.weight_mode != PB_W_LOGDEPTH && o.weight_mode != PB_W_UNIFORM_FINAL)
    return PB_EINVAL;
  if (o.eos_id < -1 || o.eos_id >= V || (o.eos_id >= 0 && o.eos_id == o.blank_id)) return PB_EINVAL;
  if (n_phrases > 0 && (!tokens || !offsets)) return PB_EINVAL;
  // Scores are sums of the weights: the kernels' arithmetic (a boost times 0 for the blank column, comparisons
  // of fused values) assumes they are finite.
  if (!std::isfinite(o.beta) || !std::isfinite(o.unk_score) || !std::isfinite(o.final_eos_score)) return PB_EINVAL;
  for (int64_t i = 0; weights && i < n_phrases; ++i)
    if (!std::isfinite(weights[i])) return PB_EINVAL;
  for (int64_t i = 0; i < n_phrases; ++i) {
    if (offsets[i] < 0 || offsets[i + 1] <= offsets[i]) return PB_EINVAL;
    for (int64_t j = offsets[i]; j < offsets[i + 1]; ++j) {
      if (tokens[j] < 0 || tokens[j] >= V) return PB_ERANGE;
      if (tokens[j] == o.blank_id || tokens[j] == o.eos_id) return PB_EINVAL;
    }
  }
  const int64_t total = n_phrases ? offsets[n_phrases] - offsets[0] : 0;
  if (total + 1 > INT32_MAX) return PB_ERANGE;

  try {
    // ---- Stage 1: insertion ---------------------------------------------------------
    std::vector<TmpNode> nodes;
    nodes.reserve(static_cast<size_t>(total) + 1);
    nodes.push_back({-1, -1, 0, 0.0, 0.0, false});
    std::unordered_map<uint64_t, int32_t> arcs;
    arcs.reserve(static_cast<size_t>(total) * 2 + 16);
    for (int64_t i = 0; i < n_phrases; ++i) {
      const double c0 = weights ? static_cast<double>(weights[i]) : 1.0;
      int32_t cur = 0;
      for (int64_t j = offsets[i]; j < offsets[i + 1]; ++j) {
        const int32_t depth = static_cast<int32_t>(j - offsets[i]) + 1;
        const uint64_t key = (static_cast<uint64_t>(static_cast<uint32_t>(cur)) << 32) |
                             static_cast<uint32_t>(tokens[j]);
        auto it = arcs.find(key);
        if (it == arcs.end()) {
          double a = c0;
          if (o.weight_mode == PB_W_LOGDEPTH && depth > 1)
            a = c0 * static_cast<double>(o.beta) + std::log(static_cast<double>(depth));
          const int32_t id = static_cast<int32_t>(nodes.size());
          nodes.push_back({cur, tokens[j], depth, a, nodes[cur].acc + a, false});
          arcs.emplace(key, id);
          cur = id;
        } else {
          cur = it->second;
        }
      }
      nodes[cur].is_final = true;
    }
    arcs.clear();
    const int32_t N = static_cast<int32_t>(nodes.size());
    if (o.weight_mode == PB_W_UNIFORM_FINAL) {
      // end-of-phrase reward: the arc into a node where a phrase ends also carries the uniform scores of
      // the whole path (node ids grow from parent to child, so one forward sweep rebuilds acc)
      std::vector<double> path(N, 0.0);
      for (int32_t id = 1; id < N; ++id) {
        TmpNode& nd = nodes[id];
        path[id] = path[nd.parent] + nd.arc;
        if (nd.is_final) nd.arc += path[id];
        nd.acc = nodes[nd.parent].acc + nd.arc;
      }
    }

    // ---- canonical numbering: breadth-first, children by ascending token -------------
    std::vector<int32_t> by_parent(N > 1 ? N - 1 : 0);
    std::iota(by_parent.begin(), by_parent.end(), 1);
    std::sort(by_parent.begin(), by_parent.end(), [&](int32_t a, int32_t b) {
      if (nodes[a].parent != nodes[b].parent) return nodes[a].parent < nodes[b].parent;
      return nodes[a].token < nodes[b].token;
    });
    std::vector<int32_t> kid_begin(N + 1, 0);
    for (int32_t id = 1; id < N; ++id) kid_begin[nodes[id].parent + 1]++;
    for (int32_t i = 0; i < N; ++i) kid_begin[i + 1] += kid_begin[i];
    std::vector<int32_t> order(N), canon(N);
    order[0] = 0;
    int32_t tail = 1;
    for (int32_t head = 0; head < tail; ++head) {
      const int32_t s = order[head];
      for (int32_t k = kid_begin[s]; k < kid_begin[s + 1]; ++k) order[tail++] = by_parent[k];
    }
    for (int32_t i = 0; i < N; ++i) canon[order[i]] = i;

    HostTree t;
    t.vocab_size = V;
    t.blank_id = o.blank_id;
    t.eos_id = o.eos_id;
    t.arc_begin.assign(N, 0);
    t.arc_count.assign(N, 0);
    t.fail.assign(N, 0);
    t.depth.assign(N, 0);
    t.parent.assign(N, -1);
    t.backoff.assign(N, 0.0f);
    t.is_final.assign(N, 0);
    t.acc.assign(N, 0.0);
    t.arc_token.assign(N > 1 ? N - 1 : 0, 0);
    t.arc_score.assign(N > 1 ? N - 1 : 0, 0.0f);
    int32_t next_arc = 0;
    for (int32_t i = 0; i < N; ++i) {
      const TmpNode& nd = nodes[order[i]];
      t.depth[i] = nd.depth;
      t.parent[i] = nd.parent < 0 ? -1 : canon[nd.parent];
      t.is_final[i] = nd.is_final ? 1 : 0;
      t.acc[i] = nd.acc;
      t.max_depth = std::max(t.max_depth, nd.depth);
      if (i > 0) {  // the arc leading into state i has index i - 1
        t.arc_token[i - 1] = nd.token;
        t.arc_score[i - 1] = static_cast<float>(nd.arc);
      }
      const int32_t s = order[i];
      t.arc_begin[i] = next_arc;
      t.arc_count[i] = kid_begin[s + 1] - kid_begin[s];
      next_arc += t.arc_count[i];
    }

    // ---- failure links, in breadth-first (= id) order ---------------------------------
    for (int32_t s = 1; s < N; ++s) {
      const int32_t p = t.parent[s];
      if (p == 0) continue;  // depth 1 fails to the root
      const int32_t tok = t.arc_token[s - 1];
      int32_t f = t.fail[p];
      for (;;) {
        const int32_t c = find_child(t, f, tok);
        if (c >= 0) { t.fail[s] = c; break; }
        if (f == 0) break;
        f = t.fail[f];
      }
    }

    // ---- Stage 2: backoff scores, dense root row, packed records -----------------------
    std::vector<int32_t> hops(N, 0);
    for (int32_t s = 1; s < N; ++s) {
      const bool zero = t.is_final[s] && o.final_zero_backoff;
      t.backoff[s] = zero ? 0.0f : static_cast<float>(t.acc[t.fail[s]] - t.acc[s]);
      hops[s] = hops[t.fail[s]] + 1;
      t.max_fail_chain = std::max(t.max_fail_chain, hops[s]);
    }
    // total backoff of each state's failure chain, summed in fp32 in the order a query pays it
    t.p_root.assign(N, 0.0f);
    for (int32_t s = 1; s < N; ++s) {
      float p = 0.0f;
      for (int32_t x = s; x != 0; x = t.fail[x]) p = p + t.backoff[x];
      t.p_root[s] = p;
    }
    if (o.eos_id >= 0) {  // EOS rule (Sec. II-C): end-of-phrase states carry the final weight
      t.final_score.assign(N, 0.0f);
      for (int32_t s = 0; s < N; ++s)
        if (t.is_final[s]) t.final_score[s] = o.final_eos_score;
    }
    t.root_score.assign(V, o.unk_score);
    t.root_next.assign(V, 0);
    t.root_degree = t.arc_count[0];
    for (int32_t j = 0; j < t.arc_count[0]; ++j) {
      t.root_score[t.arc_token[j]] = t.arc_score[j];
      t.root_next[t.arc_token[j]] = j + 1;
    }
    if (o.eos_id >= 0) {
      // EOS rule (Sec. II-C): the EOS boost of a state is the largest score any other token (the blank aside)
      // gets in that state, plus the final weight of an end-of-phrase state.  It depends on the state alone,
      // so it is tabulated here.  Per state: the arcs along the failure chain that no deeper chain state
      // shadows, each with the backoffs paid before it (fp32, in the order a query adds them), and for the
      // tokens no chain state overrides the total backoff plus the largest root score among them (fp32
      // addition is monotone, so the maximum may be taken before the sum).
      std::vector<int32_t> by_root_score;
      by_root_score.reserve(V);
      for (int32_t v = 0; v < V; ++v)
        if (v != o.eos_id && v != o.blank_id) by_root_score.push_back(v);
      std::stable_sort(by_root_score.begin(), by_root_score.end(),
                       [&](int32_t a, int32_t b) { return t.root_score[a] > t.root_score[b]; });
      std::vector<int32_t> seen(V, -1);
      t.eos_score.assign(N, 0.0f);
      for (int32_t s = 0; s < N; ++s) {
        bool any = false;
        float best = 0.0f;
        float p = 0.0f;
        for (int32_t x = s; x != 0; x = t.fail[x]) {
          for (int32_t j = t.arc_begin[x]; j < t.arc_begin[x] + t.arc_count[x]; ++j) {
            const int32_t v = t.arc_token[j];
            if (seen[v] == s) continue;  // a deeper chain state has an arc on v
            seen[v] = s;
            const float c = p + t.arc_score[j];  // (phrases hold neither the EOS nor the blank)
            if (!any || c > best) best = c;
            any = true;
          }
          p = p + t.backoff[x];
        }
        for (const int32_t v : by_root_score) {
          if (seen[v] == s) continue;
          const float c = p + t.root_score[v];
          if (!any || c > best) best = c;
          any = true;
          break;
        }
        t.eos_score[s] = (any ? best : 0.0f) + t.final_score[s];
      }
    }
    t.state.resize(N);
    for (int32_t s = 0; s < N; ++s) {
      const int32_t f = t.fail[s];
      t.state[s] = {t.arc_begin[s], t.arc_count[s], f, t.backoff[s], t.arc_begin[f], t.arc_count[f], t.fail[f], t.backoff[f]};
    }
    t.root_rec.resize(V);
    for (int32_t v = 0; v < V; ++v) {
      const int32_t n = t.root_next[v];
      t.root_rec[v] = {n, t.arc_begin[n], t.arc_count[n], t.fail[n], t.backoff[n], t.p_root[n],
                       t.eos_score.empty() ? 0.0f : t.eos_score[n], 0};
    }
    t.arc.resize(t.arc_token.size());
    for (size_t j = 0; j < t.arc.size(); ++j) t.arc[j] = {t.arc_token[j], t.arc_score[j]};
    // (finite weights can still add up to an overflow)
    for (const float v : t.arc_score)
      if (!std::isfinite(v)) return PB_ERANGE;
    for (const float v : t.p_root)
      if (!std::isfinite(v)) return PB_ERANGE;
    for (const float v : t.backoff)
      if (!std::isfinite(v)) return PB_ERANGE;
    out = std::move(t);
  } catch (const std::bad_alloc&) {
    return PB_ENOMEM;
  }
  return PB_OK;
}

}  // namespace pb
