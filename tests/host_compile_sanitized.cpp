// Host tree compiler under AddressSanitizer / UndefinedBehaviorSanitizer (no GPU, no HIP runtime):
// random phrase lists of every shape the compiler accepts, every malformed input it must reject, and the
// structural invariants of the flat arrays (Alg. 1, Stages 1 and 2).  Exit code 0 = clean.
#include <cstdint>
#include <cstdio>
#include <random>
#include <vector>

#include "pb_tree.hpp"

static int fails = 0;
#define CHECK(cond)                                                       \
  do {                                                                    \
    if (!(cond)) {                                                        \
      std::printf("check failed at line %d: %s\n", __LINE__, #cond);     \
      ++fails;                                                            \
    }                                                                     \
  } while (0)

static pb_build_opts opts(int V, int blank, int mode, int eos) {
  pb_build_opts o{};
  o.vocab_size = V;
  o.blank_id = blank;
  o.weight_mode = mode;
  o.beta = 2.0f;
  o.unk_score = 0.25f;
  o.final_zero_backoff = 1;
  o.device = -1;
  o.eos_id = eos;
  o.final_eos_score = 1.5f;
  return o;
}

static void invariants(const pb::HostTree& t, int V, int64_t total_tokens) {
  const int N = static_cast<int>(t.state.size());
  CHECK(N >= 1 && N <= total_tokens + 1);
  CHECK(static_cast<int>(t.arc.size()) == N - 1);
  CHECK(static_cast<int>(t.root_score.size()) == V && static_cast<int>(t.root_rec.size()) == V);
  int arcs = 0;
  for (int s = 0; s < N; ++s) {
    CHECK(t.arc_begin[s] == arcs);
    arcs += t.arc_count[s];
    CHECK(t.fail[s] >= 0 && t.fail[s] < N);
    if (s) CHECK(t.depth[t.fail[s]] < t.depth[s]);
    for (int j = 1; j < t.arc_count[s]; ++j) CHECK(t.arc_token[t.arc_begin[s] + j - 1] < t.arc_token[t.arc_begin[s] + j]);
    for (int j = 0; j < t.arc_count[s]; ++j) {
      const int child = t.arc_begin[s] + j + 1;
      CHECK(child < N && t.parent[child] == s && t.depth[child] == t.depth[s] + 1);
    }
  }
  CHECK(arcs == N - 1);
  for (int v = 0; v < V; ++v) CHECK(t.root_next[v] >= 0 && t.root_next[v] < N && t.root_rec[v].next == t.root_next[v]);
}

int main() {
  std::mt19937_64 rng(20250807);
  for (int trial = 0; trial < 400; ++trial) {
    const int V = 2 + static_cast<int>(rng() % 40);
    const int blank = (trial % 3 == 0) ? -1 : 0;
    const int eos = (trial % 4 == 0 && V > 3) ? V - 1 : -1;
    const int mode = trial % 3;
    const int n = static_cast<int>(rng() % 30);
    std::vector<int32_t> toks;
    std::vector<int64_t> offs{0};
    std::vector<float> w;
    for (int i = 0; i < n; ++i) {
      const int len = 1 + static_cast<int>(rng() % 7);
      for (int j = 0; j < len; ++j) {
        int tk;
        do tk = static_cast<int>(rng() % V); while (tk == blank || tk == eos);
        toks.push_back(tk);
      }
      offs.push_back(static_cast<int64_t>(toks.size()));
      w.push_back(0.25f * static_cast<float>(1 + rng() % 8));
    }
    if (V <= 2 && (blank == 0)) continue;  // no usable token besides the blank is possible only for V = 1; keep V >= 2 cases
    pb::HostTree t;
    const pb_build_opts o = opts(V, blank, mode, eos);
    const int rc = pb::compile_tree(toks.data(), offs.data(), n, (trial & 1) ? w.data() : nullptr, o, t);
    CHECK(rc == PB_OK);
    if (rc == PB_OK) invariants(t, V, static_cast<int64_t>(toks.size()));
    if (rc == PB_OK && eos >= 0) CHECK(static_cast<int>(t.final_score.size()) == static_cast<int>(t.state.size()));
  }
  // malformed inputs: an error code, never a crash
  {
    pb::HostTree t;
    const int32_t toks[] = {1, 2, 3, 4};
    const int64_t ok[] = {0, 2, 4}, empty[] = {0, 2, 2}, back[] = {0, 3, 1}, neg[] = {-1, 2, 4};
    CHECK(pb::compile_tree(toks, ok, 2, nullptr, opts(8, 0, 0, -1), t) == PB_OK);
    CHECK(pb::compile_tree(toks, empty, 2, nullptr, opts(8, 0, 0, -1), t) == PB_EINVAL);
    CHECK(pb::compile_tree(toks, back, 2, nullptr, opts(8, 0, 0, -1), t) == PB_EINVAL);
    CHECK(pb::compile_tree(toks, neg, 2, nullptr, opts(8, 0, 0, -1), t) == PB_EINVAL);
    CHECK(pb::compile_tree(toks, ok, 2, nullptr, opts(4, 0, 0, -1), t) == PB_ERANGE);   // token 4 outside V = 4
    CHECK(pb::compile_tree(toks, ok, 2, nullptr, opts(8, 2, 0, -1), t) == PB_EINVAL);   // blank inside a phrase
    CHECK(pb::compile_tree(toks, ok, 2, nullptr, opts(8, 0, 0, 3), t) == PB_EINVAL);    // EOS inside a phrase
    CHECK(pb::compile_tree(toks, ok, 2, nullptr, opts(8, 0, 0, 0), t) == PB_EINVAL);    // EOS == blank
    CHECK(pb::compile_tree(toks, ok, 2, nullptr, opts(8, 0, 7, -1), t) == PB_EINVAL);   // unknown weight mode
    CHECK(pb::compile_tree(toks, ok, 2, nullptr, opts(0, -1, 0, -1), t) == PB_EINVAL);  // empty vocabulary
    CHECK(pb::compile_tree(nullptr, nullptr, 2, nullptr, opts(8, 0, 0, -1), t) == PB_EINVAL);
    CHECK(pb::compile_tree(nullptr, nullptr, 0, nullptr, opts(8, 0, 0, -1), t) == PB_OK);  // root-only tree
    CHECK(t.state.size() == 1);
  }
  std::printf(fails ? "FAILED (%d)\n" : "clean (%d)\n", fails);
  return fails ? 1 : 0;
}
