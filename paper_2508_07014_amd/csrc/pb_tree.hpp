// Internal layout of a compiled boosting tree: host arrays plus their device mirror.
#pragma once
#include <cstdint>
#include <vector>

#include "pb.h"

namespace pb {

// One 32-byte record per state: everything a failure-chain hop needs, for the state and for the state its
// failure link leads to, so that one load serves two levels of the chain (kernels that walk level by level
// read the first half).
struct alignas(32) StateRec {
  int32_t arc_begin;  // first arc of the state in the (from_state, token)-sorted arc table
  int32_t arc_count;  // arcs leaving the state
  int32_t fail;       // failure link
  float backoff;      // backoff score paid when the state is abandoned
  int32_t f_arc_begin;  // the same four fields of state `fail`
  int32_t f_arc_count;
  int32_t f_fail;
  float f_backoff;
};

// One 8-byte record per arc; the arc with index j leads to state j + 1.
struct alignas(8) ArcRec {
  int32_t token;
  float score;
};

// One 32-byte record per token: where the root row sends the token (a depth-1 state, or the root
// itself for the c_unk self-loop) together with that state's record, so that following a root arc
// costs one load.
struct alignas(32) RootRec {
  int32_t next;       // target state
  int32_t arc_begin;  // StateRec of the target ...
  int32_t arc_count;
  int32_t fail;
  float backoff;
  float p_root;       // ... and its total backoff down to the root
  float eos_score;    // ... and its EOS boost (0 without an EOS rule)
  int32_t pad;
};

// Device mirror (one allocation, sub-arrays aligned to 256 bytes).
struct DeviceTree {
  const StateRec* state = nullptr;  // [N]
  const ArcRec* arc = nullptr;      // [N-1]
  const float* root_score = nullptr;  // [V]
  const int32_t* root_next = nullptr;  // [V]
  const float* p_root = nullptr;       // [N] backoff accumulated from the state down to the root (fp32, chain order)
  const RootRec* root_rec = nullptr;   // [V]
  const float* eos_score = nullptr;    // [N] boost of the EOS token in every state (Sec. II-C: largest score of the other
                                       // tokens plus the final weight of an end-of-phrase state); null without an EOS rule
  int32_t num_states = 0;
  int32_t vocab_size = 0;
  int32_t blank_id = -1;
  int32_t eos_id = -1;
};

// Per-row choice among several trees (a different context list per hypothesis or utterance): row i uses
// table[ids[i]].  A null table means "the one tree passed beside it".
struct TreePick {
  const DeviceTree* table = nullptr;  // device array of `count` trees
  const int32_t* ids = nullptr;       // device array, one id per hypothesis (beam step: per utterance)
  int32_t count = 0;
};

struct HostTree {
  int32_t vocab_size = 0, blank_id = -1, eos_id = -1;
  int32_t max_depth = 0, max_fail_chain = 0, root_degree = 0;
  std::vector<StateRec> state;
  std::vector<ArcRec> arc;
  std::vector<RootRec> root_rec;
  std::vector<int32_t> arc_begin, arc_count, fail, depth, parent, arc_token, root_next;
  std::vector<float> backoff, arc_score, root_score, p_root, final_score, eos_score;
  std::vector<uint8_t> is_final;
  std::vector<double> acc;
};

// Alg. 1 Stages 1-2 on the host.  Returns a pb_status.
int compile_tree(const int32_t* tokens, const int64_t* offsets, int64_t n_phrases, const float* weights,
                 const pb_build_opts& opts, HostTree& out);

}  // namespace pb

struct pb_forest {
  pb::DeviceTree* d_table = nullptr;  // device copy of the members' DeviceTree records
  pb::DeviceTree proto;               // vocabulary size and blank id common to all members
  int32_t count = 0;
  int device = -1;
};

struct pb_tree {
  pb::HostTree host;
  pb::DeviceTree dev;
  void* slab = nullptr;  // device allocation backing `dev`
  int64_t device_bytes = 0;
  int device = -1;
};
