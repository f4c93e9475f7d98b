// C ABI of the phrase-boosting tree library (declared in include/pb.h): argument checks, upload of
// the compiled tree, and dispatch to the kernel launchers.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "pb.h"
#include "pb_kernels.hpp"
#include "pb_tree.hpp"

namespace {

constexpr size_t kAlign = 256;

// Scratch of pb_fuse_frames_static: the patch workspace of the multi-frame decoder as a fixed device array, for
// callers that cannot allocate.  Every GPU the library runs on holds its own copy until the process ends.  In
// host code the array's name is only a stand-in for the symbol: its device address is looked up once per device
// (with that device current) and that address is what the launches get.
constexpr int64_t kStaticScratchBytes = 2ll << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// With `device` current: the address of this device's copy of `scratch`.
int lookup_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return PB_OK;  // (such a device simply has no static scratch)
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device] != nullptr) return PB_OK;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
    (void)hipGetLastError();
    return PB_EHIP;
  }
  g_scratch_ptr[device] = ptr;
  return PB_OK;
}

size_t padded(size_t bytes) { return (bytes + kAlign - 1) / kAlign * kAlign; }

// Uploads the flat arrays as one device allocation.  The device stays current only inside the call.
int upload(pb_tree* tr, int device) {
  const pb::HostTree& h = tr->host;
  const size_t n_state = h.state.size() * sizeof(pb::StateRec);
  const size_t n_arc = h.arc.size() * sizeof(pb::ArcRec);
  const size_t n_rs = h.root_score.size() * sizeof(float);
  const size_t n_rn = h.root_next.size() * sizeof(int32_t);
  const size_t n_pr = h.p_root.size() * sizeof(float);
  const size_t n_rr = h.root_rec.size() * sizeof(pb::RootRec);
  const size_t n_es = h.eos_score.size() * sizeof(float);
  const size_t total =
      padded(n_state) + padded(n_arc) + padded(n_rs) + padded(n_rn) + padded(n_pr) + padded(n_rr) + padded(n_es);
  // The wave kernels request the first arcs of a state without a condition, with the index clamped into the
  // state's arc range; for a state without arcs (the last state of the table included) that reads the entry
  // at arc_begin, i.e. up to one ArcRec past the arc table.  The sub-arrays that follow the arc table in the
  // allocation make that read harmless; refuse a layout that would not.
  if (total - (padded(n_state) + n_arc) < sizeof(pb::ArcRec)) return PB_EUNSUPPORTED;
  int prev = 0;
  if (hipGetDevice(&prev) != hipSuccess) { (void)hipGetLastError(); return PB_EHIP; }
  if (hipSetDevice(device) != hipSuccess) { (void)hipGetLastError(); return PB_EHIP; }
  int rc = PB_OK;
  char* slab = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&slab), total) != hipSuccess) {
    (void)hipGetLastError();
    rc = PB_ENOMEM;
  } else {
    char* p = slab;
    auto put = [&](const void* src, size_t bytes) -> const void* {
      char* dst = p;
      if (bytes && rc == PB_OK && hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice) != hipSuccess) rc = PB_EHIP;
      p += padded(bytes);
      return dst;
    };
    tr->dev.state = static_cast<const pb::StateRec*>(put(h.state.data(), n_state));
    tr->dev.arc = static_cast<const pb::ArcRec*>(put(h.arc.data(), n_arc));
    tr->dev.root_score = static_cast<const float*>(put(h.root_score.data(), n_rs));
    tr->dev.root_next = static_cast<const int32_t*>(put(h.root_next.data(), n_rn));
    tr->dev.p_root = static_cast<const float*>(put(h.p_root.data(), n_pr));
    tr->dev.root_rec = static_cast<const pb::RootRec*>(put(h.root_rec.data(), n_rr));
    tr->dev.eos_score = n_es ? static_cast<const float*>(put(h.eos_score.data(), n_es)) : nullptr;
    tr->dev.eos_id = h.eos_id;
    if (rc == PB_OK) rc = pb::prepare_wave_kernels();
    if (rc == PB_OK) rc = lookup_scratch(device);
    tr->dev.num_states = static_cast<int32_t>(h.state.size());
    tr->dev.vocab_size = h.vocab_size;
    tr->dev.blank_id = h.blank_id;
    if (rc != PB_OK) {
      (void)hipGetLastError();
      (void)hipFree(slab);
      slab = nullptr;
    }
  }
  (void)hipSetDevice(prev);
  if (rc == PB_OK) {
    tr->slab = slab;
    tr->device_bytes = static_cast<int64_t>(total);
    tr->device = device;
  }
  return rc;
}

bool on_device(const pb_tree* t) { return t && t->slab != nullptr; }

}  // namespace

extern "C" {

int pb_build(const int32_t* tokens, const int64_t* offsets, int64_t n_phrases, const float* weights,
             const pb_build_opts* opts, pb_tree** out) {
  if (!opts || !out) return PB_EINVAL;
  if (opts->device < -1) return PB_EINVAL;
  pb_tree* tr = new (std::nothrow) pb_tree();
  if (!tr) return PB_ENOMEM;
  int rc = pb::compile_tree(tokens, offsets, n_phrases, weights, *opts, tr->host);
  if (rc == PB_OK) {  // debug mode: bounds-check every index of the compiled arrays before anything uses them
    const char* dbg = std::getenv("PB_DEBUG");
    if (dbg && dbg[0] != '\0' && !(dbg[0] == '0' && dbg[1] == '\0')) rc = pb_validate(tr);
  }
  if (rc == PB_OK && opts->device >= 0) rc = upload(tr, opts->device);
  if (rc != PB_OK) {
    delete tr;
    return rc;
  }
  *out = tr;
  return PB_OK;
}

int pb_free(pb_tree* tree) {
  if (!tree) return PB_OK;
  int rc = PB_OK;
  if (tree->slab) {
    int prev = 0;
    (void)hipGetDevice(&prev);
    (void)hipSetDevice(tree->device);
    if (hipFree(tree->slab) != hipSuccess) { (void)hipGetLastError(); rc = PB_EHIP; }
    (void)hipSetDevice(prev);
  }
  delete tree;
  return rc;
}

int pb_info(const pb_tree* tree, pb_tree_info* out) {
  if (!tree || !out) return PB_EINVAL;
  const pb::HostTree& h = tree->host;
  out->num_states = static_cast<int32_t>(h.state.size());
  out->num_arcs = static_cast<int32_t>(h.arc.size());
  out->max_depth = h.max_depth;
  out->max_fail_chain = h.max_fail_chain;
  out->root_degree = h.root_degree;
  out->vocab_size = h.vocab_size;
  out->blank_id = h.blank_id;
  out->eos_id = h.eos_id;
  out->device_bytes = tree->device_bytes;
  return PB_OK;
}

int pb_host_arrays(const pb_tree* tree, pb_host_view* out) {
  if (!tree || !out) return PB_EINVAL;
  const pb::HostTree& h = tree->host;
  out->arc_begin = h.arc_begin.data();
  out->arc_count = h.arc_count.data();
  out->fail = h.fail.data();
  out->backoff = h.backoff.data();
  out->is_final = h.is_final.data();
  out->depth = h.depth.data();
  out->parent = h.parent.data();
  out->arc_token = h.arc_token.data();
  out->arc_score = h.arc_score.data();
  out->acc = h.acc.data();
  out->root_score = h.root_score.data();
  out->root_next = h.root_next.data();
  out->p_root = h.p_root.data();
  out->eos_score = h.eos_score.empty() ? nullptr : h.eos_score.data();
  return PB_OK;
}

int pb_state_prefix(const pb_tree* tree, int32_t state, int32_t* out_tokens, int32_t cap, int32_t* out_len) {
  if (!tree || !out_len || cap < 0 || (cap > 0 && !out_tokens)) return PB_EINVAL;
  const pb::HostTree& h = tree->host;
  if (state < 0 || state >= static_cast<int32_t>(h.state.size())) return PB_ERANGE;
  const int32_t len = h.depth[state];
  *out_len = len;
  int32_t s = state;
  for (int32_t d = len - 1; d >= 0; --d) {  // the arc into state s has index s - 1
    if (d < cap) out_tokens[d] = h.arc_token[s - 1];
    s = h.parent[s];
  }
  return PB_OK;
}

int pb_score(const pb_tree* tree, const int32_t* d_states, int32_t B, float* d_scores, int32_t* d_next,
             void* hip_stream) {
  if (!on_device(tree) || B < 0) return PB_EINVAL;
  if (B == 0) return PB_OK;
  if (!d_states || !d_scores) return PB_EINVAL;
  return pb::launch_score(tree->dev, pb::TreePick{}, d_states, B, d_scores, d_next,
                          static_cast<hipStream_t>(hip_stream));
}

int pb_fuse_step_select(const pb_tree* tree, const float* d_logp, int64_t row_stride, const int32_t* d_states_in,
                        const int32_t* d_last_tokens, float alpha, int32_t B, int32_t mode, int32_t* d_tokens,
                        int32_t* d_states_out, float* d_scores, void* hip_stream) {
  if (!on_device(tree) || B < 0) return PB_EINVAL;
  if (mode != PB_SELECT_FUSED && mode != PB_SELECT_TWO_STAGE && mode != PB_SELECT_TWO_STAGE_CTC) return PB_EINVAL;
  if (B == 0) return PB_OK;
  if (!d_logp || !d_states_in || !d_tokens || !d_states_out || !d_scores) return PB_EINVAL;
  if (row_stride < tree->dev.vocab_size) return PB_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (pb::wave_path_ok(tree->dev, d_logp, 0, row_stride))
    return pb::launch_step_wave(tree->dev, pb::TreePick{}, d_logp, row_stride, d_states_in, d_last_tokens, alpha, B, mode, d_tokens,
                                d_states_out, d_scores, stream);
  return pb::launch_fuse(tree->dev, pb::TreePick{}, d_logp, 0, row_stride, d_states_in, d_last_tokens, alpha, 1, B, mode, d_tokens,
                         d_states_out, d_scores, stream);
}

int pb_fuse_step(const pb_tree* tree, const float* d_logp, int64_t row_stride, const int32_t* d_states_in,
                 float alpha, int32_t B, int32_t* d_tokens, int32_t* d_states_out, float* d_scores,
                 void* hip_stream) {
  return pb_fuse_step_select(tree, d_logp, row_stride, d_states_in, nullptr, alpha, B, PB_SELECT_FUSED, d_tokens,
                             d_states_out, d_scores, hip_stream);
}

}  // extern "C"

namespace {

// pb_fuse_frames_select and pb_fuse_frames_ws: d_patches is the optional workspace (null: none).
int fuse_frames_any(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                    const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B, int32_t mode,
                    int32_t* d_tokens, int32_t* d_states, float* d_scores, int32_t* d_patches, void* hip_stream) {
  if (!on_device(tree) || B < 0 || T < 0) return PB_EINVAL;
  if (mode != PB_SELECT_FUSED && mode != PB_SELECT_TWO_STAGE && mode != PB_SELECT_TWO_STAGE_CTC) return PB_EINVAL;
  if (B == 0 || T == 0) return PB_OK;
  if (!d_logp || !d_states0 || !d_tokens || !d_states || !d_scores) return PB_EINVAL;
  if (row_stride < tree->dev.vocab_size || frame_stride < 0) return PB_EINVAL;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // (the segment decoder keeps a flag in bit 30 of the state words it stores: larger trees take the plain kernel)
  if (pb::wave_path_ok(tree->dev, d_logp, frame_stride, row_stride) && tree->dev.num_states < (1 << 30))
    return pb::launch_frames_wave(tree->dev, pb::TreePick{}, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B, mode,
                                  d_tokens, d_states, d_scores, d_patches, stream);
  return pb::launch_fuse(tree->dev, pb::TreePick{}, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B, mode, d_tokens,
                         d_states, d_scores, stream);
}

}  // namespace

extern "C" {

int pb_fuse_frames_select(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                          const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B,
                          int32_t mode, int32_t* d_tokens, int32_t* d_states, float* d_scores, void* hip_stream) {
  return fuse_frames_any(tree, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B, mode, d_tokens, d_states,
                         d_scores, nullptr, hip_stream);
}

int64_t pb_fuse_frames_workspace_bytes(const pb_tree* tree, int32_t T, int32_t B) {
  if (!tree || T < 0 || B < 0) return PB_EINVAL;
  if (T == 0 || B == 0) return 0;
  pb::DeviceTree shape;  // (a host-only tree has no device record: the size depends on the vocabulary alone)
  shape.vocab_size = tree->host.vocab_size;
  return pb::frames_workspace_bytes(shape, T, B);
}

int pb_fuse_frames_plan(const pb_tree* tree, int32_t T, int32_t B, int32_t* n_segments, int32_t* bounds) {
  if (!tree || !n_segments || T < 0 || B < 0) return PB_EINVAL;
  if (T == 0 || B == 0) {
    *n_segments = 0;
    if (bounds) bounds[0] = 0;
    return PB_OK;
  }
  const bool wide = tree->host.vocab_size > 1024;  // (rows wider than a chunk aim for fewer, longer chains)
  const pb::SegPlan plan = pb::plan_segments(T, B, wide ? pb::kWideTargetChains : pb::kTargetChains);
  *n_segments = plan.nseg;
  if (bounds)
    for (int j = 0; j <= plan.nseg; ++j) bounds[j] = pb::seg_begin(j, T, plan.nseg);
  return PB_OK;
}

int pb_fuse_frames_ws(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                      const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B, int32_t mode,
                      int32_t* d_tokens, int32_t* d_states, float* d_scores, void* d_workspace, int64_t workspace_bytes,
                      void* hip_stream) {
  if (!on_device(tree) || B < 0 || T < 0 || workspace_bytes < 0) return PB_EINVAL;
  const int64_t need = (T == 0 || B == 0) ? 0 : pb::frames_workspace_bytes(tree->dev, T, B);
  if (need > 0 && (!d_workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(d_workspace) & 7u) != 0))
    return PB_EINVAL;
  return fuse_frames_any(tree, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B, mode, d_tokens, d_states,
                         d_scores, need > 0 ? static_cast<int32_t*>(d_workspace) : nullptr, hip_stream);
}

int pb_fuse_frames_static(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                          const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B,
                          int32_t mode, int32_t* d_tokens, int32_t* d_states, float* d_scores, void* hip_stream) {
  if (!on_device(tree) || B < 0 || T < 0) return PB_EINVAL;
  const int64_t need = (T == 0 || B == 0) ? 0 : pb::frames_workspace_bytes(tree->dev, T, B);
  if (need > kStaticScratchBytes) return PB_EUNSUPPORTED;  // more segment boundaries than the fixed array holds
  void* ptr = (tree->device >= 0 && tree->device < kMaxDevices) ? g_scratch_ptr[tree->device] : nullptr;
  if (need > 0 && ptr == nullptr) return PB_EHIP;
  return fuse_frames_any(tree, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B, mode, d_tokens, d_states,
                         d_scores, need > 0 ? static_cast<int32_t*>(ptr) : nullptr, hip_stream);
}

int pb_fuse_frames(const pb_tree* tree, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                   const int32_t* d_states0, float alpha, int32_t T, int32_t B, int32_t* d_tokens,
                   int32_t* d_states, float* d_scores, void* hip_stream) {
  return pb_fuse_frames_select(tree, d_logp, frame_stride, row_stride, d_states0, nullptr, alpha, T, B,
                               PB_SELECT_FUSED, d_tokens, d_states, d_scores, hip_stream);
}

int pb_fuse_step_beam(const pb_tree* tree, const float* d_logp, int64_t row_stride, const float* d_hyp_scores,
                      const int32_t* d_states_in, float alpha, int32_t U, int32_t K, int32_t* d_tokens,
                      int32_t* d_parents, int32_t* d_states_out, float* d_scores_out, void* hip_stream) {
  if (!on_device(tree) || U < 0) return PB_EINVAL;
  if (K < 1) return PB_EINVAL;
  if (K > 32) return PB_EUNSUPPORTED;
  if (U == 0) return PB_OK;
  if (!d_logp || !d_hyp_scores || !d_states_in || !d_tokens || !d_parents || !d_states_out || !d_scores_out)
    return PB_EINVAL;
  if (row_stride < tree->dev.vocab_size) return PB_EINVAL;
  if (d_states_out == d_states_in) return PB_EINVAL;
  if (static_cast<int64_t>(K) * tree->dev.vocab_size >= INT32_MAX) return PB_EUNSUPPORTED;
  if (static_cast<int64_t>(U) * K > INT32_MAX) return PB_EUNSUPPORTED;
  if (pb::beam_wave_ok(tree->dev, d_logp, row_stride, K))
    return pb::launch_beam_wave(tree->dev, d_logp, row_stride, d_hyp_scores, d_states_in, alpha, U, K, d_tokens,
                                d_parents, d_states_out, d_scores_out, static_cast<hipStream_t>(hip_stream));
  return pb::launch_beam(tree->dev, pb::TreePick{}, d_logp, row_stride, d_hyp_scores, d_states_in, alpha, U, K, d_tokens, d_parents,
                         d_states_out, d_scores_out, static_cast<hipStream_t>(hip_stream));
}

int pb_forest_build(const pb_tree* const* trees, int32_t n_trees, pb_forest** out) {
  if (!trees || !out || n_trees < 1) return PB_EINVAL;
  for (int32_t i = 0; i < n_trees; ++i)
    if (!on_device(trees[i])) return PB_EINVAL;
  const pb_tree* first = trees[0];
  std::vector<pb::DeviceTree> table(static_cast<size_t>(n_trees));
  for (int32_t i = 0; i < n_trees; ++i) {
    const pb_tree* tr = trees[i];
    if (tr->device != first->device || tr->dev.vocab_size != first->dev.vocab_size ||
        tr->dev.blank_id != first->dev.blank_id || tr->dev.eos_id >= 0)
      return PB_EUNSUPPORTED;
    table[static_cast<size_t>(i)] = tr->dev;
  }
  pb_forest* f = new (std::nothrow) pb_forest();
  if (!f) return PB_ENOMEM;
  int prev = 0, rc = PB_OK;
  if (hipGetDevice(&prev) != hipSuccess || hipSetDevice(first->device) != hipSuccess) {
    (void)hipGetLastError();
    delete f;
    return PB_EHIP;
  }
  const size_t bytes = table.size() * sizeof(pb::DeviceTree);
  if (hipMalloc(reinterpret_cast<void**>(&f->d_table), bytes) != hipSuccess) {
    (void)hipGetLastError();
    rc = PB_ENOMEM;
  } else if (hipMemcpy(f->d_table, table.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(f->d_table);
    rc = PB_EHIP;
  }
  (void)hipSetDevice(prev);
  if (rc != PB_OK) {
    delete f;
    return rc;
  }
  f->proto = first->dev;
  for (int32_t i = 0; i < n_trees; ++i)  // the largest member decides what the others may rely on (see pb_fuse_frames_forest)
    if (trees[i]->dev.num_states > f->proto.num_states) f->proto.num_states = trees[i]->dev.num_states;
  f->count = n_trees;
  f->device = first->device;
  *out = f;
  return PB_OK;
}

int pb_forest_free(pb_forest* forest) {
  if (!forest) return PB_OK;
  int rc = PB_OK, prev = 0;
  (void)hipGetDevice(&prev);
  (void)hipSetDevice(forest->device);
  if (hipFree(forest->d_table) != hipSuccess) {
    (void)hipGetLastError();
    rc = PB_EHIP;
  }
  (void)hipSetDevice(prev);
  delete forest;
  return rc;
}

int pb_score_forest(const pb_forest* forest, const int32_t* d_tree_ids, const int32_t* d_states, int32_t B,
                    float* d_scores, int32_t* d_next, void* hip_stream) {
  if (!forest || B < 0) return PB_EINVAL;
  if (B == 0) return PB_OK;
  if (!d_tree_ids || !d_states || !d_scores) return PB_EINVAL;
  const pb::TreePick pick{forest->d_table, d_tree_ids, forest->count};
  return pb::launch_score(forest->proto, pick, d_states, B, d_scores, d_next, static_cast<hipStream_t>(hip_stream));
}

int pb_fuse_step_forest(const pb_forest* forest, const float* d_logp, int64_t row_stride, const int32_t* d_tree_ids,
                        const int32_t* d_states_in, const int32_t* d_last_tokens, float alpha, int32_t B, int32_t mode,
                        int32_t* d_tokens, int32_t* d_states_out, float* d_scores, void* hip_stream) {
  if (!forest || B < 0) return PB_EINVAL;
  if (mode != PB_SELECT_FUSED && mode != PB_SELECT_TWO_STAGE && mode != PB_SELECT_TWO_STAGE_CTC) return PB_EINVAL;
  if (B == 0) return PB_OK;
  if (!d_logp || !d_tree_ids || !d_states_in || !d_tokens || !d_states_out || !d_scores) return PB_EINVAL;
  if (row_stride < forest->proto.vocab_size) return PB_EINVAL;
  const pb::TreePick pick{forest->d_table, d_tree_ids, forest->count};
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (pb::wave_path_ok(forest->proto, d_logp, 0, row_stride))  // members share the vocabulary, so one answer fits all
    return pb::launch_step_wave(forest->proto, pick, d_logp, row_stride, d_states_in, d_last_tokens, alpha, B, mode,
                                d_tokens, d_states_out, d_scores, stream);
  return pb::launch_fuse(forest->proto, pick, d_logp, 0, row_stride, d_states_in, d_last_tokens, alpha, 1, B, mode,
                         d_tokens, d_states_out, d_scores, stream);
}

int pb_fuse_frames_forest(const pb_forest* forest, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                          const int32_t* d_tree_ids, const int32_t* d_states0, const int32_t* d_last0, float alpha,
                          int32_t T, int32_t B, int32_t mode, int32_t* d_tokens, int32_t* d_states, float* d_scores,
                          void* hip_stream) {
  if (!forest || B < 0 || T < 0) return PB_EINVAL;
  if (mode != PB_SELECT_FUSED && mode != PB_SELECT_TWO_STAGE && mode != PB_SELECT_TWO_STAGE_CTC) return PB_EINVAL;
  if (B == 0 || T == 0) return PB_OK;
  if (!d_logp || !d_tree_ids || !d_states0 || !d_tokens || !d_states || !d_scores) return PB_EINVAL;
  if (row_stride < forest->proto.vocab_size || frame_stride < 0) return PB_EINVAL;
  const pb::TreePick pick{forest->d_table, d_tree_ids, forest->count};
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (pb::wave_path_ok(forest->proto, d_logp, frame_stride, row_stride) && forest->proto.num_states < (1 << 30))
    return pb::launch_frames_wave(forest->proto, pick, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B,
                                  mode, d_tokens, d_states, d_scores, nullptr, stream);
  return pb::launch_fuse(forest->proto, pick, d_logp, frame_stride, row_stride, d_states0, d_last0, alpha, T, B, mode,
                         d_tokens, d_states, d_scores, stream);
}

int pb_fuse_step_beam_forest(const pb_forest* forest, const float* d_logp, int64_t row_stride,
                             const int32_t* d_tree_ids, const float* d_hyp_scores, const int32_t* d_states_in,
                             float alpha, int32_t U, int32_t K, int32_t* d_tokens, int32_t* d_parents,
                             int32_t* d_states_out, float* d_scores_out, void* hip_stream) {
  if (!forest || U < 0 || K < 1) return PB_EINVAL;
  if (K > 32) return PB_EUNSUPPORTED;
  if (U == 0) return PB_OK;
  if (!d_logp || !d_tree_ids || !d_hyp_scores || !d_states_in || !d_tokens || !d_parents || !d_states_out ||
      !d_scores_out)
    return PB_EINVAL;
  if (row_stride < forest->proto.vocab_size || d_states_out == d_states_in) return PB_EINVAL;
  if (static_cast<int64_t>(K) * forest->proto.vocab_size >= INT32_MAX) return PB_EUNSUPPORTED;
  if (static_cast<int64_t>(U) * K > INT32_MAX) return PB_EUNSUPPORTED;
  const pb::TreePick pick{forest->d_table, d_tree_ids, forest->count};
  return pb::launch_beam(forest->proto, pick, d_logp, row_stride, d_hyp_scores, d_states_in, alpha, U, K, d_tokens,
                         d_parents, d_states_out, d_scores_out, static_cast<hipStream_t>(hip_stream));
}

int pb_validate(const pb_tree* tree) {
  if (!tree) return PB_EINVAL;
  const pb::HostTree& h = tree->host;
  const int64_t N = static_cast<int64_t>(h.state.size()), A = static_cast<int64_t>(h.arc.size());
  const int32_t V = h.vocab_size;
  auto in = [](int64_t x, int64_t lo, int64_t hi) { return x >= lo && x < hi; };
  if (N < 1 || A != N - 1 || V <= 0) return PB_ERANGE;
  if (static_cast<int64_t>(h.arc_begin.size()) != N || static_cast<int64_t>(h.arc_count.size()) != N ||
      static_cast<int64_t>(h.fail.size()) != N || static_cast<int64_t>(h.depth.size()) != N ||
      static_cast<int64_t>(h.parent.size()) != N || static_cast<int64_t>(h.backoff.size()) != N ||
      static_cast<int64_t>(h.p_root.size()) != N || static_cast<int64_t>(h.arc_token.size()) != A ||
      static_cast<int64_t>(h.arc_score.size()) != A || static_cast<int64_t>(h.root_score.size()) != V ||
      static_cast<int64_t>(h.root_next.size()) != V || static_cast<int64_t>(h.root_rec.size()) != V)
    return PB_ERANGE;
  if (h.eos_id >= 0 && static_cast<int64_t>(h.eos_score.size()) != N) return PB_ERANGE;
  int64_t next_arc = 0;
  for (int64_t s = 0; s < N; ++s) {
    // arc rows tile the arc table in state order; every arc stays inside it
    if (h.arc_begin[s] != next_arc || h.arc_count[s] < 0 || next_arc + h.arc_count[s] > A) return PB_ERANGE;
    next_arc += h.arc_count[s];
    for (int64_t j = h.arc_begin[s]; j < h.arc_begin[s] + h.arc_count[s]; ++j) {
      const int32_t tok = h.arc_token[j];
      if (!in(tok, 0, V) || tok == h.blank_id || tok == h.eos_id) return PB_ERANGE;
      if (j > h.arc_begin[s] && h.arc_token[j - 1] >= tok) return PB_ERANGE;  // strictly ascending rows
      if (h.parent[j + 1] != s || h.depth[j + 1] != h.depth[s] + 1) return PB_ERANGE;  // arc j leads to state j + 1
      if (h.arc[j].token != tok || h.arc[j].score != h.arc_score[j]) return PB_ERANGE;
    }
    // failure links lead to strictly shallower states, so every chain ends in the root
    if (!in(h.fail[s], 0, N) || (s > 0 && h.depth[h.fail[s]] >= h.depth[s]) || (s == 0 && h.fail[s] != 0)) return PB_ERANGE;
    const pb::StateRec& r = h.state[s];
    const int32_t f = h.fail[s];
    if (r.arc_begin != h.arc_begin[s] || r.arc_count != h.arc_count[s] || r.fail != f || r.backoff != h.backoff[s] ||
        r.f_arc_begin != h.arc_begin[f] || r.f_arc_count != h.arc_count[f] || r.f_fail != h.fail[f] ||
        r.f_backoff != h.backoff[f])
      return PB_ERANGE;
  }
  if (next_arc != A) return PB_ERANGE;
  for (int32_t v = 0; v < V; ++v) {
    const int32_t n = h.root_next[v];
    if (!in(n, 0, N)) return PB_ERANGE;
    if (n != 0 && (h.parent[n] != 0 || h.arc_token[n - 1] != v)) return PB_ERANGE;
    const pb::RootRec& r = h.root_rec[v];
    if (r.next != n || r.arc_begin != h.arc_begin[n] || r.arc_count != h.arc_count[n] || r.fail != h.fail[n] ||
        r.backoff != h.backoff[n] || r.p_root != h.p_root[n])
      return PB_ERANGE;
  }
  return PB_OK;
}

int pb_validate_states(const pb_tree* tree, const int32_t* states, int64_t n, int64_t* first_bad) {
  if (!tree || n < 0 || (n > 0 && !states)) return PB_EINVAL;
  const int64_t N = static_cast<int64_t>(tree->host.state.size());
  for (int64_t i = 0; i < n; ++i) {
    if (states[i] < 0 || states[i] >= N) {
      if (first_bad) *first_bad = i;
      return PB_ERANGE;
    }
  }
  return PB_OK;
}

const char* pb_strerror(int code) {
  switch (code) {
    case PB_OK: return "ok";
    case PB_EINVAL: return "invalid argument";
    case PB_ERANGE: return "value out of range";
    case PB_ENOMEM: return "out of memory";
    case PB_EHIP: return "HIP runtime error";
    case PB_EUNSUPPORTED: return "unsupported size";
    default: return "unknown error";
  }
}

}  // extern "C"
