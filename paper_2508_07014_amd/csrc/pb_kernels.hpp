// Launch wrappers of the HIP kernels (defined in pb_kernels.hip).  Each returns a pb_status.
#pragma once
#include <hip/hip_runtime.h>

#include "pb_tree.hpp"

namespace pb {

// The tree of row i: `t` as passed, or table[ids[i]] when a table is given.  False for an id outside the table.
__device__ __forceinline__ bool pick_tree(const TreePick& p, int i, DeviceTree& t) {
  if (p.table == nullptr) return true;
  const int32_t id = p.ids[i];
  if (static_cast<uint32_t>(id) >= static_cast<uint32_t>(p.count)) return false;
  t = p.table[id];
  return true;
}

constexpr int kMaxChunk = 8192;   // tokens per LDS pass of the fused kernels (64 KiB of 8-byte entries)
#ifndef PB_SCORE_TILE
#define PB_SCORE_TILE 2048
#endif
constexpr int kScoreTile = PB_SCORE_TILE;  // tokens per workgroup of the score kernel (16 KiB of LDS)

int launch_score(const DeviceTree& t, const TreePick& pick, const int32_t* d_states, int32_t B, float* d_scores,
                 int32_t* d_next, hipStream_t stream);

// T == 1 with frame_stride == 0 is the single step.  sel is an enum pb_select_mode value; d_last0 (previous
// labels, CTC rule only) may be null.
int launch_fuse(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t frame_stride, int64_t row_stride,
                const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B, int sel,
                int32_t* d_tokens, int32_t* d_states, float* d_scores, hipStream_t stream);

// Wave-per-hypothesis greedy kernels (pb_frames.hip); usable when rows are 16-byte aligned and V % 4 == 0.
#ifndef PB_TARGET_CHAINS
#define PB_TARGET_CHAINS 4096
#endif
constexpr int kTargetChains = PB_TARGET_CHAINS;  // concurrent decode chains aimed for by the multi-frame decoder
constexpr int kMinSegLen = 8;        // shortest speculative segment, in frames
constexpr int kMaxSegments = 64;     // segments per hypothesis (one lane each in the validation pass)

constexpr int kWideMaxV = 16384;     // widest row of the wave kernels (the root scores of a row live in LDS)
#ifndef PB_WIDE_TARGET_CHAINS
#define PB_WIDE_TARGET_CHAINS 1024
#endif
constexpr int kWideTargetChains = PB_WIDE_TARGET_CHAINS;  // the same for rows wider than 1024 tokens (one wave per SIMD:
                                                          // a wave keeps three 4-KiB chunks of its rows in flight)

struct SegPlan {
  int nseg, seg_len;  // segments per hypothesis and their nominal length
};
// First frame of segment j of nseg (j == nseg: T).  The frames are split evenly, then tapered: the first segment is
// 1/kSegTaper longer than the mean, the last one as much shorter, linearly in between.  The chains of a call are
// launched in segment order and a SIMD serves older waves first -- measured, the waves launched first run about 5 %
// faster than those launched last -- so equal segments would end the kernel with the youngest waves alone on the chip.
#ifndef PB_SEG_TAPER
#define PB_SEG_TAPER 20
#endif
constexpr int kSegTaper = PB_SEG_TAPER;
__host__ __device__ inline int seg_begin(int j, int T, int nseg) {
  const long long even = static_cast<long long>(j) * T / nseg;
  const long long bulge = kSegTaper > 0 ? static_cast<long long>(T) * j * (nseg - j) / (static_cast<long long>(kSegTaper) * nseg * nseg) : 0;
  return static_cast<int>(even + bulge);
}
SegPlan plan_segments(int32_t T, int32_t B, int target_chains);

bool wave_path_ok(const DeviceTree& t, const float* d_logp, int64_t frame_stride, int64_t row_stride);
// Rows wider than 1024 tokens (pb_wide.hip); same arguments as the calls below, which forward to them.
int prepare_wide_kernels(int max_lds_bytes);
int launch_step_wide(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t row_stride,
                     const int32_t* d_states_in, const int32_t* d_last, float alpha, int32_t B, int sel,
                     int32_t* d_tokens, int32_t* d_states_out, float* d_scores, hipStream_t stream);
int launch_frames_wide(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t frame_stride,
                       int64_t row_stride, const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T,
                       int32_t B, int sel, int32_t* d_tokens, int32_t* d_states, float* d_scores, hipStream_t stream);
int prepare_wave_kernels();  // once per device, after the device has been made current
int launch_step_wave(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t row_stride,
                     const int32_t* d_states_in,
                     const int32_t* d_last, float alpha, int32_t B, int sel, int32_t* d_tokens, int32_t* d_states_out,
                     float* d_scores, hipStream_t stream);
// d_patches: optional workspace of frames_workspace_bytes(t, T, B) bytes (null: wrong boundary guesses are
// repaired by re-runs in pass 2 instead of patches from pass 1).
int64_t frames_workspace_bytes(const DeviceTree& t, int32_t T, int32_t B);
int launch_frames_wave(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t frame_stride,
                       int64_t row_stride,
                       const int32_t* d_states0, const int32_t* d_last0, float alpha, int32_t T, int32_t B, int sel,
                       int32_t* d_tokens, int32_t* d_states, float* d_scores, int32_t* d_patches, hipStream_t stream);

// Wave-per-beam kernel (pb_frames.hip): rows as for the wave path, V <= 1024 and a beam the LDS can hold.
bool beam_wave_ok(const DeviceTree& t, const float* d_logp, int64_t row_stride, int32_t K);
int launch_beam_wave(const DeviceTree& t, const float* d_logp, int64_t row_stride, const float* d_hyp,
                     const int32_t* d_states_in, float alpha, int32_t U, int32_t K, int32_t* d_tokens,
                     int32_t* d_parents, int32_t* d_states_out, float* d_scores_out, hipStream_t stream);

int launch_beam(const DeviceTree& t, const TreePick& pick, const float* d_logp, int64_t row_stride, const float* d_hyp,
                const int32_t* d_states_in, float alpha, int32_t U, int32_t K, int32_t* d_tokens, int32_t* d_parents,
                int32_t* d_states_out, float* d_scores_out, hipStream_t stream);

}  // namespace pb
