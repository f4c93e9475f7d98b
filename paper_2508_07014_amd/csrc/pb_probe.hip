// Measurement probes used by bench.py only (libpb_probe.so): no part of the method and not in the product
// library.  Plain C ABI, device pointers, asynchronous on the given stream.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

namespace {

// One lane follows i = table[i] for `hops` dependent loads.  The decode recurrence (state -> record -> arcs
// -> next state) is a chain of such loads, so the time per hop is the floor under every single-step call.
// An index outside [0, n) ends the walk (the result is then -1): a bad table cannot fault.
__global__ void chase_kernel(const int32_t* __restrict__ table, int64_t n, int32_t start, int32_t hops,
                             int32_t* __restrict__ out) {
  int32_t i = start + static_cast<int32_t>(threadIdx.x);  // launched with one thread; keeps the loads on the vector path
  for (int32_t h = 0; h < hops; ++h) {
    if (static_cast<uint64_t>(i) >= static_cast<uint64_t>(n)) {
      i = -1;
      break;
    }
    i = table[i];
  }
  *out = i;
}

// One wavefront per row: reads prev[b] (so that a chain of such launches is dependent like a decoding loop), the
// row of V floats and writes the index of its maximum (lowest index among equal maxima) -- the least a greedy step
// can do.  Its time per launch in a HIP-graph loop is the floor under pb_fuse_step in that regime.
__global__ void __launch_bounds__(64) rowmax_kernel(const float* __restrict__ logp, int64_t row_stride, int32_t V,
                                                    const int32_t* __restrict__ prev, int32_t* __restrict__ out) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int32_t p = prev[b];
  const float* row = logp + static_cast<size_t>(b) * row_stride;
  float best = -INFINITY;
  int32_t bi = INT32_MAX;
  float4 x[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {  // (V <= 1024, V % 4 == 0: checked by the caller)
    const int v = 256 * i + 4 * lane;
    x[i] = v < V ? *reinterpret_cast<const float4*>(row + v) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = 256 * i + 4 * lane;
    const float e[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (v + k < V && (e[k] > best || bi == INT32_MAX)) { best = e[k]; bi = v + k; }
  }
  for (int o = 32; o; o >>= 1) {
    const float ob = __shfl_xor(best, o);
    const int32_t oi = __shfl_xor(bi, o);
    if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
  }
  if (lane == 0) out[b] = bi == INT32_MAX ? -1 : bi + (p == INT32_MIN ? 1 : 0);
}

}  // namespace

extern "C" {

// d_logp fp32 rows of V values (0 < V <= 1024, V % 4 == 0, rows 16-byte aligned), d_prev int32[B] (read, any
// values), d_out int32[B] (may be the d_prev of the next launch).  0 on success, -1 on a bad argument, -4 when the
// launch fails.
int pb_probe_rowmax(const float* d_logp, int64_t row_stride, int32_t V, const int32_t* d_prev, int32_t* d_out, int32_t B,
                    void* hip_stream) {
  if (!d_logp || !d_prev || !d_out || B <= 0 || V <= 0 || V > 1024 || (V & 3) != 0 || row_stride < V ||
      (row_stride & 3) != 0 || (reinterpret_cast<uintptr_t>(d_logp) & 15u) != 0)
    return -1;
  hipLaunchKernelGGL(rowmax_kernel, dim3(static_cast<unsigned>(B)), dim3(64), 0, static_cast<hipStream_t>(hip_stream),
                     d_logp, row_stride, V, d_prev, d_out);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// d_table int32[n], start in [0, n), hops >= 0; *d_out receives the last index.  0 on success, -1 on a bad
// argument, -4 when the launch fails.
int pb_probe_chase(const int32_t* d_table, int64_t n, int32_t start, int32_t hops, int32_t* d_out, void* hip_stream) {
  if (!d_table || !d_out || n <= 0 || n > INT32_MAX || start < 0 || start >= n || hops < 0) return -1;
  hipLaunchKernelGGL(chase_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(hip_stream), d_table, n, start, hops,
                     d_out);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
