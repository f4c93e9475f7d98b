// Measurement probes used by bench.py only (libpb_probe.so): no part of the method and not in the product
// library.  Plain C ABI, device pointers, asynchronous on the given stream.
#include <hip/hip_runtime.h>

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

}  // namespace

extern "C" {

// d_table int32[n], start in [0, n), hops >= 0; *d_out receives the last index.  0 on success, -1 on a bad
// argument, -4 when the launch fails.
int pb_probe_chase(const int32_t* d_table, int64_t n, int32_t start, int32_t hops, int32_t* d_out, void* hip_stream) {
  if (!d_table || !d_out || n <= 0 || n > INT32_MAX || start < 0 || start >= n || hops < 0) return -1;
  hipLaunchKernelGGL(chase_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(hip_stream), d_table, n, start, hops,
                     d_out);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
