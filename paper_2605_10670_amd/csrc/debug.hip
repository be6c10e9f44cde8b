// Debug helpers that are not part of the step.
#include "eep_internal.hpp"

namespace eep {

// ---------------------------------------------------------------------------
// Debug check of a finished layout, on the device: every routed pair's row lies
// inside its slot's part of the receive buffer and src_of points back at the
// pair; every row below N has a source that points at it.  The pack and combine
// kernels index the caller's buffers with these rows without further checks, so
// this is the bounds assertion of the path, as a call instead of a build flavour.
//   bad[0] pairs whose row is outside [offset[slot], offset[slot+1])
//   bad[1] pairs whose row's src_of is not the pair
//   bad[2] rows < N whose src_of is out of range or whose pair does not hold the row
//   bad[3] routed pairs without a row (legal only after a rank was dropped
//          by failure detection in this step)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_check_layout(
    const int32_t* __restrict__ slot_of, const int32_t* __restrict__ row_of,
    const int32_t* __restrict__ src_of, const int32_t* __restrict__ offset,
    const int32_t* __restrict__ status, int32_t* __restrict__ bad, int total_pairs, int P) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= total_pairs) return;
  const int N = status[0];
  const int p = slot_of[i];
  const int row = row_of[i];
  if (p >= P || p < -1) {
    atomicAdd(&bad[0], 1);
  } else if (p >= 0) {
    if (row == -1) {
      atomicAdd(&bad[3], 1);
    } else if (row < offset[p] || row >= offset[p + 1] || row >= N) {
      atomicAdd(&bad[0], 1);
    } else if (src_of[row] != i) {
      atomicAdd(&bad[1], 1);
    }
  } else if (row != -1) {
    atomicAdd(&bad[0], 1);
  }
  if (i < N) {  // i doubles as a row index here
    const int pair = src_of[i];
    if (pair < 0 || pair >= total_pairs) atomicAdd(&bad[2], 1);
    else if (row_of[pair] != i && row_of[pair] != -1) atomicAdd(&bad[2], 1);
  } else if (src_of[i] != -1) {
    atomicAdd(&bad[2], 1);
  }
}

hipError_t launch_check_layout(eep_ctx* c, int T, int32_t* bad, hipStream_t st) {
  hipError_t e = launch_fill(bad, 0, 4, st);
  const int pairs = T * c->k;
  if (e != hipSuccess || pairs == 0) return e;
  hipLaunchKernelGGL(k_check_layout, dim3((pairs + 255) / 256), dim3(256), 0, st, c->slot_of,
                     c->row_of, c->src_of, c->offset, c->status, bad, pairs, c->P);
  return hipGetLastError();
}

}  // namespace eep
