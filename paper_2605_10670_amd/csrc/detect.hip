// GPU-side failure detection, emulated on one GPU (paper Sec. 3.4; Sec. 4.1,
// the paragraph on failure detection from the GPU side; the time-out remark in
// the listing of Fig. 7).
//
// In the paper a sender bumps the receiver's signal counter after its payload
// (RDMA atomic, or a release store over NVLink); the receiver polls its counter
// inside the kernel and, if the bump does not arrive within a timeout, clears
// the peer's `active` bit and goes on without it; the host learns about it only
// after the kernel has exited.
//
// Here the ranks are partitions of one GPU, so the round that can be reproduced
// is "expert rank r has produced its outputs of this step" (producer: the expert
// stage, which stores the step's epoch into signal[r] with release semantics;
// k_signal below) and "combine waits for the signals of the ranks it reads from"
// (consumer: the combine kernel itself, see await_late_ranks in data.hip).  A
// rank that stays silent -- on one GPU only the test knob `withhold` can make
// one -- is dropped by the kernel: active[r] = 0, report[r] = 1, and the pairs
// that were routed to it lose their row.  The next step's routing already reads
// the cleared bit; no host action and no graph change is needed for that.
#include "eep_internal.hpp"

namespace eep {

__global__ __launch_bounds__(256) void k_signal(const int32_t* __restrict__ active,
                                                const int32_t* __restrict__ withhold,
                                                const int32_t* __restrict__ step_epoch,
                                                int32_t* __restrict__ signal, int R) {
  const int epoch = *step_epoch;
  for (int r = threadIdx.x; r < R; r += blockDim.x)
    if (active[r] != 0 && withhold[r] == 0)
      __hip_atomic_store(&signal[r], epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

hipError_t launch_signal(eep_ctx* c, hipStream_t st) {
  hipLaunchKernelGGL(k_signal, dim3(1), dim3(256), 0, st, c->active, c->withhold, c->step_epoch,
                     c->signal, c->R);
  return hipGetLastError();
}

}  // namespace eep
