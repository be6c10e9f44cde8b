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
// stage, which stores the step's epoch into signal[r] with release semantics)
// and "combine waits for the signals of the active ranks" (consumer: k_await,
// launched by eep_combine when detection is on).  A rank that stays silent --
// on one GPU only the test knob `withhold` can make one -- is dropped by the
// kernel itself: active[r] = 0, report[r] = 1, and the pairs that were routed to
// it lose their row so that combine skips them.  The next step's routing already
// reads the cleared bit; no host action and no graph change is needed for that.
//
// Every wait is bounded by a wall-clock budget, so every wavefront exits.
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

__global__ __launch_bounds__(1024) void k_await(int32_t* __restrict__ active,
                                                int32_t* __restrict__ mem_version,
                                                const int32_t* __restrict__ signal,
                                                const int32_t* __restrict__ step_epoch,
                                                int32_t* __restrict__ report,
                                                const int32_t* __restrict__ slot_of,
                                                int32_t* __restrict__ row_of, int R, int S,
                                                int total_pairs, long long timeout_ticks,
                                                long long max_spins) {
  extern __shared__ int32_t s_failed[];  // [R]
  __shared__ int32_t s_any;
  const int tid = threadIdx.x;
  if (tid == 0) s_any = 0;
  for (int r = tid; r < R; r += blockDim.x) s_failed[r] = 0;
  __syncthreads();
  const int epoch = *step_epoch;
  for (int r = tid; r < R; r += blockDim.x) {
    if (active[r] == 0) continue;  // only active peers are awaited
    const long long t0 = wall_clock64();
    bool arrived = false;
    // two bounds: the wall-clock budget, and a spin count in case the clock stalls
    for (long long spin = 0; spin < max_spins; ++spin) {
      if (__hip_atomic_load(&signal[r], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == epoch) {
        arrived = true;
        break;
      }
      if (wall_clock64() - t0 > timeout_ticks) break;  // the bound every wait has
      __builtin_amdgcn_s_sleep(4);
    }
    if (!arrived) {
      active[r] = 0;  // drop the peer; later steps route around it
      report[r] = 1;  // read by the host after the kernel has exited
      s_failed[r] = 1;
      s_any = 1;
    }
  }
  __syncthreads();
  if (s_any == 0) return;
  if (tid == 0) *mem_version = *mem_version + 1;  // the membership changed: status[3] shows it
  // rare path: pairs routed to a dropped rank contribute nothing to this step
  for (int i = tid; i < total_pairs; i += blockDim.x) {
    int p = slot_of[i];
    if (p >= 0 && s_failed[p / S] != 0) row_of[i] = -1;
  }
}

hipError_t launch_signal(eep_ctx* c, hipStream_t st) {
  hipLaunchKernelGGL(k_signal, dim3(1), dim3(256), 0, st, c->active, c->withhold, c->step_epoch,
                     c->signal, c->R);
  return hipGetLastError();
}

hipError_t launch_await(eep_ctx* c, int T, hipStream_t st) {
  hipLaunchKernelGGL(k_await, dim3(1), dim3(1024), sizeof(int32_t) * c->R, st, c->active,
                     c->mem->mem_version, c->signal, c->step_epoch, c->report, c->slot_of, c->row_of, c->R, c->S,
                     T * c->k, (long long)c->detect_timeout_ticks,
                     (long long)c->detect_timeout_ticks * 8 + 1024);
  return hipGetLastError();
}

}  // namespace eep
