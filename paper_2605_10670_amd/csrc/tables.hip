// In-place table patching (paper Sec. 4.1 "In-place peer-table updates",
// Fig. 4, Fig. 8): the tables live at fixed device addresses; an update is a
// tiny kernel that carries the new contents BY VALUE in its kernel arguments,
// so no host buffer has to outlive the call and nothing is allocated, copied
// through staging memory or synchronised.
#include "eep_internal.hpp"

namespace eep {

// version_dst (may be null): a word that counts the changes of the table; it is bumped on
// the device, so that changes made by kernels (a rank dropped by the waiting kernel) and
// changes made by the host share one count.
__global__ __launch_bounds__(256) void k_patch(int32_t* __restrict__ dst, int n, PatchChunk chunk,
                                               int32_t* version_dst) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) dst[i] = chunk.v[i];
  if (version_dst != nullptr && threadIdx.x == 0) *version_dst = *version_dst + 1;
}

__global__ __launch_bounds__(256) void k_fill(int32_t* __restrict__ dst, int32_t value, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = value;
}

hipError_t launch_patch(int32_t* dst, const int32_t* src_host, int n, int32_t* version_dst,
                        hipStream_t st) {
  // The version word is bumped by the last chunk, after the data it describes.
  for (int done = 0; done < n || (n == 0 && done == 0); done += kPatchInts) {
    PatchChunk chunk;
    int m = n - done < kPatchInts ? n - done : kPatchInts;
    for (int i = 0; i < m; ++i) chunk.v[i] = src_host[done + i];
    for (int i = m; i < kPatchInts; ++i) chunk.v[i] = 0;
    bool last = done + kPatchInts >= n;
    hipLaunchKernelGGL(k_patch, dim3(1), dim3(256), 0, st, dst + done, m, chunk,
                       last ? version_dst : nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (n == 0) break;
  }
  return hipSuccess;
}

hipError_t launch_fill(int32_t* dst, int32_t value, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_fill, dim3((unsigned)blocks), dim3(256), 0, st, dst, value, n);
  return hipGetLastError();
}

}  // namespace eep
