// Measurement helpers, no part of the step: streaming kernels with a known
// byte count and a known read:write mix, as yardsticks for the data kernels.
//   k_calibration_copy    plain loads and stores, dst[i] = src[i]; the kernel
//                         that hardware HBM counters are scaled by
//   k_calibration_stream  RD reads and WR writes of 16 bytes per thread, with
//                         the access flavours of pack and combine (read-once
//                         non-temporal loads, write-through stores), perfectly
//                         sequential in every plane: what the memory system
//                         gives a kernel with the step's mix of reads and
//                         writes when nothing is scattered
#include "eep_internal.hpp"

namespace eep {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_calibration_copy(const u32x4* __restrict__ src,
                                                          u32x4* __restrict__ dst, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// Thread i reads vector i of RD source planes and writes vector i of WR
// destination planes (planes `stride` vectors apart).  The value written
// depends on everything read, so no load can be dropped.
template <int RD, int WR>
__global__ __launch_bounds__(256) void k_calibration_stream(const u32x4* __restrict__ src,
                                                            u32x4* __restrict__ dst, int64_t n,
                                                            int64_t stride) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  u32x4 v = {1u, 2u, 3u, 4u};
#pragma unroll
  for (int j = 0; j < RD; ++j) v ^= __builtin_nontemporal_load(&src[j * stride + i]);
#pragma unroll
  for (int j = 0; j < WR; ++j) {
    u32x4 o = v + (uint32_t)j;
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(&dst[j * stride + i]), "v"(o)
                 : "memory");
  }
}

}  // namespace eep

extern "C" {

int eep_calibration_copy(void* dst, const void* src, int64_t bytes, void* stream) {
  if (!dst || !src || bytes < 0 || bytes % 16 != 0 || ((uintptr_t)dst & 15) ||
      ((uintptr_t)src & 15) || bytes / 16 / 256 >= ((int64_t)1 << 31))
    return EEP_ERR_INVALID_ARG;
  if (bytes == 0) return EEP_OK;
  int64_t n = bytes / 16;
  hipLaunchKernelGGL(eep::k_calibration_copy, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, (const eep::u32x4*)src, (eep::u32x4*)dst, n);
  return hipGetLastError() == hipSuccess ? EEP_OK : EEP_ERR_HIP;
}

int eep_calibration_stream(void* dst, const void* src, int64_t plane_bytes,
                           int64_t plane_stride_bytes, int32_t reads, int32_t writes,
                           void* stream) {
  if (!dst || !src || plane_bytes < 0 || plane_bytes % 16 != 0 || plane_stride_bytes % 16 != 0 ||
      plane_stride_bytes < plane_bytes || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15) ||
      plane_bytes / 16 / 256 >= ((int64_t)1 << 31))
    return EEP_ERR_INVALID_ARG;
  const int64_t n = plane_bytes / 16, stride = plane_stride_bytes / 16;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  hipStream_t st = (hipStream_t)stream;
  const eep::u32x4* s = (const eep::u32x4*)src;
  eep::u32x4* d = (eep::u32x4*)dst;
  if (reads != 1 && reads != 8) return EEP_ERR_INVALID_ARG;
  if (writes != 1 && writes != 8) return EEP_ERR_INVALID_ARG;
  if (n == 0) return EEP_OK;
  if (reads == 1 && writes == 1)
    hipLaunchKernelGGL((eep::k_calibration_stream<1, 1>), grid, block, 0, st, s, d, n, stride);
  else if (reads == 1 && writes == 8)
    hipLaunchKernelGGL((eep::k_calibration_stream<1, 8>), grid, block, 0, st, s, d, n, stride);
  else if (reads == 8 && writes == 1)
    hipLaunchKernelGGL((eep::k_calibration_stream<8, 1>), grid, block, 0, st, s, d, n, stride);
  else
    hipLaunchKernelGGL((eep::k_calibration_stream<8, 8>), grid, block, 0, st, s, d, n, stride);
  return hipGetLastError() == hipSuccess ? EEP_OK : EEP_ERR_HIP;
}

}  // extern "C"
