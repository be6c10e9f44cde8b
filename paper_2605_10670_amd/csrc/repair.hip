// Weight movement for a planned repair (paper Sec. 3.5: local reuse, batched
// GPU-to-GPU relocation, reload from the DRAM backup; Sec. 5.1: the active mask
// is looked up when a transfer is issued).  One kernel moves the whole batch.
#include <vector>

#include "eep_internal.hpp"

using namespace eep;

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMoveThreads = 256;
constexpr int kMoveVecs = 8;                                            // 16-byte vectors per thread per pass
constexpr int kMovePasses = 2;
constexpr int kChunkVecs = kMoveThreads * kMoveVecs * kMovePasses;      // 64 KiB per workgroup

// Workgroup b copies chunk (b mod chunks_per_move) of move (b div chunks_per_move).
// Source and destination both lie in `weights` for a peer copy, so no restrict.
__global__ __launch_bounds__(kMoveThreads) void k_relocate(
    u32x4* weights, const u32x4* backup, int64_t slot_vecs, int chunks_per_move,
    const int32_t* __restrict__ mv_dst, const int32_t* __restrict__ mv_src,
    const int32_t* __restrict__ mv_expert, const int32_t* __restrict__ active, int S,
    int32_t* __restrict__ outcome) {
  const int m = blockIdx.x / chunks_per_move;
  const int chunk = blockIdx.x - m * chunks_per_move;
  const int dst = mv_dst[m], src = mv_src[m], e = mv_expert[m];
  // the mask as it stands now, not as it stood when the plan was made; only the
  // source is looked up (a destination may belong to a rank that has not joined yet)
  const bool from_peer = src >= 0 && active[src / S] != 0;
  if (chunk == 0 && threadIdx.x == 0)
    outcome[dst] = from_peer ? EEP_REPAIR_FROM_PEER
                   : src >= 0 ? EEP_REPAIR_FROM_DRAM_FALLBACK
                              : EEP_REPAIR_FROM_DRAM;
  const u32x4* from = from_peer ? weights + (int64_t)src * slot_vecs : backup + (int64_t)e * slot_vecs;
  u32x4* to = weights + (int64_t)dst * slot_vecs;
  const int64_t first = (int64_t)chunk * kChunkVecs + threadIdx.x;
  if ((int64_t)(chunk + 1) * kChunkVecs <= slot_vecs) {
    // full chunk: no per-vector guards, so all loads of a pass are in flight together
#pragma unroll
    for (int pass = 0; pass < kMovePasses; ++pass) {
      const int64_t base = first + (int64_t)pass * (kMoveThreads * kMoveVecs);
      u32x4 buf[kMoveVecs];
#pragma unroll
      for (int u = 0; u < kMoveVecs; ++u)
        buf[u] = __builtin_nontemporal_load(from + base + (int64_t)u * kMoveThreads);
#pragma unroll
      for (int u = 0; u < kMoveVecs; ++u) to[base + (int64_t)u * kMoveThreads] = buf[u];
    }
    return;
  }
  // ragged last chunk of a slot
  for (int64_t v = first; v < slot_vecs; v += kMoveThreads) to[v] = __builtin_nontemporal_load(from + v);
}

int fail_hip(eep_ctx* c, hipError_t e) {
  c->last_hip_error = (int)e;
  return EEP_ERR_HIP;
}

// Is [p, p + bytes) GPU-readable memory of the kind the contract names?  On
// success *dev_ptr is the address a kernel uses.
bool gpu_readable(const void* p, int64_t bytes, bool device_only, int device, const void** dev_ptr) {
  hipPointerAttribute_t at;
  if (hipPointerGetAttributes(&at, p) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  const bool on_device = at.type == hipMemoryTypeDevice && at.device == device;
  const bool pinned_host = at.type == hipMemoryTypeHost && !device_only && at.devicePointer != nullptr;
  if (!on_device && !pinned_host) return false;
  // the enclosing allocation must contain the whole range
  void* base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange((hipDeviceptr_t*)&base, &size, (hipDeviceptr_t)p) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  if ((const char*)p + bytes > (const char*)base + size) return false;
  *dev_ptr = p;  // pinned host memory is mapped at its host address
  return true;
}

}  // namespace

extern "C" {

int eep_apply_repair(eep_ctx* c, void* weights, const void* backup, int64_t slot_bytes,
                     const int32_t* new_p2l, const int32_t* kind, const int32_t* src_slot,
                     void* stream) {
  if (!c || !weights || !new_p2l || !kind || !src_slot || slot_bytes <= 0)
    return EEP_ERR_INVALID_ARG;
  if (slot_bytes % 16 != 0 || ((uintptr_t)weights & 15u) || ((uintptr_t)backup & 15u))
    return EEP_ERR_ALIGN;
  c = c->tables;  // a staging context names its owner's tables
  const int P = c->P, S = c->S;
  std::vector<int32_t> dst, src, expert;
  for (int p = 0; p < P; ++p) {
    const int e = new_p2l[p];
    if (e < -1 || e >= c->E) return EEP_ERR_INVALID_ARG;
    switch (kind[p]) {
      case EEP_SRC_NONE:
        break;
      case EEP_SRC_LOCAL:
        if (e < 0 || c->h_p2l[p] != e) return EEP_ERR_INVALID_ARG;
        break;
      case EEP_SRC_PEER: {
        const int q = src_slot[p];
        if (e < 0 || q < 0 || q >= P || q == p || c->h_p2l[q] != e) return EEP_ERR_INVALID_ARG;
        if (kind[q] == EEP_SRC_PEER || kind[q] == EEP_SRC_DRAM) return EEP_ERR_INVALID_ARG;
        dst.push_back(p); src.push_back(q); expert.push_back(e);
        break;
      }
      case EEP_SRC_DRAM:
        if (e < 0) return EEP_ERR_INVALID_ARG;
        dst.push_back(p); src.push_back(-1); expert.push_back(e);
        break;
      default:
        return EEP_ERR_INVALID_ARG;
    }
  }
  // Sources are looked up in the device mask per transfer, so an unread detection round
  // does not matter for the movement; the coverage check of a strict context does need a
  // current mask.
  if (c->cfg.strict_coverage) {
    if (c->mem->unread_round) return EEP_ERR_STATE;
    if (host_uncovered_experts(P, c->E, S, new_p2l, c->mem->h_active.data()) > 0)
      return EEP_ERR_COVERAGE;
  }
  const int n_moves = (int)dst.size();
  const int64_t slot_vecs = slot_bytes / 16;
  const int64_t chunks = (slot_vecs + kChunkVecs - 1) / kChunkVecs;
  if ((int64_t)n_moves * chunks > 0x7fffffffLL) return EEP_ERR_INVALID_ARG;
  const void* weights_dev = nullptr;
  const void* backup_dev = nullptr;
  if (!gpu_readable(weights, (int64_t)P * slot_bytes, true, c->device, &weights_dev))
    return EEP_ERR_INVALID_ARG;
  if (n_moves > 0) {
    if (!backup) return EEP_ERR_INVALID_ARG;
    if (!gpu_readable(backup, (int64_t)c->E * slot_bytes, false, c->device, &backup_dev))
      return EEP_ERR_INVALID_ARG;
  }

  hipStream_t st = (hipStream_t)stream;
  hipError_t e = launch_fill(c->mv_outcome, EEP_REPAIR_UNTOUCHED, P, st);
  if (e == hipSuccess && n_moves > 0) {
    e = launch_patch(c->mv_dst, dst.data(), n_moves, nullptr, st);
    if (e == hipSuccess) e = launch_patch(c->mv_src, src.data(), n_moves, nullptr, st);
    if (e == hipSuccess) e = launch_patch(c->mv_expert, expert.data(), n_moves, nullptr, st);
    if (e == hipSuccess) {
      k_relocate<<<dim3((unsigned)(n_moves * chunks)), dim3(kMoveThreads), 0, st>>>(
          (u32x4*)weights_dev, (const u32x4*)backup_dev, slot_vecs, (int)chunks, c->mv_dst,
          c->mv_src, c->mv_expert, c->active, S, c->mv_outcome);
      e = hipGetLastError();
    }
  }
  if (e != hipSuccess) return fail_hip(c, e);
  return publish_placement(c, new_p2l, true, st);
}

int eep_read_repair_outcome(eep_ctx* c, int32_t* outcome_host) {
  if (!c || !outcome_host) return EEP_ERR_INVALID_ARG;
  c = c->tables;  // the repair ran on the tables' owner, whichever context was named
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess)
    e = hipMemcpy(outcome_host, c->mv_outcome, sizeof(int32_t) * (size_t)c->P, hipMemcpyDeviceToHost);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

}  // extern "C"
