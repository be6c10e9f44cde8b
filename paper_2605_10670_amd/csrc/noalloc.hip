// eep_dispatch_layout_noalloc: the routing + layout pass for callers that cannot
// allocate device memory (code under hipGraph capture, tight serving loops,
// harnesses that forbid hipMalloc).  No context: the caller passes the tables
// and every output array; the pass's scratch (per-tile slot counts, per-tile
// prefixes, per-tile drop counters, a step counter) lives in a file-scope
// device array of fixed size instead of a context slab.  The kernels are the
// ones eep_dispatch_layout launches; they take the scratch as pointer arguments
// either way.
#include <mutex>

#include "eep_internal.hpp"

namespace {

constexpr int64_t kScratchInts = EEP_NOALLOC_SCRATCH_BYTES / (int64_t)sizeof(int32_t);
constexpr int kMaxDevices = 64;

// Every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; device addresses come from scratch_of_current_device().
static __device__ __align__(256) int32_t scratch[kScratchInts];

// Layout of the array (ints):
//   [0]                 a word nothing ever writes: stays 0 from load time
//   [64]                step counter the layout kernels bump (unused by callers)
//   [128 ...)           cnt_tile[tiles*P], base_tile[tiles*P], blk_unc[tiles], blk_msk[tiles],
//                       each rounded up to 64 ints
constexpr int64_t kZeroWord = 0, kEpochWord = 64, kFirstArray = 128;

std::mutex g_lock;
int32_t* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, once resolved

int scratch_of_current_device(int32_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return EEP_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return EEP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> hold(g_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return EEP_ERR_HIP;
    }
    g_scratch_ptr[dev] = (int32_t*)p;
  }
  *out = g_scratch_ptr[dev];
  return EEP_OK;
}

int64_t round_up64(int64_t ints) { return (ints + 63) / 64 * 64; }

}  // namespace

extern "C" {

int64_t eep_noalloc_scratch_needed(int32_t num_ranks, int32_t slots_per_rank, int32_t T) {
  if (num_ranks < 1 || slots_per_rank < 1 || T < 0 || T % num_ranks != 0) return EEP_ERR_INVALID_ARG;
  const eep::Tiling g = eep::make_tiling(T, num_ranks);
  const int64_t P = (int64_t)num_ranks * slots_per_rank;
  const int64_t ints = kFirstArray + 2 * round_up64((int64_t)g.num_tiles * P) +
                       2 * round_up64(g.num_tiles);
  return ints * (int64_t)sizeof(int32_t);
}

int eep_dispatch_layout_noalloc(const eep_layout_shape* shape, const int32_t* topk_idx,
                                const int32_t* active, const int32_t* l2p_off,
                                const int32_t* l2p_list, const int32_t* table_version,
                                const eep_layout_out* out, int32_t T, void* stream) {
  if (!shape || !out || !active || !l2p_off || !l2p_list) return EEP_ERR_INVALID_ARG;
  const int R = shape->num_ranks, S = shape->slots_per_rank, E = shape->num_logical,
            k = shape->topk;
  if (R < 1 || S < 1 || E < 1 || k < 1 || k > eep::kMaxTopk) return EEP_ERR_INVALID_ARG;
  if ((int64_t)R * S > (1 << 20) || E > (1 << 20)) return EEP_ERR_INVALID_ARG;
  if (shape->policy != EEP_SPREAD && shape->policy != EEP_FIRST_LIVE) return EEP_ERR_INVALID_ARG;
  if (T < 0 || T % R != 0 || (int64_t)T * k > (int64_t)1 << 30) return EEP_ERR_INVALID_ARG;
  if (T > 0 && !topk_idx) return EEP_ERR_INVALID_ARG;
  if (!out->slot_of || !out->row_of || !out->src_of || !out->count || !out->offset ||
      !out->rank_count || !out->rank_offset || !out->cnt_src || !out->status)
    return EEP_ERR_INVALID_ARG;
  const int P = R * S;
  if (!eep::layout_shape_fits(E, P, R, k)) return EEP_ERR_INVALID_ARG;
  if (eep_noalloc_scratch_needed(R, S, T) > EEP_NOALLOC_SCRATCH_BYTES) return EEP_ERR_SCRATCH;

  int32_t* base = nullptr;
  int rc = scratch_of_current_device(&base);
  if (rc != EEP_OK) return rc;

  const eep::Tiling g = eep::make_tiling(T, R);
  const int64_t n_tile = round_up64((int64_t)g.num_tiles * P), n_blk = round_up64(g.num_tiles);
  eep::LayoutIO io;
  io.R = R; io.S = S; io.P = P; io.E = E; io.k = k; io.policy = shape->policy;
  io.topk_idx = topk_idx;
  io.l2p_off = l2p_off; io.l2p_list = l2p_list; io.active = active;
  // status[3] = *table_version, or 0 without one: the kernels add two words
  io.tbl_version = table_version ? table_version : base + kZeroWord;
  io.mem_version = base + kZeroWord;
  io.slot_of = out->slot_of; io.row_of = out->row_of; io.src_of = out->src_of;
  io.count = out->count; io.offset = out->offset; io.rank_count = out->rank_count;
  io.rank_offset = out->rank_offset; io.cnt_src = out->cnt_src; io.status = out->status;
  // Nothing in the scratch has to start at zero: every word a kernel of this
  // pass reads was written earlier in the same pass (k_map_count fills all of
  // cnt_tile / blk_unc / blk_msk for the tiles of this T, k_tile_prefix all of
  // base_tile), so what the previous call left behind is never seen.
  io.cnt_tile = base + kFirstArray;
  io.base_tile = io.cnt_tile + n_tile;
  io.blk_unc = io.base_tile + n_tile;
  io.blk_msk = io.blk_unc + n_blk;
  io.step_epoch = base + kEpochWord;
  return eep::launch_layout(io, T, (hipStream_t)stream) == hipSuccess ? EEP_OK : EEP_ERR_HIP;
}

}  // extern "C"
