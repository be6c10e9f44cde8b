// Internal declarations shared by the HIP sources of libeep (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "eep.h"

namespace eep {

// Tokens of one layout tile never exceed this; a tile never straddles two
// source ranks.  128 tokens = 4 bitmap words per slot.
constexpr int kTileTokens = 128;
constexpr int kBitmapWords = kTileTokens / 32;
constexpr int kMaxTopk = 32;
constexpr int kDedupMaxRanks = 1024;  // the de-duplicated layout keeps per-rank bitmaps in LDS
constexpr int kPatchInts = 512;  // ints carried by value in one table-patch launch
constexpr size_t kLayoutLdsLimit = 60 * 1024;  // the layout kernels keep their tables in LDS

struct Tiling {
  int tokens_per_rank;  // T / R
  int tiles_per_rank;   // nt
  int tile_tokens;      // TT <= kTileTokens
  int num_tiles;        // NB = R * nt
};

inline Tiling make_tiling(int T, int R) {
  Tiling g;
  g.tokens_per_rank = T / R;
  g.tiles_per_rank = (g.tokens_per_rank + kTileTokens - 1) / kTileTokens;
  if (g.tiles_per_rank < 1) g.tiles_per_rank = 1;
  g.tile_tokens = (g.tokens_per_rank + g.tiles_per_rank - 1) / g.tiles_per_rank;
  g.num_tiles = (T > 0) ? R * g.tiles_per_rank : 0;
  return g;
}

// LDS bytes of the map kernel: placement CSR, active mask, live-replica table,
// per-slot token bitmaps and the tile's router indices / chosen slots.
inline size_t map_lds_bytes(int E, int P, int R, int tile_tokens, int k) {
  return sizeof(int32_t) * ((size_t)(E + 1) + P + R + E + P + (size_t)P * kBitmapWords +
                            (size_t)2 * tile_tokens * k);
}

inline int dtype_bytes(int dt) { return dt == EEP_F32 ? 4 : dt == EEP_BF16 ? 2 : 1; }

struct PatchChunk {
  int32_t v[kPatchInts];
};

}  // namespace eep

// The membership of one EP instance (the peer table's `active` column, Fig. 7):
// one device array and one host copy, shared by every context of the instance.
// It lives in the slab of the context that created it (the "root").
struct eep_membership {
  int R;
  int32_t* active;       // device [R]
  int32_t* mem_version;  // device word: membership changes (host updates + ranks dropped by kernels)
  std::vector<int32_t> h_active;
  // A combine with failure detection has been queued since the last eep_read_failures: a
  // kernel may have cleared bits of `active` that h_active still shows as set.
  bool unread_round;
  std::vector<eep_ctx*> members;  // root first
};

struct eep_ctx {
  eep_config cfg;
  eep_membership* mem;  // shared; owned by the root context
  int R, S, S_prim, P, E, k, H, T_max;
  int64_t x_row_bytes, y_row_bytes, out_row_bytes, scale_row_bytes;
  int device;
  int max_tiles;

  void* slab;  // the one device allocation everything below points into
  bool owns_slab;  // false: the caller supplied it (eep_create_with_workspace)
  // tables (fixed addresses, contents patched in place)
  int32_t *active;  // == mem->active
  int32_t *own_active, *mem_version_word;  // slab space used only when this context is the root
  int32_t *p2l, *l2p_off, *l2p_list, *tbl_version;  // tbl_version: placement updates of this context
  // per-step layout results
  int32_t *slot_of, *row_of, *src_of, *count, *offset, *rank_count, *rank_offset, *cnt_src, *status;
  // per-step scratch
  int32_t *cnt_tile, *base_tile, *blk_unc, *blk_msk;
  // GPU-side failure detection: step counter, per-rank arrival word (holds the
  // epoch of the last step whose expert outputs arrived), test knob that mutes
  // a rank, failure report written by the waiting kernel
  int32_t *step_epoch, *signal, *withhold, *report;
  int32_t* round_ok;  // epoch of the last step whose combine found every expected signal in place
  int32_t* check_bad;  // [4] violation counters of eep_debug_check_layout
  // repair batch: destination slot, source slot (-1 = backup), logical expert of
  // each move, and what the relocation kernel did per slot
  int32_t *mv_dst, *mv_src, *mv_expert, *mv_outcome;
  // de-duplicated dispatch: per pair the row in the rank-major buffer (dd_row), the same
  // but -1 unless the pair carries the row (dd_dst: what the pack kernel reads), the row of
  // the rank-major buffer behind every expert-major row (dd_expand), per-rank counts and
  // offsets, per-tile per-rank counts, {N_d}
  int32_t *dd_row, *dd_dst, *dd_expand, *dd_count, *dd_offset, *dd_tile, *dd_status;
  int dedup_T;  // T of the last eep_dedup_layout, -1 if none
  int64_t detect_timeout_ticks;  // 0 = detection off
  int wall_clock_khz;

  // host shadows of the tables (coverage is validated without touching the GPU)
  std::vector<int32_t> h_p2l;
  // Double-buffered staging: a staging context shares the placement tables (device arrays
  // and host shadow) of `tables`, the context they belong to; an ordinary context points
  // to itself.  n_staging counts the staging contexts that point here.
  eep_ctx* tables;
  int n_staging;
  hipEvent_t ev_fork, ev_join;  // created on first use by eep_staging_fork
  int layout_T;  // T of the last dispatch_layout, -1 if none yet
  int last_hip_error;
  int64_t field_ints[EEP_V_NUM_FIELDS];
};

namespace eep {

// host_logic.cpp (no GPU touched)
int host_uncovered_experts(int P, int E, int S, const int32_t* p2l, const int32_t* active);
void host_replica_lists(int P, int E, int S, int S_prim, const int32_t* p2l, int32_t* l2p_off,
                        int32_t* l2p_list);
// layout.hip
// Everything one layout pass touches, as plain device pointers: the context's
// arrays for eep_dispatch_layout, the caller's arrays plus the static scratch
// array for eep_dispatch_layout_noalloc.
struct LayoutIO {
  int R, S, P, E, k, policy;
  const int32_t *topk_idx, *l2p_off, *l2p_list, *active, *tbl_version, *mem_version;
  int32_t *slot_of, *row_of, *src_of, *count, *offset, *rank_count, *rank_offset, *cnt_src, *status;
  // scratch: per-tile slot counts and prefixes [tiles][P], per-tile drop counters [tiles],
  // the step counter
  int32_t *cnt_tile, *base_tile, *blk_unc, *blk_msk, *step_epoch;
};
bool layout_shape_fits(int E, int P, int R, int k);  // tables fit the kernels' LDS budget
hipError_t launch_layout(const LayoutIO& io, int T, hipStream_t st);
hipError_t launch_layout(eep_ctx* c, const int32_t* topk_idx, int T, hipStream_t st);
hipError_t launch_check_layout(eep_ctx* c, int T, int32_t* bad /* device [4] */, hipStream_t st);
// data.hip
hipError_t launch_pack(eep_ctx* c, const void* x, const float* x_scale, void* recv_x,
                       float* recv_scale, int T, hipStream_t st);
// pack through another row table (the de-duplicated dispatch's), payload rows only
hipError_t launch_pack_rows(eep_ctx* c, const int32_t* rows, const void* x, void* recv, int T,
                            hipStream_t st);
hipError_t launch_expand(eep_ctx* c, const void* recv_dedup, void* recv_x, int T, hipStream_t st);
hipError_t launch_dedup_layout(eep_ctx* c, int T, hipStream_t st);
hipError_t launch_pack_quant(eep_ctx* c, const void* x_bf16, void* recv_q, float* recv_scale, int T,
                             hipStream_t st);
hipError_t launch_combine(eep_ctx* c, const void* y, const float* w, void* out, int T,
                          hipStream_t st);
hipError_t launch_stub(eep_ctx* c, int kind, const void* recv_x, const float* recv_scale,
                       const float* expert_scale, void* y, int T, hipStream_t st);
// detect.hip
hipError_t launch_signal(eep_ctx* c, hipStream_t st);
// api.hip
int publish_placement(eep_ctx* c, const int32_t* p2l_host, bool mask_may_be_stale, hipStream_t st);
// tables.hip
hipError_t launch_patch(int32_t* dst, const int32_t* src_host, int n, int32_t* version_dst,
                        hipStream_t st);
hipError_t launch_fill(int32_t* dst, int32_t value, int64_t n, hipStream_t st);

}  // namespace eep
