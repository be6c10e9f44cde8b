// dispatch_layout: route every (token, j) pair to a live replica slot, count
// pairs per slot, prefix-sum the counts into receive-buffer offsets and give
// every routed pair its row, rows of one slot ordered by ascending token.
//
// Paper: Fig. 7 (the dispatch path skips peers whose `active` is 0), Sec. 5.1
// (slot -> logical expert map and all locations of each logical expert),
// Sec. 3.2 (validity contract), Sec. 4.1 (contiguous per-expert receive
// buffers as in prior work).
//
// Two or three launches, all tiny and latency-bound (the step's metadata is
// < 1 MB), so the design goal is a short chain of dependent memory round trips,
// not bandwidth.  Every kernel issues all its global loads before its first
// wait.
//   k_map_count  one workgroup per tile of <= 128 tokens of ONE source rank.
//                Placement CSR, active mask and the tile's router indices are
//                fetched into LDS with independent loads; the live-replica
//                table is then built from LDS.  For every slot the kernel
//                records a bitmap of the tile's tokens that hit it: popcount
//                of the bitmap is the tile's count, popcount of the bits below
//                a token is that pair's stable rank inside the tile.  No
//                atomics on positions, so the order is deterministic.
//   k_scan_position  (<= 64 tiles) one workgroup per tile.  Thread = slot walks
//                the [tiles][P] count matrix in registers (coalesced, no
//                cross-lane traffic) for the slot total and the pairs of
//                earlier tiles; slot totals are then scanned across the
//                workgroup; row = slot offset + pairs of earlier tiles + rank
//                in tile.  Each workgroup repeats the small scan rather than
//                wait for another kernel.
//   k_tile_prefix + k_position  (> 64 tiles) the tile prefixes are computed once
//                by a few workgroups, then a wide grid computes the rows.
#include "eep_internal.hpp"

namespace eep {

constexpr int kMapThreads = 1024;
constexpr int kPosThreads = 256;

// Tile b covers tokens [t0, t0 + ntok) of source rank b / tiles_per_rank; the
// last tile of a rank may be shorter, and no tile crosses into the next rank.
struct TileRange {
  int src_rank, sub_tile, t0, ntok;
};
__device__ inline TileRange tile_range(int b, int tokens_per_rank, int tiles_per_rank,
                                       int tile_tokens) {
  TileRange r;
  r.src_rank = b / tiles_per_rank;
  r.sub_tile = b - r.src_rank * tiles_per_rank;
  r.t0 = r.src_rank * tokens_per_rank + r.sub_tile * tile_tokens;
  int t1 = r.t0 + tile_tokens;
  const int rank_end = (r.src_rank + 1) * tokens_per_rank;
  if (t1 > rank_end) t1 = rank_end;
  r.ntok = t1 > r.t0 ? t1 - r.t0 : 0;
  return r;
}

// A token can hit a slot at most once: its k logical experts are distinct
// (repeats are masked) and a slot holds one logical expert.  So one bit per
// (slot, token of the tile) is enough.
template <int KC>  // KC = compile-time k (power of two) or 0 for any k
__global__ __launch_bounds__(kMapThreads) void k_map_count(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ l2p_off,
    const int32_t* __restrict__ l2p_list, const int32_t* __restrict__ active,
    int32_t* __restrict__ slot_of, int32_t* __restrict__ rank_in_tile,
    int32_t* __restrict__ cnt_tile, int32_t* __restrict__ blk_unc,
    int32_t* __restrict__ blk_msk, int k_rt, int E, int R, int S, int P, int tokens_per_rank,
    int tiles_per_rank, int tile_tokens, int policy) {
  const int k = KC > 0 ? KC : k_rt;
  extern __shared__ int32_t smem[];
  int32_t* s_off = smem;                         // [E+1] replica-list starts (CSR)
  int32_t* s_list = s_off + (E + 1);             // [P] replica lists, canonical order
  int32_t* s_active = s_list + P;                // [R]
  int32_t* s_nlive = s_active + R;               // [E] live replicas of expert e
  int32_t* s_live = s_nlive + E;                 // [P] live replicas, compacted per expert
  uint32_t* s_bm = (uint32_t*)(s_live + P);      // [P][kBitmapWords]
  int32_t* s_idx = (int32_t*)(s_bm + P * kBitmapWords);  // [tile_tokens*k] router indices
  int32_t* s_slot = s_idx + tile_tokens * k;             // [tile_tokens*k] chosen slots
  __shared__ int32_t s_drop[2];

  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  const TileRange tr = tile_range(b, tokens_per_rank, tiles_per_rank, tile_tokens);
  const int t0 = tr.t0;
  const int npairs = tr.ntok * k;
  const int64_t g0 = (int64_t)t0 * k;

  // every global read of this kernel is issued here, none depends on another
  for (int i = tid; i < npairs; i += kMapThreads) s_idx[i] = topk_idx[g0 + i];
  for (int i = tid; i <= E; i += kMapThreads) s_off[i] = l2p_off[i];
  for (int i = tid; i < P; i += kMapThreads) s_list[i] = l2p_list[i];
  for (int i = tid; i < R; i += kMapThreads) s_active[i] = active[i];
  for (int i = tid; i < P * kBitmapWords; i += kMapThreads) s_bm[i] = 0u;
  if (tid < 2) s_drop[tid] = 0;
  __syncthreads();

  for (int e = tid; e < E; e += kMapThreads) {
    int o = s_off[e], o1 = s_off[e + 1], n = 0;
    for (int q = o; q < o1; ++q) {
      int p = s_list[q];
      if (s_active[p / S] != 0) s_live[o + n++] = p;  // failed peers are skipped
    }
    s_nlive[e] = n;
  }
  __syncthreads();

  int n_unc = 0, n_msk = 0;
  for (int i = tid; i < npairs; i += kMapThreads) {
    int tl = i / k;
    int j = i - tl * k;
    int e = s_idx[i];
    int p = -1;
    if (e < 0 || e >= E) {
      ++n_msk;
    } else {
      bool repeated = false;
      for (int jj = 0; jj < j; ++jj) repeated |= (s_idx[tl * k + jj] == e);
      if (repeated) {
        ++n_msk;
      } else {
        int n = s_nlive[e];
        if (n == 0) {
          ++n_unc;
        } else {
          int sel = (policy == EEP_FIRST_LIVE || n == 1) ? 0 : (t0 + tl) % n;
          p = s_live[s_off[e] + sel];
          atomicOr(&s_bm[p * kBitmapWords + (tl >> 5)], 1u << (tl & 31));
        }
      }
    }
    s_slot[i] = p;
    slot_of[g0 + i] = p;
  }
  if (n_unc) atomicAdd(&s_drop[0], n_unc);
  if (n_msk) atomicAdd(&s_drop[1], n_msk);
  __syncthreads();

  for (int i = tid; i < npairs; i += kMapThreads) {
    int p = s_slot[i];
    int r = -1;
    if (p >= 0) {
      int tl = i / k;
      int w = tl >> 5;
      const uint32_t* bm = &s_bm[p * kBitmapWords];
      r = __popc(bm[w] & ((1u << (tl & 31)) - 1u));
      for (int ww = 0; ww < w; ++ww) r += __popc(bm[ww]);
    }
    rank_in_tile[g0 + i] = r;
  }
  for (int p = tid; p < P; p += kMapThreads) {
    int c = 0;
#pragma unroll
    for (int w = 0; w < kBitmapWords; ++w) c += __popc(s_bm[p * kBitmapWords + w]);
    cnt_tile[(int64_t)b * P + p] = c;
  }
  if (tid == 0) {
    blk_unc[b] = s_drop[0];
    blk_msk[b] = s_drop[1];
  }
}

// inclusive scan inside aligned groups of `seg` lanes (seg a power of two <= 64)
__device__ inline int seg_inclusive_scan(int v, int seg) {
  const int sl = (threadIdx.x & 63) & (seg - 1);
  for (int d = 1; d < seg; d <<= 1) {
    int o = __shfl_up(v, d, 64);
    if (sl >= d) v += o;
  }
  return v;
}

// Exclusive scan of s_count[0..P) into s_offset[0..P] by the whole workgroup
// (NT threads, NT/64 <= 16 wavefronts).  Ends with a barrier.
template <int NT>
__device__ inline void block_exclusive_scan(const int32_t* s_count, int32_t* s_offset,
                                            int32_t* s_wave, int P) {
  const int tid = threadIdx.x;
  const int ipt = (P + NT - 1) / NT;
  const int lo = tid * ipt;
  int hi = lo + ipt;
  if (hi > P) hi = P;
  int local = 0;
  for (int p = lo; p < hi; ++p) local += s_count[p];
  int incl = seg_inclusive_scan(local, 64);
  if ((tid & 63) == 63) s_wave[tid >> 6] = incl;
  __syncthreads();
  int wave_base = 0;
  for (int w = 0; w < (tid >> 6); ++w) wave_base += s_wave[w];
  int run = wave_base + incl - local;
  for (int p = lo; p < hi; ++p) {
    s_offset[p] = run;
    run += s_count[p];
  }
  if (tid == NT - 1) s_offset[P] = wave_base + incl;
  __syncthreads();
}

// Per-step tables every consumer needs, written once by one workgroup
// (`count` may be null when another kernel has already written it).
template <int NT>
__device__ inline void write_step_tables(const int32_t* s_count, const int32_t* s_offset,
                                         int dropped_unc, int dropped_msk, int version,
                                         int32_t* __restrict__ count, int32_t* __restrict__ offset,
                                         int32_t* __restrict__ rank_count,
                                         int32_t* __restrict__ rank_offset,
                                         int32_t* __restrict__ status,
                                         int32_t* __restrict__ step_epoch, int R, int S, int P) {
  const int tid = threadIdx.x;
  for (int p = tid; p <= P; p += NT) {
    offset[p] = s_offset[p];
    if (count != nullptr && p < P) count[p] = s_count[p];
  }
  for (int r = tid; r < R; r += NT) {
    rank_offset[r] = s_offset[r * S];
    rank_count[r] = s_offset[(r + 1) * S] - s_offset[r * S];
  }
  if (tid == 0) {
    rank_offset[R] = s_offset[P];
    status[0] = s_offset[P];
    status[1] = dropped_unc;
    status[2] = dropped_msk;
    status[3] = version;
    *step_epoch = *step_epoch + 1;  // one increment per step, on the device (graph replays too)
  }
}

// ---------------------------------------------------------------------------
// Few tiles (<= 64, the decode regime): scan and position fused.  Every
// workgroup (one per tile) re-derives what it needs from the [tiles][P] count
// matrix -- slot totals and the pairs of earlier tiles -- with thread = slot and
// the tiles walked in registers, so that the kernel has one round of global
// loads (two beyond 32 tiles), all issued before the first wait.
// ---------------------------------------------------------------------------
constexpr int kFusedThreads = 512;
constexpr int kFusedPairs = 4;    // pairs of the tile kept in registers per thread
constexpr int kTileBatch = 32;    // count-matrix rows fetched per round

template <int KC>
__global__ __launch_bounds__(kFusedThreads) void k_scan_position(
    const int32_t* __restrict__ cnt_tile, const int32_t* __restrict__ blk_unc,
    const int32_t* __restrict__ blk_msk, const int32_t* __restrict__ tbl_version,
    const int32_t* __restrict__ mem_version, const int32_t* __restrict__ slot_of,
    int32_t* __restrict__ row_of,
    int32_t* __restrict__ src_of, int32_t* __restrict__ count, int32_t* __restrict__ offset,
    int32_t* __restrict__ rank_count, int32_t* __restrict__ rank_offset,
    int32_t* __restrict__ cnt_src, int32_t* __restrict__ status,
    int32_t* __restrict__ step_epoch, int k_rt, int num_tiles, int tokens_per_rank,
    int tiles_per_rank, int tile_tokens, int R, int S, int P) {
  const int k = KC > 0 ? KC : k_rt;
  extern __shared__ int32_t smem[];
  int32_t* s_count = smem;           // [P]   pairs per slot, all tiles
  int32_t* s_offset = s_count + P;   // [P+1] exclusive scan of s_count
  int32_t* s_pre = s_offset + P + 1; // [P]   pairs per slot in tiles before this one
  __shared__ int32_t s_wave[kFusedThreads / 64];
  __shared__ int32_t s_drop[2];
  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  const TileRange tr = tile_range(b, tokens_per_rank, tiles_per_rank, tile_tokens);
  const int src_rank = tr.src_rank, sub_tile = tr.sub_tile;
  const int npairs = tr.ntok * k;
  const int g0 = tr.t0 * k;
  const int first = src_rank * tiles_per_rank;  // tiles [first, first + tiles_per_rank) share
                                                // this tile's source rank

  int my_slot[kFusedPairs], my_rank[kFusedPairs];
#pragma unroll
  for (int u = 0; u < kFusedPairs; ++u) {
    int i = tid + u * kFusedThreads;
    my_slot[u] = i < npairs ? slot_of[g0 + i] : -1;
    my_rank[u] = i < npairs ? row_of[g0 + i] : 0;  // rank inside the tile
  }
  int du = 0, dm = 0, version = 0;
  if (b == 0) {
    for (int i = tid; i < num_tiles; i += kFusedThreads) {
      du += blk_unc[i];
      dm += blk_msk[i];
    }
    if (tid == 0) version = *tbl_version + *mem_version;
  }
  if (tid < 2) s_drop[tid] = 0;
  for (int p = tid; p < P; p += kFusedThreads) {
    int total = 0, before = 0, src_part = 0;
    for (int tb = 0; tb < num_tiles; tb += kTileBatch) {
      int v[kTileBatch];
#pragma unroll
      for (int u = 0; u < kTileBatch; ++u)
        v[u] = tb + u < num_tiles ? cnt_tile[(int64_t)(tb + u) * P + p] : 0;
#pragma unroll
      for (int u = 0; u < kTileBatch; ++u) {
        int tile = tb + u;
        total += v[u];
        before += tile < b ? v[u] : 0;
        src_part += (tile >= first && tile < first + tiles_per_rank) ? v[u] : 0;
      }
    }
    s_count[p] = total;
    s_pre[p] = before;
    if (sub_tile == 0) cnt_src[(int64_t)src_rank * P + p] = src_part;
  }
  __syncthreads();
  if (du) atomicAdd(&s_drop[0], du);  // zeroed before the barrier, read after the scan's barriers
  if (dm) atomicAdd(&s_drop[1], dm);
  block_exclusive_scan<kFusedThreads>(s_count, s_offset, s_wave, P);

  const int N = s_offset[P];
#pragma unroll
  for (int u = 0; u < kFusedPairs; ++u) {
    int i = tid + u * kFusedThreads;
    if (i < npairs) {
      int p = my_slot[u];
      int row = -1;
      if (p >= 0) {
        row = s_offset[p] + s_pre[p] + my_rank[u];
        src_of[row] = g0 + i;
      }
      row_of[g0 + i] = row;
      if (g0 + i >= N) src_of[g0 + i] = -1;  // rows past the last routed pair
    }
  }
  if (b == 0)
    write_step_tables<kFusedThreads>(s_count, s_offset, s_drop[0], s_drop[1], version, count,
                                     offset, rank_count, rank_offset, status, step_epoch, R, S, P);
}

// ---------------------------------------------------------------------------
// Small batches (T <= 192 tokens and T*k <= 1536 pairs: a few tokens per rank,
// the low-concurrency decode regime): ONE workgroup does the whole layout in one
// launch -- map, count, scan and position -- with a token bitmap per slot that
// spans the whole batch.  No tiles, no second kernel.  Measured at 32 ranks,
// top-8: the step drops from 17.3 / 18.8 / 22.7 us to 14.5 / 16.0 / 20.1 us at
// T = 32 / 64 / 128, and by 0.7 us at T = 160 and 192; from 2 pairs per thread
// on, the tiled two-launch path is as fast or faster, hence the limits.
// ---------------------------------------------------------------------------
constexpr int kSmallTokens = 192;
constexpr int kSmallPairs = 1536;

inline size_t small_lds_bytes(int E, int P, int R, int T, int k) {
  const int stride = ((T + 31) / 32) | 1;  // odd LDS row stride of the bitmaps
  return sizeof(int32_t) * ((size_t)(E + 1) + P + R + E + P + P + (P + 1) + (size_t)P * stride +
                            (size_t)2 * T * k);
}

// bits [lo, hi) of a bitmap, lo < hi
__device__ inline int popc_range(const uint32_t* bm, int lo, int hi) {
  int c = 0;
  for (int w = lo >> 5; w <= (hi - 1) >> 5; ++w) {
    uint32_t m = bm[w];
    const int base = w << 5;
    if (lo > base) m &= ~0u << (lo - base);
    if (hi < base + 32) m &= (1u << (hi - base)) - 1u;
    c += __popc(m);
  }
  return c;
}

template <int KC>
__global__ __launch_bounds__(kMapThreads) void k_layout_small(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ l2p_off,
    const int32_t* __restrict__ l2p_list, const int32_t* __restrict__ active,
    const int32_t* __restrict__ tbl_version, const int32_t* __restrict__ mem_version,
    int32_t* __restrict__ slot_of, int32_t* __restrict__ row_of, int32_t* __restrict__ src_of,
    int32_t* __restrict__ count, int32_t* __restrict__ offset, int32_t* __restrict__ rank_count,
    int32_t* __restrict__ rank_offset, int32_t* __restrict__ cnt_src,
    int32_t* __restrict__ status, int32_t* __restrict__ step_epoch, int k_rt, int E, int R, int S,
    int P, int T, int tokens_per_rank, int policy) {
  const int k = KC > 0 ? KC : k_rt;
  const int words = (T + 31) >> 5;
  const int stride = words | 1;  // odd: lanes on different slots reading the same word index hit different banks
  const int npairs = T * k;
  extern __shared__ int32_t smem[];
  int32_t* s_off = smem;                              // [E+1] replica-list starts (CSR)
  int32_t* s_list = s_off + (E + 1);                  // [P] replica lists, canonical order
  int32_t* s_active = s_list + P;                     // [R]
  int32_t* s_nlive = s_active + R;                    // [E] live replicas of expert e
  int32_t* s_live = s_nlive + E;                      // [P] live replicas, compacted per expert
  int32_t* s_count = s_live + P;                      // [P] pairs per slot
  int32_t* s_offset = s_count + P;                    // [P+1] exclusive scan of s_count
  uint32_t* s_bm = (uint32_t*)(s_offset + P + 1);     // [P][stride] token bitmap per slot
  int32_t* s_idx = (int32_t*)(s_bm + P * stride);     // [T*k] router indices
  int32_t* s_slot = s_idx + npairs;                   // [T*k] chosen slots
  __shared__ int32_t s_drop[2];
  __shared__ int32_t s_wave[kMapThreads / 64];
  const int tid = threadIdx.x;

  // every global read of this kernel is issued here, none depends on another
  for (int i = tid; i < npairs; i += kMapThreads) s_idx[i] = topk_idx[i];
  for (int i = tid; i <= E; i += kMapThreads) s_off[i] = l2p_off[i];
  for (int i = tid; i < P; i += kMapThreads) s_list[i] = l2p_list[i];
  for (int i = tid; i < R; i += kMapThreads) s_active[i] = active[i];
  const int version = tid == 0 ? *tbl_version + *mem_version : 0;
  for (int i = tid; i < P * stride; i += kMapThreads) s_bm[i] = 0u;
  if (tid < 2) s_drop[tid] = 0;
  __syncthreads();

  for (int e = tid; e < E; e += kMapThreads) {
    int o = s_off[e], o1 = s_off[e + 1], n = 0;
    for (int q = o; q < o1; ++q) {
      int p = s_list[q];
      if (s_active[p / S] != 0) s_live[o + n++] = p;  // failed peers are skipped
    }
    s_nlive[e] = n;
  }
  __syncthreads();

  int n_unc = 0, n_msk = 0;
  for (int i = tid; i < npairs; i += kMapThreads) {
    int t = i / k;
    int j = i - t * k;
    int e = s_idx[i];
    int p = -1;
    if (e < 0 || e >= E) {
      ++n_msk;
    } else {
      bool repeated = false;
      for (int jj = 0; jj < j; ++jj) repeated |= (s_idx[t * k + jj] == e);
      if (repeated) {
        ++n_msk;
      } else {
        int n = s_nlive[e];
        if (n == 0) {
          ++n_unc;
        } else {
          int sel = (policy == EEP_FIRST_LIVE || n == 1) ? 0 : t % n;
          p = s_live[s_off[e] + sel];
          atomicOr(&s_bm[p * stride + (t >> 5)], 1u << (t & 31));
        }
      }
    }
    s_slot[i] = p;
    slot_of[i] = p;
  }
  if (n_unc) atomicAdd(&s_drop[0], n_unc);
  if (n_msk) atomicAdd(&s_drop[1], n_msk);
  __syncthreads();

  for (int p = tid; p < P; p += kMapThreads) {
    int c = 0;
    for (int w = 0; w < words; ++w) c += __popc(s_bm[p * stride + w]);
    s_count[p] = c;
  }
  // pairs per (source rank, slot): the tokens of a source rank are a bit range;
  // wavefronts take source ranks, lanes take slots
  for (int b = tid >> 6; b < R; b += kMapThreads / 64)
    for (int p = tid & 63; p < P; p += 64)
      cnt_src[b * P + p] =
          popc_range(&s_bm[p * stride], b * tokens_per_rank, (b + 1) * tokens_per_rank);
  __syncthreads();
  block_exclusive_scan<kMapThreads>(s_count, s_offset, s_wave, P);

  const int N = s_offset[P];
  for (int i = tid; i < npairs; i += kMapThreads) {
    int p = s_slot[i];
    int row = -1;
    if (p >= 0) {
      int t = i / k;
      const uint32_t* bm = &s_bm[p * stride];
      int rank = __popc(bm[t >> 5] & ((1u << (t & 31)) - 1u));  // earlier tokens in this slot
      for (int w = 0; w < (t >> 5); ++w) rank += __popc(bm[w]);
      row = s_offset[p] + rank;
      src_of[row] = i;
    }
    row_of[i] = row;
    if (i >= N) src_of[i] = -1;  // rows past the last routed pair
  }
  write_step_tables<kMapThreads>(s_count, s_offset, s_drop[0], s_drop[1], version, count, offset,
                                 rank_count, rank_offset, status, step_epoch, R, S, P);
}

// ---------------------------------------------------------------------------
// Many tiles (> 64, the prefill regime): three launches.
//   k_tile_prefix  one workgroup per 64 slots (lane = slot, coalesced rows of the
//                  [tiles][P] count matrix); its 16 wavefronts split the tiles,
//                  each sums its share (one round of loads when the share is
//                  <= 32 tiles), the shares are combined through LDS, and every
//                  wavefront writes pre_tile[tile][slot] = pairs of the slot in
//                  earlier tiles, plus the slot totals.
//   k_position     a wide grid; every workgroup scans the P slot totals in LDS
//                  (cheap, and it saves a launch), then row = slot offset +
//                  earlier-tile pairs + rank in tile.  Workgroup 0 publishes the
//                  per-step tables.
// ---------------------------------------------------------------------------
constexpr int kPrefixThreads = 1024;
constexpr int kPrefixWaves = kPrefixThreads / 64;

__global__ __launch_bounds__(kPrefixThreads) void k_tile_prefix(
    const int32_t* __restrict__ cnt_tile, int32_t* __restrict__ pre_tile,
    int32_t* __restrict__ count, int num_tiles, int tiles_per_wave, int P) {
  __shared__ int32_t s_part[kPrefixWaves][64];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int p = blockIdx.x * 64 + lane;
  const int b_lo = wave * tiles_per_wave;
  int b_hi = b_lo + tiles_per_wave;
  if (b_hi > num_tiles) b_hi = num_tiles;
  const bool single = tiles_per_wave <= kTileBatch;  // the share fits one batch: keep it in registers
  int v[kTileBatch];
  int part = 0;
  if (p < P) {
    for (int tb = b_lo; tb < b_hi; tb += kTileBatch) {
#pragma unroll
      for (int u = 0; u < kTileBatch; ++u)
        v[u] = tb + u < b_hi ? cnt_tile[(int64_t)(tb + u) * P + p] : 0;
#pragma unroll
      for (int u = 0; u < kTileBatch; ++u) part += v[u];
    }
  }
  s_part[wave][lane] = part;
  __syncthreads();
  if (p >= P) return;
  int run = 0;
  for (int w = 0; w < wave; ++w) run += s_part[w][lane];
  if (wave == 0) {
    int total = 0;
    for (int w = 0; w < kPrefixWaves; ++w) total += s_part[w][lane];
    count[p] = total;
  }
  for (int tb = b_lo; tb < b_hi; tb += kTileBatch) {
    if (!single) {
#pragma unroll
      for (int u = 0; u < kTileBatch; ++u)
        v[u] = tb + u < b_hi ? cnt_tile[(int64_t)(tb + u) * P + p] : 0;
    }
#pragma unroll
    for (int u = 0; u < kTileBatch; ++u) {
      if (tb + u < b_hi) pre_tile[(int64_t)(tb + u) * P + p] = run;
      run += v[u];
    }
  }
}

template <int KC>
__global__ __launch_bounds__(kPosThreads) void k_position(
    const int32_t* __restrict__ slot_of, const int32_t* __restrict__ pre_tile,
    const int32_t* __restrict__ count_in, const int32_t* __restrict__ blk_unc,
    const int32_t* __restrict__ blk_msk, const int32_t* __restrict__ tbl_version,
    const int32_t* __restrict__ mem_version, int32_t* __restrict__ row_of,
    int32_t* __restrict__ src_of, int32_t* __restrict__ cnt_src,
    int32_t* __restrict__ offset, int32_t* __restrict__ rank_count,
    int32_t* __restrict__ rank_offset, int32_t* __restrict__ status,
    int32_t* __restrict__ step_epoch, int k_rt, int tokens_per_rank, int tiles_per_rank,
    int tile_tokens, int num_tiles, int total_pairs, int R, int S, int P) {
  const int k = KC > 0 ? KC : k_rt;
  extern __shared__ int32_t smem[];
  int32_t* s_count = smem;           // [P]
  int32_t* s_offset = s_count + P;   // [P+1]
  __shared__ int32_t s_wave[kPosThreads / 64];
  __shared__ int32_t s_drop[2];
  const int tid = threadIdx.x;
  const int g = blockIdx.x * kPosThreads + tid;

  // this thread's pair, fetched together with the slot totals
  int p = -1, rank_in_tile = 0;
  if (g < total_pairs) {
    p = slot_of[g];
    rank_in_tile = row_of[g];
  }
  for (int q = tid; q < P; q += kPosThreads) s_count[q] = count_in[q];
  int du = 0, dm = 0, version = 0;
  if (blockIdx.x == 0) {
    for (int b = tid; b < num_tiles; b += kPosThreads) {
      du += blk_unc[b];
      dm += blk_msk[b];
    }
    if (tid == 0) version = *tbl_version + *mem_version;
  }
  if (tid < 2) s_drop[tid] = 0;
  __syncthreads();
  if (du) atomicAdd(&s_drop[0], du);
  if (dm) atomicAdd(&s_drop[1], dm);
  block_exclusive_scan<kPosThreads>(s_count, s_offset, s_wave, P);

  // pairs per (source rank, slot): difference of the tile prefixes at the source
  // rank's first tile and at the next source rank's first tile
  for (int i = g; i < R * P; i += gridDim.x * kPosThreads) {
    int bs = i / P;
    int q = i - bs * P;
    int first = bs * tiles_per_rank, next = first + tiles_per_rank;
    int lo_v = pre_tile[(int64_t)first * P + q];
    int hi_v = next < num_tiles ? pre_tile[(int64_t)next * P + q] : s_count[q];
    cnt_src[i] = hi_v - lo_v;
  }
  if (g < total_pairs) {
    const int t = g / k;
    const int src_rank = t / tokens_per_rank;
    const int tile = src_rank * tiles_per_rank + (t - src_rank * tokens_per_rank) / tile_tokens;
    const int N = s_offset[P];
    int row = -1;
    if (p >= 0) {
      row = s_offset[p] + pre_tile[(int64_t)tile * P + p] + rank_in_tile;
      src_of[row] = g;
    }
    row_of[g] = row;
    if (g >= N) src_of[g] = -1;  // rows past the last routed pair
  }
  if (blockIdx.x == 0)
    write_step_tables<kPosThreads>(s_count, s_offset, s_drop[0], s_drop[1], version, nullptr,
                                   offset, rank_count, rank_offset, status, step_epoch, R, S, P);
}

// T == 0: nothing is routed; publish empty tables.
__global__ __launch_bounds__(256) void k_empty_step(
    const int32_t* __restrict__ tbl_version, const int32_t* __restrict__ mem_version,
    int32_t* __restrict__ count, int32_t* __restrict__ offset, int32_t* __restrict__ rank_count,
    int32_t* __restrict__ rank_offset, int32_t* __restrict__ cnt_src,
    int32_t* __restrict__ status, int32_t* __restrict__ step_epoch, int R, int P) {
  for (int p = threadIdx.x; p <= P; p += 256) {
    offset[p] = 0;
    if (p < P) count[p] = 0;
  }
  for (int r = threadIdx.x; r <= R; r += 256) {
    rank_offset[r] = 0;
    if (r < R) rank_count[r] = 0;
  }
  for (int i = threadIdx.x; i < R * P; i += 256) cnt_src[i] = 0;
  if (threadIdx.x == 0) {
    status[0] = status[1] = status[2] = 0;
    status[3] = *tbl_version + *mem_version;
    *step_epoch = *step_epoch + 1;
  }
}

// ---------------------------------------------------------------------------
// De-duplicated dispatch (a data-path variant): one row per (token, destination
// rank).  Two launches after the ordinary layout, built like it: per tile a
// token bitmap per RANK gives the tile's count and the stable rank of a token
// inside the tile; then every workgroup derives the rank offsets and the pairs
// of earlier tiles from the small [tiles][R] count matrix.
//   dd_row[t,j]  row of token t in rank r's part of the rank-major buffer
//   dd_dst[t,j]  the same for the pair that carries the row (lowest j on that
//                rank), -1 for the others: the row table the pack kernel reads
//   dd_expand[row] for every expert-major row, the rank-major row behind it
// ---------------------------------------------------------------------------
template <int KC>
__global__ __launch_bounds__(kMapThreads) void k_dedup_count(
    const int32_t* __restrict__ slot_of, int32_t* __restrict__ dd_row,
    int32_t* __restrict__ dd_dst, int32_t* __restrict__ dd_tile, int k_rt, int R, int S,
    int tokens_per_rank, int tiles_per_rank, int tile_tokens) {
  const int k = KC > 0 ? KC : k_rt;
  extern __shared__ int32_t smem[];
  uint32_t* s_bm = (uint32_t*)smem;                       // [R][kBitmapWords]
  int32_t* s_slot = smem + R * kBitmapWords;              // [tile_tokens*k]
  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  const TileRange tr = tile_range(b, tokens_per_rank, tiles_per_rank, tile_tokens);
  const int npairs = tr.ntok * k;
  const int64_t g0 = (int64_t)tr.t0 * k;
  for (int i = tid; i < npairs; i += kMapThreads) s_slot[i] = slot_of[g0 + i];
  for (int i = tid; i < R * kBitmapWords; i += kMapThreads) s_bm[i] = 0u;
  __syncthreads();
  for (int i = tid; i < npairs; i += kMapThreads) {
    const int p = s_slot[i];
    if (p >= 0) {
      const int tl = i / k;
      atomicOr(&s_bm[(p / S) * kBitmapWords + (tl >> 5)], 1u << (tl & 31));
    }
  }
  __syncthreads();
  for (int i = tid; i < npairs; i += kMapThreads) {
    const int p = s_slot[i];
    int rank = -1, lead = 0;
    if (p >= 0) {
      const int r = p / S;
      const int tl = i / k;
      const int j = i - tl * k;
      lead = 1;
      for (int jj = 0; jj < j; ++jj) {
        const int q = s_slot[tl * k + jj];
        if (q >= 0 && q / S == r) lead = 0;
      }
      const uint32_t* bm = &s_bm[r * kBitmapWords];
      const int w = tl >> 5;
      rank = __popc(bm[w] & ((1u << (tl & 31)) - 1u));
      for (int ww = 0; ww < w; ++ww) rank += __popc(bm[ww]);
    }
    dd_row[g0 + i] = rank;  // rank inside the tile; the position kernel turns it into the row
    dd_dst[g0 + i] = lead;
  }
  for (int r = tid; r < R; r += kMapThreads) {
    int c = 0;
#pragma unroll
    for (int w = 0; w < kBitmapWords; ++w) c += __popc(s_bm[r * kBitmapWords + w]);
    dd_tile[(int64_t)b * R + r] = c;
  }
}

template <int KC>
__global__ __launch_bounds__(kMapThreads) void k_dedup_position(
    const int32_t* __restrict__ slot_of, const int32_t* __restrict__ row_of,
    const int32_t* __restrict__ status, const int32_t* __restrict__ dd_tile,
    int32_t* __restrict__ dd_row, int32_t* __restrict__ dd_dst, int32_t* __restrict__ dd_expand,
    int32_t* __restrict__ dd_count, int32_t* __restrict__ dd_offset,
    int32_t* __restrict__ dd_status, int k_rt, int R, int S, int num_tiles, int tokens_per_rank,
    int tiles_per_rank, int tile_tokens) {
  const int k = KC > 0 ? KC : k_rt;
  extern __shared__ int32_t smem[];
  int32_t* s_cnt = smem;           // [R]   tokens per rank, all tiles
  int32_t* s_off = s_cnt + R;      // [R+1] exclusive scan of s_cnt
  int32_t* s_pre = s_off + R + 1;  // [R]   tokens per rank in tiles before this one
  __shared__ int32_t s_wave[kMapThreads / 64];
  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  const TileRange tr = tile_range(b, tokens_per_rank, tiles_per_rank, tile_tokens);
  const int npairs = tr.ntok * k;
  const int64_t g0 = (int64_t)tr.t0 * k;
  const int N = status[0];
  for (int r = tid; r < R; r += kMapThreads) {
    int total = 0, before = 0;
    for (int tb = 0; tb < num_tiles; tb += kTileBatch) {
      int v[kTileBatch];
#pragma unroll
      for (int u = 0; u < kTileBatch; ++u)
        v[u] = tb + u < num_tiles ? dd_tile[(int64_t)(tb + u) * R + r] : 0;
#pragma unroll
      for (int u = 0; u < kTileBatch; ++u) {
        total += v[u];
        before += tb + u < b ? v[u] : 0;
      }
    }
    s_cnt[r] = total;
    s_pre[r] = before;
  }
  __syncthreads();
  block_exclusive_scan<kMapThreads>(s_cnt, s_off, s_wave, R);
  for (int i = tid; i < npairs; i += kMapThreads) {
    const int p = slot_of[g0 + i];
    int row_d = -1, dst = -1;
    if (p >= 0) {
      const int r = p / S;
      row_d = s_off[r] + s_pre[r] + dd_row[g0 + i];
      if (dd_dst[g0 + i] != 0) dst = row_d;
      const int row = row_of[g0 + i];
      if (row >= 0) dd_expand[row] = row_d;  // (a row withdrawn by failure detection stays -1)
    }
    dd_row[g0 + i] = row_d;
    dd_dst[g0 + i] = dst;
    if (g0 + i >= N) dd_expand[g0 + i] = -1;  // rows past the last routed pair
  }
  if (b == 0) {
    for (int r = tid; r <= R; r += kMapThreads) {
      dd_offset[r] = s_off[r];
      if (r < R) dd_count[r] = s_cnt[r];
    }
    if (tid == 0) dd_status[0] = s_off[R];
  }
}

hipError_t launch_dedup_layout(eep_ctx* c, int T, hipStream_t st) {
  Tiling g = make_tiling(T, c->R);
  if (g.num_tiles == 0) {
    hipError_t e = launch_fill(c->dd_count, 0, c->R, st);
    if (e == hipSuccess) e = launch_fill(c->dd_offset, 0, c->R + 1, st);
    if (e == hipSuccess) e = launch_fill(c->dd_status, 0, 1, st);
    return e;
  }
  const bool k8 = c->k == 8;
  {
    size_t lds = sizeof(int32_t) * ((size_t)c->R * kBitmapWords + (size_t)g.tile_tokens * c->k);
    auto kern = k8 ? k_dedup_count<8> : k_dedup_count<0>;
    hipLaunchKernelGGL(kern, dim3(g.num_tiles), dim3(kMapThreads), lds, st, c->slot_of, c->dd_row,
                       c->dd_dst, c->dd_tile, c->k, c->R, c->S, g.tokens_per_rank,
                       g.tiles_per_rank, g.tile_tokens);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  size_t lds = sizeof(int32_t) * ((size_t)3 * c->R + 1);
  auto kern = k8 ? k_dedup_position<8> : k_dedup_position<0>;
  hipLaunchKernelGGL(kern, dim3(g.num_tiles), dim3(kMapThreads), lds, st, c->slot_of, c->row_of,
                     c->status, c->dd_tile, c->dd_row, c->dd_dst, c->dd_expand, c->dd_count,
                     c->dd_offset, c->dd_status, c->k, c->R, c->S, g.num_tiles, g.tokens_per_rank,
                     g.tiles_per_rank, g.tile_tokens);
  return hipGetLastError();
}

bool layout_shape_fits(int E, int P, int R, int k) {
  return map_lds_bytes(E, P, R, kTileTokens, k) <= kLayoutLdsLimit &&
         sizeof(int32_t) * ((size_t)3 * P + 1) <= kLayoutLdsLimit;
}

hipError_t launch_layout(const LayoutIO& c, int T, hipStream_t st) {
  Tiling g = make_tiling(T, c.R);
  const bool k8 = c.k == 8;
  if (g.num_tiles == 0) {
    hipLaunchKernelGGL(k_empty_step, dim3(1), dim3(256), 0, st, c.tbl_version, c.mem_version,
                       c.count, c.offset, c.rank_count, c.rank_offset, c.cnt_src, c.status,
                       c.step_epoch, c.R, c.P);
    return hipGetLastError();
  }
  if (T <= kSmallTokens && T * c.k <= kSmallPairs &&
      small_lds_bytes(c.E, c.P, c.R, T, c.k) <= kLayoutLdsLimit) {
    auto kern = k8 ? k_layout_small<8> : k_layout_small<0>;
    hipLaunchKernelGGL(kern, dim3(1), dim3(kMapThreads), small_lds_bytes(c.E, c.P, c.R, T, c.k),
                       st, c.topk_idx, c.l2p_off, c.l2p_list, c.active, c.tbl_version,
                       c.mem_version, c.slot_of, c.row_of, c.src_of, c.count, c.offset,
                       c.rank_count, c.rank_offset, c.cnt_src, c.status, c.step_epoch, c.k, c.E,
                       c.R, c.S, c.P, T, g.tokens_per_rank, c.policy);
    return hipGetLastError();
  }
  {
    size_t lds = map_lds_bytes(c.E, c.P, c.R, g.tile_tokens, c.k);
    auto kern = k8 ? k_map_count<8> : k_map_count<0>;
    hipLaunchKernelGGL(kern, dim3(g.num_tiles), dim3(kMapThreads), lds, st, c.topk_idx, c.l2p_off,
                       c.l2p_list, c.active, c.slot_of, c.row_of, c.cnt_tile, c.blk_unc, c.blk_msk,
                       c.k, c.E, c.R, c.S, c.P, g.tokens_per_rank, g.tiles_per_rank, g.tile_tokens,
                       c.policy);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const bool fused = g.num_tiles <= 64 && g.tile_tokens * c.k <= kFusedThreads * kFusedPairs;
  if (fused) {
    size_t lds = sizeof(int32_t) * ((size_t)3 * c.P + 1);
    auto kern = k8 ? k_scan_position<8> : k_scan_position<0>;
    hipLaunchKernelGGL(kern, dim3(g.num_tiles), dim3(kFusedThreads), lds, st, c.cnt_tile,
                       c.blk_unc, c.blk_msk, c.tbl_version, c.mem_version, c.slot_of, c.row_of,
                       c.src_of, c.count, c.offset, c.rank_count, c.rank_offset, c.cnt_src,
                       c.status, c.step_epoch, c.k, g.num_tiles, g.tokens_per_rank,
                       g.tiles_per_rank, g.tile_tokens, c.R, c.S, c.P);
    return hipGetLastError();
  }
  int tiles_per_wave = (g.num_tiles + kPrefixWaves - 1) / kPrefixWaves;
  hipLaunchKernelGGL(k_tile_prefix, dim3((c.P + 63) / 64), dim3(kPrefixThreads), 0, st, c.cnt_tile,
                     c.base_tile, c.count, g.num_tiles, tiles_per_wave, c.P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  int total_pairs = T * c.k;
  size_t lds_pos = sizeof(int32_t) * ((size_t)2 * c.P + 1);
  auto kern = k8 ? k_position<8> : k_position<0>;
  hipLaunchKernelGGL(kern, dim3((total_pairs + kPosThreads - 1) / kPosThreads), dim3(kPosThreads),
                     lds_pos, st, c.slot_of, c.base_tile, c.count, c.blk_unc, c.blk_msk,
                     c.tbl_version, c.mem_version, c.row_of, c.src_of, c.cnt_src, c.offset,
                     c.rank_count, c.rank_offset, c.status, c.step_epoch, c.k, g.tokens_per_rank,
                     g.tiles_per_rank, g.tile_tokens, g.num_tiles, total_pairs, c.R, c.S, c.P);
  return hipGetLastError();
}

hipError_t launch_layout(eep_ctx* c, const int32_t* topk_idx, int T, hipStream_t st) {
  LayoutIO io;
  io.R = c->R; io.S = c->S; io.P = c->P; io.E = c->E; io.k = c->k; io.policy = c->cfg.policy;
  io.topk_idx = topk_idx;
  io.l2p_off = c->l2p_off; io.l2p_list = c->l2p_list; io.active = c->active;
  io.tbl_version = c->tbl_version; io.mem_version = c->mem->mem_version;
  io.slot_of = c->slot_of; io.row_of = c->row_of; io.src_of = c->src_of;
  io.count = c->count; io.offset = c->offset; io.rank_count = c->rank_count;
  io.rank_offset = c->rank_offset; io.cnt_src = c->cnt_src; io.status = c->status;
  io.cnt_tile = c->cnt_tile; io.base_tile = c->base_tile; io.blk_unc = c->blk_unc;
  io.blk_msk = c->blk_msk; io.step_epoch = c->step_epoch;
  return launch_layout(io, T, st);
}

}  // namespace eep
