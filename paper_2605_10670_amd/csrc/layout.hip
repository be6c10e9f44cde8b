// dispatch_layout: route every (token, j) pair to a live replica slot, count
// pairs per slot, prefix-sum the counts into receive-buffer offsets and give
// every routed pair its row, rows of one slot ordered by ascending token.
//
// Paper: Fig. 7 (the dispatch path skips peers whose `active` is 0), Sec. 5.1
// (slot -> logical expert map and all locations of each logical expert),
// Sec. 3.2 (validity contract), Sec. 4.1 (contiguous per-expert receive
// buffers as in prior work).
//
// Three launches, all tiny and latency-bound (the step's metadata is < 1 MB):
//   k_map_count  one workgroup per tile of <= 128 tokens of ONE source rank:
//                builds the live-replica table in LDS from the placement CSR and
//                the active mask, maps its pairs, and records for every slot a
//                bitmap of the tile's tokens that hit it.  popcount of the
//                bitmap is the tile's count; popcount of the bits below a token
//                is that pair's stable rank inside the tile.  No atomics on
//                positions, so the order is deterministic.
//   k_scan       one workgroup: column sums over tiles, exclusive scan over
//                slots, per-tile bases, per-rank and per-source-rank tables.
//   k_position   one workgroup per tile: row = tile base + rank in tile; also
//                writes the inverse permutation.
#include "eep_internal.hpp"

namespace eep {

constexpr int kMapThreads = 256;
constexpr int kScanThreads = 512;

// A token can hit a slot at most once: its k logical experts are distinct
// (repeats are masked) and a slot holds one logical expert.  So one bit per
// (slot, token of the tile) is enough.
__global__ __launch_bounds__(kMapThreads) void k_map_count(
    const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ l2p_off,
    const int32_t* __restrict__ l2p_list, const int32_t* __restrict__ active,
    int32_t* __restrict__ slot_of, int32_t* __restrict__ rank_in_tile,
    int32_t* __restrict__ cnt_tile, int32_t* __restrict__ blk_unc, int32_t* __restrict__ blk_msk,
    int k, int E, int S, int P, int tokens_per_rank, int tiles_per_rank, int tile_tokens,
    int policy) {
  extern __shared__ int32_t smem[];
  int32_t* s_nlive = smem;                       // [E] live replicas of expert e
  int32_t* s_off = s_nlive + E;                  // [E] start of e's replica list
  int32_t* s_live = s_off + E;                   // [P] live replicas, compacted per expert
  uint32_t* s_bm = (uint32_t*)(s_live + P);      // [P][kBitmapWords]
  int32_t* s_idx = (int32_t*)(s_bm + P * kBitmapWords);  // [tile_tokens*k] router indices
  int32_t* s_slot = s_idx + tile_tokens * k;             // [tile_tokens*k] chosen slots
  __shared__ int32_t s_drop[2];

  const int tid = threadIdx.x;
  const int b = blockIdx.x;
  const int src_rank = b / tiles_per_rank;
  const int sub = b - src_rank * tiles_per_rank;
  const int t0 = src_rank * tokens_per_rank + sub * tile_tokens;
  int t1 = t0 + tile_tokens;
  const int rank_end = (src_rank + 1) * tokens_per_rank;
  if (t1 > rank_end) t1 = rank_end;
  const int ntok = t1 > t0 ? t1 - t0 : 0;
  const int npairs = ntok * k;
  const int64_t g0 = (int64_t)t0 * k;

  for (int i = tid; i < npairs; i += kMapThreads) s_idx[i] = topk_idx[g0 + i];
  for (int e = tid; e < E; e += kMapThreads) {
    int o = l2p_off[e], o1 = l2p_off[e + 1], n = 0;
    for (int q = o; q < o1; ++q) {
      int p = l2p_list[q];
      if (active[p / S] != 0) s_live[o + n++] = p;  // failed peers are skipped
    }
    s_nlive[e] = n;
    s_off[e] = o;
  }
  for (int i = tid; i < P * kBitmapWords; i += kMapThreads) s_bm[i] = 0u;
  if (tid < 2) s_drop[tid] = 0;
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
    for (int w = 0; w < kBitmapWords; ++w) c += __popc(s_bm[p * kBitmapWords + w]);
    cnt_tile[(int64_t)b * P + p] = c;
  }
  if (tid == 0) {
    blk_unc[b] = s_drop[0];
    blk_msk[b] = s_drop[1];
  }
}

__device__ inline int wave_inclusive_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

__global__ __launch_bounds__(kScanThreads) void k_scan(
    const int32_t* __restrict__ cnt_tile, const int32_t* __restrict__ blk_unc,
    const int32_t* __restrict__ blk_msk, const int32_t* __restrict__ tbl_version,
    int32_t* __restrict__ count, int32_t* __restrict__ offset, int32_t* __restrict__ rank_count,
    int32_t* __restrict__ rank_offset, int32_t* __restrict__ cnt_src,
    int32_t* __restrict__ base_tile, int32_t* __restrict__ status, int num_tiles,
    int tiles_per_rank, int R, int S, int P) {
  extern __shared__ int32_t smem[];
  int32_t* s_count = smem;           // [P]
  int32_t* s_offset = s_count + P;   // [P+1]
  __shared__ int32_t s_wave[kScanThreads / 64];
  __shared__ int32_t s_drop[2];
  const int tid = threadIdx.x;
  const int n_src = num_tiles > 0 ? R : 0;

  if (tid < 2) s_drop[tid] = 0;
  // column sums: pairs per slot, and per (source rank, slot)
  for (int p = tid; p < P; p += kScanThreads) {
    int total = 0;
    for (int bs = 0; bs < n_src; ++bs) {
      int part = 0;
      for (int sub = 0; sub < tiles_per_rank; ++sub)
        part += cnt_tile[(int64_t)(bs * tiles_per_rank + sub) * P + p];
      cnt_src[bs * P + p] = part;
      total += part;
    }
    for (int bs = n_src; bs < R; ++bs) cnt_src[bs * P + p] = 0;
    s_count[p] = total;
    count[p] = total;
  }
  __syncthreads();

  // exclusive scan over slots: each thread owns a contiguous chunk
  const int ipt = (P + kScanThreads - 1) / kScanThreads;
  const int lo = tid * ipt;
  int hi = lo + ipt;
  if (hi > P) hi = P;
  int local = 0;
  for (int p = lo; p < hi; ++p) local += s_count[p];
  int incl = wave_inclusive_scan(local);
  if ((tid & 63) == 63) s_wave[tid >> 6] = incl;
  __syncthreads();
  int wave_base = 0;
  for (int w = 0; w < (tid >> 6); ++w) wave_base += s_wave[w];
  int run = wave_base + incl - local;
  for (int p = lo; p < hi; ++p) {
    s_offset[p] = run;
    run += s_count[p];
  }
  if (tid == kScanThreads - 1) s_offset[P] = wave_base + incl;
  // dropped-pair totals
  int du = 0, dm = 0;
  for (int b = tid; b < num_tiles; b += kScanThreads) {
    du += blk_unc[b];
    dm += blk_msk[b];
  }
  if (du) atomicAdd(&s_drop[0], du);
  if (dm) atomicAdd(&s_drop[1], dm);
  __syncthreads();

  for (int p = tid; p <= P; p += kScanThreads) offset[p] = s_offset[p];
  for (int r = tid; r < R; r += kScanThreads) {
    rank_offset[r] = s_offset[r * S];
    rank_count[r] = s_offset[(r + 1) * S] - s_offset[r * S];
  }
  if (tid == 0) {
    rank_offset[R] = s_offset[P];
    status[0] = s_offset[P];
    status[1] = s_drop[0];
    status[2] = s_drop[1];
    status[3] = *tbl_version;
  }
  // first row of every (tile, slot): slot offset + pairs of earlier tiles
  for (int p = tid; p < P; p += kScanThreads) {
    int acc = s_offset[p];
    for (int b = 0; b < num_tiles; ++b) {
      base_tile[(int64_t)b * P + p] = acc;
      acc += cnt_tile[(int64_t)b * P + p];
    }
  }
}

__global__ __launch_bounds__(kMapThreads) void k_position(
    const int32_t* __restrict__ slot_of, const int32_t* __restrict__ base_tile,
    const int32_t* __restrict__ status, int32_t* __restrict__ row_of, int32_t* __restrict__ src_of,
    int k, int P, int tokens_per_rank, int tiles_per_rank, int tile_tokens) {
  const int b = blockIdx.x;
  const int src_rank = b / tiles_per_rank;
  const int sub = b - src_rank * tiles_per_rank;
  const int t0 = src_rank * tokens_per_rank + sub * tile_tokens;
  int t1 = t0 + tile_tokens;
  const int rank_end = (src_rank + 1) * tokens_per_rank;
  if (t1 > rank_end) t1 = rank_end;
  const int npairs = (t1 > t0 ? t1 - t0 : 0) * k;
  const int g0 = t0 * k;
  const int N = status[0];
  const int32_t* base = base_tile + (int64_t)b * P;
  for (int i = threadIdx.x; i < npairs; i += kMapThreads) {
    int g = g0 + i;
    int p = slot_of[g];
    int row = -1;
    if (p >= 0) {
      row = base[p] + row_of[g];  // row_of still holds the rank inside the tile
      src_of[row] = g;
    }
    row_of[g] = row;
    if (g >= N) src_of[g] = -1;  // rows past the last routed pair
  }
}

hipError_t launch_layout(eep_ctx* c, const int32_t* topk_idx, int T, hipStream_t st) {
  Tiling g = make_tiling(T, c->R);
  if (g.num_tiles > 0) {
    size_t lds = sizeof(int32_t) * ((size_t)2 * c->E + c->P + (size_t)c->P * kBitmapWords +
                                    (size_t)2 * g.tile_tokens * c->k);
    hipLaunchKernelGGL(k_map_count, dim3(g.num_tiles), dim3(kMapThreads), lds, st, topk_idx,
                       c->l2p_off, c->l2p_list, c->active, c->slot_of, c->row_of, c->cnt_tile,
                       c->blk_unc, c->blk_msk, c->k, c->E, c->S, c->P, g.tokens_per_rank,
                       g.tiles_per_rank, g.tile_tokens, c->cfg.policy);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  size_t lds_scan = sizeof(int32_t) * ((size_t)2 * c->P + 1);
  hipLaunchKernelGGL(k_scan, dim3(1), dim3(kScanThreads), lds_scan, st, c->cnt_tile, c->blk_unc,
                     c->blk_msk, c->tbl_version, c->count, c->offset, c->rank_count,
                     c->rank_offset, c->cnt_src, c->base_tile, c->status, g.num_tiles,
                     g.tiles_per_rank, c->R, c->S, c->P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (g.num_tiles > 0) {
    hipLaunchKernelGGL(k_position, dim3(g.num_tiles), dim3(kMapThreads), 0, st, c->slot_of,
                       c->base_tile, c->status, c->row_of, c->src_of, c->k, c->P,
                       g.tokens_per_rank, g.tiles_per_rank, g.tile_tokens);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace eep
