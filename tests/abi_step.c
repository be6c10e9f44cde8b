/* A consumer of the C ABI with no Python and no torch in the process: one small
 * step (layout, dispatch, scalar expert stand-in, combine) with a failed rank,
 * driven from plain C through include/eep.h with buffers from hipMalloc, and
 * compared with the C oracle function by function (integers and bytes exactly,
 * the combine output against the oracle's fp32 chain).  Built by
 * tests/abi_step_build.py; run on a GPU by tests/test_gpu_c_abi.py. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "eep.h"

/* oracle/eep_oracle.c */
int eeo_tables(int P, int E, int S, int S_prim, const int32_t* p2l, int32_t* l2p_off, int32_t* l2p_list);
void eeo_map(int T, int k, int E, int S, int policy, const int32_t* topk_idx, const int32_t* l2p_off,
             const int32_t* l2p_list, const int32_t* active, int32_t* slot_of, int64_t* counters);
void eeo_layout(int T, int k, int R, int S, const int32_t* slot_of, int32_t* count, int32_t* rank_count,
                int32_t* cnt_src, int32_t* offset, int32_t* rank_offset, int32_t* row_of, int32_t* src_of,
                int32_t* cursor);
void eeo_pack(int T, int k, int64_t row_bytes, const uint8_t* x, const int32_t* row_of, uint8_t* recv);
void eeo_stub_scale(int N, int H, int P, int dtype, const void* recv, const int32_t* offset,
                    const int32_t* p2l, const float* expert_scale, void* y);
void eeo_combine_chain32(int T, int k, int H, int y_dtype, const void* y, const float* w,
                         const int32_t* row_of, float* out);

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      printf("abi_step FAILED at line %d: %s\n", __LINE__, #cond);         \
      return 1;                                                            \
    }                                                                      \
  } while (0)

static uint32_t lcg_state = 260510670u;
static uint32_t lcg(void) {
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return lcg_state >> 8;
}

enum { R = 4, S = 6, S_PRIM = 4, P = R * S, E = 16, K = 2, T = 128, H = 1024 };

int main(void) {
  /* placement: primaries in place, rank 2 failed, its experts 8..11 on redundant slots elsewhere */
  int32_t p2l[P], active[R] = {1, 1, 0, 1};
  for (int p = 0; p < P; ++p) p2l[p] = -1;
  for (int r = 0; r < R; ++r)
    for (int s = 0; s < S_PRIM; ++s) p2l[r * S + s] = r * S_PRIM + s;
  p2l[0 * S + 4] = 8; p2l[0 * S + 5] = 9; p2l[1 * S + 4] = 10; p2l[3 * S + 4] = 11;
  p2l[3 * S + 5] = 0;                                   /* and one ordinary replica */

  static int32_t idx[T * K];
  static float w[T * K], x[T * H], scale[E];
  for (int t = 0; t < T; ++t) {
    idx[t * K] = (int32_t)(lcg() % E);
    do idx[t * K + 1] = (int32_t)(lcg() % E); while (idx[t * K + 1] == idx[t * K]);
    w[t * K] = (float)(lcg() % 1000) / 1000.0f;
    w[t * K + 1] = 1.0f - w[t * K];
  }
  for (int i = 0; i < T * H; ++i) x[i] = (float)((int)(lcg() % 2001) - 1000) / 256.0f;
  for (int e = 0; e < E; ++e) scale[e] = 1.0f + (float)e / 16.0f;

  /* ---- the library ---- */
  eep_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.num_ranks = R; cfg.slots_per_rank = S; cfg.primary_slots = S_PRIM; cfg.num_logical = E;
  cfg.max_tokens = T; cfg.topk = K; cfg.hidden = H;
  cfg.x_dtype = EEP_F32; cfg.y_dtype = EEP_F32; cfg.out_dtype = EEP_F32;
  cfg.policy = EEP_SPREAD; cfg.strict_coverage = 1;
  eep_ctx* ctx = NULL;
  CHECK(eep_create(&cfg, &ctx) == EEP_OK);
  CHECK(eep_update_placement(ctx, p2l, NULL) == EEP_OK);
  CHECK(eep_set_membership(ctx, active, NULL) == EEP_OK);
  int32_t alone[R] = {1, 0, 0, 1};                      /* would orphan expert 10: refused */
  CHECK(eep_set_membership(ctx, alone, NULL) == EEP_ERR_COVERAGE);

  void *d_idx, *d_w, *d_x, *d_scale, *d_recv, *d_y, *d_out;
  CHECK(hipMalloc(&d_idx, sizeof idx) == hipSuccess && hipMalloc(&d_w, sizeof w) == hipSuccess);
  CHECK(hipMalloc(&d_x, sizeof x) == hipSuccess && hipMalloc(&d_scale, sizeof scale) == hipSuccess);
  CHECK(hipMalloc(&d_recv, (size_t)T * K * H * 4) == hipSuccess);
  CHECK(hipMalloc(&d_y, (size_t)T * K * H * 4) == hipSuccess && hipMalloc(&d_out, sizeof x) == hipSuccess);
  CHECK(hipMemcpy(d_idx, idx, sizeof idx, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(hipMemcpy(d_w, w, sizeof w, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(hipMemcpy(d_x, x, sizeof x, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(hipMemcpy(d_scale, scale, sizeof scale, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(hipMemset(d_recv, 0, (size_t)T * K * H * 4) == hipSuccess);
  hipStream_t st;
  CHECK(hipStreamCreate(&st) == hipSuccess);
  CHECK(eep_combine(ctx, d_y, (const float*)d_w, d_out, T, st) == EEP_ERR_STATE);  /* no layout yet */
  CHECK(eep_dispatch_layout(ctx, (const int32_t*)d_idx, T, st) == EEP_OK);
  CHECK(eep_dispatch(ctx, d_x, NULL, d_recv, NULL, T, st) == EEP_OK);
  CHECK(eep_expert_stub(ctx, EEP_STUB_SCALE, d_recv, NULL, (const float*)d_scale, d_y, T, st) == EEP_OK);
  CHECK(eep_combine(ctx, d_y, (const float*)d_w, d_out, T, st) == EEP_OK);
  CHECK(hipStreamSynchronize(st) == hipSuccess);

  static int32_t g_slot[T * K], g_row[T * K], g_src[T * K], g_count[P], g_offset[P + 1], g_rcount[R],
      g_status[4], bad[4];
  CHECK(eep_read_view(ctx, EEP_V_SLOT_OF, g_slot, T * K, st) == EEP_OK);
  CHECK(eep_read_view(ctx, EEP_V_ROW_OF, g_row, T * K, st) == EEP_OK);
  CHECK(eep_read_view(ctx, EEP_V_SRC_OF, g_src, T * K, st) == EEP_OK);
  CHECK(eep_read_view(ctx, EEP_V_COUNT, g_count, P, st) == EEP_OK);
  CHECK(eep_read_view(ctx, EEP_V_OFFSET, g_offset, P + 1, st) == EEP_OK);
  CHECK(eep_read_view(ctx, EEP_V_RANK_COUNT, g_rcount, R, st) == EEP_OK);
  CHECK(eep_read_view(ctx, EEP_V_STATUS, g_status, 4, st) == EEP_OK);
  CHECK(eep_debug_check_layout(ctx, T, bad, st) == EEP_OK);
  CHECK(bad[0] == 0 && bad[1] == 0 && bad[2] == 0 && bad[3] == 0);
  static float g_recv[T * K * H], g_out[T * H];
  CHECK(hipMemcpy(g_recv, d_recv, sizeof g_recv, hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(hipMemcpy(g_out, d_out, sizeof g_out, hipMemcpyDeviceToHost) == hipSuccess);

  /* ---- the oracle ---- */
  static int32_t off[E + 1], lst[P], o_slot[T * K], o_row[T * K], o_src[T * K], o_count[P], o_rcount[R],
      o_cnt_src[R * P], o_offset[P + 1], o_roff[R + 1], cursor[P];
  int64_t dropped[2];
  CHECK(eeo_tables(P, E, S, S_PRIM, p2l, off, lst) == 0);
  eeo_map(T, K, E, S, 0, idx, off, lst, active, o_slot, dropped);
  eeo_layout(T, K, R, S, o_slot, o_count, o_rcount, o_cnt_src, o_offset, o_roff, o_row, o_src, cursor);
  const int N = o_offset[P];
  static float o_recv[T * K * H], o_y[T * K * H], o_out[T * H];
  memset(o_recv, 0, sizeof o_recv);
  eeo_pack(T, K, (int64_t)H * 4, (const uint8_t*)x, o_row, (uint8_t*)o_recv);
  eeo_stub_scale(N, H, P, 0, o_recv, o_offset, p2l, scale, o_y);
  eeo_combine_chain32(T, K, H, 0, o_y, w, o_row, o_out);

  CHECK(dropped[0] == 0 && dropped[1] == 0 && N == T * K);
  CHECK(g_status[0] == N && g_status[1] == 0 && g_status[2] == 0);
  CHECK(memcmp(g_slot, o_slot, sizeof g_slot) == 0 && memcmp(g_row, o_row, sizeof g_row) == 0);
  CHECK(memcmp(g_src, o_src, sizeof g_src) == 0 && memcmp(g_count, o_count, sizeof g_count) == 0);
  CHECK(memcmp(g_offset, o_offset, sizeof g_offset) == 0 && memcmp(g_rcount, o_rcount, sizeof g_rcount) == 0);
  CHECK(g_rcount[2] == 0);                                        /* the failed rank receives nothing */
  CHECK(memcmp(g_recv, o_recv, sizeof g_recv) == 0);              /* packed rows, byte for byte */
  CHECK(memcmp(g_out, o_out, sizeof g_out) == 0);                 /* fp32 chain, bit for bit */

  CHECK(eep_destroy(ctx) == EEP_OK);
  CHECK(hipFree(d_idx) == hipSuccess && hipFree(d_w) == hipSuccess && hipFree(d_x) == hipSuccess);
  CHECK(hipFree(d_scale) == hipSuccess && hipFree(d_recv) == hipSuccess && hipFree(d_y) == hipSuccess);
  CHECK(hipFree(d_out) == hipSuccess && hipStreamDestroy(st) == hipSuccess);
  printf("abi_step ok: N = %d rows, rank 2 got %d\n", N, g_rcount[2]);
  return 0;
}
