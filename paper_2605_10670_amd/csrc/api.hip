// C ABI of libeep: argument checks, context and table state, kernel launches.
// See include/eep.h for the contract of every entry point.
#include <new>

#include "eep_internal.hpp"

using namespace eep;

namespace {

int fail_hip(eep_ctx* c, hipError_t e) {
  if (c) c->last_hip_error = (int)e;
  return EEP_ERR_HIP;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

extern "C" {

const char* eep_strerror(int code) {
  switch (code) {
    case EEP_OK: return "ok";
    case EEP_ERR_INVALID_ARG: return "invalid argument";
    case EEP_ERR_ALIGN: return "row size or pointer not 16-byte aligned";
    case EEP_ERR_COVERAGE: return "a logical expert would have no live replica";
    case EEP_ERR_HIP: return "HIP runtime error";
    case EEP_ERR_STATE: return "call order violated";
    case EEP_ERR_SCRATCH: return "batch needs more scratch than the static array holds";
    default: return "unknown error";
  }
}

int eep_last_hip_error(eep_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

}  // extern "C"

namespace {

// One routine behind eep_create, eep_create_attached, eep_create_with_workspace and
// eep_workspace_bytes (size_only: validate, report the slab size, touch no GPU).
int create_impl(const eep_config* cfg, eep_ctx* parent, void* workspace, int64_t workspace_bytes,
                int64_t* size_only, eep_ctx** out, eep_ctx* staging_of = nullptr) {
  if (!out && !size_only) return EEP_ERR_INVALID_ARG;
  if (out) *out = nullptr;
  if (!cfg) return EEP_ERR_INVALID_ARG;
  if (parent && cfg->num_ranks != parent->R) return EEP_ERR_INVALID_ARG;
  const eep_config& f = *cfg;
  if (f.num_ranks < 1 || f.slots_per_rank < 1 || f.primary_slots < 0 ||
      f.primary_slots > f.slots_per_rank || f.num_logical < 1 || f.max_tokens < 0 || f.topk < 1 ||
      f.topk > kMaxTopk || f.hidden < 1)
    return EEP_ERR_INVALID_ARG;
  if ((int64_t)f.num_ranks * f.slots_per_rank > (1 << 20) || f.num_logical > (1 << 20) ||
      (int64_t)f.max_tokens * f.topk > (int64_t)1 << 30)
    return EEP_ERR_INVALID_ARG;
  auto dtype_ok = [](int d) { return d == EEP_F32 || d == EEP_BF16; };
  if (!(dtype_ok(f.x_dtype) || f.x_dtype == EEP_FP8_E4M3) || !dtype_ok(f.y_dtype) ||
      !dtype_ok(f.out_dtype))
    return EEP_ERR_INVALID_ARG;
  if (f.policy != EEP_SPREAD && f.policy != EEP_FIRST_LIVE) return EEP_ERR_INVALID_ARG;
  if (f.x_dtype == EEP_FP8_E4M3) {
    if (f.scale_group < 16 || f.scale_group % 16 != 0 || f.hidden % f.scale_group != 0)
      return EEP_ERR_INVALID_ARG;
  } else if (f.scale_group != 0) {
    return EEP_ERR_INVALID_ARG;
  }

  eep_ctx* c = new (std::nothrow) eep_ctx();
  if (!c) return EEP_ERR_INVALID_ARG;
  c->cfg = f;
  c->R = f.num_ranks;
  c->S = f.slots_per_rank;
  c->S_prim = f.primary_slots;
  c->P = c->R * c->S;
  c->E = f.num_logical;
  c->k = f.topk;
  c->H = f.hidden;
  c->T_max = f.max_tokens;
  c->x_row_bytes = (int64_t)c->H * dtype_bytes(f.x_dtype);
  c->y_row_bytes = (int64_t)c->H * dtype_bytes(f.y_dtype);
  c->out_row_bytes = (int64_t)c->H * dtype_bytes(f.out_dtype);
  c->scale_row_bytes = f.x_dtype == EEP_FP8_E4M3 ? (int64_t)(c->H / f.scale_group) * 4 : 0;
  c->layout_T = -1;
  c->last_hip_error = 0;
  c->slab = nullptr;
  if (c->x_row_bytes % 16 || c->y_row_bytes % 16 || c->out_row_bytes % 16 ||
      c->scale_row_bytes % 16) {
    delete c;
    return EEP_ERR_ALIGN;
  }
  Tiling g = make_tiling(c->T_max - c->T_max % c->R, c->R);
  c->max_tiles = g.num_tiles > 0 ? g.num_tiles : 1;
  // the map kernel keeps its tables in LDS; refuse shapes that do not fit 64 KiB
  if (!layout_shape_fits(c->E, c->P, c->R, c->k)) {
    delete c;
    return EEP_ERR_INVALID_ARG;
  }

  const int64_t pairs = (int64_t)c->T_max * c->k;
  int64_t* n = c->field_ints;
  n[EEP_V_ACTIVE] = c->R;
  n[EEP_V_PHYS_TO_LOGICAL] = c->P;
  n[EEP_V_L2P_OFF] = c->E + 1;
  n[EEP_V_L2P_LIST] = c->P;
  n[EEP_V_SLOT_OF] = pairs;
  n[EEP_V_ROW_OF] = pairs;
  n[EEP_V_SRC_OF] = pairs;
  n[EEP_V_COUNT] = c->P;
  n[EEP_V_OFFSET] = c->P + 1;
  n[EEP_V_RANK_COUNT] = c->R;
  n[EEP_V_RANK_OFFSET] = c->R + 1;
  n[EEP_V_CNT_SRC] = (int64_t)c->R * c->P;
  n[EEP_V_STATUS] = 4;
  int32_t** field_ptr[EEP_V_NUM_FIELDS] = {
      &c->own_active, &c->p2l,   &c->l2p_off, &c->l2p_list,   &c->slot_of,     &c->row_of, &c->src_of,
      &c->count,  &c->offset, &c->rank_count, &c->rank_offset, &c->cnt_src, &c->status};
  // carve one slab; every array starts on a 256-byte boundary
  auto round_up = [](int64_t ints) { return (ints + 63) / 64 * 64; };
  int64_t total = 0;
  for (int i = 0; i < EEP_V_NUM_FIELDS; ++i) total += round_up(n[i] > 0 ? n[i] : 1);
  const int64_t n_tile = (int64_t)c->max_tiles * c->P;
  total += 2 * round_up(n_tile) + 2 * round_up(c->max_tiles) + 5 * round_up(1) +
           3 * round_up(c->R) + 4 * round_up(c->P);
  const int64_t n_dd_tile = (int64_t)c->max_tiles * c->R;
  total += 3 * round_up(pairs > 0 ? pairs : 1) + round_up(c->R) + round_up(c->R + 1) +
           round_up(n_dd_tile) + round_up(1);
  if (size_only) {
    *size_only = total * (int64_t)sizeof(int32_t);
    delete c;
    return EEP_OK;
  }

  hipError_t e = hipGetDevice(&c->device);
  if (e != hipSuccess) { delete c; return EEP_ERR_HIP; }
  if (parent && parent->device != c->device) { delete c; return EEP_ERR_INVALID_ARG; }
  if (workspace) {
    // caller-owned slab: device memory of this GPU, 256-byte aligned, large enough
    hipPointerAttribute_t at;
    void* base = nullptr;
    size_t size = 0;
    if (((uintptr_t)workspace & 255u) || workspace_bytes < total * (int64_t)sizeof(int32_t) ||
        hipPointerGetAttributes(&at, workspace) != hipSuccess || at.type != hipMemoryTypeDevice ||
        at.device != c->device ||
        hipMemGetAddressRange((hipDeviceptr_t*)&base, &size, (hipDeviceptr_t)workspace) != hipSuccess ||
        (const char*)workspace + workspace_bytes > (const char*)base + size) {
      (void)hipGetLastError();
      delete c;
      return EEP_ERR_INVALID_ARG;
    }
    c->slab = workspace;
    c->owns_slab = false;
  } else {
    e = hipMalloc(&c->slab, (size_t)total * sizeof(int32_t));
    if (e != hipSuccess) { delete c; return EEP_ERR_HIP; }
    c->owns_slab = true;
  }
  int32_t* cur = (int32_t*)c->slab;
  for (int i = 0; i < EEP_V_NUM_FIELDS; ++i) {
    *field_ptr[i] = cur;
    cur += round_up(n[i] > 0 ? n[i] : 1);
  }
  c->cnt_tile = cur;  cur += round_up(n_tile);
  c->base_tile = cur; cur += round_up(n_tile);
  c->blk_unc = cur;   cur += round_up(c->max_tiles);
  c->blk_msk = cur;   cur += round_up(c->max_tiles);
  c->tbl_version = cur; cur += round_up(1);
  c->mem_version_word = cur; cur += round_up(1);
  c->step_epoch = cur;  cur += round_up(1);
  c->round_ok = cur;    cur += round_up(1);
  c->check_bad = cur;   cur += round_up(1);
  c->signal = cur;      cur += round_up(c->R);
  c->withhold = cur;    cur += round_up(c->R);
  c->report = cur;      cur += round_up(c->R);
  c->mv_dst = cur;      cur += round_up(c->P);
  c->mv_src = cur;      cur += round_up(c->P);
  c->mv_expert = cur;   cur += round_up(c->P);
  c->mv_outcome = cur;  cur += round_up(c->P);
  c->dd_row = cur;      cur += round_up(pairs > 0 ? pairs : 1);
  c->dd_dst = cur;      cur += round_up(pairs > 0 ? pairs : 1);
  c->dd_expand = cur;   cur += round_up(pairs > 0 ? pairs : 1);
  c->dd_count = cur;    cur += round_up(c->R);
  c->dd_offset = cur;   cur += round_up(c->R + 1);
  c->dd_tile = cur;     cur += round_up(n_dd_tile);
  c->dd_status = cur;
  c->dedup_T = -1;
  c->detect_timeout_ticks = 0;
  c->wall_clock_khz = 0;

  // membership: a new instance (all ranks live), or the parent's
  if (parent) {
    c->mem = parent->mem;
  } else {
    c->mem = new (std::nothrow) eep_membership();
    if (!c->mem) { if (c->owns_slab) (void)hipFree(c->slab); delete c; return EEP_ERR_INVALID_ARG; }
    c->mem->R = c->R;
    c->mem->active = c->own_active;
    c->mem->mem_version = c->mem_version_word;
    c->mem->h_active.assign(c->R, 1);
    c->mem->unread_round = false;
  }
  c->active = c->mem->active;
  c->tables = c;
  c->n_staging = 0;
  c->ev_fork = c->ev_join = nullptr;
  // initial state: every slot empty, nothing laid out
  c->h_p2l.assign(c->P, -1);
  hipStream_t st = nullptr;
  e = hipMemsetAsync(c->slab, 0, (size_t)total * sizeof(int32_t), st);
  if (e == hipSuccess) e = launch_fill(c->own_active, 1, c->R, st);
  if (e == hipSuccess) e = launch_fill(c->p2l, -1, c->P, st);
  if (e == hipSuccess) e = launch_fill(c->l2p_list, -1, c->P, st);
  if (e == hipSuccess) e = launch_fill(c->slot_of, -1, pairs, st);
  if (e == hipSuccess) e = launch_fill(c->row_of, -1, pairs, st);
  if (e == hipSuccess) e = launch_fill(c->src_of, -1, pairs, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) {
    if (c->owns_slab) (void)hipFree(c->slab);
    if (!parent) delete c->mem;
    delete c;
    return EEP_ERR_HIP;
  }
  if (staging_of) {
    // a second staging set of the same layer: the placement tables are the owner's
    eep_ctx* owner = staging_of->tables;
    c->tables = owner;
    c->p2l = owner->p2l;
    c->l2p_off = owner->l2p_off;
    c->l2p_list = owner->l2p_list;
    c->tbl_version = owner->tbl_version;
    owner->n_staging += 1;
  }
  c->mem->members.push_back(c);
  *out = c;
  return EEP_OK;
}

}  // namespace

extern "C" {

int eep_create(const eep_config* cfg, eep_ctx** out) {
  return create_impl(cfg, nullptr, nullptr, 0, nullptr, out);
}

int eep_workspace_bytes(const eep_config* cfg, int64_t* bytes) {
  if (!bytes) return EEP_ERR_INVALID_ARG;
  *bytes = 0;
  return create_impl(cfg, nullptr, nullptr, 0, bytes, nullptr);
}

int eep_create_with_workspace(const eep_config* cfg, void* workspace, int64_t workspace_bytes,
                              eep_ctx** out) {
  if (!workspace) {
    if (out) *out = nullptr;
    return EEP_ERR_INVALID_ARG;
  }
  return create_impl(cfg, nullptr, workspace, workspace_bytes, nullptr, out);
}

int eep_create_attached(const eep_config* cfg, eep_ctx* parent, eep_ctx** out) {
  if (!parent) {
    if (out) *out = nullptr;
    return EEP_ERR_INVALID_ARG;
  }
  return create_impl(cfg, parent, nullptr, 0, nullptr, out);
}

int eep_create_staging(eep_ctx* of, eep_ctx** out) {
  if (!of) {
    if (out) *out = nullptr;
    return EEP_ERR_INVALID_ARG;
  }
  return create_impl(&of->cfg, of, nullptr, 0, nullptr, out, of);
}

int eep_destroy(eep_ctx* ctx) {
  if (!ctx) return EEP_OK;
  eep_membership* m = ctx->mem;
  const bool is_root = m->members.front() == ctx;
  if (is_root && m->members.size() > 1) return EEP_ERR_STATE;  // attached contexts go first
  if (ctx->n_staging > 0) return EEP_ERR_STATE;  // so do the staging sets that use its tables
  hipError_t e = hipDeviceSynchronize();
  if (ctx->tables != ctx) ctx->tables->n_staging -= 1;
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
  for (size_t i = 0; i < m->members.size(); ++i)
    if (m->members[i] == ctx) {
      m->members.erase(m->members.begin() + i);
      break;
    }
  hipError_t e2 = ctx->owns_slab ? hipFree(ctx->slab) : hipSuccess;
  if (is_root) delete m;
  delete ctx;
  return (e == hipSuccess && e2 == hipSuccess) ? EEP_OK : EEP_ERR_HIP;
}

int eep_set_membership(eep_ctx* c, const int32_t* active_host, void* stream) {
  if (!c || !active_host) return EEP_ERR_INVALID_ARG;
  eep_membership* m = c->mem;
  // A waiting kernel may have dropped a rank that the host's copy of the mask still shows
  // as live; rewriting the whole mask from the caller's array would bring it back.
  if (m->unread_round) return EEP_ERR_STATE;
  std::vector<int32_t> a(c->R);
  for (int r = 0; r < c->R; ++r) a[r] = active_host[r] != 0 ? 1 : 0;
  // the mask is shared: every context of the instance that asked for strict
  // coverage must stay covered under its own placement
  for (eep_ctx* o : m->members)
    if (o->tables == o && o->cfg.strict_coverage &&
        host_uncovered_experts(o->P, o->E, o->S, o->h_p2l.data(), a.data()) > 0)
      return EEP_ERR_COVERAGE;
  hipError_t e = launch_patch(m->active, a.data(), c->R, m->mem_version, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(c, e);
  m->h_active = a;
  return EEP_OK;
}

}  // extern "C"

namespace eep {

// Checks and publishes a placement.  `mask_may_be_stale`: the caller has dealt with an
// unread detection round itself (eep_apply_repair looks the device mask up per transfer).
int publish_placement(eep_ctx* c, const int32_t* p2l_host, bool mask_may_be_stale,
                      hipStream_t st) {
  c = c->tables;  // a staging context names its owner's tables
  for (int p = 0; p < c->P; ++p)
    if (p2l_host[p] < -1 || p2l_host[p] >= c->E) return EEP_ERR_INVALID_ARG;
  if (c->cfg.strict_coverage) {
    // coverage is judged against the host's copy of the mask, which must be current
    if (c->mem->unread_round && !mask_may_be_stale) return EEP_ERR_STATE;
    if (host_uncovered_experts(c->P, c->E, c->S, p2l_host, c->mem->h_active.data()) > 0)
      return EEP_ERR_COVERAGE;
  }
  std::vector<int32_t> off(c->E + 1), list(c->P);
  host_replica_lists(c->P, c->E, c->S, c->S_prim, p2l_host, off.data(), list.data());
  hipError_t e = launch_patch(c->p2l, p2l_host, c->P, nullptr, st);
  if (e == hipSuccess) e = launch_patch(c->l2p_off, off.data(), c->E + 1, nullptr, st);
  if (e == hipSuccess) e = launch_patch(c->l2p_list, list.data(), c->P, c->tbl_version, st);
  if (e != hipSuccess) return fail_hip(c, e);
  c->h_p2l.assign(p2l_host, p2l_host + c->P);
  return EEP_OK;
}

}  // namespace eep

extern "C" {

int eep_update_placement(eep_ctx* c, const int32_t* p2l_host, void* stream) {
  if (!c || !p2l_host) return EEP_ERR_INVALID_ARG;
  return publish_placement(c, p2l_host, false, (hipStream_t)stream);
}

int eep_dispatch_layout(eep_ctx* c, const int32_t* topk_idx, int32_t T, void* stream) {
  if (!c || T < 0 || T > c->T_max || T % c->R != 0) return EEP_ERR_INVALID_ARG;
  if (T > 0 && !topk_idx) return EEP_ERR_INVALID_ARG;
  hipError_t e = launch_layout(c, topk_idx, T, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(c, e);
  c->layout_T = T;
  c->dedup_T = -1;  // the de-duplicated tables belong to the previous layout
  return EEP_OK;
}

int eep_dispatch(eep_ctx* c, const void* x, const float* x_scale, void* recv_x, float* recv_scale,
                 int32_t T, void* stream) {
  if (!c || T < 0 || T > c->T_max) return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T) return EEP_ERR_STATE;
  if (T == 0) return EEP_OK;
  if (!x || !recv_x) return EEP_ERR_INVALID_ARG;
  const bool fp8 = c->cfg.x_dtype == EEP_FP8_E4M3;
  if (fp8 != (x_scale != nullptr) || fp8 != (recv_scale != nullptr)) return EEP_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(recv_x) || !aligned16(x_scale) || !aligned16(recv_scale))
    return EEP_ERR_ALIGN;
  hipError_t e = launch_pack(c, x, x_scale, recv_x, recv_scale, T, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_staging_fork(eep_ctx* c, const int32_t* topk_idx, const void* x, const float* x_scale,
                     void* recv_x, float* recv_scale, int32_t T, void* stream, void* side_stream) {
  if (!c || !stream || !side_stream || stream == side_stream) return EEP_ERR_INVALID_ARG;
  hipError_t e = hipSuccess;
  if (!c->ev_fork) e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess && !c->ev_join) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
  // the side stream starts after everything queued on `stream` so far
  if (e == hipSuccess) e = hipEventRecord(c->ev_fork, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamWaitEvent((hipStream_t)side_stream, c->ev_fork, 0);
  if (e != hipSuccess) return fail_hip(c, e);
  int rc = eep_dispatch_layout(c, topk_idx, T, side_stream);
  if (rc == EEP_OK) rc = eep_dispatch(c, x, x_scale, recv_x, recv_scale, T, side_stream);
  // Whatever happened, the side stream is joined again by eep_staging_join; a stream left
  // forked would make an enclosing capture fail.
  return rc;
}

int eep_staging_join(eep_ctx* c, void* stream, void* side_stream) {
  if (!c || !stream || !side_stream || stream == side_stream) return EEP_ERR_INVALID_ARG;
  if (!c->ev_join) return EEP_ERR_STATE;  // no eep_staging_fork before
  hipError_t e = hipEventRecord(c->ev_join, (hipStream_t)side_stream);
  if (e == hipSuccess) e = hipStreamWaitEvent((hipStream_t)stream, c->ev_join, 0);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_dispatch_quant(eep_ctx* c, const void* x_bf16, void* recv_x, float* recv_scale, int32_t T,
                       void* stream) {
  if (!c || T < 0 || T > c->T_max) return EEP_ERR_INVALID_ARG;
  if (c->cfg.x_dtype != EEP_FP8_E4M3) return EEP_ERR_INVALID_ARG;
  const int lanes_per_group = c->cfg.scale_group / 16;
  if (lanes_per_group > 64 || (lanes_per_group & (lanes_per_group - 1)) != 0 ||
      c->H / c->cfg.scale_group > 8192)
    return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T) return EEP_ERR_STATE;
  if (T == 0) return EEP_OK;
  if (!x_bf16 || !recv_x || !recv_scale) return EEP_ERR_INVALID_ARG;
  if (!aligned16(x_bf16) || !aligned16(recv_x) || ((uintptr_t)recv_scale & 3u))
    return EEP_ERR_ALIGN;
  hipError_t e = launch_pack_quant(c, x_bf16, recv_x, recv_scale, T, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_combine(eep_ctx* c, const void* y, const float* topk_w, void* out, int32_t T,
                void* stream) {
  if (!c || T < 0 || T > c->T_max) return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T) return EEP_ERR_STATE;
  if (T == 0) return EEP_OK;
  if (!y || !topk_w || !out) return EEP_ERR_INVALID_ARG;
  if (!aligned16(y) || !aligned16(out)) return EEP_ERR_ALIGN;
  // with detection on, the kernel itself waits for the ranks' signals and may drop one
  if (c->detect_timeout_ticks > 0) c->mem->unread_round = true;  // until eep_read_failures
  hipError_t e = launch_combine(c, y, topk_w, out, T, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_expert_stub(eep_ctx* c, int32_t kind, const void* recv_x, const float* recv_scale,
                    const float* expert_scale, void* y, int32_t T, void* stream) {
  if (!c || T < 0 || T > c->T_max) return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T) return EEP_ERR_STATE;
  if (T == 0) return EEP_OK;
  if (!recv_x || !y) return EEP_ERR_INVALID_ARG;
  if (!aligned16(recv_x) || !aligned16(y)) return EEP_ERR_ALIGN;
  switch (kind) {
    case EEP_STUB_IDENTITY:
      if (c->cfg.x_dtype != c->cfg.y_dtype) return EEP_ERR_INVALID_ARG;
      break;
    case EEP_STUB_SCALE:
      if (c->cfg.x_dtype != c->cfg.y_dtype || !expert_scale) return EEP_ERR_INVALID_ARG;
      break;
    case EEP_STUB_DEQUANT:
      if (c->cfg.x_dtype != EEP_FP8_E4M3 || c->cfg.y_dtype != EEP_BF16 || !recv_scale)
        return EEP_ERR_INVALID_ARG;
      break;
    default:
      return EEP_ERR_INVALID_ARG;
  }
  hipError_t e =
      launch_stub(c, kind, recv_x, recv_scale, expert_scale, y, T, (hipStream_t)stream);
  if (e == hipSuccess && c->detect_timeout_ticks > 0) e = launch_signal(c, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_set_detection(eep_ctx* c, int64_t timeout_ns) {
  if (!c || timeout_ns < 0 || timeout_ns > 2000000000LL || c->R > 8192)
    return EEP_ERR_INVALID_ARG;
  if (timeout_ns == 0) {
    c->detect_timeout_ticks = 0;
    return EEP_OK;
  }
  if (c->wall_clock_khz == 0) {
    int khz = 0;
    hipError_t e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, c->device);
    if (e != hipSuccess || khz <= 0) return fail_hip(c, e);
    c->wall_clock_khz = khz;
  }
  int64_t ticks = (timeout_ns * c->wall_clock_khz + 999999) / 1000000;
  c->detect_timeout_ticks = ticks > 0 ? ticks : 1;
  return EEP_OK;
}

int eep_signal_experts_done(eep_ctx* c, void* stream) {
  if (!c) return EEP_ERR_INVALID_ARG;
  hipError_t e = launch_signal(c, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_debug_withhold_signal(eep_ctx* c, const int32_t* withhold_host, void* stream) {
  if (!c || !withhold_host) return EEP_ERR_INVALID_ARG;
  std::vector<int32_t> w(c->R);
  for (int r = 0; r < c->R; ++r) w[r] = withhold_host[r] != 0;
  hipError_t e = launch_patch(c->withhold, w.data(), c->R, nullptr, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_read_failures(eep_ctx* c, int32_t* failed_host, void* stream) {
  if (!c || !failed_host) return EEP_ERR_INVALID_ARG;
  eep_membership* m = c->mem;
  hipStream_t st = (hipStream_t)stream;
  // the mask is shared by every context of the instance, so every context's report counts;
  // their steps may run on other streams
  hipError_t e = m->members.size() > 1 ? hipDeviceSynchronize() : hipStreamSynchronize(st);
  if (e != hipSuccess) return fail_hip(c, e);
  for (int r = 0; r < c->R; ++r) failed_host[r] = 0;
  std::vector<int32_t> rep(c->R);
  for (eep_ctx* o : m->members) {
    e = hipMemcpy(rep.data(), o->report, sizeof(int32_t) * c->R, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(c, e);
    bool any = false;
    for (int r = 0; r < c->R; ++r)
      if (rep[r] != 0) {
        failed_host[r] = 1;
        m->h_active[r] = 0;  // the kernel already cleared the device copy
        any = true;
      }
    if (any) {
      e = launch_fill(o->report, 0, c->R, st);
      if (e != hipSuccess) return fail_hip(c, e);
    }
  }
  m->unread_round = false;
  return EEP_OK;
}

int eep_dedup_layout(eep_ctx* c, int32_t T, void* stream) {
  if (!c || T < 0 || T > c->T_max) return EEP_ERR_INVALID_ARG;
  if (c->R > kDedupMaxRanks) return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T) return EEP_ERR_STATE;
  hipError_t e = launch_dedup_layout(c, T, (hipStream_t)stream);
  if (e != hipSuccess) return fail_hip(c, e);
  c->dedup_T = T;
  return EEP_OK;
}

int eep_dispatch_dedup(eep_ctx* c, const void* x, void* recv_dedup, int32_t T, void* stream) {
  if (!c || T < 0 || T > c->T_max || c->cfg.x_dtype == EEP_FP8_E4M3) return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T || c->dedup_T != T) return EEP_ERR_STATE;
  if (T == 0) return EEP_OK;
  if (!x || !recv_dedup) return EEP_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(recv_dedup)) return EEP_ERR_ALIGN;
  hipError_t e = launch_pack_rows(c, c->dd_dst, x, recv_dedup, T, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_expand(eep_ctx* c, const void* recv_dedup, void* recv_x, int32_t T, void* stream) {
  if (!c || T < 0 || T > c->T_max || c->cfg.x_dtype == EEP_FP8_E4M3) return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T || c->dedup_T != T) return EEP_ERR_STATE;
  if (T == 0) return EEP_OK;
  if (!recv_dedup || !recv_x || recv_dedup == recv_x) return EEP_ERR_INVALID_ARG;
  if (!aligned16(recv_dedup) || !aligned16(recv_x)) return EEP_ERR_ALIGN;
  hipError_t e = launch_expand(c, recv_dedup, recv_x, T, (hipStream_t)stream);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_read_dedup(eep_ctx* c, int32_t field, int32_t* host_dst, int64_t n, void* stream) {
  if (!c || field < 0 || field >= EEP_D_NUM_FIELDS || n < 0) return EEP_ERR_INVALID_ARG;
  const int64_t pairs = (int64_t)c->T_max * c->k;
  const int64_t size[EEP_D_NUM_FIELDS] = {c->R, c->R + 1, pairs, pairs, pairs, 1};
  const int32_t* src[EEP_D_NUM_FIELDS] = {c->dd_count, c->dd_offset, c->dd_row,
                                          c->dd_dst,   c->dd_expand, c->dd_status};
  if (n > size[field]) return EEP_ERR_INVALID_ARG;
  if (n == 0) return EEP_OK;
  if (!host_dst) return EEP_ERR_INVALID_ARG;
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e == hipSuccess)
    e = hipMemcpy(host_dst, src[field], (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_debug_check_layout(eep_ctx* c, int32_t T, int32_t violations_host[4], void* stream) {
  if (!c || !violations_host || T < 0 || T > c->T_max) return EEP_ERR_INVALID_ARG;
  if (c->layout_T != T) return EEP_ERR_STATE;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = launch_check_layout(c, T, c->check_bad, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e == hipSuccess)
    e = hipMemcpy(violations_host, c->check_bad, 4 * sizeof(int32_t), hipMemcpyDeviceToHost);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

int eep_get_dedup_view(eep_ctx* c, eep_dedup_view* out) {
  if (!c || !out) return EEP_ERR_INVALID_ARG;
  out->dedup_count = c->dd_count;
  out->dedup_offset = c->dd_offset;
  out->dedup_row = c->dd_row;
  out->dedup_dst = c->dd_dst;
  out->expand_of = c->dd_expand;
  out->status = c->dd_status;
  return EEP_OK;
}

int eep_get_view(eep_ctx* c, eep_view* out) {
  if (!c || !out) return EEP_ERR_INVALID_ARG;
  out->active = c->active;
  out->phys_to_logical = c->p2l;
  out->l2p_off = c->l2p_off;
  out->l2p_list = c->l2p_list;
  out->slot_of = c->slot_of;
  out->row_of = c->row_of;
  out->src_of = c->src_of;
  out->count = c->count;
  out->offset = c->offset;
  out->rank_count = c->rank_count;
  out->rank_offset = c->rank_offset;
  out->cnt_src = c->cnt_src;
  out->status = c->status;
  return EEP_OK;
}

int eep_read_view(eep_ctx* c, int32_t field, int32_t* host_dst, int64_t n, void* stream) {
  if (!c || field < 0 || field >= EEP_V_NUM_FIELDS || n < 0) return EEP_ERR_INVALID_ARG;
  if (n > c->field_ints[field]) return EEP_ERR_INVALID_ARG;
  if (n == 0) return EEP_OK;
  if (!host_dst) return EEP_ERR_INVALID_ARG;
  const int32_t* src[EEP_V_NUM_FIELDS] = {c->active, c->p2l,    c->l2p_off,    c->l2p_list,
                                          c->slot_of, c->row_of, c->src_of,     c->count,
                                          c->offset,  c->rank_count, c->rank_offset, c->cnt_src,
                                          c->status};
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e == hipSuccess)
    e = hipMemcpy(host_dst, src[field], (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost);
  return e == hipSuccess ? EEP_OK : fail_hip(c, e);
}

}  // extern "C"
