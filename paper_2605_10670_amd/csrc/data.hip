// The bandwidth-bound half of the step: pack (dispatch), the expert stand-ins,
// and the weighted gather-reduce (combine).
//
// Paper: Fig. 7 (dispatch writes one token row per (token, destination)),
// Sec. 4.1 (combine reduces the expert outputs), Sec. 6.2 (dispatch and
// combine dominate the cost of EP serving).  Nothing here is a contraction:
// every kernel is bound by HBM traffic, so the design rules are 16-byte
// accesses, whole 64-lane wavefronts on contiguous 1 KiB spans, each input byte
// read once, and enough independent loads in flight per lane.
#include "eep_internal.hpp"

namespace eep {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// pack: recv[row_of[t, j]] = x[t].  One wavefront per token reads the row once
// into registers (up to kPackVecs 16-byte vectors per lane per pass, every load
// issued before the first store) and stores it to the token's k rows; each
// store instruction covers 1 KiB of contiguous row.  Measured on MI355X at the
// decode shape: fatter workgroups, persistent grids, column-split tokens and
// destination-ordered (gather) forms were all slower; stores marked
// write-through at system scope were ~5 % faster than plain or non-temporal
// stores.
// ---------------------------------------------------------------------------
constexpr int kPackVecs = 14;
constexpr int kPackSplitBelow = 1024;  // batches below this many tokens split a row over wavefronts

__device__ inline void store_through(u32x4* p, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
}

// U = 16-byte vectors per lane per pass.  EXACT: the row is a whole number of
// passes (row_vecs % (64 * U) == 0), so no load or store needs a bounds guard
// and the compiler keeps all U loads of a pass in flight; otherwise every
// access is guarded (any row size).  `parts` wavefronts share a token, taking
// every parts-th pass each: 1 for large batches (a whole row per wavefront
// measured fastest there), more for small ones, which would otherwise leave
// most of the chip idle.
// SPLIT selects at compile time: the one-wavefront-per-token form keeps its simpler
// indexing (2 us faster at the decode shape than the general form with parts = 1).
template <int U, bool EXACT, bool SPLIT>
__global__ __launch_bounds__(64) void k_pack(const u32x4* __restrict__ x,
                                             u32x4* __restrict__ recv,
                                             const int32_t* __restrict__ row_of, int k,
                                             int row_vecs, int parts) {
  const int t = SPLIT ? blockIdx.x / parts : blockIdx.x;
  const int part = SPLIT ? blockIdx.x - t * parts : 0;
  const int step = SPLIT ? parts * 64 * U : 64 * U;
  const int lane = threadIdx.x;
  const int32_t* rows = row_of + (int64_t)t * k;
  const u32x4* src = x + (int64_t)t * row_vecs;
  for (int v0 = part * 64 * U; v0 < row_vecs; v0 += step) {
    u32x4 buf[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int v = v0 + u * 64 + lane;
      if (EXACT || v < row_vecs) buf[u] = __builtin_nontemporal_load(&src[v]);
    }
    // Touch every loaded register here, so that the waits for the loads sit in
    // front of the row loop and the stores of consecutive rows stream out
    // without a wait between them.
    if (EXACT) {
#pragma unroll
      for (int u = 0; u < U; ++u) asm volatile("" ::"v"(buf[u]));
    }
    for (int j = 0; j < k; ++j) {
      int row = rows[j];
      if (row < 0) continue;
      u32x4* dst = recv + (int64_t)row * row_vecs;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        int v = v0 + u * 64 + lane;
        if (EXACT || v < row_vecs) store_through(&dst[v], buf[u]);
      }
    }
  }
}

// Several tokens per wavefront: all TPW * U loads of the wavefront are issued
// before its first store, then the TPW * k rows stream out.  Measured on MI355X
// (T = 16384, 7 KiB rows): 212 us with one token per wavefront, 201 with four,
// 192 with eight; what counts is that the launch comes down to about 2048
// wavefronts -- two per SIMD, all resident at once, every load of the launch in
// flight before the stores start.  Fewer wavefronts than that, or a loop over
// token groups inside a wavefront, are slower again.  T % TPW == 0, rows exact.
template <int U, int TPW>
__global__ __launch_bounds__(64) void k_pack_multi(const u32x4* __restrict__ x,
                                                   u32x4* __restrict__ recv,
                                                   const int32_t* __restrict__ row_of, int k,
                                                   int row_vecs) {
  const int t0 = blockIdx.x * TPW;
  const int lane = threadIdx.x;
  u32x4 buf[TPW][U];
#pragma unroll
  for (int q = 0; q < TPW; ++q) {
    const u32x4* src = x + (int64_t)(t0 + q) * row_vecs;
#pragma unroll
    for (int u = 0; u < U; ++u) buf[q][u] = __builtin_nontemporal_load(&src[u * 64 + lane]);
  }
#pragma unroll
  for (int q = 0; q < TPW; ++q) {
#pragma unroll
    for (int u = 0; u < U; ++u) asm volatile("" ::"v"(buf[q][u]));  // waits sit before the stores
  }
#pragma unroll
  for (int q = 0; q < TPW; ++q) {
    const int32_t* rows = row_of + (int64_t)(t0 + q) * k;
    for (int j = 0; j < k; ++j) {
      int row = rows[j];
      if (row < 0) continue;
      u32x4* dst = recv + (int64_t)row * row_vecs;
#pragma unroll
      for (int u = 0; u < U; ++u) store_through(&dst[u * 64 + lane], buf[q][u]);
    }
  }
}

// Scale rows of fp8 payloads (H/group fp32 values per row; 224 bytes at the
// prefill shape), written in DESTINATION order: a thread owns one 16-byte
// vector of the receive scale buffer, finds the token behind its row through
// src_of, and copies the vector from the small [T][H/group] source table (3.6 MB
// at T = 16384, read 8 times, from cache).  All stores are contiguous.
// Measured at T = 16384 inside the step (payload, scales, combine in a loop):
// token-ordered scatter with one token per wavefront +27 us, with four tokens
// per wavefront +20 us, this form +10 us, for 33 MB; 224-byte rows scattered
// among the payload's write stream are what is expensive, not the launch.
constexpr int kScaleThreads = 256;
constexpr int kScaleVecs = 4;  // vectors per thread, each an independent chain of lookups
                               // (measured at T = 16384: 2 per thread -1.5 us, 4 -3 us, 8 +5 us
                               // against one vector per thread)

// max_vecs = T * k * scale_vecs (every row the buffers hold); the rows of this step end at
// status[0], which is read beside the first lookups rather than ahead of them.
__global__ __launch_bounds__(kScaleThreads) void k_scale_rows(
    const u32x4* __restrict__ x_scale, u32x4* __restrict__ recv_scale,
    const int32_t* __restrict__ src_of, const int32_t* __restrict__ status, int k, int scale_vecs,
    int64_t max_vecs) {
  const int64_t v0 = (int64_t)blockIdx.x * (kScaleThreads * kScaleVecs) + threadIdx.x;
  int pair[kScaleVecs], col[kScaleVecs];
#pragma unroll
  for (int u = 0; u < kScaleVecs; ++u) {
    const int64_t v = v0 + u * kScaleThreads;
    const int row = (int)(v / scale_vecs);
    col[u] = (int)(v - (int64_t)row * scale_vecs);
    pair[u] = v < max_vecs ? src_of[row] : -1;
  }
  const int64_t n_vecs = (int64_t)status[0] * scale_vecs;  // rows >= N are left untouched
  u32x4 val[kScaleVecs];
#pragma unroll
  for (int u = 0; u < kScaleVecs; ++u) {
    if (v0 + u * kScaleThreads >= n_vecs) pair[u] = -1;
    if (pair[u] >= 0) val[u] = x_scale[(int64_t)(pair[u] / k) * scale_vecs + col[u]];
  }
#pragma unroll
  for (int u = 0; u < kScaleVecs; ++u)
    if (pair[u] >= 0) store_through(&recv_scale[v0 + u * kScaleThreads], val[u]);
}

template <int U, bool EXACT>
static hipError_t launch_pack_t(eep_ctx* c, const int32_t* rows, const void* x, void* recv_x,
                                int T, int parts, hipStream_t st) {
  if (parts > 1)
    hipLaunchKernelGGL((k_pack<U, EXACT, true>), dim3((unsigned)((int64_t)T * parts)), dim3(64), 0,
                       st, (const u32x4*)x, (u32x4*)recv_x, rows, c->k,
                       (int)(c->x_row_bytes / 16), parts);
  else
    hipLaunchKernelGGL((k_pack<U, EXACT, false>), dim3(T), dim3(64), 0, st, (const u32x4*)x,
                       (u32x4*)recv_x, rows, c->k, (int)(c->x_row_bytes / 16), 1);
  return hipGetLastError();
}

template <int U, int TPW>
static hipError_t launch_pack_multi_t(eep_ctx* c, const int32_t* rows, const void* x, void* recv_x,
                                      int T, hipStream_t st) {
  hipLaunchKernelGGL((k_pack_multi<U, TPW>), dim3(T / TPW), dim3(64), 0, st, (const u32x4*)x,
                     (u32x4*)recv_x, rows, c->k, (int)(c->x_row_bytes / 16));
  return hipGetLastError();
}

// Below 8192 tokens one wavefront per token already fits the chip in one round (8192
// resident wavefronts), and at the decode shape (T = 4096, 14 KiB rows) two tokens per
// wavefront made the step 3 us slower: pack itself no faster, the combine after it slower.
constexpr int kPackMultiMinTokens = 8192;
constexpr int kPackMultiMinWaves = 2048;  // two wavefronts per SIMD of the 256 CUs
constexpr int kPackMultiMaxVecs = 56;     // 16-byte vectors a lane holds at once

static hipError_t launch_pack_payload(eep_ctx* c, const int32_t* rows, const void* x, void* recv_x,
                                      int T, hipStream_t st) {
  const int row_vecs = (int)(c->x_row_bytes / 16);
  if (row_vecs % 64 == 0) {
    // Large batches: one wavefront per token, the largest pass width <= kPackVecs that
    // divides the per-lane vector count (a whole 14 KiB row per wavefront at the decode
    // shape).  Small batches (< kPackSplitBelow tokens) would leave most of the chip idle
    // that way, so a row is split over wavefronts, each taking one pass of the smallest
    // width >= 2: measured at 32 ranks, top-8, 14 KiB rows, 2 KiB per wavefront and row is
    // about twice as fast as 1 KiB or 7 KiB pieces for 64 <= T <= 256 (1 KiB pieces are
    // no better than whole rows), and nothing differs from T = 1024 on.
    const int per_lane = row_vecs / 64;
    int u, parts;
    if (T < kPackSplitBelow && per_lane > 1) {
      u = 2;
      while (per_lane % u != 0) ++u;  // ends at per_lane at the latest
      if (u > kPackVecs) u = 1;       // a large prime: fall back to single vectors
      parts = per_lane / u;
    } else {
      u = kPackVecs;
      while (per_lane % u != 0) --u;
      parts = 1;
      // Very large batches (>= kPackMultiMinTokens) of whole-row passes: several tokens per
      // wavefront, as many as keep >= kPackMultiMinWaves wavefronts and <= kPackMultiMaxVecs
      // vectors per lane.
      if (u == per_lane) {
        int tpw = 1;
        while (T >= kPackMultiMinTokens && tpw < 8 && T % (tpw * 2) == 0 &&
               T / (tpw * 2) >= kPackMultiMinWaves &&
               per_lane * tpw * 2 <= kPackMultiMaxVecs)
          tpw *= 2;
        if (tpw > 1) {
          switch (tpw * 16 + u) {
#define EEP_PACK_MULTI(TPW, U) \
  case TPW * 16 + U: return launch_pack_multi_t<U, TPW>(c, rows, x, recv_x, T, st);
            EEP_PACK_MULTI(2, 1) EEP_PACK_MULTI(2, 2) EEP_PACK_MULTI(2, 3) EEP_PACK_MULTI(2, 4)
            EEP_PACK_MULTI(2, 5) EEP_PACK_MULTI(2, 6) EEP_PACK_MULTI(2, 7) EEP_PACK_MULTI(2, 8)
            EEP_PACK_MULTI(2, 9) EEP_PACK_MULTI(2, 10) EEP_PACK_MULTI(2, 11) EEP_PACK_MULTI(2, 12)
            EEP_PACK_MULTI(2, 13) EEP_PACK_MULTI(2, 14)
            EEP_PACK_MULTI(4, 1) EEP_PACK_MULTI(4, 2) EEP_PACK_MULTI(4, 3) EEP_PACK_MULTI(4, 4)
            EEP_PACK_MULTI(4, 5) EEP_PACK_MULTI(4, 6) EEP_PACK_MULTI(4, 7) EEP_PACK_MULTI(4, 8)
            EEP_PACK_MULTI(4, 9) EEP_PACK_MULTI(4, 10) EEP_PACK_MULTI(4, 11) EEP_PACK_MULTI(4, 12)
            EEP_PACK_MULTI(4, 13) EEP_PACK_MULTI(4, 14)
            EEP_PACK_MULTI(8, 1) EEP_PACK_MULTI(8, 2) EEP_PACK_MULTI(8, 3) EEP_PACK_MULTI(8, 4)
            EEP_PACK_MULTI(8, 5) EEP_PACK_MULTI(8, 6) EEP_PACK_MULTI(8, 7)
#undef EEP_PACK_MULTI
          }
        }
      }
    }
    switch (u) {
#define EEP_PACK_CASE(U) \
  case U: return launch_pack_t<U, true>(c, rows, x, recv_x, T, parts, st);
      EEP_PACK_CASE(14) EEP_PACK_CASE(13) EEP_PACK_CASE(12) EEP_PACK_CASE(11) EEP_PACK_CASE(10)
      EEP_PACK_CASE(9) EEP_PACK_CASE(8) EEP_PACK_CASE(7) EEP_PACK_CASE(6) EEP_PACK_CASE(5)
      EEP_PACK_CASE(4) EEP_PACK_CASE(3) EEP_PACK_CASE(2) EEP_PACK_CASE(1)
#undef EEP_PACK_CASE
    }
  }
  return launch_pack_t<kPackVecs, false>(c, rows, x, recv_x, T, 1, st);
}

static hipError_t launch_pack_any(eep_ctx* c, const int32_t* rows, const void* x,
                                  const float* x_scale, void* recv_x, float* recv_scale, int T,
                                  hipStream_t st) {
  if (T == 0) return hipSuccess;
  hipError_t e = launch_pack_payload(c, rows, x, recv_x, T, st);
  if (e != hipSuccess || x_scale == nullptr) return e;
  const int scale_vecs = (int)(c->scale_row_bytes / 16);
  const int64_t vecs = (int64_t)T * c->k * scale_vecs;
  const int64_t per_block = (int64_t)kScaleThreads * kScaleVecs;
  const int64_t blocks = (vecs + per_block - 1) / per_block;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_scale_rows, dim3((unsigned)blocks), dim3(kScaleThreads), 0, st,
                     (const u32x4*)x_scale, (u32x4*)recv_scale, c->src_of, c->status, c->k,
                     scale_vecs, vecs);
  return hipGetLastError();
}

hipError_t launch_pack(eep_ctx* c, const void* x, const float* x_scale, void* recv_x,
                       float* recv_scale, int T, hipStream_t st) {
  return launch_pack_any(c, c->row_of, x, x_scale, recv_x, recv_scale, T, st);
}

hipError_t launch_pack_rows(eep_ctx* c, const int32_t* rows, const void* x, void* recv, int T,
                            hipStream_t st) {
  return launch_pack_any(c, rows, x, nullptr, recv, nullptr, T, st);
}

// ---------------------------------------------------------------------------
// Expansion on the destination of a de-duplicated dispatch:
// recv[row] = recv_d[expand_of[row]] for the N routed rows.  One wavefront per
// row; the grid covers T*k rows and reads N from device memory.
// ---------------------------------------------------------------------------
constexpr int kExpandVecs = 7;

__global__ __launch_bounds__(64) void k_expand(const u32x4* __restrict__ recv_d,
                                               u32x4* __restrict__ recv,
                                               const int32_t* __restrict__ expand_of,
                                               const int32_t* __restrict__ status, int row_vecs) {
  const int row = blockIdx.x;
  if (row >= status[0]) return;
  const int from = expand_of[row];
  if (from < 0) return;
  const u32x4* src = recv_d + (int64_t)from * row_vecs;
  u32x4* dst = recv + (int64_t)row * row_vecs;
  for (int v0 = threadIdx.x; v0 < row_vecs; v0 += 64 * kExpandVecs) {
    u32x4 buf[kExpandVecs];
#pragma unroll
    for (int u = 0; u < kExpandVecs; ++u)
      if (v0 + u * 64 < row_vecs) buf[u] = __builtin_nontemporal_load(&src[v0 + u * 64]);
#pragma unroll
    for (int u = 0; u < kExpandVecs; ++u)
      if (v0 + u * 64 < row_vecs) store_through(&dst[v0 + u * 64], buf[u]);
  }
}

hipError_t launch_expand(eep_ctx* c, const void* recv_dedup, void* recv_x, int T, hipStream_t st) {
  const int64_t rows = (int64_t)T * c->k;
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(k_expand, dim3((unsigned)rows), dim3(64), 0, st, (const u32x4*)recv_dedup,
                     (u32x4*)recv_x, c->dd_expand, c->status, (int)(c->x_row_bytes / 16));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// number formats
// ---------------------------------------------------------------------------
__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// binary32 -> bfloat16 bits, round to nearest even, NaN stays (quiet) NaN
__device__ inline uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// OCP e4m3fn byte -> binary32 (1-4-3, bias 7, no inf, S.1111.111 = NaN)
__device__ inline float e4m3_to_f32(uint32_t q) {
  uint32_t mag = q & 0x7fu;
  uint32_t sign = (q & 0x80u) << 24;
  uint32_t bits;
  if (mag == 0x7fu) bits = 0x7fc00000u;
  else if (mag >= 8u) bits = (mag << 20) + (120u << 23);
  else bits = __float_as_uint((float)mag * 0x1p-9f);
  return __uint_as_float(bits | sign);
}

// binary32 -> OCP e4m3fn byte, round to nearest even, saturating at +-448
// (NaN -> 0x7f).  Normal results round the 23-bit significand to 3 bits with an
// integer add so that a carry moves into the exponent; results below 2^-6 are
// multiples of 2^-9.
__device__ inline uint32_t f32_to_e4m3(float f) {
  uint32_t u = __float_as_uint(f);
  uint32_t sign = (u >> 24) & 0x80u;
  uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return sign | 0x7fu;      // NaN
  if (a >= 0x43e00000u) return sign | 0x7eu;     // |f| >= 448: saturate
  uint32_t code;
  if (a < 0x3c800000u) {                         // |f| < 2^-6: subnormal range
    float scaled = __uint_as_float(a) * 512.0f;  // exact; in [0, 8)
    code = (uint32_t)__float2int_rn(scaled);     // ties to even; 8 is the smallest normal
  } else {
    uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u);
    code = (r >> 20) - ((127u - 7u) << 3);
    if (code > 0x7eu) code = 0x7eu;              // 448 < |f| rounded past the top
  }
  return sign | code;
}

// ---------------------------------------------------------------------------
// pack with quantisation fused in (a data-path variant the paper's Sec. 4.1
// leaves to prior work): x is bf16, the receive rows are e4m3 codes plus one
// fp32 scale per `group` channels.  Per token and group: scale = max|x| / 448
// (1 if the group is all zero), code = e4m3(x / scale).  One wavefront per
// token; a lane owns 16 consecutive channels (32 bytes in, 16 bytes out), so
// the lanes of a group are neighbours and the group maximum is a few
// xor-shuffles.  The token is quantised once and stored to its k rows.
// ---------------------------------------------------------------------------
constexpr int kQuantVecs = 7;  // 16-channel vectors per lane per pass (7 * 64 * 16 = 7168)

__global__ __launch_bounds__(64) void k_pack_quant(const u32x4* __restrict__ x,
                                                   u32x4* __restrict__ recv_q,
                                                   float* __restrict__ recv_scale,
                                                   const int32_t* __restrict__ row_of, int k,
                                                   int out_vecs, int lanes_per_group,
                                                   int groups) {
  extern __shared__ float s_scale[];  // [groups] scales of this token
  const int t = blockIdx.x;
  const int lane = threadIdx.x;
  const int32_t* rows = row_of + (int64_t)t * k;
  const u32x4* src = x + (int64_t)t * out_vecs * 2;
  for (int w0 = 0; w0 < out_vecs; w0 += 64 * kQuantVecs) {
    u32x4 in[kQuantVecs][2];
#pragma unroll
    for (int u = 0; u < kQuantVecs; ++u) {
      int w = w0 + u * 64 + lane;
      if (w < out_vecs) {
        in[u][0] = __builtin_nontemporal_load(&src[2 * w]);
        in[u][1] = __builtin_nontemporal_load(&src[2 * w + 1]);
      } else {
        in[u][0] = in[u][1] = u32x4{0, 0, 0, 0};
      }
    }
    u32x4 q[kQuantVecs];
#pragma unroll
    for (int u = 0; u < kQuantVecs; ++u) {
      int w = w0 + u * 64 + lane;
      float v[16];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint32_t d = in[u][i >> 2][i & 3];
        v[2 * i] = bf16_lo(d);
        v[2 * i + 1] = bf16_hi(d);
      }
      float amax = 0.0f;
#pragma unroll
      for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
      for (int m = 1; m < lanes_per_group; m <<= 1) amax = fmaxf(amax, __shfl_xor(amax, m, 64));
      float scale = amax / 448.0f;
      if (scale == 0.0f) scale = 1.0f;
      if (w < out_vecs && (lane & (lanes_per_group - 1)) == 0) s_scale[w / lanes_per_group] = scale;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        q[u][i] = f32_to_e4m3(v[4 * i] / scale) | (f32_to_e4m3(v[4 * i + 1] / scale) << 8) |
                  (f32_to_e4m3(v[4 * i + 2] / scale) << 16) |
                  (f32_to_e4m3(v[4 * i + 3] / scale) << 24);
    }
    for (int j = 0; j < k; ++j) {
      int row = rows[j];
      if (row < 0) continue;
      u32x4* dst = recv_q + (int64_t)row * out_vecs;
#pragma unroll
      for (int u = 0; u < kQuantVecs; ++u) {
        int w = w0 + u * 64 + lane;
        if (w < out_vecs) store_through(&dst[w], q[u]);
      }
    }
  }
  __syncthreads();
  for (int g = lane; g < groups; g += 64) {
    float sc = s_scale[g];
    for (int j = 0; j < k; ++j) {
      int row = rows[j];
      if (row >= 0) recv_scale[(int64_t)row * groups + g] = sc;
    }
  }
}

hipError_t launch_pack_quant(eep_ctx* c, const void* x_bf16, void* recv_q, float* recv_scale, int T,
                             hipStream_t st) {
  if (T == 0) return hipSuccess;
  int out_vecs = c->H / 16;
  int groups = c->H / c->cfg.scale_group;
  hipLaunchKernelGGL(k_pack_quant, dim3(T), dim3(64), sizeof(float) * groups, st,
                     (const u32x4*)x_bf16, (u32x4*)recv_q, recv_scale, c->row_of, c->k, out_vecs,
                     c->cfg.scale_group / 16, groups);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// combine: out[t] = sum_j w[t,j] * y[row_of[t,j]], fp32 fused multiply-add chain
// in ascending j.  A lane owns 16-byte columns of the row and issues the k row
// loads of its columns back to back.
// ---------------------------------------------------------------------------
template <bool Y_BF16>
struct YVec {
  static constexpr int kElems = Y_BF16 ? 8 : 4;
};

template <bool Y_BF16>
__device__ inline void accumulate(float (&acc)[YVec<Y_BF16>::kElems], u32x4 v, float w) {
  if constexpr (Y_BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = fmaf(w, bf16_lo(v[i]), acc[2 * i]);
      acc[2 * i + 1] = fmaf(w, bf16_hi(v[i]), acc[2 * i + 1]);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(w, __uint_as_float(v[i]), acc[i]);
  }
}

template <bool Y_BF16, bool OUT_BF16>
__device__ inline void store_out(void* out_row, int v, const float (&acc)[YVec<Y_BF16>::kElems]) {
  if constexpr (Y_BF16 && OUT_BF16) {
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = pack_bf16x2(acc[2 * i], acc[2 * i + 1]);
    __builtin_nontemporal_store(o, (u32x4*)out_row + v);
  } else if constexpr (Y_BF16 && !OUT_BF16) {
    f32x4 a = {acc[0], acc[1], acc[2], acc[3]}, b = {acc[4], acc[5], acc[6], acc[7]};
    __builtin_nontemporal_store(a, (f32x4*)out_row + 2 * v);
    __builtin_nontemporal_store(b, (f32x4*)out_row + 2 * v + 1);
  } else if constexpr (!Y_BF16 && OUT_BF16) {
    u32x2 o = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3])};
    __builtin_nontemporal_store(o, (u32x2*)out_row + v);
  } else {
    f32x4 a = {acc[0], acc[1], acc[2], acc[3]};
    __builtin_nontemporal_store(a, (f32x4*)out_row + v);
  }
}

// ---------------------------------------------------------------------------
// GPU-side failure detection inside combine (paper Sec. 3.4; Sec. 4.1, the
// paragraph on failure detection from the GPU side): before a wavefront reduces
// a token's rows it looks at the signal word of every rank those rows come
// from.  The expert stage stores the step's epoch there once the rank's outputs
// are in place.  A word that does not show the epoch sends the wavefront into
// the wait below; a rank that stays silent past the time-out is dropped by the
// kernel: its `active` entry is cleared, it is put on the report that the host
// reads after the kernel, the membership version is bumped, and the pairs
// routed to it contribute nothing (their row_of entry becomes -1).
// In a healthy step the first wavefront of the launch finds every expected
// signal in place and publishes that in one word (round_ok = epoch); the others
// read that word (one agent-scope load, issued beside the row loads) and go
// straight on.  Wavefronts that run before the word is published, and all
// wavefronts of a step in which a signal is missing, look at the signals of
// their own rows' ranks.  Those first looks use plain loads: the signal words
// were written by an earlier launch of the same stream.  The wait itself uses agent-scope loads,
// so that a rank dropped by a wavefront on another XCD is seen at once and all
// waiting wavefronts together spend about one time-out, not one each.  Every
// wait is bounded by the wall clock and by a poll count.
// ---------------------------------------------------------------------------
struct DetectArgs {
  const int32_t* slot_of;     // [T, k]
  int32_t* row_of;            // [T, k], entries of dropped pairs are set to -1
  const int32_t* signal;      // [R] epoch of the last step whose outputs arrived
  const int32_t* step_epoch;  // current step
  int32_t* active;            // [R]
  int32_t* report;            // [R]
  int32_t* mem_version;
  const int32_t* rank_count;  // [R] rows each rank holds in this step
  int32_t* round_ok;          // epoch of the last step in which every expected signal was there
  int R, S;
  long long timeout_ticks, max_polls;
};

// pending: bit j set = pair j's rank has not signalled.  Returns the bits of the pairs whose
// rank was dropped (by this wavefront or by another).  Uniform across the wavefront.
__device__ __forceinline__ uint32_t await_late_ranks(const DetectArgs& d, int64_t pair0, uint32_t pending,
                                                  int epoch) {
  uint32_t failed = 0;
  const long long t0 = wall_clock64();
  long long polls = 0;
  while (pending != 0) {
    for (uint32_t m = pending; m != 0; m &= m - 1) {
      const int j = __ffs(m) - 1;
      const int rank = d.slot_of[pair0 + j] / d.S;
      if (__hip_atomic_load(&d.signal[rank], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == epoch) {
        pending &= ~(1u << j);  // arrived late
      } else if (__hip_atomic_load(&d.active[rank], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
        pending &= ~(1u << j);  // dropped meanwhile
        failed |= 1u << j;
      }
    }
    if (pending == 0) break;
    if (++polls > d.max_polls || wall_clock64() - t0 > d.timeout_ticks) {
      // time-out: drop every rank still awaited; the first wavefront to clear the entry
      // also reports it
      for (uint32_t m = pending; m != 0; m &= m - 1) {
        const int j = __ffs(m) - 1;
        const int rank = d.slot_of[pair0 + j] / d.S;
        if (threadIdx.x == 0 &&
            __hip_atomic_exchange(&d.active[rank], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
          __hip_atomic_store(&d.report[rank], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_fetch_add(d.mem_version, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        failed |= 1u << j;
      }
      break;
    }
    __builtin_amdgcn_s_sleep(8);
  }
  if (threadIdx.x == 0)
    for (uint32_t m = failed; m != 0; m &= m - 1) d.row_of[pair0 + __ffs(m) - 1] = -1;
  return failed;
}

// First look (plain loads) at the signals of the ranks a token's rows come from; the wait only
// if one is missing.  Returns the bits of the pairs whose rank was dropped.
__device__ __forceinline__ uint32_t ranks_dropped(const DetectArgs& d, int64_t pair0, int k,
                                                  const int32_t* rows, int epoch) {
  uint32_t pending = 0;
  for (int j = 0; j < k; ++j) {
    const int p = d.slot_of[pair0 + j];
    if (p >= 0 && rows[j] >= 0 && d.signal[p / d.S] != epoch) pending |= 1u << j;
  }
  return pending != 0 ? await_late_ranks(d, pair0, pending, epoch) : 0u;
}

// One wavefront per (token, part): a part is kCombineCols * 64 16-byte columns
// of the row (2 KiB of each source row at the decode shape), so a lane has
// kCombineCols * k independent loads in flight.  Small single-wavefront
// workgroups measured ~10 % faster than one workgroup per token.
constexpr int kCombineCols = 2;

// DETECT: the wait for the ranks' signals is part of the kernel (DetectArgs above); row_of
// is then not read-only, because dropped pairs are struck from it.
template <bool Y_BF16, bool OUT_BF16, int K, bool DETECT>
__global__ __launch_bounds__(64) void k_combine(const u32x4* __restrict__ y,
                                                const float* __restrict__ topk_w,
                                                const int32_t* row_of, void* __restrict__ out,
                                                int k, int row_vecs, int parts,
                                                int64_t out_row_bytes, DetectArgs det) {
  constexpr int NE = YVec<Y_BF16>::kElems;
  const int t = blockIdx.x / parts;
  const int part = blockIdx.x - t * parts;
  const int v0 = part * (64 * kCombineCols) + threadIdx.x;
  const int32_t* rows = row_of + (int64_t)t * k;
  const float* ws = topk_w + (int64_t)t * k;
  void* out_row = (char*)out + (int64_t)t * out_row_bytes;

  int round_flag = 0, epoch = 0;
  if constexpr (DETECT) {
    epoch = *det.step_epoch;
    if (blockIdx.x == 0) {
      // the first wavefront looks at every rank that holds rows of this step
      bool ok = true;
      for (int r = threadIdx.x; r < det.R; r += 64)
        ok &= det.active[r] == 0 || det.rank_count[r] == 0 || det.signal[r] == epoch;
      if (__all(ok) && threadIdx.x == 0)
        __hip_atomic_store(det.round_ok, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    round_flag = __hip_atomic_load(det.round_ok, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  if constexpr (K > 0) {
    // fast path: compile-time k and every pair routed -> no branch between loads
    int r[K];
    float w[K];
    bool all = true;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      r[j] = rows[j];
      w[j] = ws[j];
      all &= (r[j] >= 0);
    }
    if (all) {
      u32x4 d[kCombineCols][K];
#pragma unroll
      for (int q = 0; q < kCombineCols; ++q) {
        int v = v0 + q * 64;
        if (v < row_vecs) {
#pragma unroll
          for (int j = 0; j < K; ++j)
            d[q][j] = __builtin_nontemporal_load(&y[(int64_t)r[j] * row_vecs + v]);
        }
      }
      // the look at the ranks' signals comes after the row loads have been issued, so that
      // its two dependent table lookups overlap with them; rows of a rank that turns out to
      // be dropped are loaded and not used
      uint32_t dropped = 0;
      if constexpr (DETECT)
        if (round_flag != epoch) dropped = ranks_dropped(det, (int64_t)t * k, k, rows, epoch);
#pragma unroll
      for (int q = 0; q < kCombineCols; ++q) {
        int v = v0 + q * 64;
        if (v < row_vecs) {
          float acc[NE];
#pragma unroll
          for (int i = 0; i < NE; ++i) acc[i] = 0.0f;
#pragma unroll
          for (int j = 0; j < K; ++j)
            if (!DETECT || !((dropped >> j) & 1u)) accumulate<Y_BF16>(acc, d[q][j], w[j]);
          store_out<Y_BF16, OUT_BF16>(out_row, v, acc);
        }
      }
      return;
    }
  }
  uint32_t dropped = 0;  // bit j: pair j's rank was dropped in this step
  if constexpr (DETECT)
    if (round_flag != epoch) dropped = ranks_dropped(det, (int64_t)t * k, k, rows, epoch);
  for (int q = 0; q < kCombineCols; ++q) {
    int v = v0 + q * 64;
    if (v >= row_vecs) break;
    float acc[NE];
#pragma unroll
    for (int i = 0; i < NE; ++i) acc[i] = 0.0f;
    for (int j = 0; j < k; ++j) {
      int row = rows[j];
      if (row < 0 || ((dropped >> j) & 1u)) continue;
      u32x4 d = __builtin_nontemporal_load(&y[(int64_t)row * row_vecs + v]);
      accumulate<Y_BF16>(acc, d, ws[j]);
    }
    store_out<Y_BF16, OUT_BF16>(out_row, v, acc);
  }
}

template <bool Y_BF16, bool OUT_BF16>
static hipError_t launch_combine_t(eep_ctx* c, const void* y, const float* w, void* out, int T,
                                   hipStream_t st) {
  int row_vecs = (int)(c->y_row_bytes / 16);
  int parts = (row_vecs + 64 * kCombineCols - 1) / (64 * kCombineCols);
  if ((int64_t)T * parts > 0x7fffffffLL) return hipErrorInvalidValue;  // grid size limit
  dim3 grid((unsigned)((int64_t)T * parts)), block(64);
  DetectArgs det = {};
  if (c->detect_timeout_ticks > 0) {
    // the wait for the ranks' signals runs inside the kernel
    det.slot_of = c->slot_of; det.row_of = c->row_of; det.signal = c->signal;
    det.step_epoch = c->step_epoch; det.active = c->active; det.report = c->report;
    det.mem_version = c->mem->mem_version; det.S = c->S; det.R = c->R;
    det.rank_count = c->rank_count; det.round_ok = c->round_ok;
    det.timeout_ticks = c->detect_timeout_ticks;
    det.max_polls = c->detect_timeout_ticks * 8 + 1024;
    if (c->k == 8)
      hipLaunchKernelGGL((k_combine<Y_BF16, OUT_BF16, 8, true>), grid, block, 0, st,
                         (const u32x4*)y, w, c->row_of, out, c->k, row_vecs, parts,
                         c->out_row_bytes, det);
    else
      hipLaunchKernelGGL((k_combine<Y_BF16, OUT_BF16, 0, true>), grid, block, 0, st,
                         (const u32x4*)y, w, c->row_of, out, c->k, row_vecs, parts,
                         c->out_row_bytes, det);
    return hipGetLastError();
  }
  if (c->k == 8)
    hipLaunchKernelGGL((k_combine<Y_BF16, OUT_BF16, 8, false>), grid, block, 0, st,
                       (const u32x4*)y, w, c->row_of, out, c->k, row_vecs, parts,
                       c->out_row_bytes, det);
  else
    hipLaunchKernelGGL((k_combine<Y_BF16, OUT_BF16, 0, false>), grid, block, 0, st,
                       (const u32x4*)y, w, c->row_of, out, c->k, row_vecs, parts,
                       c->out_row_bytes, det);
  return hipGetLastError();
}

hipError_t launch_combine(eep_ctx* c, const void* y, const float* w, void* out, int T,
                          hipStream_t st) {
  if (T == 0) return hipSuccess;
  bool yb = c->cfg.y_dtype == EEP_BF16, ob = c->cfg.out_dtype == EEP_BF16;
  if (yb && ob) return launch_combine_t<true, true>(c, y, w, out, T, st);
  if (yb && !ob) return launch_combine_t<true, false>(c, y, w, out, T, st);
  if (!yb && ob) return launch_combine_t<false, true>(c, y, w, out, T, st);
  return launch_combine_t<false, false>(c, y, w, out, T, st);
}

// ---------------------------------------------------------------------------
// expert stand-ins (outside the measured path): one workgroup per receive row,
// rows >= N (read from device memory) are skipped.  Same streaming access
// policy as pack and combine: read-once loads are non-temporal, stores write
// through.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_stub_copy(const u32x4* __restrict__ recv,
                                                   u32x4* __restrict__ y,
                                                   const int32_t* __restrict__ status,
                                                   int row_vecs) {
  const int row = blockIdx.x;
  if (row >= status[0]) return;
  for (int v = threadIdx.x; v < row_vecs; v += blockDim.x)
    store_through(&y[(int64_t)row * row_vecs + v],
                  __builtin_nontemporal_load(&recv[(int64_t)row * row_vecs + v]));
}

template <bool BF16>
__global__ __launch_bounds__(256) void k_stub_scale(
    const u32x4* __restrict__ recv, u32x4* __restrict__ y, const int32_t* __restrict__ status,
    const int32_t* __restrict__ src_of, const int32_t* __restrict__ slot_of,
    const int32_t* __restrict__ p2l, const float* __restrict__ expert_scale, int row_vecs) {
  const int row = blockIdx.x;
  if (row >= status[0]) return;
  const int e = p2l[slot_of[src_of[row]]];
  const float s = e >= 0 ? expert_scale[e] : 0.0f;
  for (int v = threadIdx.x; v < row_vecs; v += blockDim.x) {
    u32x4 d = __builtin_nontemporal_load(&recv[(int64_t)row * row_vecs + v]);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (BF16) o[i] = pack_bf16x2(s * bf16_lo(d[i]), s * bf16_hi(d[i]));
      else o[i] = __float_as_uint(s * __uint_as_float(d[i]));
    }
    store_through(&y[(int64_t)row * row_vecs + v], o);
  }
}

// 16 fp8 codes in, 16 bf16 out per thread step; all 16 share one scale
// (group is a multiple of 16).
__global__ __launch_bounds__(256) void k_stub_dequant(const u32x4* __restrict__ q,
                                                      const float* __restrict__ scale,
                                                      u32x4* __restrict__ y,
                                                      const int32_t* __restrict__ status,
                                                      int row_vecs, int group, int groups_per_row) {
  const int row = blockIdx.x;
  if (row >= status[0]) return;
  for (int v = threadIdx.x; v < row_vecs; v += blockDim.x) {
    u32x4 d = __builtin_nontemporal_load(&q[(int64_t)row * row_vecs + v]);
    float sc = scale[(int64_t)row * groups_per_row + (v * 16) / group];
    u32x4 o[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float f0 = sc * e4m3_to_f32(d[i] & 0xffu);
      float f1 = sc * e4m3_to_f32((d[i] >> 8) & 0xffu);
      float f2 = sc * e4m3_to_f32((d[i] >> 16) & 0xffu);
      float f3 = sc * e4m3_to_f32(d[i] >> 24);
      o[i >> 1][(i & 1) * 2] = pack_bf16x2(f0, f1);
      o[i >> 1][(i & 1) * 2 + 1] = pack_bf16x2(f2, f3);
    }
    store_through(&y[((int64_t)row * row_vecs + v) * 2], o[0]);
    store_through(&y[((int64_t)row * row_vecs + v) * 2 + 1], o[1]);
  }
}

hipError_t launch_stub(eep_ctx* c, int kind, const void* recv_x, const float* recv_scale,
                       const float* expert_scale, void* y, int T, hipStream_t st) {
  int64_t rows = (int64_t)T * c->k;
  if (rows == 0) return hipSuccess;
  int row_vecs = (int)(c->x_row_bytes / 16);
  dim3 grid((unsigned)rows), block(256);
  if (kind == EEP_STUB_IDENTITY) {
    hipLaunchKernelGGL(k_stub_copy, grid, block, 0, st, (const u32x4*)recv_x, (u32x4*)y,
                       c->status, row_vecs);
  } else if (kind == EEP_STUB_SCALE) {
    if (c->cfg.x_dtype == EEP_BF16)
      hipLaunchKernelGGL(k_stub_scale<true>, grid, block, 0, st, (const u32x4*)recv_x, (u32x4*)y,
                         c->status, c->src_of, c->slot_of, c->p2l, expert_scale, row_vecs);
    else
      hipLaunchKernelGGL(k_stub_scale<false>, grid, block, 0, st, (const u32x4*)recv_x,
                         (u32x4*)y, c->status, c->src_of, c->slot_of, c->p2l, expert_scale,
                         row_vecs);
  } else {
    hipLaunchKernelGGL(k_stub_dequant, grid, block, 0, st, (const u32x4*)recv_x, recv_scale,
                       (u32x4*)y, c->status, row_vecs, c->cfg.scale_group,
                       c->H / c->cfg.scale_group);
  }
  return hipGetLastError();
}

}  // namespace eep
