// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "heterospec.h"

namespace hs {

// Records the message for hs_last_error() and returns `st`.
hs_status fail(hs_status st, const char* fmt, ...);
void clear_error();

inline hs_status launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(HS_ERR_RUNTIME, "%s: %s", what, hipGetErrorString(e));
  return HS_OK;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of the caller's workspace.
struct Carver {
  char* base;
  size_t used = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  template <typename T>
  T* take(size_t n) {
    T* r = reinterpret_cast<T*>(base + used);
    used += align_up(n * sizeof(T), 256);
    return r;
  }
};

// Row scan shared by hs_draft_entropy_topk and hs_verify_accept (defined in entropy_topk.hip).
size_t row_topk_workspace(int R, int V, int K);
// `slices` (may be NULL): when the rows had to be cut into slices, the merge launch is left to the
// caller, who receives the per-slice results instead: entry (row * count + slice) * K + k of
// val / idx is the slice's k-th best pair (an unused entry has index INT_MAX).  count == 1 means
// the outputs were written in full.
// `row_active` (device, may be NULL): one byte per row; a row whose byte is 0 is neither read nor
// written.  `row_index` (device, may be NULL): result row r is computed from logits row
// row_index[r]; a negative entry leaves row r's results as they are.  `logits2` (may be NULL):
// rows rows1, rows1 + 1, ... are rows 0, 1, ... of this second array (same row stride).
// `prepared`: the workspace was cleared by hs_workspace_prepare and has since been used by completed
// calls of this kind only; rows cut into slices are then merged by the scan's own launch.
struct ScanSlices {
  const float* val;
  const int32_t* idx;
  int count;
  bool pairs_only = false;  // in: the caller wants the slices' best pairs only, no softmax statistics
};
hs_status row_topk_launch(const float* logits, int64_t row_stride, int R, int V, int K, float temperature,
                          int32_t* topk_idx, float* topk_logp, float* ent_topk, float* ent_full, float* lse,
                          void* workspace, hipStream_t stream, ScanSlices* slices = nullptr,
                          const uint8_t* row_active = nullptr, const int32_t* row_index = nullptr,
                          const float* logits2 = nullptr, int rows1 = 0, bool prepared = false);

#define HS_REQUIRE(cond, st, ...) \
  do {                            \
    if (!(cond)) return ::hs::fail(st, __VA_ARGS__); \
  } while (0)

// ------------------------------------------------------------------ device helpers
#define HS_INF __builtin_huge_valf()

// Strict total order on (value, index): larger value first, then lower index.
__device__ __forceinline__ bool better(float av, int ai, float bv, int bi) {
  return av > bv || (av == bv && ai < bi);
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Running softmax statistics of a set of raw logits x, with y = x * inv_t:
//   m  = max x (raw units, so comparisons stay exact);
//   s1 = sum exp(y - y_max) over all elements but ONE instance of the max;
//   t  = sum exp(y - y_max) (y - y_max)   (every term <= 0).
// Keeping the max's own unit out of s1 keeps entropy and lse accurate for nearly one-hot rows:
//   lse = m * inv_t + log1p(s1),  entropy = log1p(s1) - t / (1 + s1).
struct Stats {
  float m, s1, t;
};

__device__ __forceinline__ Stats stats_empty() { return Stats{-HS_INF, 0.f, 0.f}; }

__device__ __forceinline__ Stats stats_merge(Stats a, Stats b, float inv_t) {
  if (b.m == -HS_INF) return a;
  if (a.m == -HS_INF) return b;
  if (b.m > a.m) {
    Stats x = a;
    a = b;
    b = x;
  }
  float d = (b.m - a.m) * inv_t;  // <= 0
  float e = exp2_fast(d * 1.4426950408889634f);
  float w = 1.f + b.s1;
  return Stats{a.m, a.s1 + e * w, a.t + e * (b.t + d * w)};
}

// Reductions over the 64 lanes of a wave with DPP moves (no LDS traffic): partial results travel
// right inside each row of 16 lanes, then from row to row; lane 63 ends up with the total, which
// is broadcast.  `idle` is what a lane without a source takes (the identity of the operation).
template <typename Op>
__device__ __forceinline__ float wave_reduce_dpp(float x, float idle, Op op) {
  const int id = __builtin_bit_cast(int, idle);
#define HS_DPP_STEP(ctrl, rows, banks)                                                                        \
  x = op(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(id, __builtin_bit_cast(int, x), ctrl, rows, \
                                                                  banks, false)))
  HS_DPP_STEP(0x111, 0xf, 0xf);  // row_shr:1
  HS_DPP_STEP(0x112, 0xf, 0xf);  // row_shr:2
  HS_DPP_STEP(0x114, 0xf, 0xe);  // row_shr:4
  HS_DPP_STEP(0x118, 0xf, 0xc);  // row_shr:8
  HS_DPP_STEP(0x142, 0xa, 0xf);  // row_bcast:15
  HS_DPP_STEP(0x143, 0xc, 0xf);  // row_bcast:31
#undef HS_DPP_STEP
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
// Inclusive prefix sums over the lanes of a wave, same DPP steps: lane l receives x_0 + ... + x_l.
__device__ __forceinline__ int wave_prefix_sum(int x) {
#define HS_DPP_STEP(ctrl, rows, banks) x += __builtin_amdgcn_update_dpp(0, x, ctrl, rows, banks, false)
  HS_DPP_STEP(0x111, 0xf, 0xf);  // row_shr:1
  HS_DPP_STEP(0x112, 0xf, 0xf);  // row_shr:2
  HS_DPP_STEP(0x114, 0xf, 0xe);  // row_shr:4
  HS_DPP_STEP(0x118, 0xf, 0xc);  // row_shr:8
  HS_DPP_STEP(0x142, 0xa, 0xf);  // row_bcast:15
  HS_DPP_STEP(0x143, 0xc, 0xf);  // row_bcast:31
#undef HS_DPP_STEP
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
  return wave_reduce_dpp(x, -HS_INF, [](float a, float b) { return fmaxf(a, b); });
}
__device__ __forceinline__ float wave_sum(float x) {
  return wave_reduce_dpp(x, 0.f, [](float a, float b) { return a + b; });
}

__device__ __forceinline__ Stats stats_shfl_xor(Stats a, int mask) {
  return Stats{__shfl_xor(a.m, mask), __shfl_xor(a.s1, mask), __shfl_xor(a.t, mask)};
}

__device__ __forceinline__ Stats stats_wave_reduce(Stats a, float inv_t) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) a = stats_merge(a, stats_shfl_xor(a, off), inv_t);
  return a;
}

}  // namespace hs
