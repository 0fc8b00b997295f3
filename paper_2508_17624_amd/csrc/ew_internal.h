// Internal helpers shared by the translation units of libexpertweave (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "expertweave.h"

#include "ffn_ws_plan.h"

namespace ew {

// Records a printf-style message for ew_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline int hip_fail(hipError_t e, const char* what) {
  return fail(e == hipErrorOutOfMemory ? EW_ERR_OOM : EW_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define EW_HIP(call)                                    \
  do {                                                  \
    hipError_t _e = (call);                             \
    if (_e != hipSuccess) return ::ew::hip_fail(_e, #call); \
  } while (0)

// Checks the launch that was just enqueued.
#define EW_LAUNCH_CHECK(name)                                   \
  do {                                                          \
    hipError_t _e = hipGetLastError();                          \
    if (_e != hipSuccess) return ::ew::hip_fail(_e, "launch " name); \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int ilog2_ceil(int v) {  // smallest b with (1<<b) >= v, at least 1
  int b = 1;
  while ((1 << b) < v) ++b;
  return b;
}


// ffn_gemm.hip: LDS-tiled grouped GEMM path of moe_grouped_ffn (bf16, many rows per slot).
size_t ffn_gemm_plan_ints(int rows, int P);
int launch_ffn_gemm(const void* x, int rows, int k, int H, int I, int P, const int32_t* counts, const int32_t* offsets,
                    const int32_t* por, const void* w13, const void* w2, void* act, void* y, int32_t* plan, hipStream_t st);


// ffn_ws.hip: weight-stationary streaming path of moe_grouped_ffn (bf16; weights and gathered token
// rows both reach LDS by LDS-direct loads, persistent workgroups pull items from per-XCD work
// lists).  nf = 32-token fragments per row chunk (1, 2, 4 or 8).
int ffn_ws_frags(int max_rows_per_slot, int rows, int slots, int nf_override);
size_t ffn_ws_plan_ints(int rows, int P, int nf);
// Plan shape of a call with `rows` rows in all and `slots` slots (shared experts included).
// merge: let the two products share a launch where the shape allows it.
WsPlanShape ffn_ws_plan_shape(int rows, int slots, int nf, int chunk_frags, bool merge);
// The plan kernel alone (what launch_ffn_ws runs first unless plan_ready).
int launch_ffn_ws_plan(const int32_t* counts, const int32_t* offsets, int P, int S, int T, int rows_routed, const WsPlanShape& sh,
                       int32_t* plan, hipStream_t st);
// S > 0: slots P .. P+S-1 are shared experts (weights w13_sh / w2_sh) that every one of the rows_routed / k tokens
// visits; their rows follow the routed ones in act and y, and plan must be sized for all rows and P + S slots.
int launch_ffn_ws(const void* x, int rows_routed, int k, int H, int I, int P, int S, const WsPlanShape& sh, bool plan_ready,
                  const int32_t* counts, const int32_t* offsets, const int32_t* por, const void* w13, const void* w2,
                  const void* w13_sh, const void* w2_sh, void* act, void* y, int32_t* plan, int wait_ticks, hipStream_t st);

// Whether moe_grouped_ffn / moe_grouped_ffn_with_shared with these dimensions runs the weight-stationary kernel, and
// if so with which plan shape (defined beside the tuning state it depends on).
bool ffn_ws_shape_of_call(int dtype, int T, int k, int H, int I, int P, int S, WsPlanShape* sh);

}  // namespace ew
