// Internal helpers shared by the HIP translation units of libsymi (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <vector>

#include "symi.h"

namespace symi {

void set_error(const char* fmt, ...);
int check_cfg(const symi_cfg* cfg, const char* who);

// Kernel ids for the optional event timing (symi_timing_*).
enum KernelId {
  K_FILL = 0, K_ROUTE, K_ROUTE_BWD, K_PLACE, K_CHUNK_COUNT, K_CHUNK_SCAN, K_CHUNK_RANK, K_GATHER,
  K_TILE_MAP, K_GEMM_FWD1, K_GEMM_FWD2, K_GEMM_BWD_DH, K_GEMM_BWD_DX, K_GEMM_WGRAD2, K_GEMM_WGRAD1,
  K_COMBINE, K_COMBINE_BWD, K_DISPATCH_BWD, K_ADAM, K_REPLICA_AR, K_ROUTER_FWD, K_ROUTER_DX, K_ROUTER_DW, K_SLICE_SUM, K_COUNT
};
struct TimedLaunch { int kid; hipEvent_t a, b; };

#define SYMI_REQUIRE(cond, who, msg)                      \
  do {                                                    \
    if (!(cond)) {                                        \
      symi::set_error("%s: %s", who, msg);                \
      return SYMI_EINVAL;                                 \
    }                                                     \
  } while (0)

#define SYMI_LAUNCH_CHECK(who)                                            \
  do {                                                                    \
    hipError_t e_ = hipGetLastError();                                    \
    if (e_ != hipSuccess) {                                               \
      symi::set_error("%s: launch failed: %s", who, hipGetErrorString(e_)); \
      return SYMI_EHIP;                                                   \
    }                                                                     \
  } while (0)

// Every device call starts with this: checks the context, makes `cfg` its configuration.
#define SYMI_ENTER(ctx, who)                               \
  if (int rc_enter_ = symi::enter(ctx, who)) return rc_enter_; \
  const symi_cfg* const cfg = &(ctx)->cfg

static inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

// bf16 <-> fp32 on raw 16-bit patterns.  Round to nearest, ties to even; NaN kept quiet.
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// two values at once: the gfx950 packed conversion (same rounding; NaNs come out canonical)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Workspace layout (byte offsets inside the caller's `ws`), one place for all users.
struct WsLayout {
  size_t blk_counts;   // dispatch: [nblk][E] i32 per-block class counts, then bases
  size_t class_tab;    // capacity-limited dispatch: per class {offset, kept offset, capacity}
  size_t tile_map;     // expert fwd/bwd: m-tile table, see gemm.hip
  size_t class_order;  // expert bwd: classes by decreasing row count
  size_t duv;          // expert bwd: dUV [A,2f] in the activation dtype
  size_t split_part;   // expert fwd/bwd: partial tiles of sliced reductions, see gemm.hip
  size_t router_partial;  // router bwd (bf16): partial weight gradients [chunks,E,d] f32
  size_t router_bias_partial;  // router bwd: partial bias gradients [chunks,E] f32
  size_t total;
};
WsLayout ws_layout(const symi_cfg* cfg);

constexpr int DISPATCH_CHUNK = 1024;  // assignments ranked by one workgroup
constexpr int GEMM_BM = 256;          // rows of one m-tile in the tile map
// Sliced reductions (gemm.hip): at most SPLIT_CUS partial tiles of 256 x 256 fp32 = 256 KB each.
constexpr int SPLIT_CUS = 256;        // compute units the slicing fills (at most)
constexpr size_t SPLIT_TILE_BYTES = 256 * 256 * sizeof(float);

}  // namespace symi

// The opaque context of include/symi.h: the validated configuration plus everything the
// library owns for it.  Created and destroyed by symi_create / symi_destroy; the hot calls
// only read it (the event list of the optional timing is the one thing they append to).
struct symi_ctx {
  uint32_t magic;
  symi_cfg cfg;
  unsigned flags;
  int device;            // the device that was current in symi_create
  int cus;               // its compute units
  symi::WsLayout L;      // layout of the caller's workspace for cfg
  bool overlap, slicing, timing;
  // helper stream of the expert backward with its fork / hand-over / join events
  // (nullptr when the flags or the shape rule it out)
  hipStream_t side;
  hipEvent_t fork, mid, join;
  // device address of the static scratch of symi_dispatch_noalloc on `device`
  void* static_scratch;
  mutable std::vector<symi::TimedLaunch> launches;
  mutable hipEvent_t open[symi::K_COUNT];
};

namespace symi {
constexpr uint32_t CTX_MAGIC = 0x53594d49u;   // "SYMI"
int enter(const symi_ctx* ctx, const char* who);
void timing_begin(const symi_ctx* ctx, int kid, hipStream_t st);
void timing_end(const symi_ctx* ctx, int kid, hipStream_t st);
int static_scratch_address(int device, void** out);   // dispatch.hip
void launch_fill_i32(const symi_ctx* ctx, int32_t* p, int n, int32_t val, hipStream_t st);
}  // namespace symi

// Brackets one kernel launch with events when the context was created with SYMI_CTX_TIMING.
#define SYMI_TIMED(ctx, kid, st, launch)                      \
  do {                                                        \
    if ((ctx)->timing) symi::timing_begin(ctx, kid, st);      \
    launch;                                                   \
    if ((ctx)->timing) symi::timing_end(ctx, kid, st);        \
  } while (0)
