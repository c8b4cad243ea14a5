// Host-side parts of libsymi: configuration checks, error text, workspace layout.
#include <stdarg.h>
#include <string.h>

#include <new>
#include <vector>

#include "common.h"

namespace symi {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int check_cfg(const symi_cfg* c, const char* who) {
  if (!c) {
    set_error("%s: cfg is NULL", who);
    return SYMI_EINVAL;
  }
#define BAD(cond, msg)                   \
  if (cond) {                            \
    set_error("%s: %s", who, msg);       \
    return SYMI_EINVAL;                  \
  }
  BAD(c->T < 0, "T < 0");
  BAD(c->E < 1 || c->E > 1024, "E outside [1, 1024]");
  BAD(c->k < 1 || c->k > c->E || c->k > 16, "k outside [1, min(E, 16)]");
  BAD(c->d < 8 || c->d % 8, "d must be a positive multiple of 8");
  BAD(c->f < 8 || c->f % 8, "f must be a positive multiple of 8");
  // Sec. 3.4: at least one instance per expert class, so the slot budget must cover E.
  BAD(c->S_tot < c->E, "S_tot < E: every class needs one slot");
  BAD(c->S_tot > 4096, "S_tot > 4096");
  BAD(c->N < 1, "N < 1");
  BAD(c->shard < 0 || c->shard >= c->N, "shard outside [0, N)");
  BAD(c->dtype != SYMI_F32 && c->dtype != SYMI_BF16, "dtype must be SYMI_F32 or SYMI_BF16");
  BAD(c->renorm != 0 && c->renorm != 1, "renorm must be 0 or 1");
  long long Pe = 3LL * c->d * c->f;
  BAD(Pe % c->N, "P_e = 3*d*f is not divisible by N");
  BAD((Pe / c->N) % 8, "P_e / N is not a multiple of 8");
  BAD((long long)c->T * c->k > 0x7fffffffLL / 2, "T*k too large for int32 indexing");
#undef BAD
#define UNSUPPORTED(cond, msg)           \
  if (cond) {                            \
    set_error("%s: %s", who, msg);       \
    return SYMI_EUNSUPPORTED;            \
  }
  // launch limits of the kernels: the m-tile index of the grouped GEMM (one per 64 rows in the
  // fp32 twin, plus the slices of a cut last round) and the router's 128-token tiles are grid.y
  // coordinates; the GEMM's per-lane element offsets inside a slot's weights are 32 bits
  const long long A = (long long)c->T * c->k;
  const long long mtiles = A / GEMM_BM + c->S_tot;
  UNSUPPORTED(c->dtype == SYMI_BF16 ? mtiles + 256 > 65535 : 4 * mtiles > 65535,
              "T*k/256 + S_tot (m-tiles of the grouped GEMM; four times that for fp32) exceeds the grid limit");
  UNSUPPORTED(((long long)c->T + 127) / 128 > 65535, "T/128 exceeds the grid limit of the router kernels");
  // the grouped GEMM addresses an operand tile with 32-bit per-lane byte offsets (8 KB of bias
  // included): a weight panel spans up to 2*f*d elements, 256 tile rows up to 256*max(d, 2f)
  UNSUPPORTED(2LL * c->f * c->d > (1LL << 31) - 8192, "2*f*d must not exceed 2^31 - 8192");
  UNSUPPORTED(c->d > (1 << 22) || c->f > (1 << 21), "d must not exceed 2^22 and f 2^21");
#undef UNSUPPORTED
  return SYMI_OK;
}

WsLayout ws_layout(const symi_cfg* c) {
  WsLayout L;
  const size_t A = (size_t)c->T * c->k;
  const size_t w = c->dtype == SYMI_BF16 ? 2 : 4;
  const size_t nblk = (A + DISPATCH_CHUNK - 1) / DISPATCH_CHUNK;
  const size_t mtiles = A / GEMM_BM + c->S_tot + 1;
  size_t off = 0;
  L.blk_counts = off;
  off += align_up((nblk + 1) * c->E * sizeof(int32_t), 256);
  L.class_tab = off;
  off += align_up((size_t)3 * c->E * sizeof(int32_t), 256);
  L.tile_map = off;
  off += align_up((4 + 4 * mtiles) * sizeof(int32_t), 256);
  L.class_order = off;
  off += align_up((size_t)c->E * sizeof(int32_t), 256);
  L.duv = off;
  off += align_up(A * 2 * c->f * w, 256);
  L.split_part = off;
  off += c->dtype == SYMI_BF16 ? (size_t)SPLIT_CUS * SPLIT_TILE_BYTES : 0;
  L.router_partial = off;
  off += align_up(((size_t)c->T + 511) / 512 * c->E * c->d * sizeof(float), 256);
  L.router_bias_partial = off;
  off += align_up(((size_t)c->T + 255) / 256 * c->E * sizeof(float), 256);
  L.total = off + 256;
  return L;
}

// ---- optional per-kernel event timing (contexts created with SYMI_CTX_TIMING; used by the
// benchmark)
static const char* const g_names[K_COUNT] = {
    "fill_i32", "route", "route_bwd", "place", "chunk_count", "chunk_scan", "chunk_rank",
    "gather_rows", "tile_map", "gemm_fwd1", "gemm_fwd2", "gemm_bwd_dh", "gemm_bwd_dx",
    "gemm_wgrad2", "gemm_wgrad1", "combine", "combine_bwd", "dispatch_bwd", "adam_to_replicas",
    "replica_allreduce", "router_fwd", "router_dx", "router_dw", "slice_sum"};

void timing_begin(const symi_ctx* ctx, int kid, hipStream_t st) {
  hipEvent_t e;
  if (hipEventCreate(&e) != hipSuccess) return;
  (void)hipEventRecord(e, st);
  ctx->open[kid] = e;
}
void timing_end(const symi_ctx* ctx, int kid, hipStream_t st) {
  hipEvent_t e;
  if (!ctx->open[kid] || hipEventCreate(&e) != hipSuccess) return;
  (void)hipEventRecord(e, st);
  ctx->launches.push_back({kid, ctx->open[kid], e});
  ctx->open[kid] = nullptr;
}

int enter(const symi_ctx* ctx, const char* who) {
  if (!ctx || ctx->magic != CTX_MAGIC) {
    set_error("%s: ctx is NULL or not a live context of symi_create", who);
    return SYMI_EINVAL;
  }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device) {
    (void)hipGetLastError();
    set_error("%s: the context was created on device %d, the current device is %d", who, ctx->device, dev);
    return SYMI_EINVAL;
  }
  return SYMI_OK;
}

// The expert backward runs its weight-gradient chain on a stream of its own while the products
// are only a few rounds of workgroups (gemm.hip); larger shapes fill the chip anyway.
static bool wants_side_stream(const symi_cfg* c, int cus) {
  const long long A = (long long)c->T * c->k;
  const long long max_mtiles = A / GEMM_BM + c->S_tot;
  return A > 0 && max_mtiles * cdiv(c->d, 256) < 8LL * cus;
}

static void release(symi_ctx* ctx) {
  for (auto& l : ctx->launches) {
    (void)hipEventDestroy(l.a);
    (void)hipEventDestroy(l.b);
  }
  ctx->launches.clear();
  for (auto& e : ctx->open)
    if (e) { (void)hipEventDestroy(e); e = nullptr; }
  if (ctx->fork) (void)hipEventDestroy(ctx->fork);
  if (ctx->mid) (void)hipEventDestroy(ctx->mid);
  if (ctx->join) (void)hipEventDestroy(ctx->join);
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  ctx->fork = ctx->mid = ctx->join = nullptr;
  ctx->side = nullptr;
}

}  // namespace symi

extern "C" {

int symi_create(const symi_cfg* cfg, unsigned flags, symi_ctx** out) {
  if (!out) {
    symi::set_error("symi_create: out is NULL");
    return SYMI_EINVAL;
  }
  *out = nullptr;
  if (int rc = symi::check_cfg(cfg, "symi_create")) return rc;
  if (flags & ~(unsigned)(SYMI_CTX_NO_OVERLAP | SYMI_CTX_NO_SLICING | SYMI_CTX_TIMING)) {
    symi::set_error("symi_create: unknown flag bits 0x%x", flags);
    return SYMI_EINVAL;
  }
  int dev = -1, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
    (void)hipGetLastError();
    symi::set_error("symi_create: no usable HIP device is current");
    return SYMI_EHIP;
  }
  symi_ctx* ctx = new (std::nothrow) symi_ctx();
  if (!ctx) {
    symi::set_error("symi_create: out of host memory");
    return SYMI_EHIP;
  }
  ctx->cfg = *cfg;
  ctx->flags = flags;
  ctx->device = dev;
  ctx->cus = cus;
  ctx->L = symi::ws_layout(cfg);
  ctx->overlap = !(flags & SYMI_CTX_NO_OVERLAP);
  ctx->slicing = !(flags & SYMI_CTX_NO_SLICING);
  ctx->timing = (flags & SYMI_CTX_TIMING) != 0;
  ctx->side = nullptr;
  ctx->fork = ctx->mid = ctx->join = nullptr;
  for (auto& e : ctx->open) e = nullptr;
  ctx->static_scratch = nullptr;
  if (int rc = symi::static_scratch_address(dev, &ctx->static_scratch)) {
    delete ctx;
    return rc;
  }
  if (ctx->overlap && symi::wants_side_stream(cfg, cus)) {
    // default priority, non-blocking with respect to the NULL stream
    const bool ok = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) == hipSuccess &&
                    hipEventCreateWithFlags(&ctx->fork, hipEventDisableTiming) == hipSuccess &&
                    hipEventCreateWithFlags(&ctx->mid, hipEventDisableTiming) == hipSuccess &&
                    hipEventCreateWithFlags(&ctx->join, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
      symi::set_error("symi_create: creating the helper stream failed: %s", hipGetErrorString(hipGetLastError()));
      symi::release(ctx);
      delete ctx;
      return SYMI_EHIP;
    }
  }
  ctx->magic = symi::CTX_MAGIC;
  *out = ctx;
  return SYMI_OK;
}

int symi_destroy(symi_ctx* ctx) {
  if (!ctx) return SYMI_OK;
  if (ctx->magic != symi::CTX_MAGIC) {
    symi::set_error("symi_destroy: not a live context of symi_create");
    return SYMI_EINVAL;
  }
  ctx->magic = 0;
  symi::release(ctx);
  delete ctx;
  return SYMI_OK;
}

int symi_timing_reset(const symi_ctx* ctx) {
  if (!ctx || ctx->magic != symi::CTX_MAGIC) {
    symi::set_error("symi_timing_reset: bad context");
    return SYMI_EINVAL;
  }
  for (auto& l : ctx->launches) {
    (void)hipEventDestroy(l.a);
    (void)hipEventDestroy(l.b);
  }
  ctx->launches.clear();
  return SYMI_OK;
}

int symi_timing_read(const symi_ctx* ctx, int kernel_id, double* total_ms, int* launches) {
  if (!ctx || ctx->magic != symi::CTX_MAGIC || kernel_id < 0 || kernel_id >= symi::K_COUNT || !total_ms || !launches) {
    symi::set_error("symi_timing_read: bad argument");
    return SYMI_EINVAL;
  }
  double tot = 0.0;
  int n = 0;
  for (auto& l : ctx->launches) {
    if (l.kid != kernel_id) continue;
    if (hipEventSynchronize(l.b) != hipSuccess) {
      symi::set_error("symi_timing_read: hipEventSynchronize failed");
      return SYMI_EHIP;
    }
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, l.a, l.b) != hipSuccess) {
      symi::set_error("symi_timing_read: hipEventElapsedTime failed");
      return SYMI_EHIP;
    }
    tot += ms;
    ++n;
  }
  *total_ms = tot;
  *launches = n;
  return SYMI_OK;
}

int symi_kernel_count(void) { return symi::K_COUNT; }

const char* symi_kernel_name(int kernel_id) {
  return kernel_id >= 0 && kernel_id < symi::K_COUNT ? symi::g_names[kernel_id] : "";
}

int symi_validate(const symi_cfg* cfg) { return symi::check_cfg(cfg, "symi_validate"); }

size_t symi_workspace_bytes(const symi_cfg* cfg) {
  if (symi::check_cfg(cfg, "symi_workspace_bytes") != SYMI_OK) return 0;
  return symi::ws_layout(cfg).total;
}

const char* symi_last_error(void) { return symi::g_err; }

}  // extern "C"
