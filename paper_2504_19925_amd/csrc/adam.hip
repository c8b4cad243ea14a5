// symi_adam_to_replicas: the Symi Optimizer's step on this GPU's static 1/N partition of
// every expert class, fused with the weight write into the replica slots of the NEXT
// placement (paper Sec. 3.2 steps 4-8, Sec. 3.3 "weight communication phase", Sec. 4.4).
//
// Pure streaming: per parameter 16 B are read (grad, master weight, m, v), 12 B are
// written back, and the fresh weight goes once to every replica slot of its class, so a
// slot never sees the master copy round-trip through HBM.  The number of slot bytes is
// S_tot * P_e / N * sizeof(weight) for any placement.  One thread owns 8 consecutive
// parameters (two float4 per state tensor, one 16-byte bf16 store per replica).
#include <math.h>

#include "common.h"

#ifndef SYMI_ADAM_NT
#define SYMI_ADAM_NT false   // measured: non-temporal stores 4.9 TB/s, loads+stores 3.7, plain 5.1
#endif
#ifndef SYMI_ADAM_BLOCK
#define SYMI_ADAM_BLOCK 256
#endif
#ifndef SYMI_ADAM_UNROLL
#define SYMI_ADAM_UNROLL 1   // 8-parameter groups a thread has in flight at once
#endif

namespace symi {

struct AdamScalars {
  float lr, beta1, beta2, eps, wd, gscale, inv_bc1, inv_bc2;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// NT marks loads and stores non-temporal (streamed past the caches).  Every byte here is
// touched once per step, yet on MI355X the plain path is the faster one, so NT is off.
template <bool NT, typename V>
__device__ __forceinline__ V ld_stream(const V* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT, typename V>
__device__ __forceinline__ void st_stream(V v, V* p) {
  if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}

template <bool BF16, bool NT, int U>
__global__ __launch_bounds__(SYMI_ADAM_BLOCK) void adam_to_replicas_kernel(
    const float* __restrict__ dW1, const float* __restrict__ dW2, float* __restrict__ mw,
    float* __restrict__ m, float* __restrict__ v, const int32_t* __restrict__ first_next,
    void* __restrict__ W1s, void* __restrict__ W2s, long long n1, long long n2, long long per,
    long long lo, AdamScalars hp, const int32_t* __restrict__ slot_offsets,
    const int32_t* __restrict__ first_slot) {
  const int e = blockIdx.y;
  // a class that had no rows this iteration: its gradient is zero and is not read
  const bool has_g = !slot_offsets || slot_offsets[first_slot[e + 1]] > slot_offsets[first_slot[e]];
  const long long groups = per / 8;
  const int q0 = first_next[e], q1 = first_next[e + 1];
  const long long stride = (long long)gridDim.x * SYMI_ADAM_BLOCK;
  for (long long g0 = (long long)blockIdx.x * SYMI_ADAM_BLOCK + threadIdx.x; g0 < groups; g0 += stride * U) {
    f32x4 g[U][2], w[U][2], mm[U][2], vv[U][2];
    // all loads of the U groups first, then the arithmetic and the stores
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long gi = g0 + u * stride;
      if (gi >= groups) continue;
      const long long s = gi * 8;       // offset inside this partition's range
      const long long p = lo + s;       // offset inside the flat class vector [W1 | W2]
      const bool in1 = p < n1;          // 8-element groups never straddle n1 (n1 % 8 == 0)
      const float* gsrc = in1 ? dW1 + (long long)e * n1 + p : dW2 + (long long)e * n2 + (p - n1);
      const long long so = (long long)e * per + s;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        g[u][h] = has_g ? ld_stream<NT>(reinterpret_cast<const f32x4*>(gsrc) + h) : f32x4{0.f, 0.f, 0.f, 0.f};
        w[u][h] = ld_stream<NT>(reinterpret_cast<const f32x4*>(mw + so) + h);
        mm[u][h] = ld_stream<NT>(reinterpret_cast<const f32x4*>(m + so) + h);
        vv[u][h] = ld_stream<NT>(reinterpret_cast<const f32x4*>(v + so) + h);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long gi = g0 + u * stride;
      if (gi >= groups) continue;
      const long long s = gi * 8;
      const long long p = lo + s;
      const bool in1 = p < n1;
      const long long so = (long long)e * per + s;
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float gr = hp.gscale * g[u][h][i];
          mm[u][h][i] = hp.beta1 * mm[u][h][i] + (1.f - hp.beta1) * gr;
          vv[u][h][i] = hp.beta2 * vv[u][h][i] + (1.f - hp.beta2) * gr * gr;
          const float mhat = mm[u][h][i] * hp.inv_bc1;
          const float vhat = vv[u][h][i] * hp.inv_bc2;
          w[u][h][i] = w[u][h][i] - hp.lr * (mhat / (sqrtf(vhat) + hp.eps) + hp.wd * w[u][h][i]);
        }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        st_stream<NT>(w[u][h], reinterpret_cast<f32x4*>(mw + so) + h);
        st_stream<NT>(mm[u][h], reinterpret_cast<f32x4*>(m + so) + h);
        st_stream<NT>(vv[u][h], reinterpret_cast<f32x4*>(v + so) + h);
      }
      // the weight phase: every replica of class e in the next placement gets the range
      const long long slot_stride = in1 ? n1 : n2;
      const long long in_slot = in1 ? p : p - n1;
      if (BF16) {
        u32x4 pk;
        pk[0] = pack_bf16x2(w[u][0][0], w[u][0][1]); pk[1] = pack_bf16x2(w[u][0][2], w[u][0][3]);
        pk[2] = pack_bf16x2(w[u][1][0], w[u][1][1]); pk[3] = pack_bf16x2(w[u][1][2], w[u][1][3]);
        uint16_t* basep = static_cast<uint16_t*>(in1 ? W1s : W2s);
        for (int q = q0; q < q1; ++q)
          st_stream<NT>(pk, reinterpret_cast<u32x4*>(basep + (long long)q * slot_stride + in_slot));
      } else {
        float* basep = static_cast<float*>(in1 ? W1s : W2s);
        for (int q = q0; q < q1; ++q) {
          f32x4* dst = reinterpret_cast<f32x4*>(basep + (long long)q * slot_stride + in_slot);
          st_stream<NT>(w[u][0], dst);
          st_stream<NT>(w[u][1], dst + 1);
        }
      }
    }
  }
}

}  // namespace symi

using namespace symi;

static int adam_impl(const char* who, const symi_ctx* ctx, const symi_adam* hp,
                     const float* dW1_class, const float* dW2_class, float* master_w, float* m,
                     float* v, const int32_t* slot_offsets, const int32_t* first_slot,
                     const int32_t* first_slot_next, void* W1_slots, void* W2_slots, void* stream) {
  SYMI_ENTER(ctx, who);
  SYMI_REQUIRE(hp && dW1_class && dW2_class && master_w && m && v && first_slot_next && W1_slots &&
                   W2_slots, who, "NULL pointer");
  SYMI_REQUIRE(hp->step >= 1, who, "step must be >= 1");
  SYMI_REQUIRE(hp->beta1 >= 0.f && hp->beta1 < 1.f && hp->beta2 >= 0.f && hp->beta2 < 1.f,
               who, "betas must lie in [0, 1)");
  const long long n1 = 2LL * cfg->f * cfg->d, n2 = (long long)cfg->d * cfg->f;
  const long long per = (n1 + n2) / cfg->N;
  const long long lo = per * cfg->shard;
  AdamScalars s;
  s.lr = hp->lr; s.beta1 = hp->beta1; s.beta2 = hp->beta2; s.eps = hp->eps;
  s.wd = hp->weight_decay; s.gscale = hp->grad_scale;
  // bias corrections evaluated once in double, then applied as fp32 factors
  s.inv_bc1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, hp->step)));
  s.inv_bc2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, hp->step)));
  const long long per_block = (long long)SYMI_ADAM_BLOCK * SYMI_ADAM_UNROLL;
  long long gx = (per / 8 + per_block - 1) / per_block;
  if (gx > 8192) gx = 8192;
  if (gx < 1) gx = 1;
  dim3 grid((unsigned)gx, (unsigned)cfg->E);
  hipStream_t st = as_stream(stream);
  if (cfg->dtype == SYMI_BF16)
    SYMI_TIMED(ctx, K_ADAM, st, (adam_to_replicas_kernel<true, SYMI_ADAM_NT, SYMI_ADAM_UNROLL><<<grid, SYMI_ADAM_BLOCK, 0, st>>>(
        dW1_class, dW2_class, master_w, m, v, first_slot_next, W1_slots, W2_slots, n1, n2, per, lo, s, slot_offsets, first_slot)));
  else
    SYMI_TIMED(ctx, K_ADAM, st, (adam_to_replicas_kernel<false, SYMI_ADAM_NT, SYMI_ADAM_UNROLL><<<grid, SYMI_ADAM_BLOCK, 0, st>>>(
        dW1_class, dW2_class, master_w, m, v, first_slot_next, W1_slots, W2_slots, n1, n2, per, lo, s, slot_offsets, first_slot)));
  SYMI_LAUNCH_CHECK(who);
  return SYMI_OK;
}

extern "C" int symi_adam_to_replicas(const symi_ctx* ctx, const symi_adam* hp,
                                     const float* dW1_class, const float* dW2_class,
                                     float* master_w, float* m, float* v,
                                     const int32_t* first_slot_next, void* W1_slots,
                                     void* W2_slots, void* stream) {
  return adam_impl("symi_adam_to_replicas", ctx, hp, dW1_class, dW2_class, master_w, m, v, nullptr,
                   nullptr, first_slot_next, W1_slots, W2_slots, stream);
}

extern "C" int symi_adam_to_replicas_active(const symi_ctx* ctx, const symi_adam* hp,
                                            const float* dW1_class, const float* dW2_class,
                                            float* master_w, float* m, float* v,
                                            const int32_t* slot_offsets, const int32_t* first_slot,
                                            const int32_t* first_slot_next, void* W1_slots,
                                            void* W2_slots, void* stream) {
  if (!slot_offsets || !first_slot) {
    set_error("symi_adam_to_replicas_active: NULL pointer");
    return SYMI_EINVAL;
  }
  return adam_impl("symi_adam_to_replicas_active", ctx, hp, dW1_class, dW2_class, master_w, m, v,
                   slot_offsets, first_slot, first_slot_next, W1_slots, W2_slots, stream);
}
