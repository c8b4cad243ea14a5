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

namespace symi {

struct AdamScalars {
  float lr, beta1, beta2, eps, wd, gscale, inv_bc1, inv_bc2;
};

template <bool BF16>
__global__ __launch_bounds__(256) void adam_to_replicas_kernel(
    const float* __restrict__ dW1, const float* __restrict__ dW2, float* __restrict__ mw,
    float* __restrict__ m, float* __restrict__ v, const int32_t* __restrict__ first_next,
    void* __restrict__ W1s, void* __restrict__ W2s, long long n1, long long n2, long long per,
    long long lo, AdamScalars hp) {
  const int e = blockIdx.y;
  const long long groups = per / 8;
  const int q0 = first_next[e], q1 = first_next[e + 1];
  for (long long gi = (long long)blockIdx.x * 256 + threadIdx.x; gi < groups;
       gi += (long long)gridDim.x * 256) {
    const long long s = gi * 8;       // offset inside this partition's range
    const long long p = lo + s;       // offset inside the flat class vector [W1 | W2]
    const bool in1 = p < n1;          // 8-element groups never straddle n1 (n1 % 8 == 0)
    const float* gsrc = in1 ? dW1 + (long long)e * n1 + p : dW2 + (long long)e * n2 + (p - n1);
    const long long so = (long long)e * per + s;
    float g[8], w[8], mm[8], vv[8];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float4 a = reinterpret_cast<const float4*>(gsrc)[h];
      const float4 b = reinterpret_cast<const float4*>(mw + so)[h];
      const float4 c = reinterpret_cast<const float4*>(m + so)[h];
      const float4 d = reinterpret_cast<const float4*>(v + so)[h];
      g[4 * h] = a.x; g[4 * h + 1] = a.y; g[4 * h + 2] = a.z; g[4 * h + 3] = a.w;
      w[4 * h] = b.x; w[4 * h + 1] = b.y; w[4 * h + 2] = b.z; w[4 * h + 3] = b.w;
      mm[4 * h] = c.x; mm[4 * h + 1] = c.y; mm[4 * h + 2] = c.z; mm[4 * h + 3] = c.w;
      vv[4 * h] = d.x; vv[4 * h + 1] = d.y; vv[4 * h + 2] = d.z; vv[4 * h + 3] = d.w;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float gr = hp.gscale * g[i];
      mm[i] = hp.beta1 * mm[i] + (1.f - hp.beta1) * gr;
      vv[i] = hp.beta2 * vv[i] + (1.f - hp.beta2) * gr * gr;
      const float mhat = mm[i] * hp.inv_bc1;
      const float vhat = vv[i] * hp.inv_bc2;
      w[i] = w[i] - hp.lr * (mhat / (sqrtf(vhat) + hp.eps) + hp.wd * w[i]);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      reinterpret_cast<float4*>(mw + so)[h] = make_float4(w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]);
      reinterpret_cast<float4*>(m + so)[h] = make_float4(mm[4 * h], mm[4 * h + 1], mm[4 * h + 2], mm[4 * h + 3]);
      reinterpret_cast<float4*>(v + so)[h] = make_float4(vv[4 * h], vv[4 * h + 1], vv[4 * h + 2], vv[4 * h + 3]);
    }
    // the weight phase: every replica of class e in the next placement gets the range
    const long long slot_stride = in1 ? n1 : n2;
    const long long in_slot = in1 ? p : p - n1;
    if (BF16) {
      uint4 pk;
      pk.x = pack_bf16x2(w[0], w[1]); pk.y = pack_bf16x2(w[2], w[3]);
      pk.z = pack_bf16x2(w[4], w[5]); pk.w = pack_bf16x2(w[6], w[7]);
      uint16_t* basep = static_cast<uint16_t*>(in1 ? W1s : W2s);
      for (int q = q0; q < q1; ++q)
        *reinterpret_cast<uint4*>(basep + (long long)q * slot_stride + in_slot) = pk;
    } else {
      float* basep = static_cast<float*>(in1 ? W1s : W2s);
      for (int q = q0; q < q1; ++q) {
        float4* dst = reinterpret_cast<float4*>(basep + (long long)q * slot_stride + in_slot);
        dst[0] = make_float4(w[0], w[1], w[2], w[3]);
        dst[1] = make_float4(w[4], w[5], w[6], w[7]);
      }
    }
  }
}

}  // namespace symi

using namespace symi;

extern "C" int symi_adam_to_replicas(const symi_cfg* cfg, const symi_adam* hp,
                                     const float* dW1_class, const float* dW2_class,
                                     float* master_w, float* m, float* v,
                                     const int32_t* first_slot_next, void* W1_slots,
                                     void* W2_slots, void* stream) {
  if (int rc = check_cfg(cfg, "symi_adam_to_replicas")) return rc;
  SYMI_REQUIRE(hp && dW1_class && dW2_class && master_w && m && v && first_slot_next && W1_slots &&
                   W2_slots, "symi_adam_to_replicas", "NULL pointer");
  SYMI_REQUIRE(hp->step >= 1, "symi_adam_to_replicas", "step must be >= 1");
  SYMI_REQUIRE(hp->beta1 >= 0.f && hp->beta1 < 1.f && hp->beta2 >= 0.f && hp->beta2 < 1.f,
               "symi_adam_to_replicas", "betas must lie in [0, 1)");
  const long long n1 = 2LL * cfg->f * cfg->d, n2 = (long long)cfg->d * cfg->f;
  const long long per = (n1 + n2) / cfg->N;
  const long long lo = per * cfg->shard;
  AdamScalars s;
  s.lr = hp->lr; s.beta1 = hp->beta1; s.beta2 = hp->beta2; s.eps = hp->eps;
  s.wd = hp->weight_decay; s.gscale = hp->grad_scale;
  // bias corrections evaluated once in double, then applied as fp32 factors
  s.inv_bc1 = (float)(1.0 / (1.0 - pow((double)hp->beta1, hp->step)));
  s.inv_bc2 = (float)(1.0 / (1.0 - pow((double)hp->beta2, hp->step)));
  long long gx = (per / 8 + 255) / 256;
  if (gx > 4096) gx = 4096;
  if (gx < 1) gx = 1;
  dim3 grid((unsigned)gx, (unsigned)cfg->E);
  hipStream_t st = as_stream(stream);
  if (cfg->dtype == SYMI_BF16)
    SYMI_TIMED(K_ADAM, st, (adam_to_replicas_kernel<true><<<grid, 256, 0, st>>>(
        dW1_class, dW2_class, master_w, m, v, first_slot_next, W1_slots, W2_slots, n1, n2, per, lo, s)));
  else
    SYMI_TIMED(K_ADAM, st, (adam_to_replicas_kernel<false><<<grid, 256, 0, st>>>(
        dW1_class, dW2_class, master_w, m, v, first_slot_next, W1_slots, W2_slots, n1, n2, per, lo, s)));
  SYMI_LAUNCH_CHECK("symi_adam_to_replicas");
  return SYMI_OK;
}
