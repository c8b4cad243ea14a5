// symi_route / symi_route_bwd: top-k gating with the per-class popularity histogram
// (paper Sec. 2.1 and Sec. 3.2 step 1).
//
// A token's logits row is shared by a group of G lanes (G a power of two, G*4*NV >= E),
// each lane holding NV float4 pieces, so that global loads are coalesced 16-byte
// accesses and the arg-max of each top-k round is a log2(G)-step butterfly inside the
// 64-wide wavefront.  A wavefront serves 64/G tokens at a time.  Ties go to the lower
// class index because every comparison orders (value, -index) pairs.  The histogram is
// accumulated with integer atomics (LDS per workgroup, then one global add per class
// and workgroup): integer sums do not depend on the order of the adds.
#include <float.h>
#include <limits.h>

#include "common.h"

namespace symi {

constexpr int ROUTE_THREADS = 256;
constexpr int ROUTE_THREADS_MAX = 1024;   // route_kernel on large batches
constexpr int MAX_K = 16;

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t val) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = val;
}

void launch_fill_i32(const symi_ctx* ctx, int32_t* p, int n, int32_t val, hipStream_t st) {
  if (n > 0) SYMI_TIMED(ctx, K_FILL, st, (fill_i32_kernel<<<cdiv(n, 256), 256, 0, st>>>(p, n, val)));
}

template <int NV>
__device__ __forceinline__ void load_row(const float* __restrict__ row, int E, int G, int g,
                                         bool valid, float (&z)[NV * 4]) {
  const bool vec_ok = (E & 3) == 0;
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int col0 = (v * G + g) * 4;
    if (valid && vec_ok && col0 + 3 < E) {
      const float4 q = *reinterpret_cast<const float4*>(row + col0);
      z[v * 4 + 0] = q.x; z[v * 4 + 1] = q.y; z[v * 4 + 2] = q.z; z[v * 4 + 3] = q.w;
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c)
        z[v * 4 + c] = (valid && col0 + c < E) ? row[col0 + c] : -INFINITY;
    }
  }
}

// Softmax statistics of the row held by a lane group: max and sum of exp(z - max).
template <int NV>
__device__ __forceinline__ void row_stats(const float (&z)[NV * 4], int E, int G, int g,
                                          float& zmax, float& zsum) {
  float mx = -INFINITY;
#pragma unroll
  for (int c = 0; c < NV * 4; ++c) mx = fmaxf(mx, z[c]);
  for (int m = G >> 1; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NV * 4; ++c) {
    const int col = ((c >> 2) * G + g) * 4 + (c & 3);
    if (col < E) s += expf(z[c] - mx);
  }
  for (int m = G >> 1; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
  zmax = mx;
  zsum = s;
}

// Order-preserving integer image of a float (an involution): a > b  <=>  key(a) > key(b) for all
// non-NaN floats, -inf included.  INT_MIN is no float's key: it marks what can never be chosen
// (a column beyond E, a NaN).
__device__ __forceinline__ int order_key(float z) {
  const int i = __float_as_int(z);
  return i ^ ((i >> 31) & 0x7fffffff);
}
constexpr int KEY_NONE = INT_MIN;

// G lanes share a token's row, NV float4 pieces each (both compile-time: the column of a lane's
// c-th value is then a constant plus 4 g).  Each of the k rounds scans the lane's own values in
// increasing column order with a strict comparison (so the lowest column wins ties inside a
// lane without comparing columns), skips the values retired in earlier rounds by a bit mask, and
// settles the winner across the group by a butterfly over (key, column) pairs.
// Workgroups of 256 or 1024 threads (blockDim.x): every workgroup adds its histogram to the
// global one with E atomics, so a large batch takes the large workgroup (a quarter of the
// atomics on the same E addresses).
template <int G, int NV>
__global__ __launch_bounds__(ROUTE_THREADS_MAX) void route_kernel(
    const float* __restrict__ logits, int32_t* __restrict__ idx, float* __restrict__ gate,
    int32_t* __restrict__ hist, int T, int E, int k, int renorm) {
  extern __shared__ int32_t hist_s[];
  const int nthreads = blockDim.x;
  for (int i = threadIdx.x; i < E; i += nthreads) hist_s[i] = 0;
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane & (G - 1), sub = lane / G;
  constexpr int tpw = 64 / G;
  const int tpb = (nthreads / 64) * tpw;
  constexpr int NVAL = NV * 4;
  auto col_of = [&](int c) { return ((c >> 2) * G + g) * 4 + (c & 3); };

  for (long long t0 = (long long)blockIdx.x * tpb; t0 < T; t0 += (long long)gridDim.x * tpb) {
    const long long t = t0 + wave * tpw + sub;
    const bool valid = t < T;
    float z[NVAL];
    load_row<NV>(logits + (valid ? t : 0) * E, E, G, g, valid, z);
    float zmax, zsum;
    row_stats<NV>(z, E, G, g, zmax, zsum);
    int key[NVAL];
#pragma unroll
    for (int c = 0; c < NVAL; ++c)
      key[c] = (col_of(c) < E && z[c] == z[c]) ? order_key(z[c] + 0.f) : KEY_NONE;   // -0 counts as +0

    unsigned taken = 0;   // NVAL <= 32 values per lane
    float pj[MAX_K];
    int ij[MAX_K];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) {
      pj[j] = 0.f;
      ij[j] = 0;
      if (j < k) {
        int bk = KEY_NONE, bc = 0;
#pragma unroll
        for (int c = 0; c < NVAL; ++c) {
          const bool better = !((taken >> c) & 1u) && key[c] > bk;
          bk = better ? key[c] : bk;
          bc = better ? c : bc;
        }
        int bi = bk == KEY_NONE ? INT_MAX : col_of(bc);
        const int mine = bi;
#pragma unroll
        for (int m = G >> 1; m >= 1; m >>= 1) {
          const int ok = __shfl_xor(bk, m, 64);
          const int oi = __shfl_xor(bi, m, 64);
          const bool other = ok > bk || (ok == bk && oi < bi);
          bk = other ? ok : bk;
          bi = other ? oi : bi;
        }
        // the lane that owns the winner retires it
        if (bi != INT_MAX && bi == mine) taken |= 1u << bc;
        const float bv = __int_as_float(bk ^ ((bk >> 31) & 0x7fffffff));
        pj[j] = bi != INT_MAX ? expf(bv - zmax) / zsum : 0.f;
        ij[j] = bi;
        psum += pj[j];
      }
    }
    if (valid) {
#pragma unroll
      for (int j = 0; j < MAX_K; ++j) {
        if (j < k && g == (j & (G - 1))) {
          idx[t * k + j] = ij[j];
          gate[t * k + j] = renorm ? pj[j] / psum : pj[j];
          if ((unsigned)ij[j] < (unsigned)E) atomicAdd(&hist_s[ij[j]], 1);  // false only for NaN rows
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < E; i += nthreads)
    if (hist_s[i]) atomicAdd(&hist[i], hist_s[i]);
}

template <int NV>
__global__ __launch_bounds__(ROUTE_THREADS) void route_bwd_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ idx,
    const float* __restrict__ gate, const float* __restrict__ dgate,
    float* __restrict__ dlogits, int T, int E, int k, int G, int renorm) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane & (G - 1), sub = lane / G, tpw = 64 / G;
  const int tpb = (ROUTE_THREADS / 64) * tpw;

  for (long long t0 = (long long)blockIdx.x * tpb; t0 < T; t0 += (long long)gridDim.x * tpb) {
    const long long t = t0 + wave * tpw + sub;
    const bool valid = t < T;
    const float* row = logits + (valid ? t : 0) * E;
    float z[NV * 4];
    load_row<NV>(row, E, G, g, valid, z);
    float zmax, zsum;
    row_stats<NV>(z, E, G, g, zmax, zsum);

    int ij[MAX_K];
    float ps[MAX_K], dg[MAX_K];
    float ssum = 0.f, dot = 0.f;
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) {
      ij[j] = -1; ps[j] = 0.f; dg[j] = 0.f;
      if (j < k && valid) {
        ij[j] = idx[t * k + j];
        ps[j] = (unsigned)ij[j] < (unsigned)E ? expf(row[ij[j]] - zmax) / zsum : 0.f;
        dg[j] = dgate[t * k + j];
        ssum += ps[j];
        dot += dg[j] * gate[t * k + j];
      }
    }
    // gradient w.r.t. the selected probabilities, then its inner product with p
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < MAX_K; ++j) {
      if (j < k) {
        if (renorm) dg[j] = (dg[j] - dot) / ssum;
        s += dg[j] * ps[j];
      }
    }
    if (!valid) continue;
    const bool vec_ok = (E & 3) == 0;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col0 = (v * G + g) * 4;
      float out[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int col = col0 + c;
        float dp = 0.f;
#pragma unroll
        for (int j = 0; j < MAX_K; ++j)
          if (j < k && ij[j] == col) dp = dg[j];
        const float p = col < E ? expf(z[v * 4 + c] - zmax) / zsum : 0.f;
        out[c] = p * (dp - s);
      }
      float* dst = dlogits + t * E + col0;
      if (vec_ok && col0 + 3 < E) {
        *reinterpret_cast<float4*>(dst) = make_float4(out[0], out[1], out[2], out[3]);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (col0 + c < E) dst[c] = out[c];
      }
    }
  }
}

static void route_shape(int E, int& G, int& NV) {
  const int vecs = (E + 3) / 4;
  G = 1;
  while (G < vecs && G < 64) G <<= 1;
  const int need = (vecs + G - 1) / G;
  NV = need <= 1 ? 1 : (need <= 2 ? 2 : 4);
}

// The forward kernel spends its time in the k selection rounds: few lanes per token (a short
// butterfly) with up to 32 values each, scanned locally, cost a third of the instructions of
// one float4 per lane.
static void route_fwd_shape(int E, int T, int& G, int& NV) {
  const int vecs = (E + 3) / 4;
  G = 1;
  while (G * 8 < vecs && G < 64) G <<= 1;
  // a small batch is spread over more lanes per token instead, so that the chip is filled:
  // at least 512 workgroups of (256 / G) tokens, as long as a lane still has a float4
  while (G < vecs && G < 64 && (long long)T * G < 512LL * ROUTE_THREADS) G <<= 1;
  const int need = (vecs + G - 1) / G;
  NV = need <= 1 ? 1 : (need <= 2 ? 2 : (need <= 4 ? 4 : 8));
}

static int route_grid(int T, int G) {
  const int tpb = (ROUTE_THREADS / 64) * (64 / G);
  int grid = cdiv(T, tpb);
  return grid < 1 ? 1 : (grid > 8192 ? 8192 : grid);
}

}  // namespace symi

using namespace symi;

extern "C" int symi_route(const symi_ctx* ctx, const float* logits, int32_t* idx, float* gate,
                          int32_t* hist, void* stream) {
  SYMI_ENTER(ctx, "symi_route");
  SYMI_REQUIRE(hist && (cfg->T == 0 || (logits && idx && gate)), "symi_route", "NULL pointer");
  hipStream_t st = as_stream(stream);
  const int E = cfg->E;
  launch_fill_i32(ctx, hist, E, 0, st);
  if (cfg->T > 0) {
    int G, NV;
    route_fwd_shape(E, cfg->T, G, NV);
    int grid = route_grid(cfg->T, G);
    // four workgroups of 256 per compute unit or more: one of 1024 each instead
    const int threads = grid >= 4 * ctx->cus ? ROUTE_THREADS_MAX : ROUTE_THREADS;
    if (threads == ROUTE_THREADS_MAX) grid = cdiv(grid, ROUTE_THREADS_MAX / ROUTE_THREADS);
    const size_t sh = (size_t)E * sizeof(int32_t);
#define SYMI_ROUTE_CASE(GG, NN)                                                                  \
  case GG * 16 + NN:                                                                             \
    SYMI_TIMED(ctx, K_ROUTE, st, (route_kernel<GG, NN><<<grid, threads, sh, st>>>(          \
        logits, idx, gate, hist, cfg->T, E, cfg->k, cfg->renorm)));                              \
    break;
#define SYMI_ROUTE_G(GG) SYMI_ROUTE_CASE(GG, 1) SYMI_ROUTE_CASE(GG, 2) SYMI_ROUTE_CASE(GG, 4) SYMI_ROUTE_CASE(GG, 8)
    switch (G * 16 + NV) {
      SYMI_ROUTE_G(1) SYMI_ROUTE_G(2) SYMI_ROUTE_G(4) SYMI_ROUTE_G(8) SYMI_ROUTE_G(16) SYMI_ROUTE_G(32) SYMI_ROUTE_G(64)
      default:
        set_error("symi_route: no kernel for %d lanes x %d pieces per token", G, NV);
        return SYMI_EUNSUPPORTED;
    }
#undef SYMI_ROUTE_G
#undef SYMI_ROUTE_CASE
  }
  SYMI_LAUNCH_CHECK("symi_route");
  return SYMI_OK;
}

extern "C" int symi_route_bwd(const symi_ctx* ctx, const float* logits, const int32_t* idx,
                              const float* gate, const float* dgate, float* dlogits,
                              void* stream) {
  SYMI_ENTER(ctx, "symi_route_bwd");
  if (cfg->T == 0) return SYMI_OK;
  SYMI_REQUIRE(logits && idx && gate && dgate && dlogits, "symi_route_bwd", "NULL pointer");
  hipStream_t st = as_stream(stream);
  int G, NV;
  route_shape(cfg->E, G, NV);
  const int grid = route_grid(cfg->T, G);
  if (NV == 1)
    SYMI_TIMED(ctx, K_ROUTE_BWD, st, (route_bwd_kernel<1><<<grid, ROUTE_THREADS, 0, st>>>(logits, idx, gate, dgate, dlogits, cfg->T, cfg->E, cfg->k, G, cfg->renorm)));
  else if (NV == 2)
    SYMI_TIMED(ctx, K_ROUTE_BWD, st, (route_bwd_kernel<2><<<grid, ROUTE_THREADS, 0, st>>>(logits, idx, gate, dgate, dlogits, cfg->T, cfg->E, cfg->k, G, cfg->renorm)));
  else
    SYMI_TIMED(ctx, K_ROUTE_BWD, st, (route_bwd_kernel<4><<<grid, ROUTE_THREADS, 0, st>>>(logits, idx, gate, dgate, dlogits, cfg->T, cfg->E, cfg->k, G, cfg->renorm)));
  SYMI_LAUNCH_CHECK("symi_route_bwd");
  return SYMI_OK;
}
