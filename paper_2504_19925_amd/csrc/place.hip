// symi_place / symi_place_host: the Expert Placement Scheduler (paper App. A.3,
// Algorithm 1; Sec. 3.4) in exact integer arithmetic.
//
// goal_i = pop_i * S_tot / P is never formed: the rounding error diff_i = counts_i -
// goal_i is carried as its numerator D_i = counts_i * P - pop_i * S_tot (int64).
// The shrinking loop of the algorithm also visits classes pinned at one replica; such a
// visit only lowers that class's own diff and never changes which class with more than
// one replica is shrunk next, so both versions here pick "first maximum among classes
// with more than one replica" directly: identical counts in at most E steps.
//
// Device version: one 64-lane wavefront; lane l owns classes l, l+64, ...; the arg-max /
// arg-min is a strided scan followed by a butterfly over (D, index) pairs.  It runs on
// the stream between the histogram and the optimizer step, so no host round trip is
// needed to learn the next placement.
#include <vector>

#include "common.h"

namespace symi {

constexpr int PLACE_MAX_E = 1024;

__device__ __forceinline__ long long wave_sum_ll(long long x) {
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}

__global__ __launch_bounds__(64) void place_kernel(const int32_t* __restrict__ pop,
                                                   int32_t* __restrict__ counts,
                                                   int32_t* __restrict__ placement,
                                                   int32_t* __restrict__ first_slot, int E, int S) {
  __shared__ long long D[PLACE_MAX_E];
  __shared__ int cnt[PLACE_MAX_E];
  __shared__ int first[PLACE_MAX_E + 1];
  const int lane = threadIdx.x;

  long long psum = 0;
  for (int i = lane; i < E; i += 64) psum += pop[i] > 0 ? pop[i] : 0;
  psum = wave_sum_ll(psum);
  const bool uniform = psum == 0;  // no popularity recorded yet: treat all classes alike
  const long long P = uniform ? E : psum;

  long long tot = 0;
  for (int i = lane; i < E; i += 64) {
    const long long p = uniform ? 1 : (pop[i] > 0 ? pop[i] : 0);
    long long c = p * S / P;  // floor(goal)
    if (c < 1) c = 1;         // every class stays reachable
    cnt[i] = (int)c;
    D[i] = c * P - p * S;
    tot += c;
  }
  long long total = wave_sum_ll(tot);
  __syncthreads();

  // too many replicas: shrink the class whose count exceeds its goal the most
  for (int it = 0; total > S && it < E + S; ++it) {
    long long bd = 0;
    int bi = INT32_MAX;
    for (int i = lane; i < E; i += 64)
      if (cnt[i] > 1 && (bi == INT32_MAX || D[i] > bd)) { bd = D[i]; bi = i; }
    for (int m = 32; m >= 1; m >>= 1) {
      const long long od = __shfl_xor(bd, m, 64);
      const int oi = __shfl_xor(bi, m, 64);
      if (oi != INT32_MAX && (bi == INT32_MAX || od > bd || (od == bd && oi < bi))) { bd = od; bi = oi; }
    }
    if (bi == INT32_MAX) break;
    if (lane == 0) { cnt[bi] -= 1; D[bi] -= P; }
    total -= 1;
    __syncthreads();
  }
  // too few: grow the class that lags its goal the most
  for (int it = 0; total < S && it < E + S; ++it) {
    long long bd = 0;
    int bi = INT32_MAX;
    for (int i = lane; i < E; i += 64)
      if (bi == INT32_MAX || D[i] < bd) { bd = D[i]; bi = i; }
    for (int m = 32; m >= 1; m >>= 1) {
      const long long od = __shfl_xor(bd, m, 64);
      const int oi = __shfl_xor(bi, m, 64);
      if (oi != INT32_MAX && (bi == INT32_MAX || od < bd || (od == bd && oi < bi))) { bd = od; bi = oi; }
    }
    if (lane == 0) { cnt[bi] += 1; D[bi] += P; }
    total += 1;
    __syncthreads();
  }

  // first_slot = exclusive prefix sum of counts, 64 classes per step
  int carry = 0;
  for (int base = 0; base < E; base += 64) {
    const int i = base + lane;
    const int c = i < E ? cnt[i] : 0;
    int incl = c;
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (i < E) {
      first[i] = carry + incl - c;
      first_slot[i] = carry + incl - c;
      counts[i] = c;
    }
    carry += __shfl(incl, 63, 64);
  }
  if (lane == 0) { first[E] = carry; first_slot[E] = carry; }
  __syncthreads();

  // same-class instances are contiguous: slot q belongs to the class whose run holds q
  for (int q = lane; q < S; q += 64) {
    int lo = 0, hi = E - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (first[mid] <= q) lo = mid; else hi = mid - 1;
    }
    placement[q] = lo;
  }
}

static void place_host(const int32_t* pop_in, int E, int S, int32_t* counts, int32_t* placement,
                       int32_t* first_slot) {
  std::vector<long long> pop(E), D(E);
  long long P = 0;
  for (int i = 0; i < E; ++i) { pop[i] = pop_in[i] > 0 ? pop_in[i] : 0; P += pop[i]; }
  if (P == 0) { for (int i = 0; i < E; ++i) pop[i] = 1; P = E; }
  long long total = 0;
  for (int i = 0; i < E; ++i) {
    long long c = pop[i] * S / P;
    if (c < 1) c = 1;
    counts[i] = (int32_t)c;
    D[i] = c * P - pop[i] * S;
    total += c;
  }
  while (total > S) {
    int bi = -1;
    for (int i = 0; i < E; ++i)
      if (counts[i] > 1 && (bi < 0 || D[i] > D[bi])) bi = i;
    if (bi < 0) break;
    counts[bi] -= 1; D[bi] -= P; total -= 1;
  }
  while (total < S) {
    int bi = 0;
    for (int i = 1; i < E; ++i)
      if (D[i] < D[bi]) bi = i;
    counts[bi] += 1; D[bi] += P; total += 1;
  }
  int q = 0;
  for (int i = 0; i < E; ++i) {
    first_slot[i] = q;
    for (int c = 0; c < counts[i]; ++c) placement[q++] = i;
  }
  first_slot[E] = q;
}

}  // namespace symi

using namespace symi;

extern "C" int symi_place(const symi_cfg* cfg, const int32_t* popularity, int32_t* counts,
                          int32_t* placement, int32_t* first_slot, void* stream) {
  if (int rc = check_cfg(cfg, "symi_place")) return rc;
  SYMI_REQUIRE(popularity && counts && placement && first_slot, "symi_place", "NULL pointer");
  hipStream_t st = as_stream(stream);
  SYMI_TIMED(K_PLACE, st, (place_kernel<<<1, 64, 0, st>>>(popularity, counts, placement, first_slot,
                                                        cfg->E, cfg->S_tot)));
  SYMI_LAUNCH_CHECK("symi_place");
  return SYMI_OK;
}

extern "C" int symi_place_host(const symi_cfg* cfg, const int32_t* popularity, int32_t* counts,
                               int32_t* placement, int32_t* first_slot) {
  if (int rc = check_cfg(cfg, "symi_place_host")) return rc;
  SYMI_REQUIRE(popularity && counts && placement && first_slot, "symi_place_host", "NULL pointer");
  place_host(popularity, cfg->E, cfg->S_tot, counts, placement, first_slot);
  return SYMI_OK;
}
