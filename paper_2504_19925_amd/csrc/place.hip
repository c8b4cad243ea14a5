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
// Device version: one 64-lane wavefront; lane l keeps classes l, l+64, ... in registers and
// the correction loops are evaluated in closed form (see place_kernel).  It runs on
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

__device__ __forceinline__ int wave_sum_i(int x) {
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}

// NPL = classes per lane (class lane + 64*i lives in register i of its lane).
//
// The two correction loops of the algorithm are evaluated in closed form.  Shrinking: a
// class with more than one replica starts with diff in (-1, 0]; each removal lowers its
// diff by exactly 1, below every class not yet visited in the same round.  The loop
// therefore proceeds in rounds over the classes in (diff descending, index ascending)
// order, a class dropping out once it is down to one replica.  With X replicas to remove,
// R = the largest number of full rounds with sum_i min(counts_i - 1, R) <= X, and the
// remaining X - that sum removals go to the first classes of that order still holding
// more than one replica.  Growing: the deficit Y is smaller than the number of classes
// that were not lifted to one replica, so the Y classes with the smallest (diff, index)
// get one replica each.
template <int NPL>
__global__ __launch_bounds__(64) void place_kernel(const int32_t* __restrict__ pop,
                                                   int32_t* __restrict__ counts,
                                                   int32_t* __restrict__ placement,
                                                   int32_t* __restrict__ first_slot, int E, int S) {
  __shared__ long long Dl[PLACE_MAX_E];
  __shared__ int cl[PLACE_MAX_E];
  __shared__ int first[PLACE_MAX_E + 1];
  const int lane = threadIdx.x;

  long long p[NPL];
  long long psum = 0;
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    const int c = lane + 64 * i;
    p[i] = (c < E && pop[c] > 0) ? pop[c] : 0;
    psum += p[i];
  }
  psum = wave_sum_ll(psum);
  const bool uniform = psum == 0;  // no popularity recorded yet: treat all classes alike
  const long long P = uniform ? E : psum;

  long long D[NPL];
  int cnt[NPL];
  int tot = 0;
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    const int c = lane + 64 * i;
    const long long pi = uniform ? 1 : p[i];
    long long k = pi * S / P;  // floor(goal)
    if (k < 1) k = 1;          // every class stays reachable
    cnt[i] = c < E ? (int)k : 0;
    D[i] = k * P - pi * S;
    tot += cnt[i];
  }
  const int total = wave_sum_i(tot);

  if (total > S) {
    const int X = total - S;
    int lo = 0, hi = S;       // full rounds
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      int f = 0;
#pragma unroll
      for (int i = 0; i < NPL; ++i) f += min(max(cnt[i] - 1, 0), mid);
      if (wave_sum_i(f) <= X) lo = mid; else hi = mid - 1;
    }
    const int R = lo;
    int f = 0;
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      const int dec = min(max(cnt[i] - 1, 0), R);
      cnt[i] -= dec;
      f += dec;
    }
    const int rem = X - wave_sum_i(f);
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      const int c = lane + 64 * i;
      if (c < E) { Dl[c] = D[i]; cl[c] = cnt[i]; }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      const int c = lane + 64 * i;
      if (c < E && cnt[i] > 1 && rem > 0) {
        int rank = 0;   // classes still shrinkable that come earlier in (diff desc, index asc)
        for (int j = 0; j < E; ++j)
          rank += (cl[j] > 1 && (Dl[j] > D[i] || (Dl[j] == D[i] && j < c))) ? 1 : 0;
        if (rank < rem) cnt[i] -= 1;
      }
    }
  } else if (total < S) {
    const int Y = S - total;
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      const int c = lane + 64 * i;
      if (c < E) Dl[c] = D[i];
    }
    __syncthreads();
    const int full = Y / E, rem = Y % E;   // full is 0 for any popularity; kept for safety
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      const int c = lane + 64 * i;
      if (c < E) {
        int rank = 0;   // classes that come earlier in (diff asc, index asc)
        for (int j = 0; j < E; ++j) rank += (Dl[j] < D[i] || (Dl[j] == D[i] && j < c)) ? 1 : 0;
        cnt[i] += full + (rank < rem ? 1 : 0);
      }
    }
  }

  // first_slot = exclusive prefix sum of counts, 64 classes per step
  int carry = 0;
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    const int c = lane + 64 * i;
    int incl = cnt[i];
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (c < E) {
      first[c] = carry + incl - cnt[i];
      first_slot[c] = carry + incl - cnt[i];
      counts[c] = cnt[i];
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

extern "C" int symi_place(const symi_ctx* ctx, const int32_t* popularity, int32_t* counts,
                          int32_t* placement, int32_t* first_slot, void* stream) {
  SYMI_ENTER(ctx, "symi_place");
  SYMI_REQUIRE(popularity && counts && placement && first_slot, "symi_place", "NULL pointer");
  hipStream_t st = as_stream(stream);
  const int E = cfg->E, S = cfg->S_tot;
  if (E <= 64)
    SYMI_TIMED(ctx, K_PLACE, st, (place_kernel<1><<<1, 64, 0, st>>>(popularity, counts, placement, first_slot, E, S)));
  else if (E <= 128)
    SYMI_TIMED(ctx, K_PLACE, st, (place_kernel<2><<<1, 64, 0, st>>>(popularity, counts, placement, first_slot, E, S)));
  else if (E <= 256)
    SYMI_TIMED(ctx, K_PLACE, st, (place_kernel<4><<<1, 64, 0, st>>>(popularity, counts, placement, first_slot, E, S)));
  else
    SYMI_TIMED(ctx, K_PLACE, st, (place_kernel<16><<<1, 64, 0, st>>>(popularity, counts, placement, first_slot, E, S)));
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
