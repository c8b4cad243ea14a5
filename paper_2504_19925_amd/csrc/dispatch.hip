// symi_dispatch / symi_dispatch_bwd / symi_combine / symi_combine_bwd: the token ->
// replica permutation of paper Sec. 3.2 step 2 and the data movement around the expert
// FFN (the all-to-all scatter/gather of Sec. 2.1, which on one GPU is a local
// permutation).
//
// The permutation is a stable counting sort of the A = T*k assignments by class, made
// deterministic without ordered atomics:
//   1. every workgroup counts the classes of its chunk of DISPATCH_CHUNK assignments;
//   2. one workgroup per class turns the per-chunk counts into exclusive bases (class
//      offset O_e + rows of that class in earlier chunks) and writes the class's
//      entries of slot_offsets from O_e, c_e and the placement;
//   3. every workgroup ranks its chunk again: inside a wavefront the rank among equal
//      classes is a popcount over a match mask built from ballots, across wavefronts
//      and passes it is a small LDS prefix.
// Row moves are 16-byte vector loads/stores, one row spread over consecutive lanes.
//
// symi_dispatch_capacity is the same permutation under the capacity rule of Sec. 3.4:
// class e may occupy slot_capacity * r_e rows (r_e = its replicas in the current
// placement); its assignments beyond that, in stable order, are dropped (row -1), the
// kept ones are packed without gaps and spread over the replicas as before.
#include <math.h>

#include <mutex>

#include "common.h"

// Scratch of symi_dispatch_noalloc (the per-chunk class counts and the per-class capacity
// table that symi_dispatch keeps in the caller's workspace).  Every GPU the library runs on
// holds its own copy at its own address until the process ends; host code never uses this name
// as an address, only the pointer hipGetSymbolAddress returned for the device in question.
static __device__ __align__(256) unsigned char scratch[SYMI_DISPATCH_NOALLOC_SCRATCH_BYTES];

namespace symi {

constexpr int DT = 256;                      // threads per workgroup
constexpr int DPASS = DISPATCH_CHUNK / DT;   // passes of 256 assignments per chunk

__global__ __launch_bounds__(DT) void chunk_count_kernel(const int32_t* __restrict__ cls, int A,
                                                         int E, int32_t* __restrict__ blk_counts) {
  extern __shared__ int32_t cnt_s[];
  for (int i = threadIdx.x; i < E; i += DT) cnt_s[i] = 0;
  __syncthreads();
  const int base = blockIdx.x * DISPATCH_CHUNK;
#pragma unroll
  for (int p = 0; p < DPASS; ++p) {
    const int a = base + p * DT + threadIdx.x;
    if (a < A && (unsigned)cls[a] < (unsigned)E) atomicAdd(&cnt_s[cls[a]], 1);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < E; i += DT) blk_counts[(size_t)blockIdx.x * E + i] = cnt_s[i];
}

// grid = E workgroups; workgroup e scans column e of blk_counts in place into bases.
// slot_cap > 0 switches the capacity rule on: class i keeps min(hist[i], slot_cap * counts[i])
// rows; slot_offsets then describes the kept rows only and tab[3e..] = {O_e, offset of the
// class among the kept rows, capacity of the class} tells the ranking kernel what to drop.
__global__ __launch_bounds__(DT) void chunk_scan_kernel(int32_t* __restrict__ blk_counts, int nblk,
                                                        int E, int S, int A,
                                                        const int32_t* __restrict__ hist,
                                                        const int32_t* __restrict__ counts,
                                                        const int32_t* __restrict__ first_slot,
                                                        int32_t* __restrict__ slot_offsets,
                                                        int slot_cap, int32_t* __restrict__ tab) {
  __shared__ int32_t wsum[DT / 64];
  __shared__ int32_t carry_s;
  __shared__ int32_t red[2][DT / 64];
  const int e = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  auto cap_of = [&](int i) -> int {
    if (slot_cap <= 0) return A;
    const long long c = (long long)slot_cap * counts[i];
    return c < A ? (int)c : A;
  };

  // class offset O_e = rows of all lower classes (all of them / the kept ones)
  int part = 0, partk = 0;
  for (int i = threadIdx.x; i < e; i += DT) {
    part += hist[i];
    partk += min(hist[i], cap_of(i));
  }
  for (int m = 32; m >= 1; m >>= 1) {
    part += __shfl_xor(part, m, 64);
    partk += __shfl_xor(partk, m, 64);
  }
  if (lane == 0) { red[0][wave] = part; red[1][wave] = partk; }
  __syncthreads();
  int O_e = 0, Ok_e = 0;
  for (int w = 0; w < DT / 64; ++w) { O_e += red[0][w]; Ok_e += red[1][w]; }
  if (threadIdx.x == 0) carry_s = O_e;
  __syncthreads();

  for (int b0 = 0; b0 < nblk; b0 += DT) {
    const int b = b0 + threadIdx.x;
    const int c = b < nblk ? blk_counts[(size_t)b * E + e] : 0;
    int incl = c;
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int before = carry_s;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    if (b < nblk) blk_counts[(size_t)b * E + e] = before + incl - c;
    __syncthreads();
    if (threadIdx.x == DT - 1) carry_s = before + incl;
    __syncthreads();
  }

  // replica i of class e owns rows O_e + floor(i*c_e/r_e) .. O_e + floor((i+1)*c_e/r_e)
  // (c_e and O_e counted over the kept rows)
  const int r = counts[e], F = first_slot[e];
  const int c_e = min(hist[e], cap_of(e));
  for (int i = threadIdx.x; i < r; i += DT)
    slot_offsets[F + i] = Ok_e + (int)(((long long)i * c_e) / r);
  if (e == E - 1 && threadIdx.x == 0) slot_offsets[S] = Ok_e + c_e;
  if (tab && threadIdx.x == 0) {
    tab[3 * e] = O_e;
    tab[3 * e + 1] = Ok_e;
    tab[3 * e + 2] = cap_of(e);
  }
}

__global__ __launch_bounds__(DT) void chunk_rank_kernel(const int32_t* __restrict__ cls, int A, int E,
                                                        const int32_t* __restrict__ bases,
                                                        int32_t* __restrict__ row_of_assign,
                                                        int32_t* __restrict__ assign_of_row,
                                                        const int32_t* __restrict__ tab) {
  extern __shared__ int32_t sm[];
  int32_t* running = sm;           // [E] rows of class e already placed by this workgroup (+ base)
  int32_t* wcnt = sm + E;          // [4][E] per-wavefront counts of the current pass
  constexpr int NW = DT / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < E; i += DT) running[i] = bases[(size_t)blockIdx.x * E + i];
  for (int i = threadIdx.x; i < NW * E; i += DT) wcnt[i] = 0;
  __syncthreads();
  int ebits = 0;
  while ((1 << ebits) < E) ++ebits;
  const unsigned long long lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  const int base = blockIdx.x * DISPATCH_CHUNK;

  for (int p = 0; p < DPASS; ++p) {
    const int a = base + p * DT + threadIdx.x;
    const int c_raw = a < A ? cls[a] : 0;
    const bool valid = a < A && (unsigned)c_raw < (unsigned)E;   // a class outside [0,E) is skipped
    const int c = valid ? c_raw : 0;
    // lanes of this wavefront that hold the same class
    unsigned long long mask = __ballot(valid);
    for (int b = 0; b < ebits; ++b) {
      const unsigned long long bal = __ballot((c >> b) & 1);
      mask &= ((c >> b) & 1) ? bal : ~bal;
    }
    const int rank_in_wave = __popcll(mask & lt);
    if (valid && rank_in_wave == 0) wcnt[wave * E + c] = __popcll(mask);
    __syncthreads();
    if (valid) {
      int row = running[c] + rank_in_wave;
      for (int w = 0; w < wave; ++w) row += wcnt[w * E + c];
      if (tab) {
        // capacity rule: the first cap_e assignments of the class (stable order) are kept
        const int rho = row - tab[3 * c];
        row = rho < tab[3 * c + 2] ? tab[3 * c + 1] + rho : -1;
      }
      row_of_assign[a] = row;
      if ((unsigned)row < (unsigned)A) assign_of_row[row] = a;   // false if dropped (or hist disagrees with idx)
    }
    __syncthreads();
    for (int i = threadIdx.x; i < E; i += DT) {
      int s = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) { s += wcnt[w * E + i]; wcnt[w * E + i] = 0; }
      running[i] += s;
    }
    __syncthreads();
  }
}

// Xp[row_of_assign[t*k + j]] = X[t] for every choice j of token t, rows of `vec_per_row`
// 16-byte pieces.  Walking the tokens (not the rows) reads every token once, whatever k is;
// the k destination rows are whole contiguous rows.  Dropped assignments (row -1) are skipped.
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4* __restrict__ src,
                                                           uint4* __restrict__ dst,
                                                           const int32_t* __restrict__ roa, int k,
                                                           long long n_vec, int vec_per_row) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n_vec;
       i += (long long)gridDim.x * 256) {
    const long long t = i / vec_per_row;
    const int c = (int)(i - t * vec_per_row);
    const uint4 x = src[i];
    for (int j = 0; j < k; ++j) {
      const long long row = roa[t * k + j];
      if (row >= 0) dst[row * vec_per_row + c] = x;
    }
  }
}

struct f8 { float v[8]; };

template <bool BF16>
__device__ __forceinline__ int load_piece(const void* p, long long piece, float (&out)[8]) {
  if (BF16) {
    const uint4 q = reinterpret_cast<const uint4*>(p)[piece];
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
    return 8;
  } else {
    const float4 q = reinterpret_cast<const float4*>(p)[piece];
    out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    return 4;
  }
}

template <bool BF16>
__device__ __forceinline__ void store_piece(void* p, long long piece, const float (&in)[8]) {
  if (BF16) {
    uint4 q;
    q.x = pack_bf16x2(in[0], in[1]); q.y = pack_bf16x2(in[2], in[3]);
    q.z = pack_bf16x2(in[4], in[5]); q.w = pack_bf16x2(in[6], in[7]);
    reinterpret_cast<uint4*>(p)[piece] = q;
  } else {
    reinterpret_cast<float4*>(p)[piece] = make_float4(in[0], in[1], in[2], in[3]);
  }
}

// out[t] = sum_j w[t,j] * src[row_of_assign[t*k+j]]   (w == nullptr: plain sum)
template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const void* __restrict__ src,
                                                      const int32_t* __restrict__ roa,
                                                      const float* __restrict__ w,
                                                      void* __restrict__ out, int T, int k,
                                                      int pieces_per_row) {
  constexpr int PW = BF16 ? 8 : 4;
  const long long n = (long long)T * pieces_per_row;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n;
       i += (long long)gridDim.x * 256) {
    const long long t = i / pieces_per_row;
    const int c = (int)(i - t * pieces_per_row);
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = 0; j < k; ++j) {
      const long long row = roa[t * k + j];
      if (row < 0) continue;   // dropped by the capacity rule: contributes nothing
      const float g = w ? w[t * k + j] : 1.f;
      float x[8];
      load_piece<BF16>(src, row * pieces_per_row + c, x);
#pragma unroll
      for (int q = 0; q < PW; ++q) acc[q] = fmaf(g, x[q], acc[q]);
    }
    store_piece<BF16>(out, i, acc);
  }
}

// One wavefront per token: dYp[row] = gate*dY[t] and dgate[t,j] = <dY[t], Yp[row]>.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_bwd_kernel(const void* __restrict__ dY,
                                                          const void* __restrict__ Yp,
                                                          const int32_t* __restrict__ roa,
                                                          const float* __restrict__ gate,
                                                          void* __restrict__ dYp,
                                                          float* __restrict__ dgate, int T, int k,
                                                          int pieces_per_row) {
  constexpr int PW = BF16 ? 8 : 4;
  const int lane = threadIdx.x & 63;
  const long long wave0 = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  for (long long t = wave0; t < T; t += (long long)gridDim.x * 4) {
    for (int j = 0; j < k; ++j) {
      const long long row = roa[t * k + j];
      if (row < 0) {   // dropped by the capacity rule: the output does not depend on this gate
        if (lane == 0) dgate[t * k + j] = 0.f;
        continue;
      }
      const float g = gate[t * k + j];
      float dot = 0.f;
      for (int c = lane; c < pieces_per_row; c += 64) {
        float dy[8], yp[8], o[8];
        load_piece<BF16>(dY, t * pieces_per_row + c, dy);
        load_piece<BF16>(Yp, row * pieces_per_row + c, yp);
#pragma unroll
        for (int q = 0; q < PW; ++q) {
          dot = fmaf(dy[q], yp[q], dot);
          o[q] = g * dy[q];
        }
        store_piece<BF16>(dYp, row * pieces_per_row + c, o);
      }
      for (int m = 32; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, 64);
      if (lane == 0) dgate[t * k + j] = dot;
    }
  }
}

// Device address of `scratch` on `device`, which must be the current device: looked up once per
// device and kept (each GPU holds its own copy of the array at its own address).
int static_scratch_address(int device, void** out) {
  constexpr int MAX_DEV = 64;
  static std::mutex mu;
  static void* addr[MAX_DEV] = {};
  *out = nullptr;
  if (device < 0 || device >= MAX_DEV) {
    set_error("symi_create: device ordinal %d outside [0, %d)", device, MAX_DEV);
    return SYMI_EUNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      set_error("symi_create: hipGetSymbolAddress of the static scratch failed on device %d: %s", device,
                hipGetErrorString(e));
      return SYMI_EHIP;
    }
    addr[device] = p;
  }
  *out = addr[device];
  return SYMI_OK;
}

static int grid_for(long long work_items, int per_block) {
  long long g = (work_items + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > 16384) g = 16384;
  return (int)g;
}

}  // namespace symi

using namespace symi;

static int dispatch_impl(const char* who, const symi_ctx* ctx, int slot_cap, const void* X,
                         const int32_t* idx, const int32_t* hist, const int32_t* counts,
                         const int32_t* first_slot, int32_t* row_of_assign, int32_t* assign_of_row,
                         int32_t* slot_offsets, void* Xp, void* ws, void* stream) {
  SYMI_ENTER(ctx, who);
  SYMI_REQUIRE(hist && counts && first_slot && slot_offsets && ws, who, "NULL pointer");
  SYMI_REQUIRE(cfg->T == 0 || (X && idx && row_of_assign && assign_of_row && Xp), who, "NULL pointer");
  hipStream_t st = as_stream(stream);
  const int E = cfg->E, A = cfg->T * cfg->k;
  const WsLayout& L = ctx->L;
  int32_t* blk = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.blk_counts);
  int32_t* tab = slot_cap > 0 ? reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.class_tab) : nullptr;
  const int nblk = cdiv(A, DISPATCH_CHUNK);
  if (nblk > 0)
    SYMI_TIMED(ctx, K_CHUNK_COUNT, st, (chunk_count_kernel<<<nblk, DT, E * sizeof(int32_t), st>>>(idx, A, E, blk)));
  SYMI_TIMED(ctx, K_CHUNK_SCAN, st, (chunk_scan_kernel<<<E, DT, 0, st>>>(blk, nblk, E, cfg->S_tot, A, hist, counts,
                                                                    first_slot, slot_offsets, slot_cap, tab)));
  if (nblk > 0) {
    SYMI_TIMED(ctx, K_CHUNK_RANK, st, (chunk_rank_kernel<<<nblk, DT, (size_t)(1 + DT / 64) * E * sizeof(int32_t), st>>>(
        idx, A, E, blk, row_of_assign, assign_of_row, tab)));
    const int w = cfg->dtype == SYMI_BF16 ? 2 : 4;
    const int vpr = cfg->d * w / 16;
    const long long nvec = (long long)cfg->T * vpr;
    SYMI_TIMED(ctx, K_GATHER, st, (scatter_rows_kernel<<<grid_for(nvec, 256 * 2), 256, 0, st>>>(
        static_cast<const uint4*>(X), static_cast<uint4*>(Xp), row_of_assign, cfg->k, nvec, vpr)));
  }
  SYMI_LAUNCH_CHECK(who);
  return SYMI_OK;
}

extern "C" int symi_dispatch(const symi_ctx* ctx, const void* X, const int32_t* idx,
                             const int32_t* hist, const int32_t* counts, const int32_t* first_slot,
                             int32_t* row_of_assign, int32_t* assign_of_row, int32_t* slot_offsets,
                             void* Xp, void* ws, void* stream) {
  return dispatch_impl("symi_dispatch", ctx, 0, X, idx, hist, counts, first_slot, row_of_assign,
                       assign_of_row, slot_offsets, Xp, ws, stream);
}

extern "C" int symi_dispatch_noalloc(const symi_ctx* ctx, const void* X, const int32_t* idx,
                                     const int32_t* hist, const int32_t* counts,
                                     const int32_t* first_slot, int32_t* row_of_assign,
                                     int32_t* assign_of_row, int32_t* slot_offsets, void* Xp,
                                     void* stream) {
  const char* who = "symi_dispatch_noalloc";
  if (int rc = enter(ctx, who)) return rc;
  // a timing context creates two events per launch, which allocates
  SYMI_REQUIRE(!ctx->timing, who, "the context was created with SYMI_CTX_TIMING");
  // the same layout as the head of the caller's workspace: counts of every chunk, class table
  const size_t need = ctx->L.tile_map;
  if (need > (size_t)SYMI_DISPATCH_NOALLOC_SCRATCH_BYTES) {
    set_error("%s: T*k = %lld assignments in %d classes need %zu bytes of scratch, the static buffer holds %zu "
              "((ceil(T*k/1024)+1)*E*4 + 12*E, each rounded up to 256): use symi_dispatch with a workspace",
              who, (long long)ctx->cfg.T * ctx->cfg.k, ctx->cfg.E, need, (size_t)SYMI_DISPATCH_NOALLOC_SCRATCH_BYTES);
    return SYMI_EUNSUPPORTED;
  }
  SYMI_REQUIRE(ctx->static_scratch != nullptr, who, "the context holds no address of the static scratch");
  return dispatch_impl(who, ctx, 0, X, idx, hist, counts, first_slot, row_of_assign, assign_of_row,
                       slot_offsets, Xp, ctx->static_scratch, stream);
}

extern "C" int symi_slot_capacity(const symi_cfg* cfg, double capacity_factor) {
  if (int rc = check_cfg(cfg, "symi_slot_capacity")) return rc;
  SYMI_REQUIRE(capacity_factor > 0.0 && capacity_factor <= 1e6, "symi_slot_capacity",
               "capacity_factor must lie in (0, 1e6]");
  // slot_capacity = capacity_factor * tokens_per_batch / (s N), evaluated in binary64 in this
  // order and rounded up to whole rows
  const double x = capacity_factor * (double)((long long)cfg->T * cfg->k) / (double)cfg->S_tot;
  const double c = ceil(x);
  if (c < 1.0) return 1;
  if (c > 2147483647.0) return 2147483647;
  return (int)c;
}

extern "C" int symi_dispatch_capacity(const symi_ctx* ctx, int slot_capacity, const void* X,
                                      const int32_t* idx, const int32_t* hist, const int32_t* counts,
                                      const int32_t* first_slot, int32_t* row_of_assign,
                                      int32_t* assign_of_row, int32_t* slot_offsets, void* Xp,
                                      void* ws, void* stream) {
  SYMI_REQUIRE(slot_capacity >= 1, "symi_dispatch_capacity", "slot_capacity must be >= 1");
  return dispatch_impl("symi_dispatch_capacity", ctx, slot_capacity, X, idx, hist, counts, first_slot,
                       row_of_assign, assign_of_row, slot_offsets, Xp, ws, stream);
}

extern "C" int symi_dispatch_bwd(const symi_ctx* ctx, const void* dXp, const int32_t* row_of_assign,
                                 void* dX, void* stream) {
  SYMI_ENTER(ctx, "symi_dispatch_bwd");
  if (cfg->T == 0) return SYMI_OK;
  SYMI_REQUIRE(dXp && row_of_assign && dX, "symi_dispatch_bwd", "NULL pointer");
  hipStream_t st = as_stream(stream);
  if (cfg->dtype == SYMI_BF16) {
    const int ppr = cfg->d / 8;
    SYMI_TIMED(ctx, K_DISPATCH_BWD, st, (combine_kernel<true><<<grid_for((long long)cfg->T * ppr, 256), 256, 0, st>>>(
        dXp, row_of_assign, nullptr, dX, cfg->T, cfg->k, ppr)));
  } else {
    const int ppr = cfg->d / 4;
    SYMI_TIMED(ctx, K_DISPATCH_BWD, st, (combine_kernel<false><<<grid_for((long long)cfg->T * ppr, 256), 256, 0, st>>>(
        dXp, row_of_assign, nullptr, dX, cfg->T, cfg->k, ppr)));
  }
  SYMI_LAUNCH_CHECK("symi_dispatch_bwd");
  return SYMI_OK;
}

extern "C" int symi_combine(const symi_ctx* ctx, const void* Yp, const int32_t* row_of_assign,
                            const float* gate, void* Y, void* stream) {
  SYMI_ENTER(ctx, "symi_combine");
  if (cfg->T == 0) return SYMI_OK;
  SYMI_REQUIRE(Yp && row_of_assign && gate && Y, "symi_combine", "NULL pointer");
  hipStream_t st = as_stream(stream);
  if (cfg->dtype == SYMI_BF16) {
    const int ppr = cfg->d / 8;
    SYMI_TIMED(ctx, K_COMBINE, st, (combine_kernel<true><<<grid_for((long long)cfg->T * ppr, 256), 256, 0, st>>>(
        Yp, row_of_assign, gate, Y, cfg->T, cfg->k, ppr)));
  } else {
    const int ppr = cfg->d / 4;
    SYMI_TIMED(ctx, K_COMBINE, st, (combine_kernel<false><<<grid_for((long long)cfg->T * ppr, 256), 256, 0, st>>>(
        Yp, row_of_assign, gate, Y, cfg->T, cfg->k, ppr)));
  }
  SYMI_LAUNCH_CHECK("symi_combine");
  return SYMI_OK;
}

extern "C" int symi_combine_bwd(const symi_ctx* ctx, const void* dY, const void* Yp,
                                const int32_t* row_of_assign, const float* gate, void* dYp,
                                float* dgate, void* stream) {
  SYMI_ENTER(ctx, "symi_combine_bwd");
  if (cfg->T == 0) return SYMI_OK;
  SYMI_REQUIRE(dY && Yp && row_of_assign && gate && dYp && dgate, "symi_combine_bwd", "NULL pointer");
  hipStream_t st = as_stream(stream);
  if (cfg->dtype == SYMI_BF16)
    SYMI_TIMED(ctx, K_COMBINE_BWD, st, (combine_bwd_kernel<true><<<grid_for(cfg->T, 4), 256, 0, st>>>(
        dY, Yp, row_of_assign, gate, dYp, dgate, cfg->T, cfg->k, cfg->d / 8)));
  else
    SYMI_TIMED(ctx, K_COMBINE_BWD, st, (combine_bwd_kernel<false><<<grid_for(cfg->T, 4), 256, 0, st>>>(
        dY, Yp, row_of_assign, gate, dYp, dgate, cfg->T, cfg->k, cfg->d / 4)));
  SYMI_LAUNCH_CHECK("symi_combine_bwd");
  return SYMI_OK;
}
