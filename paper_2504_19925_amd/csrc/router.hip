// symi_router_fwd / symi_router_bwd: the learned gate network in front of symi_route
// (paper Sec. 2.1: the router scores every token against every expert class):
//   logits = X Wr^T + b          dWr = dlogits^T X,  db = sum_t dlogits,  dX += dlogits Wr
// Three skinny products (one side is E <= 1024 wide) that share one small tiled kernel:
// 128 x 128 output tile, 4 wavefronts of 64 x 64 (2 x 2 MFMA 32x32x16 bf16 tiles), reduction
// step 64.  Operands pass through registers into LDS (rows padded to 144 bytes; the next
// step's global loads are in flight while the current one feeds the MFMAs) so that either
// side may be bf16 or fp32 in memory and reduction-contiguous (LDS tile [row][k], fragments
// are plain 16-byte reads) or reduction-strided (LDS tile [k][row] as in memory, fragments come
// from the transposing LDS read ds_read_b64_tr_b16); several workgroups per compute unit hide
// the latency.
// The weight gradient's reduction runs over all T tokens: it is cut into chunks of at least
// 512 tokens whose partial products are summed by a second kernel in a fixed order.
// With E <= 128 (a multiple of 8) the two backward products run in one kernel that reads X,
// dX and dlogits once (router_bwd_fused_kernel below); other E take the shared kernel twice.
// fp32 configurations take a plain FMA kernel (one output per thread) instead.
#include <type_traits>

#include "common.h"

namespace symi {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 rbf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float rfloatx16;

constexpr int RT = 128;        // tile rows and columns
constexpr int RK = 64;         // reduction step
constexpr int RLD = RK + 8;    // padded LDS row of a [row][k] tile (elements; 144 B)
constexpr int RLS = RT + 32;   // padded LDS row of a [k][row] tile (320 B: four k-rows cover 64 banks)
constexpr int RTILE = RT * RLD > RK * RLS ? RT * RLD : RK * RLS;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short rshortx4;
typedef unsigned int ru32x4 __attribute__((ext_vector_type(4)));
constexpr int RCHUNK = 512;    // tokens per partial weight gradient, at least

enum { R_FWD = 0, R_DX = 1, R_DW = 2 };

struct RouterParams {
  const void* X;        // [T,d] activations (bf16)
  const void* Wr;       // [E,d] router weights (bf16)
  const float* b;       // [E] or null
  const float* dl;      // [T,E] dlogits
  float* logits;        // [T,E]
  void* dX;             // [T,d] accumulated into
  float* partial;       // [nchunk,E,d]
  int T, E, d;
  int chunk;            // tokens per partial weight gradient
};

__device__ __forceinline__ uint4 pack8(const float (&v)[8]) {
  return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                    pack_bf16x2(v[6], v[7]));
}

// 8 consecutive reduction indices k..k+7 of operand row `r`, as bf16, zero outside.
//   contiguous bf16:  src[r*ld + k ..]            strided bf16:  src[(k+i)*ld + r]
//   contiguous fp32:  src[r*ld + k ..] converted  strided fp32:  src[(k+i)*ld + r] converted
template <bool CONTIG, bool F32>
__device__ __forceinline__ uint4 load8(const void* src, long long ld, int r, int rows, int k, int kend) {
  if (r >= rows || k >= kend) return make_uint4(0, 0, 0, 0);
  float v[8];
  if (CONTIG && !F32 && k + 8 <= kend) {
    return *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(src) + (long long)r * ld + k);
  }
  if (CONTIG && F32 && k + 8 <= kend && (ld & 3) == 0) {
    const float4 a = *reinterpret_cast<const float4*>(static_cast<const float*>(src) + (long long)r * ld + k);
    const float4 c = *reinterpret_cast<const float4*>(static_cast<const float*>(src) + (long long)r * ld + k + 4);
    return make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(c.x, c.y), pack_bf16x2(c.z, c.w));
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const long long at = CONTIG ? (long long)r * ld + k + i : (long long)(k + i) * ld + r;
    if (k + i < kend)
      v[i] = F32 ? static_cast<const float*>(src)[at] : bf16_to_f32(static_cast<const uint16_t*>(src)[at]);
    else
      v[i] = 0.f;
  }
  return pack8(v);
}

// A reduction-strided operand (memory [k][r], r contiguous) is fetched with one vector load per
// (k-row, 8 consecutive r) and stored to its [k][r] LDS tile as it is.
template <bool F32>
__device__ __forceinline__ uint4 load8_strided(const void* src, long long ld, int r, int rows, int k, int kend) {
  if (k >= kend || r >= rows) return make_uint4(0, 0, 0, 0);
  if (r + 7 < rows && (ld & (F32 ? 3 : 7)) == 0) {
    if (F32) {
      const float4 a = *reinterpret_cast<const float4*>(static_cast<const float*>(src) + (long long)k * ld + r);
      const float4 c = *reinterpret_cast<const float4*>(static_cast<const float*>(src) + (long long)k * ld + r + 4);
      return make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(c.x, c.y), pack_bf16x2(c.z, c.w));
    }
    return *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(src) + (long long)k * ld + r);
  }
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    v[i] = 0.f;
    if (r + i < rows)
      v[i] = F32 ? static_cast<const float*>(src)[(long long)k * ld + r + i]
                 : bf16_to_f32(static_cast<const uint16_t*>(src)[(long long)k * ld + r + i]);
  }
  return pack8(v);
}
template <int MODE>
__global__ __launch_bounds__(256) void router_gemm_kernel(RouterParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t As[RTILE];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[RTILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // output rows M, columns N, reduction range [kbeg, kend)
  const int M = MODE == R_DW ? p.E : p.T;
  const int N = MODE == R_FWD ? p.E : p.d;
  const int m0 = blockIdx.y * RT, n0 = blockIdx.x * RT;
  int kbeg = 0, kend = MODE == R_FWD ? p.d : MODE == R_DX ? p.E : p.T;
  if (MODE == R_DW) {
    kbeg = blockIdx.z * p.chunk;
    kend = min(p.T, kbeg + p.chunk);
  }
  rfloatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // per operand and step 128 rows x 64 reduction indices = 1024 pieces of 8, four per thread.
  // Reduction-contiguous operands: piece u -> (row u/8, k-piece u%8), committed with one 16-byte
  // LDS store at [row][k]; strided ones: piece u -> (k-row u/16, rows 8*(u%16) ..), one 16-byte
  // LDS store at [k][row].
  constexpr bool A_CONTIG = MODE != R_DW, B_CONTIG = MODE == R_FWD;
  uint4 ra[4], rb[4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int u = tid + 256 * h;
      if (MODE == R_FWD) ra[h] = load8<true, false>(p.X, p.d, m0 + (u >> 3), M, k0 + 8 * (u & 7), kend);
      else if (MODE == R_DX) ra[h] = load8<true, true>(p.dl, p.E, m0 + (u >> 3), M, k0 + 8 * (u & 7), kend);
      else ra[h] = load8_strided<true>(p.dl, p.E, m0 + 8 * (u & 15), M, k0 + (u >> 4), kend);
      if (MODE == R_FWD) rb[h] = load8<true, false>(p.Wr, p.d, n0 + (u >> 3), N, k0 + 8 * (u & 7), kend);
      else rb[h] = load8_strided<false>(MODE == R_DX ? p.Wr : p.X, p.d, n0 + 8 * (u & 15), N, k0 + (u >> 4), kend);
    }
  };
  auto commit = [&]() {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int u = tid + 256 * h;
      if (A_CONTIG) *reinterpret_cast<uint4*>(&As[(u >> 3) * RLD + 8 * (u & 7)]) = ra[h];
      else *reinterpret_cast<uint4*>(&As[(u >> 4) * RLS + 8 * (u & 15)]) = ra[h];
      if (B_CONTIG) *reinterpret_cast<uint4*>(&Bs[(u >> 3) * RLD + 8 * (u & 7)]) = rb[h];
      else *reinterpret_cast<uint4*>(&Bs[(u >> 4) * RLS + 8 * (u & 15)]) = rb[h];
    }
  };

  // R_DX adds into dX: the old values of the whole tile are requested before the reduction
  // starts, in the layout the epilogue works in (a lane: 8 consecutive columns of a row), so
  // that their latency is paid once, next to the first operand loads.  The loads carry no
  // branch (lanes past the edge read the last row / the last 8 columns; never stored).
  uint4 old[2][4];
  if (MODE == R_DX && (N & 7) == 0) {
    const uint16_t* const dXp = static_cast<const uint16_t*>(p.dX);
    const int col = min(n0 + wn * 64 + (lane & 7) * 8, N - 8);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int row = min(m0 + wm * 64 + i * 32 + it * 8 + (lane >> 3), M - 1);
        old[i][it] = *reinterpret_cast<const uint4*>(dXp + (long long)row * N + col);
      }
  }
  // the MFMAs of one 64-deep step from the two LDS tiles
  auto mma = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int ks = 0; ks < RK / 16; ++ks) {
      rbf16x8 af[2], bfr[2];
      // [row][k] tile: lane -> row lane%32, 8 k at 16*ks + 8*(lane/32).  [k][row] tile: lane =
      // 16*g + jj addresses k-row 16*ks + 8*(g>>1) + jj/4 (+4 for the second half), the 8-byte
      // piece jj%4 of rows 16*(g&1) ..; the transposing read hands it row lane%32's 4 + 4 k-values
      auto frag = [&](const uint16_t* tile, bool contig, int rbase) -> rbf16x8 {
        if (contig)
          return *reinterpret_cast<const rbf16x8*>(&tile[(rbase + (lane & 31)) * RLD + ks * 16 + 8 * (lane >> 5)]);
        const int g = lane >> 4, jj = lane & 15;
        const uint16_t* q = tile + (16 * ks + 8 * (g >> 1) + (jj >> 2)) * RLS + rbase + 16 * (g & 1) + 4 * (jj & 3);
        const rshortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) rshortx4*)((void __attribute__((address_space(3)))*)(q)));
        const rshortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) rshortx4*)((void __attribute__((address_space(3)))*)(q + 4 * RLS)));
        union { rshortx4 h[2]; rbf16x8 v; } u;
        u.h[0] = lo;
        u.h[1] = hi;
        return u.v;
      };
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = frag(As, A_CONTIG, wm * 64 + i * 32);
        bfr[i] = frag(Bs, B_CONTIG, wn * 64 + i * 32);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
  };
  if constexpr (MODE == R_FWD) {
    // The forward streams X once with few workgroups per compute unit (T / 128 of them): two
    // steps are kept in flight in two register sets.  Every load is unconditional (clamped
    // address; pieces past the reduction's end are zeroed on both sides, rows past the tile's
    // edge only reach outputs that are never stored) and the steps come in pairs, so the loop
    // has no branch and the wait for one set's loads does not wait for the other's.
    const uint16_t* const Xb = static_cast<const uint16_t*>(p.X);
    const uint16_t* const Wb = static_cast<const uint16_t*>(p.Wr);
    ru32x4 xa[2][4], xb[2][4];
    auto fetch2 = [&](auto setc, int k0) __attribute__((always_inline)) {
      constexpr int S = decltype(setc)::value;
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const int u = tid + 256 * h;
        const int kp = k0 + 8 * (u & 7), kc = min(kp, kend - 8);
        xa[S][h] = *reinterpret_cast<const ru32x4*>(Xb + (long long)min(m0 + (u >> 3), M - 1) * p.d + kc);
        xb[S][h] = *reinterpret_cast<const ru32x4*>(Wb + (long long)min(n0 + (u >> 3), N - 1) * p.d + kc);
      }
    };
    auto commit2 = [&](auto setc, int k0) __attribute__((always_inline)) {
      constexpr int S = decltype(setc)::value;
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const int u = tid + 256 * h;
        const bool in = k0 + 8 * (u & 7) < kend;   // the values are only looked at here
        const ru32x4 zero = {0u, 0u, 0u, 0u};
        *reinterpret_cast<ru32x4*>(&As[(u >> 3) * RLD + 8 * (u & 7)]) = in ? xa[S][h] : zero;
        *reinterpret_cast<ru32x4*>(&Bs[(u >> 3) * RLD + 8 * (u & 7)]) = in ? xb[S][h] : zero;
      }
    };
    const int nk2 = ((kend - kbeg + RK - 1) / RK + 1) / 2 * 2;
    fetch2(std::integral_constant<int, 0>{}, kbeg);
    fetch2(std::integral_constant<int, 1>{}, kbeg + RK);
    __builtin_amdgcn_sched_barrier(0);
    for (int s2 = 0; s2 < nk2; s2 += 2) {
      const int k0 = kbeg + s2 * RK;
      commit2(std::integral_constant<int, 0>{}, k0);
      __syncthreads();
      fetch2(std::integral_constant<int, 0>{}, k0 + 2 * RK);
      __builtin_amdgcn_sched_barrier(0);   // the requests go out here, not behind the MFMAs
      mma();
      __syncthreads();
      commit2(std::integral_constant<int, 1>{}, k0 + RK);
      __syncthreads();
      fetch2(std::integral_constant<int, 1>{}, k0 + 3 * RK);
      __builtin_amdgcn_sched_barrier(0);
      mma();
      __syncthreads();
    }
  } else {
    if (kbeg < kend) fetch(kbeg);
    for (int k0 = kbeg; k0 < kend; k0 += RK) {
      commit();
      __syncthreads();
      if (k0 + RK < kend) fetch(k0 + RK);   // in flight while this step feeds the MFMAs
      mma();
      __syncthreads();
    }
  }

  // a lane owns output row lane%32 of each 32 x 32 block and, per 8-column group g, the 4
  // columns 8g + 4*(lane/32) ..
  if (MODE == R_DX && (N & 7) == 0) {
    // dX is read, added to and written back.  In the MFMA layout an access would touch 32 rows
    // with 8 bytes each; every wavefront turns its 32 x 64 blocks around through the (now free)
    // operand tiles instead, so that a lane handles 8 consecutive columns of a row (16 bytes of
    // bf16) and an instruction covers 8 rows x 128 bytes.
    constexpr int LDT = 68;   // fp32 row of 64 columns + pad
    float* const stg = reinterpret_cast<float*>(wave < 2 ? As : Bs) + (wave & 1) * (32 * LDT);
    uint16_t* const dXp = static_cast<uint16_t*>(p.dX);
    const int r32 = lane & 31, hw = lane >> 5;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(stg + r32 * LDT + 32 * j + 8 * g + 4 * hw) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): the block is in LDS (wavefront-private area)
      const int col = n0 + wn * 64 + (lane & 7) * 8;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int rr = it * 8 + (lane >> 3);
        const int row = m0 + wm * 64 + i * 32 + rr;
        const float4 x0 = *reinterpret_cast<const float4*>(stg + rr * LDT + (lane & 7) * 8);
        const float4 x1 = *reinterpret_cast<const float4*>(stg + rr * LDT + (lane & 7) * 8 + 4);
        if (row < M && col < N) {
          const uint4 o = old[i][it];
          *reinterpret_cast<uint4*>(dXp + (long long)row * N + col) = make_uint4(
              pack_bf16x2(__uint_as_float(o.x << 16) + x0.x, __uint_as_float(o.x & 0xffff0000u) + x0.y),
              pack_bf16x2(__uint_as_float(o.y << 16) + x0.z, __uint_as_float(o.y & 0xffff0000u) + x0.w),
              pack_bf16x2(__uint_as_float(o.z << 16) + x1.x, __uint_as_float(o.z & 0xffff0000u) + x1.y),
              pack_bf16x2(__uint_as_float(o.w << 16) + x1.z, __uint_as_float(o.w & 0xffff0000u) + x1.w));
        }
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);   // the next block's writes must not pass these reads
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = m0 + wm * 64 + i * 32 + (lane & 31);
    if (row >= M) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * 64 + j * 32 + 8 * g + 4 * (lane >> 5);
        if (col >= N) continue;
        float x[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) x[c] = acc[i][j][4 * g + c];
        const long long at = (long long)row * N + col;
        if (col + 3 < N && (N & 3) == 0) {   // 4 columns at once (16 bytes fp32, 8 bytes bf16)
          if (MODE == R_FWD) {
            float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p.b) bb = make_float4(p.b[col], p.b[col + 1], p.b[col + 2], p.b[col + 3]);
            *reinterpret_cast<float4*>(p.logits + at) = make_float4(x[0] + bb.x, x[1] + bb.y, x[2] + bb.z, x[3] + bb.w);
          } else if (MODE == R_DX) {
            uint2* o = reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.dX) + at);
            const uint2 old = *o;
            *o = make_uint2(pack_bf16x2(__uint_as_float(old.x << 16) + x[0], __uint_as_float(old.x & 0xffff0000u) + x[1]),
                            pack_bf16x2(__uint_as_float(old.y << 16) + x[2], __uint_as_float(old.y & 0xffff0000u) + x[3]));
          } else {
            *reinterpret_cast<float4*>(p.partial + (long long)blockIdx.z * M * N + at) = make_float4(x[0], x[1], x[2], x[3]);
          }
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            if (col + c >= N) continue;
            if (MODE == R_FWD) {
              p.logits[at + c] = x[c] + (p.b ? p.b[col + c] : 0.f);
            } else if (MODE == R_DX) {
              uint16_t* o = static_cast<uint16_t*>(p.dX) + at + c;
              *o = f32_to_bf16(bf16_to_f32(*o) + x[c]);
            } else {
              p.partial[(long long)blockIdx.z * M * N + at + c] = x[c];
            }
          }
        }
      }
  }
}

// ---- both backward products in one pass (bf16, E <= 128 and a multiple of 8)
// Workgroup = one column tile of 128 (of d) x one chunk of tokens, walked in row blocks of 128:
//   dX[t, n] += sum_e dl[t, e] Wr[e, n]      (reduction over the classes)
//   dWr[e, n] += sum_t dl[t, e] X[t, n]      (reduction over the block's tokens, kept in the
//                                             accumulators over the whole chunk)
// The column tile of Wr stays in LDS; a block of dlogits is fetched and converted once and
// serves both products (read along e for the first, transposed for the second); X, the old dX
// values and the dlogits of the next block are in flight while the current one is worked on.
// Every global load is unconditional (clamped address, value zeroed where it must not count), so
// the compiler can count the loads in flight instead of waiting for all of them.
constexpr int FSD = RT + 8;     // dlogits block [t][e]: 272-byte rows (plain 16-byte reads are conflict-free)
constexpr int FSW = RT + 32;    // Wr and X tiles [k][n]: 320-byte rows (transposing reads are conflict-free)

__global__ __launch_bounds__(256) void router_bwd_fused_kernel(RouterParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t DLt[RT * FSD];
  __shared__ __attribute__((aligned(16))) uint16_t WRt[RT * FSW];
  __shared__ __attribute__((aligned(16))) uint16_t XT[RT * FSW];   // later the epilogue's staging
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int T = p.T, E = p.E, d = p.d;
  const int n0 = blockIdx.x * RT;
  const int t_beg = blockIdx.y * p.chunk, t_end = min(T, t_beg + p.chunk);
  const uint16_t* const X = static_cast<const uint16_t*>(p.X);
  const uint16_t* const Wr = static_cast<const uint16_t*>(p.Wr);
  uint16_t* const dX = static_cast<uint16_t*>(p.dX);

  // piece u = tid + 256 h (h < 8) of a 128 x 128 tile: row u / 16, 8 consecutive columns at 8 (u % 16)
  const int pr = tid >> 4, pc = (tid & 15) * 8;       // row of piece h: pr + 16 h
  const int ncol = min(n0 + pc, d - 8);               // clamped: columns past d are never stored
  const int ecol = min(pc, E - 8);
  const bool e_ok = pc < E;
  // epilogue layout of the dX tile: block i (32 rows), pass it: row 8 it + lane / 8, 8 columns
  const int ocol = min(n0 + wn * 64 + (lane & 7) * 8, d - 8);

  // Wr tile, once: rows e >= E are zero
#pragma unroll
  for (int h = 0; h < 8; ++h) {
    const int e = pr + 16 * h;
    uint4 w = *reinterpret_cast<const uint4*>(Wr + (long long)min(e, E - 1) * d + ncol);
    if (e >= E) w = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(&WRt[e * FSW + pc]) = w;
  }

  // two register sets: while block b is worked on, the operands of blocks b + 1 and b + 2 are
  // on their way (one set would leave a block's requests only the time of one block's MFMAs
  // and epilogue to arrive)
  float4 rd[2][8][2];   // dlogits pieces (fp32)
  ru32x4 rx[2][8];      // X pieces
  uint4 ro[2][4];       // old dX values
  auto fetch = [&](auto setc, int t0) __attribute__((always_inline)) {
    constexpr int S = decltype(setc)::value;
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      const long long t = min(t0 + pr + 16 * h, T - 1);
      const float* q = p.dl + t * E + ecol;
      rd[S][h][0] = *reinterpret_cast<const float4*>(q);
      rd[S][h][1] = *reinterpret_cast<const float4*>(q + 4);
      rx[S][h] = *reinterpret_cast<const ru32x4*>(X + t * d + ncol);
    }
  };
  auto fetch_old = [&](int t0) __attribute__((always_inline)) {   // requested behind the previous block's stores
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const long long t = min(t0 + wm * 64 + i * 32 + it * 8 + (lane >> 3), T - 1);
        ro[i][it] = *reinterpret_cast<const uint4*>(dX + t * d + ocol);
      }
  };

  rfloatx16 accw[2][2];   // dWr tile of the chunk
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) accw[i][j][r] = 0.f;

  // fragments: plain = [row][k] tile, a lane reads 8 k of row lane % 32; transposing = [k][row]
  // tile, lane 16 g + jj addresses k-row 8 (g >> 1) + jj / 4 (+4 for the second half), the
  // 8-byte piece jj % 4 of rows 16 (g & 1) .., and receives row lane % 32's 4 + 4 k-values
  auto frag_plain = [&](const uint16_t* tile, int stride, int rbase, int ks) __attribute__((always_inline)) -> rbf16x8 {
    return *reinterpret_cast<const rbf16x8*>(&tile[(rbase + (lane & 31)) * stride + ks * 16 + 8 * (lane >> 5)]);
  };
  auto frag_tr = [&](const uint16_t* tile, int stride, int rbase, int ks) __attribute__((always_inline)) -> rbf16x8 {
    const int g = lane >> 4, jj = lane & 15;
    const uint16_t* q = tile + (16 * ks + 8 * (g >> 1) + (jj >> 2)) * stride + rbase + 16 * (g & 1) + 4 * (jj & 3);
    const rshortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) rshortx4*)((void __attribute__((address_space(3)))*)(q)));
    const rshortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) rshortx4*)((void __attribute__((address_space(3)))*)(q + 4 * stride)));
    union { rshortx4 h[2]; rbf16x8 v; } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
  };

  // one row block; FULL: all its rows and columns exist and another block follows, so neither
  // the stores of the epilogue nor the requests for the next block sit under a branch (behind a
  // branch the compiler no longer knows how many memory operations are in flight, and every
  // wait for a loaded value becomes a wait for everything issued so far)
  auto block = [&](int t0, auto fullc, auto setc) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(fullc)::value;
    constexpr int S = decltype(setc)::value;
    // this block's operands to LDS; rows past T and classes past E count as zero
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      const bool ok = e_ok && t0 + pr + 16 * h < T;
      uint4 v = make_uint4(pack_bf16x2(rd[S][h][0].x, rd[S][h][0].y), pack_bf16x2(rd[S][h][0].z, rd[S][h][0].w),
                           pack_bf16x2(rd[S][h][1].x, rd[S][h][1].y), pack_bf16x2(rd[S][h][1].z, rd[S][h][1].w));
      if (!ok) v = make_uint4(0, 0, 0, 0);
      *reinterpret_cast<uint4*>(&DLt[(pr + 16 * h) * FSD + pc]) = v;
      *reinterpret_cast<ru32x4*>(&XT[(pr + 16 * h) * FSW + pc]) = rx[S][h];
    }
    __syncthreads();
    if (FULL || t0 + 2 * RT < t_end) fetch(setc, t0 + 2 * RT);   // in flight for the next two blocks
    __builtin_amdgcn_sched_barrier(0);   // the requests go out here, not behind the MFMAs

    rfloatx16 accx[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) accx[i][j][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < RT / 16; ++ks) {
      rbf16x8 af[2], bfr[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = frag_plain(DLt, FSD, wm * 64 + i * 32, ks);
        bfr[i] = frag_tr(WRt, FSW, wn * 64 + i * 32, ks);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          accx[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], accx[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int ks = 0; ks < RT / 16; ++ks) {
      rbf16x8 af[2], bfr[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = frag_tr(DLt, FSD, wm * 64 + i * 32, ks);
        bfr[i] = frag_tr(XT, FSW, wn * 64 + i * 32, ks);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          accw[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], accw[i][j], 0, 0, 0);
    }
    __syncthreads();   // nobody reads XT any more: it becomes the staging area

    // dX += : a lane owns output row lane % 32 of a 32 x 32 block and 4 columns per group of 8;
    // every wavefront turns its 32 x 64 blocks around through a private part of XT so that a lane
    // handles 8 consecutive columns of a row and a store instruction covers 8 rows x 128 bytes
    constexpr int LDT = 68;
    float* const stg = reinterpret_cast<float*>(XT) + wave * (32 * LDT);
    const int r32 = lane & 31, hw = lane >> 5;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(stg + r32 * LDT + 32 * j + 8 * g + 4 * hw) =
              make_float4(accx[i][j][4 * g], accx[i][j][4 * g + 1], accx[i][j][4 * g + 2], accx[i][j][4 * g + 3]);
      __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): wavefront-private area
      const int col = n0 + wn * 64 + (lane & 7) * 8;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int rr = it * 8 + (lane >> 3);
        const int row = t0 + wm * 64 + i * 32 + rr;
        const float4 x0 = *reinterpret_cast<const float4*>(stg + rr * LDT + (lane & 7) * 8);
        const float4 x1 = *reinterpret_cast<const float4*>(stg + rr * LDT + (lane & 7) * 8 + 4);
        if (FULL || (row < T && col < d)) {
          const uint4 o = ro[i][it];
          *reinterpret_cast<uint4*>(dX + (long long)row * d + col) = make_uint4(
              pack_bf16x2(__uint_as_float(o.x << 16) + x0.x, __uint_as_float(o.x & 0xffff0000u) + x0.y),
              pack_bf16x2(__uint_as_float(o.y << 16) + x0.z, __uint_as_float(o.y & 0xffff0000u) + x0.w),
              pack_bf16x2(__uint_as_float(o.z << 16) + x1.x, __uint_as_float(o.z & 0xffff0000u) + x1.y),
              pack_bf16x2(__uint_as_float(o.w << 16) + x1.z, __uint_as_float(o.w & 0xffff0000u) + x1.w));
        }
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);   // the next block's writes must not pass these reads
    }
    if (FULL || t0 + RT < t_end) fetch_old(t0 + RT);
    __syncthreads();   // the staging area is XT again
  };
  const std::integral_constant<int, 0> set0;
  const std::integral_constant<int, 1> set1;
  if (t_beg < t_end) {
    fetch(set0, t_beg);
    fetch_old(t_beg);
    fetch(set1, t_beg + RT);   // clamped to existing rows if there is no second block
  }
  int t0 = t_beg;
  if (n0 + RT <= d)   // pairs of full blocks that are followed by two more blocks
    for (; t0 + 3 * RT < t_end; t0 += 2 * RT) {
      block(t0, std::true_type{}, set0);
      block(t0 + RT, std::true_type{}, set1);
    }
  while (t0 < t_end) {
    block(t0, std::false_type{}, set0);
    t0 += RT;
    if (t0 >= t_end) break;
    block(t0, std::false_type{}, set1);
    t0 += RT;
  }

  // the chunk's partial weight gradient: row e = lane % 32 of each 32 x 32 block, 4 columns per group
  float* const part = p.partial + (long long)blockIdx.y * E * d;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int e = wm * 64 + i * 32 + (lane & 31);
    if (e >= E) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * 64 + j * 32 + 8 * g + 4 * (lane >> 5);
        if (col < d)   // d is a multiple of 8: the four columns are inside together
          *reinterpret_cast<float4*>(part + (long long)e * d + col) =
              make_float4(accw[i][j][4 * g], accw[i][j][4 * g + 1], accw[i][j][4 * g + 2], accw[i][j][4 * g + 3]);
      }
  }
}

// dWr[e,n] = sum over chunks of partial[chunk,e,n], chunks in ascending order
__global__ __launch_bounds__(256) void router_reduce_kernel(const float* __restrict__ partial, int nchunk,
                                                            long long n, float* __restrict__ dWr) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
    float s = 0.f;
    for (int c = 0; c < nchunk; ++c) s += partial[(long long)c * n + i];
    dWr[i] = s;
  }
}

// db[e] = sum_t dl[t,e] in two fixed-order stages: per chunk of 256 tokens, then over the
// chunks.  First stage: threads along e (every row is read contiguously), and where E < 256
// the rows of the chunk are dealt out over 256 / E groups of threads whose sums are added in
// group order; eight independent loads in flight per thread.
__global__ __launch_bounds__(256) void router_bias_partial_kernel(const float* __restrict__ dl, int T, int E,
                                                                  float* __restrict__ part) {
  __shared__ double red[256];
  const int tid = threadIdx.x;
  const int t0 = blockIdx.x * 256, t1 = min(T, t0 + 256);
  const int cols = min(E, 256), groups = 256 / cols;
  const int g = tid / cols, ec = tid - g * cols;
  for (int eb = 0; eb < E; eb += cols) {   // the same trip count for every thread
    const int e = eb + ec;
    double s = 0.0;   // the summands cancel heavily: accumulate in binary64
    if (g < groups && e < E) {
#pragma unroll 8
      for (int t = t0 + g; t < t1; t += groups) s += (double)dl[(long long)t * E + e];
    }
    red[tid] = s;
    __syncthreads();
    if (g == 0 && e < E) {
      for (int q = 1; q < groups; ++q) s += red[q * cols + ec];
      part[(long long)blockIdx.x * E + e] = (float)s;
    }
    __syncthreads();
  }
}
// Second stage, one workgroup per class: thread c adds chunks c, c + 256, ... in ascending
// order, then the 256 sums are added pairwise in a fixed tree.
__global__ __launch_bounds__(256) void router_bias_final_kernel(const float* __restrict__ part, int nchunk,
                                                                int E, float* __restrict__ db) {
  __shared__ double red[256];
  const int e = blockIdx.x, tid = threadIdx.x;
  double s = 0.0;
  for (int c = tid; c < nchunk; c += 256) s += (double)part[(long long)c * E + e];
  red[tid] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) red[tid] += red[tid + w];
    __syncthreads();
  }
  if (tid == 0) db[e] = (float)red[0];
}

// ---- fp32 configurations: one output element per thread, plain FMAs in index order
__global__ __launch_bounds__(256) void router_fwd_f32_kernel(const float* __restrict__ X,
                                                             const float* __restrict__ Wr,
                                                             const float* __restrict__ b,
                                                             float* __restrict__ logits, int T, int E, int d) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)T * E) return;
  const int t = (int)(i / E), e = (int)(i - (long long)t * E);
  float s = 0.f;
  for (int k = 0; k < d; ++k) s = fmaf(X[(long long)t * d + k], Wr[(long long)e * d + k], s);
  logits[i] = s + (b ? b[e] : 0.f);
}
__global__ __launch_bounds__(256) void router_dx_f32_kernel(const float* __restrict__ dl,
                                                            const float* __restrict__ Wr,
                                                            float* __restrict__ dX, int T, int E, int d) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)T * d) return;
  const int t = (int)(i / d), n = (int)(i - (long long)t * d);
  float s = 0.f;
  for (int e = 0; e < E; ++e) s = fmaf(dl[(long long)t * E + e], Wr[(long long)e * d + n], s);
  dX[i] += s;
}
__global__ __launch_bounds__(256) void router_dw_f32_kernel(const float* __restrict__ dl,
                                                            const float* __restrict__ X,
                                                            float* __restrict__ dWr, int T, int E, int d) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)E * d) return;
  const int e = (int)(i / d), n = (int)(i - (long long)e * d);
  // two-level sum: 16-token partial sums first (keeps the rounding error of a long
  // reduction near sqrt(T/16) ulps)
  float s = 0.f;
  for (int t0 = 0; t0 < T; t0 += 16) {
    float part = 0.f;
    const int t1 = min(T, t0 + 16);
    for (int t = t0; t < t1; ++t) part = fmaf(dl[(long long)t * E + e], X[(long long)t * d + n], part);
    s += part;
  }
  dWr[i] = s;
}

}  // namespace symi

using namespace symi;

extern "C" int symi_router_fwd(const symi_ctx* ctx, const void* X, const void* Wr, const float* b,
                               float* logits, void* stream) {
  SYMI_ENTER(ctx, "symi_router_fwd");
  if (cfg->T == 0) return SYMI_OK;
  SYMI_REQUIRE(X && Wr && logits, "symi_router_fwd", "NULL pointer");
  hipStream_t st = as_stream(stream);
  const int T = cfg->T, E = cfg->E, d = cfg->d;
  if (cfg->dtype == SYMI_BF16) {
    RouterParams p = {};
    p.X = X; p.Wr = Wr; p.b = b; p.logits = logits; p.T = T; p.E = E; p.d = d;
    SYMI_TIMED(ctx, K_ROUTER_FWD, st, (router_gemm_kernel<R_FWD><<<dim3(cdiv(E, RT), cdiv(T, RT)), 256, 0, st>>>(p)));
  } else {
    SYMI_TIMED(ctx, K_ROUTER_FWD, st, (router_fwd_f32_kernel<<<cdiv((long long)T * E, 256), 256, 0, st>>>(
        static_cast<const float*>(X), static_cast<const float*>(Wr), b, logits, T, E, d)));
  }
  SYMI_LAUNCH_CHECK("symi_router_fwd");
  return SYMI_OK;
}

extern "C" int symi_router_bwd(const symi_ctx* ctx, const void* X, const void* Wr, const float* dlogits,
                               float* dWr, float* db, void* dX, void* ws, void* stream) {
  SYMI_ENTER(ctx, "symi_router_bwd");
  SYMI_REQUIRE(dWr && ws, "symi_router_bwd", "NULL pointer");
  SYMI_REQUIRE(cfg->T == 0 || (X && Wr && dlogits && dX), "symi_router_bwd", "NULL pointer");
  hipStream_t st = as_stream(stream);
  const int T = cfg->T, E = cfg->E, d = cfg->d;
  const WsLayout& L = ctx->L;
  if (cfg->dtype == SYMI_BF16) {
    RouterParams p = {};
    p.X = X; p.Wr = Wr; p.dl = dlogits; p.dX = dX; p.T = T; p.E = E; p.d = d;
    p.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + L.router_partial);
    // chunks of 512 tokens, doubled while that leaves more than 1024 workgroups: fewer partial
    // products to write and read back (a function of the configuration only: same bits every run)
    const int tiles = cdiv(d, RT) * cdiv(E, RT);
    int chunk = RCHUNK;
    while ((long long)cdiv(T, chunk) * tiles > 1024 && chunk < 16384) chunk *= 2;
    const bool fused = E <= RT && E % 8 == 0;
    if (fused) {
      // one workgroup per compute unit at a time (its LDS): as many chunks as give every unit
      // one workgroup, each then walks its row blocks with the next one in flight
      const int per = std::max(1, ctx->cus / cdiv(d, RT));
      chunk = std::max(RCHUNK, cdiv(cdiv(T, per), RT) * RT);
    }
    p.chunk = chunk;
    const int nchunk = cdiv(T, chunk);
    if (T > 0 && fused) {
      // both products in one pass over X, dX and dlogits
      SYMI_TIMED(ctx, K_ROUTER_DX, st, (router_bwd_fused_kernel<<<dim3(cdiv(d, RT), nchunk), 256, 0, st>>>(p)));
    } else if (T > 0) {
      SYMI_TIMED(ctx, K_ROUTER_DX, st, (router_gemm_kernel<R_DX><<<dim3(cdiv(d, RT), cdiv(T, RT)), 256, 0, st>>>(p)));
      SYMI_TIMED(ctx, K_ROUTER_DW, st, (router_gemm_kernel<R_DW><<<dim3(cdiv(d, RT), cdiv(E, RT), nchunk), 256, 0, st>>>(p)));
    }
    const long long n = (long long)E * d;
    SYMI_TIMED(ctx, K_ROUTER_DW, st, (router_reduce_kernel<<<cdiv(n, 256), 256, 0, st>>>(p.partial, nchunk, n, dWr)));
  } else {
    if (T > 0)
      SYMI_TIMED(ctx, K_ROUTER_DX, st, (router_dx_f32_kernel<<<cdiv((long long)T * d, 256), 256, 0, st>>>(
          dlogits, static_cast<const float*>(Wr), static_cast<float*>(dX), T, E, d)));
    SYMI_TIMED(ctx, K_ROUTER_DW, st, (router_dw_f32_kernel<<<cdiv((long long)E * d, 256), 256, 0, st>>>(
        dlogits, static_cast<const float*>(X), dWr, T, E, d)));
  }
  if (db) {
    float* part = reinterpret_cast<float*>(static_cast<char*>(ws) + L.router_bias_partial);
    const int nb = cdiv(T, 256);
    if (nb > 0)
      SYMI_TIMED(ctx, K_ROUTER_DW, st, (router_bias_partial_kernel<<<nb, 256, 0, st>>>(dlogits, T, E, part)));
    SYMI_TIMED(ctx, K_ROUTER_DW, st, (router_bias_final_kernel<<<E, 256, 0, st>>>(part, nb, E, db)));
  }
  SYMI_LAUNCH_CHECK("symi_router_bwd");
  return SYMI_OK;
}
