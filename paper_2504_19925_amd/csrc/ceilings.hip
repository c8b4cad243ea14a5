// libsymi_ceilings.so: in-bounds microbenchmarks of what one MI355X sustains with the
// instruction and access mixes of the hot path's kernels.  Measurement aid only (bench.py
// --ceiling): not part of libsymi, nothing of the method is computed here.
//
//   symi_ceiling_mfma        16 independent MFMA 32x32x16 bf16 chains per wavefront, operands in
//                            registers: the rate of the matrix pipes alone with the given data
//   symi_ceiling_gemm_loop   the reduction loop of the grouped GEMM (256x256 tile, 64-deep steps,
//                            direct-to-LDS loads into two stages in the scalar-base form with one
//                            M0 write per operand and stage, fragment reads by hand, four phases
//                            of 16 MFMAs) on a plain C = A B^T, whole or with one of its three
//                            ingredients taken out
//   symi_ceiling_adam_streams the Adam step's memory streams (4 fp32 reads, 3 fp32 writes, bf16
//                            replica writes) without the optimizer's meaning, in three layouts
// All pointers are device pointers of the caller, all launches go to the caller's stream.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));

#define GPTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define LPTR(p) ((void __attribute__((address_space(3)))*)(p))

namespace {

template <int V> struct IC { static constexpr int value = V; };

// ------------------------------------------------------------------ MFMA from registers
__global__ __launch_bounds__(256) void mfma_regs_kernel(const uint16_t* __restrict__ operands,
                                                        float* __restrict__ out, int iters) {
  // every lane takes its own 16 + 16 bytes of operand data (random or zero: the power drawn by
  // the matrix pipes, and with it the clock, depends on the bits)
  const uint4 qa = reinterpret_cast<const uint4*>(operands)[(blockIdx.x * 256 + threadIdx.x) * 2];
  const uint4 qb = reinterpret_cast<const uint4*>(operands)[(blockIdx.x * 256 + threadIdx.x) * 2 + 1];
  const bf16x8 a = __builtin_bit_cast(bf16x8, qa), b = __builtin_bit_cast(bf16x8, qb);
  floatx16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// ------------------------------------------------------------------ the GEMM's reduction loop
constexpr int BM = 256, BN = 256, BK = 64;

template <int OFF>
__device__ __forceinline__ bf16x8 ds128(unsigned addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

// VARIANT 0: the whole loop; 1: no global loads (LDS reads + MFMA); 2: no LDS reads (loads +
// MFMA on whatever the fragment registers hold); 3: no MFMA (loads + LDS reads).
// C = A[M,K] B[N,K]^T with M, N multiples of 256 and K a multiple of 128 (checked by the host).
template <int VARIANT>
__global__ __launch_bounds__(256) void gemm_loop_kernel(const uint16_t* __restrict__ A,
                                                        const uint16_t* __restrict__ B,
                                                        uint16_t* __restrict__ C, int M, int N, int K) {
  constexpr bool DMA = VARIANT != 1, LDS = VARIANT != 2, MFMA = VARIANT != 3;
  __shared__ __attribute__((aligned(1024))) uint16_t sA0[BM * BK];
  __shared__ __attribute__((aligned(1024))) uint16_t sB0[BN * BK];
  __shared__ __attribute__((aligned(1024))) uint16_t sA1[BM * BK];
  __shared__ __attribute__((aligned(1024))) uint16_t sB1[BN * BK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int lrow = lane >> 3, pch = lane & 7;
  // the loads in the form the grouped GEMM uses: scalar base (operand + step, 4 KB low), 32-bit
  // per-lane byte offset, immediate; the LDS base (M0) written once per operand and stage
  unsigned vo[2][8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int par = j & 1;
    const int kc = pch ^ ((4 * par + (lane >> 4)) & 7);
    const long long rowA = m0 + wave * 64 + par * 8 + lrow + (j >> 1) * 16, rowB = n0 + wave * 64 + par * 8 + lrow + (j >> 1) * 16;
    vo[0][j] = (unsigned)((rowA * K + kc * 8) * 2 + 4096 - (j - 4) * 1024);
    vo[1][j] = (unsigned)((rowB * K + kc * 8) * 2 + 4096 - (j - 4) * 1024);
  }
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // q = 0..7: instruction q of the left operand, 8..15: instruction q - 8 of the right one
  auto dma_q = [&](uint16_t* sA, uint16_t* sB, int k0, auto qc) {
    constexpr int Q = decltype(qc)::value, j = Q & 7;
    constexpr bool right = Q >= 8;
    if (j == 0) {
      const unsigned l = (unsigned)(size_t)LPTR((right ? sB : sA) + wave_u * 64 * BK + 4 * 8 * BK);
      asm volatile("s_mov_b32 m0, %0" ::"s"(l) : "memory");
    }
    const char* sb = reinterpret_cast<const char*>(right ? B : A) + (long long)k0 * 2 - 4096;   // wave-uniform
    const unsigned v = vo[right ? 1 : 0][j];
    asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(v), "s"(sb), "n"((j - 4) * 1024) : "memory");
  };
  floatx16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lsw = (lane >> 1) & 7;
  unsigned aad[2][4], bad[2][4];   // LDS byte address of this lane's fragment piece per stage and sub-step
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int koff = (((ks * 2 + (lane >> 5)) ^ lsw) * 8);
    const int arow = (wm * 128 + (lane & 31)) * BK, brow = (wn * 128 + (lane & 31)) * BK;
    aad[0][ks] = (unsigned)(size_t)LPTR(sA0) + 2u * (arow + koff);
    aad[1][ks] = (unsigned)(size_t)LPTR(sA1) + 2u * (arow + koff);
    bad[0][ks] = (unsigned)(size_t)LPTR(sB0) + 2u * (brow + koff);
    bad[1][ks] = (unsigned)(size_t)LPTR(sB1) + 2u * (brow + koff);
  }
  bf16x8 fa[2][4], fb[2][4];
  auto load_frags = [&](auto bufc, unsigned aa, unsigned ba) {
    constexpr int bu = decltype(bufc)::value;
    fa[bu][0] = ds128<0>(aa); fb[bu][0] = ds128<0>(ba);
    fa[bu][1] = ds128<4096>(aa); fb[bu][1] = ds128<4096>(ba);
    fa[bu][2] = ds128<8192>(aa); fb[bu][2] = ds128<8192>(ba);
    fa[bu][3] = ds128<12288>(aa); fb[bu][3] = ds128<12288>(ba);
  };
  // one phase = the 16 MFMAs of one 16-deep sub-step of step t (stage S = t & 1)
  auto phase = [&](auto ksc, auto sc, int t) {
    constexpr int KS = decltype(ksc)::value, S = decltype(sc)::value;
    constexpr int bu = KS & 1;
    uint16_t* const cA = S ? sA1 : sA0; uint16_t* const cB = S ? sB1 : sB0;
    uint16_t* const oA = S ? sA0 : sA1; uint16_t* const oB = S ? sB0 : sB1;
    __builtin_amdgcn_s_waitcnt(0xC07F);            // fragments of this phase have arrived
    if (KS == 3) {
      __builtin_amdgcn_s_waitcnt(0x0F70);          // my loads of step t+1 have landed
      __builtin_amdgcn_s_barrier();                // ... everybody's have, and stage S is no longer read
    }
    __builtin_amdgcn_sched_barrier(0);
    if (LDS) load_frags(IC<bu ^ 1>{}, KS == 3 ? aad[S ^ 1][0] : aad[S][(KS + 1) & 3], KS == 3 ? bad[S ^ 1][0] : bad[S][(KS + 1) & 3]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (MFMA) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[bu][j], fa[bu][i], acc[i][j], 0, 0, 0);
        else asm volatile("" :: "v"(fb[bu][j]), "v"(fa[bu][i]));
      }
      if (DMA && (KS == 3 || KS == 0)) {
        auto two = [&](auto ic) {
          constexpr int I = decltype(ic)::value;
          if (KS == 3) { dma_q(cA, cB, (t + 2) * BK, IC<2 * I>{}); dma_q(cA, cB, (t + 2) * BK, IC<2 * I + 1>{}); }
          else { dma_q(oA, oB, (t + 1) * BK, IC<8 + 2 * I>{}); dma_q(oA, oB, (t + 1) * BK, IC<8 + 2 * I + 1>{}); }
        };
        if (i == 0) two(IC<0>{});
        if (i == 1) two(IC<1>{});
        if (i == 2) two(IC<2>{});
        if (i == 3) two(IC<3>{});
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  const int nk = K / BK;   // even
  // the loop prefetches two steps ahead: A and B carry one tile of slack rows behind them
  // (the host checks the buffer sizes), so the loads of steps nk, nk+1 stay in bounds
  auto eight = [&](uint16_t* a, uint16_t* b, int k0, auto basec) {
    constexpr int Q0 = decltype(basec)::value;
    dma_q(a, b, k0, IC<Q0 + 0>{}); dma_q(a, b, k0, IC<Q0 + 1>{}); dma_q(a, b, k0, IC<Q0 + 2>{}); dma_q(a, b, k0, IC<Q0 + 3>{});
    dma_q(a, b, k0, IC<Q0 + 4>{}); dma_q(a, b, k0, IC<Q0 + 5>{}); dma_q(a, b, k0, IC<Q0 + 6>{}); dma_q(a, b, k0, IC<Q0 + 7>{});
  };
  eight(sA0, sB0, 0, IC<0>{});
  eight(sA0, sB0, 0, IC<8>{});
  eight(sA1, sB1, BK, IC<0>{});
  __builtin_amdgcn_s_waitcnt(0x0F78);
  __builtin_amdgcn_s_barrier();
  load_frags(IC<0>{}, aad[0][0], bad[0][0]);
  if (!LDS) load_frags(IC<1>{}, aad[0][1], bad[0][1]);
  for (int t = 0; t < nk; t += 2) {
    phase(IC<0>{}, IC<0>{}, t); phase(IC<1>{}, IC<0>{}, t); phase(IC<2>{}, IC<0>{}, t); phase(IC<3>{}, IC<0>{}, t);
    phase(IC<0>{}, IC<1>{}, t + 1); phase(IC<1>{}, IC<1>{}, t + 1); phase(IC<2>{}, IC<1>{}, t + 1); phase(IC<3>{}, IC<1>{}, t + 1);
  }
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  const int colq = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + wm * 128 + i * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * 128 + j * 32 + g * 8 + colq;
        uint2 o;
        o.x = (__float_as_uint(acc[i][j][g * 4]) >> 16) | (__float_as_uint(acc[i][j][g * 4 + 1]) & 0xffff0000u);
        o.y = (__float_as_uint(acc[i][j][g * 4 + 2]) >> 16) | (__float_as_uint(acc[i][j][g * 4 + 3]) & 0xffff0000u);
        *reinterpret_cast<uint2*>(C + (long long)row * N + col) = o;
      }
  }
}

// ------------------------------------------------------------------ the Adam step's streams
__device__ __forceinline__ unsigned pk(float a, float b) {
  return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xffff0000u);
}
__device__ __forceinline__ f4 upd(f4 g, f4& w, f4& m, f4& v) {
  m = 0.9f * m + 0.1f * g;
  v = 0.99f * v + 0.01f * g * g;
  f4 r;
  for (int i = 0; i < 4; ++i) r[i] = w[i] - 1e-3f * (m[i] / (sqrtf(v[i]) + 1e-8f));
  w = r;
  return r;
}
// lane-contiguous 16-byte accesses, U per thread and tensor, spaced by the workgroup's span
template <int U>
__global__ __launch_bounds__(256) void adam_lc_kernel(const f4* g, f4* w, f4* m, f4* v, u2* s0, u2* s1,
                                                      long long n4, long long half) {
  for (long long base = (long long)blockIdx.x * 256 * U; base < n4; base += (long long)gridDim.x * 256 * U) {
    f4 G[U], W[U], M[U], V[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long i = base + u * 256 + threadIdx.x;
      if (i < n4) { G[u] = g[i]; W[u] = w[i]; M[u] = m[i]; V[u] = v[i]; }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long i = base + u * 256 + threadIdx.x;
      if (i < n4) {
        const f4 r = upd(G[u], W[u], M[u], V[u]);
        w[i] = W[u]; m[i] = M[u]; v[i] = V[u];
        const u2 p = {pk(r[0], r[1]), pk(r[2], r[3])};
        s0[i] = p;
        if (i < half) s1[i] = p;
      }
    }
  }
}
// a thread owns 8 consecutive parameters (two 16-byte accesses per tensor, one 16-byte bf16 store
// per replica): the layout of adam_to_replicas
__global__ __launch_bounds__(256) void adam_p8_kernel(const f4* g, f4* w, f4* m, f4* v, u4* s0, u4* s1,
                                                      long long n8, long long half) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long long)gridDim.x * 256) {
    f4 G[2], W[2], M[2], V[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) { G[h] = g[2 * i + h]; W[h] = w[2 * i + h]; M[h] = m[2 * i + h]; V[h] = v[2 * i + h]; }
    const f4 r0 = upd(G[0], W[0], M[0], V[0]), r1 = upd(G[1], W[1], M[1], V[1]);
#pragma unroll
    for (int h = 0; h < 2; ++h) { w[2 * i + h] = W[h]; m[2 * i + h] = M[h]; v[2 * i + h] = V[h]; }
    const u4 p = {pk(r0[0], r0[1]), pk(r0[2], r0[3]), pk(r1[0], r1[1]), pk(r1[2], r1[3])};
    s0[i] = p;
    if (i < half) s1[i] = p;
  }
}

}  // namespace

extern "C" {

// operands: 256 * blocks * 32 bytes; out: 256 * blocks floats.  Flops = blocks * 4 * iters * 16 * 32768.
int symi_ceiling_mfma(const void* operands, float* out, int blocks, int iters, void* stream) {
  if (!operands || !out || blocks < 1 || iters < 1) return -1;
  mfma_regs_kernel<<<blocks, 256, 0, (hipStream_t)stream>>>((const uint16_t*)operands, out, iters);
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

// C [M,N] bf16 = A [M,K] B [N,K]^T.  a_elems / b_elems: elements the A and B buffers hold; they
// must cover (M + 256) * K and (N + 256) * K (the loop prefetches two steps past the end).
int symi_ceiling_gemm_loop(int variant, const void* A, const void* B, void* C, int M, int N, int K,
                           long long a_elems, long long b_elems, void* stream) {
  if (!A || !B || !C || M < 256 || N < 256 || K < 128 || M % 256 || N % 256 || K % 128) return -1;
  if (a_elems < (long long)(M + 256) * K || b_elems < (long long)(N + 256) * K) return -1;
  // the per-lane byte offsets of the loads are 32 bits wide
  if ((long long)(M + 256) * K * 2 >= (1LL << 32) || (long long)(N + 256) * K * 2 >= (1LL << 32)) return -1;
  const dim3 grid(N / BN, M / BM);
  hipStream_t st = (hipStream_t)stream;
  const uint16_t* a = (const uint16_t*)A;
  const uint16_t* b = (const uint16_t*)B;
  uint16_t* c = (uint16_t*)C;
  switch (variant) {
    case 0: gemm_loop_kernel<0><<<grid, 256, 0, st>>>(a, b, c, M, N, K); break;
    case 1: gemm_loop_kernel<1><<<grid, 256, 0, st>>>(a, b, c, M, N, K); break;
    case 2: gemm_loop_kernel<2><<<grid, 256, 0, st>>>(a, b, c, M, N, K); break;
    case 3: gemm_loop_kernel<3><<<grid, 256, 0, st>>>(a, b, c, M, N, K); break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

// n parameters (a multiple of 2048): g, w, m, v fp32 [n]; s0 bf16 [n], s1 bf16 [n/2] (1.5 replicas
// per parameter on average, as 96 slots over 64 classes).  layout 0: 8 consecutive parameters per
// thread; 1 / 2 / 4: lane-contiguous 16-byte accesses, that many per thread.  grid_stride != 0:
// 2048 workgroups looping instead of one pass.  Bytes moved: n * (16 + 12 + 3).
int symi_ceiling_adam_streams(int layout, const float* g, float* w, float* m, float* v, void* s0, void* s1,
                              long long n, int grid_stride, void* stream) {
  if (!g || !w || !m || !v || !s0 || !s1 || n < 2048 || n % 2048) return -1;
  hipStream_t st = (hipStream_t)stream;
  const long long n4 = n / 4, n8 = n / 8;
  auto grid = [&](long long items, int per) {
    const long long b = (items + per - 1) / per;
    return (unsigned)(grid_stride ? (b < 2048 ? b : 2048) : b);
  };
  switch (layout) {
    case 0: adam_p8_kernel<<<grid(n8, 256), 256, 0, st>>>((const f4*)g, (f4*)w, (f4*)m, (f4*)v, (u4*)s0, (u4*)s1, n8, n8 / 2); break;
    case 1: adam_lc_kernel<1><<<grid(n4, 256), 256, 0, st>>>((const f4*)g, (f4*)w, (f4*)m, (f4*)v, (u2*)s0, (u2*)s1, n4, n4 / 2); break;
    case 2: adam_lc_kernel<2><<<grid(n4, 512), 256, 0, st>>>((const f4*)g, (f4*)w, (f4*)m, (f4*)v, (u2*)s0, (u2*)s1, n4, n4 / 2); break;
    case 4: adam_lc_kernel<4><<<grid(n4, 1024), 256, 0, st>>>((const f4*)g, (f4*)w, (f4*)m, (f4*)v, (u2*)s0, (u2*)s1, n4, n4 / 2); break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

}  // extern "C"
