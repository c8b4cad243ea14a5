// symi_expert_fwd / symi_expert_bwd: the expert SwiGLU FFN over replica slots as
// variable-group grouped GEMMs (paper Sec. 2.1; the expert compute of Fig. 5; the
// intra-rank part of the replica gradient reduction of Sec. 4.1 is fused into the
// weight-gradient GEMM, which sums over every row of a class at once).
//
// Six products share one tiled kernel (bf16 inputs, fp32 accumulation on the gfx950
// MFMA 32x32x16 bf16 instruction; a plain-FMA twin serves fp32 configurations):
//   FWD1   [u|v] = Xp  * W1^T      + SwiGLU epilogue writing u, v and h = silu(u)*v
//   FWD2   Yp    = H   * W2^T
//   BWD_DH dh    = dYp * W2        turned into du, dv from the saved u, v in the epilogue
//   BWD_DX dXp   = dUV * W1
//   WGRAD2 dW2_e = dYp^T * H       over all rows of class e
//   WGRAD1 dW1_e = dUV^T * Xp      over all rows of class e
// The first four have a variable number of rows per group (one group per slot); a small
// kernel turns slot_offsets into a table of 256-row m-tiles so that no workgroup spans
// two slots.  The last two have a variable reduction length (the rows of a class).  The two
// narrow products (FWD2, BWD_DX) may cut the reduction of their last round's tiles into slices
// that a second small kernel adds up (tail_slices, slice_sum_kernel).
//
// The MFMA is issued with the weight tile as its first operand, so a lane ends up with 4
// consecutive output columns of one output row; the epilogue turns the blocks around through
// LDS so that stores cover whole cache lines.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace symi {

enum { FWD1 = 0, FWD2 = 1, BWD_DH = 2, BWD_DX = 3, WGRAD2 = 4, WGRAD1 = 5 };

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

struct GemmParams {
  const void* A;       // activations (left operand source)
  const void* B;       // weights per slot, or the second activation for weight gradients
  void* C;             // main output
  const void* UV;      // BWD_DH: saved u|v
  void* UVout;         // FWD1: u|v out
  void* H;             // FWD1: h out
  const int32_t* tile_map;      // [4 + 4*i]: header {n_tiles}, then {row0, row1, slot, -}
  const int32_t* slot_offsets;  // weight gradients: class row ranges
  const int32_t* first_slot;
  long long b_group_stride;     // elements between consecutive slots' weights
  long long c_group_stride;     // elements between consecutive classes' gradients
  int M;   // fixed row count of the output (weight gradients)
  int N;   // output columns (FWD1: f, counted once)
  int K;   // reduction length when fixed
  int d, f;
  const int32_t* class_order;   // weight gradients: classes by decreasing row count
  int per_slot;                 // weight gradients: one output per slot instead of per class
  int skip_empty;               // weight gradients: a group without rows is not written at all
  float* partials;              // partial tiles of sliced reductions (nullptr: never slice)
  int cus;                      // compute units a round of tiles is spread over
};

__device__ __forceinline__ float silu_f(float u) { return u / (1.f + expf(-u)); }
__device__ __forceinline__ float sigmoid_f(float u) { return 1.f / (1.f + expf(-u)); }
// bf16 path: hardware exp2/rcp (relative error ~1e-6, far below the bf16 rounding of the result)
__device__ __forceinline__ float sigmoid_fast(float u) {
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.4426950408889634f * u));
}

// ---------------------------------------------------------------- m-tile table
// map[0] = number of m-tiles, map[4 + 4i ..] = {first row, end row, slot} of m-tile i.
// order[c] = the class with the c-th largest number of rows (ties: lower index first).
__global__ __launch_bounds__(256) void tile_map_kernel(const int32_t* __restrict__ slot_offsets,
                                                       const int32_t* __restrict__ first_slot, int S,
                                                       int E, int32_t* __restrict__ map,
                                                       int32_t* __restrict__ order) {
  __shared__ int32_t part[256];
  __shared__ int32_t rows[1024];
  const int tid = threadIdx.x;
  const int per = (S + 255) / 256;
  const int q0 = tid * per, q1 = min(S, q0 + per);
  int mine = 0;
  for (int q = q0; q < q1; ++q) mine += (slot_offsets[q + 1] - slot_offsets[q] + GEMM_BM - 1) / GEMM_BM;
  part[tid] = mine;
  if (first_slot) {
    for (int e = tid; e < E; e += 256) rows[e] = slot_offsets[first_slot[e + 1]] - slot_offsets[first_slot[e]];
  }
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {  // Hillis-Steele inclusive scan
    const int add = tid >= o ? part[tid - o] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  int t = part[tid] - mine;
  if (tid == 255) map[0] = part[255];
  for (int q = q0; q < q1; ++q) {
    const int b = slot_offsets[q], e = slot_offsets[q + 1];
    for (int r = b; r < e; r += GEMM_BM, ++t) {
      map[4 + 4 * t + 0] = r;
      map[4 + 4 * t + 1] = min(e, r + GEMM_BM);
      map[4 + 4 * t + 2] = q;
      map[4 + 4 * t + 3] = 0;
    }
  }
  if (first_slot) {
    for (int e = tid; e < E; e += 256) {
      int rank = 0;
      for (int j = 0; j < E; ++j) rank += (rows[j] > rows[e] || (rows[j] == rows[e] && j < e)) ? 1 : 0;
      order[rank] = e;
    }
  }
}

// ---------------------------------------------------------------- bf16 MFMA kernel
// Output tile 256 x 256 per workgroup, reduction step 64, 4 wavefronts in a 2 x 2 grid,
// each owning 128 x 128 outputs = 4 x 4 MFMA 32x32x16 tiles (256 fp32 accumulators per
// lane).  Tiles travel HBM -> LDS with the gfx950 direct-to-LDS loads (16 bytes per
// lane, no staging registers) into two stages of 2 x 32 KB; the next stage is in flight
// while the current one feeds the MFMAs.  LDS bandwidth is the scarce resource at this
// shape: 8 fragment reads of 1 KB per 16 MFMAs per wavefront.
//
// LDS layouts (all conflict-free for the access pattern that reads them):
//   reduction-contiguous operand: [256 rows][64 k], 16-byte chunk c of row r stored at
//     chunk c ^ ((r >> 1) & 7); fragments are plain 16-byte reads.
//   reduction-strided operand (memory [k][r], r contiguous): [64 k][256 r] as loaded,
//     16-byte chunk c of row k stored at c ^ 10*(k & 1) ^ 4*((k >> 1) & 1): the 32 lanes
//     the LDS serves per cycle (4 k-rows x 64 B) then fall into 64 distinct banks;
//     fragments come from the transposing LDS read (ds_read_b64_tr_b16), which hands
//     lane j of a 16-lane group the four k-values of column j.
// A direct-to-LDS load cannot zero-fill: rows or columns beyond the tile's extent are clamped
// to a valid one (they only reach outputs that are never stored), reduction indices beyond K
// load from a block of zeros.
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GT = 256;

__device__ __attribute__((aligned(16))) uint16_t g_zero_chunk[8] = {0, 0, 0, 0, 0, 0, 0, 0};

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short shortx4;
#define SYMI_GPTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define SYMI_LPTR(p) ((void __attribute__((address_space(3)))*)(p))

__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <int V> struct IC { static constexpr int value = V; };

// LDS reads with an immediate byte offset; nothing waits for them (see the kernel)
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
// transposing read: 4 k-values of one column per 8-byte half; the second half sits 4 k-rows
// (2048 bytes) further
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_tr(unsigned addr) {
  shortx4 lo, hi;
  asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
               : "=&v"(lo), "=&v"(hi) : "v"(addr), "n"(OFF), "n"(OFF + 2048));
  union { shortx4 h[2]; bf16x8 v; } u;
  u.h[0] = lo;
  u.h[1] = hi;
  return u.v;
}

// Reduction slices of the narrow variable-row products (FWD2, BWD_DX).  Their tiles run in
// launch order, one workgroup per tile, in rounds of `cus`.  If the last round would leave at
// least half the chip idle (config c2: 300 tiles, a second round of 44), each of its tiles is
// cut into `sl` slices of at least 16 reduction steps, as many as fill the round (at most 8);
// a slice leaves its accumulators as a plain fp32 tile in a partial slot and slice_sum_kernel,
// launched behind the product, adds them up in slice order.  full = tiles that stay whole.
// (Letting the slice that finishes last add up the partials inside the product was measured
// slower than no slicing at all: device-scope fences write back / invalidate the whole L2 of
// an XCD under the other tiles' feet, and without fences one workgroup reads a megabyte of
// uncached partials at some 16 GB/s.  Slicing the weight gradients of very popular classes the
// same way cost more in partial traffic than the shorter tail returned.)
__device__ __forceinline__ void tail_slices(int n_tiles, int cus, int K, int& full, int& sl) {
  full = n_tiles;
  sl = 1;
  const int rem = n_tiles % cus;
  if (rem > 0 && 2 * rem <= cus) {
    const int s = min(min(cus / rem, 8), (K + BK - 1) / BK / 16);
    if (s >= 2) { sl = s; full = n_tiles - rem; }
  }
}

// One tile of one product.  MI = 32-row blocks per wavefront: 4 for the 256-row tile (each of the
// 2 x 2 wavefronts 128 x 128), 2 for the 128-row tile that holds the ragged end of a slot when
// it has at most 128 rows (each wavefront 64 x 128: half the MFMAs, and the two wavefronts whose
// 64-row band of the left operand lies beyond the tile load nothing of it).
template <int MODE, int MI>
__device__ __forceinline__ void gemm_tile(const GemmParams& p, uint16_t* const smem, const int row0,
                                          const int row1, const int group, const int kbeg, const int K,
                                          const int bx, const int nsl, const int kofs, const int pslot) {
  // [left stage 0 | left stage 1 | right stage 0 | right stage 1], 32 KB each: the two
  // stages of an operand differ by an immediate offset of the LDS read instructions
  uint16_t* const sA0 = smem;
  uint16_t* const sA1 = smem + BM * BK;
  uint16_t* const sB0 = smem + 2 * BM * BK;
  uint16_t* const sB1 = smem + 2 * BM * BK + BN * BK;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, and known to be
  const int wm = wave >> 1, wn = wave & 1;
  constexpr bool VARM = MODE <= BWD_DX;
  constexpr bool A_KC = VARM;                       // left operand reduction-contiguous
  constexpr bool B_KC = MODE == FWD1 || MODE == FWD2;
  constexpr int WROWS = 32 * MI;                    // output rows of one wavefront
  static_assert(MI == 4 || (MI == 2 && VARM), "the 128-row tile serves the variable-row products");
  // a wavefront whose 64 rows of the left tile lie beyond a 128-row tile loads nothing of it
  const bool skip_left = MI == 2 && wave >= 2;
  // FWD1: a tile holds 128 hidden units; every 64 tile columns are 32 gate columns
  // followed by the 32 up columns of the same hidden units.
  const int n0 = bx * (MODE == FWD1 ? BN / 2 : BN);

  if (!VARM && K == 0) {
    if (p.skip_empty) return;   // the caller treats this gradient as zero without reading it
    // a class without rows: its gradient tile is zero; stream it out with one 1 KB row
    // segment per wavefront store
    float* Co = static_cast<float*>(p.C) + (long long)group * p.c_group_stride;
    const int col = n0 + lane * 4;
    if (col < p.N) {
      for (int r = row0 + wave; r < row1; r += GT / 64)
        *reinterpret_cast<float4*>(Co + (long long)r * p.N + col) = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    return;
  }

  const uint16_t* A = static_cast<const uint16_t*>(p.A);
  const uint16_t* B = static_cast<const uint16_t*>(p.B) + (VARM ? (long long)group * p.b_group_stride : 0);
  const long long lda = MODE == FWD1 ? p.d : MODE == FWD2 ? p.f : MODE == BWD_DH ? p.d
                        : MODE == BWD_DX ? 2LL * p.f : MODE == WGRAD2 ? p.d : 2LL * p.f;
  const long long ldb = MODE == FWD1 ? p.d : MODE == FWD2 ? p.f : MODE == BWD_DH ? p.f
                        : MODE == BWD_DX ? p.d : MODE == WGRAD2 ? p.f : p.d;
  const uint16_t* zero = g_zero_chunk;

  // ---- direct-to-LDS loads: a wave-uniform base per reduction step plus a 32-bit per-lane
  // element offset, one per instruction j (0..7) and operand.
  // reduction-contiguous tile: wavefront w, instruction j fills tile rows w*64 + 8j .. +8;
  //   lane -> (row + lane/8, physical chunk lane%8)
  // reduction-strided tile: wavefront w, instruction j fills k-rows w*16 + 2j, +1;
  //   lane -> (k-row + lane/32, physical chunk lane%32)
  // Rows / column chunks beyond the operand's extent are clamped to a valid one: what
  // they bring in only reaches outputs that are never stored.
  // The main loop takes its 16 offsets from registers (no vector arithmetic next to the
  // MFMAs).  The last iterations, which load the partial step or steps beyond K, recompute
  // them from five lane constants and point every reduction index beyond K at a block of
  // zeros.
  int kc_row = wave * 64 + (lane >> 3);                        // tile row of instruction 0
  int kc_c0 = (lane & 7) ^ ((lane >> 4) & 7);                  // logical chunk for even j
  int ks_kb = wave * 16 + (lane >> 5);                         // k-row of instruction 0
  int ks_c0 = (lane & 31) ^ (10 * (lane >> 5));                // logical chunk, j-dependent bits to come
  int f1_row = wave * 32 + (lane >> 3);                        // FWD1 weights: hidden unit of instruction 0

  const uint16_t* a_base;   // element (first tile row / column, reduction index 0)
  const uint16_t* b_base;
  int a_lim, b_lim;         // KC: last valid tile row; KS: number of valid columns
  if (A_KC) {
    a_base = A + (long long)row0 * lda + kofs;
    a_lim = row1 - row0 - 1;
  } else {
    a_base = A + (long long)kbeg * lda + row0;
    a_lim = row1 - row0;
  }
  if (B_KC) {
    b_base = (MODE == FWD1 ? B : B + (long long)n0 * ldb) + kofs;
    b_lim = MODE == FWD1 ? p.f - 1 : p.N - n0 - 1;
  } else {
    b_base = (VARM ? B + (long long)kofs * ldb : B + (long long)kbeg * ldb) + n0;
    b_lim = p.N - n0;
  }
  // LDS destination of instruction j (wave-uniform): both layouts advance 1 KB per j
  const int wdst = wave * 8 * 512;  // elements: 8 instructions x 512 elements per wavefront
  // q = 0..15: even = left operand, odd = right operand, instruction j = q/2
  // offset of this lane's 16 bytes for instruction j, and its reduction index within the step
  auto lane_off = [&](bool right, int j, int& krel) -> unsigned {
    const bool kcontig = right ? B_KC : A_KC;
    const int ld = (int)(right ? ldb : lda);
    const int lim = right ? b_lim : a_lim;
    if (kcontig) {
      const int kc = kc_c0 ^ (4 * (j & 1));
      krel = kc * 8;
      if (right && MODE == FWD1) {
        // tile row t -> hidden unit n0 + (t>>7)*64 + ((t>>6)&1)*32 + (t&31), up half if (t>>5)&1
        const int hu = min(n0 + f1_row + 8 * (j & 3), lim);
        return (unsigned)(((j >> 2) * p.f + hu) * ld + kc * 8);
      }
      return (unsigned)(min(kc_row + 8 * j, lim) * ld + kc * 8);
    }
    const int c = ks_c0 ^ (4 * (j & 1));
    krel = ks_kb + 2 * j;
    return (unsigned)((ks_kb + 2 * j) * ld + (c * 8 < lim ? c : 0) * 8);
  };
  // The main loop's loads take the cheapest form the instruction has: a scalar base (operand +
  // reduction step), a 32-bit per-lane byte offset from a register and an immediate, with the
  // LDS base (M0) written once per operand and stage: the 8 instructions of an operand write 8
  // consecutive KB, reached from an M0 in their middle through immediates of -4 .. +3 KB, which
  // the per-lane offset takes back out of the global address (the scalar base sits 4 KB low so
  // that the offset stays positive).  Measured in the loop's microbenchmark: an M0 write in front
  // of every load and a 64-bit vector add for its address cost 26-36 cycles of MFMA issue per
  // load, this form 4-8 (a 64-deep step 2750 -> 2340 cycles).  All direct-to-LDS loads of this
  // kernel are inline assembly, so that nothing else ever writes M0.
  unsigned voA[8], voB[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int unused;
    voA[j] = lane_off(false, j, unused) * 2u + 4096u - (unsigned)((j - 4) * 1024);
    voB[j] = lane_off(true, j, unused) * 2u + 4096u - (unsigned)((j - 4) * 1024);
  }
  auto set_m0 = [&](unsigned lds_byte_addr) {
    asm volatile("s_mov_b32 m0, %0" ::"s"(lds_byte_addr) : "memory");
  };
  auto load_fast = [&](auto jc, unsigned voff, const void* sbase) {
    constexpr int J = decltype(jc)::value;
    asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(voff), "s"(sbase), "n"((J - 4) * 1024) : "memory");
  };
  // q = 0..7: instruction j = q of the left operand, q = 8..15: instruction j = q - 8 of the right one
  auto dma_one = [&](uint16_t* sA, uint16_t* sB, int k0, auto qc, auto partial) {
    constexpr int Q = decltype(qc)::value;
    constexpr int j = Q & 7;
    constexpr bool right = Q >= 8;
    if (MI == 2 && !right && skip_left) return;
    const bool kcontig = right ? B_KC : A_KC;
    const uint16_t* base = right ? b_base : a_base;
    const long long ld = right ? ldb : lda;
    const uint16_t* sbase = kcontig ? base + k0 : base + (long long)k0 * ld;   // wave-uniform
    const unsigned lds0 = (unsigned)(size_t)SYMI_LPTR((right ? sB : sA) + wdst);   // this wavefront's 8 KB
    if (decltype(partial)::value) {
      int krel;
      const unsigned off = lane_off(right, j, krel);
      const uint16_t* src = k0 + krel < K ? sbase + (size_t)off : zero;
      set_m0(lds0 + j * 1024);
      asm volatile("global_load_lds_dwordx4 %0, off" ::"v"(src) : "memory");
    } else {
      if (j == 0) set_m0(lds0 + 4096);
      load_fast(IC<j>{}, right ? voB[j] : voA[j], reinterpret_cast<const char*>(sbase) - 4096);
    }
  };
  // ---- fragment reads.  Byte address of this lane's piece inside stage 0 of its operand,
  // everything else (32-row block, 16-deep sub-step, stage) is an immediate offset.
  // KC: row (sub*32 + lane%32), chunk (2*ks + lane/32) ^ ((lane%32 >> 1) & 7); the xor makes the
  //   sub-step a per-lane quantity, so there is one address per sub-step.
  // KS: lane = 16*g + jj supplies the address of k-row (16*ks + 8*(g>>1) + 4*e + jj/4),
  //   8-byte piece (jj%4) of columns sub*32 + 16*(g&1) ..; it receives column sub*32 + lane%32;
  //   one address per 32-column block, the sub-step is an immediate (16 k-rows of 512 B).
  const int r31 = lane & 31;
  const int g4 = lane >> 4, jj = lane & 15;
  const int ks_h2 = (10 * ((jj >> 2) & 1)) ^ (4 * ((jj >> 3) & 1));   // swizzle of this lane's k-row
  const int ks_row = (8 * (g4 >> 1) + (jj >> 2)) * 256;
  unsigned adA[4], adB[4];
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const int kc = r31 * BK + (((2 * x + (lane >> 5)) ^ ((r31 >> 1) & 7)) * 8);             // x = sub-step
    const int ksc = ks_row + (((4 * x + 2 * (g4 & 1) + ((jj & 3) >> 1)) ^ ks_h2) * 8) + 4 * (jj & 1);  // x = block
    adA[x] = (unsigned)(size_t)SYMI_LPTR(sA0) + 2u * (unsigned)(A_KC ? wm * WROWS * BK + kc : wm * WROWS + ksc);
    adB[x] = (unsigned)(size_t)SYMI_LPTR(sB0) + 2u * (unsigned)(B_KC ? wn * 128 * BK + kc : wn * 128 + ksc);
  }
  // All LDS reads are inline assembly: the compiler cannot tell the stage being read from the
  // one being filled by direct-to-LDS loads and would wait for the prefetch before every
  // read.  Completion is awaited by hand (lgkmcnt(0)) at the start of the phase that uses them.
  bf16x8 fa[2][MI], fb[2][4];   // two register sets: one feeds the MFMAs, the other is being filled
  // half = 0 / 1: fragments 0, 1 / 2, 3 of both operands; 2: all of them
  auto load_frags = [&](auto bufc, auto stagec, auto ksc, auto halfc) {
    constexpr int bu = decltype(bufc)::value, S = decltype(stagec)::value, KS = decltype(ksc)::value;
    constexpr int HF = decltype(halfc)::value;
    constexpr int SO = S * BM * BK * 2;   // stage offset in bytes
    constexpr bool LO = HF != 1, HI = HF != 0;
#pragma unroll
    for (int x = 0; x < MI; ++x) {
      if (!(x < MI / 2 ? LO : HI)) continue;
      if (A_KC) {
        if (x == 0) fa[bu][0] = lds_read_b128<SO + 0 * 4096>(adA[KS]);
        if (x == 1) fa[bu][1] = lds_read_b128<SO + 1 * 4096>(adA[KS]);
        if (x == 2) fa[bu][x] = lds_read_b128<SO + 2 * 4096>(adA[KS]);
        if (x == 3) fa[bu][x] = lds_read_b128<SO + 3 * 4096>(adA[KS]);
      } else {
        fa[bu][x] = lds_read_tr<SO + KS * 8192>(adA[x]);
      }
    }
    if (B_KC) {
      if (LO) fb[bu][0] = lds_read_b128<SO + 0 * 4096>(adB[KS]);
      if (LO) fb[bu][1] = lds_read_b128<SO + 1 * 4096>(adB[KS]);
      if (HI) fb[bu][2] = lds_read_b128<SO + 2 * 4096>(adB[KS]);
      if (HI) fb[bu][3] = lds_read_b128<SO + 3 * 4096>(adB[KS]);
    } else {
      if (LO) fb[bu][0] = lds_read_tr<SO + KS * 8192>(adB[0]);
      if (LO) fb[bu][1] = lds_read_tr<SO + KS * 8192>(adB[1]);
      if (HI) fb[bu][2] = lds_read_tr<SO + KS * 8192>(adB[2]);
      if (HI) fb[bu][3] = lds_read_tr<SO + KS * 8192>(adB[3]);
    }
  };

  floatx16 acc[MI][4];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- main loop.  A reduction step (64 deep, stage S = step & 1) is four phases of 16
  // MFMAs.  Phase ks consumes register set ks & 1 while the fragments of the next phase are
  // read into the other set.  Phase 3 first waits for the loads of the next step, meets the
  // other wavefronts (after which nobody reads stage S any more: its last fragments already
  // sit in registers), reads the first fragments of the other stage and starts loading step
  // + 2 into stage S; phase 0 of the next step issues the second half of those loads.  A
  // load therefore has three to four phases to arrive, and neither an LDS round trip nor a
  // load latency is exposed to the MFMA pipe.  Steps beyond the last one load zeros (dummy
  // loads keep the loop free of branches, which is what lets the 256 accumulators stay put).
  const int nk = (K + BK - 1) / BK;
  auto phase = [&](auto ksc, auto stagec, int step, auto partial) {
    constexpr int KS = decltype(ksc)::value, S = decltype(stagec)::value;
    constexpr int bu = KS & 1;
    uint16_t* const cA = S ? sA1 : sA0;
    uint16_t* const cB = S ? sB1 : sB0;
    uint16_t* const oA = S ? sA0 : sA1;
    uint16_t* const oB = S ? sB0 : sB1;
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): the fragments of this phase
    if (KS == 3) {
      wait_vmcnt0();                      // my share of the next step has landed
      __builtin_amdgcn_s_barrier();       // ... so has everybody's, and stage S is free
    }
    __builtin_amdgcn_sched_barrier(0);
    if (decltype(partial)::value && (KS == 3 || KS == 0)) {
      // keep the address arithmetic of these loads inside the phase (not hoisted into registers)
      asm volatile("" : "+v"(kc_row), "+v"(kc_c0), "+v"(ks_kb), "+v"(ks_c0), "+v"(f1_row));
    }
    constexpr int LPI = 8 / MI;   // loads issued behind each MFMA group of a phase that loads
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[bu][j], fa[bu][i], acc[i][j], 0, 0, 0);
      // the next phase's fragments, half of them behind each of the first two MFMA groups: the
      // matrix pipe has work queued while the reads issue, and they still have half a phase to land
      if (i == 0) {
        if (KS == 3) load_frags(IC<bu ^ 1>{}, IC<S ^ 1>{}, IC<0>{}, IC<0>{});
        else load_frags(IC<bu ^ 1>{}, IC<S>{}, IC<(KS + 1) & 3>{}, IC<0>{});
      } else if (i == 1) {
        if (KS == 3) load_frags(IC<bu ^ 1>{}, IC<S ^ 1>{}, IC<0>{}, IC<1>{});
        else load_frags(IC<bu ^ 1>{}, IC<S>{}, IC<(KS + 1) & 3>{}, IC<1>{});
      }
      // phase 3: the left operand of step + 2 into the stage just freed; phase 0: the right one
      auto issue = [&](auto uc) {
        constexpr int U = decltype(uc)::value;
        if (i == 0) { if (KS == 3) dma_one(cA, cB, (step + 2) * BK, IC<0 * LPI + U>{}, partial); else dma_one(oA, oB, (step + 1) * BK, IC<8 + 0 * LPI + U>{}, partial); }
        if (i == 1) { if (KS == 3) dma_one(cA, cB, (step + 2) * BK, IC<1 * LPI + U>{}, partial); else dma_one(oA, oB, (step + 1) * BK, IC<8 + 1 * LPI + U>{}, partial); }
        if (MI == 4 && i == 2) { if (KS == 3) dma_one(cA, cB, (step + 2) * BK, IC<(2 * LPI + U) & 7>{}, partial); else dma_one(oA, oB, (step + 1) * BK, IC<8 + ((2 * LPI + U) & 7)>{}, partial); }
        if (MI == 4 && i == 3) { if (KS == 3) dma_one(cA, cB, (step + 2) * BK, IC<(3 * LPI + U) & 7>{}, partial); else dma_one(oA, oB, (step + 1) * BK, IC<8 + ((3 * LPI + U) & 7)>{}, partial); }
      };
      if (KS == 3 || KS == 0) {
        issue(IC<0>{});
        issue(IC<1>{});
        if (LPI == 4) { issue(IC<2>{}); issue(IC<3>{}); }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto pair = [&](int t, auto partial) {
    phase(IC<0>{}, IC<0>{}, t, partial);
    phase(IC<1>{}, IC<0>{}, t, partial);
    phase(IC<2>{}, IC<0>{}, t, partial);
    phase(IC<3>{}, IC<0>{}, t, partial);
    phase(IC<0>{}, IC<1>{}, t + 1, partial);
    phase(IC<1>{}, IC<1>{}, t + 1, partial);
    phase(IC<2>{}, IC<1>{}, t + 1, partial);
    phase(IC<3>{}, IC<1>{}, t + 1, partial);
  };
  auto prologue = [&](auto partial) {
    auto all16 = [&](uint16_t* a, uint16_t* b, int k0, auto halfc) {
      dma_one(a, b, k0, IC<0>{}, partial); dma_one(a, b, k0, IC<1>{}, partial); dma_one(a, b, k0, IC<2>{}, partial);
      dma_one(a, b, k0, IC<3>{}, partial); dma_one(a, b, k0, IC<4>{}, partial); dma_one(a, b, k0, IC<5>{}, partial);
      dma_one(a, b, k0, IC<6>{}, partial); dma_one(a, b, k0, IC<7>{}, partial);
      if (decltype(halfc)::value) return;
      dma_one(a, b, k0, IC<8>{}, partial); dma_one(a, b, k0, IC<9>{}, partial); dma_one(a, b, k0, IC<10>{}, partial);
      dma_one(a, b, k0, IC<11>{}, partial); dma_one(a, b, k0, IC<12>{}, partial); dma_one(a, b, k0, IC<13>{}, partial);
      dma_one(a, b, k0, IC<14>{}, partial); dma_one(a, b, k0, IC<15>{}, partial);
    };
    all16(sA0, sB0, 0, std::false_type{});   // step 0, both operands
    all16(sA1, sB1, BK, std::true_type{});   // step 1, left operand (the right one follows in phase 0)
  };
  if (K >= 2 * BK) prologue(std::false_type{}); else prologue(std::true_type{});
  // step 0 has landed, the left operand of step 1 (8 loads) may still fly; in a half-height
  // tile the wavefronts that skip the left operand have nothing of step 1 in flight: all wait
  // for everything there
  if (MI == 4) __builtin_amdgcn_s_waitcnt(0x0F78); else wait_vmcnt0();
  __builtin_amdgcn_s_barrier();
  load_frags(IC<0>{}, IC<0>{}, IC<0>{}, IC<2>{});
  // always pairs of steps: for an odd step count the second stage holds the zeros of the
  // dummy loads and adds nothing (a mid-loop exit would cost more than the idle step).  A
  // pair starting at step t loads steps up to t + 3.
  int t = 0;
  for (; (t + 4) * BK <= K; t += 2) pair(t, std::false_type{});
  for (; t < nk; t += 2) pair(t, std::true_type{});
  // dummy loads and the fragment read of the last phase are still in flight: they must
  // not outlive the workgroup's LDS allocation
  __builtin_amdgcn_s_waitcnt(0xC07F);
  wait_vmcnt0();

  // ---- epilogue.  After the MFMA a lane owns one output row (lane%32) of each 32-row
  // block and, per 8-column group g, the 4 columns 8g + 4*(lane/32) ..: stored like that, a
  // wavefront store would touch 64 cache lines with 16 bytes each, and the store path is
  // paid per line touched.  The operand stages are free now, so every wavefront turns its
  // 32-row blocks around through a private piece of LDS (written in the MFMA layout, read
  // back row by row, 16 bytes per lane) and each store instruction writes whole lines:
  // 4 rows x 256 B (bf16 outputs), 8 rows x 128 B (u, v, h) or 2 rows x 512 B (fp32).
  __syncthreads();   // every wavefront's dummy loads have landed, nobody reads operands any more
  const int hw = lane >> 5, r32 = lane & 31;
  uint16_t* const stg = smem + wave * (16 * 1024);   // 32 KB per wavefront
  constexpr int LDB = 136;   // bf16 row of 128 columns + pad (272 B, a multiple of 16)
  constexpr int LDH = 72;    // u / v / h rows of 64 hidden units + pad (144 B)
  constexpr int LDF = 132;   // fp32 row of 128 columns + pad (528 B)
  uint4 uvu[2][8], uvv[2][8];   // BWD_DH: saved u, v of the current and the next 32-row block
  // a slice stores its accumulators the way a weight gradient is stored: fp32, pitch 256
  const bool to_partial = (MODE == FWD2 || MODE == BWD_DX) && nsl > 1;
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int rbase = row0 + wm * WROWS + i * 32;   // first output row of this block
    if (MODE == FWD1) {
      uint16_t* const su = stg;
      uint16_t* const sv = stg + 32 * LDH;
      uint16_t* const sh = stg + 64 * LDH;
#pragma unroll
      for (int hb = 0; hb < 2; ++hb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          unsigned pu[2], pv[2], ph[2];
#pragma unroll
          for (int c2 = 0; c2 < 2; ++c2) {
            const int r = g * 4 + 2 * c2;
            const float u0 = acc[i][2 * hb][r], u1 = acc[i][2 * hb][r + 1];
            const float v0 = acc[i][2 * hb + 1][r], v1 = acc[i][2 * hb + 1][r + 1];
            pu[c2] = pack_bf16x2(u0, u1);
            pv[c2] = pack_bf16x2(v0, v1);
            ph[c2] = pack_bf16x2(u0 * sigmoid_fast(u0) * v0, u1 * sigmoid_fast(u1) * v1);
          }
          const int at = r32 * LDH + hb * 32 + 8 * g + 4 * hw;
          *reinterpret_cast<uint2*>(su + at) = make_uint2(pu[0], pu[1]);
          *reinterpret_cast<uint2*>(sv + at) = make_uint2(pv[0], pv[1]);
          *reinterpret_cast<uint2*>(sh + at) = make_uint2(ph[0], ph[1]);
        }
      __builtin_amdgcn_s_waitcnt(0xC07F);
      uint16_t* UVo = static_cast<uint16_t*>(p.UVout);
      uint16_t* Ho = static_cast<uint16_t*>(p.H);
      const int hu = n0 + wn * 64 + (lane & 7) * 8;
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int rr = it * 8 + (lane >> 3);
        const int row = rbase + rr;
        const uint4 xu = *reinterpret_cast<const uint4*>(su + rr * LDH + (lane & 7) * 8);
        const uint4 xv = *reinterpret_cast<const uint4*>(sv + rr * LDH + (lane & 7) * 8);
        const uint4 xh = *reinterpret_cast<const uint4*>(sh + rr * LDH + (lane & 7) * 8);
        if (row < row1 && hu < p.f) {
          const long long o = (long long)row * 2 * p.f + hu;
          *reinterpret_cast<uint4*>(UVo + o) = xu;
          *reinterpret_cast<uint4*>(UVo + o + p.f) = xv;
          *reinterpret_cast<uint4*>(Ho + (long long)row * p.f + hu) = xh;
        }
      }
    } else if (MODE == BWD_DH) {
      // dh stays in fp32: staged like a weight-gradient block, then every lane takes 8
      // consecutive hidden units of one row, combines them with the saved u and v (16 bytes
      // each, whole lines per instruction) and writes du = dh v s (1 + u (1 - s)),
      // dv = dh u s, s = sigmoid(u).  The u, v loads of block i + 1 are issued before block i
      // is worked on, so their latency hides behind it.  They are unconditional: a lane past
      // the tile's last row or column reads the last valid row / the last 8 columns instead
      // (its result is never stored).  A load under a branch would make the compiler lose
      // count of the memory operations in flight and wait for all of them, the stores of the
      // previous rows included, before every use of a loaded value.
      float* const sf = reinterpret_cast<float*>(stg);
      const uint16_t* UVi = static_cast<const uint16_t*>(p.UV);
      uint16_t* Co = static_cast<uint16_t*>(p.C);
      const int col = n0 + wn * 128 + (lane & 15) * 8;
      const int colc = min(col, p.N - 8);
      const int twof = 2 * p.f;
      auto load_uv = [&](int blk, uint4 (&uu)[8], uint4 (&vv)[8]) {
        const int rb = row0 + wm * WROWS + blk * 32;
        const uint16_t* const q0 = UVi + (long long)rb * twof + colc;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int dr = min(rb + it * 4 + (lane >> 4), row1 - 1) - rb;   // may be negative
          const uint16_t* const q = q0 + (long long)dr * twof;
          uu[it] = *reinterpret_cast<const uint4*>(q);
          vv[it] = *reinterpret_cast<const uint4*>(q + p.f);
        }
      };
      if (i == 0) load_uv(0, uvu[0], uvv[0]);
      if (i + 1 < MI) load_uv(i + 1, uvu[(i + 1) & 1], uvv[(i + 1) & 1]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(sf + r32 * LDF + 32 * j + 8 * g + 4 * hw) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      __builtin_amdgcn_s_waitcnt(0xC07F);
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int rr = it * 4 + (lane >> 4);
        const int row = rbase + rr;
        const float4 d0 = *reinterpret_cast<const float4*>(sf + rr * LDF + (lane & 15) * 8);
        const float4 d1 = *reinterpret_cast<const float4*>(sf + rr * LDF + (lane & 15) * 8 + 4);
        if (row < row1 && col < p.N) {
          const long long o = (long long)row * 2 * p.f + col;
          const uint4 uu = uvu[i & 1][it], vv = uvv[i & 1][it];
          const float dh[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
          const uint32_t uw[4] = {uu.x, uu.y, uu.z, uu.w}, vw[4] = {vv.x, vv.y, vv.z, vv.w};
          uint32_t du[4], dv[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float o_du[2], o_dv[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const float u_ = __uint_as_float(h ? (uw[q] & 0xffff0000u) : (uw[q] << 16));
              const float v_ = __uint_as_float(h ? (vw[q] & 0xffff0000u) : (vw[q] << 16));
              const float sg = sigmoid_fast(u_);
              o_du[h] = dh[2 * q + h] * v_ * sg * (1.f + u_ * (1.f - sg));
              o_dv[h] = dh[2 * q + h] * u_ * sg;
            }
            du[q] = pack_bf16x2(o_du[0], o_du[1]);
            dv[q] = pack_bf16x2(o_dv[0], o_dv[1]);
          }
          *reinterpret_cast<uint4*>(Co + o) = make_uint4(du[0], du[1], du[2], du[3]);
          *reinterpret_cast<uint4*>(Co + o + p.f) = make_uint4(dv[0], dv[1], dv[2], dv[3]);
        }
      }
    } else if ((MODE == FWD2 || MODE == BWD_DX) && !to_partial) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<uint2*>(stg + r32 * LDB + 32 * j + 8 * g + 4 * hw) =
              make_uint2(pack_bf16x2(acc[i][j][4 * g], acc[i][j][4 * g + 1]),
                         pack_bf16x2(acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]));
      __builtin_amdgcn_s_waitcnt(0xC07F);
      uint16_t* Co = static_cast<uint16_t*>(p.C);
      const int col = n0 + wn * 128 + (lane & 15) * 8;
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int rr = it * 4 + (lane >> 4);
        const int row = rbase + rr;
        const uint4 x = *reinterpret_cast<const uint4*>(stg + rr * LDB + (lane & 15) * 8);
        if (row < row1 && col < p.N) *reinterpret_cast<uint4*>(Co + (long long)row * p.N + col) = x;
      }
    } else {   // weight gradients, fp32
      float* const sf = reinterpret_cast<float*>(stg);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(sf + r32 * LDF + 32 * j + 8 * g + 4 * hw) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      __builtin_amdgcn_s_waitcnt(0xC07F);
      if (VARM) {   // a slice's partial tile
        float* Co = p.partials + (size_t)pslot * (BM * BN) + (wm * WROWS + i * 32) * BN + wn * 128 + (lane & 31) * 4;
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          const int rr = it * 2 + (lane >> 5);
          *reinterpret_cast<float4*>(Co + rr * BN) = *reinterpret_cast<const float4*>(sf + rr * LDF + (lane & 31) * 4);
        }
      } else {
        float* Co = static_cast<float*>(p.C) + (long long)group * p.c_group_stride;
        const int col = n0 + wn * 128 + (lane & 31) * 4;
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          const int rr = it * 2 + (lane >> 5);
          const int row = rbase + rr;
          const float4 x = *reinterpret_cast<const float4*>(sf + rr * LDF + (lane & 31) * 4);
          if (row < row1 && col < p.N) *reinterpret_cast<float4*>(Co + (long long)row * p.N + col) = x;
        }
      }
    }
    // the next block reuses the staging area: its writes must not pass these reads
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Workgroups go to the eight XCDs (each with an L2 of its own) round robin in launch order:
// workgroup b runs on XCD b mod 8.  With the column index fastest an XCD would see two (ntx = 16)
// or one (ntx = 4) column tile of every m-tile, so every activation tile is fetched by four to
// eight L2s.  Instead a round of R consecutive workgroups (R / 8 per XCD, R / ntx m-tiles) is dealt
// out in blocks: XCD c takes 4 column tiles x R / 32 m-tiles, so an operand tile along either
// edge of the block is fetched by that L2 once for the whole block.  b -> tile is a permutation
// inside the round; the caller leaves rounds that are not whole in launch order.
__device__ __forceinline__ void xcd_block(int b, int ntx, int R, int& tile) {
  if (ntx != 4 && ntx != 8 && ntx != 16 && ntx != 32) return;
  const int l = b % R, c = l & 7, s = l >> 3;
  const int xn = ntx >> 2;   // XCDs side by side along the columns
  const int n = 4 * (c % xn) + (s & 3);
  const int m = (b / R) * (R / ntx) + (R >> 5) * (c / xn) + (s >> 2);
  tile = m * ntx + n;
}

template <int MODE>
__global__ __launch_bounds__(GT) void gemm_bf16_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * BM * BK + 2 * BN * BK];
  constexpr bool VARM = MODE <= BWD_DX;
  int row0, row1, group, kbeg = 0, K, bx = blockIdx.x;
  // this workgroup reduces slice zsl of nsl, starting at reduction index kofs; if nsl > 1 its
  // accumulators go to partial slot pslot
  int nsl = 1, zsl = 0, kofs = 0, pslot = 0;
  if (VARM) {
    // tiles in launch order (column index fastest); the last round's tiles may be sliced
    const int ntx = gridDim.x;
    const int n_tiles = p.tile_map[0] * ntx;
    const int b = blockIdx.y * ntx + blockIdx.x;
    int full = n_tiles, sl = 1;
    if ((MODE == FWD2 || MODE == BWD_DX) && p.partials) tail_slices(n_tiles, p.cus, p.K, full, sl);
    int tile = b;
    if (ntx == 4 || ntx == 8 || ntx == 16 || ntx == 32) {
      if (b < (full & ~255)) xcd_block(b, ntx, 256, tile);
    } else if (ntx < 32) {
      // other column counts: rounds of 8 m-tiles, XCD c takes all column tiles of the round's
      // m-tile c (launch order would scatter an m-tile's columns over all eight L2s)
      const int R = 8 * ntx;
      if (b < full - full % R) {
        const int l = b % R;
        tile = (b / R * 8 + (l & 7)) * ntx + (l >> 3);
      }
    }
    if (b >= full) {
      tile = full + (b - full) / sl;
      zsl = (b - full) % sl;
      nsl = sl;
    }
    if (tile >= n_tiles) return;
    const int mt = tile / ntx;
    bx = tile - mt * ntx;
    row0 = p.tile_map[4 + 4 * mt];
    row1 = p.tile_map[4 + 4 * mt + 1];
    group = p.tile_map[4 + 4 * mt + 2];
    K = p.K;
    if (nsl > 1) {
      const int nk_all = (p.K + BK - 1) / BK;
      const int len = ((nk_all + nsl - 1) / nsl + 1) / 2 * 2 * BK;   // whole pairs of steps
      kofs = zsl * len;
      K = max(0, min(len, p.K - kofs));
      pslot = (tile - full) * nsl + zsl;
    }
  } else {
    // classes in order of decreasing row count: the long reductions start first and the
    // short (or empty, store-only) tiles fill in behind them
    group = p.per_slot ? blockIdx.z : p.class_order[blockIdx.z];
    // the tiles of one class (or slot): whole rounds of 256, 128 or 64 workgroups are dealt out
    // in blocks per XCD (a group starts on XCD 0 whenever its tile count is a multiple of 8)
    const int ntx = gridDim.x, nt = ntx * gridDim.y;
    int tile = blockIdx.y * ntx + blockIdx.x;
    const int R = nt % 256 == 0 ? 256 : nt % 128 == 0 ? 128 : nt % 64 == 0 ? 64 : 0;
    if (R) xcd_block(tile, ntx, R, tile);
    const int mt = tile / ntx;
    bx = tile - mt * ntx;
    row0 = mt * BM;
    row1 = min(p.M, row0 + BM);
    if (p.per_slot) {   // the rows of one replica slot
      kbeg = p.slot_offsets[group];
      K = p.slot_offsets[group + 1] - kbeg;
    } else {            // the rows of all replica slots of a class
      kbeg = p.slot_offsets[p.first_slot[group]];
      K = p.slot_offsets[p.first_slot[group + 1]] - kbeg;
    }
  }
  if constexpr (VARM) {
    // the ragged end of a slot: at most 128 rows take the half-height tile
    if (__builtin_amdgcn_readfirstlane(row1 - row0) <= BM / 2) {
      gemm_tile<MODE, 2>(p, smem, row0, row1, group, kbeg, K, bx, nsl, kofs, pslot);
      return;
    }
  }
  gemm_tile<MODE, 4>(p, smem, row0, row1, group, kbeg, K, bx, nsl, kofs, pslot);
}

// ---------------------------------------------------------------- sum of reduction slices
// Runs behind FWD2 / BWD_DX (same stream): adds the partial tiles of every sliced tile in slice
// order and writes the bf16 rows of the product.  Workgroup = 16 rows of a tile, a lane four
// consecutive columns of four rows.  Returns at once if the product's tail was not sliced.
__global__ __launch_bounds__(256) void slice_sum_kernel(GemmParams p, int ntx) {
  const int tid = threadIdx.x;
  const int n_tiles = p.tile_map[0] * ntx;
  int full, sl;
  tail_slices(n_tiles, p.cus, p.K, full, sl);
  const int tile = full + blockIdx.y;
  if (sl < 2 || tile >= n_tiles) return;
  const int mt = tile / ntx;
  const int row0 = p.tile_map[4 + 4 * mt], row1 = p.tile_map[4 + 4 * mt + 1];
  const int n0 = (tile - mt * ntx) * BN;
  const float* part = p.partials + (size_t)blockIdx.y * sl * (BM * BN);
  const int c = (tid & 63) * 4;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int r = blockIdx.x * 16 + it * 4 + (tid >> 6);
    const int row = row0 + r, col = n0 + c;
    if (row >= row1 || col >= p.N) continue;
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z = 0; z < sl; ++z) {
      const float4 x = *reinterpret_cast<const float4*>(part + (size_t)z * (BM * BN) + r * BN + c);
      sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
    }
    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.C) + (long long)row * p.N + col) =
        make_uint2(pack_bf16x2(sum.x, sum.y), pack_bf16x2(sum.z, sum.w));
  }
}

// ---------------------------------------------------------------- fp32 FMA twin
// Same six products for fp32 activations/weights: 64x64 output tile, 16-deep reduction
// steps, each thread a 4x4 micro-tile, plain FMAs in fp32.
// The weight gradients of a small batch are few tiles with long reductions: they also come with
// a 32x32 tile (2x2 micro-tile) that makes four times as many workgroups.
constexpr int FK = 16;

template <int MODE, int FB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams p) {
  constexpr int MT = FB / 16;             // micro-tile edge of a thread
  constexpr int NH = FB * FK / 256;       // elements per operand a thread carries per step
  static_assert(FB == 64 || (FB == 32 && MODE >= WGRAD2), "32x32 tiles serve the weight gradients");
  __shared__ float As[FK][FB + 4];
  __shared__ float Bs[FK][FB + 4];
  const int tid = threadIdx.x;
  constexpr bool VARM = MODE <= BWD_DX;
  int row0, row1, group, kbeg = 0, K;
  if (VARM) {
    // fp32 tiles are 64 rows: each 256-row entry of the table is walked in four quarters
    const int mt = blockIdx.y >> 2;
    if (mt >= p.tile_map[0]) return;
    row0 = p.tile_map[4 + 4 * mt] + (blockIdx.y & 3) * FB;
    row1 = p.tile_map[4 + 4 * mt + 1];
    if (row0 >= row1) return;
    row1 = min(row1, row0 + FB);
    group = p.tile_map[4 + 4 * mt + 2];
    K = p.K;
  } else {
    group = blockIdx.z;
    row0 = blockIdx.y * FB;
    row1 = min(p.M, row0 + FB);
    if (p.per_slot) {
      kbeg = p.slot_offsets[group];
      K = p.slot_offsets[group + 1] - kbeg;
    } else {
      kbeg = p.slot_offsets[p.first_slot[group]];
      K = p.slot_offsets[p.first_slot[group + 1]] - kbeg;
    }
    if (K == 0 && p.skip_empty) return;
  }
  const int n0 = blockIdx.x * (MODE == FWD1 ? FB / 2 : FB);
  const float* A = static_cast<const float*>(p.A);
  const float* B = static_cast<const float*>(p.B) + (VARM ? (long long)group * p.b_group_stride : 0);
  const long long d = p.d, f = p.f;

  // element (tile row i, reduction index k) of each operand, or 0 outside
  auto a_at = [&](int i, int k) -> float {
    const int r = row0 + i;
    if (r >= row1 || k >= K) return 0.f;
    switch (MODE) {
      case FWD1: return A[r * d + k];
      case FWD2: return A[r * f + k];
      case BWD_DH: return A[r * d + k];
      case BWD_DX: return A[r * 2 * f + k];
      case WGRAD2: return A[(long long)(kbeg + k) * d + r];
      default: return A[(long long)(kbeg + k) * 2 * f + r];
    }
  };
  auto b_at = [&](int j, int k) -> float {
    if (k >= K) return 0.f;
    switch (MODE) {
      case FWD1: {  // tile columns 0..31 gate, 32..63 up of hidden units n0..n0+31
        const int hu = n0 + (j & 31);
        if (hu >= f) return 0.f;
        return B[((j >> 5) ? f + hu : hu) * d + k];
      }
      case FWD2: return n0 + j < p.N ? B[(long long)(n0 + j) * f + k] : 0.f;
      case BWD_DH: return n0 + j < p.N ? B[(long long)k * f + n0 + j] : 0.f;
      case BWD_DX: return n0 + j < p.N ? B[(long long)k * d + n0 + j] : 0.f;
      case WGRAD2: return n0 + j < p.N ? B[(long long)(kbeg + k) * f + n0 + j] : 0.f;
      default: return n0 + j < p.N ? B[(long long)(kbeg + k) * d + n0 + j] : 0.f;
    }
  };
  constexpr bool A_KC = VARM, B_KC = MODE == FWD1 || MODE == FWD2;

  float acc[MT][MT] = {};
  const int ty = tid >> 4, tx = tid & 15;  // rows ty*MT.., cols tx + 16*c (FWD1 pairs gate/up)
  // each thread carries 4 + 4 elements of a step from memory to LDS; the elements of the next
  // step are fetched into registers before the current step's FMAs, so their latency hides
  // behind them.  Operands are walked along their contiguous index for coalescing.
  float na[NH], nb[NH];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const int e = tid + 256 * h;
      const int ai = A_KC ? e / FK : e % FB, ak = A_KC ? e % FK : e / FB;
      na[h] = a_at(ai, k0 + ak);
      const int bj = B_KC ? e / FK : e % FB, bk = B_KC ? e % FK : e / FB;
      nb[h] = b_at(bj, k0 + bk);
    }
  };
  if (K > 0) fetch(0);
  for (int k0 = 0; k0 < K; k0 += FK) {
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const int e = tid + 256 * h;
      const int ai = A_KC ? e / FK : e % FB, ak = A_KC ? e % FK : e / FB;
      As[ak][ai] = na[h];
      const int bj = B_KC ? e / FK : e % FB, bk = B_KC ? e % FK : e / FB;
      Bs[bk][bj] = nb[h];
    }
    __syncthreads();
    if (k0 + FK < K) fetch(k0 + FK);
    // two-level summation: each 16-deep partial sum is formed on its own and then added,
    // which keeps the rounding error of long reductions (weight gradients) near sqrt(K/16)
    float part[MT][MT] = {};
#pragma unroll
    for (int k = 0; k < FK; ++k) {
      float a[MT], b[MT];
#pragma unroll
      for (int i = 0; i < MT; ++i) a[i] = As[k][ty * MT + i];
#pragma unroll
      for (int c = 0; c < MT; ++c) b[c] = Bs[k][tx + 16 * c];
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int c = 0; c < MT; ++c) part[i][c] = fmaf(a[i], b[c], part[i][c]);
    }
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int c = 0; c < MT; ++c) acc[i][c] += part[i][c];
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int row = row0 + ty * MT + i;
    if (row >= row1) continue;
    if constexpr (MODE == FWD1) {
      // columns tx, tx+16 are gate of hidden units n0+tx, n0+tx+16; tx+32, tx+48 their up
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int hu = n0 + tx + 16 * c;
        if (hu >= f) continue;
        const float u = acc[i][c], v = acc[i][c + 2];
        float* UVo = static_cast<float*>(p.UVout);
        UVo[row * 2 * f + hu] = u;
        UVo[row * 2 * f + f + hu] = v;
        static_cast<float*>(p.H)[row * f + hu] = silu_f(u) * v;
      }
    } else {
#pragma unroll
      for (int c = 0; c < MT; ++c) {
        const int col = n0 + tx + 16 * c;
        if (col >= p.N) continue;
        const float x = acc[i][c];
        if (MODE == FWD2 || MODE == BWD_DX) {
          static_cast<float*>(p.C)[(long long)row * p.N + col] = x;
        } else if (MODE == BWD_DH) {
          const float* UVi = static_cast<const float*>(p.UV);
          const float u = UVi[row * 2 * f + col], v = UVi[row * 2 * f + f + col];
          const float sg = sigmoid_f(u);
          float* Co = static_cast<float*>(p.C);
          Co[row * 2 * f + col] = x * v * sg * (1.f + u * (1.f - sg));
          Co[row * 2 * f + f + col] = x * u * sg;
        } else {
          (static_cast<float*>(p.C) + (long long)group * p.c_group_stride)[(long long)row * p.N + col] = x;
        }
      }
    }
  }
}

template <int MODE>
static void launch_gemm(const symi_ctx* ctx, const GemmParams& p, int n_cols, int max_mtiles,
                        hipStream_t st) {
  const symi_cfg* const cfg = &ctx->cfg;
  if (cfg->dtype == SYMI_BF16) {
    const int bn = MODE == FWD1 ? BN / 2 : BN;
    const int ntx = cdiv(n_cols, bn);
    // FWD2, BWD_DX: room for the slices of the last round's tiles (at most cus workgroups more)
    const bool may_slice = (MODE == FWD2 || MODE == BWD_DX) && p.partials && cdiv(p.K, BK) / 16 >= 2;
    const int extra = may_slice ? cdiv(p.cus, ntx) : 0;
    dim3 grid(ntx, MODE <= BWD_DX ? max_mtiles + extra : cdiv(p.M, BM), MODE <= BWD_DX ? 1 : (p.per_slot ? cfg->S_tot : cfg->E));
    SYMI_TIMED(ctx, K_GEMM_FWD1 + MODE, st, (gemm_bf16_kernel<MODE><<<grid, GT, 0, st>>>(p)));
    if (may_slice)   // the sliced round holds at most cus / 2 tiles
      SYMI_TIMED(ctx, K_SLICE_SUM, st, (slice_sum_kernel<<<dim3(BM / 16, std::max(1, p.cus / 2)), 256, 0, st>>>(p, ntx)));
  } else {
    constexpr int FB = 64;
    const int bn = MODE == FWD1 ? FB / 2 : FB;
    const int groups = p.per_slot ? cfg->S_tot : cfg->E;
    if constexpr (MODE >= WGRAD2) {
      // few tiles (a small batch leaves most of them to a handful of classes): quarter tiles
      if ((long long)cdiv(n_cols, FB) * cdiv(p.M, FB) * groups < 4LL * ctx->cus) {
        dim3 grid(cdiv(n_cols, 32), cdiv(p.M, 32), groups);
        SYMI_TIMED(ctx, K_GEMM_FWD1 + MODE, st, (gemm_f32_kernel<MODE, 32><<<grid, 256, 0, st>>>(p)));
        return;
      }
    }
    dim3 grid(cdiv(n_cols, bn), MODE <= BWD_DX ? 4 * max_mtiles : cdiv(p.M, FB), MODE <= BWD_DX ? 1 : groups);
    SYMI_TIMED(ctx, K_GEMM_FWD1 + MODE, st, (gemm_f32_kernel<MODE, 64><<<grid, 256, 0, st>>>(p)));
  }
}

// where sliced reductions keep their partial tiles (bf16 configurations only)
static void set_split(const symi_ctx* ctx, void* ws, GemmParams& p) {
  p.cus = std::min(ctx->cus, SPLIT_CUS);
  p.partials = ctx->slicing && ctx->cfg.dtype == SYMI_BF16
                   ? reinterpret_cast<float*>(static_cast<char*>(ws) + ctx->L.split_part) : nullptr;
}

}  // namespace symi

using namespace symi;

extern "C" int symi_expert_fwd(const symi_ctx* ctx, const void* Xp, const int32_t* slot_offsets,
                               const void* W1_slots, const void* W2_slots, void* UV, void* H,
                               void* Yp, void* ws, void* stream) {
  SYMI_ENTER(ctx, "symi_expert_fwd");
  const long long A = (long long)cfg->T * cfg->k;
  if (A == 0) return SYMI_OK;
  SYMI_REQUIRE(Xp && slot_offsets && W1_slots && W2_slots && UV && H && Yp && ws, "symi_expert_fwd",
               "NULL pointer");
  hipStream_t st = as_stream(stream);
  const WsLayout& L = ctx->L;
  int32_t* map = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.tile_map);
  const int max_mtiles = (int)(A / GEMM_BM) + cfg->S_tot;
  SYMI_TIMED(ctx, K_TILE_MAP, st, (tile_map_kernel<<<1, 256, 0, st>>>(slot_offsets, nullptr, cfg->S_tot, cfg->E, map, nullptr)));

  GemmParams p = {};
  p.tile_map = map;
  set_split(ctx, ws, p);
  p.d = cfg->d;
  p.f = cfg->f;
  // u|v = Xp W1^T, h = silu(u)*v
  p.A = Xp; p.B = W1_slots; p.UVout = UV; p.H = H;
  p.b_group_stride = 2LL * cfg->f * cfg->d;
  p.N = cfg->f; p.K = cfg->d;
  launch_gemm<FWD1>(ctx, p, cfg->f, max_mtiles, st);
  // Yp = h W2^T
  p.A = H; p.B = W2_slots; p.C = Yp;
  p.b_group_stride = (long long)cfg->d * cfg->f;
  p.N = cfg->d; p.K = cfg->f;
  launch_gemm<FWD2>(ctx, p, cfg->d, max_mtiles, st);
  SYMI_LAUNCH_CHECK("symi_expert_fwd");
  return SYMI_OK;
}

// The backward's five products form two chains that only meet at du|dv:
//   dh -> du|dv -> dXp          and          dW2 (needs dYp, H only) -> dW1 (needs du|dv)
// Run back to back each launch rounds its tile count up to whole rounds of 256 workgroups
// (config c2: 296 tiles of the dXp product are two rounds, the second one 84 % empty) and
// the store-bound zero tiles of the weight gradients never meet the MFMA-bound tiles.  The
// second chain is therefore enqueued on the context's helper stream (created by symi_create
// when the flags allow it and the dXp product has fewer than 8 rounds of tiles; default
// priority, non-blocking), forked from and joined back into the caller's stream with events,
// so workgroups of both chains share the chip.  Otherwise everything stays on the caller's
// stream, in order.

// per_slot = false: dW1_out / dW2_out are per class (all replica slots summed in the GEMM);
// per_slot = true: one gradient per replica slot (its own rows only)
static int expert_bwd_impl(const char* who, const symi_ctx* ctx, const void* dYp, const void* Xp,
                           const void* UV, const void* H, const int32_t* slot_offsets,
                           const int32_t* first_slot, const void* W1_slots, const void* W2_slots,
                           void* dXp, float* dW1_class, float* dW2_class, void* ws, void* stream,
                           bool per_slot, bool skip_empty = false) {
  SYMI_ENTER(ctx, who);
  const long long A = (long long)cfg->T * cfg->k;
  SYMI_REQUIRE(slot_offsets && first_slot && dW1_class && dW2_class && ws, who, "NULL pointer");
  SYMI_REQUIRE(A == 0 || (dYp && Xp && UV && H && W1_slots && W2_slots && dXp), who, "NULL pointer");
  hipStream_t st = as_stream(stream);
  const WsLayout& L = ctx->L;
  int32_t* map = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.tile_map);
  void* dUV = static_cast<char*>(ws) + L.duv;
  const int max_mtiles = (int)(A / GEMM_BM) + cfg->S_tot;

  int32_t* order = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + L.class_order);
  GemmParams p = {};
  p.tile_map = map;
  p.slot_offsets = slot_offsets;
  p.first_slot = first_slot;
  p.class_order = order;
  p.per_slot = per_slot ? 1 : 0;
  p.skip_empty = skip_empty ? 1 : 0;
  set_split(ctx, ws, p);
  p.d = cfg->d;
  p.f = cfg->f;
  SYMI_TIMED(ctx, K_TILE_MAP, st, (tile_map_kernel<<<1, 256, 0, st>>>(slot_offsets, first_slot, cfg->S_tot, cfg->E, map, order)));
  // worth it only while a product is a few rounds of workgroups: with many rounds the chip is
  // full anyway and two kernels sharing it only disturb each other's L2 locality (symi_create
  // decides; the context then holds the helper stream)
  const bool side = ctx->side != nullptr && A > 0;
  hipStream_t sw = st;   // stream of the weight-gradient chain
  if (side) {
    if (hipEventRecord(ctx->fork, st) != hipSuccess || hipStreamWaitEvent(ctx->side, ctx->fork, 0) != hipSuccess) {
      set_error("%s: forking onto the helper stream failed", who);
      return SYMI_EHIP;
    }
    sw = ctx->side;
  }
  // class gradients, first half (classes without rows get zeros: their reduction is empty)
  GemmParams pw = p;
  pw.A = dYp; pw.B = H; pw.C = dW2_class;
  pw.c_group_stride = (long long)cfg->d * cfg->f;
  pw.M = cfg->d; pw.N = cfg->f;
  launch_gemm<WGRAD2>(ctx, pw, cfg->f, 0, sw);
  if (A > 0) {
    // dh = dYp W2, turned into du, dv in the epilogue (dh itself never reaches memory)
    p.A = dYp; p.B = W2_slots; p.C = dUV; p.UV = UV;
    p.b_group_stride = (long long)cfg->d * cfg->f;
    p.N = cfg->f; p.K = cfg->d;
    launch_gemm<BWD_DH>(ctx, p, cfg->f, max_mtiles, st);
    if (side) {   // du|dv is complete: the other chain may go on to dW1
      if (hipEventRecord(ctx->mid, st) != hipSuccess || hipStreamWaitEvent(ctx->side, ctx->mid, 0) != hipSuccess) {
        set_error("%s: event hand-over between the two streams failed", who);
        return SYMI_EHIP;
      }
    }
    // dXp = dUV W1
    p.A = dUV; p.B = W1_slots; p.C = dXp;
    p.b_group_stride = 2LL * cfg->f * cfg->d;
    p.N = cfg->d; p.K = 2 * cfg->f;
    launch_gemm<BWD_DX>(ctx, p, cfg->d, max_mtiles, st);
  }
  pw.A = dUV; pw.B = Xp; pw.C = dW1_class;
  pw.c_group_stride = 2LL * cfg->f * cfg->d;
  pw.M = 2 * cfg->f; pw.N = cfg->d;
  launch_gemm<WGRAD1>(ctx, pw, cfg->d, 0, sw);
  if (side) {
    if (hipEventRecord(ctx->join, ctx->side) != hipSuccess || hipStreamWaitEvent(st, ctx->join, 0) != hipSuccess) {
      set_error("%s: joining the helper stream failed", who);
      return SYMI_EHIP;
    }
  }
  SYMI_LAUNCH_CHECK(who);
  return SYMI_OK;
}

extern "C" int symi_expert_bwd(const symi_ctx* ctx, const void* dYp, const void* Xp, const void* UV,
                               const void* H, const int32_t* slot_offsets, const int32_t* first_slot,
                               const void* W1_slots, const void* W2_slots, void* dXp,
                               float* dW1_class, float* dW2_class, void* ws, void* stream) {
  return expert_bwd_impl("symi_expert_bwd", ctx, dYp, Xp, UV, H, slot_offsets, first_slot, W1_slots,
                         W2_slots, dXp, dW1_class, dW2_class, ws, stream, false);
}

extern "C" int symi_expert_bwd_active(const symi_ctx* ctx, const void* dYp, const void* Xp,
                                      const void* UV, const void* H, const int32_t* slot_offsets,
                                      const int32_t* first_slot, const void* W1_slots,
                                      const void* W2_slots, void* dXp, float* dW1_class,
                                      float* dW2_class, void* ws, void* stream) {
  return expert_bwd_impl("symi_expert_bwd_active", ctx, dYp, Xp, UV, H, slot_offsets, first_slot,
                         W1_slots, W2_slots, dXp, dW1_class, dW2_class, ws, stream, false, true);
}

extern "C" int symi_expert_bwd_slots(const symi_ctx* ctx, const void* dYp, const void* Xp,
                                     const void* UV, const void* H, const int32_t* slot_offsets,
                                     const int32_t* first_slot, const void* W1_slots,
                                     const void* W2_slots, void* dXp, float* dW1_slot,
                                     float* dW2_slot, void* ws, void* stream) {
  return expert_bwd_impl("symi_expert_bwd_slots", ctx, dYp, Xp, UV, H, slot_offsets, first_slot,
                         W1_slots, W2_slots, dXp, dW1_slot, dW2_slot, ws, stream, true);
}

// ---------------------------------------------------------------- replica all-reduce
// The intra-rank part of the paper's all-reduce (Sec. 4.1): for every class the first of its
// slots is the representative; the other slots add their gradient to it (slot order), the
// sum is scaled and copied back to all of them.  16 bytes per lane, one class per blockIdx.y.
namespace symi {
__global__ __launch_bounds__(256) void replica_allreduce_kernel(float4* __restrict__ g,
                                                                const int32_t* __restrict__ first_slot,
                                                                long long n4, float scale) {
  const int e = blockIdx.y;
  const int q0 = first_slot[e], q1 = first_slot[e + 1];
  if (q1 - q0 == 1 && scale == 1.f) return;   // a single replica: nothing to exchange
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long long)gridDim.x * 256) {
    float4 a = g[(long long)q0 * n4 + i];
    for (int q = q0 + 1; q < q1; ++q) {
      const float4 b = g[(long long)q * n4 + i];
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    a.x *= scale; a.y *= scale; a.z *= scale; a.w *= scale;
    for (int q = q0; q < q1; ++q) g[(long long)q * n4 + i] = a;
  }
}
}  // namespace symi

extern "C" int symi_replica_allreduce(const symi_ctx* ctx, const int32_t* first_slot, float scale,
                                      float* dW1_slot, float* dW2_slot, void* stream) {
  SYMI_ENTER(ctx, "symi_replica_allreduce");
  SYMI_REQUIRE(first_slot && dW1_slot && dW2_slot, "symi_replica_allreduce", "NULL pointer");
  hipStream_t st = as_stream(stream);
  const long long n1 = 2LL * cfg->f * cfg->d / 4, n2 = (long long)cfg->d * cfg->f / 4;
  auto blocks = [](long long n4) { long long b = (n4 + 255) / 256; return (unsigned)(b > 2048 ? 2048 : (b < 1 ? 1 : b)); };
  SYMI_TIMED(ctx, K_REPLICA_AR, st, (replica_allreduce_kernel<<<dim3(blocks(n1), cfg->E), 256, 0, st>>>(
      reinterpret_cast<float4*>(dW1_slot), first_slot, n1, scale)));
  SYMI_TIMED(ctx, K_REPLICA_AR, st, (replica_allreduce_kernel<<<dim3(blocks(n2), cfg->E), 256, 0, st>>>(
      reinterpret_cast<float4*>(dW2_slot), first_slot, n2, scale)));
  SYMI_LAUNCH_CHECK("symi_replica_allreduce");
  return SYMI_OK;
}
