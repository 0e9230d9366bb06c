// MFMA GEMM kernels of the coded products (O1, O2) and of the coded rank-b update (O3).
//
// One kernel template serves the three contractions of a layer step.  With
// "A[i][k]" the operand whose index i is contiguous in the result and "B[j][k]"
// the other one, the result is C[j][i] = sum_k A[i][k] B[j][k]:
//   forward  : i = coded row of W~,    j = batch, k = base column;  A = W~ (k contiguous),
//              B = [x; x~] batch-major (k contiguous)
//   backward : i = coded column of W~, j = batch, k = base row;     A = W~ (k strided),
//              B = [delta; delta~] batch-major (k contiguous)
//   update   : i = coded column, j = coded row, k = batch;          A = [x; x~], B = [delta; delta~]
//              (both k strided), C = W~ accumulated in place.
// All operands are float32 in memory and are multiplied with v_mfma_f32_32x32x2_f32
// (the bf16 mode has kernels of its own, gemm_bf16.hip).  The update of a thin batch into a
// large matrix has a kernel of its own as well (update_thin_kernel, below).
//
// Tiling: 256 threads = 4 wavefronts in a 2 x 2 arrangement, each owning
// FM x FN MFMA tiles of 32 x 32, so a workgroup computes (64 FM) x (64 FN).
// A k-slab is 8 chunks of 16 bytes per operand row (32 floats); LDS
// rows are 128 bytes, chunk c of row r sits at slot c ^ swz(r), which keeps
// both the 16-byte fragment reads (32 consecutive rows, one chunk) and the
// transposing writes (rows 4 apart, one chunk) free of bank conflicts.
// Global loads are staged in registers one slab ahead (double-buffered LDS,
// one barrier per slab).  Operands stored k-strided are transposed in
// registers between the global load and the LDS write, so no transposed copy
// of W~ exists anywhere.
#include "codenet_internal.h"

namespace codenet {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int swz(int row) { return ((row & 7) + (row >> 3)) & 7; }

__device__ __forceinline__ float f4get(const float4 &v, int e) {
  return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
}

__device__ __forceinline__ uint4 pack_f32x4(float a0, float a1, float a2, float a3) {
  float4 t = make_float4(a0, a1, a2, a3);
  return __builtin_bit_cast(uint4, t);
}

// Stages one operand slab (T rows x 8 chunks) from global memory to LDS.
template <int T, bool KC>
struct Loader {
  static constexpr int EPC = 4;                            // elements per 16-byte chunk
  static constexpr int NTASK = KC ? T * 8 : (T / 4) * 8;   // KC: (row, chunk); else (4 rows, chunk)
  static constexpr int PER = (NTASK + 255) / 256;
  static constexpr int NF4 = KC ? EPC / 4 : EPC;           // float4 loads per task
  float4 st[PER][NF4];

  __device__ __forceinline__ void load(const float *__restrict__ src, long ld, int row0, int rows,
                                       int k0, int K, int tid) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      const int q = tid + p * 256;
      const bool live = (NTASK % 256 == 0) || q < NTASK;
      if (KC) {
        const int row = q >> 3, c = q & 7;
        const int gr = row0 + row, gk = k0 + c * EPC;
        const bool okr = live && gr < rows;
        const float *ptr = src + (long)gr * ld + gk;
#pragma unroll
        for (int f = 0; f < NF4; ++f)
          st[p][f] = (okr && gk + 4 * f < K) ? *reinterpret_cast<const float4 *>(ptr + 4 * f)
                                             : make_float4(0.f, 0.f, 0.f, 0.f);
      } else {
        const int ig = q % (T / 4), kg = q / (T / 4);
        const int gr = row0 + ig * 4;
        const bool okr = live && gr < rows;
#pragma unroll
        for (int f = 0; f < NF4; ++f) {
          const int gk = k0 + kg * EPC + f;
          st[p][f] = (okr && gk < K) ? *reinterpret_cast<const float4 *>(src + (long)gk * ld + gr)
                                     : make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
    }
  }

  __device__ __forceinline__ void store(uint4 *lds, int tid) const {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      const int q = tid + p * 256;
      if (!((NTASK % 256 == 0) || q < NTASK)) continue;
      if (KC) {
        const int row = q >> 3, c = q & 7;
        lds[row * 8 + (c ^ swz(row))] = __builtin_bit_cast(uint4, st[p][0]);
      } else {
        const int ig = q % (T / 4), kg = q / (T / 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int row = ig * 4 + e;
          lds[row * 8 + (kg ^ swz(row))] = pack_f32x4(f4get(st[p][0], e), f4get(st[p][1], e), f4get(st[p][2], e),
                                                       f4get(st[p][3], e));
        }
      }
    }
  }
};

template <int FM, int FN, bool AKC, bool BKC, bool ACCUM>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
  constexpr int TI = 64 * FM, TJ = 64 * FN;
  constexpr int EPC = 4, KT = 8 * EPC;
  constexpr int STAGE = (TI + TJ) * 8;                     // chunks per LDS stage
  extern __shared__ uint4 lds[];

  // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs (8 of
  // them, one L2 each); give each XCD a contiguous run of tiles so that tiles
  // sharing an operand panel share an L2.
  const int nt = g.tiles_i * g.tiles_j * g.splits;
  const int per = (nt + 7) >> 3;
  const int logical = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
  if (logical >= nt) return;
  const int split = logical % g.splits, tile = logical / g.splits;
  const int tj = tile % g.tiles_j, ti = tile / g.tiles_j;
  const int i0 = ti * TI, j0 = tj * TJ;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wi = wave & 1, wj = wave >> 1;
  const int l32 = lane & 31, h = lane >> 5;

  Loader<TI, AKC> la;
  Loader<TJ, BKC> lb;

  floatx16 acc[FM][FN];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  // this workgroup's share of the slabs (all of them unless the contraction is split)
  const int nk_all = (g.K + KT - 1) / KT;
  const int kb = (int)((long)split * nk_all / g.splits), nk = (int)((long)(split + 1) * nk_all / g.splits);
  la.load(g.A, g.lda, i0, g.I, kb * KT, g.K, tid);
  lb.load(g.B, g.ldb, j0, g.J, kb * KT, g.K, tid);
  la.store(lds, tid);
  lb.store(lds + TI * 8, tid);
  __syncthreads();

  for (int kt = kb; kt < nk; ++kt) {
    const int cur = (kt - kb) & 1;
    if (kt + 1 < nk) {
      la.load(g.A, g.lda, i0, g.I, (kt + 1) * KT, g.K, tid);
      lb.load(g.B, g.ldb, j0, g.J, (kt + 1) * KT, g.K, tid);
    }
    const uint4 *sa = lds + cur * STAGE;
    const uint4 *sb = sa + TI * 8;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int c = 2 * s + h;
      uint4 av[FM], bv[FN];
#pragma unroll
      for (int a = 0; a < FM; ++a) {
        const int row = (wi * FM + a) * 32 + l32;
        av[a] = sa[row * 8 + (c ^ swz(row))];
      }
#pragma unroll
      for (int b = 0; b < FN; ++b) {
        const int row = (wj * FN + b) * 32 + l32;
        bv[b] = sb[row * 8 + (c ^ swz(row))];
      }
#pragma unroll
      for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b) {
          const float4 af = __builtin_bit_cast(float4, av[a]);
          const float4 bf = __builtin_bit_cast(float4, bv[b]);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af.x, bf.x, acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af.y, bf.y, acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af.z, bf.z, acc[a][b], 0, 0, 0);
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af.w, bf.w, acc[a][b], 0, 0, 0);
        }
    }
    if (kt + 1 < nk) {
      uint4 *nx = lds + (cur ^ 1) * STAGE;
      la.store(nx, tid);
      lb.store(nx + TI * 8, tid);
    }
    __syncthreads();
  }

  // Accumulator element 4 g + e of a 32 x 32 tile is (i = 8 g + 4 h + e, j = lane % 32):
  // four consecutive i per lane.
  if (ACCUM) {
    // Read-modify-write of C through an LDS copy of the tile, so that every global access is a
    // whole row segment (a wavefront instruction moves 1 KB of one or a few rows).  Straight from
    // the accumulators, a lane's float4 is a 16-byte piece of its own row: 64 rows per
    // instruction, every 128-byte line requested eight times -- the 18432 x 18432 update of a
    // batch of 64 spent 1.07 ms on 170 M such requests.
    constexpr int PITCH = TI + 4;                          // floats; 16-byte aligned rows, skewed banks
    float *tile = reinterpret_cast<float *>(lds);          // the operand stages are free (barrier above)
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
      for (int b = 0; b < FN; ++b) {
        const int jl = (wj * FN + b) * 32 + l32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int il = (wi * FM + a) * 32 + 8 * q + 4 * h;
          *reinterpret_cast<float4 *>(tile + jl * PITCH + il) =
              make_float4(acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
        }
      }
    __syncthreads();
    constexpr int QPR = TI / 4;                            // float4 per tile row
    constexpr int PASSES = TJ * QPR / 256;
    constexpr int CH = PASSES < 8 ? PASSES : 8;            // accesses in flight per thread
    static_assert(TJ * QPR % 256 == 0 && PASSES % CH == 0, "tile rows divide among the threads");
    for (int p0 = 0; p0 < PASSES; p0 += CH) {
      float4 o[CH], v[CH];
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const int idx = tid + 256 * (p0 + u);
        const int jl = idx / QPR, il = (idx % QPR) * 4;
        const bool in = j0 + jl < g.J && i0 + il < g.I;
        o[u] = in ? *reinterpret_cast<const float4 *>(g.C + (long)(j0 + jl) * g.ldc + i0 + il) : make_float4(0.f, 0.f, 0.f, 0.f);
        v[u] = *reinterpret_cast<const float4 *>(tile + jl * PITCH + il);
      }
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const int idx = tid + 256 * (p0 + u);
        const int jl = idx / QPR, il = (idx % QPR) * 4;
        if (j0 + jl < g.J && i0 + il < g.I)
          *reinterpret_cast<float4 *>(g.C + (long)(j0 + jl) * g.ldc + i0 + il) =
              make_float4(o[u].x + g.alpha * v[u].x, o[u].y + g.alpha * v[u].y, o[u].z + g.alpha * v[u].z,
                          o[u].w + g.alpha * v[u].w);
      }
    }
    return;
  }
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b) {
      const int j = j0 + (wj * FN + b) * 32 + l32;
      if (j >= g.J) continue;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int i = i0 + (wi * FM + a) * 32 + 8 * q + 4 * h;
        if (i >= g.I) continue;
        *reinterpret_cast<float4 *>(g.C + (long)split * g.split_stride + (long)j * g.ldc + i) =
            make_float4(acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
      }
    }
}

// ---------------------------------------------------------------------------
// Coded update of a thin batch in float32: C[j][i] += alpha * sum_k A[k][i] B[k][j] with a
// contraction of a few dozen to a few hundred (the batch), which makes it a read-modify-write of
// the coded matrix with the rate of v_mfma_f32_32x32x2_f32 next to it: at a batch of 64 the MFMAs
// of the 18432 x 18432 update take 277 us at the chip's fp32 matrix peak (525 us measured for this
// kernel's contraction alone, one or two wavefronts per SIMD), the 2.7 GB of the matrix about
// 500 us at the rate a plain in-place pass reaches.
//
// One 128 (i) x 128 (j) tile per workgroup of four wavefronts (2 x 2, 64 x 64 each), two
// workgroups per compute unit: while one contracts, the other's loads and stores are under way.
// (One resident workgroup per compute unit that requests the next tile's operands and old values
// during the contraction of the current one was slower, 805 us against 645 us: it is the second
// wavefront on each SIMD that fills the gaps of the first.)
// The operands are stored batch-major, which is k-major here: a k-row of a tile is 512 contiguous
// bytes, and it goes to LDS as it is (direct-to-LDS loads, 64 k-rows per operand and stage).  The
// MFMA takes one k per half wavefront and one row or column index per lane: the x~ side is the
// column index (lane % 32) and a lane reads columns 2 (lane % 32) and the next with one
// ds_read_b64 as its fragments a = 0, 1, the delta~ side is the row index, one ds_read_b32 per
// fragment.  The matrix does not pass through LDS: a lane owns two adjacent columns of 32 rows;
// their old values are requested (dwordx2, 256 contiguous bytes per half wavefront) before the
// contraction and used after it, the new ones leave with dwordx2 stores.
// ---------------------------------------------------------------------------
typedef float f32x2 __attribute__((ext_vector_type(2)));

#if defined(__HIP_DEVICE_COMPILE__)
#define CN_GEMM_ASM 1
#else
#define CN_GEMM_ASM 0
#endif

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void update_thin_kernel(GemmArgs g) {
  constexpr int KROWS = 64;                    // k-rows per stage
  constexpr int OPB = KROWS * 512;             // bytes of one operand's stage
  extern __shared__ uint4 lds[];
  char *const lds_c = reinterpret_cast<char *>(lds);
  const int nt = g.tiles_i * g.tiles_j;
  const int per = (nt + 7) >> 3;
  const int logical = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
  if (logical >= nt) return;
  // Tiles in bands of eight tile columns (i), walked row by row (j) inside a band: the workgroups
  // resident on an XCD at one time (64) then share eight operand panels of either side.  Walked
  // along j alone they share one x~ panel and use 64 delta~ panels once each, which the matrix
  // streaming through the L2 has evicted when the next tile column wants them again (measured at
  // 18432 x 18432, batch 64: 0.68 GB of operand panels fetched from memory next to the 1.36 GB matrix).
  const int band = logical / (8 * g.tiles_j), rem = logical % (8 * g.tiles_j);
  const int hb = g.tiles_i - 8 * band < 8 ? g.tiles_i - 8 * band : 8;
  const int tj = rem / hb, ti = 8 * band + rem % hb;
  const int i0 = ti * 128, j0 = tj * 128;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wi = wave & 1, wj = wave >> 1;
  const int l32 = lane & 31, h = lane >> 5;

  // fill: load u of a wavefront brings k-rows 2 (4 u + wave) and the next of both operands, 16 bytes per lane
  int ca = i0 + 4 * l32, cb = j0 + 4 * l32;
  ca = ca < g.I ? ca : g.I - 4;
  cb = cb < g.J ? cb : g.J - 4;
  auto fill = [&](int k0) __attribute__((always_inline)) {
#if CN_GEMM_ASM
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int k = k0 + 2 * (4 * u + wave) + h;
      k = k < g.K ? k : g.K - 1;
      __builtin_amdgcn_global_load_lds(g.A + (long)k * g.lda + ca,
                                       (__attribute__((address_space(3))) void *)(lds_c + (4 * u + wave) * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(g.B + (long)k * g.ldb + cb,
                                       (__attribute__((address_space(3))) void *)(lds_c + OPB + (4 * u + wave) * 1024), 16, 0, 0);
    }
#else
    (void)k0;
#endif
  };
  fill(0);
#if CN_GEMM_ASM
  asm volatile("" ::: "memory");            // the old values are requested after the fill: the first wait counts on it
#endif
  __builtin_amdgcn_sched_barrier(0);

  // old values: element x = 4 q + e of fragment row b is row 64 wj + 32 b + 8 q + 4 h + e, columns 64 wi + 2 l32, + 1
  const int ci = i0 + 64 * wi + 2 * l32, rj = j0 + 64 * wj + 4 * h;
  const bool col_in = ci < g.I;
  const float *const pold = g.C + (col_in ? ci : g.I - 2);
  f32x2 old[2][16];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      int row = rj + 32 * b + 8 * (x >> 2) + (x & 3);
      row = row < g.J ? row : g.J - 1;
      old[b][x] = *reinterpret_cast<const f32x2 *>(pold + (long)row * g.ldc);
    }

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  // LDS addresses of this lane's operands in k-row h of a pair
  const unsigned addr_x = (unsigned)(h * 512 + (64 * wi + 2 * l32) * 4);
  const unsigned addr_d = (unsigned)(OPB + h * 512 + (64 * wj + l32) * 4);
  auto read_x = [&](unsigned at) __attribute__((always_inline)) {
    f32x2 v = {0.f, 0.f};
#if CN_GEMM_ASM
    asm volatile("ds_read_b64 %0, %1" : "=v"(v) : "v"(at) : "memory");
#endif
    return v;
  };
  auto read_d = [&](unsigned at, int b) __attribute__((always_inline)) {
    float v = 0.f;
#if CN_GEMM_ASM
    if (b == 0) asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(at) : "memory");
    else asm volatile("ds_read_b32 %0, %1 offset:128" : "=v"(v) : "v"(at) : "memory");
#endif
    return v;
  };

  for (int k0 = 0; k0 < g.K; k0 += KROWS) {
    // everything but the old values (issued after the first fill) has landed
#if CN_GEMM_ASM
    if (k0 == 0) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
    __builtin_amdgcn_s_barrier();
    const int left = g.K - k0;
    const int steps = left >= KROWS ? KROWS / 2 : (left + 1) / 2;
    f32x2 xv = read_x(addr_x);
    float d0 = read_d(addr_d, 0), d1 = read_d(addr_d, 1);
    for (int ks = 0; ks < steps; ++ks) {
      const unsigned nxt = (unsigned)((ks + 1 < steps ? ks + 1 : ks) * 1024);
      const f32x2 xn = read_x(addr_x + nxt);
      const float e0 = read_d(addr_d + nxt, 0), e1 = read_d(addr_d + nxt, 1);
#if CN_GEMM_ASM
      asm volatile("s_waitcnt lgkmcnt(3)" : "+v"(xv), "+v"(d0), "+v"(d1)::"memory");
#endif
      const bool live = 2 * ks + h < left;        // a batch of odd size: its last k-row has no partner
      const float a0 = live ? d0 : 0.f, a1 = live ? d1 : 0.f;
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, xv[0], acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, xv[1], acc[1][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, xv[0], acc[0][1], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, xv[1], acc[1][1], 0, 0, 0);
      xv = xn; d0 = e0; d1 = e1;
    }
#if CN_GEMM_ASM
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(xv), "+v"(d0), "+v"(d1)::"memory");
#endif
    if (k0 + KROWS < g.K) {
      __builtin_amdgcn_s_barrier();              // every wavefront is done with the stage (its reads have returned)
      fill(k0 + KROWS);
    }
  }

  // The old values pass through an empty asm statement: the compiler waits for them once, here, and
  // not before each of the 32 uses below (with a direct-to-LDS load behind it, it waits for everything
  // outstanding every time: each store would wait for the one before it).
#if CN_GEMM_ASM
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int x = 0; x < 16; ++x) asm volatile("" : "+v"(old[b][x]));
#endif
  float *const pnew = g.C + ci;
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      const int row = rj + 32 * b + 8 * (x >> 2) + (x & 3);
      if (col_in && row < g.J)
        *reinterpret_cast<f32x2 *>(pnew + (long)row * g.ldc) =
            f32x2{fmaf(g.alpha, acc[0][b][x], old[b][x][0]), fmaf(g.alpha, acc[1][b][x], old[b][x][1])};
    }
}

namespace {

struct TileChoice { int fm, fn; double eff; };
const TileChoice kTiles[] = {{4, 2, 1.00}, {2, 2, 0.95}, {2, 1, 0.80}, {1, 2, 0.80}, {1, 1, 0.60}};

int pick_tile(const GemmArgs &g) {
  // Cheapest estimated time: rounds of resident workgroups x tile area / tile efficiency.
  int best = 0;
  double best_cost = 1e300;
  for (int t = 0; t < 5; ++t) {
    const int ti = 64 * kTiles[t].fm, tj = 64 * kTiles[t].fn;
    const long nt = (long)((g.I + ti - 1) / ti) * ((g.J + tj - 1) / tj);
    const int lds = 2 * (ti + tj) * 128;
    const int occ = lds * 2 <= 160 * 1024 ? 2 : 1;
    const long rounds = (nt + 256L * occ - 1) / (256L * occ);
    const double cost = (double)rounds * occ * ti * tj / kTiles[t].eff;
    if (cost < best_cost) { best_cost = cost; best = t; }
  }
  return best;
}

template <int FM, int FN, bool AKC, bool BKC, bool ACCUM>
hipError_t launch_one(GemmArgs g, hipStream_t s) {
  constexpr int TI = 64 * FM, TJ = 64 * FN;
  constexpr int stages = 2 * (TI + TJ) * 128, ctile = ACCUM ? TJ * (TI + 4) * 4 : 0;
  constexpr int lds = stages > ctile ? stages : ctile;
  static_assert(lds <= 160 * 1024, "the tile of C does not fit in LDS");
  g.tiles_i = (g.I + TI - 1) / TI;
  g.tiles_j = (g.J + TJ - 1) / TJ;
  // Split-k for products whose tiles do not fill the chip while the contraction is long (thin
  // batches: the kernel then streams the matrix, and a workgroup keeps only one 128-byte slab per
  // row in flight): enough pieces for about eight workgroups per CU, at least 16 slabs each.
  float *final_out = g.C;
  g.splits = 1;
  g.split_stride = 0;
  constexpr int KT = 32;
  const int tiles = g.tiles_i * g.tiles_j, slabs = (g.K + KT - 1) / KT;
  if (!ACCUM && g.workspace != nullptr && tiles < 512 && slabs >= 64) {
    int sp = (2048 + tiles - 1) / tiles;
    if (sp > slabs / 16) sp = slabs / 16;
    if (sp > g.max_splits) sp = g.max_splits;
    if (sp > 1) {
      g.splits = sp;
      g.split_stride = (long)g.J * g.ldc;
      g.C = g.workspace;
    }
  }
  const int nt = tiles * g.splits;
  const int grid = ((nt + 7) / 8) * 8;
  auto kern = gemm_kernel<FM, FN, AKC, BKC, ACCUM>;
  static LdsOnce attr_done;
  hipError_t e = allow_lds(kern, lds, &attr_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, s, g);
  e = hipGetLastError();
  if (e != hipSuccess || g.splits == 1) return e;
  return launch_reduce_partials(g.workspace, g.split_stride, g.splits, final_out, g.split_stride, s);
}

// The update of a thin batch: one 128 x 128 tile per workgroup, 64 KB of LDS (two per compute unit).
hipError_t launch_update_thin(GemmArgs g, hipStream_t s) {
  constexpr int lds = 2 * 64 * 512;
  g.tiles_i = (g.I + 127) / 128;
  g.tiles_j = (g.J + 127) / 128;
  const int nt = g.tiles_i * g.tiles_j;
  const int grid = ((nt + 7) / 8) * 8;
  static LdsOnce attr_done;
  hipError_t e = allow_lds(update_thin_kernel, lds, &attr_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(update_thin_kernel, dim3(grid), dim3(256), lds, s, g);
  return hipGetLastError();
}

template <bool AKC, bool BKC, bool ACCUM>
hipError_t launch_layout(const GemmArgs &g, hipStream_t s) {
  // A short contraction into a large C is a read-modify-write of C with the contraction next to it.
  if (ACCUM && g.K <= 256 && g.I >= 1024 && g.J >= 1024 && (g.ldc & 1) == 0) return launch_update_thin(g, s);
  switch (pick_tile(g)) {
    case 0: return launch_one<4, 2, AKC, BKC, ACCUM>(g, s);
    case 1: return launch_one<2, 2, AKC, BKC, ACCUM>(g, s);
    case 2: return launch_one<2, 1, AKC, BKC, ACCUM>(g, s);
    case 3: return launch_one<1, 2, AKC, BKC, ACCUM>(g, s);
    default: return launch_one<1, 1, AKC, BKC, ACCUM>(g, s);
  }
}

}  // namespace

hipError_t launch_gemm(GemmLayout layout, const GemmArgs &args, hipStream_t stream) {
  // The kernels use 16-byte accesses along every contiguous dimension.
  if ((args.lda & 3) || (args.ldb & 3) || (args.ldc & 3) || (args.I & 3)) return hipErrorInvalidValue;
  if (layout != kUpd && (args.K & 3)) return hipErrorInvalidValue;
  if (layout == kUpd && (args.J & 3)) return hipErrorInvalidValue;
  switch (layout) {
    case kFwd: return launch_layout<true, true, false>(args, stream);
    case kBwd: return launch_layout<false, true, false>(args, stream);
    default: return launch_layout<false, false, true>(args, stream);
  }
}

}  // namespace codenet
