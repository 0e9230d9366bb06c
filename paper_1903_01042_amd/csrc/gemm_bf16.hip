// bf16 MFMA kernels of the coded products (O1, O2) and of the coded update (O3) for gfx950.
//
// C[j][i] (+)= sum_k A[i][k] B[j][k] with A and B bf16 in memory, k contiguous
// ("shadow" copies of the fp32 coded matrix and of the coded vectors, k padded
// with zeros to a multiple of 64), fp32 accumulation, fp32 result.
//
// At the benchmark shape (5120 x 512 x 4096) the MFMA rate is not the bound: per CU the
// global -> LDS fill of a slab takes longer than its MFMAs, and its rate is set by the bytes a
// CU keeps in flight (see product_kernel and product_check_kernel).  Common to the kernels below:
//  * slabs go global -> LDS directly (global_load_lds_dwordx4, no VGPR staging),
//    NS stages deep; a stage is consumed NS-1 iterations after it was requested;
//  * completion is tracked by hand: s_waitcnt vmcnt(n) leaves the younger
//    slabs in flight, one s_barrier per slab;
//  * fragments are read from LDS with ds_read_b128 issued from inline asm one
//    k-step ahead of the MFMAs that use them (the compiler would otherwise
//    drain every outstanding direct-to-LDS load before each LDS read);
//  * LDS rows are 128 bytes (64 bf16), their 16-byte chunks XOR-swizzled by the
//    row (swizzle_of_row below) so that fragment reads are free of bank conflicts;
//    the direct-to-LDS writes are linear per wavefront, and the swizzle is applied
//    by choosing which global chunk each lane fetches;
//  * workgroup ids are dealt to the 8 XCDs round-robin by the hardware; the
//    id -> tile maps give every XCD tiles that share operand panels, hence an L2.
// Kernels: product_kernel (8 wavefronts with separate roles, the two products),
// product_check_kernel (the forward product on tiles of whole codewords with the check's first
// pass in its epilogue), update2_kernel (update, one tile per workgroup), update3_kernel (update,
// persistent and wave-specialised), shadow_kernel.
#include "codenet_internal.h"

namespace codenet {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#define CN_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// The inline asm below only exists in the device pass: the host pass must still
// be able to instantiate the kernel template to emit its launch stub.
#if defined(__HIP_DEVICE_COMPILE__)
#define CN_DEVICE_ASM 1
#else
#define CN_DEVICE_ASM 0
#endif

template <int OFF>
__device__ __forceinline__ u32x4 lds_read16(unsigned addr) {
  u32x4 v = {0u, 0u, 0u, 0u};
#if CN_DEVICE_ASM
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
#endif
  return v;
}

// N fragments of 32 rows each (4096 bytes apart) at the same chunk slot
template <int N>
__device__ __forceinline__ void read_frags(u32x4 (&f)[N], unsigned addr) {
  f[0] = lds_read16<0>(addr);
  if constexpr (N > 1) f[1] = lds_read16<4096>(addr);
  if constexpr (N > 2) f[2] = lds_read16<8192>(addr);
  if constexpr (N > 3) f[3] = lds_read16<12288>(addr);
}

// Transposing LDS read of gfx950 (16-bit elements): in every group of 16 lanes, lane s points at
// four consecutive elements, columns 4 (s % 4) .. + 3 of row s / 4 of a 4 x 16 block, and lane n
// receives column n of that block, rows 0 .. 3 (checked on the device with an index pattern).
template <int OFF>
__device__ __forceinline__ u32x2 lds_read_tr8(unsigned addr) {
  u32x2 v;
#if CN_DEVICE_ASM
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
#else
  v = u32x2{addr, 0u};
#endif
  return v;
}

template <int N>
__device__ __forceinline__ void wait_lgkm() {
#if CN_DEVICE_ASM
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
#endif
}
template <int N>
__device__ __forceinline__ void wait_vm() {
#if CN_DEVICE_ASM
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
#endif
}
// LDS traffic of this wavefront complete, then the workgroup barrier; one asm
// statement with a memory clobber, so no LDS access is moved across it
__device__ __forceinline__ void lds_barrier() {
#if CN_DEVICE_ASM
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#endif
}
// orders the consumers of v after every asm statement issued before this one
__device__ __forceinline__ void pin(u32x4 &v) {
#if CN_DEVICE_ASM
  asm volatile("" : "+v"(v));
#endif
}
__device__ __forceinline__ void pin(u32x2 &v) {
#if CN_DEVICE_ASM
  asm volatile("" : "+v"(v));
#endif
}

// LDS layout of an operand tile: row r (128 bytes = eight 16-byte chunks of k) keeps its
// chunk c at slot c ^ swizzle_of_row(r).  A ds_read_b128 serves 16 lanes at a time; the 16
// rows they read (same chunk) must cover the sixteen 16-byte bank groups: the group is
// 8 (r % 2) + slot, so the swizzle has to take its three bits from r / 2 (with r % 8, rows
// r and r + 8 collide: half of all LDS cycles were bank conflicts).  Every row group that
// a direct-to-LDS load fills starts at a multiple of 8 rows, and 8 * (4 u + wave) or
// 8 * (8 u + wave) differ from 8 * wave by a multiple of 16: one formula serves all loads.
__device__ __forceinline__ int swizzle_of_row(int r) { return (r >> 1) & 7; }

// Main loop shared by the product and the update kernels: acc[a][b] += A-tile x B-tile^T
// over slabs [kb, kb + nk) of 64.  acc rows (MFMA row index) run over j (B rows),
// acc columns (lane % 32) over i (A rows): the B-side fragment is the first MFMA operand.
template <int FM, int FN, int NS>
__device__ __forceinline__ void mainloop(const __bf16 *__restrict__ A, long lda, const __bf16 *__restrict__ B,
                                         long ldb, int I, int J, int i0, int j0, int kb, int nk, char *lds_c,
                                         floatx16 (&acc)[FM][FN]) {
  constexpr int TI = 64 * FM, TJ = 64 * FN;
  constexpr int STAGE = (TI + TJ) * 128;              // bytes per stage
  constexpr int LA = TI / 32, LB = TJ / 32;           // direct-to-LDS loads per lane and slab
  constexpr int LPS = LA + LB;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wi = wave & 1, wj = wave >> 1;
  const int l32 = lane & 31, h = lane >> 5;

  // per-lane sources: lane l of load u fetches, for slot l & 7 of row 8 (4 u + wave) + (l >> 3), the chunk that belongs there
  const int lrow = lane >> 3;
  const int chunk = (lane & 7) ^ swizzle_of_row(8 * wave + lrow);
  const __bf16 *srcA[LA];
  const __bf16 *srcB[LB];
#pragma unroll
  for (int u = 0; u < LA; ++u) {
    int row = i0 + 8 * (4 * u + wave) + lrow;
    row = row < I ? row : I - 1;
    srcA[u] = A + (long)row * lda + (long)kb * 64 + chunk * 8;
  }
#pragma unroll
  for (int u = 0; u < LB; ++u) {
    int row = j0 + 8 * (4 * u + wave) + lrow;
    row = row < J ? row : J - 1;
    srcB[u] = B + (long)row * ldb + (long)kb * 64 + chunk * 8;
  }

  // load u (0 .. LPS-1) of slab kt: A rows first, then B rows
  auto issue_one = [&](int kt, int u) {
#if CN_DEVICE_ASM
    char *sbase = lds_c + (kt % NS) * STAGE;
    if (u < LA)
      __builtin_amdgcn_global_load_lds(srcA[u] + (long)kt * 64, CN_LDS_PTR(sbase + (4 * u + wave) * 1024), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds(srcB[u - LA] + (long)kt * 64,
                                       CN_LDS_PTR(sbase + TI * 128 + (4 * (u - LA) + wave) * 1024), 16, 0, 0);
#else
    (void)kt; (void)u;
#endif
  };
  auto issue = [&](int kt) {
#pragma unroll
    for (int u = 0; u < LPS; ++u) issue_one(kt, u);
  };

  // fragment read addresses (bytes inside a stage) for the 4 k-steps of a slab
  unsigned offA[4], offB[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const unsigned slot = (unsigned)(((2 * s + h) ^ swizzle_of_row(l32)) * 16);
    offA[s] = (unsigned)((wi * FM * 32 + l32) * 128) + slot;
    offB[s] = (unsigned)(TI * 128 + (wj * FN * 32 + l32) * 128) + slot;
  }

#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nk) issue(s);

  for (int kt = 0; kt < nk; ++kt) {
    // slab kt must have landed; up to NS-2 younger slabs stay in flight
    const int later = nk - 1 - kt;
    if (NS >= 4 && later >= 2) wait_vm<2 * LPS>();
    else if (NS >= 3 && later >= 1) wait_vm<LPS>();
    else wait_vm<0>();
    __builtin_amdgcn_s_barrier();
    // The loads of slab kt + NS - 1 are issued a few at a time between the MFMAs
    // of this slab: a wavefront issues in order, and a burst of direct-to-LDS
    // loads would hold back its own MFMAs while the memory pipeline accepts them.
    const bool prefetch = kt + NS - 1 < nk;

    const unsigned sb = (unsigned)((kt % NS) * STAGE);
    u32x4 fa[2][FM], fb[2][FN];
    read_frags<FM>(fa[0], sb + offA[0]);
    read_frags<FN>(fb[0], sb + offB[0]);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int cur = s & 1, nxt = cur ^ 1;
      if (s < 3) {
        read_frags<FM>(fa[nxt], sb + offA[s + 1]);
        read_frags<FN>(fb[nxt], sb + offB[s + 1]);
        wait_lgkm<FM + FN>();      // LDS returns in order: the older step's fragments are in
      } else {
        wait_lgkm<0>();
      }
#pragma unroll
      for (int a = 0; a < FM; ++a) pin(fa[cur][a]);
#pragma unroll
      for (int b = 0; b < FN; ++b) pin(fb[cur][b]);
      constexpr int LQ = LPS / 4;            // loads issued during one k-step
      constexpr int MPL = (FM * FN) / LQ;    // MFMAs between two loads
#pragma unroll
      for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b) {
          const int m = a * FN + b;
          if (m % MPL == 0 && m / MPL < LQ) {
            if (prefetch) issue_one(kt + NS - 1, s * LQ + m / MPL);
            __builtin_amdgcn_sched_barrier(0);
          }
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[cur][b]),
                                                              __builtin_bit_cast(bf16x8, fa[cur][a]), acc[a][b], 0, 0, 0);
        }
    }
  }
}

// workgroup id -> (tile, split): consecutive ids land on different XCDs, so give
// every XCD a contiguous run of logical tiles (tiles sharing an A panel share an L2)
__device__ __forceinline__ int logical_workgroup(int total) {
  const int per = (total + 7) >> 3;
  const int logical = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
  return logical < total ? logical : -1;
}

// ---------------------------------------------------------------------------
// The product kernel (forward and backward products of the bf16 mode): the fill on a SIMD of
// its own.  Wavefront w of a workgroup runs on SIMD w % 4.  Wavefronts 3 and 7 (SIMD 3) only
// issue the direct-to-LDS loads; the other six (two on each of SIMDs 0-2) only read fragments
// and issue MFMAs: a 96 (i) x 128 (j) tile as 3 x 2 wavefronts of 32 x 64, 64-deep slabs of
// 28 KB, five stages (four slabs in flight), one barrier per slab for all eight wavefronts.
// Three quarters of the MFMA units work, on 216 instead of 160 tiles at 5120 x 512.
//
// Why this shape was chosen, and what is known since.  Measured at 5120 x 512 x 4096 with
// ablation builds of a 128 x 128 kernel whose four MFMA wavefronts (one per SIMD, 64 x 64 each)
// and four loader wavefronts are separate (shader clock 2.05 GHz under this load): launch,
// barriers and the epilogue's 10.5 MB of stores 7.5 to 11 us; MFMAs alone 10 to 14 us; fragment
// reads alone 6 us; fill alone 18 us, whether the weights come from HBM or, with every tile
// reading one L2-resident panel, from L2.  Loads + MFMAs 37 us, reads + MFMAs 29 us, all three
// 42 us; the same with the roles mixed in every wavefront (39 to 42 us), with loaders that stage
// through registers (39 us), with a sixth wavefront that prefetches into L2 (46 us), with
// fragments requested one, two or four k-steps ahead (42 to 45 us), and with 160 x 64 tiles on
// all 256 CUs (41 us).  With the loaders on SIMDs 2 and 3 and the MFMA wavefronts on SIMDs 0 and
// 1, loads + MFMAs take 38 us where the MFMAs alone take 36.  This kernel: 31 to 33 us (the
// 128 x 128 kernel with mixed roles: 41.3 us in the same run; hipBLASLt's kernel for this
// product, 160 x 64 x 128 tiles: 32 us).  Kernels that issue only one kind of instruction show
// that the pipes themselves do not get in each other's way: one wavefront per SIMD keeps the
// MFMA pipe 99.8 % busy, LDS reads run at up to 230 bytes per clock and CU, the direct-to-LDS
// fill at up to 57 (50 from HBM), and all three at once at the same rates.  What the structure
// above buys is bytes in flight: a slab period is the loaded latency of a slab's loads divided
// by the slabs in flight, about 650 clocks with 4 x 28 KB here, whatever else the CU does.
// ---------------------------------------------------------------------------
// AT: the A operand is stored k-major, A[k][i] with i contiguous (the row-major bf16 copy of the
// coded matrix seen from the backward product).  Its slab then sits in LDS as 64 rows (k) of
// 96 elements, filled by the same direct-to-LDS loads, and the MFMA wavefronts fetch their
// fragments with the transposing LDS read: two 8-byte reads per fragment instead of one of 16.
template <bool AT>
__global__ __launch_bounds__(512) void product_kernel(Gemm2Args g) {
  constexpr int NS = 5;
  constexpr int A_BYTES = 96 * 128, STAGE = A_BYTES + 128 * 128;
  extern __shared__ uint4 lds[];
  char *const lds_c = reinterpret_cast<char *>(lds);
  const int logical = logical_workgroup(g.tiles_i * g.tiles_j);
  if (logical < 0) return;
  const int tj = logical % g.tiles_j, ti = logical / g.tiles_j;
  const int i0 = ti * 96, j0 = tj * 128;
  const int nk = g.K >> 6;
  const int tid = threadIdx.x;
  const int lane = tid & 63, hw = tid >> 6;

  if ((hw & 3) == 3) {
    // loader lw takes the row groups 2 u + lw of the 28 (12 of A, 16 of B); all of them have
    // the parity of lw inside their operand, so one swizzle serves the fourteen loads
    const int lw = hw >> 2;
    const int lrow = lane >> 3, chunk = (lane & 7) ^ ((4 * lw + (lrow >> 1)) & 7);
    const __bf16 *src[14];
#pragma unroll
    for (int u = 0; u < 14; ++u) {
      const int grp = 2 * u + lw;
      if (u < 6) {
        if (AT) {
          // load grp fills bytes 1024 grp .. + 1023 of the slab: rows of 192 bytes
          const int o = 1024 * grp + 16 * lane;
          int col = i0 + (o % 192) / 2;
          col = col + 8 <= (int)g.lda ? col : (int)g.lda - 8;    // stay inside the row; such columns are never stored
          src[u] = g.A + (long)(o / 192) * g.lda + col;
        } else {
          int row = i0 + 8 * grp + lrow;
          row = row < g.I ? row : g.I - 1;
          src[u] = g.A + (long)row * g.lda + chunk * 8;
        }
      } else {
        int row = j0 + 8 * (grp - 12) + lrow;
        row = row < g.J ? row : g.J - 1;
        src[u] = g.B + (long)row * g.ldb + chunk * 8;
      }
    }
    auto issue = [&](int kt) {
#if CN_DEVICE_ASM
      char *stage = lds_c + (kt % NS) * STAGE;
#pragma unroll
      for (int u = 0; u < 14; ++u)
        __builtin_amdgcn_global_load_lds(src[u] + ((AT && u < 6) ? (long)kt * 64 * g.lda : (long)kt * 64),
                                         CN_LDS_PTR(stage + (2 * u + lw) * 1024), 16, 0, 0);
#else
      (void)kt;
#endif
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (s < nk) issue(s);
    for (int kt = 0; kt < nk; ++kt) {
      // slab kt has landed when only the younger slabs' loads are outstanding
      const int later = nk - 1 - kt;
      if (later >= 3) wait_vm<42>();
      else if (later >= 2) wait_vm<28>();
      else if (later >= 1) wait_vm<14>();
      else wait_vm<0>();
      __builtin_amdgcn_s_barrier();
      // every MFMA wavefront is done with slab kt - 1: its stage takes slab kt + NS - 1
      if (kt + NS - 1 < nk) issue(kt + NS - 1);
    }
    return;
  }

  const int m = (hw & 3) + 3 * (hw >> 2);     // 0 .. 5
  const int wi = m % 3, wj = m / 3;           // 3 x 2 wavefronts over (i, j)
  const int l32 = lane & 31, h = lane >> 5;
  unsigned offA[4], offB[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const unsigned slot = (unsigned)(((2 * s + h) ^ swizzle_of_row(l32)) * 16);
    offA[s] = (unsigned)((wi * 32 + l32) * 128) + slot;
    offB[s] = (unsigned)(A_BYTES + (wj * 64 + l32) * 128) + slot;
  }
  // AT: lane's row of the 4 x 16 block that its group of 16 lanes reads: k = 8 h + (lane % 16) / 4 (+ 4 for the
  // second read, + 16 per k-step), columns wi * 32 + 16 (lane / 16 % 2) + 4 (lane % 4) .. + 3
  const unsigned baseAT = (unsigned)((8 * h + ((lane & 15) >> 2)) * 192 + (wi * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);
  // The halves of a transposed fragment stay two values until their wait has passed: joined
  // earlier, the join could be a register move that reads them before they have landed.
  u32x2 alo[2], ahi[2];
  auto read_a = [&](int slot, unsigned sb, int s, u32x4 &f) {
    if constexpr (AT) {
      const unsigned a = sb + baseAT + (unsigned)(s * 3072);
      alo[slot] = lds_read_tr8<0>(a);
      ahi[slot] = lds_read_tr8<768>(a);
    } else {
      f = lds_read16<0>(sb + offA[s]);
    }
  };
  constexpr int READS = AT ? 4 : 3;            // LDS reads of one k-step
  floatx16 acc[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;

  for (int kt = 0; kt < nk; ++kt) {
    __builtin_amdgcn_s_barrier();
    const unsigned sb = (unsigned)((kt % NS) * STAGE);
    u32x4 fa[2][1], fb[2][2];
    read_a(0, sb, 0, fa[0][0]);
    read_frags<2>(fb[0], sb + offB[0]);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int cur = s & 1, nxt = cur ^ 1;
      if (s < 3) {
        read_a(nxt, sb, s + 1, fa[nxt][0]);
        read_frags<2>(fb[nxt], sb + offB[s + 1]);
        wait_lgkm<READS>();
      } else {
        wait_lgkm<0>();
      }
      if constexpr (AT) {
        pin(alo[cur]); pin(ahi[cur]);
        fa[cur][0] = u32x4{alo[cur][0], alo[cur][1], ahi[cur][0], ahi[cur][1]};
      } else {
        pin(fa[cur][0]);
      }
      pin(fb[cur][0]); pin(fb[cur][1]);
#pragma unroll
      for (int b = 0; b < 2; ++b)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fb[cur][b]),
                                                         __builtin_bit_cast(bf16x8, fa[cur][0]), acc[b], 0, 0, 0);
    }
  }
  // element 4 q + e of fragment b is (j = 8 q + 4 h + e, i = lane % 32)
  const int i = i0 + wi * 32 + l32;
  if (i >= g.I) return;
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = j0 + (wj * 2 + b) * 32 + 8 * q + 4 * h + e;
        if (j < g.J) g.C[(long)j * g.ldc + i] = acc[b][4 * q + e];
      }
}

// ---------------------------------------------------------------------------
// The coded product with the check's first pass in its epilogue (General Error-Detection
// Method: every consistency check is a linear combination of block outputs that sit side by
// side once the tile holds whole codewords).
//
// Tile: 160 rows x 64 batch columns, the rows being the same 16 positions of up to ten blocks
// (row a of the tile is position p0 + a % 16 of block a / 16), so that a workgroup owns
// 16 x 64 complete codewords.  With L = 10 blocks of 512 positions and a batch of 512 that is
// 32 x 8 = 256 tiles: one per compute unit, none idle.  Eight wavefronts: four issue MFMAs
// (v_mfma_f32_16x16x32_bf16, 2 x 2 wavefronts of 80 rows x 32 columns: five blocks times two
// column groups = ten accumulators), four only issue the direct-to-LDS loads.
//
// What bounds the main loop (measured on this kernel and on kernels that issue only one kind of
// instruction): a compute unit takes direct-to-LDS data at up to 57 bytes per clock, MFMAs, these
// loads and LDS fragment reads run side by side without slowing each other, and the MFMAs of a
// 64-deep slab are 320 clocks per wavefront -- yet a slab takes about 650 clocks, with or without
// the MFMAs.  The period is the loaded latency of a slab's loads divided by the slabs in flight
// (NS - 1 = 4 stages of 28 KB, all the LDS that the epilogue leaves), so the loop is bound by bytes
// in flight per compute unit, not by a pipe.  Reading the fragments one k-step ahead, across the
// barrier, is kept because it costs nothing; it gained nothing either.
//
// Only the product with k contiguous in both operands runs here.  The backward product reads
// the row-major matrix k-major: gathering this tile's rows from it takes 32-byte pieces (three
// times the L2 requests) and the transposing LDS reads then conflict two ways; measured at twice
// the time of product_kernel<true> plus detect_kernel, which that product therefore keeps.
//
// Epilogue: the accumulators are stored as the coded output and, from the same registers, each
// lane forms its share of the r syndromes (a lane holds one position of five blocks for four
// batch columns; the two wavefronts that share a column group exchange their halves through
// LDS), writes them for the correction pass, and the workgroup leaves one record of partial sums
// -- squared norms of the blocks, Gram matrix of the syndromes, float64, fixed order -- exactly
// what detect_kernel leaves per workgroup.  The decision kernel then runs on these records.
// ---------------------------------------------------------------------------
template <int R>
__global__ __launch_bounds__(512) void product_check_kernel(Gemm2Args g, CheckArgs c) {
  constexpr int NS = 5;
  constexpr int A_BYTES = 160 * 128, STAGE = A_BYTES + 64 * 128;      // 28 KB
  constexpr int NG = R * (R + 1) / 2;
  extern __shared__ uint4 lds[];
  char *const lds_c = reinterpret_cast<char *>(lds);
  const int logical = logical_workgroup(g.tiles_i * g.tiles_j);
  if (logical < 0) return;
  const int tj = logical % g.tiles_j, tp = logical / g.tiles_j;
  const int p0 = tp * 16, j0 = tj * 64;
  const int nk = g.K >> 6;
  const int tid = threadIdx.x;
  const int lane = tid & 63, hw = tid >> 6;
  const int L = c.L, Bp = c.Bp;

  if (hw >= 4) {
    // ------------------------------------------------------------------ loaders
    // 28 wavefront-loads of 1 KB per slab (20 of A, 8 of B); loader lw takes loads lw, lw + 4, ...
    const int lw = hw - 4;
    const int lrow = lane >> 3;
    const __bf16 *src[7];
#pragma unroll
    for (int u = 0; u < 7; ++u) {
      const int grp = 4 * u + lw;
      if (grp < 20) {
        const int a = 8 * grp + lrow;                    // tile row
        const int blk = a >> 4, pos = p0 + (a & 15);
        const bool ok = blk < L && pos < Bp;
        const int chunk = (lane & 7) ^ swizzle_of_row(a);
        src[u] = g.A + (ok ? (long)blk * Bp + pos : 0) * g.lda + chunk * 8;
      } else {
        const int row = 8 * (grp - 20) + lrow;
        int j = j0 + row;
        j = j < g.J ? j : g.J - 1;
        const int chunk = (lane & 7) ^ swizzle_of_row(row);
        src[u] = g.B + (long)j * g.ldb + chunk * 8;
      }
    }
    auto issue = [&](int kt) {
#if CN_DEVICE_ASM
      char *stage = lds_c + (kt % NS) * STAGE;
#pragma unroll
      for (int u = 0; u < 7; ++u)
        __builtin_amdgcn_global_load_lds(src[u] + (long)kt * 64, CN_LDS_PTR(stage + (4 * u + lw) * 1024), 16, 0, 0);
#else
      (void)kt;
#endif
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (s < nk) issue(s);
    for (int kt = 0; kt < nk; ++kt) {
      const int later = nk - 1 - kt;
      if (later >= 3) wait_vm<21>();
      else if (later >= 2) wait_vm<14>();
      else if (later >= 1) wait_vm<7>();
      else wait_vm<0>();
      __builtin_amdgcn_s_barrier();
      if (kt + NS - 1 < nk) issue(kt + NS - 1);
    }
    // the epilogue's barriers: one before LDS is reused, one for the exchange, three per reduction round
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int c0 = 0; c0 < 10 + NG; c0 += 16) {
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_s_barrier();
    }
    return;
  }

  // ------------------------------------------------------------------ MFMA wavefronts
  const int wi = hw & 1, wj = hw >> 1;
  const int l16 = lane & 15, gq = lane >> 4;
  // fragment addresses inside a stage for the two k-steps of a slab (block s5 adds 2048 / 32 bytes)
  unsigned offA[2], offB[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const unsigned slot = (unsigned)((((4 * ks + gq) ^ (l16 >> 1)) & 7) * 16);
    offB[ks] = (unsigned)(A_BYTES + (32 * wj) * 128 + l16 * 128) + slot;
    offA[ks] = (unsigned)((80 * wi) * 128 + l16 * 128) + slot;
  }
  floatx4 acc[5][2];
#pragma unroll
  for (int s5 = 0; s5 < 5; ++s5)
#pragma unroll
    for (int bj = 0; bj < 2; ++bj) acc[s5][bj] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Fragments are read one k-step ahead of the MFMAs that use them, across the slab boundary as well.
  u32x4 fa[2][5], fb[2][2];
  constexpr int READS = 7;                       // LDS reads of one k-step
  auto read_step = [&](unsigned sb, int ks) {
    const unsigned a = sb + offA[ks], b = sb + offB[ks];
    fa[ks][0] = lds_read16<0>(a);
    fa[ks][1] = lds_read16<2048>(a);
    fa[ks][2] = lds_read16<4096>(a);
    fa[ks][3] = lds_read16<6144>(a);
    fa[ks][4] = lds_read16<8192>(a);
    fb[ks][0] = lds_read16<0>(b);
    fb[ks][1] = lds_read16<2048>(b);
  };
  auto mfma_step = [&](int ks) {
#pragma unroll
    for (int s5 = 0; s5 < 5; ++s5) pin(fa[ks][s5]);
    pin(fb[ks][0]); pin(fb[ks][1]);
#pragma unroll
    for (int s5 = 0; s5 < 5; ++s5)
#pragma unroll
      for (int bj = 0; bj < 2; ++bj)
        acc[s5][bj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fb[ks][bj]),
                                                             __builtin_bit_cast(bf16x8, fa[ks][s5]), acc[s5][bj], 0, 0, 0);
  };
  __builtin_amdgcn_s_barrier();                  // slab 0 has landed
  read_step(0u, 0);
  for (int kt = 0; kt < nk; ++kt) {
    const unsigned sb = (unsigned)((kt % NS) * STAGE);
    read_step(sb, 1);
    wait_lgkm<READS>();                          // LDS returns in order: the first k-step's fragments are in
    mfma_step(0);
    wait_lgkm<0>();                              // all of this wavefront's reads of slab kt are done
    if (kt + 1 < nk) {
      __builtin_amdgcn_s_barrier();              // slab kt + 1 has landed; the loaders may refill the stage of slab kt
      read_step((unsigned)(((kt + 1) % NS) * STAGE), 0);
    }
    mfma_step(1);
  }
  __builtin_amdgcn_s_barrier();                  // every wavefront is done with the operand stages

  // element e of accumulator (s5, bj): block 5 wi + s5, position p0 + lane % 16,
  // batch column j0 + 32 wj + 16 bj + 4 (lane / 16) + e
  const int pos = p0 + l16;
  float sq[5];
  float ps[R][2][4];
#pragma unroll
  for (int k = 0; k < R; ++k)
#pragma unroll
    for (int bj = 0; bj < 2; ++bj)
#pragma unroll
      for (int e = 0; e < 4; ++e) ps[k][bj][e] = 0.f;
#pragma unroll
  for (int s5 = 0; s5 < 5; ++s5) {
    const int blk = 5 * wi + s5;
    const bool row_ok = blk < L && pos < Bp;
    float ssum = 0.f;
#pragma unroll
    for (int bj = 0; bj < 2; ++bj)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = j0 + 32 * wj + 16 * bj + 4 * gq + e;
        const bool ok = row_ok && j < g.J;
        const float v = ok ? acc[s5][bj][e] : 0.f;
        if (ok) g.C[(long)j * g.ldc + (long)blk * Bp + pos] = v;
        ssum = fmaf(v, v, ssum);
#pragma unroll
        for (int k = 0; k < R; ++k) ps[k][bj][e] = fmaf(c.Hf[k][blk < 10 ? blk : 9], v, ps[k][bj][e]);
      }
    sq[s5] = ssum;
  }
  // the halves of the syndromes meet: wavefronts with wi = 1 hand theirs over
  float *const exch = reinterpret_cast<float *>(lds_c + 40960) + wj * (R * 8 * 64);
  if (wi == 1) {
#pragma unroll
    for (int k = 0; k < R; ++k)
#pragma unroll
      for (int bj = 0; bj < 2; ++bj)
#pragma unroll
        for (int e = 0; e < 4; ++e) exch[(k * 8 + bj * 4 + e) * 64 + lane] = ps[k][bj][e];
  }
  __syncthreads();
  float gram[NG];
#pragma unroll
  for (int q = 0; q < NG; ++q) gram[q] = 0.f;
  if (wi == 0) {
#pragma unroll
    for (int k = 0; k < R; ++k)
#pragma unroll
      for (int bj = 0; bj < 2; ++bj)
#pragma unroll
        for (int e = 0; e < 4; ++e) ps[k][bj][e] += exch[(k * 8 + bj * 4 + e) * 64 + lane];
#pragma unroll
    for (int bj = 0; bj < 2; ++bj)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = j0 + 32 * wj + 16 * bj + 4 * gq + e;
        if (pos < Bp && j < g.J) {
#pragma unroll
          for (int k = 0; k < R; ++k) c.syn[((long)k * g.J + j) * Bp + pos] = ps[k][bj][e];
        }
        int q = 0;
#pragma unroll
        for (int k = 0; k < R; ++k)
#pragma unroll
          for (int k2 = k; k2 < R; ++k2, ++q) gram[q] = fmaf(ps[k][bj][e], ps[k2][bj][e], gram[q]);
      }
  }
  // The workgroup's record: ten block norms, then the Gram entries; float64, a 16 x 16 tree per
  // entry over the 256 lanes of the MFMA wavefronts, the same order on every run.
  double (*red)[256] = reinterpret_cast<double (*)[256]>(lds_c);
  double (*red2)[16] = reinterpret_cast<double (*)[16]>(lds_c + 16 * 256 * 8);
#pragma unroll
  for (int c0 = 0; c0 < 10 + NG; c0 += 16) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int en = c0 + u;                       // compile-time after unrolling
      float v = 0.f;
      if (en < 10) v = (en / 5 == wi) ? sq[en % 5] : 0.f;
      else if (en - 10 < NG) v = wi == 0 ? gram[en - 10 < NG ? en - 10 : 0] : 0.f;
      red[u][tid] = (double)v;
    }
    __syncthreads();
    {
      const int u = tid >> 4, part = tid & 15;
      double a = 0.0;
#pragma unroll
      for (int q = 0; q < 16; ++q) a += red[u][part + 16 * q];
      red2[u][part] = a;
    }
    __syncthreads();
    if (tid < 16 && c0 + tid < 10 + NG) {
      double a = 0.0;
#pragma unroll
      for (int q = 0; q < 16; ++q) a += red2[tid][q];
      const int en = c0 + tid;
      const int entry = en < 10 ? en : CODENET_MAX_L + (en - 10);
      if (en >= 10 || en < L) c.partials[(long)entry * kDetectParts + logical] = a;
    }
    __syncthreads();
  }
}

// out = sum over splits of the partial results, in split order
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float4 *__restrict__ part, long stride4,
                                                              int splits, float4 *__restrict__ out, long count4) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= count4) return;
  float4 v = part[idx];
  for (int s = 1; s < splits; ++s) {
    const float4 w = part[(long)s * stride4 + idx];
    v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
  }
  out[idx] = v;
}

// ---------------------------------------------------------------------------
// Coded update (O3 with the three block rules, corner included):
//   W~[j][i] += eta * sum_k delta~[j][k] x~[i][k]      (j coded row, i coded column, k batch)
// Operands are the feature-major bf16 copies of the cached coded vectors.  The
// epilogue reads-modifies-writes the fp32 matrix with fully coalesced dword
// accesses and refreshes its bf16 copy, staged through LDS so that it leaves as
// 16-byte stores.
// ---------------------------------------------------------------------------
__device__ __forceinline__ unsigned pack2_bf16(float lo, float hi) {
  const __bf16 a = (__bf16)lo, b = (__bf16)hi;
  return (unsigned)__builtin_bit_cast(unsigned short, a) | ((unsigned)__builtin_bit_cast(unsigned short, b) << 16);
}

template <int FM, int FN, int NS>
__global__ __launch_bounds__(256, (FM * FN <= 4 ? 2 : 1)) void update2_kernel(Update2Args g) {
  constexpr int TI = 64 * FM, TJ = 64 * FN;
  constexpr int PR = TI * 2 + 16;       // pitch of the staging tile [j][i], bytes
  extern __shared__ uint4 lds[];
  char *const lds_c = reinterpret_cast<char *>(lds);
  const int logical = logical_workgroup(g.tiles_i * g.tiles_j);
  if (logical < 0) return;
  const int ti = logical % g.tiles_i, tj = logical / g.tiles_i;
  const int i0 = ti * TI, j0 = tj * TJ;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wi = wave & 1, wj = wave >> 1, l32 = lane & 31, h = lane >> 5;

  // The fp32 tile this workgroup will read-modify-write is requested before the
  // main loop, so that its HBM latency is hidden behind the contraction.  Element
  // x of fragment (a, b) is (j = 8 (x / 4) + 4 h + x % 4, i = lane % 32): for one x
  // a half-wavefront touches 128 contiguous bytes of a row.
  float old[FM][FN][16];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b) {
      const int i = i0 + (wi * FM + a) * 32 + l32;
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int j = j0 + (wj * FN + b) * 32 + 8 * (x >> 2) + 4 * h + (x & 3);
        old[a][b][x] = (i < g.I && j < g.J) ? g.W[(long)j * g.ldw + i] : 0.f;
      }
    }

  floatx16 acc[FM][FN];
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
  mainloop<FM, FN, NS>(g.XT, g.ldx, g.DT, g.ldd, g.I, g.J, i0, j0, 0, g.K >> 6, lds_c, acc);

  __syncthreads();                       // every wavefront is done with the operand stages
#pragma unroll
  for (int a = 0; a < FM; ++a)
#pragma unroll
    for (int b = 0; b < FN; ++b) {
      const int il = (wi * FM + a) * 32 + l32;
      const int i = i0 + il;
      // 1. fp32 matrix: w = W~ + eta * acc, written back; entries outside the matrix become 0
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int j = j0 + (wj * FN + b) * 32 + 8 * (x >> 2) + 4 * h + (x & 3);
        const bool in = i < g.I && j < g.J;
        const float w = in ? fmaf(g.eta, acc[a][b][x], old[a][b][x]) : 0.f;
        if (in) g.W[(long)j * g.ldw + i] = w;
        acc[a][b][x] = w;
      }
      // 2. stage the bf16 value of w, row-major [j][i]
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int jl = (wj * FN + b) * 32 + 8 * (x >> 2) + 4 * h + (x & 3);
        const __bf16 v = (__bf16)acc[a][b][x];
        *reinterpret_cast<unsigned short *>(lds_c + jl * PR + il * 2) = __builtin_bit_cast(unsigned short, v);
      }
    }
  __syncthreads();
  // 3. the copy leaves as rows of 16-byte chunks (the pitch is a multiple of 64
  //    elements: whole chunks fit, and entries beyond the matrix are zeros)
  for (int id = tid; id < TJ * (TI / 8); id += 256) {
    const int row = id / (TI / 8), ci = id % (TI / 8);
    const int j = j0 + row, i = i0 + ci * 8;
    if (j < g.J && i < g.ldWb)
      *reinterpret_cast<uint4 *>(g.Wb + (long)j * g.ldWb + i) = *reinterpret_cast<const uint4 *>(lds_c + row * PR + ci * 16);
  }
}

// ---------------------------------------------------------------------------
// Coded update, persistent and wave-specialised (batch of at least 256).
//
// update2_kernel spends 40 us in its contraction and 54 us streaming the fp32
// matrix and its bf16 copy, one after the other.  Here a workgroup of 8
// wavefronts stays resident and walks over 128 x 128 tiles, with three roles
// that meet only at the per-slab workgroup barriers (every wavefront executes
// the same number of s_barrier: one per slab, one at the end of a tile):
//  * wavefronts 0-3 (MMA) run one flat slab pipeline across all tiles of the
//    workgroup (direct-to-LDS loads three stages deep, MFMAs); their vmcnt only
//    ever counts those loads.  At the end of a tile they add eta * acc to the
//    fp32 tile that waits in LDS, in place;
//  * wavefronts 4-5 (loaders) fetch the fp32 tile of the matrix from HBM into
//    registers a whole tile period ahead and drop it into LDS in four groups during
//    the last slabs of the tile, once the storers have released the buffer; no other
//    wavefront ever waits on HBM;
//  * wavefronts 6-7 (storers) work one tile behind: during the first slabs they gather
//    rows of the matrix from the LDS tile and store them and their bf16
//    copy; every store instruction writes whole 64-byte segments (the L2 request
//    rate, not its bandwidth, is what this kernel runs into).  They only ever issue
//    stores, so they never wait for memory.
// Which piece follows which barrier is described at the roles' code below.
// One counter covers a wavefront's loads and stores, and with a direct-to-LDS load
// outstanding the compiler waits for all of them wherever it places a wait of its own: a
// wavefront that fills LDS, loads the matrix and stores it would drain everything at every
// use of a loaded value, which is why the roles are split this way.  (A kernel in which eight
// identical wavefronts read and write the matrix straight from the accumulators of 256 x 128
// tiles, with hand-placed waits, ran no faster: 69 to 71 us.)  Tiles are dealt so that every XCD owns one rectangle of a
// 2 x 4 partition of the tile grid and needs only the operand panels of that rectangle.
// Streaming accesses stay ordinary cached ones: the matrix and its copy largely live in
// the 256 MB memory-side cache from one step to the next, and non-temporal stores forfeit
// that (150 us vs 84 us); non-temporal loads of the fp32 tile change nothing.  Write-through
// stores (sc1) keep the operand panels in L2 (operand traffic falls from 95 MB to 43 MB, close
// to the 31 MB that the partition makes compulsory) but are slower themselves: 100 us.
// Unlike in product_kernel, moving the roles apart by SIMD does not pay here (MMA wavefronts
// on SIMDs 0 and 1, loaders on 2, storers on 3: 86.5 us against 82.5 us): the MFMAs are the
// smaller part and the kernel runs at the rate the memory system takes the traffic.
// The roles' times mostly add up.  Measured while the kernel still wrote a second, transposed
// bf16 copy for the backward product: MMA role alone 42 us, the streaming roles alone 58 us,
// all 79 us; without the transposed copy 72, without the row-major copy 70, without the fp32
// stores 64, without the fp32 loads 67 us.  That is why the transposed copy went (the backward
// product now reads the row-major one through transposing LDS reads): 70 us in the step for
// 357 MB of traffic, 5.1 TB/s; a plain pass over the same matrix (shadow_kernel) reaches 5.8.
// ---------------------------------------------------------------------------
struct TileWalk {
  int tiles_i, tiles_j, tiw, tjh, total, i_base, j_base, step, q;
  bool reverse;
  // XCD x (workgroup id % 8) owns the rectangle of tiles (x / 4, x % 4) of a 2 x 4 partition and
  // walks it row by row: the tiw column panels of the rectangle (1.3 MB at 40 x 40 tiles) are in
  // use all the time and stay in that XCD's L2, the row panels pass through once.
  __device__ void init(int ti, int tj, bool rev = false) {
    reverse = rev;
    tiles_i = ti; tiles_j = tj;
    tiw = (ti + 3) >> 2;
    tjh = (tj + 1) >> 1;
    total = tiw * tjh;
    const int x = blockIdx.x & 7;
    i_base = (x & 3) * tiw;
    j_base = (x >> 2) * tjh;
    step = gridDim.x >> 3;
    q = (int)(blockIdx.x >> 3) - step;
  }
  // next valid tile of this workgroup; false when there is none
  __device__ bool next(int &ti, int &tj) {
    for (q += step; q < total; q += step) {
      const int qq = reverse ? total - 1 - q : q;
      ti = i_base + qq % tiw;
      tj = j_base + qq / tiw;
      if (ti < tiles_i && tj < tiles_j) return true;
    }
    return false;
  }
};

__global__ __launch_bounds__(512) void update3_kernel(Update2Args g) {
  constexpr int STAGE = 256 * 128;            // bytes: 128 A rows + 128 B rows of 128 bytes
  constexpr int TILE = 3 * STAGE;             // fp32 tile of the matrix, 64 KB: 160 KB in all
  extern __shared__ uint4 lds[];
  char *const lds_c = reinterpret_cast<char *>(lds);
  // The fp32 tile sits in LDS as the matrix does in memory, [j][i] with 512-byte rows: the
  // loaders and the storers move whole rows, and an MMA lane owns four consecutive i of one j
  // (the A-side fragment is the first MFMA operand here).  The 16-byte piece i / 4 of row j
  // sits at piece (i / 4) ^ (j % 32): the MMA lanes (32 consecutive j, one piece) spread over
  // all banks, a row's pieces stay a permutation of the row.
  auto cell = [&](int jl, int il) -> char * {
    return lds_c + TILE + jl * 512 + ((((il >> 2) ^ jl) & 31) << 4) + ((il & 3) << 2);
  };
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int KS = g.K >> 6;                    // slabs per tile (>= 4)

  TileWalk walk;
  walk.init(g.tiles_i, g.tiles_j, g.reverse != 0);
  int ti, tj;
  if (!walk.next(ti, tj)) return;             // uniform: nothing for this workgroup

  if (wave < 4) {
    // ---------------------------------------------------------------------- MMA
    const int wi = wave & 1, wj = wave >> 1;
    const int l32 = lane & 31, h = lane >> 5;
    const int lrow = lane >> 3, chunk = (lane & 7) ^ swizzle_of_row(8 * wave + lrow);
    unsigned offA[4], offB[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const unsigned slot = (unsigned)(((2 * s + h) ^ swizzle_of_row(l32)) * 16);
      offA[s] = (unsigned)((wi * 64 + l32) * 128) + slot;
      offB[s] = (unsigned)(128 * 128 + (wj * 64 + l32) * 128) + slot;
    }
    const __bf16 *src[8];                     // 4 A loads then 4 B loads of the slab being requested
    auto point_at = [&](int pti, int ptj) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int row = pti * 128 + 8 * (4 * u + wave) + lrow;
        row = row < g.I ? row : g.I - 1;
        src[u] = g.XT + (long)row * g.ldx + chunk * 8;
        row = ptj * 128 + 8 * (4 * u + wave) + lrow;
        row = row < g.J ? row : g.J - 1;
        src[4 + u] = g.DT + (long)row * g.ldd + chunk * 8;
      }
    };
    auto issue_one = [&](int kslab, int stage, int u) {
#if CN_DEVICE_ASM
      char *dst = lds_c + stage * STAGE + (u < 4 ? 0 : 128 * 128) + (4 * (u & 3) + wave) * 1024;
      __builtin_amdgcn_global_load_lds(src[u] + (long)kslab * 64, CN_LDS_PTR(dst), 16, 0, 0);
#else
      (void)kslab; (void)stage; (void)u;
#endif
    };
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    point_at(ti, tj);
#pragma unroll
    for (int u = 0; u < 8; ++u) issue_one(0, 0, u);
#pragma unroll
    for (int u = 0; u < 8; ++u) issue_one(1, 1, u);
    int nti = 0, ntj = 0;
    bool more = walk.next(nti, ntj);
    int stage = 0;                            // stage of the slab being consumed; the pipeline is flat across tiles
    for (;;) {
      for (int kt = 0; kt < KS; ++kt) {
        // the slab after this one was requested one round ago and may still be in flight
        if (kt + 1 < KS || more) wait_vm<8>();
        else wait_vm<0>();
        lds_barrier();
        // requested during this slab: two slabs ahead, in this tile or at the start of the next one
        const bool wraps = kt + 2 >= KS;
        const bool prefetch = !wraps || more;
        if (kt + 2 == KS && more) point_at(nti, ntj);
        const int pk = wraps ? kt + 2 - KS : kt + 2;
        const int pstage = stage == 0 ? 2 : stage - 1;
        const unsigned sb = (unsigned)(stage * STAGE);
        stage = stage == 2 ? 0 : stage + 1;
        u32x4 fa[2][2], fb[2][2];
        read_frags<2>(fa[0], sb + offA[0]);
        read_frags<2>(fb[0], sb + offB[0]);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const int cur = s & 1, nxt = cur ^ 1;
          if (s < 3) {
            read_frags<2>(fa[nxt], sb + offA[s + 1]);
            read_frags<2>(fb[nxt], sb + offB[s + 1]);
            wait_lgkm<4>();
          } else {
            wait_lgkm<0>();
          }
          pin(fa[cur][0]); pin(fa[cur][1]); pin(fb[cur][0]); pin(fb[cur][1]);
#pragma unroll
          for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
              const int m = a * 2 + b;
              if ((m & 1) == 0) {
                if (prefetch) issue_one(pk, pstage, s * 2 + (m >> 1));
                __builtin_amdgcn_sched_barrier(0);
              }
              acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[cur][a]),
                                                                  __builtin_bit_cast(bf16x8, fb[cur][b]), acc[a][b], 0, 0, 0);
            }
        }
      }
      // end of the tile: the loaders' fp32 tile is in; add eta * acc in place.  Elements
      // 4 q .. 4 q + 3 of fragment (a, b) are i = 8 q + 4 h .. + 3 of row j = lane % 32.
      lds_barrier();
      // all sixteen reads first: read, add, write one piece at a time is sixteen LDS round trips
      // in a row (the compiler keeps their order: it cannot tell that the pieces are distinct)
      f32x4 w[2][2][4];
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            w[a][b][q] = *reinterpret_cast<const f32x4 *>(cell((wj * 2 + b) * 32 + l32, (wi * 2 + a) * 32 + 8 * q + 4 * h));
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              w[a][b][q][e] += g.eta * acc[a][b][4 * q + e];
              acc[a][b][4 * q + e] = 0.f;
            }
            *reinterpret_cast<f32x4 *>(cell((wj * 2 + b) * 32 + l32, (wi * 2 + a) * 32 + 8 * q + 4 * h)) = w[a][b][q];
          }
      if (!more) break;
      ti = nti; tj = ntj;
      more = walk.next(nti, ntj);
    }
    // the storers finish the last tile after this one
    lds_barrier();
    return;
  }

  // Schedule of the other two roles inside a tile period (barriers B0 .. B(KS-1), then
  // the end-of-tile barrier).  With 8 slabs or more the storers empty the tile buffer in four
  // pieces after B0 .. B3, half a row quarter each (they read their rows from the
  // tile and push 24 KB of stores per piece; as whole quarters they took twice a
  // slab of the MMA role, which then waited 1900 clocks at each of the next barriers -- seen
  // in time stamps that one MMA wavefront took at every barrier), and the loaders refill it
  // with one group after each of B4 .. B7.  With fewer slabs the quarters follow B0 and B1
  // and the groups pair up after B2 and B3.
  const bool wide = KS >= 8;

  if (wave < 6) {
    // ------------------------------------------------------------------ loaders
    // Lane v holds, as item n, the values of row j = 4 n + v / 32, columns i = 4 (v % 32) .. + 3;
    // group q is items 8 q .. 8 q + 7.  As soon as a group is in LDS, the same registers
    // request that group of the next tile: the HBM latency has a whole tile period.
    const int v = tid - 256;
    f32x4 old[32];                            // native vectors: an array of HIP's float4 struct ends up in scratch here
    // item n goes to row 4 n + v / 32, piece (v % 32) ^ (row % 32) = ((v % 32) ^ (v / 32)) ^ (4 n % 32)
    char *const wbase = lds_c + TILE + (v >> 5) * 512;
    int wpiece = (((v & 31) ^ (v >> 5)) << 4);
    auto request_group = [&](int gq, int rti, int rtj) {
      if ((rti + 1) * 128 <= g.I && (rtj + 1) * 128 <= g.J) {
        // whole tile inside the matrix: one base address, uniform strides
        const float *src = g.W + (long)(rtj * 128 + (v >> 5)) * g.ldw + rti * 128 + (v & 31) * 4;
#pragma unroll
        for (int n8 = 0; n8 < 8; ++n8) {
          const int n = gq * 8 + n8;
          old[n] = *reinterpret_cast<const f32x4 *>(src + (long)(4 * n) * g.ldw);
        }
        return;
      }
      const int col = rti * 128 + (v & 31) * 4;
      const float *src = g.W + (col < g.I ? col : g.I - 4);
#pragma unroll
      for (int n8 = 0; n8 < 8; ++n8) {
        const int n = gq * 8 + n8;
        int row = rtj * 128 + 4 * n + (v >> 5);
        row = row < g.J ? row : g.J - 1;
        old[n] = *reinterpret_cast<const f32x4 *>(src + (long)row * g.ldw);
      }
    };
    auto write_group = [&](int gq) {
#if CN_DEVICE_ASM
      // recompute the addresses of a group here: hoisted out of the tile loop they cost 32 registers
      asm volatile("" : "+v"(wpiece));
#endif
#pragma unroll
      for (int n8 = 0; n8 < 8; ++n8) {
        const int n = gq * 8 + n8;
        *reinterpret_cast<f32x4 *>(wbase + 2048 * n + (wpiece ^ (((4 * n) & 31) << 4))) = old[n];
      }
    };
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) request_group(gq, ti, tj);
    bool have = true;
    while (have) {
      for (int e = wide ? 5 : 3; e > 0; --e) lds_barrier();
      have = walk.next(ti, tj);
      // Two copies of the sequence, with and without the requests for the next tile: with the
      // requests under a condition of their own, the compiler's count of the loads in flight
      // has to assume the smaller number at every join, and the last group then waits for
      // vmcnt(0), i.e. for the requests issued a moment ago (a full HBM latency at the
      // end-of-tile barrier, where the MMA wavefronts wait for this role).
      if (have) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          if (gq > 0 && (wide || gq == 2)) lds_barrier();
          write_group(gq);
          request_group(gq, ti, tj);
        }
      } else {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          if (gq > 0 && (wide || gq == 2)) lds_barrier();
          write_group(gq);
        }
      }
      for (int e = KS - (wide ? 8 : 4); e > 0; --e) lds_barrier();
      lds_barrier();                                      // end of the tile
    }
    lds_barrier();
    return;
  }

  // -------------------------------------------------------------------- storers
  const int v = tid - 384;                    // 0 .. 127
  int pti = 0, ptj = 0;                       // tile being stored (one behind the MMA role)
  // quarters 0, 1 (rows 0 .. 63 and 64 .. 127 of the tile): fp32 matrix and its bf16 copy;
  // item k is row j = 8 k + v / 16, columns i = 4 (v % 16) .. + 3 and 64 + 4 (v % 16) .. + 3: sixteen lanes
  // of one store instruction cover 256 contiguous bytes of a row (with eight adjacent columns per lane, as
  // two stores, each instruction wrote every other 16-byte piece and every 64-byte write request left the
  // L1 half full: 4.1 M write requests per launch for 2.46 M segments).
  // The two pieces are v % 16 and 16 + v % 16, at (piece ^ row % 32) = ((v % 16) ^ (v / 16)) ^ (8 k % 32) (^ 16)
  const char *const rbase = lds_c + TILE + (v >> 4) * 512;
  int rpiece = ((((v & 15)) ^ (v >> 4)) << 4);
  // qt: rows 64 qt .. 64 qt + 63 of the tile; hsel: -1 all of them, 0 / 1 one half (four of the eight row groups)
  auto quarter = [&](int qt, int hsel = -1) {
    // a tile that lies inside the matrix takes the branch-free path: all LDS reads of the
    // quarter first, then the stores; an edge tile masks every access
    const bool interior = (pti + 1) * 128 <= g.I && (ptj + 1) * 128 <= g.J;
    {
#if CN_DEVICE_ASM
      asm volatile("" : "+v"(rpiece));
#endif
      // byte offset of item k's first piece from rbase; the second piece is that offset ^ 256
      auto piece0 = [&](int k) -> int { return 4096 * k + (rpiece ^ (((8 * k) & 31) << 4)); };
      const int j0 = ptj * 128 + (v >> 4), i = pti * 128 + (v & 15) * 4;
      float *const pw = g.W + (long)j0 * g.ldw + i;
      __bf16 *const pb = g.Wb + (long)j0 * g.ldWb + i;
      if (interior) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          if (hsel >= 0 && half != hsel) continue;
          f32x4 c[4][2];
#pragma unroll
          for (int k4 = 0; k4 < 4; ++k4) {
            const int o = piece0(qt * 8 + half * 4 + k4);
            c[k4][0] = *reinterpret_cast<const f32x4 *>(rbase + o);
            c[k4][1] = *reinterpret_cast<const f32x4 *>(rbase + (o ^ 256));
          }
#pragma unroll
          for (int k4 = 0; k4 < 4; ++k4) {
            const int k = qt * 8 + half * 4 + k4;
            const f32x4 w0 = c[k4][0], w1 = c[k4][1];
            *reinterpret_cast<f32x4 *>(pw + (long)(8 * k) * g.ldw) = w0;
            *reinterpret_cast<f32x4 *>(pw + (long)(8 * k) * g.ldw + 64) = w1;
            *reinterpret_cast<u32x2 *>(pb + (long)(8 * k) * g.ldWb) = u32x2{pack2_bf16(w0[0], w0[1]), pack2_bf16(w0[2], w0[3])};
            *reinterpret_cast<u32x2 *>(pb + (long)(8 * k) * g.ldWb + 64) = u32x2{pack2_bf16(w1[0], w1[1]), pack2_bf16(w1[2], w1[3])};
          }
        }
        return;
      }
#pragma unroll 2
      for (int k8 = (hsel == 1 ? 4 : 0); k8 < (hsel == 0 ? 4 : 8); ++k8) {
        const int k = qt * 8 + k8;
        const int o = piece0(k);
        const f32x4 c0 = *reinterpret_cast<const f32x4 *>(rbase + o);
        const f32x4 c1 = *reinterpret_cast<const f32x4 *>(rbase + (o ^ 256));
        float4 w0 = make_float4(c0[0], c0[1], c0[2], c0[3]), w1 = make_float4(c1[0], c1[1], c1[2], c1[3]);
        const int j = j0 + 8 * k;
        const bool in0 = j < g.J && i < g.I, in1 = j < g.J && i + 64 < g.I;
        if (!in0) w0 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!in1) w1 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in0) *reinterpret_cast<float4 *>(pw + (long)(8 * k) * g.ldw) = w0;
        if (in1) *reinterpret_cast<float4 *>(pw + (long)(8 * k) * g.ldw + 64) = w1;
        if (j < g.J && i < g.ldWb)
          *reinterpret_cast<uint2 *>(pb + (long)(8 * k) * g.ldWb) = make_uint2(pack2_bf16(w0.x, w0.y), pack2_bf16(w0.z, w0.w));
        if (j < g.J && i + 64 < g.ldWb)
          *reinterpret_cast<uint2 *>(pb + (long)(8 * k) * g.ldWb + 64) = make_uint2(pack2_bf16(w1.x, w1.y), pack2_bf16(w1.z, w1.w));
      }
    }
  };
  bool have_prev = false, more = true;
  while (more) {
    if (wide) {
      // a whole quarter takes twice as long as a slab of the MMA role: half a quarter per barrier
      lds_barrier();
      if (have_prev) quarter(0, 0);
      lds_barrier();
      if (have_prev) quarter(0, 1);
      lds_barrier();
      if (have_prev) quarter(1, 0);
      lds_barrier();
      if (have_prev) quarter(1, 1);
      for (int e = KS - 4; e > 0; --e) lds_barrier();
    } else {
      lds_barrier();
      if (have_prev) quarter(0);
      lds_barrier();
      if (have_prev) quarter(1);
      for (int e = KS - 2; e > 0; --e) lds_barrier();
    }
    lds_barrier();                                        // end of the tile
    pti = ti; ptj = tj;
    have_prev = true;
    more = walk.next(ti, tj);
  }
  lds_barrier();
  quarter(0); quarter(1);
}

namespace {

template <int FM, int FN, int NS>
hipError_t launch_upd2(Update2Args g, hipStream_t s) {
  constexpr int TI = 64 * FM, TJ = 64 * FN;
  constexpr int stage = NS * (TI + TJ) * 128, st = TJ * (TI * 2 + 16);
  constexpr int lds = stage > st ? stage : st;
  static_assert(lds <= 160 * 1024, "the staging tile does not fit in LDS");
  g.tiles_i = (g.I + TI - 1) / TI;
  g.tiles_j = (g.J + TJ - 1) / TJ;
  const int nt = g.tiles_i * g.tiles_j;
  const int grid = ((nt + 7) / 8) * 8;
  static LdsOnce attr_done;
  hipError_t e = allow_lds(update2_kernel<FM, FN, NS>, lds, &attr_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((update2_kernel<FM, FN, NS>), dim3(grid), dim3(256), lds, s, g);
  return hipGetLastError();
}

hipError_t launch_upd3(Update2Args g, hipStream_t s) {
  constexpr int lds = 3 * 256 * 128 + 128 * 128 * 4;   // 160 KB
  g.tiles_i = (g.I + 127) / 128;
  g.tiles_j = (g.J + 127) / 128;
  static LdsOnce attr_done;
  hipError_t e = allow_lds(update3_kernel, lds, &attr_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(update3_kernel, dim3(256), dim3(512), lds, s, g);
  return hipGetLastError();
}

}  // namespace

// C = A B^T for bf16 operands (k contiguous and zero padded to a multiple of 64, or A stored
// k-major), fp32 result.
hipError_t launch_product(Gemm2Args g, hipStream_t s) {
  if ((g.K & 63) || (g.lda & 7) || (g.ldb & 7) || (g.ldc & 3) || (g.I & 3) || g.I < 1 || g.J < 1)
    return hipErrorInvalidValue;
  constexpr int lds = 5 * (96 + 128) * 128;
  static LdsOnce attr_done;
  static LdsOnce attr_t_done;
  hipError_t e = g.a_k_major ? allow_lds(product_kernel<true>, lds, &attr_t_done) : allow_lds(product_kernel<false>, lds, &attr_done);
  if (e != hipSuccess) return e;
  g.tiles_i = (g.I + 95) / 96;
  g.tiles_j = (g.J + 127) / 128;
  const int total = g.tiles_i * g.tiles_j;
  const dim3 grid((unsigned)(((total + 7) / 8) * 8));
  if (g.a_k_major) hipLaunchKernelGGL(product_kernel<true>, grid, dim3(512), lds, s, g);
  else hipLaunchKernelGGL(product_kernel<false>, grid, dim3(512), lds, s, g);
  return hipGetLastError();
}

// Whether launch_product_check takes a product: whole codewords of at most ten blocks in a tile, at
// most four parity blocks, one record per tile within the check's record buffer.
bool product_check_fits(int L, int Bp, int r, int J) {
  if (L < 1 || L > 10 || r < 1 || r > 4 || Bp < 1 || J < 1) return false;
  const long tiles = (long)((Bp + 15) / 16) * ((J + 63) / 64);
  return tiles <= kDetectParts;
}

// C = A B^T as launch_product (k contiguous in both operands only), on tiles of whole codewords,
// with the pass-1 records of the check and the syndromes left behind (*n_parts records).
hipError_t launch_product_check(Gemm2Args g, CheckArgs c, int *n_parts, hipStream_t s) {
  if ((g.K & 63) || (g.lda & 7) || (g.ldb & 7) || g.a_k_major || !product_check_fits(c.L, c.Bp, c.r, g.J) ||
      g.I != c.L * c.Bp)
    return hipErrorInvalidValue;
  constexpr int lds = 5 * (160 + 64) * 128;
  g.tiles_i = (c.Bp + 15) / 16;
  g.tiles_j = (g.J + 63) / 64;
  const int total = g.tiles_i * g.tiles_j;
  *n_parts = total;
  const dim3 grid((unsigned)(((total + 7) / 8) * 8));
#define CODENET_PC(RV)                                                                                 \
  {                                                                                                    \
    static LdsOnce once;                                                                               \
    hipError_t e = allow_lds(product_check_kernel<RV>, lds, &once);                                    \
    if (e != hipSuccess) return e;                                                                     \
    hipLaunchKernelGGL((product_check_kernel<RV>), grid, dim3(512), lds, s, g, c);                     \
    return hipGetLastError();                                                                          \
  }
  switch (c.r) { case 1: CODENET_PC(1) case 2: CODENET_PC(2) case 3: CODENET_PC(3) default: CODENET_PC(4) }
#undef CODENET_PC
}

hipError_t launch_reduce_partials(const float *part, long stride, int splits, float *out, long count, hipStream_t s) {
  if ((stride & 3) || (count & 3) || splits < 1) return hipErrorInvalidValue;
  const long count4 = count / 4;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<const float4 *>(part), stride / 4, splits, reinterpret_cast<float4 *>(out), count4);
  return hipGetLastError();
}

// The coded update: the persistent kernel for batches of 256 and more (its slab pipeline needs at
// least four slabs per tile), one tile per workgroup below.
hipError_t launch_update2(Update2Args g, hipStream_t s) {
  if ((g.K & 63) || (g.ldx & 7) || (g.ldd & 7) || (g.ldWb & 63) || g.I < 1 || g.J < 1)
    return hipErrorInvalidValue;
  if (g.K >= 256 && (g.I & 3) == 0 && (g.J & 3) == 0) return launch_upd3(g, s);
  return launch_upd2<4, 2, 2>(g, s);
}

// ---------------------------------------------------------------------------
// Shadow refresh: the bf16 copy of the fp32 coded matrix (row-major; the forward product
// reads it as it is, the backward product through transposing LDS reads).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void shadow_kernel(const float *__restrict__ Wt, int Mr, int Nc,
                                                     __bf16 *__restrict__ Wb, long ldWb) {
  // 64 x 64 tiles: thread t handles float4 (t & 15) of rows (t >> 4) + 16 p
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int t = threadIdx.x;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int r = r0 + (t >> 4) + 16 * p, c = c0 + (t & 15) * 4;
    if (r < Mr && c < Nc) {
      const float4 v = *reinterpret_cast<const float4 *>(Wt + (long)r * Nc + c);
      uint2 pk;
      pk.x = pack2_bf16(v.x, v.y);
      pk.y = pack2_bf16(v.z, v.w);
      *reinterpret_cast<uint2 *>(Wb + (long)r * ldWb + c) = pk;
    }
  }
}

hipError_t launch_shadow(const float *Wt, int Mr, int Nc, void *Wb, long ldWb, hipStream_t s) {
  dim3 grid((unsigned)((Nc + 63) / 64), (unsigned)((Mr + 63) / 64));
  hipLaunchKernelGGL(shadow_kernel, grid, dim3(256), 0, s, Wt, Mr, Nc, (__bf16 *)Wb, ldWb);
  return hipGetLastError();
}

}  // namespace codenet
