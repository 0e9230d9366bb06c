// Memory-bound and tiny kernels of the coded layer step: one-time encoding of W,
// additional encoding of the input vectors, syndrome / Gram reduction, the
// decision (locate) kernel, the correction + decode kernel, soft-error
// injection and weight export.
#include "codenet_internal.h"

namespace codenet {

// ---------------------------------------------------------------------------
// Pre-processing (Claim 1): W~ block (i, j) = sum_{i', j'} G_r[i'][i] G_c[j'][j] W_{i', j'}.
// One thread per coded element, float64 accumulation, one rounding to float32.
// G = [I | P] and H = [P^T | -I], so G[i'][a + k] = H[k][i'].
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_matrix_kernel(const float *__restrict__ W, float *__restrict__ Wt,
                                                            const DevCode *__restrict__ cr,
                                                            const DevCode *__restrict__ cc, int Mr, int Nc,
                                                            int n_out, int n_in) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)Mr * Nc) return;
  const int R = (int)(idx / Nc), C = (int)(idx % Nc);
  const int i = R / cr->B, rho = R % cr->B;
  const int j = C / cc->B, kap = C % cc->B;
  double acc = 0.0;
  if (rho < cr->B0 && kap < cc->B0) {
    const int i_lo = i < cr->a ? i : 0, i_hi = i < cr->a ? i + 1 : cr->a;
    const int j_lo = j < cc->a ? j : 0, j_hi = j < cc->a ? j + 1 : cc->a;
    for (int i2 = i_lo; i2 < i_hi; ++i2) {
      const int g = i2 * cr->B0 + rho;
      if (g >= n_out) continue;
      const double gr = i < cr->a ? 1.0 : cr->H[i - cr->a][i2];
      for (int j2 = j_lo; j2 < j_hi; ++j2) {
        const int hcol = j2 * cc->B0 + kap;
        if (hcol >= n_in) continue;
        const double gc = j < cc->a ? 1.0 : cc->H[j - cc->a][j2];
        acc += gr * gc * (double)W[(long)g * n_in + hcol];
      }
    }
  }
  Wt[idx] = (float)acc;
}

hipError_t launch_encode_matrix(const float *W, float *Wt, const DevCode *code_r, const DevCode *code_c,
                                int Mr, int Nc, int n_out, int n_in, hipStream_t s) {
  const long total = (long)Mr * Nc;
  const unsigned grid = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(encode_matrix_kernel, dim3(grid), dim3(256), 0, s, W, Wt, code_r, code_c, Mr, Nc,
                     n_out, n_in);
  return hipGetLastError();
}

// Systematic part without padding (inverse of the block padding above).
__global__ __launch_bounds__(256) void export_weights_kernel(const float *__restrict__ Wt, float *__restrict__ W,
                                                             int Br, int B0r, int Bc, int B0c, int Nc,
                                                             int n_out, int n_in) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)n_out * n_in) return;
  const int g = (int)(idx / n_in), hcol = (int)(idx % n_in);
  const int R = (g / B0r) * Br + g % B0r, C = (hcol / B0c) * Bc + hcol % B0c;
  W[idx] = Wt[(long)R * Nc + C];
}

hipError_t launch_export_weights(const float *Wt, float *W, const DevCode &cr, const DevCode &cc, int Nc,
                                 int n_out, int n_in, hipStream_t s) {
  const long total = (long)n_out * n_in;
  hipLaunchKernelGGL(export_weights_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, Wt, W,
                     cr.B, cr.B0, cc.B, cc.B0, Nc, n_out, n_in);
  return hipGetLastError();
}

// Block geometry by value: kernels that take it need no dependent load from the code table
// before they can form their first address.
struct Geometry { int B, B0, a, r, L, N; };
static inline Geometry geometry_of(const DevCode &c) { return Geometry{c.B, c.B0, c.a, c.r, c.L, c.N}; }

// ---------------------------------------------------------------------------
// Additional encoding step (step 4 of the feedforward and backpropagation
// stages): [v; v~] = (G^T (x) I) v for every batch row.  Input is the caller's
// dense [b][N]; output is the block-padded [b][(a + r) B] that the products and
// the update read.  One thread per (batch row, 4 positions inside a block).
// ---------------------------------------------------------------------------
template <bool ALIGNED>
__global__ __launch_bounds__(256) void encode_vector_kernel(const float *__restrict__ V, long ldv, float *__restrict__ Vt,
                                                            const DevCode *__restrict__ code, int b,
                                                            __bf16 *__restrict__ Vb, long ldVb,
                                                            float4 *__restrict__ zero, long zero_count4,
                                                            Geometry geo) {
  const int B = geo.B, B0 = geo.B0, a = geo.a, r = geo.r, N = geo.N;
  const int quads = B >> 2;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  const int job = blockIdx.y;            // 0 .. a-1: copy systematic block `job`; a: the r parity blocks
  if (zero != nullptr && job == 0)
    for (long z = idx; z < zero_count4; z += (long)gridDim.x * 256) zero[z] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (idx >= (long)b * quads) return;
  const int beta = (int)(idx / quads), rho = (int)(idx % quads) * 4;
  const float *src = V + (long)beta * ldv;
  float *dst = Vt + (long)beta * (a + r) * B;
  // Entries rho .. rho + 3 of block i.  Unconditional loads (the address moves to the start of the
  // row where the entry is padding, and the value is dropped): a guarded load would wait for its
  // data in a branch of its own.  ALIGNED: N and B0 multiples of 4, V 16-byte aligned -- whole
  // quads are real or padding.
  auto fetch = [&](int i, float (&v)[4]) {
    if constexpr (ALIGNED) {
      const int g = i * B0 + rho;
      const bool ok = g < N;
      const float4 q = *reinterpret_cast<const float4 *>(src + (ok ? g : 0));
      v[0] = ok ? q.x : 0.f; v[1] = ok ? q.y : 0.f; v[2] = ok ? q.z : 0.f; v[3] = ok ? q.w : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int g = i * B0 + rho + e;
        const bool ok = rho + e < B0 && g < N;
        const float q = src[ok ? g : 0];
        v[e] = ok ? q : 0.f;
      }
    }
  };
  if (job < a) {
    const int i = job;
    float v[4];
    fetch(i, v);
    *reinterpret_cast<float4 *>(dst + i * B + rho) = make_float4(v[0], v[1], v[2], v[3]);
    if (Vb != nullptr) {
      const __bf16 b0 = (__bf16)v[0], b1 = (__bf16)v[1], b2 = (__bf16)v[2], b3 = (__bf16)v[3];
      uint2 pk;
      pk.x = (unsigned)__builtin_bit_cast(unsigned short, b0) | ((unsigned)__builtin_bit_cast(unsigned short, b1) << 16);
      pk.y = (unsigned)__builtin_bit_cast(unsigned short, b2) | ((unsigned)__builtin_bit_cast(unsigned short, b3) << 16);
      *reinterpret_cast<uint2 *>(Vb + (long)beta * ldVb + i * B + rho) = pk;
    }
    return;
  }
  if (r == 0) return;
  // parity block k = sum_i H[k][i] block_i, i ascending, eight blocks' loads in flight at a time
  // (beyond the last block: block a - 1 again, with weight zero)
  float par[CODENET_MAX_R][4];
#pragma unroll
  for (int k = 0; k < CODENET_MAX_R; ++k) par[k][0] = par[k][1] = par[k][2] = par[k][3] = 0.f;
  for (int i0 = 0; i0 < a; i0 += 8) {
    float v[8][4];
#pragma unroll
    for (int u = 0; u < 8; ++u) fetch(i0 + u < a ? i0 + u : a - 1, v[u]);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool live = i0 + u < a;
      const int i = live ? i0 + u : a - 1;
#pragma unroll
      for (int k = 0; k < CODENET_MAX_R; ++k)
        if (k < r) {
          const float p = code->Hf[k][i];
#pragma unroll
          for (int e = 0; e < 4; ++e) par[k][e] = live ? fmaf(p, v[u][e], par[k][e]) : par[k][e];
        }
    }
  }
#pragma unroll
  for (int k = 0; k < CODENET_MAX_R; ++k)
    if (k < r)
      *reinterpret_cast<float4 *>(dst + (a + k) * B + rho) = make_float4(par[k][0], par[k][1], par[k][2], par[k][3]);
}


hipError_t launch_encode_vector(const float *V, long ldv, float *Vt, const DevCode *code_dev, const DevCode &code_host,
                                int b, void *Vb, long ldVb, float *zero, long zero_count4, hipStream_t s) {
  const long total = (long)b * (code_host.B >> 2);
  dim3 grid((unsigned)((total + 255) / 256), (unsigned)(code_host.a + 1));
  const int aligned = (code_host.N % 4 == 0) && (code_host.B0 % 4 == 0) && (ldv % 4 == 0) && ((reinterpret_cast<uintptr_t>(V) & 15) == 0);
  if (aligned)
    hipLaunchKernelGGL(encode_vector_kernel<true>, grid, dim3(256), 0, s, V, ldv, Vt, code_dev, b, (__bf16 *)Vb, ldVb,
                       reinterpret_cast<float4 *>(zero), zero_count4, geometry_of(code_host));
  else
    hipLaunchKernelGGL(encode_vector_kernel<false>, grid, dim3(256), 0, s, V, ldv, Vt, code_dev, b, (__bf16 *)Vb, ldVb,
                       reinterpret_cast<float4 *>(zero), zero_count4, geometry_of(code_host));
  return hipGetLastError();
}


// The same encoding for the bf16 mode, one 64 (batch) x TP (positions) tile of one
// output block per workgroup (TP = 32: 1280 workgroups at 4096 x 512 were measured at 6.8 us,
// 640 of 64 x 64 at 7.7, 2560 of 64 x 16 at 8.6).  It writes the two bf16 arrays that the MFMA kernels
// read (nothing in this mode reads an fp32 coded vector, so none is written): the
// batch-major systematic part (operand of the product) and, through an LDS
// transposition, the feature-major coded vector (operand of the update);
// batch columns b .. Rpad-1 of the latter are written as zeros.  Jobs 0 .. a-1 copy
// a systematic block, job a + k computes parity block k.
template <bool ALIGNED, int TP>
__global__ __launch_bounds__(256) void encode_vector_bf16_kernel(const float *__restrict__ V, long ldv,
                                                                 const DevCode *__restrict__ code, int b,
                                                                 __bf16 *__restrict__ Vb, long ldVb,
                                                                 __bf16 *__restrict__ VTb, long ldVT, int Rpad,
                                                                 Geometry geo) {
  constexpr int PER_ROW = TP / 4, ROWS = 256 / PER_ROW, P = 64 / ROWS;   // threads per batch row, rows per pass, passes
  static_assert(TP == 16 || TP == 32 || TP == 64, "tile width in positions");
  __shared__ unsigned short tile[64][TP + 2];
  const int B = geo.B, B0 = geo.B0, a = geo.a, r = geo.r, N = geo.N;
  // the parity jobs read all a blocks: they are dispatched first so that they do not form the tail
  const int rho0 = blockIdx.x * TP, beta0 = blockIdx.y * 64;
  const int job = (int)blockIdx.z < r ? a + (int)blockIdx.z : (int)blockIdx.z - r;
  const int t = threadIdx.x;
  const int c = (t % PER_ROW) * 4, rho = rho0 + c;
  // Four entries rho .. rho + 3 of block i of one batch row.  The loads are unconditional, from an
  // address moved into the array where the entry is padding or the row is beyond the batch, and the
  // value is dropped afterwards: a load under a condition would sit in a branch of its own and wait
  // for its data there, one memory latency per load instead of one per batch of loads.
  // ALIGNED: N and B0 multiples of 4, V 16-byte aligned -- whole quads are real or padding.
  auto fetch = [&](int beta, int i, float (&v)[4]) {
    const bool row_ok = beta < b && rho < B;
    const float *src = V + (long)(beta < b ? beta : b - 1) * ldv;
    if constexpr (ALIGNED) {
      const int g = i * B0 + rho;
      const bool ok = row_ok && rho < B0 && g < N;
      const float4 q = *reinterpret_cast<const float4 *>(src + (ok ? g : 0));
      v[0] = ok ? q.x : 0.f; v[1] = ok ? q.y : 0.f; v[2] = ok ? q.z : 0.f; v[3] = ok ? q.w : 0.f;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int g = i * B0 + rho + e;
        const bool ok = row_ok && rho + e < B0 && g < N;
        const float q = src[ok ? g : 0];
        v[e] = ok ? q : 0.f;
      }
    }
  };
  // this thread's four rows: rr = t / 16 + 16 p
  float v[P][4];
  if (job < a) {
#pragma unroll
    for (int p = 0; p < P; ++p) fetch(beta0 + t / PER_ROW + ROWS * p, job, v[p]);
  } else {
    // parity block k = sum_i H[k][i] block_i, i ascending; eight blocks x four rows of loads in flight
    // at a time (beyond the last block: block a - 1 again, with weight zero)
#pragma unroll
    for (int p = 0; p < P; ++p) v[p][0] = v[p][1] = v[p][2] = v[p][3] = 0.f;
    const int k = job - a;
    for (int i0 = 0; i0 < a; i0 += 8) {
      float x[8][P][4];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int p = 0; p < P; ++p) fetch(beta0 + t / PER_ROW + ROWS * p, i0 + u < a ? i0 + u : a - 1, x[u][p]);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool live = i0 + u < a;
        const float h = code->Hf[k][live ? i0 + u : a - 1];
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
          for (int e = 0; e < 4; ++e) v[p][e] = live ? fmaf(h, x[u][p][e], v[p][e]) : v[p][e];
      }
    }
  }
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int rr = t / PER_ROW + ROWS * p, beta = beta0 + rr;
    const __bf16 b0 = (__bf16)v[p][0], b1 = (__bf16)v[p][1], b2 = (__bf16)v[p][2], b3 = (__bf16)v[p][3];
    const unsigned short u0 = __builtin_bit_cast(unsigned short, b0), u1 = __builtin_bit_cast(unsigned short, b1),
                         u2 = __builtin_bit_cast(unsigned short, b2), u3 = __builtin_bit_cast(unsigned short, b3);
    tile[rr][c] = u0; tile[rr][c + 1] = u1; tile[rr][c + 2] = u2; tile[rr][c + 3] = u3;
    if (job < a && beta < b && rho < B) {
      uint2 pk;
      pk.x = (unsigned)u0 | ((unsigned)u1 << 16);
      pk.y = (unsigned)u2 | ((unsigned)u3 << 16);
      *reinterpret_cast<uint2 *>(Vb + (long)beta * ldVb + (long)job * B + rho) = pk;
    }
  }
  __syncthreads();
  // feature-major: thread t writes batch rows 4 (t % 16) .. + 3 of positions t / 16 + 16 p
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int cc = (t >> 4) + 16 * p, rr = (t & 15) * 4;
    if (rho0 + cc < B && beta0 + rr < Rpad) {
      uint2 pk;
      pk.x = (unsigned)tile[rr][cc] | ((unsigned)tile[rr + 1][cc] << 16);
      pk.y = (unsigned)tile[rr + 2][cc] | ((unsigned)tile[rr + 3][cc] << 16);
      *reinterpret_cast<uint2 *>(VTb + ((long)job * B + rho0 + cc) * ldVT + beta0 + rr) = pk;
    }
  }
}

hipError_t launch_encode_vector_bf16(const float *V, long ldv, const DevCode *code_dev, const DevCode &code_host,
                                     int b, void *Vb, long ldVb, void *VTb, long ldVT, hipStream_t s) {
  const int Rpad = (b + 63) & ~63;
  const int aligned = (code_host.N % 4 == 0) && (code_host.B0 % 4 == 0) && (ldv % 4 == 0) && ((reinterpret_cast<uintptr_t>(V) & 15) == 0);
  // 64 x 32 tiles (see the kernel's comment for the other widths measured)
  const dim3 grid((unsigned)((code_host.B + 31) / 32), (unsigned)(Rpad / 64), (unsigned)(code_host.a + code_host.r));
  if (aligned)
    hipLaunchKernelGGL((encode_vector_bf16_kernel<true, 32>), grid, dim3(256), 0, s, V, ldv, code_dev, b, (__bf16 *)Vb, ldVb,
                       (__bf16 *)VTb, ldVT, Rpad, geometry_of(code_host));
  else
    hipLaunchKernelGGL((encode_vector_bf16_kernel<false, 32>), grid, dim3(256), 0, s, V, ldv, code_dev, b, (__bf16 *)Vb, ldVb,
                       (__bf16 *)VTb, ldVT, Rpad, geometry_of(code_host));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Consistency check, pass 2: the decision (decoding algorithm of the
// appendix), one workgroup, float64.  With Gamma the Gram matrix of the
// syndromes, the least-squares residual of a support A is
//   ||out^||^2 - tr((H_A^T H_A)^-1 H_A^T Gamma H_A),
// so the search over supports touches only a few dozen scalars.
// ---------------------------------------------------------------------------
struct Support {
  int k;
  int idx[CODENET_MAX_T];
};

// k-subset number `rank` of {0..L-1} in lexicographic order
__device__ void unrank_support(long rank, int L, int k, int *idx) {
  int x = 0;
  for (int pos = 0; pos < k; ++pos) {
    for (;; ++x) {
      // subsets that keep x at this position: C(L - x - 1, k - pos - 1)
      long c = 1;
      const int nn = L - x - 1, kk = k - pos - 1;
      if (kk > nn) c = 0;
      else for (int q = 1; q <= kk; ++q) c = c * (nn - kk + q) / q;
      if (rank < c) break;
      rank -= c;
    }
    idx[pos] = x++;
  }
}

__device__ long n_choose_k(int n, int k) {
  if (k > n) return 0;
  long c = 1;
  for (int q = 1; q <= k; ++q) c = c * (n - k + q) / q;
  return c;
}

// Cholesky factor of M = H_A^T H_A (k x k, lower), returns false if not positive definite
__device__ bool support_factor(const double (*H)[CODENET_MAX_L], int r, const int *idx, int k,
                               double Lo[CODENET_MAX_T][CODENET_MAX_T]) {
  for (int p = 0; p < k; ++p)
    for (int q = 0; q <= p; ++q) {
      double m = 0.0;
      for (int c = 0; c < r; ++c) m += H[c][idx[p]] * H[c][idx[q]];
      for (int u = 0; u < q; ++u) m -= Lo[p][u] * Lo[q][u];
      if (p == q) {
        if (m <= 1e-300) return false;
        Lo[p][p] = sqrt(m);
      } else {
        Lo[p][q] = m / Lo[q][q];
      }
    }
  return true;
}

__device__ double support_residual2(const double (*H)[CODENET_MAX_L], int r, const double (*G)[CODENET_MAX_R],
                                    double trG, const int *idx, int k) {
  double Lo[CODENET_MAX_T][CODENET_MAX_T];
  if (!support_factor(H, r, idx, k, Lo)) return trG;
  // N = H_A^T Gamma H_A
  double T[CODENET_MAX_R][CODENET_MAX_T];
  for (int c = 0; c < r; ++c)
    for (int p = 0; p < k; ++p) {
      double v = 0.0;
      for (int d = 0; d < r; ++d) v += G[c][d] * H[d][idx[p]];
      T[c][p] = v;
    }
  double N[CODENET_MAX_T][CODENET_MAX_T];
  for (int p = 0; p < k; ++p)
    for (int q = 0; q < k; ++q) {
      double v = 0.0;
      for (int c = 0; c < r; ++c) v += H[c][idx[p]] * T[c][q];
      N[p][q] = v;
    }
  // tr(M^-1 N) = tr(Lo^-1 N Lo^-T): forward-substitute rows, then columns
  double Y[CODENET_MAX_T][CODENET_MAX_T];
  for (int q = 0; q < k; ++q)
    for (int p = 0; p < k; ++p) {
      double v = N[p][q];
      for (int u = 0; u < p; ++u) v -= Lo[p][u] * Y[u][q];
      Y[p][q] = v / Lo[p][p];
    }
  double tr = 0.0;
  for (int p = 0; p < k; ++p) {
    // (Y Lo^-T)[p][p]: solve z Lo^T = Y[p][:] up to column p
    double z[CODENET_MAX_T];
    for (int q = 0; q <= p; ++q) {
      double v = Y[p][q];
      for (int u = 0; u < q; ++u) v -= z[u] * Lo[q][u];
      z[q] = v / Lo[q][q];
    }
    tr += z[p];
  }
  const double res = trG - tr;
  return res > 0.0 ? res : 0.0;
}

// Executed by all 256 threads of one workgroup.  GENERIC = supports of two or more
// blocks may be needed (r >= 4); without it the kernel needs no private scratch.
// Always inlined: with several kernels using it the compiler would otherwise emit a call,
// which costs the finishing kernel about 2 us.
template <bool GENERIC>
__device__ __forceinline__ void decide_body(const double *partials, int n_parts, const DevCode *__restrict__ code,
                            DevPlan *__restrict__ plan, codenet_report *__restrict__ report) {
  __shared__ double tot[kMaxEntries];
  __shared__ double G[CODENET_MAX_R][CODENET_MAX_R];
  __shared__ double best_res[4];
  __shared__ long best_rank[4];
  __shared__ int s_verdict, s_k;
  __shared__ long s_rank;
  __shared__ double s_resid, s_trG;
  const int t = threadIdx.x;
  const int L = code->L, r = code->r;
  const int tcap = r / 2 < CODENET_MAX_T ? r / 2 : CODENET_MAX_T;
  // the parity-check matrix is read many times by single threads below: keep it in LDS
  __shared__ double H[CODENET_MAX_R][CODENET_MAX_L];
  for (int idx = t; idx < CODENET_MAX_R * CODENET_MAX_L; idx += 256)
    H[idx / CODENET_MAX_L][idx % CODENET_MAX_L] = code->H[idx / CODENET_MAX_L][idx % CODENET_MAX_L];
  const double tau_detect = code->tau_detect, tau_resid = code->tau_resid;

  // Totals of the per-workgroup records (stored entry-major), live entries only, 16 entries at
  // a time: thread t adds records t and t + 256 of each (independent loads), then a 16 x 16
  // tree through LDS per entry -- the same arithmetic on every run and in every workgroup.
  __shared__ double red[16][256];
  __shared__ double red2[16][16];
  const int n_live = L + r * (r + 1) / 2;
  if (t < kMaxEntries) tot[t] = 0.0;
  for (int c0 = 0; c0 < n_live; c0 += 16) {
    double v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int k = c0 + u;
      const int e = k < L ? k : CODENET_MAX_L + (k - L);
      double a = 0.0, b2 = 0.0;
      if (k < n_live && t < n_parts) a = partials[(long)e * kDetectParts + t];
      if (k < n_live && t + 256 < n_parts) b2 = partials[(long)e * kDetectParts + t + 256];
      v[u] = a + b2;
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) red[u][t] = v[u];
    __syncthreads();
    {
      const int u = t >> 4, part = t & 15;
      double acc = 0.0;
#pragma unroll
      for (int q = 0; q < 16; ++q) acc += red[u][part + 16 * q];
      red2[u][part] = acc;
    }
    __syncthreads();
    if (t < 16 && c0 + t < n_live) {
      double acc = 0.0;
#pragma unroll
      for (int q = 0; q < 16; ++q) acc += red2[t][q];
      const int k = c0 + t;
      tot[k < L ? k : CODENET_MAX_L + (k - L)] = acc;
    }
    __syncthreads();
  }
  if (t == 0) {
    int e = CODENET_MAX_L;
    double trG = 0.0;
    for (int k = 0; k < r; ++k)
      for (int k2 = k; k2 < r; ++k2, ++e) G[k][k2] = G[k2][k] = tot[e];
    bool clean = true;
    for (int k = 0; k < r; ++k) {
      trG += G[k][k];
      double ref2 = 0.0;
      for (int i = 0; i < L; ++i) ref2 += H[k][i] * H[k][i] * tot[i];
      const double rel = ref2 > 0.0 ? sqrt(G[k][k] / ref2) : 0.0;
      if (report) report->syn_rel[k] = (float)rel;
      // a non-finite ratio (NaN / Inf in the output) must not pass as clean
      if (!(rel <= tau_detect)) clean = false;
    }
    if (report)
      for (int k = r; k < CODENET_MAX_R; ++k) report->syn_rel[k] = 0.f;
    s_trG = trG;
    s_verdict = clean ? CODENET_CLEAN : CODENET_UNCORRECTABLE;
    s_k = 0;
    s_rank = -1;
    s_resid = 0.0;
  }
  __syncthreads();

  if (s_verdict != CODENET_CLEAN && isfinite(s_trG) && s_trG > 0.0) {
    for (int k = 1; k <= tcap; ++k) {
      const long count = n_choose_k(L, k);
      double my_res = 1e300;
      long my_rank = -1;
      for (long rank = t; rank < count; rank += 256) {
        double res2;
        if (k == 1) {
          // one block i: residual^2 = tr(Gamma) - (h^T Gamma h) / (h^T h), h = H[:, i]
          double hh = 0.0, hgh = 0.0;
          for (int c = 0; c < r; ++c) {
            const double hc = H[c][rank];
            hh += hc * hc;
            double gh = 0.0;
            for (int d = 0; d < r; ++d) gh += G[c][d] * H[d][rank];
            hgh += hc * gh;
          }
          res2 = hh > 0.0 ? s_trG - hgh / hh : s_trG;
          if (res2 < 0.0) res2 = 0.0;
        } else if constexpr (GENERIC) {
          int idx[CODENET_MAX_T];
          unrank_support(rank, L, k, idx);
          res2 = support_residual2(H, r, G, s_trG, idx, k);
        } else {
          res2 = s_trG;
        }
        if (res2 < my_res) { my_res = res2; my_rank = rank; }
      }
      // smallest (residual, rank) pair: shuffle tree inside a wavefront, then the four leaders
      // (an LDS tree as for the sums was no faster here)
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        const double o_res = __shfl_down(my_res, off, 64);
        const long o_rank = __shfl_down(my_rank, off, 64);
        if (o_rank >= 0 && (my_rank < 0 || o_res < my_res || (o_res == my_res && o_rank < my_rank))) {
          my_res = o_res;
          my_rank = o_rank;
        }
      }
      if ((t & 63) == 0) {
        best_res[t >> 6] = my_res;
        best_rank[t >> 6] = my_rank;
      }
      __syncthreads();
      if (t == 0) {
        double br = 1e300;
        long bk = -1;
        for (int u = 0; u < 4; ++u)
          if (best_rank[u] >= 0 && (bk < 0 || best_res[u] < br || (best_res[u] == br && best_rank[u] < bk))) {
            br = best_res[u];
            bk = best_rank[u];
          }
        const double rel = bk >= 0 ? sqrt(br / s_trG) : 1e300;
        s_resid = rel;
        if (bk >= 0 && rel <= tau_resid) {
          s_verdict = CODENET_CORRECTED;
          s_k = k;
          s_rank = bk;
        }
      }
      __syncthreads();
      if (s_verdict == CODENET_CORRECTED) break;
    }
  }

  if (t == 0) {
    int idx[CODENET_MAX_T];
    for (int p = 0; p < CODENET_MAX_T; ++p) idx[p] = -1;
    const int k = s_verdict == CODENET_CORRECTED ? s_k : 0;
    if (k == 1) {
      idx[0] = (int)s_rank;
      double hh = 0.0;
      for (int c = 0; c < r; ++c) hh += H[c][idx[0]] * H[c][idx[0]];
      for (int c = 0; c < r; ++c) plan->coef[0][c] = (float)(H[c][idx[0]] / hh);
    } else if (GENERIC && k > 1) {
      unrank_support(s_rank, L, k, idx);
      // error block p = sum_c pinv[p][c] syndrome_c with pinv = (H_A^T H_A)^-1 H_A^T
      double Lo[CODENET_MAX_T][CODENET_MAX_T];
      support_factor(H, r, idx, k, Lo);
      for (int c = 0; c < r; ++c) {
        double y[CODENET_MAX_T], x[CODENET_MAX_T];
        for (int p = 0; p < k; ++p) {
          double v = H[c][idx[p]];
          for (int u = 0; u < p; ++u) v -= Lo[p][u] * y[u];
          y[p] = v / Lo[p][p];
        }
        for (int p = k - 1; p >= 0; --p) {
          double v = y[p];
          for (int u = p + 1; u < k; ++u) v -= Lo[u][p] * x[u];
          x[p] = v / Lo[p][p];
        }
        for (int p = 0; p < k; ++p) plan->coef[p][c] = (float)x[p];
      }
    }
    plan->verdict = s_verdict;
    plan->n_located = k;
    for (int p = 0; p < CODENET_MAX_T; ++p) plan->located[p] = idx[p];
    if (report) {
      report->verdict = s_verdict;
      report->n_located = k;
      for (int p = 0; p < CODENET_MAX_T; ++p) report->located[p] = idx[p];
      report->resid_rel = (float)(s_resid < 3e38 ? s_resid : 3e38);
    }
  }
}

// ---------------------------------------------------------------------------
// Consistency check, pass 1 (General Error-Detection Method): syndromes
// out^_k = sum_i H[k][i] out_i for every position of a block, written out for
// the correction pass, plus what the decision needs: ||out_i||^2 for every
// block and the r x r Gram matrix sum_pos out^(pos) out^(pos)^T.  HBM-bound:
// the coded output is read once.  (Letting the last workgroup to finish take the
// decision in the same kernel was tried: the device-scope fence it needs writes
// back the L2 of every XCD and cost 25 us; a second tiny kernel costs 3-10 us.)
// Per-thread float32 sums over a few positions, then float64 across lanes,
// wavefronts and workgroups in a fixed order (no atomics), so the decision is
// reproducible -- and two evaluations of it are bit-identical, which the verified
// check relies on.
// ---------------------------------------------------------------------------
template <int R, int CH>
__global__ __launch_bounds__(256) void detect_kernel(const float *__restrict__ out, float *__restrict__ syn,
                                                     double *__restrict__ partials,
                                                     const DevCode *__restrict__ code, int b, int iters,
                                                     int shift, Geometry geo) {
  // A second, independent evaluation of the same checks (verification step 1) runs with
  // shift > 0: workgroup w does the work and fills the record of workgroup w + shift, so that
  // every record is computed on another compute unit, in the same order of operations.
  unsigned wg = blockIdx.x + (unsigned)shift;
  if (wg >= gridDim.x) wg -= gridDim.x;
  const int B = geo.B, L = geo.L;
  const int quads = B >> 2;
  const long npos = (long)b * quads;
  constexpr int NG = R * (R + 1) / 2;
  float sq[CODENET_MAX_L];
  float gram[NG];
#pragma unroll
  for (int i = 0; i < CODENET_MAX_L; ++i) sq[i] = 0.f;
#pragma unroll
  for (int e = 0; e < NG; ++e) gram[e] = 0.f;

  for (int it = 0; it < iters; ++it) {
    const long idx = ((long)it * gridDim.x + wg) * 256 + threadIdx.x;
    if (idx >= npos) break;
    const int beta = (int)(idx / quads), rho = (int)(idx % quads) * 4;
    const float *row = out + (long)beta * L * B + rho;
    float4 sy[R];
#pragma unroll
    for (int k = 0; k < R; ++k) sy[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    // CH blocks at a time, all their loads issued before the first is used.  A load guarded
    // by "i < L" would sit in a branch of its own and wait for its data there (one memory
    // latency per block); instead every load is unconditional, from a clamped block index,
    // and a block beyond the code contributes through a zero weight (H is zero there).
#pragma unroll
    for (int i0 = 0; i0 < CODENET_MAX_L; i0 += CH) {
      if (i0 >= L) break;
      float4 v[CH];
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const int i = i0 + u < L ? i0 + u : L - 1;
        v[u] = *reinterpret_cast<const float4 *>(row + i * B);
      }
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        constexpr int last = CODENET_MAX_L - 1;
        const int i = i0 + u < last ? i0 + u : last;   // compile-time after unrolling
        const bool live = i0 + u < L;
        const float4 x = v[u];
        sq[i] += live ? x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w : 0.f;
#pragma unroll
        for (int k = 0; k < R; ++k) {
          const float hk = code->Hf[k][i];            // zero for i >= L
          sy[k].x = fmaf(hk, x.x, sy[k].x);
          sy[k].y = fmaf(hk, x.y, sy[k].y);
          sy[k].z = fmaf(hk, x.z, sy[k].z);
          sy[k].w = fmaf(hk, x.w, sy[k].w);
        }
      }
    }
    int e = 0;
#pragma unroll
    for (int k = 0; k < R; ++k) {
      if (syn) *reinterpret_cast<float4 *>(syn + ((long)k * b + beta) * B + rho) = sy[k];
#pragma unroll
      for (int k2 = k; k2 < R; ++k2, ++e)
        gram[e] += sy[k].x * sy[k2].x + sy[k].y * sy[k2].y + sy[k].z * sy[k2].z + sy[k].w * sy[k2].w;
    }
  }

  // Reduce over the 256 threads, 16 entries at a time, through LDS: a 16 x 16 tree per entry
  // (each thread adds 16 values a fixed stride apart, then 16 threads add the 16 partial sums).
  // Float64, fixed order.  (Shuffle trees of doubles cost about 2 us here: two ds_bpermute
  // and their address arithmetic per step, 6 steps, 13 entries.)  Live entries are numbered
  // Gram first (their count is a compile-time constant), then the L block norms.
  __shared__ double red[16][256];
  __shared__ double red2[16][16];
  const int t = threadIdx.x;
  const int n_live = NG + L;
#pragma unroll
  for (int c0 = 0; c0 < NG + CODENET_MAX_L; c0 += 16) {
    if (c0 >= n_live) break;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int k = c0 + u;
      float v = 0.f;
      if (k < NG) v = gram[k < NG ? k : 0];
      else if (k - NG < CODENET_MAX_L && k - NG < L) v = sq[k - NG < CODENET_MAX_L ? k - NG : 0];
      red[u][t] = (double)v;
    }
    __syncthreads();
    {
      const int u = t >> 4, part = t & 15;
      double acc = 0.0;
#pragma unroll
      for (int q = 0; q < 16; ++q) acc += red[u][part + 16 * q];
      red2[u][part] = acc;
    }
    __syncthreads();
    if (t < 16 && c0 + t < n_live) {
      double acc = 0.0;
#pragma unroll
      for (int q = 0; q < 16; ++q) acc += red2[t][q];
      const int k = c0 + t;
      const int e = k < NG ? CODENET_MAX_L + k : k - NG;
      partials[(long)e * kDetectParts + wg] = acc;
    }
    __syncthreads();
  }
}

hipError_t launch_detect(const float *out, float *syn, double *partials, int *n_parts, const DevCode *code_dev,
                         const DevCode &ch, int b, bool second_evaluation, hipStream_t s) {
  const long npos = (long)b * (ch.B >> 2);
  long wgs = (npos + 255) / 256;
  int iters = 1;
  if (wgs > kDetectParts) {
    iters = (int)((wgs + kDetectParts - 1) / kDetectParts);
    wgs = (npos + 256L * iters - 1) / (256L * iters);
  }
  *n_parts = (int)wgs;
  // an odd shift near half the grid: another compute unit in another XCD
  const int shift = second_evaluation && wgs > 1 ? (int)(((wgs / 2) | 1) % wgs) : 0;
  dim3 grid((unsigned)wgs), block(256);
  // blocks loaded at a time: the whole codeword when it has at most 16 blocks
  const bool wide = ch.L > 8 && ch.L <= 16;
  switch (ch.r) {
#define CODENET_DETECT_CASE(RR)                                                                                     \
  case RR:                                                                                                          \
    if (wide)                                                                                                       \
      hipLaunchKernelGGL((detect_kernel<RR, 16>), grid, block, 0, s, out, syn, partials, code_dev, b, iters, shift,  \
                         geometry_of(ch));                                                                          \
    else                                                                                                            \
      hipLaunchKernelGGL((detect_kernel<RR, 8>), grid, block, 0, s, out, syn, partials, code_dev, b, iters, shift,   \
                         geometry_of(ch));                                                                          \
    break;
    CODENET_DETECT_CASE(1) CODENET_DETECT_CASE(2) CODENET_DETECT_CASE(3) CODENET_DETECT_CASE(4)
    CODENET_DETECT_CASE(5) CODENET_DETECT_CASE(6) CODENET_DETECT_CASE(7) CODENET_DETECT_CASE(8)
#undef CODENET_DETECT_CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Consistency check, passes 2 + 3 in one kernel: every workgroup first takes the
// decision from the pass-1 records (the same deterministic arithmetic in each of
// them -- cheaper than a single-workgroup kernel in between, whose chain of
// dependent loads cost 8-10 us), then subtracts the reconstructed error blocks on
// the accepted support and emits the decoded (systematic, unpadded) output.
// Workgroup 0 writes the report.
// ---------------------------------------------------------------------------
// With VERIFY the two verification steps of Error Model 2 ride along.  Step 1: the pass-1
// records of a second evaluation of the checks are compared, bit for bit, with the ones the
// decision was taken from (every workgroup compares all of them); a difference makes the
// verdict DISAGREE and nothing is corrected.  Step 2: every workgroup is one evaluator of the
// decision and leaves its verdict and list of erroneous nodes as one word in votes[]; a
// single-workgroup kernel (verify_kernel) compares the words afterwards.
template <bool GENERIC, bool VERIFY>
__global__ __launch_bounds__(256) void finish_kernel(float *__restrict__ out, const float *__restrict__ syn,
                                                     const double *__restrict__ partials, int n_parts,
                                                     const DevCode *__restrict__ code, int b,
                                                     float *__restrict__ decoded, int aligned, int in_place,
                                                     codenet_report *__restrict__ report, int epi,
                                                     const float *__restrict__ aux, VerifyArgs ver, Geometry geo) {
  __shared__ DevPlan plan;
  decide_body<GENERIC>(partials, n_parts, code, &plan, blockIdx.x == 0 ? report : nullptr);
  __syncthreads();
  const int B = geo.B, B0 = geo.B0, L = geo.L, a = geo.a, r = geo.r, N = geo.N;
  if constexpr (VERIFY) {
    // eight live entries at a time, this thread's two records of each from both evaluations: 32
    // unconditional loads in flight (indices beyond the end are clamped: those records are compared
    // again, which changes nothing)
    const int n_live = L + r * (r + 1) / 2;
    static_assert(kDetectParts <= 512, "a thread compares records t and t + 256");
    int differ = 0;
    for (int k0 = 0; k0 < n_live; k0 += 8) {
      long long xa[8][2], xb[8][2];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int k = k0 + u < n_live ? k0 + u : n_live - 1;
        const long e = k < L ? k : CODENET_MAX_L + (k - L);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int q = (int)threadIdx.x + 256 * h;
          const long at = e * kDetectParts + (q < n_parts ? q : 0);
          xa[u][h] = __double_as_longlong(partials[at]);
          xb[u][h] = __double_as_longlong(ver.partials_b[at]);
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) differ |= (xa[u][0] != xb[u][0]) | (xa[u][1] != xb[u][1]);
    }
    differ = __syncthreads_or(differ);
    if (threadIdx.x == 0) {
      if (differ) {
        plan.verdict = CODENET_DISAGREE;
        plan.n_located = 0;
        for (int p = 0; p < CODENET_MAX_T; ++p) plan.located[p] = -1;
        if (blockIdx.x == 0 && report) {
          report->verdict = CODENET_DISAGREE;
          report->n_located = 0;
          for (int p = 0; p < CODENET_MAX_T; ++p) report->located[p] = -1;
        }
      } else if ((int)blockIdx.x == ver.faulty_evaluator) {
        // planted error in this evaluator's decision (tests of step 2)
        if (plan.verdict == CODENET_CORRECTED) plan.located[0] = (plan.located[0] + 1) % L;
        else plan.verdict = plan.verdict == CODENET_CLEAN ? CODENET_UNCORRECTABLE : CODENET_CLEAN;
      }
      unsigned long long word = (unsigned long long)plan.verdict | ((unsigned long long)plan.n_located << 8);
      for (int p = 0; p < CODENET_MAX_T; ++p)
        word |= (unsigned long long)((plan.located[p] + 1) & 0xff) << (16 + 8 * p);
      ver.votes[blockIdx.x] = word;
    }
    __syncthreads();
  }
  const int corrected = plan.verdict == CODENET_CORRECTED ? plan.n_located : 0;
  // in_place: the caller reads the systematic part where it is (decoded is null then); only an
  // elementwise step still has work to do on a clean output
  const bool act_in_place = in_place && epi != CODENET_EPI_NONE;
  if (corrected == 0 && decoded == nullptr && !act_in_place) return;
  const int quads = B >> 2;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)b * quads) return;
  const int beta = (int)(idx / quads), rho = (int)(idx % quads) * 4;
  float *row = out + (long)beta * L * B + rho;

  for (int p = 0; p < corrected; ++p) {
    // the located block and the r syndromes of this position: loads issued together
    const int i = plan.located[p];
    float4 v = *reinterpret_cast<float4 *>(row + i * B);
    float4 e = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int c = 0; c < r; ++c) {
      const float4 s = *reinterpret_cast<const float4 *>(syn + ((long)c * b + beta) * B + rho);
      const float w = plan.coef[p][c];
      e.x = fmaf(w, s.x, e.x); e.y = fmaf(w, s.y, e.y); e.z = fmaf(w, s.z, e.z); e.w = fmaf(w, s.w, e.w);
    }
    v.x -= e.x; v.y -= e.y; v.z -= e.z; v.w -= e.w;
    *reinterpret_cast<float4 *>(row + i * B) = v;
  }
  if (decoded == nullptr && !act_in_place) return;
  float *dst = decoded ? decoded + (long)beta * N : nullptr;
  const float *ax = aux ? aux + (long)beta * N : nullptr;
  // the elementwise primary step that follows the product, applied to the decoded copy only:
  // activation f = ReLU (feedforward), or the diagonal post-multiplication by g(x) (backpropagation)
  auto act = [&](float v, int g) -> float {
    if (epi == CODENET_EPI_RELU) return v > 0.f ? v : 0.f;
    if (epi == CODENET_EPI_MASK_POS) return ax[g] > 0.f ? v : 0.f;
    if (epi == CODENET_EPI_MUL) return v * ax[g];
    return v;
  };
  if (act_in_place) {
    // the elementwise step on the real entries of the systematic blocks, where they are
    for (int i = 0; i < a; ++i) {
      float4 v = *reinterpret_cast<const float4 *>(row + i * B);
      float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int g = i * B0 + rho + e;
        if (rho + e < B0 && g < N) vv[e] = act(vv[e], g);
      }
      *reinterpret_cast<float4 *>(row + i * B) = make_float4(vv[0], vv[1], vv[2], vv[3]);
    }
    return;
  }
  // eight blocks at a time: all loads first, then the stores (one block at a time would
  // expose a load latency per block)
  for (int i0 = 0; i0 < a; i0 += 8) {
    float4 blk[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (i0 + u < a) blk[u] = *reinterpret_cast<const float4 *>(row + (i0 + u) * B);   // own writes above are visible to this thread
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = i0 + u;
      if (i >= a) break;
      const float4 v = blk[u];
      if (aligned && epi == CODENET_EPI_NONE) {
        const int g = i * B0 + rho;
        if (g < N) *reinterpret_cast<float4 *>(dst + g) = v;
        continue;
      }
      const float vv[4] = {v.x, v.y, v.z, v.w};
      if (aligned) {
        const int g = i * B0 + rho;
        if (g < N)
          *reinterpret_cast<float4 *>(dst + g) = make_float4(act(vv[0], g), act(vv[1], g + 1), act(vv[2], g + 2), act(vv[3], g + 3));
        continue;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int g = i * B0 + rho + e;
        if (rho + e < B0 && g < N) dst[g] = act(vv[e], g);
      }
    }
  }
}

// Verification step 2: do all evaluators' words agree?  One workgroup; the report's verdict
// becomes DISAGREE if not.
__global__ __launch_bounds__(256) void verify_kernel(const unsigned long long *__restrict__ votes, int n,
                                                     codenet_report *__restrict__ report) {
  const unsigned long long first = votes[0];
  int differ = 0;
  // four words per thread and trip, loaded together (beyond the end: the last word again)
  for (int q0 = 0; q0 < n; q0 += 1024) {
    unsigned long long w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = q0 + 256 * u + (int)threadIdx.x;
      w[u] = votes[q < n ? q : n - 1];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) differ |= w[u] != first;
  }
  differ = __syncthreads_or(differ);
  if (differ && threadIdx.x == 0) {
    report->verdict = CODENET_DISAGREE;
    report->n_located = 0;
    for (int p = 0; p < CODENET_MAX_T; ++p) report->located[p] = -1;
  }
}

// Planted error in one evaluation of the checks (tests of verification step 1): one pass-1
// record of the first check's squared norm becomes (1 + scale) * record + scale.
__global__ void record_fault_kernel(double *record, double scale) { *record = (1.0 + scale) * *record + scale; }

hipError_t launch_record_fault(double *partials, int part, double scale, hipStream_t s) {
  hipLaunchKernelGGL(record_fault_kernel, dim3(1), dim3(1), 0, s, partials + (long)CODENET_MAX_L * kDetectParts + part,
                     scale);
  return hipGetLastError();
}

// workgroups of the finishing kernel; a verified check has at least two (two evaluators of the
// decision even when one workgroup covers the whole output)
long finish_workgroups(const DevCode &ch, int b, bool verified) {
  const long wgs = ((long)b * (ch.B >> 2) + 255) / 256;
  return verified && wgs < 2 ? 2 : wgs;
}

hipError_t launch_finish(float *out, const float *syn, const double *partials, int n_parts, const DevCode *code_dev,
                         const DevCode &ch, int b, float *decoded, codenet_report *report, int epi, const float *aux,
                         const VerifyArgs *ver, hipStream_t s) {
  const int in_place = decoded != nullptr && decoded == out;
  if (in_place) decoded = nullptr;
  const int aligned = (ch.N % 4 == 0) && (ch.B0 % 4 == 0) && ((reinterpret_cast<uintptr_t>(decoded) & 15) == 0);
  dim3 grid((unsigned)finish_workgroups(ch, b, ver != nullptr)), block(256);
  const VerifyArgs none{};
#define CODENET_FINISH(GEN, VER)                                                                                    \
  hipLaunchKernelGGL((finish_kernel<GEN, VER>), grid, block, 0, s, out, syn, partials, n_parts, code_dev, b, decoded, \
                     aligned, in_place, report, epi, aux, ver ? *ver : none, geometry_of(ch))
  if (ver) {
    if (ch.r >= 4) CODENET_FINISH(true, true); else CODENET_FINISH(false, true);
  } else {
    if (ch.r >= 4) CODENET_FINISH(true, false); else CODENET_FINISH(false, false);
  }
#undef CODENET_FINISH
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && ver) {
    hipLaunchKernelGGL(verify_kernel, dim3(1), dim3(256), 0, s, ver->votes, (int)grid.x, report);
    e = hipGetLastError();
  }
  return e;
}

// ---------------------------------------------------------------------------
// Regeneration of the stored blocks at located nodes.  Along the axis of the
// phase's code, the L blocks of every line of the coded matrix form a codeword:
// parity block q is sum_i P[i][q] block_i.  The k <= t located blocks are
// rebuilt from a good systematic blocks' worth of others: the good systematic
// blocks and, for ks located systematic blocks, the first ks good parity blocks
// (a ks x ks system in the entries of P, nonsingular for an MDS generator).
// Every workgroup derives the k x L coefficient table itself (float64, one
// thread, a few hundred flops) from the report that the decision left on the
// device: no host round trip, and nothing happens unless the verdict is
// CORRECTED.  One workgroup rebuilds a 64 x 64 tile of one located block:
// fp32 matrix and its bf16 copy.
// ---------------------------------------------------------------------------
template <int TR>      // tile height: TR rows x 64 columns per workgroup
__global__ __launch_bounds__(256) void regen_kernel(RegenArgs g, const DevCode *__restrict__ code,
                                                    const codenet_report *__restrict__ report) {
  __shared__ float coef[CODENET_MAX_L];
  __shared__ int src_blk[CODENET_MAX_L];
  __shared__ int s_target, s_n_src;      // s_n_src < 0: the located blocks cannot be rebuilt (singular system)
  const int t = threadIdx.x;
  const int slot = blockIdx.z;
  if (report->verdict != CODENET_CORRECTED || slot >= report->n_located) return;
  const int a = code->a, r = code->r, L = code->L;
  // a report that does not fit this code (another phase's, or not a report at all) is ignored:
  // at most r / 2 distinct block indices below L
  {
    const int k = report->n_located;
    if (k < 1 || k > CODENET_MAX_T || 2 * k > r) return;
    for (int p = 0; p < k; ++p) {
      const int i = report->located[p];
      if (i < 0 || i >= L) return;
      for (int q = 0; q < p; ++q)
        if (report->located[q] == i) return;
    }
  }
  // work arrays of the one thread that derives the coefficients: in LDS, because dynamically
  // indexed private arrays live in scratch memory, where every dependent access is a memory latency
  __shared__ bool bad[CODENET_MAX_L];
  __shared__ int As[CODENET_MAX_T], Q[CODENET_MAX_T];
  __shared__ double M[CODENET_MAX_T][2 * CODENET_MAX_T];
  __shared__ double cs[CODENET_MAX_T][CODENET_MAX_L];
  if (t == 0) {
    const int k = report->n_located;
    for (int i = 0; i < L; ++i) bad[i] = false;
    int ks = 0;
    for (int p = 0; p < k; ++p) {
      const int i = report->located[p];
      bad[i] = true;
      if (i < a) As[ks++] = i;
    }
    int nq = 0;
    for (int q = 0; q < r && nq < ks; ++q)
      if (!bad[a + q]) Q[nq++] = q;
    // M[x][y] = P[As[y]][Q[x]] = H[Q[x]][As[y]]; Gauss-Jordan with partial pivoting -> Minv
    for (int x = 0; x < ks; ++x)
      for (int y = 0; y < ks; ++y) {
        M[x][y] = code->H[Q[x]][As[y]];
        M[x][ks + y] = x == y ? 1.0 : 0.0;
      }
    bool singular = false;
    for (int c = 0; c < ks && !singular; ++c) {
      int piv = c;
      for (int x = c + 1; x < ks; ++x)
        if (fabs(M[x][c]) > fabs(M[piv][c])) piv = x;
      // a generator that passed the MDS check has no vanishing pivot here; one that was only
      // sampled might: nothing is rebuilt then (the matrix stays as it is, the next check reports it)
      if (!(fabs(M[piv][c]) > 1e-12)) { singular = true; break; }
      for (int y = 0; y < 2 * ks; ++y) { const double tmp = M[c][y]; M[c][y] = M[piv][y]; M[piv][y] = tmp; }
      const double inv = 1.0 / M[c][c];
      for (int y = 0; y < 2 * ks; ++y) M[c][y] *= inv;
      for (int x = 0; x < ks; ++x)
        if (x != c) {
          const double f = M[x][c];
          for (int y = 0; y < 2 * ks; ++y) M[x][y] -= f * M[c][y];
        }
    }
    // located systematic block As[y] = sum_x Minv[y][x] (parity_Q[x] - sum_{good i'} P[i'][Q[x]] block_i')
    for (int y = 0; y < ks; ++y) {
      for (int i = 0; i < L; ++i) cs[y][i] = 0.0;
      for (int x = 0; x < ks; ++x) {
        const double mi = M[y][ks + x];
        cs[y][a + Q[x]] += mi;
        for (int i = 0; i < a; ++i)
          if (!bad[i]) cs[y][i] -= mi * code->H[Q[x]][i];
      }
    }
    const int target = report->located[slot];
    s_target = target;
    if (target < a) {
      int y = 0;
      while (As[y] != target) ++y;
      for (int i = 0; i < L; ++i) coef[i] = (float)cs[y][i];
    } else {
      const int q = target - a;
      for (int i = 0; i < L; ++i) {
        double c = (i < a && !bad[i]) ? code->H[q][i] : 0.0;
        for (int y = 0; y < ks; ++y) c += code->H[q][As[y]] * cs[y][i];
        coef[i] = (float)c;
      }
    }
    int n = 0;
    for (int i = 0; i < L; ++i)
      if (coef[i] != 0.f) src_blk[n++] = i;
    s_n_src = singular ? -1 : n;
  }
  __syncthreads();
  const int target = s_target, n_src = s_n_src;
  if (n_src < 0) return;
  const int B = code->B;
  // tile (r0, c0) of the located block; along the code's axis the block offset is target * B
  constexpr int P = TR / 16;
  static_assert(TR == 16 || TR == 32 || TR == 64, "tile height");
  const int r0 = blockIdx.y * TR, c0 = blockIdx.x * 64;
  const int rows = g.axis == 0 ? B : g.Mr, cols = g.axis == 0 ? g.Nc : B;
  const long blk = g.axis == 0 ? (long)B * g.Nc : (long)B;      // distance between consecutive blocks of a line
  const int gr0 = g.axis == 0 ? target * B + r0 : r0;           // row / column of the tile in the coded matrix
  const int gc0 = g.axis == 0 ? c0 : target * B + c0;
  // This thread's four rows rr = t / 16 + 16 p, columns cc .. cc + 3.  Source blocks (nonzero
  // coefficient) in ascending order, eight at a time for all four rows: 32 loads in flight, all
  // unconditional (rows / columns beyond the tile and sources beyond the last are clamped and
  // enter with weight zero or are not stored) -- a guarded load would wait for its data in a
  // branch of its own.
  const int cc = (t & 15) * 4;
  const int ccl = c0 + cc < cols ? c0 + cc : cols - 4;
  const float *first[P];
  bool in[P];
  float4 v[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int rr = (t >> 4) + 16 * p;
    in[p] = r0 + rr < rows && c0 + cc < cols;
    const int rrl = r0 + rr < rows ? r0 + rr : rows - 1;
    first[p] = g.W + (long)rrl * g.Nc + ccl;     // the same position in block 0 of the line; block sb is sb * blk further
    v[p] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  for (int q0 = 0; q0 < n_src; q0 += 8) {
    float4 x[P][8];
    long off[8];
    float w[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int sb = src_blk[q0 + u < n_src ? q0 + u : n_src - 1];
      off[u] = sb * blk;
      w[u] = q0 + u < n_src ? coef[sb] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int p = 0; p < P; ++p) x[p][u] = *reinterpret_cast<const float4 *>(first[p] + off[u]);
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int p = 0; p < P; ++p) {
        v[p].x = fmaf(w[u], x[p][u].x, v[p].x); v[p].y = fmaf(w[u], x[p][u].y, v[p].y);
        v[p].z = fmaf(w[u], x[p][u].z, v[p].z); v[p].w = fmaf(w[u], x[p][u].w, v[p].w);
      }
  }
#pragma unroll
  for (int p = 0; p < P; ++p) {
    if (!in[p]) continue;
    const int rr = (t >> 4) + 16 * p;
    *reinterpret_cast<float4 *>(g.W + (long)(gr0 + rr) * g.Nc + gc0 + cc) = v[p];
    if (g.Wb != nullptr) {
      const __bf16 b0 = (__bf16)v[p].x, b1 = (__bf16)v[p].y, b2 = (__bf16)v[p].z, b3 = (__bf16)v[p].w;
      const unsigned short u0 = __builtin_bit_cast(unsigned short, b0), u1 = __builtin_bit_cast(unsigned short, b1),
                           u2 = __builtin_bit_cast(unsigned short, b2), u3 = __builtin_bit_cast(unsigned short, b3);
      uint2 pk;
      pk.x = (unsigned)u0 | ((unsigned)u1 << 16);
      pk.y = (unsigned)u2 | ((unsigned)u3 << 16);
      *reinterpret_cast<uint2 *>(g.Wb + (long)(gr0 + rr) * g.ldWb + gc0 + cc) = pk;
    }
  }
}

hipError_t launch_regen(RegenArgs g, const DevCode *code_dev, const DevCode &ch, const codenet_report *report,
                        hipStream_t s) {
  const int tcap = ch.r / 2 < CODENET_MAX_T ? ch.r / 2 : CODENET_MAX_T;
  if (tcap < 1) return hipSuccess;
  const int rows = g.axis == 0 ? ch.B : g.Mr, cols = g.axis == 0 ? g.Nc : ch.B;
  // 32 x 64 tiles: 20.3 us at 5120 x 5120 against 20.9 (64 rows) and 21.2 (16 rows)
  hipLaunchKernelGGL(regen_kernel<32>, dim3((unsigned)((cols + 63) / 64), (unsigned)((rows + 31) / 32), (unsigned)tcap), dim3(256), 0, s,
                     g, code_dev, report);
  return hipGetLastError();
}

// One lane stores the constant-rate wall clock (s_memrealtime) with an ordinary vector store.
__global__ void timestamp_kernel(unsigned long long *dst) {
  if (threadIdx.x == 0) *dst = wall_clock64();
}

hipError_t launch_timestamp(unsigned long long *dst, hipStream_t s) {
  hipLaunchKernelGGL(timestamp_kernel, dim3(1), dim3(64), 0, s, dst);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Soft-error injection.  Noise element idx of a fault is a pure function of
// (seed, step, phase, bi, bj, idx) through the SplitMix64 output function
// (Steele, Lea, Flood 2014): z = mix(key + idx); bits 0..31 decide a sparse
// hit, bits 32..55 give u in [0, 1) in steps of 2^-24, bit 63 the sign.
// ---------------------------------------------------------------------------
__host__ __device__ inline unsigned long long mix64(unsigned long long x) {
  unsigned long long z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

unsigned long long fault_key(unsigned long long seed, unsigned long long step, int phase, int bi, int bj) {
  unsigned long long k = mix64(seed);
  k = mix64(k ^ step);
  return mix64(k ^ (((unsigned long long)phase << 40) | ((unsigned long long)bi << 20) | (unsigned long long)bj));
}

// sum of squares of the (still clean) target payload, kFaultParts partial sums
__global__ __launch_bounds__(256) void fault_stats_kernel(FaultBatch fb) {
  const FaultArgs &fa = fb.f[blockIdx.y];
  if (fa.mode != CODENET_NOISE_DENSE_REL) return;
  const long total = (long)fa.n_outer * fa.n_inner;
  // eight elements of the grid-stride sequence at a time: loads first, then the sum (in order)
  const bool small = total <= 0x7fffffffL;     // 32-bit index arithmetic (a 64-bit division is ~100 instructions)
  double acc = 0.0;
  const long stride = (long)gridDim.x * 256;
  for (long e0 = (long)blockIdx.x * 256 + threadIdx.x; e0 < total; e0 += 8 * stride) {
    // unconditional loads (index clamped, value dropped beyond the end): guarded ones would each
    // wait for their data in a branch of their own
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const long e = e0 + u * stride;
      const long ec = e < total ? e : total - 1;
      long o, in;
      if (small) {
        const unsigned q = (unsigned)ec / (unsigned)fa.n_inner;
        o = q; in = (unsigned)ec - q * (unsigned)fa.n_inner;
      } else {
        o = ec / fa.n_inner; in = ec % fa.n_inner;
      }
      const float x = fa.base[o * fa.stride_outer + in];
      v[u] = e < total ? x : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += (double)v[u] * (double)v[u];
  }
  __shared__ double red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
  if (lane == 0) red[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) fa.partials[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void fault_apply_kernel(FaultBatch fb) {
  const FaultArgs &fa = fb.f[blockIdx.y];
  const long total = (long)fa.n_outer * fa.n_inner;
  const long e = (long)blockIdx.x * 256 + threadIdx.x;
  // rms of the clean block from the kFaultParts partial sums of squares: one load per thread,
  // then a fixed-order tree (16 sums of 8, one sum of 16)
  __shared__ float s_scale;
  __shared__ double s_part[kFaultParts];
  __shared__ double s_sum[16];
  static_assert(kFaultParts == 128, "the tree below adds 16 x 8 partial sums");
  const bool dense = fa.mode == CODENET_NOISE_DENSE_REL;
  if (threadIdx.x < kFaultParts) s_part[threadIdx.x] = dense ? fa.partials[threadIdx.x] : 0.0;
  __syncthreads();
  if (threadIdx.x < 16) {
    double a = 0.0;
#pragma unroll
    for (int q = 0; q < 8; ++q) a += s_part[8 * threadIdx.x + q];
    s_sum[threadIdx.x] = a;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double ss = 0.0;
#pragma unroll
    for (int q = 0; q < 16; ++q) ss += s_sum[q];
    s_scale = dense ? (float)sqrt(ss / (double)total) : 1.f;
  }
  __syncthreads();
  if (e >= total) return;
  long o, in;
  if (total <= 0x7fffffffL) {
    const unsigned q = (unsigned)e / (unsigned)fa.n_inner;
    o = q; in = (unsigned)e - q * (unsigned)fa.n_inner;
  } else {
    o = e / fa.n_inner; in = e % fa.n_inner;
  }
  const unsigned long long idx = (unsigned long long)o * fa.idx_outer + (unsigned long long)in * fa.idx_inner;
  const unsigned long long z = mix64(fa.key + idx);
  const float u = (float)((z >> 32) & 0xFFFFFFull) * (1.0f / 16777216.0f);
  float val = fa.lo + (fa.hi - fa.lo) * u;
  if (fa.mode == CODENET_NOISE_DENSE_REL) {
    val *= s_scale;
    if (z >> 63) val = -val;
  } else if ((unsigned int)(z & 0xFFFFFFFFull) >= fa.hit_below) {
    return;
  }
  float *p = fa.base + o * fa.stride_outer + in;
  *p += val;
}

// One launch per batch of faults with pairwise distinct targets (grid.y = fault)
hipError_t launch_faults(const FaultBatch &fb, hipStream_t s, bool stats_pass) {
  if (fb.n < 1) return hipSuccess;
  if (stats_pass) {
    hipLaunchKernelGGL(fault_stats_kernel, dim3(kFaultParts, (unsigned)fb.n), dim3(256), 0, s, fb);
  } else {
    long most = 1;
    for (int f = 0; f < fb.n; ++f) {
      const long total = (long)fb.f[f].n_outer * fb.f[f].n_inner;
      most = total > most ? total : most;
    }
    hipLaunchKernelGGL(fault_apply_kernel, dim3((unsigned)((most + 255) / 256), (unsigned)fb.n), dim3(256), 0, s, fb);
  }
  return hipGetLastError();
}

}  // namespace codenet
