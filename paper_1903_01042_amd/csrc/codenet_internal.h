// Internal declarations shared by the HIP translation units of libcodenet.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "codenet.h"

namespace codenet {

// A kernel that needs more than 64 KB of LDS has to be told so once per device; one of these per
// kernel remembers on which devices that has happened (a bit per device ordinal).
struct LdsOnce { std::atomic<unsigned long long> devices{0}; };
template <typename K>
inline hipError_t allow_lds(K kern, int lds_bytes, LdsOnce *once) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (once->devices.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (e == hipSuccess) once->devices.fetch_or(bit, std::memory_order_release);
  return e;
}

constexpr int kDetectParts = 512;      // most per-workgroup partial records of one check
constexpr int kFaultParts = 128;       // partial sums of squares per fault
constexpr int kMaxGram = CODENET_MAX_R * (CODENET_MAX_R + 1) / 2;
constexpr int kMaxEntries = CODENET_MAX_L + kMaxGram;

// One systematic (a + r, a) code as the kernels see it (device memory).
struct DevCode {
  int a, r, L;                                   // L = a + r
  int B;                                         // block pitch (multiple of 4)
  int B0;                                        // real block size ceil(N / a)
  int N;                                         // logical length a dimension is cut from
  double H[CODENET_MAX_R][CODENET_MAX_L];        // parity check [P^T | -I]
  float Hf[CODENET_MAX_R][CODENET_MAX_L];        // the same, float32
  double tau_detect, tau_resid;
};

// What the decision kernel leaves for the correction kernel.
struct DevPlan {
  int verdict;
  int n_located;
  int located[CODENET_MAX_T];
  float coef[CODENET_MAX_T][CODENET_MAX_R];      // error block a = sum_k coef[a][k] * syndrome_k
};

struct GemmArgs {
  const float *A; long lda;     // operand A, logical A[i][k]
  const float *B; long ldb;     // operand B, logical B[j][k]
  float *C; long ldc;           // C[j][i], i contiguous
  int I, J, K;
  float alpha;                  // accumulate variant: C += alpha * A B^T
  int tiles_i, tiles_j;
  // split-k (products of thin batches): with a workspace of max_splits x J x ldc floats the launcher
  // may cut the contraction in pieces whose partial results are then added in split order
  float *workspace; int max_splits;
  int splits; long split_stride;   // set by the launcher
};
// out[idx] = sum over s < splits of part[s * stride + idx], in split order (count a multiple of 4)
hipError_t launch_reduce_partials(const float *part, long stride, int splits, float *out, long count, hipStream_t s);

enum GemmLayout { kFwd = 0, kBwd = 1, kUpd = 2 };
// float32 operands: fwd: A k-contiguous, B k-contiguous, C = A B^T
//                   bwd: A k-strided   , B k-contiguous, C = A B^T
//                   upd: A k-strided   , B k-strided   , C += alpha A B^T
hipError_t launch_gemm(GemmLayout layout, const GemmArgs &args, hipStream_t stream);

// bf16 operands, k contiguous and zero padded to a multiple of 64; C[j][i] fp32
struct Gemm2Args {
  const __bf16 *A; long lda;
  const __bf16 *B; long ldb;
  float *C; long ldc;
  int I, J, K;
  int tiles_i, tiles_j;          // set by the launcher
  int a_k_major;                 // A is stored A[k][i], i contiguous
};
struct Update2Args {
  const __bf16 *XT; long ldx;    // [I = coded columns][batch padded to 64]
  const __bf16 *DT; long ldd;    // [J = coded rows][batch padded to 64]
  float *W; long ldw;            // fp32 coded matrix [J][I]
  __bf16 *Wb; long ldWb;         // its bf16 copy (row-major)
  int I, J, K;
  float eta;
  int tiles_i, tiles_j;
  int reverse;                   // walk the tiles in the opposite order (alternates from call to call)
};
// pass 1 of the check, taken in the epilogue of the product (launch_product_check)
struct CheckArgs {
  float *syn;                    // syndromes [r][J][Bp], written for the correction pass
  double *partials;              // one record per tile, entry-major as detect_kernel's
  float Hf[4][10];               // H[k][block], zero beyond the code
  int L, Bp, r;                  // blocks per codeword, block pitch, parity blocks
};
constexpr int kMaxSplits = 8;
hipError_t launch_product(Gemm2Args g, hipStream_t s);
bool product_check_fits(int L, int Bp, int r, int J);
hipError_t launch_product_check(Gemm2Args g, CheckArgs c, int *n_parts, hipStream_t s);
hipError_t launch_update2(Update2Args g, hipStream_t s);
hipError_t launch_shadow(const float *Wt, int Mr, int Nc, void *Wb, long ldWb, hipStream_t s);

// Regeneration of located blocks: axis 0 = block-rows (code along the rows), 1 = block-columns
struct RegenArgs {
  float *W; int Mr, Nc;          // fp32 coded matrix [Mr][Nc]
  __bf16 *Wb; long ldWb;         // bf16 copy (null in the f32 mode)
  int axis;
};
hipError_t launch_regen(RegenArgs g, const DevCode *code_dev, const DevCode &code_host, const codenet_report *report,
                        hipStream_t s);

hipError_t launch_timestamp(unsigned long long *dst, hipStream_t s);

struct FaultArgs {
  float *base;                  // first element of the target payload
  long stride_outer;            // element (outer, inner) at base[outer * stride_outer + inner]
  int n_outer, n_inner;
  unsigned long long idx_outer, idx_inner;   // element index = outer * idx_outer + inner * idx_inner
  unsigned long long key;       // hash key of (seed, step, phase, bi, bj)
  float lo, hi;
  unsigned int hit_below;       // SPARSE_ABS: hit iff low 32 hash bits < hit_below
  int mode;
  double *partials;             // kFaultParts partial sums of squares of this fault
};
constexpr int kFaultBatch = 8;
struct FaultBatch {
  int n;
  FaultArgs f[kFaultBatch];
};

hipError_t launch_encode_matrix(const float *W, float *Wt, const DevCode *code_r, const DevCode *code_c,
                                int Mr, int Nc, int n_out, int n_in, hipStream_t s);
// Vb (optional): bf16 batch-major copy of the systematic part, pitch ldVb.
// zero (optional): zero_count4 float4 of a buffer to clear in the same pass.
hipError_t launch_encode_vector(const float *V, long ldv, float *Vt, const DevCode *code_dev, const DevCode &code_host,
                                int b, void *Vb, long ldVb, float *zero, long zero_count4, hipStream_t s);
hipError_t launch_encode_vector_bf16(const float *V, long ldv, const DevCode *code_dev, const DevCode &code_host,
                                     int b, void *Vb, long ldVb, void *VTb, long ldVT, hipStream_t s);
// pass 1 of a check.  second_evaluation: the same records computed by other workgroups (another
// compute unit for every record); syn may then be null (the syndromes are not written again)
hipError_t launch_detect(const float *out, float *syn, double *partials, int *n_parts,
                         const DevCode *code_dev, const DevCode &code_host, int b, bool second_evaluation,
                         hipStream_t s);
// Verification steps of Error Model 2 (null = none)
struct VerifyArgs {
  const double *partials_b;      // pass-1 records of the second evaluation
  unsigned long long *votes;     // one word per workgroup of the finishing kernel: its verdict and located nodes
  int faulty_evaluator;          // workgroup whose decision gets a planted error; -1 = none
};
long finish_workgroups(const DevCode &code_host, int b, bool verified);
hipError_t launch_record_fault(double *partials, int part, double scale, hipStream_t s);
// passes 2 + 3 of a check: decision (every workgroup, from the pass-1 records), correction, decoded output;
// with ver, the comparison of the two evaluations and of the workgroups' decisions as well
hipError_t launch_finish(float *out, const float *syn, const double *partials, int n_parts,
                         const DevCode *code_dev, const DevCode &code_host, int b, float *decoded,
                         codenet_report *report, int epilogue, const float *aux, const VerifyArgs *ver,
                         hipStream_t s);
hipError_t launch_faults(const FaultBatch &fb, hipStream_t s, bool stats_pass);
hipError_t launch_export_weights(const float *Wt, float *W, const DevCode &cr, const DevCode &cc,
                                 int Nc, int n_out, int n_in, hipStream_t s);

unsigned long long fault_key(unsigned long long seed, unsigned long long step, int phase, int bi, int bj);

}  // namespace codenet
