// C ABI of libcodenet: argument checking, the layer object, and the order in
// which the kernels of each call are enqueued.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "codenet_internal.h"

using namespace codenet;

struct codenet_layer {
  codenet_desc desc;            // P_r / P_c pointers are cleared after encode
  DevCode code_r, code_c;       // host copies: rows (forward check), columns (backward check)
  DevCode *code_r_dev = nullptr, *code_c_dev = nullptr;
  int Mr = 0, Nc = 0;           // coded sizes
  float *Wt = nullptr;          // [Mr][Nc]
  float *Xt = nullptr;          // [max_batch][Nc]   cached [x; x~]          (f32 mode only)
  float *Dt = nullptr;          // [max_batch][Mr]   cached [delta; delta~]  (f32 mode only)
  float *syn = nullptr;         // [max r][max_batch][max B]
  double *partials = nullptr;   // [kDetectParts][kMaxEntries]
  // pass 1 of the check as the product's epilogue left it (bf16 mode, codes that fit the kernel), per phase:
  // syndromes, records, and which output buffer / batch / number of records they describe (null: none)
  float *syn_p[2] = {nullptr, nullptr};
  double *partials_p[2] = {nullptr, nullptr};
  const float *rec_out[2] = {nullptr, nullptr};
  int rec_b[2] = {0, 0}, rec_parts[2] = {0, 0};
  double *fault_partials = nullptr;   // [CODENET_MAX_FAULTS][kFaultParts]
  double *partials_b = nullptr; // records of the second evaluation of the checks (verified check), as partials
  unsigned long long *votes = nullptr;  // one decision word per workgroup of the finishing kernel (verified check)
  // pending CODENET_CHECK fault, planted into the next verified check: target -1 = none
  int check_target = -1, check_who = 0;
  unsigned long long check_seed = 0;
  double check_scale = 0.0;
  // bf16 mode only: bf16 operands of the products and of the update
  __bf16 *Wb = nullptr;         // [max(Mr, KpD)][ldWb]  bf16 copy of W~, operand of both products
  __bf16 *Xb = nullptr;         // [max_batch][ldXb]  x, zero beyond the base columns
  __bf16 *Db = nullptr;         // [max_batch][ldDb]  delta, zero beyond the base rows
  __bf16 *XTb = nullptr;        // [Nc][ldT]    feature-major [x; x~] (update)
  __bf16 *DTb = nullptr;        // [Mr][ldT]    feature-major [delta; delta~] (update)
  float *part = nullptr;        // split-k partial results of the f32 products at thin batches: [kMaxSplits][max_batch][max(Mr, Nc)]
  long ldWb = 0;
  int KpX = 0, KpD = 0, bpad = 0;   // contraction lengths (multiples of 64): base columns, base rows, batch
  long ldXb = 0, ldDb = 0, ldT = 0; // pitches of Xb, Db and of XTb / DTb
  int fwd_b = 0, bwd_b = 0;     // batch of the cached vectors (0 = none)
  unsigned long updates = 0;    // number of updates enqueued so far
  unsigned long long *stamps = nullptr;   // profiling aid: four device time stamps around the product kernels (caller's memory)
  bool bf16 = false;
};

namespace {

int map_hip(hipError_t e, const char *what) {
  std::fprintf(stderr, "libcodenet: %s: %s\n", what, hipGetErrorString(e));
  (void)hipGetLastError();
  return e == hipErrorOutOfMemory ? CODENET_E_ALLOC : CODENET_E_HIP;
}

#define CN_HIP(expr)                                   \
  do {                                                 \
    hipError_t _e = (expr);                            \
    if (_e != hipSuccess) return map_hip(_e, #expr);   \
  } while (0)

int round_up4(int v) { return (v + 3) & ~3; }

double det_small(std::vector<double> a, int k) {   // Gaussian elimination with partial pivoting
  double det = 1.0;
  for (int c = 0; c < k; ++c) {
    int piv = c;
    for (int r = c + 1; r < k; ++r)
      if (std::fabs(a[r * k + c]) > std::fabs(a[piv * k + c])) piv = r;
    if (a[piv * k + c] == 0.0) return 0.0;
    if (piv != c) {
      for (int q = 0; q < k; ++q) std::swap(a[piv * k + q], a[c * k + q]);
      det = -det;
    }
    det *= a[c * k + c];
    for (int r = c + 1; r < k; ++r) {
      const double f = a[r * k + c] / a[c * k + c];
      for (int q = c; q < k; ++q) a[r * k + q] -= f * a[c * k + q];
    }
  }
  return det;
}

// next k-subset of {0..n-1} in lexicographic order; false when exhausted
bool next_subset(std::vector<int> &s, int n) {
  const int k = (int)s.size();
  int p = k - 1;
  while (p >= 0 && s[p] == n - k + p) --p;
  if (p < 0) return false;
  ++s[p];
  for (int q = p + 1; q < k; ++q) s[q] = s[q - 1] + 1;
  return true;
}

// |det| of the k x k minor of P on (rows, cols), relative to the product of the Euclidean norms of its
// columns (Hadamard's bound): 1 for orthogonal columns, 0 for dependent ones, whatever the scale of P.
double relative_minor(const double *P, int r, const std::vector<int> &rows, const std::vector<int> &cols) {
  const int k = (int)rows.size();
  std::vector<double> sub((size_t)k * k);
  double bound = 1.0;
  for (int y = 0; y < k; ++y) {
    double n2 = 0.0;
    for (int x = 0; x < k; ++x) {
      const double v = P[rows[x] * r + cols[y]];
      sub[x * k + y] = v;
      n2 += v * v;
    }
    bound *= std::sqrt(n2);
  }
  return bound > 0.0 ? std::fabs(det_small(sub, k)) / bound : 0.0;
}

double binomial(int n, int k) {
  double c = 1.0;
  for (int q = 1; q <= k; ++q) c = c * (n - k + q) / q;
  return c;
}

// G = [I | P] is MDS iff every square minor of P is non-zero (taken as: above 1e-9 of Hadamard's
// bound).  All minors of all orders are checked while there are at most 4e6 of them; a longer code
// gets every order checked on a share of that budget: completely where the order has few enough
// minors, otherwise on minors drawn by a fixed linear congruential sequence -- such a generator
// is verified by sampling only.
bool generator_is_mds(const double *P, int a, int r) {
  const double tol = 1e-9;
  const double budget = 4e6;
  const int orders = std::min(a, r);
  double total = 0.0;
  for (int k = 1; k <= orders; ++k) total += binomial(a, k) * binomial(r, k);
  const double share = total <= budget ? budget : budget / orders;
  unsigned long long lcg = 0x2545F4914F6CDD1Dull;
  for (int k = 1; k <= orders; ++k) {
    std::vector<int> rows(k), cols(k);
    if (binomial(a, k) * binomial(r, k) <= share) {
      for (int q = 0; q < k; ++q) rows[q] = q;
      do {
        for (int q = 0; q < k; ++q) cols[q] = q;
        do {
          if (!(relative_minor(P, r, rows, cols) > tol)) return false;
        } while (next_subset(cols, r));
      } while (next_subset(rows, a));
      continue;
    }
    auto draw = [&](std::vector<int> &set, int n) {      // k distinct indices below n, ascending
      std::vector<char> used((size_t)n, 0);
      for (int got = 0; got < k;) {
        lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
        const int v = (int)((lcg >> 33) % (unsigned long long)n);
        if (!used[v]) { used[v] = 1; ++got; }
      }
      for (int v = 0, q = 0; v < n; ++v) if (used[v]) set[q++] = v;
    };
    for (long trial = 0; trial < (long)share; ++trial) {
      draw(rows, a);
      draw(cols, r);
      if (!(relative_minor(P, r, rows, cols) > tol)) return false;
    }
  }
  return true;
}

void fill_code(DevCode &c, int a, int r, int N, const double *P, double tau_detect, double tau_resid) {
  std::memset(&c, 0, sizeof(c));
  c.a = a; c.r = r; c.L = a + r; c.N = N;
  c.B0 = (N + a - 1) / a;
  c.B = round_up4(c.B0);
  c.tau_detect = tau_detect; c.tau_resid = tau_resid;
  for (int k = 0; k < r; ++k) {
    for (int i = 0; i < a; ++i) c.H[k][i] = P[i * r + k];
    c.H[k][a + k] = -1.0;
    for (int i = 0; i < a + r; ++i) c.Hf[k][i] = (float)c.H[k][i];
  }
}

int real_entries(const DevCode &c, int block) {
  if (block >= c.a) return c.B0;
  const int left = c.N - block * c.B0;
  return left < 0 ? 0 : (left < c.B0 ? left : c.B0);
}

void free_layer(codenet_layer *l) {
  if (!l) return;
  (void)hipFree(l->Wt); (void)hipFree(l->Xt); (void)hipFree(l->Dt); (void)hipFree(l->syn);
  (void)hipFree(l->partials); (void)hipFree(l->fault_partials);
  (void)hipFree(l->partials_b); (void)hipFree(l->votes);
  for (int ph = 0; ph < 2; ++ph) { (void)hipFree(l->syn_p[ph]); (void)hipFree(l->partials_p[ph]); }
  (void)hipFree(l->code_r_dev); (void)hipFree(l->code_c_dev);
  (void)hipFree(l->Wb); (void)hipFree(l->Xb); (void)hipFree(l->Db);
  (void)hipFree(l->XTb); (void)hipFree(l->DTb); (void)hipFree(l->part);
  delete l;
}

}  // namespace

// Scratch of codenet_inject_noalloc: the partial sums of squares of up to CODENET_MAX_FAULTS faults
// (kFaultParts doubles each, 64 KB).  Every GPU holds its own copy of the array at its own address
// for the life of the process; that address is looked up once per device (scratch_address below)
// and is what host code passes around -- the array's name is only a handle on the host side.
static __device__ __align__(256) double scratch[CODENET_MAX_FAULTS * kFaultParts];

extern "C" {

const char *codenet_strerror(int code) {
  switch (code) {
    case CODENET_OK: return "ok";
    case CODENET_E_NULL: return "null pointer";
    case CODENET_E_SHAPE: return "bad shape";
    case CODENET_E_BATCH: return "batch out of range";
    case CODENET_E_ORDER: return "update needs a forward and a backward call with the same batch first";
    case CODENET_E_CODE: return "generator is not MDS or the code is too long";
    case CODENET_E_FAULT: return "fault names an inactive node";
    case CODENET_E_HIP: return "HIP runtime error";
    case CODENET_E_DTYPE: return "unknown dtype, phase or mode";
    case CODENET_E_ALLOC: return "out of device memory";
    default: return "unknown error";
  }
}

int codenet_encode(const codenet_desc *d, const float *W_dev, void *stream, codenet_layer **out) {
  if (!d || !W_dev || !out) return CODENET_E_NULL;
  *out = nullptr;
  if (d->n_out < 1 || d->n_in < 1 || d->m < 1 || d->n < 1 || d->r_rows < 0 || d->r_cols < 0 ||
      d->m > d->n_out || d->n > d->n_in)
    return CODENET_E_SHAPE;
  if (d->max_batch < 1) return CODENET_E_BATCH;
  if (d->dtype != CODENET_F32 && d->dtype != CODENET_BF16_F32ACC) return CODENET_E_DTYPE;
  if (d->r_rows > CODENET_MAX_R || d->r_cols > CODENET_MAX_R || d->m + d->r_rows > CODENET_MAX_L ||
      d->n + d->r_cols > CODENET_MAX_L)
    return CODENET_E_CODE;
  if ((d->r_rows > 0 && !d->P_r) || (d->r_cols > 0 && !d->P_c)) return CODENET_E_NULL;
  if (!(d->tau_detect >= 0.0) || !(d->tau_resid >= 0.0)) return CODENET_E_SHAPE;
  if (d->r_rows > 0 && !generator_is_mds(d->P_r, d->m, d->r_rows)) return CODENET_E_CODE;
  if (d->r_cols > 0 && !generator_is_mds(d->P_c, d->n, d->r_cols)) return CODENET_E_CODE;

  codenet_layer *l = new (std::nothrow) codenet_layer();
  if (!l) return CODENET_E_ALLOC;
  l->desc = *d;
  l->desc.P_r = l->desc.P_c = nullptr;
  l->bf16 = d->dtype == CODENET_BF16_F32ACC;
  fill_code(l->code_r, d->m, d->r_rows, d->n_out, d->P_r, d->tau_detect, d->tau_resid);
  fill_code(l->code_c, d->n, d->r_cols, d->n_in, d->P_c, d->tau_detect, d->tau_resid);
  l->Mr = l->code_r.L * l->code_r.B;
  l->Nc = l->code_c.L * l->code_c.B;
  hipStream_t s = (hipStream_t)stream;
  const size_t mb = (size_t)d->max_batch;
  const int rmax = std::max(std::max(d->r_rows, d->r_cols), 1);
  const int bmax = std::max(l->code_r.B, l->code_c.B);
  hipError_t e = hipSuccess;
  const char *what = "hipMalloc";
  auto alloc = [&](void **p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes ? bytes : 16); };
  alloc((void **)&l->Wt, sizeof(float) * (size_t)l->Mr * l->Nc);
  // fp32 coded vectors [x; x~], [delta; delta~]: operands of the f32 kernels only
  alloc((void **)&l->Xt, l->bf16 ? 0 : sizeof(float) * mb * l->Nc);
  alloc((void **)&l->Dt, l->bf16 ? 0 : sizeof(float) * mb * l->Mr);
  // split-k workspace of the f32 products: thin batches only (their tiles do not fill the chip)
  if (!l->bf16 && mb <= 256)
    alloc((void **)&l->part, sizeof(float) * (size_t)kMaxSplits * mb * std::max(l->Mr, l->Nc));
  alloc((void **)&l->syn, sizeof(float) * (size_t)rmax * mb * bmax);
  alloc((void **)&l->partials, sizeof(double) * (size_t)kDetectParts * kMaxEntries);
  alloc((void **)&l->fault_partials, sizeof(double) * (size_t)CODENET_MAX_FAULTS * kFaultParts);
  alloc((void **)&l->partials_b, sizeof(double) * (size_t)kDetectParts * kMaxEntries);
  alloc((void **)&l->votes, sizeof(unsigned long long) * ((mb * (size_t)(bmax / 4) + 255) / 256 + 1));
  alloc((void **)&l->code_r_dev, sizeof(DevCode));
  alloc((void **)&l->code_c_dev, sizeof(DevCode));
  if (l->bf16) {
    auto up64 = [](long v) { return (v + 63) & ~63L; };
    // A row pitch that is a multiple of 2 KB puts the same 128-byte column of every row of an
    // operand tile on one L2 channel, and all workgroups of an XCD walk those columns together:
    // such pitches get one more line (64 elements), so that consecutive rows change channel.
    auto pitch = [&](long v) { v = up64(v); return (v * 2) % 2048 == 0 ? v + 64 : v; };
    l->ldWb = pitch(l->Nc);
    l->KpX = (int)up64((long)l->code_c.a * l->code_c.B);
    l->KpD = (int)up64((long)l->code_r.a * l->code_r.B);
    l->ldXb = pitch(l->KpX);
    l->ldDb = pitch(l->KpD);
    // the backward product reads rows 0 .. KpD - 1 of the row-major copy: with no parity rows the 64-padding
    // of the contraction can reach past the matrix, so the copy has that many rows (the extra ones stay zero)
    const size_t szWb = 2 * (size_t)std::max(l->Mr, l->KpD) * l->ldWb;
    const size_t szXb = 2 * mb * l->ldXb, szDb = 2 * mb * l->ldDb;
    l->bpad = (int)up64((long)mb);
    l->ldT = pitch(l->bpad);
    alloc((void **)&l->XTb, 2 * (size_t)l->Nc * l->ldT);
    alloc((void **)&l->DTb, 2 * (size_t)l->Mr * l->ldT);
    // Only the forward product (k contiguous in both operands) can leave the check's records behind.
    if (product_check_fits(l->code_r.L, l->code_r.B, l->code_r.r, 1)) {
      alloc((void **)&l->syn_p[CODENET_FWD], sizeof(float) * (size_t)l->code_r.r * mb * l->code_r.B);
      alloc((void **)&l->partials_p[CODENET_FWD], sizeof(double) * (size_t)kDetectParts * kMaxEntries);
    }
    alloc((void **)&l->Wb, szWb);
    alloc((void **)&l->Xb, szXb);
    alloc((void **)&l->Db, szDb);
    // pitch padding and the tails beyond the base blocks stay zero for the layer's life
    what = "clearing the bf16 operands";
    if (e == hipSuccess) e = hipMemsetAsync(l->Wb, 0, szWb, s);
    if (e == hipSuccess) e = hipMemsetAsync(l->Xb, 0, szXb, s);
    if (e == hipSuccess) e = hipMemsetAsync(l->Db, 0, szDb, s);
  }
  if (e == hipSuccess) {
    what = "copy of the code tables";
    e = hipMemcpyAsync(l->code_r_dev, &l->code_r, sizeof(DevCode), hipMemcpyHostToDevice, s);
  }
  if (e == hipSuccess) e = hipMemcpyAsync(l->code_c_dev, &l->code_c, sizeof(DevCode), hipMemcpyHostToDevice, s);
  if (e == hipSuccess) {
    what = "encode kernel launch";
    e = launch_encode_matrix(W_dev, l->Wt, l->code_r_dev, l->code_c_dev, l->Mr, l->Nc, d->n_out, d->n_in, s);
  }
  if (e == hipSuccess && l->bf16) {
    what = "bf16 copies of the coded matrix";
    e = launch_shadow(l->Wt, l->Mr, l->Nc, l->Wb, l->ldWb, s);
  }
  // the host copies of the code tables must outlive the asynchronous copies above
  if (e == hipSuccess) {
    what = "encode stream synchronize";
    e = hipStreamSynchronize(s);
  }
  if (e != hipSuccess) {
    const int rc = map_hip(e, what);
    free_layer(l);
    return rc;
  }
  *out = l;
  return CODENET_OK;
}

int codenet_layer_geometry(const codenet_layer *l, int *B_r, int *B_c, int *coded_rows, int *coded_cols) {
  if (!l) return CODENET_E_NULL;
  if (B_r) *B_r = l->code_r.B;
  if (B_c) *B_c = l->code_c.B;
  if (coded_rows) *coded_rows = l->Mr;
  if (coded_cols) *coded_cols = l->Nc;
  return CODENET_OK;
}

namespace {
// The bf16 product of a phase: on tiles of whole codewords with the check's first pass in the
// epilogue where the operand layout and the code fit that kernel (the forward product), else the
// plain product (the check then reads the output).
int bf16_product(codenet_layer *l, int phase, Gemm2Args g2, const float *out, int b, hipStream_t s) {
  const DevCode &cd = phase == CODENET_FWD ? l->code_r : l->code_c;
  l->rec_out[phase] = nullptr;
  if (l->stamps) CN_HIP(launch_timestamp(l->stamps + 2 * phase, s));
  if (l->syn_p[phase] && !g2.a_k_major && product_check_fits(cd.L, cd.B, cd.r, b)) {
    CheckArgs c{};
    c.syn = l->syn_p[phase];
    c.partials = l->partials_p[phase];
    c.L = cd.L; c.Bp = cd.B; c.r = cd.r;
    for (int k = 0; k < cd.r; ++k)
      for (int i = 0; i < cd.L; ++i) c.Hf[k][i] = cd.Hf[k][i];
    int n_parts = 0;
    CN_HIP(launch_product_check(g2, c, &n_parts, s));
    l->rec_out[phase] = out;
    l->rec_b[phase] = b;
    l->rec_parts[phase] = n_parts;
  } else {
    CN_HIP(launch_product(g2, s));
  }
  if (l->stamps) CN_HIP(launch_timestamp(l->stamps + 2 * phase + 1, s));
  return CODENET_OK;
}
}  // namespace

int codenet_forward(codenet_layer *l, const float *X_dev, int b, float *S_coded_dev, void *stream) {
  return codenet_forward_ld(l, X_dev, l ? l->desc.n_in : 0, b, S_coded_dev, stream);
}

int codenet_forward_ld(codenet_layer *l, const float *X_dev, long ldx, int b, float *S_coded_dev, void *stream) {
  if (!l || !X_dev || !S_coded_dev) return CODENET_E_NULL;
  if (b < 1 || b > l->desc.max_batch) return CODENET_E_BATCH;
  if (ldx < l->desc.n_in) return CODENET_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  l->fwd_b = 0;
  if (l->bf16) {
    // coded input: batch-major bf16 x (product operand) and feature-major bf16 [x; x~] (update operand)
    CN_HIP(launch_encode_vector_bf16(X_dev, ldx, l->code_c_dev, l->code_c, b, l->Xb, l->ldXb, l->XTb, l->ldT, s));
    Gemm2Args g2{};
    g2.A = l->Wb; g2.lda = l->ldWb;
    g2.B = l->Xb; g2.ldb = l->ldXb;
    g2.C = S_coded_dev; g2.ldc = l->Mr;
    g2.I = l->Mr; g2.J = b; g2.K = l->KpX;
    const int rc = bf16_product(l, CODENET_FWD, g2, S_coded_dev, b, s);
    if (rc != CODENET_OK) return rc;
    l->fwd_b = b;
    return CODENET_OK;
  }
  CN_HIP(launch_encode_vector(X_dev, ldx, l->Xt, l->code_c_dev, l->code_c, b, nullptr, 0, nullptr, 0, s));
  GemmArgs g{};
  g.A = l->Wt; g.lda = l->Nc;                 // A[i][k] = W~[i][k], k over the base columns
  g.B = l->Xt; g.ldb = l->Nc;                 // B[j][k] = x[j][k]
  g.C = S_coded_dev; g.ldc = l->Mr;
  g.I = l->Mr; g.J = b; g.K = l->code_c.a * l->code_c.B;
  g.alpha = 1.f;
  g.workspace = l->part; g.max_splits = kMaxSplits;
  if (l->stamps) CN_HIP(launch_timestamp(l->stamps + 0, s));
  CN_HIP(launch_gemm(kFwd, g, s));
  if (l->stamps) CN_HIP(launch_timestamp(l->stamps + 1, s));
  l->fwd_b = b;
  return CODENET_OK;
}

int codenet_backward(codenet_layer *l, const float *D_dev, int b, float *C_coded_dev, void *stream) {
  return codenet_backward_ld(l, D_dev, l ? l->desc.n_out : 0, b, C_coded_dev, stream);
}

int codenet_backward_ld(codenet_layer *l, const float *D_dev, long ldd, int b, float *C_coded_dev, void *stream) {
  if (!l || !D_dev || !C_coded_dev) return CODENET_E_NULL;
  if (b < 1 || b > l->desc.max_batch) return CODENET_E_BATCH;
  if (ldd < l->desc.n_out) return CODENET_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  l->bwd_b = 0;
  if (l->bf16) {
    CN_HIP(launch_encode_vector_bf16(D_dev, ldd, l->code_r_dev, l->code_r, b, l->Db, l->ldDb, l->DTb, l->ldT, s));
    Gemm2Args g2{};
    // A[i][k] = W~[k][i]: the row-major copy, read k-major (transposing LDS reads in the kernel)
    g2.A = l->Wb; g2.lda = l->ldWb; g2.a_k_major = 1;
    g2.B = l->Db; g2.ldb = l->ldDb;
    g2.C = C_coded_dev; g2.ldc = l->Nc;
    g2.I = l->Nc; g2.J = b; g2.K = l->KpD;
    const int rc = bf16_product(l, CODENET_BWD, g2, C_coded_dev, b, s);
    if (rc != CODENET_OK) return rc;
    l->bwd_b = b;
    return CODENET_OK;
  }
  CN_HIP(launch_encode_vector(D_dev, ldd, l->Dt, l->code_r_dev, l->code_r, b, nullptr, 0, nullptr, 0, s));
  GemmArgs g{};
  g.A = l->Wt; g.lda = l->Nc;                 // A[i][k] = W~[k][i], k over the base rows
  g.B = l->Dt; g.ldb = l->Mr;                 // B[j][k] = delta[j][k]
  g.C = C_coded_dev; g.ldc = l->Nc;
  g.I = l->Nc; g.J = b; g.K = l->code_r.a * l->code_r.B;
  g.alpha = 1.f;
  g.workspace = l->part; g.max_splits = kMaxSplits;
  if (l->stamps) CN_HIP(launch_timestamp(l->stamps + 2, s));
  CN_HIP(launch_gemm(kBwd, g, s));
  if (l->stamps) CN_HIP(launch_timestamp(l->stamps + 3, s));
  l->bwd_b = b;
  return CODENET_OK;
}

int codenet_update(codenet_layer *l, float eta, void *stream) {
  if (!l) return CODENET_E_NULL;
  if (l->fwd_b < 1 || l->fwd_b != l->bwd_b) return CODENET_E_ORDER;
  hipStream_t s = (hipStream_t)stream;
  if (l->bf16) {
    const int bp = (l->fwd_b + 63) & ~63;
    Update2Args u{};
    u.XT = l->XTb; u.ldx = l->ldT;
    u.DT = l->DTb; u.ldd = l->ldT;
    u.W = l->Wt; u.ldw = l->Nc;
    u.Wb = l->Wb; u.ldWb = l->ldWb;
    u.I = l->Nc; u.J = l->Mr; u.K = bp; u.eta = eta;
    // The matrix and its copies are a little more than the memory-side cache holds; sweeping them
    // in the same order every step is the worst case for its LRU replacement, so the direction
    // alternates: what the last update wrote last is read first.
    u.reverse = (int)(l->updates & 1);
    ++l->updates;
    CN_HIP(launch_update2(u, s));
    return CODENET_OK;
  }
  GemmArgs g{};
  g.A = l->Xt; g.lda = l->Nc;                 // A[i][k] = x~[k][i]     (i = coded column, k = batch)
  g.B = l->Dt; g.ldb = l->Mr;                 // B[j][k] = delta~[k][j] (j = coded row)
  g.C = l->Wt; g.ldc = l->Nc;
  g.I = l->Nc; g.J = l->Mr; g.K = l->fwd_b;
  g.alpha = eta;
  CN_HIP(launch_gemm(kUpd, g, s));
  return CODENET_OK;
}

int codenet_detect_decode(codenet_layer *l, int phase, float *coded_out_dev, int b, float *decoded_dev,
                          codenet_report *report_dev, void *stream) {
  return codenet_detect_decode_act(l, phase, coded_out_dev, b, decoded_dev, report_dev, CODENET_EPI_NONE, nullptr,
                                   stream);
}

namespace {
int check_call(codenet_layer *l, int phase, float *coded_out_dev, int b, float *decoded_dev, codenet_report *report_dev,
               int epilogue, const float *aux_dev, bool verified, void *stream);
}

int codenet_detect_decode_act(codenet_layer *l, int phase, float *coded_out_dev, int b, float *decoded_dev,
                              codenet_report *report_dev, int epilogue, const float *aux_dev, void *stream) {
  return check_call(l, phase, coded_out_dev, b, decoded_dev, report_dev, epilogue, aux_dev, false, stream);
}

int codenet_detect_decode_verified(codenet_layer *l, int phase, float *coded_out_dev, int b, float *decoded_dev,
                                   codenet_report *report_dev, int epilogue, const float *aux_dev, void *stream) {
  if (!report_dev) return CODENET_E_NULL;
  return check_call(l, phase, coded_out_dev, b, decoded_dev, report_dev, epilogue, aux_dev, true, stream);
}

namespace {
int check_call(codenet_layer *l, int phase, float *coded_out_dev, int b, float *decoded_dev, codenet_report *report_dev,
               int epilogue, const float *aux_dev, bool verified, void *stream) {
  if (!l || !coded_out_dev) return CODENET_E_NULL;
  if (epilogue < CODENET_EPI_NONE || epilogue > CODENET_EPI_MUL) return CODENET_E_DTYPE;
  if (epilogue != CODENET_EPI_NONE && !decoded_dev) return CODENET_E_NULL;
  if (aux_dev && aux_dev == decoded_dev) return CODENET_E_SHAPE;
  if ((epilogue == CODENET_EPI_MASK_POS || epilogue == CODENET_EPI_MUL) && !aux_dev) return CODENET_E_NULL;
  if (phase != CODENET_FWD && phase != CODENET_BWD) return CODENET_E_DTYPE;
  if (b < 1 || b > l->desc.max_batch) return CODENET_E_BATCH;
  hipStream_t s = (hipStream_t)stream;
  const DevCode &ch = phase == CODENET_FWD ? l->code_r : l->code_c;
  const DevCode *cd = phase == CODENET_FWD ? l->code_r_dev : l->code_c_dev;
  int n_parts = 0;
  // The product of this phase may have left the first pass behind (its records describe this very
  // buffer as the product wrote it: nothing but this call has touched it since).  Whatever happens
  // now, they are used up: the check may correct the buffer in place.
  const bool taken = !verified && ch.r > 0 && l->rec_out[phase] == coded_out_dev && l->rec_b[phase] == b;
  const float *syn = taken ? l->syn_p[phase] : l->syn;
  const double *partials = taken ? l->partials_p[phase] : l->partials;
  if (taken) n_parts = l->rec_parts[phase];
  l->rec_out[phase] = nullptr;
  if (ch.r > 0 && !taken) {
    CN_HIP(launch_detect(coded_out_dev, l->syn, l->partials, &n_parts, cd, ch, b, false, s));
  }
  if (verified && ch.r > 0) {
    CN_HIP(launch_detect(coded_out_dev, nullptr, l->partials_b, &n_parts, cd, ch, b, true, s));
    VerifyArgs ver{l->partials_b, l->votes, -1};
    if (l->check_target == CODENET_CHECK_EVALUATION)
      CN_HIP(launch_record_fault(l->check_who % 2 ? l->partials_b : l->partials, (int)(l->check_seed % (unsigned)n_parts),
                                 l->check_scale, s));
    else if (l->check_target == CODENET_CHECK_LIST)
      ver.faulty_evaluator = (int)(l->check_who % finish_workgroups(ch, b, true));
    l->check_target = -1;
    CN_HIP(launch_finish(coded_out_dev, l->syn, l->partials, n_parts, cd, ch, b, decoded_dev, report_dev, epilogue,
                         aux_dev, &ver, s));
    return CODENET_OK;
  }
  // with r = 0 there is nothing to check: zero records make the decision CLEAN
  CN_HIP(launch_finish(coded_out_dev, syn, partials, n_parts, cd, ch, b, decoded_dev, report_dev, epilogue,
                       aux_dev, nullptr, s));
  return CODENET_OK;
}
}  // namespace

namespace {

constexpr int kMaxDevices = 64;
std::atomic<double *> scratch_of_device[kMaxDevices];

// Device address of `scratch` on the current device; the first call on a device asks the runtime.
int scratch_address(double **out) {
  int dev = 0;
  CN_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CODENET_E_HIP;
  double *p = scratch_of_device[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    CN_HIP(hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch)));
    if (p == nullptr) return CODENET_E_HIP;
    scratch_of_device[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return CODENET_OK;
}

// Both injection entry points.  partials: kFaultParts doubles per fault, written by the first pass
// of every call before the second pass reads them (nothing has to be cleared between calls).
int inject_faults(codenet_layer *l, const codenet_fault *faults, int n_faults, float *coded_out_dev, int b,
                  double *partials, void *stream) {
  if (!l) return CODENET_E_NULL;
  if (n_faults == 0) return CODENET_OK;
  if (!faults) return CODENET_E_NULL;
  if (n_faults < 0 || n_faults > CODENET_MAX_FAULTS) return CODENET_E_SHAPE;
  const int phase = faults[0].phase;
  if (phase == CODENET_CHECK) {
    const codenet_fault &ft = faults[0];
    if (n_faults != 1) return CODENET_E_SHAPE;
    if ((ft.bi != CODENET_CHECK_EVALUATION && ft.bi != CODENET_CHECK_LIST) || ft.bj < 0) return CODENET_E_FAULT;
    l->check_target = ft.bi;
    l->check_who = ft.bj;
    l->check_seed = ft.seed;
    l->check_scale = (double)ft.hi;
    return CODENET_OK;
  }
  if (phase != CODENET_FWD && phase != CODENET_BWD && phase != CODENET_WEIGHT) return CODENET_E_DTYPE;
  if (phase != CODENET_WEIGHT) {
    if (!coded_out_dev) return CODENET_E_NULL;
    if (b < 1 || b > l->desc.max_batch) return CODENET_E_BATCH;
    l->rec_out[phase] = nullptr;      // the output changes: what the product recorded about it is stale
  }
  const DevCode &cr = l->code_r, &cc = l->code_c;
  FaultArgs fa[CODENET_MAX_FAULTS];
  for (int f = 0; f < n_faults; ++f) {
    const codenet_fault &ft = faults[f];
    if (ft.phase != phase) return CODENET_E_FAULT;
    if (ft.mode != CODENET_NOISE_DENSE_REL && ft.mode != CODENET_NOISE_SPARSE_ABS) return CODENET_E_DTYPE;
    if (ft.bi < 0 || ft.bj < 0) return CODENET_E_FAULT;
    bool active;
    if (phase == CODENET_FWD) active = ft.bi < cr.L && ft.bj < cc.a;
    else if (phase == CODENET_BWD) active = ft.bi < cr.a && ft.bj < cc.L;
    else active = ft.bi < cr.L && ft.bj < cc.L && (ft.bi < cr.a || ft.bj < cc.a);
    if (!active) return CODENET_E_FAULT;
    FaultArgs &a = fa[f];
    a.key = fault_key(ft.seed, ft.step, ft.phase, ft.bi, ft.bj);
    a.lo = ft.lo; a.hi = ft.hi; a.mode = ft.mode;
    double hb = std::floor((double)ft.density * 4294967296.0);
    a.hit_below = hb <= 0.0 ? 0u : (hb >= 4294967295.0 ? 4294967295u : (unsigned int)hb);
    a.partials = partials + (size_t)f * kFaultParts;
    if (phase == CODENET_FWD) {
      a.base = coded_out_dev + (size_t)ft.bi * cr.B;
      a.stride_outer = l->Mr; a.n_outer = b; a.n_inner = real_entries(cr, ft.bi);
      a.idx_outer = 1; a.idx_inner = (unsigned long long)b;
    } else if (phase == CODENET_BWD) {
      a.base = coded_out_dev + (size_t)ft.bj * cc.B;
      a.stride_outer = l->Nc; a.n_outer = b; a.n_inner = real_entries(cc, ft.bj);
      a.idx_outer = 1; a.idx_inner = (unsigned long long)b;
    } else {
      a.base = l->Wt + (size_t)ft.bi * cr.B * l->Nc + (size_t)ft.bj * cc.B;
      a.stride_outer = l->Nc; a.n_outer = real_entries(cr, ft.bi); a.n_inner = real_entries(cc, ft.bj);
      a.idx_outer = (unsigned long long)cc.B0; a.idx_inner = 1;
    }
  }
  hipStream_t s = (hipStream_t)stream;
  // Every rms is taken from the still clean data, then the noises are added in the order
  // given.  Faults go to the GPU in batches of up to kFaultBatch, one launch per batch; a
  // fault whose target block is already in the batch starts a new one, so that two noises
  // on one block are still added one after the other.
  for (int pass = 0; pass < 2; ++pass) {
    FaultBatch fb{};
    for (int f = 0; f < n_faults; ++f) {
      bool clash = false;
      for (int q = 0; q < fb.n; ++q) clash = clash || fb.f[q].base == fa[f].base;
      if (fb.n == kFaultBatch || (pass == 1 && clash)) {
        CN_HIP(launch_faults(fb, s, pass == 0));
        fb.n = 0;
      }
      if (pass == 1 || fa[f].mode == CODENET_NOISE_DENSE_REL) fb.f[fb.n++] = fa[f];
    }
    CN_HIP(launch_faults(fb, s, pass == 0));
  }
  if (phase == CODENET_WEIGHT && l->bf16)
    CN_HIP(launch_shadow(l->Wt, l->Mr, l->Nc, l->Wb, l->ldWb, s));
  return CODENET_OK;
}

}  // namespace

int codenet_inject(codenet_layer *l, const codenet_fault *faults, int n_faults, float *coded_out_dev, int b,
                   void *stream) {
  if (!l) return CODENET_E_NULL;
  return inject_faults(l, faults, n_faults, coded_out_dev, b, l->fault_partials, stream);
}

int codenet_inject_noalloc(codenet_layer *l, const codenet_fault *faults, int n_faults, float *coded_out_dev, int b,
                           void *stream) {
  if (!l) return CODENET_E_NULL;
  double *partials = nullptr;
  const int rc = scratch_address(&partials);
  if (rc != CODENET_OK) return rc;
  return inject_faults(l, faults, n_faults, coded_out_dev, b, partials, stream);
}

int codenet_regenerate(codenet_layer *l, int phase, const codenet_report *report_dev, void *stream) {
  if (!l || !report_dev) return CODENET_E_NULL;
  if (phase != CODENET_FWD && phase != CODENET_BWD) return CODENET_E_SHAPE;
  RegenArgs g{};
  g.W = l->Wt; g.Mr = l->Mr; g.Nc = l->Nc;
  g.Wb = l->bf16 ? l->Wb : nullptr; g.ldWb = l->ldWb;
  g.axis = phase == CODENET_FWD ? 0 : 1;
  // the forward output is checked by the code along the rows, so its located nodes are block-rows
  const bool rows = phase == CODENET_FWD;
  CN_HIP(launch_regen(g, rows ? l->code_r_dev : l->code_c_dev, rows ? l->code_r : l->code_c, report_dev,
                      (hipStream_t)stream));
  return CODENET_OK;
}

int codenet_export_coded(codenet_layer *l, float *Wc_dev, void *stream) {
  if (!l || !Wc_dev) return CODENET_E_NULL;
  CN_HIP(hipMemcpyAsync(Wc_dev, l->Wt, sizeof(float) * (size_t)l->Mr * l->Nc, hipMemcpyDeviceToDevice,
                        (hipStream_t)stream));
  return CODENET_OK;
}

int codenet_export_weights(codenet_layer *l, float *W_dev, void *stream) {
  if (!l || !W_dev) return CODENET_E_NULL;
  CN_HIP(launch_export_weights(l->Wt, W_dev, l->code_r, l->code_c, l->Nc, l->desc.n_out, l->desc.n_in,
                               (hipStream_t)stream));
  return CODENET_OK;
}

int codenet_destroy(codenet_layer *l) {
  if (!l) return CODENET_E_NULL;
  (void)hipDeviceSynchronize();
  free_layer(l);
  return CODENET_OK;
}

int codenet_output_modified(codenet_layer *l, int phase) {
  if (!l) return CODENET_E_NULL;
  if (phase != CODENET_FWD && phase != CODENET_BWD) return CODENET_E_DTYPE;
  l->rec_out[phase] = nullptr;
  return CODENET_OK;
}

int codenet_profile_stamps(codenet_layer *l, uint64_t *stamps_dev) {
  if (!l) return CODENET_E_NULL;
  l->stamps = reinterpret_cast<unsigned long long *>(stamps_dev);
  return CODENET_OK;
}

int codenet_timestamp(uint64_t *dst_dev, void *stream, int *ticks_per_us) {
  if (!dst_dev) return CODENET_E_NULL;
  if (ticks_per_us) {
    int dev = 0, khz = 0;
    CN_HIP(hipGetDevice(&dev));
    CN_HIP(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    *ticks_per_us = khz / 1000;
  }
  CN_HIP(launch_timestamp(reinterpret_cast<unsigned long long *>(dst_dev), (hipStream_t)stream));
  return CODENET_OK;
}

}  // extern "C"
