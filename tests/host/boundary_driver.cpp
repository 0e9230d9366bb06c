// Host-side walk over the C-ABI's argument checks and error paths, for a build of the library whose
// host code is instrumented (AddressSanitizer + UndefinedBehaviorSanitizer).  Runs without a GPU: every
// call below must come back with an error code (or succeed without touching a device) and leave nothing
// behind.  tests/test_host_sanitizers.py builds and runs it.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "codenet.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static std::vector<double> vandermonde(int a, int r) {
  std::vector<double> P((size_t)a * r);
  for (int i = 0; i < a; ++i) {
    double x = 1.0 + (double)i / a, p = 1.0;
    for (int k = 0; k < r; ++k) { P[(size_t)i * r + k] = p; p *= x; }
  }
  return P;
}

int main() {
  codenet_layer *layer = nullptr;
  float dummy = 0.f;
  // null arguments
  EXPECT(codenet_encode(nullptr, &dummy, nullptr, &layer) == CODENET_E_NULL);
  codenet_desc d{};
  d.n_out = 64; d.n_in = 64; d.m = 4; d.n = 4; d.r_rows = 2; d.r_cols = 2;
  auto P = vandermonde(4, 2);
  d.P_r = P.data(); d.P_c = P.data();
  d.dtype = 0; d.max_batch = 8; d.tau_detect = 1e-3; d.tau_resid = 2e-3;
  EXPECT(codenet_encode(&d, nullptr, nullptr, &layer) == CODENET_E_NULL);
  EXPECT(codenet_encode(&d, &dummy, nullptr, nullptr) == CODENET_E_NULL);
  // shapes
  codenet_desc e = d; e.m = 0;
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_SHAPE);
  e = d; e.n = 65;
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_SHAPE);
  e = d; e.n_out = -1;
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_SHAPE);
  e = d; e.max_batch = 0;
  { const int rc = codenet_encode(&e, &dummy, nullptr, &layer); EXPECT(rc == CODENET_E_BATCH || rc == CODENET_E_SHAPE); }
  e = d; e.dtype = 77;
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_DTYPE);
  // codes: too many parity blocks, a generator with a vanishing minor, one with proportional rows, a missing generator
  e = d; e.r_rows = CODENET_MAX_R + 1;
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_CODE);
  std::vector<double> bad = P; bad[2 * 2 + 1] = 0.0; bad[2 * 2 + 0] = 0.0;
  e = d; e.P_r = bad.data();
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_CODE);
  std::vector<double> prop = P; prop[1 * 2 + 0] = 2.0 * prop[0]; prop[1 * 2 + 1] = 2.0 * prop[1];
  e = d; e.P_c = prop.data();
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_CODE);
  e = d; e.P_r = nullptr;
  EXPECT(codenet_encode(&e, &dummy, nullptr, &layer) == CODENET_E_NULL);
  // the MDS check on the largest code the library takes (all orders of minors within its budget, then samples)
  {
    const int a = CODENET_MAX_L - CODENET_MAX_R, r = CODENET_MAX_R;
    std::vector<double> big((size_t)a * r);
    unsigned long long s = 12345;
    for (auto &v : big) { s = s * 6364136223846793005ULL + 1442695040888963407ULL; v = 0.3 + (double)(s >> 40) / (1 << 24); }
    e = d; e.n_out = 4 * a; e.n_in = 64; e.m = a; e.r_rows = r; e.P_r = big.data();
    // without a device this ends in an allocation or HIP error after the generator has been accepted,
    // or in CODENET_E_CODE if a sampled minor vanishes; either way the error path must release everything
    const int rc = codenet_encode(&e, &dummy, nullptr, &layer);
    EXPECT(rc != CODENET_OK || layer != nullptr);
    if (rc == CODENET_OK) codenet_destroy(layer);
    layer = nullptr;
  }
  // a valid description: without a device the allocations fail and the half-built layer is released
  {
    const int rc = codenet_encode(&d, &dummy, nullptr, &layer);
    if (rc == CODENET_OK) { codenet_destroy(layer); layer = nullptr; std::printf("note: a device is present\n"); }
    else EXPECT(rc == CODENET_E_HIP || rc == CODENET_E_ALLOC);
  }
  // calls on a null layer
  codenet_report rep{};
  codenet_fault f{};
  EXPECT(codenet_forward(nullptr, &dummy, 1, &dummy, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_backward(nullptr, &dummy, 1, &dummy, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_update(nullptr, 0.1f, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_detect_decode(nullptr, CODENET_FWD, &dummy, 1, &dummy, &rep, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_inject(nullptr, &f, 1, &dummy, 1, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_inject_noalloc(nullptr, &f, 1, &dummy, 1, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_regenerate(nullptr, CODENET_FWD, &rep, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_output_modified(nullptr, CODENET_FWD) == CODENET_E_NULL);
  int B = -1;
  EXPECT(codenet_layer_geometry(nullptr, &B, nullptr, nullptr, nullptr) == CODENET_E_NULL);
  EXPECT(codenet_destroy(nullptr) == CODENET_E_NULL || codenet_destroy(nullptr) == CODENET_OK);
  std::printf(failures ? "boundary driver: %d check(s) failed\n" : "boundary driver: all checks passed\n", failures);
  return failures ? 1 : 0;
}
