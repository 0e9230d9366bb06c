/*
 * codenet.h -- C ABI of the MI355X (gfx950) CodeNet coded layer step.
 *
 * CodeNet (arXiv 1903.01042) splits a layer's weight matrix W (N_out x N_in)
 * into an m x n grid of blocks, encodes it once with two systematic real MDS
 * codes into a grid of (m + r_rows) x (n + r_cols) blocks, and then runs every
 * training step on the coded matrix: coded forward product, coded backward
 * product, a parity check on each product that detects, locates and corrects
 * erroneous block outputs, and a coded update that keeps the code structure
 * without re-encoding W.  The paper's error-prone nodes are blocks of one
 * GPU's work here; soft errors are injected by codenet_inject.
 *
 * Conventions
 *  - Every function returns CODENET_OK (0) or a negative CODENET_E* code and
 *    never throws.  codenet_strerror() names a code.
 *  - "dev" pointers are device memory (or host memory the GPU can address,
 *    such as pinned allocations); "host" pointers are ordinary host memory and
 *    are only read during the call.
 *  - All GPU work is enqueued on `stream` (a hipStream_t passed as void*;
 *    NULL = the default stream) and is asynchronous; no call synchronises
 *    except codenet_encode (once, at set-up) and codenet_destroy.
 *  - Activations are batch-major, row-major, float32: X is [b][N_in],
 *    Delta is [b][N_out], decoded S is [b][N_out], decoded C is [b][N_in],
 *    densely packed.  W is [N_out][N_in] row-major float32.
 *  - Block geometry.  A dimension of N entries split in `parts` equal parts
 *    uses blocks of ceil(N / parts) entries, zero padded at the end of the
 *    dimension; the library stores each block with a pitch B rounded up to a
 *    multiple of 4.  Coded outputs use that geometry: the forward coded output
 *    is [b][(m + r_rows) * B_r] with block i in columns [i*B_r, (i+1)*B_r)
 *    (real entries first, then zeros); the backward one is
 *    [b][(n + r_cols) * B_c].  codenet_layer_geometry() reports B_r, B_c.
 *  - Ownership.  The caller owns W, X, Delta, the coded / decoded output
 *    buffers and the report.  The layer owns the coded weights, the cached
 *    coded inputs [x; x~] (from codenet_forward) and [delta; delta~] (from
 *    codenet_backward) that codenet_update consumes, and all scratch memory,
 *    all allocated by codenet_encode and released by codenet_destroy.
 *  - Calls on one layer must not overlap in time (they share scratch memory), and are made
 *    with the device current that was current in codenet_encode (the layer's memory lives
 *    there).  Different layers may be driven from different host threads.
 */
#ifndef CODENET_H
#define CODENET_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CODENET_MAX_T 4          /* largest number of correctable blocks per product */
#define CODENET_MAX_R 8          /* largest number of parity blocks per dimension    */
#define CODENET_MAX_L 40         /* largest codeword length m + r (n + r)            */
#define CODENET_MAX_FAULTS 64    /* faults per codenet_inject call                   */

typedef struct codenet_layer codenet_layer;   /* opaque */

typedef enum { CODENET_F32 = 0, CODENET_BF16_F32ACC = 1 } codenet_dtype;
typedef enum { CODENET_FWD = 0, CODENET_BWD = 1, CODENET_WEIGHT = 2, CODENET_CHECK = 3 } codenet_phase;
typedef enum { CODENET_CLEAN = 0, CODENET_CORRECTED = 1, CODENET_UNCORRECTABLE = 2,
               CODENET_DISAGREE = 3 /* codenet_detect_decode_verified only */ } codenet_verdict;
/* what a CODENET_CHECK fault hits (its `bi`) */
typedef enum { CODENET_CHECK_EVALUATION = 0, CODENET_CHECK_LIST = 1 } codenet_check_target;
typedef enum { CODENET_NOISE_DENSE_REL = 0, CODENET_NOISE_SPARSE_ABS = 1 } codenet_noise_mode;

enum {
  CODENET_OK = 0,
  CODENET_E_NULL = -1,      /* a required pointer is NULL                          */
  CODENET_E_SHAPE = -2,     /* non-positive or inconsistent sizes                  */
  CODENET_E_BATCH = -3,     /* b < 1 or b > max_batch                              */
  CODENET_E_ORDER = -4,     /* update without a forward and a backward before it   */
  CODENET_E_CODE = -5,      /* generator not MDS, or r / m + r beyond the limits   */
  CODENET_E_FAULT = -6,     /* fault names a node that is not active in its phase  */
  CODENET_E_HIP = -7,       /* a HIP runtime call failed                           */
  CODENET_E_DTYPE = -8,     /* unknown dtype / phase / mode                        */
  CODENET_E_ALLOC = -9      /* out of device memory                                */
};

/* Layer description (all host memory, read only during codenet_encode). */
typedef struct {
  int n_out, n_in;          /* logical shape of W                                              */
  int m, n;                 /* base node grid (Section "Some Notations"); 1 <= m <= n_out,
                               1 <= n <= n_in, else CODENET_E_SHAPE                         */
  int r_rows, r_cols;       /* parity block-rows / block-columns; the paper uses 2t of each to
                               correct t errors per product (Theorem 1); 0 = uncoded          */
  const double *P_r;        /* m x r_rows, row-major: parity part of G_r = [I | P_r]          */
  const double *P_c;        /* n x r_cols, row-major: parity part of G_c = [I | P_c]          */
  int dtype;                /* codenet_dtype: arithmetic of the three products                */
  int max_batch;            /* largest b any later call will use                              */
  double tau_detect;        /* a product is clean iff every relative syndrome norm is <= this */
  double tau_resid;         /* a located support is accepted iff its relative residual <= this */
} codenet_desc;

/* Result of one check, written by the GPU to caller memory (device or pinned host). */
typedef struct {
  int verdict;                      /* codenet_verdict                                          */
  int n_located;                    /* 0 .. t                                                   */
  int located[CODENET_MAX_T];       /* ascending coded block index along the codeword
                                       (block-row for FWD, block-column for BWD); unused = -1   */
  float syn_rel[CODENET_MAX_R];     /* ||syndrome_k||_F / ref_k, ref_k^2 = sum_i H[k,i]^2 ||out_i||_F^2 */
  float resid_rel;                  /* relative least-squares residual of the best support tried */
} codenet_report;

/* One soft error (Error Model 2: additive continuous noise on a node's output). */
typedef struct {
  int phase;                /* codenet_phase: product whose output is hit, WEIGHT (update stage) or CHECK */
  int bi, bj;               /* node (block-row, block-column) in the coded grid                  */
  int mode;                 /* codenet_noise_mode                                                 */
  uint64_t seed, step;      /* noise is a pure function of (seed, step, phase, bi, bj, element)   */
  float lo, hi;             /* magnitude range                                                    */
  float density;            /* SPARSE_ABS only: fraction of elements hit                          */
  int reserved;
} codenet_fault;

/*
 * Pre-processing (Claim 1; appendix on the coding technique): build
 * W~ = (G_r^T (x) I) W (G_c (x) I), parity x parity corner included, in float32
 * (float64 accumulation), and allocate everything later calls need.
 * W_dev: [n_out][n_in] float32, device.  *out receives the layer.
 * Checks that both generators are MDS (every square minor of P non-singular).
 * Synchronises the stream before returning.
 */
int codenet_encode(const codenet_desc *desc, const float *W_dev, void *stream, codenet_layer **out);

/* Block pitches and coded sizes: coded_rows = (m + r_rows) * B_r, coded_cols = (n + r_cols) * B_c.
 * Any output pointer may be NULL. */
int codenet_layer_geometry(const codenet_layer *layer, int *B_r, int *B_c, int *coded_rows, int *coded_cols);

/*
 * Feedforward stage, steps 2-4: additional encoding x~ = (G_c^T (x) I) x (cached
 * for the update) and the coded product s~ = W~[:, base columns] x over the
 * active nodes (all block-rows, base block-columns), partial results summed
 * along each grid row.  X_dev: [b][n_in].  S_coded_dev: [b][coded_rows], written.
 */
int codenet_forward(codenet_layer *layer, const float *X_dev, int b, float *S_coded_dev, void *stream);

/*
 * Backpropagation stage, steps 2-4: delta~ = (G_r^T (x) I) delta (cached) and
 * c~^T = delta^T W~[base rows, :] over the active nodes (base block-rows, all
 * block-columns), summed along each grid column.  D_dev: [b][n_out].
 * C_coded_dev: [b][coded_cols], written.
 */
int codenet_backward(codenet_layer *layer, const float *D_dev, int b, float *C_coded_dev, void *stream);

/*
 * The same two calls for an input whose rows are ldx (ldd) floats apart, ldx >= n_in (ldd >= n_out;
 * else CODENET_E_SHAPE).  For inputs that are a part of wider rows: the decoded output of another
 * layer's check left in place in its coded buffer (codenet_detect_decode with decoded_dev =
 * coded_out_dev) is such an input when that layer's blocks carry no padding (its width a multiple of
 * its block count and the block a multiple of 4 entries): X_dev = its coded buffer, ldx = its coded width.
 */
int codenet_forward_ld(codenet_layer *layer, const float *X_dev, long ldx, int b, float *S_coded_dev, void *stream);
int codenet_backward_ld(codenet_layer *layer, const float *D_dev, long ldd, int b, float *C_coded_dev, void *stream);

/*
 * Soft-error injection (Error Models 1 / 2; the experiment's sparse law is
 * mode SPARSE_ABS).  All faults of one call must have the same phase.
 * FWD: node (bi, bj), bi < m + r_rows, bj < n, adds noise to block-row bi of
 * coded_out_dev ([b][coded_rows]); BWD: node (bi < m, bj < n + r_cols) adds noise to
 * block-column bj of coded_out_dev ([b][coded_cols]); WEIGHT: the stored block
 * W~_{bi,bj} (not in the corner) is corrupted, coded_out_dev is ignored.
 * DENSE_REL: every real element gets sign * U[lo, hi) * rms(clean target block);
 * SPARSE_ABS: a fraction `density` of the elements gets U[lo, hi).
 * faults_host: n_faults <= CODENET_MAX_FAULTS entries, host memory.
 * CHECK (errors in the error detection or in the decoding themselves, Error Model 2;
 * n_faults must be 1, coded_out_dev and b are ignored): nothing is enqueued; the fault is
 * kept and planted into the next codenet_detect_decode_verified call on this layer, then
 * forgotten.  bi = CODENET_CHECK_EVALUATION: one record of evaluation `bj % 2` of the
 * consistency checks (the partial squared norm of the first check kept by workgroup
 * `seed % workgroups`) becomes (1 + hi) * record + hi.  bi = CODENET_CHECK_LIST: evaluator
 * `bj % evaluators` of the decision gets a wrong list (first located node replaced by the
 * next block) or, with nothing located, a flipped verdict (CLEAN <-> UNCORRECTABLE).
 */
int codenet_inject(codenet_layer *layer, const codenet_fault *faults_host, int n_faults,
                   float *coded_out_dev, int b, void *stream);

/*
 * codenet_inject for callers that cannot allocate device memory or have the library use memory
 * it allocated earlier for its intermediate results: code under HIP graph capture, serving loops
 * and harnesses that forbid hipMalloc.  Same arguments, same results, bit for bit.  The partial
 * sums that the noise scale is taken from (128 per fault) live in a fixed array inside the
 * library's device code instead of in the layer: 64 KB per GPU, held until the process ends, enough
 * for CODENET_MAX_FAULTS faults -- more faults than that are refused with CODENET_E_SHAPE, as by
 * codenet_inject.  The call allocates and frees nothing, on the host or on the device.  All layers
 * on one GPU share the array: calls of this function that overlap in time on one GPU race (calls
 * on one stream are ordered and safe); nothing has to be cleared between calls, every call
 * writes the sums it reads.
 */
int codenet_inject_noalloc(codenet_layer *layer, const codenet_fault *faults_host, int n_faults,
                           float *coded_out_dev, int b, void *stream);

/*
 * Error detection and decoding (General Error-Detection Method; Lemma 2 and
 * the decoding algorithm of the appendix): syndromes (H (x) I) out with
 * H = [P^T | -I]; clean iff all relative syndrome norms <= tau_detect;
 * otherwise the support of at most t = floor(r/2) blocks with the smallest
 * least-squares residual is searched by increasing cardinality and accepted
 * if its relative residual <= tau_resid; accepted blocks are corrected in
 * place in coded_out_dev.  More errors than t: verdict UNCORRECTABLE,
 * coded_out_dev untouched (the caller rolls back; not an API error).
 * phase: CODENET_FWD or CODENET_BWD.  decoded_dev: [b][n_out] (FWD) or
 * [b][n_in] (BWD), receives the systematic part without padding; may be NULL, or
 * coded_out_dev itself ("in place": nothing is copied, the systematic part stays
 * where it is -- block i in columns [i * B, i * B + real entries) of each row of
 * coded_out_dev -- and a clean check writes nothing at all); any other overlap of
 * the two buffers is not allowed.  report_dev: written by the GPU; may be NULL.
 *
 * Where the consistency checks are evaluated.  In the bf16 mode, for row codes of at most ten
 * blocks and four parity blocks, the coded forward product computes them in its epilogue, while
 * the outputs of a codeword still sit side by side in registers, and leaves them with the layer
 * (the backward product reads the matrix the other way and does not);
 * this call then starts from them instead of reading the output again.  They are used only if
 * coded_out_dev is the buffer that the layer's last product of this phase wrote, with the same
 * b, and no codenet_inject or check has touched it since (both discard them, as does a
 * verified check, which evaluates the checks twice itself).  A caller that changes that buffer
 * by any other means between the product and the check must say so with
 * codenet_output_modified(), or the change goes unchecked.
 */
int codenet_detect_decode(codenet_layer *layer, int phase, float *coded_out_dev, int b,
                          float *decoded_dev, codenet_report *report_dev, void *stream);

/* The coded output of the last product of `phase` was modified by the caller: the check reads it afresh. */
int codenet_output_modified(codenet_layer *layer, int phase);

/*
 * The same with the elementwise primary step that follows the product applied
 * to the decoded output on its way out (the per-layer algorithm's "generate
 * x^{l+1} = f(s^l)" in the feedforward stage and the diagonal post-multiplication
 * delta^{l-1} = g(x^l) (.) c^l in the backpropagation stage, with g(f(u)) = f'(u)):
 *   CODENET_EPI_RELU      decoded = max(decoded, 0)                  (f = ReLU)
 *   CODENET_EPI_MASK_POS  decoded = aux > 0 ? decoded : 0            (g of ReLU; aux = x^l)
 *   CODENET_EPI_MUL       decoded = decoded * aux                    (any f', supplied by the caller)
 * aux_dev has the shape of decoded_dev ([b][n_out] for FWD, [b][n_in] for BWD) and
 * is required by the last two; decoded_dev is required by all three.  The coded
 * output buffer keeps the (corrected) values before the elementwise step -- unless
 * decoded_dev is coded_out_dev, where the step is applied in place to the real entries
 * of the systematic blocks.
 */
typedef enum { CODENET_EPI_NONE = 0, CODENET_EPI_RELU = 1, CODENET_EPI_MASK_POS = 2, CODENET_EPI_MUL = 3 } codenet_epilogue;
int codenet_detect_decode_act(codenet_layer *layer, int phase, float *coded_out_dev, int b,
                              float *decoded_dev, codenet_report *report_dev, int epilogue,
                              const float *aux_dev, void *stream);

/*
 * The same check with the two verification steps that the decentralized
 * implementation adds under Error Model 2 ("Errors in Error-Detection" and
 * "Errors in decoding": the nodes exchange and compare their evaluations of the
 * 2t consistency checks, and later their lists of erroneous nodes; any
 * disagreement means that the checking itself went wrong and the network is
 * restored from the last checkpoint).  On one GPU: (1) the consistency checks are
 * evaluated twice, the second time with every partial result computed on another
 * compute unit, and the two sets of partial results are compared bit for bit;
 * (2) every workgroup of the correcting kernel takes the decision (verdict and
 * list of erroneous nodes) for itself and the decisions are compared.  Agreement:
 * exactly the results of codenet_detect_decode_act.  Disagreement: verdict
 * CODENET_DISAGREE, n_located 0; after a disagreement in step 1 nothing has been
 * corrected, after one in step 2 the contents of coded_out_dev and decoded_dev
 * are unspecified (an evaluator may have acted on its wrong decision) -- either
 * way the caller restores its checkpoint.  report_dev is required.  With r = 0
 * there is nothing to verify and the call equals codenet_detect_decode_act.
 */
int codenet_detect_decode_verified(codenet_layer *layer, int phase, float *coded_out_dev, int b,
                                   float *decoded_dev, codenet_report *report_dev, int epilogue,
                                   const float *aux_dev, void *stream);

/*
 * Update stage (the three block rules, plus the same rule on the corner):
 * W~ += eta * [delta; delta~] [x; x~]^T summed over the batch, using the vectors
 * cached by the last forward and backward calls (which must have used the same b).
 * The cached vectors stay valid until the next forward / backward call replaces
 * them: a second update applies the same gradient again.  (The check is made
 * when the call is enqueued; forward and backward calls replayed from a captured
 * graph refresh the vectors on the device without the host noticing.)
 */
int codenet_update(codenet_layer *layer, float eta, void *stream);

/*
 * Regeneration of the stored data at located nodes (Sec. "Errors in the update
 * stage" and the regeneration step of the per-layer algorithm; the worked
 * example W_{1,0} = W~_{2,0} - W_{0,0}).  report_dev is the report that
 * codenet_detect_decode left on the device for `phase`.  If its verdict is
 * CORRECTED, every stored block of the located block-rows (FWD) or
 * block-columns (BWD) is rebuilt from good blocks of the same grid column
 * (row): the good systematic blocks plus as many good parity blocks as there are
 * located systematic ones.  Any other verdict, or a located set that does not fit
 * the code of `phase` (more than r / 2 blocks, an index beyond the grid, a
 * repeated index), leaves the matrix untouched.  The
 * report is read on the device: the call never synchronises with the host.  In
 * the bf16 mode the bf16 copy of the rebuilt blocks is refreshed as well.
 * The cached vectors [x; x~], [delta; delta~] need no regeneration here: they
 * are re-encoded from the caller's inputs on every forward / backward call.
 */
int codenet_regenerate(codenet_layer *layer, int phase, const codenet_report *report_dev, void *stream);

/* Copy out the coded matrix, [coded_rows][coded_cols] float32 (drift checks, tests). */
int codenet_export_coded(codenet_layer *layer, float *Wc_dev, void *stream);

/* Copy out the systematic part without padding, [n_out][n_in] float32. */
int codenet_export_weights(codenet_layer *layer, float *W_dev, void *stream);

/* Waits for the device, frees everything the layer owns. */
int codenet_destroy(codenet_layer *layer);

/*
 * Time stamp on the device: when `stream` reaches this point, the GPU's
 * constant-rate wall clock is written to *dst_dev (one 64-bit count).
 * *ticks_per_us, if not NULL, receives the clock's rate during the call.  A
 * kernel like the others: it can be captured into a hipGraph together with the
 * calls above, where host-recorded events cannot stamp individual kernels.
 * The difference of two stamps around a call is that call's time on the GPU
 * plus one kernel boundary.
 */
int codenet_timestamp(uint64_t *dst_dev, void *stream, int *ticks_per_us);

/*
 * Profiling aid.  While stamps_dev is not NULL, codenet_forward and codenet_backward on this layer
 * put a device time stamp (as codenet_timestamp) before and after the kernel(s) of their coded
 * product: stamps_dev[0], [1] around the forward product, [2], [3] around the backward one (four
 * 64-bit counts, device memory of the caller's).  The vector encoding that the same calls run
 * first is outside the stamps.  NULL switches the stamps off again.
 */
int codenet_profile_stamps(codenet_layer *layer, uint64_t *stamps_dev);

const char *codenet_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CODENET_H */
