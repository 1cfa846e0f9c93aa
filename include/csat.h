/*
 * csat.h -- C ABI of the compressed-sensing attention (CSAT) forward pass for AMD MI355X (gfx950).
 *
 * The operations follow section 3 ("Mathematical Framework") of "CS-VLM: Compressed Sensing
 * Attention for Efficient Vision-Language Representation Learning":
 *
 *   measurement            K~ = Phi K,  V~ = Phi V                       (Phi in R^{m x n}, m <= n)
 *   compressed attention   A~ = softmax(Q K~^T / sqrt(d_k)),  Z = A~ V~
 *   sparse recovery        ISTA on  min 1/2 ||y - Phi x||^2 + lambda ||x||_1  (the l1 decoder the
 *                          section names), x^0 = 0, x <- eta_{mu*lambda}(x + mu Phi^T (y - Phi x)),
 *                          exactly `iters` iterations, one problem per query row with y = A~[i, :]
 *   synthesis              C^_i = Psi alpha^_i with Psi = V^T, i.e.  C^ = X V
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless the comment says "host".  The caller owns every
 *     buffer; the library keeps no reference to caller memory after a call returns and never
 *     frees it.  The only library-owned object is the opaque context.
 *   - Tensors are row-major and contiguous: Q [B,H,n_q,d]; K, V [B,H,n,d]; Phi [m,n], shared by
 *     all batches and heads; Kc, Vc [B,H,m,d]; A [B,H,n_q,m]; Z, C [B,H,n_q,d]; X [B,H,n_q,n].
 *   - `dtype` is the element type of Q, K, V, Phi and of the Kc, Vc, Z, C outputs
 *     (CSAT_F32: float, CSAT_BF16: bfloat16).  A, Y and X are always float.  In CSAT_BF16 mode
 *     MFMA operands are bf16 and every accumulation, the softmax and the decoder state are fp32.
 *   - Calls are asynchronous on `stream` (a hipStream_t, NULL = the default stream) and must not
 *     overlap with another call that uses the same workspace.
 *   - Every call validates its arguments on the host before touching the device; on any error
 *     status no output buffer has been written.  A status covers what the host can know when the
 *     call returns; what a kernel finds out later is reported by csat_decoder_status (below).
 *   - Data pointers and the workspace must be 16-byte aligned, d must be a multiple of 8.
 */
#ifndef CSAT_H
#define CSAT_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CSAT_OK = 0,
    CSAT_ERR_NULL = -1,       /* a required pointer is NULL */
    CSAT_ERR_SHAPE = -2,      /* non-positive dimension, m > n, or d not a multiple of 8 */
    CSAT_ERR_DTYPE = -3,      /* dtype is neither CSAT_F32 nor CSAT_BF16 */
    CSAT_ERR_ALIGN = -4,      /* a pointer is not 16-byte aligned */
    CSAT_ERR_WORKSPACE = -5,  /* workspace missing or smaller than csat_workspace_bytes() */
    CSAT_ERR_PARAM = -6,      /* lambda < 0, step <= 0 (or not finite), iters < 0 */
    CSAT_ERR_HIP = -7,        /* a HIP runtime call or kernel launch failed */
    CSAT_ERR_TIMEOUT = -8     /* csat_decoder_status only: the decoder of the last call gave up, its outputs are invalid */
} csat_status;

typedef enum { CSAT_F32 = 0, CSAT_BF16 = 1 } csat_dtype;

/* Problem shape.  n_q may differ from n (cross-attention).  m == n is legal (Phi = I case). */
typedef struct {
    int B, H, n_q, n, d, m;
    csat_dtype dtype;
} csat_dims;

/* Context: host object, holds no device memory.  create/destroy never touch the GPU. */
csat_status csat_create(void** ctx);
csat_status csat_destroy(void* ctx);

/* Static, host, NUL-terminated description of a status code. */
const char* csat_status_string(csat_status s);

/* Host-only query: bytes of device workspace that any of the calls below needs for these
 * dims and this iteration count (the maximum over the four entry points). */
csat_status csat_workspace_bytes(const csat_dims* dims, int iters, size_t* bytes);

/* Host helper (setup, off the hot path): draws a measurement matrix of one of the ensembles section 3 names
 * (its sentence on random Gaussian, Rademacher and structured matrices) into the HOST array phi_host [m, n],
 * row-major, caller-owned.  kind CSAT_PHI_GAUSSIAN: entries N(0, 1/m); CSAT_PHI_RADEMACHER: entries
 * +-1/sqrt(m).  The scaling and the generator are this library's choice, not the paper's: element i = r n + c
 * is drawn from words 2 i and 2 i + 1 of the SplitMix64 sequence started at `seed` (Gaussian by Box-Muller in
 * double precision, rounded to float; Rademacher from the top bit of the first word), so the same seed gives the
 * same matrix on every machine and any element can be drawn on its own.  Errors: CSAT_ERR_NULL, CSAT_ERR_SHAPE
 * (m or n not positive), CSAT_ERR_PARAM (unknown kind); nothing is written then. */
enum { CSAT_PHI_GAUSSIAN = 0, CSAT_PHI_RADEMACHER = 1 };
csat_status csat_phi_fill(int kind, unsigned long long seed, int m, int n, float* phi_host);

/* Host helper (setup, off the hot path): L = ||Phi||_2^2, the largest eigenvalue of Phi Phi^T,
 * in double precision from a HOST float matrix Phi [m,n]; ISTA's step is mu = 1/L. */
csat_status csat_phi_opnorm2(const float* phi_host, int m, int n, double* L);

/* Measurement (section 3, K~ = Phi_K K, V~ = Phi_V V with one shared Phi):
 * Kc[b,h] = Phi K[b,h], Vc[b,h] = Phi V[b,h]. */
csat_status csat_measure(void* ctx, const csat_dims* dims, const void* Phi, const void* K, const void* V,
                         void* Kc, void* Vc, void* workspace, size_t workspace_bytes, void* stream);

/* Compressed attention (section 3, A~ = softmax(Q K~^T / sqrt(d_k)), Z = A~ V~): row softmax over
 * the m compressed keys, no mask.  A (float, [B,H,n_q,m]) may be NULL when only Z is wanted. */
csat_status csat_compressed_attention(void* ctx, const csat_dims* dims, const void* Q, const void* Kc,
                                      const void* Vc, float* A, void* Z,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* Sparse recovery (section 3, ISTA decoder and C^_i = Psi alpha^_i): rows = B*H*n_q independent
 * problems.  Y [rows,m] float -> X [rows,n] float after exactly `iters` iterations from x = 0 with
 * threshold step*lambda; the support of row i is {j : X[i,j] != 0}.  X may be NULL when only C is
 * wanted.  If V and C are both non-NULL also writes C[b,h,i,:] = sum_j X[b,h,i,j] V[b,h,j,:]
 * (V and C in dims->dtype).  At least one of X, C must be requested.  iters == 0 gives X = 0, C = 0. */
csat_status csat_recover(void* ctx, const csat_dims* dims, const float* Y, const void* Phi,
                         float lambda, float step, int iters,
                         float* X, const void* V, void* C,
                         void* workspace, size_t workspace_bytes, void* stream);

/* The whole block: measurement, compressed attention, recovery, synthesis.  C is required;
 * Z (compressed output, dims->dtype) and X (float codes) are optional outputs.
 * iters == 0 skips the decoder and writes C = Z. */
csat_status csat_forward(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                         const void* Phi, float lambda, float step, int iters,
                         void* C, void* Z, float* X,
                         void* workspace, size_t workspace_bytes, void* stream);

/* The block under the column-wise reading of the recovery passage (section 3; the paper's claim of
 * a cost linear in n): self-attention only, dims->n_q == dims->n, else CSAT_ERR_SHAPE.  After the
 * compressed block, Y = Phi Z (m x d per head) is formed and each of the d feature columns of Y is
 * decoded by the same ISTA iteration into a length-n column of C: B*H*d problems instead of
 * B*H*n_q.  C [B,H,n,d] is required; Z (compressed output, dims->dtype) is optional.
 * iters == 0 skips the decoder and writes C = Z.  Needs the workspace csat_workspace_bytes reports
 * for these dims (it includes the second decoder's buffers whenever n_q == n). */
csat_status csat_forward_rd(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                            const void* Phi, float lambda, float step, int iters,
                            void* C, void* Z,
                            void* workspace, size_t workspace_bytes, void* stream);

/* The same three calls with the two measurement matrices of section 3 given separately
 * (K~ = Phi_K K, V~ = Phi_V V): PhiK and PhiV are both [m,n] in dims->dtype (device, 16-byte aligned,
 * required; they may be the same pointer, which is exactly the shared-Phi call).  PhiK is used for K~
 * only.  PhiV measures V and is the decoder's matrix, as the recovery passage states (Phi = Phi_V,
 * "reused for decoding"): it forms Y in the column-wise reading and is the Phi of every ISTA step, and
 * `step` is 1 / ||PhiV||_2^2.  Everything else (arguments, outputs, workspace, errors) as in
 * csat_measure / csat_forward / csat_forward_rd. */
csat_status csat_measure_kv(void* ctx, const csat_dims* dims, const void* PhiK, const void* PhiV,
                            const void* K, const void* V, void* Kc, void* Vc,
                            void* workspace, size_t workspace_bytes, void* stream);
csat_status csat_forward_kv(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                            const void* PhiK, const void* PhiV, float lambda, float step, int iters,
                            void* C, void* Z, float* X,
                            void* workspace, size_t workspace_bytes, void* stream);
csat_status csat_forward_rd_kv(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                               const void* PhiK, const void* PhiV, float lambda, float step, int iters,
                               void* C, void* Z,
                               void* workspace, size_t workspace_bytes, void* stream);

/* The unrolled (LISTA) form of the decoder (section 3, alpha^(t+1) = eta_theta(S alpha^(t) + B y)) with
 * caller-supplied weights: S [n,n] and Bw [n,m] in dims->dtype (device), thetas[iters] one threshold
 * per layer (HOST array, read before the call returns), alpha^(0) = 0.  Y, X, V, C as in csat_recover.
 * With S = I - step Phi^T Phi, Bw = step Phi^T and thetas[t] = step*lambda it computes what
 * csat_recover computes.  S is applied as I + (S - I): the iterate itself stays in fp32 and only the
 * correction goes through the bf16 product.  A negative or non-finite threshold gives CSAT_ERR_PARAM.
 * Needs the workspace csat_lista_workspace_bytes reports (host-only query). */
csat_status csat_lista_workspace_bytes(const csat_dims* dims, int iters, size_t* bytes);
csat_status csat_recover_lista(void* ctx, const csat_dims* dims, const float* Y, const void* S, const void* Bw,
                               const float* thetas, int iters,
                               float* X, const void* V, void* C,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Orthogonal matching pursuit, the greedy decoder the paper names next to ISTA (introduction,
 * limitations); standard algorithm: per row, k times pick the column of Phi with the largest
 * |phi_j^T r| (lowest index on a tie, no column twice), refit the picked coefficients by least
 * squares, update the residual r = y - Phi_S x_S.  Y [rows,m] float; outputs, each optional but at
 * least one required: X [rows,n] float (k non-zeros per row), picks [rows,k] int32 (device; column
 * indices in the order chosen), and C = X V when V and C are given (dims->dtype).
 * 0 <= k <= min(32, m) else CSAT_ERR_PARAM; m <= 1024 else CSAT_ERR_SHAPE; k == 0 gives zeros.
 * Correlations are computed with the operands in dims->dtype (bf16: the residual is rounded to
 * bf16 for the product), so near-ties may be decided differently from exact arithmetic.
 * Needs the workspace csat_omp_workspace_bytes reports (host-only query). */
csat_status csat_omp_workspace_bytes(const csat_dims* dims, int k, size_t* bytes);
csat_status csat_recover_omp(void* ctx, const csat_dims* dims, const float* Y, const void* Phi, int k,
                             float* X, int* picks, const void* V, void* C,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ISTA recovery for a structured measurement matrix (section 3, the sentence on measurement ensembles, names
 * structured Hadamard matrices next to Gaussian and Rademacher ones; the subsampling of rows, the random column
 * signs and the 1/sqrt(m) scale are this library's own construction), applied by fast Walsh-Hadamard transforms
 * instead of products with a stored Phi:
 *   Phi[l][j] = H_N[rows_of_h[l]][j] * signs[j] / sqrt(m),  j < n,
 * H_N the Walsh-Hadamard matrix of order N = smallest power of two >= n in natural ordering
 * (H[i][j] = (-1)^popcount(i & j)); rows_of_h [m] int32 distinct rows (device), signs [N] +-1 as
 * signed char (device).  In bf16 mode 1/sqrt(m) is taken rounded to bf16, as a stored bf16 Phi would
 * hold it.  Everything else (Y, lambda, step, iters, X, V, C, zero iterations) as in csat_recover.
 * n <= 16384, and a row's transform buffer and measurements must fit the 160 KB of LDS:
 * (N + N/32 + 2 m) * 4 bytes for N >= 512, (2 N + N/32 + 2 m) * 4 bytes below; else CSAT_ERR_SHAPE.  Workspace: csat_workspace_bytes. */
csat_status csat_recover_hadamard(void* ctx, const csat_dims* dims, const float* Y, const int* rows_of_h,
                                  const signed char* signs, float lambda, float step, int iters,
                                  float* X, const void* V, void* C,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* Completion status of the ISTA decoder (no passage of the paper: this is error reporting).  The fused
 * decoder (bf16, m <= 512) passes its rows from one workgroup to another between segments of the iterations
 * and bounds the wait for such a hand-over; if a wait ever ran out, the rows concerned were left unfinished.
 * The launching call has returned CSAT_OK long before (calls are asynchronous), so the kernel records the
 * failure in the workspace and a trailing kernel overwrites X (and, through the synthesis product, C) of that
 * call with NaN.  csat_decoder_status waits for `stream` (host-blocking), reads that record for the last
 * csat_recover / csat_forward* call that used `workspace` (device, the same pointer those calls were given; NULL
 * means the scratch of csat_forward_static on the current device) and returns CSAT_OK or CSAT_ERR_TIMEOUT.
 * Meaningful only after such a call has been issued on this workspace. */
csat_status csat_decoder_status(void* ctx, const void* workspace, void* stream);

/* Kernel-selection overrides (no passage of the paper: for A/B measurements and for tests that must reach a
 * particular kernel).  Options live in the context and apply to every later call made with it; value 0 is
 * the library's own choice for every key.  Results of a call depend on its arguments and these options only,
 * never on the process environment; csat_workspace_bytes does not depend on them.  An unknown key gives CSAT_ERR_PARAM. */
typedef enum {
    CSAT_OPT_DECODER = 0,          /* 1: ISTA as one GEMM pair per iteration even where the fused decoder applies; 2: the fused decoder wherever it fits (bf16, m <= 512), also on launches with few rows */
    CSAT_OPT_GEMM = 1,             /* 1: every contraction on the 128-wide GEMM kernel */
    CSAT_OPT_RASTER = 2,           /* low 3 bits: 1 the large-tile GEMM's column-fastest tile order everywhere, 2..5 its XCD-owned column groups of 1, 2, 4, 8 tiles; +8 / +16: never / always load its row operand with the non-temporal hint */
    CSAT_OPT_STATE = 3,            /* fused decoder's fp32 iterate in memory: 1 dense, 2 sparse; + 4 / + 8: its accesses always / never with the non-temporal hint */
    CSAT_OPT_FUSED_SEGMENTS = 4,   /* k >= 1: cut the fused decoder's iterations into k segments per row group; k <= -1: the two-chunk kernel's group-iterations in -k equal shares */
    CSAT_OPT_FUSED_THIN = 5,       /* 1: 128-row workgroups even for launches with few rows */
    CSAT_OPT_LISTA = 6,            /* 1: the unrolled decoder's layers on the element-wise epilogue */
    CSAT_OPT_HADAMARD = 7,         /* 1: the transform-based decoder with its iterate in LDS */
    CSAT_OPT_FUSED_SPIN_LIMIT = 8, /* k > 0: polls before a hand-over wait gives up; k < 0: give up at the first unmet poll */
    CSAT_OPT_INJECT_DECODER_ERROR = 9, /* 1 (tests): the decoder starts with its error record set, as if a wait had run out */
    CSAT_OPT_ATTENTION = 10,       /* 1: compressed attention as separate score, softmax and output kernels; 2: as one kernel for every shape */
    CSAT_OPT_FUSED_SCHEDULE = 11,  /* 1: the fused decoder's one-chunk-per-step schedule for every launch */
    CSAT_OPT_MEASURE = 12,         /* 1: the measurement as two GEMMs over transposed copies of K and V for every shape; 2: one kernel, but V~ transposed for a product GEMM, not as the attention kernel's fragments */
    CSAT_OPT_SYNTHESIS = 13,       /* 1: the synthesis C = X V always as a product kernel behind the decoder; 2: that kernel always the GEMM over a transposed copy of V */
    CSAT_OPT_Y_LAYOUT = 14,        /* 1: A~ row-major between the attention kernel and the fused decoder for every shape */
    CSAT_OPT_COUNT = 15
} csat_option;
csat_status csat_set_option(void* ctx, int key, int value);

/* csat_forward for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): the same block, the same kernels, the same arguments without a workspace.  The
 * workspace is a static array in the library's own device memory, csat_static_workspace_bytes() bytes (48 MiB)
 * per device, there from the moment the library is loaded until the process ends; the call allocates nothing
 * and calls no allocating routine (per-kernel timing, csat_profile_enable, is ignored here for that reason).
 * Problems whose csat_forward carving exceeds that size are refused with CSAT_ERR_WORKSPACE before anything is
 * launched.  Every call on a device uses that device's one array: calls that overlap on a device race, whatever
 * their streams; the array keeps the previous call's contents and every call clears what it needs cleared.
 * csat_decoder_status(ctx, NULL, stream) reports on the last such call. */
csat_status csat_static_workspace_bytes(size_t* bytes);
csat_status csat_forward_static(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                                const void* Phi, float lambda, float step, int iters,
                                void* C, void* Z, float* X, void* stream);

/* ------------------------------------------------------------------------------------------------------
 * Everything below this line is benchmark instrumentation and reference kernels: not part of the method,
 * not needed by a user of the block.
 * ------------------------------------------------------------------------------------------------------ */

/* Benchmark instrumentation (not part of the method).  When enabled, every kernel launch of the
 * calls above is bracketed by a pair of HIP events on the caller's stream, tagged with the id of
 * the step it belongs to; csat_profile_read waits for those events and returns the summed elapsed
 * milliseconds and the number of bracketed launches for one id.  Enabling or disabling discards
 * earlier records.  Event creation allocates: leave this off in production and under graph capture. */
typedef enum {
    CSAT_K_LAYOUT = 0,     /* operand packing / transposes */
    CSAT_K_MEASURE = 1,    /* K~ = Phi K, V~ = Phi V */
    CSAT_K_SCORES = 2,     /* Q K~^T / sqrt(d) */
    CSAT_K_SOFTMAX = 3,    /* row softmax over m */
    CSAT_K_OUTPUT = 4,     /* Z = A~ V~ */
    CSAT_K_RESIDUAL = 5,   /* ISTA: r = y - Phi x */
    CSAT_K_UPDATE = 6,     /* ISTA: x <- eta(x + mu Phi^T r) */
    CSAT_K_SYNTHESIS = 7,  /* C^ = X V */
    CSAT_K_COUNT = 8
} csat_kernel_id;
csat_status csat_profile_enable(void* ctx, int on);
csat_status csat_profile_read(void* ctx, int kernel_id, double* total_ms, int* launches);
/* Which kernel the last ISTA decoder call on this context launched (for the benchmark's kernel names):
 * -1 not the fused decoder (or no decoder call yet); fused decoder, one chunk per step: 0 dense state, 1 sparse
 * state, 2 one 32-row tile per workgroup; two chunks per step: 3 dense state, 4 sparse state. */
csat_status csat_profile_decoder_kernel(void* ctx, int* kernel);

/* Measurement (section 3, K~ = Phi K, V~ = Phi V) for the same structured Phi, by transforms: one Walsh-Hadamard
 * transform of length N per head and feature column, no stored matrix and no workspace.  rows_of_h, signs as in
 * csat_recover_hadamard; K, V [B,H,n,d] -> Kc, Vc [B,H,m,d] in dims->dtype (device, 16-byte aligned).
 * n <= 16384 and B*H <= 65535, else CSAT_ERR_SHAPE. */
csat_status csat_measure_hadamard(void* ctx, const csat_dims* dims, const int* rows_of_h, const signed char* signs,
                                  const void* K, const void* V, void* Kc, void* Vc, void* stream);

/* The whole block (csat_forward's arguments and outputs) with the structured Phi given by rows_of_h and signs:
 * measurement and decoder by transforms, no stored matrix.  step = 1 / ||Phi||_2^2 of that matrix (1 <= ||Phi||_2^2
 * <= N / m; the caller computes it, e.g. from the explicit matrix once).  Limits as in csat_recover_hadamard and
 * csat_measure_hadamard; workspace: csat_workspace_bytes. */
csat_status csat_forward_hadamard(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                                  const int* rows_of_h, const signed char* signs, float lambda, float step, int iters,
                                  void* C, void* Z, float* X,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* csat_forward_rd (the column-wise reading; dims->n_q == dims->n) with the structured Phi: Y = Phi Z and the
 * decoder by transforms, no stored matrix.  Arguments as in csat_forward_rd with rows_of_h, signs in place of Phi;
 * limits as in csat_recover_hadamard with B*H*d decoder problems. */
csat_status csat_forward_rd_hadamard(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                                     const int* rows_of_h, const signed char* signs, float lambda, float step,
                                     int iters, void* C, void* Z,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Reference launches for the benchmark (not on the product path): what the device delivers for the two
 * roofs the kernels are priced against, and for instruction issue next to the MFMAs.
 * csat_peak_copy: one streaming copy of `bytes` (a multiple of 16) from src to dst, both device, 16-byte
 *   aligned, not overlapping; it moves 2*bytes through HBM.
 * csat_peak_mfma: a register-resident v_mfma_f32_32x32x16_bf16 loop on every compute unit (two wavefronts
 *   per SIMD, `iters` x 16 MFMAs each); writes the number of floating-point operations of the launch to
 *   *flops (host) and per-lane sums to out (device, at least 2 * CUs * 1024 bytes, else
 *   CSAT_ERR_WORKSPACE; 1 MiB is enough for any device).
 * csat_peak_mfma_issue: the same MFMA with ONE wavefront per SIMD (the fused decoder's occupancy) and, behind
 *   every MFMA, valu_per_mfma independent fp32 fmas and lds_reads_per_mfma 16-byte LDS reads per lane
 *   (`iters` x 8 MFMAs per wavefront): how much else a single wavefront can issue before its MFMAs are delayed.
 *   (valu_per_mfma, lds_reads_per_mfma) is one of (0,0) (3,0) (6,0) (9,0) (12,0) (0,1) (3,1) (6,1) (0,2), else
 *   CSAT_ERR_PARAM; out and *flops as for csat_peak_mfma (at least CUs * 1024 bytes).
 * All are asynchronous on `stream`; the caller times them. */
csat_status csat_peak_copy(void* ctx, const void* src, void* dst, size_t bytes, void* stream);
csat_status csat_peak_mfma(void* ctx, float* out, size_t out_bytes, int iters, double* flops, void* stream);
csat_status csat_peak_mfma_issue(void* ctx, float* out, size_t out_bytes, int iters, int valu_per_mfma, int lds_reads_per_mfma,
                                 double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CSAT_H */
