/*
 * gecc -- grid-code protected matrix product for AMD MI355X (gfx950).
 *
 * C ABI of the library.  The calls follow the paper's statement of the
 * problem: encode A and B (Section III), multiply the encoded operands
 * (Section III, C-bar = A-bar B-bar), verify (Section V step 1), correct
 * (Section V step 2), and return the corrected C plus the located errors.
 *
 * Conventions
 *   - All indices in this ABI are 0-based; the weight of 0-based index i in a
 *     weighted parity is i+1 (the paper's index sets start at 1, Section II-A).
 *   - Logical shapes: A is n x k, B is k x m, C is n x m (Section II-A).
 *   - "dev" pointers are device (HBM) addresses, "host" pointers host
 *     addresses.  Every device buffer is allocated and owned by the caller;
 *     the library allocates no device memory and frees none.
 *   - All work is enqueued on the HIP stream handed in (a hipStream_t passed
 *     as void*; NULL = the default stream).  No call synchronises except
 *     gecc_report_to_host, gecc_syndromes_to_host, gecc_timing_read and
 *     gecc_protected_gemm_retry (which reads its reports back after every attempt).
 *   - Return value: 0 = ok, negative = usage or HIP error (see
 *     gecc_strerror); nothing throws or aborts.  The outcome of decoding
 *     travels in gecc_report.status, not in the return value.
 *   - Calls on one context must not overlap in time (they share the context's
 *     workspace); use one context per concurrent stream.
 */
#ifndef GECC_H
#define GECC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gecc_ctx gecc_ctx; /* opaque */

/* element type of A and B; products accumulate in fp32 and C is fp32 */
enum { GECC_F32 = 0, GECC_BF16 = 1 };

/* decode outcome */
enum {
  GECC_CLEAN = 0,         /* every syndrome inside its threshold                    */
  GECC_CORRECTED = 1,     /* errors located and removed                             */
  GECC_UNCORRECTABLE = 2, /* pattern beyond the code: recompute (Section V, step 1) */
  GECC_DETECTED = 3       /* gecc_verify found flagged lines; gecc_correct not run  */
};

/* which matrix a located error sits in */
enum { GECC_MAT_A = 0, GECC_MAT_B = 1, GECC_MAT_C = 2 };

/* error codes */
enum {
  GECC_OK = 0,
  GECC_ERR_ARG = -1,       /* null pointer, non-positive size, bad enum, bad leading dim */
  GECC_ERR_WORKSPACE = -2, /* workspace missing or too small                             */
  GECC_ERR_HIP = -3,       /* a HIP runtime call failed (launch, copy)                   */
  GECC_ERR_SCRATCH = -5,   /* gecc_protected_gemm_static: the problem needs more scratch than
                              GECC_STATIC_SCRATCH_BYTES                                   */
  GECC_ERR_ALIGN = -4      /* a device pointer is not aligned to its element type (A, B: 2 or
                              4 bytes; C: 4; parity buffers: 8; workspace: 256).  Operands
                              whose base and rows are 16-byte aligned (lda/ldb multiples of 8
                              bf16 or 4 fp32 elements, ldc a multiple of 4) take the vector
                              paths; others are correct but slower                        */
};

typedef struct {
  int32_t n, k, m;          /* logical sizes, each >= 1                                   */
  int32_t batch;            /* number of independent products, >= 1                       */
  int32_t dtype;            /* GECC_F32 or GECC_BF16                                      */
  int32_t trans_a;          /* 0: A stored n x k row-major (k contiguous), lda >= k
                               1: A stored k x n row-major (n contiguous), lda >= n       */
  int32_t trans_b;          /* 0: B stored k x m row-major (m contiguous), ldb >= m
                               1: B stored m x k row-major (k contiguous), ldb >= k       */
  int32_t refine;           /* 1: after Section V's subtraction, every patched symbol of C
                               is re-evaluated as its k-term dot product in fp64 (removes
                               the sqrt(n)-fold rounding noise the subtraction inherits)  */
  int64_t lda, ldb, ldc;    /* leading dimensions in elements; C is n x m row-major       */
  int64_t stride_a, stride_b, stride_c; /* element distance between batch items           */
  /* detection thresholds, one per syndrome family (the delta of Section V):
     row plain, row weighted, column plain, column weighted; operand audit */
  double tau_r1, tau_r2, tau_q1, tau_q2, tau_op;
  /* relative rounding allowance after an operand repair: a symbol of C whose running sum held
     the corrupted term f = e * b_lj may be off by tau_rep * sqrt(k) * |f|; the thresholds of the
     lines such a repair touched are widened accordingly in the second pass of Section V
     (root-sum-square over a whole repaired line).  16 * 2^-24 suits fp32 accumulation. */
  double tau_rep;
  /* relative rounding allowance of a syndrome value: when an estimate is verified, a syndrome y
     (a difference of fp32 sums) is trusted to tau + tau_rel * |y|.  Detection uses tau alone.
     2^-20 suits fp32 partial sums. */
  double tau_rel;
  /* 1: the grid code of Section III, two parities per line (the default of every binding).
     0: single-checksum mode, the conventional checksum scheme Section VI compares with (Table 1):
        the same kernels run, but detection and correction read the plain parities only -- errors
        confined to one row or one column of C are corrected (Appendix A, cases s = t = 1 and
        s = 1), everything else, a wrong operand symbol included (one parity names its line, not
        its place in it), is GECC_UNCORRECTABLE.  tau_r2 / tau_q2 are ignored, max_abs_synd[1] and
        [3] read 0. */
  int32_t weighted;
  /* Blocked grid code: block_n = block_m = 0 (the default) encodes the whole product as one
     codeword, as Section III does.  block_n, block_m > 0 (multiples of 128 that divide n and m;
     batch = 1, weighted = 1) apply Section III to every block_n x block_m block of C on its own:
     block (I, J) = A[rows of I, :] B[:, columns of J] gets two parity rows over its row block of A
     (weights 1 .. block_n), two parity columns over its column block of B (weights 1 .. block_m)
     and its own parity blocks P_r, P_c, P_g; Section V runs per block.  Up to two errors are
     corrected per block, the weights (and with them the rounding noise of the weighted sums,
     hence tau_r2 / tau_q2) are bounded by the block size, and no syndrome crosses a block.  The
     four thresholds are those of one block.  Buffer shapes in this mode, with NI = n / block_n,
     NJ = m / block_m, item (I, J) = I * NJ + J:
       A_par  NI x [2][k]      B_par  NJ x [2][k]
       C_par  NI * NJ items x { P_r [2][block_n], P_c [2][block_m], P_g [4] }
       reports, syndromes      one per item, positions relative to the block (operand errors: row
                               inside the row block of A / column inside the column block of B)
     gecc_item_count() gives NI * NJ; gecc_a_par_len() etc. give the sizes above.  The parity blocks
     P_r, P_c are formed on the matrix units (A times the parity columns of all column blocks at
     once, split into three bf16 pieces each for bf16 operands), in fp32 like C itself. */
  int32_t block_n, block_m;
  int32_t reserved;
} gecc_params;

/* one located error: `magnitude` is the additive offset that was removed */
typedef struct {
  int32_t matrix, row, col, reserved;
  double magnitude;
} gecc_err;

#define GECC_MAX_ERR 8

/* per batch item, written to device memory by verify / correct */
typedef struct {
  int32_t status;            /* GECC_CLEAN / CORRECTED / UNCORRECTABLE / DETECTED         */
  int32_t s, t;              /* flagged rows / columns at first detection (Section V)     */
  int32_t n_err;             /* entries used in err[], sorted by (matrix, row, col)       */
  gecc_err err[GECC_MAX_ERR];
  double max_abs_synd[4];    /* max |r1|, |r2|, |q1|, |q2| at first detection             */
  int32_t n_total;           /* located errors in all; err[] lists the first n_err of them
                                (more than GECC_MAX_ERR only for the patterns of Theorem 2:
                                many errors in at most two rows or columns of C)           */
  int32_t reserved;
} gecc_report;

/* a fault to be planted into the product while it is computed (E3 of Section II-A):
   offset is added to data symbol (row, col) of batch item `batch` before the
   syndromes are formed and before C is stored.  Positions in one list must be distinct. */
typedef struct {
  int32_t batch, row, col;
  float offset;
} gecc_fault;

#define GECC_MAX_FAULTS 1024

/* ---- context ------------------------------------------------------------------------ */

/* Validates *p and builds a context (host memory only). *out receives it.
   Reads the environment variable GECC_CU_COUNT once, here: if set to a positive number the
   bf16 product plans its rounds of tiles as for that many compute units instead of the
   device's own count (for tests of the k-split of a half-empty last round on small shapes;
   any value gives correct results).  Likewise GECC_TILE_MIN: operands of that many elements or
   more are encoded by the one-pass scan (default 2^25; tests set 1 to reach it with small shapes). */
int gecc_create(gecc_ctx** out, const gecc_params* p);
void gecc_destroy(gecc_ctx* ctx);

/* Bytes of device workspace the context needs (partial syndromes, syndromes, decoder
   state, audit parities, scan scratch, the partial tiles of a k-split product).  The caller
   allocates it (256-byte aligned) and hands it over; it stays the caller's.  Its contents need
   not be initialised: its first 64 KiB are counters that the library keeps at zero between
   launches, and the first compute call after gecc_set_workspace clears them with a small kernel
   on that call's stream (so a workspace is attached before, not while, a graph is captured, or
   the clear is captured with it, which is harmless).  Contexts may share one workspace when
   their calls are ordered on a stream; calls that overlap in time on one workspace race. */
size_t gecc_workspace_bytes(const gecc_ctx* ctx);
int gecc_set_workspace(gecc_ctx* ctx, void* dev_workspace, size_t bytes);

/* Sizes (in doubles, per batch item) of the parity buffers below (blocked mode: see gecc_params). */
size_t gecc_a_par_len(const gecc_ctx* ctx); /* 2*k           */
size_t gecc_b_par_len(const gecc_ctx* ctx); /* 2*k           */
size_t gecc_c_par_len(const gecc_ctx* ctx); /* 2*n + 2*m + 4 */
/* Number of reports (and of syndrome records) a call fills: batch, or the number of blocks. */
int32_t gecc_item_count(const gecc_ctx* ctx);

/* ---- the path ----------------------------------------------------------------------- */

/* S1, Section III (A_P = [P_n1; P_n2] A).  dev_A: the operand, read only.
   dev_A_par (out): batch x [2][k] doubles; [0][l] = sum_i a_il, [1][l] = sum_i (i+1) a_il. */
int gecc_encode_a(gecc_ctx* ctx, const void* dev_A, double* dev_A_par, void* stream);

/* S2, Section III (B_P = B [P_m1^T P_m2^T]).
   dev_B_par (out): batch x [2][k] doubles; [0][l] = sum_j b_lj, [1][l] = sum_j (j+1) b_lj. */
int gecc_encode_b(gecc_ctx* ctx, const void* dev_B, double* dev_B_par, void* stream);

/* S3, Section III (C-bar = A-bar B-bar).  Writes the data block C (fp32, n x m, ldc) and
   the parity blocks into dev_C_par: batch x { P_r [2][n], P_c [2][m], P_g [4] } doubles with
   P_r[0][i] = cbar_{i,m+1}, P_r[1][i] = cbar_{i,m+2}, P_c[0][j] = cbar_{n+1,j},
   P_c[1][j] = cbar_{n+2,j}, P_g = {cbar_{n+1,m+1}, cbar_{n+1,m+2}, cbar_{n+2,m+1},
   cbar_{n+2,m+2}}.  The product kernel also leaves per-tile partial row/column sums of the
   C it computed in the workspace, for gecc_verify(fused=1).
   dev_faults: NULL or n_faults (<= GECC_MAX_FAULTS) entries in device memory. */
int gecc_multiply(gecc_ctx* ctx, const void* dev_A, const double* dev_A_par, const void* dev_B,
                  const double* dev_B_par, float* dev_C, double* dev_C_par,
                  const gecc_fault* dev_faults, int32_t n_faults, void* stream);

/* S4 + S5, Section V step 1: the four syndrome families and the threshold tests.
   fused = 1: use the partial sums the immediately preceding gecc_multiply left in the workspace
              (C is not read; that call also reset the detection counters, so verify once per
              multiply);
   fused = 0: scan dev_C (for a C modified after the product, or produced elsewhere).
   dev_report (out): batch entries; status = GECC_CLEAN or GECC_DETECTED, s, t,
   max_abs_synd filled. */
int gecc_verify(gecc_ctx* ctx, const float* dev_C, const double* dev_C_par,
                gecc_report* dev_report, int32_t fused, void* stream);

/* S6 + S7, Section V step 2 and the operand audit: locates and removes the errors.
   Order: at most two flagged rows and two flagged columns: Section V's rule, every estimate
   verified against the syndromes.  Anything else, or a failed verification: both operands are
   re-encoded and compared with their stored parities (Section III: every column of A-bar, every
   row of B-bar is a codeword of its own); located operand symbols are patched and their
   rank-one footprint is taken out of C-bar; what is left goes through Section V's rule again or,
   with errors in many columns of at most two flagged rows (or the mirror image), through the
   decoder of Theorem 2 (Appendix B).
   Patches dev_A / dev_B / dev_C / dev_C_par in place; dev_report must be the one
   gecc_verify just filled.  All work is gated on device-side state, so the call is cheap
   when the report says CLEAN.  On GECC_UNCORRECTABLE the buffers hold whatever the attempt
   left behind and the product has to be recomputed. */
int gecc_correct(gecc_ctx* ctx, void* dev_A, const double* dev_A_par, void* dev_B,
                 const double* dev_B_par, float* dev_C, double* dev_C_par,
                 gecc_report* dev_report, void* stream);

/* encode_a, encode_b, multiply, verify(fused), correct in stream order (the larger operand is read
   once for its encoding and its parity block of C-bar).  No faults can be planted through this
   entry point: tests that want a fault inside the product use gecc_protected_gemm_retry with
   max_retries = 0, or the staged calls. */
int gecc_protected_gemm(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, double* dev_A_par,
                        double* dev_B_par, double* dev_C_par, gecc_report* dev_report,
                        void* stream);

/* Per-k-panel verification.  The code of Section III is linear in the operands: with the k index
   cut into `panels` consecutive panels, C-bar is the sum of the partial products
   A-bar[:, g] B-bar[g, :], and each of them has the grid structure of Definition 1 on its own, with
   the panel's slices of A_P and B_P as its operand parities.  This call runs the whole path --
   encode, multiply, verify (fused), correct -- on one panel after the other and adds the corrected
   partial products up in dev_C, so that a fault is caught, located and removed in the panel it
   strikes (two faults in two panels are two single faults), at the price of one more pass over C
   per panel after the first.  batch must be 1.
   Panel g covers k indices [g * step, min(k, (g + 1) * step)), step = k / panels rounded up to a
   multiple of 64; gecc_panel_count(ctx, panels) says how many of them are not empty (P below).
     dev_C_partial   n x ldc floats of scratch (may be null when P = 1)
     dev_A_par, dev_B_par   2 k doubles each: panel after panel, [2][k_g] of the panel's slice
     dev_C_par       P x (2 n + 2 m + 4) doubles: the parity blocks of every partial product
     dev_report      P reports; operand errors carry the column (of A) / row (of B) inside the panel
     dev_faults      NULL or n_faults test faults; the `batch` field of a fault names its panel
   The detection thresholds of a panel are the context's scaled by k_g / k (rounding noise of an
   fp32-accumulated sum grows with its number of terms).  The workspace of the context serves
   every panel in turn. */
int32_t gecc_panel_count(const gecc_ctx* ctx, int32_t panels);
int gecc_protected_gemm_panels(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, float* dev_C_partial,
                               double* dev_A_par, double* dev_B_par, double* dev_C_par,
                               gecc_report* dev_report, int32_t panels, const gecc_fault* dev_faults,
                               int32_t n_faults, void* stream);

/* For callers that cannot allocate device memory or hand a workspace over (code under HIP graph
   capture, tight serving loops, harnesses that forbid hipMalloc): gecc_protected_gemm on a scratch
   buffer that lives inside the library, a static device array of GECC_STATIC_SCRATCH_BYTES per GPU,
   held until the process ends.  Needs no gecc_set_workspace and calls no allocating routine.
   Returns GECC_ERR_SCRATCH, before anything is enqueued, when gecc_workspace_bytes(ctx) exceeds
   GECC_STATIC_SCRATCH_BYTES (a 16384 x 4096 x 14336 product needs 45 MiB in any storage layout,
   256 products of 512^3 need 37 MiB).  All calls on one GPU share that GPU's array, whatever their context:
   two such calls that overlap in time on one GPU race; calls in stream order on one stream are
   safe, and nothing has to be cleared between them (the first call on a GPU clears the array's
   counters with a small kernel on its stream).  The fused verification state lives in that
   array too, so gecc_syndromes_to_host does not see this call's syndromes.  The device current at
   the time of the call must be the one `stream` belongs to. */
#define GECC_STATIC_SCRATCH_BYTES (48u << 20)
int gecc_protected_gemm_static(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C,
                               double* dev_A_par, double* dev_B_par, double* dev_C_par,
                               gecc_report* dev_report, void* stream);

/* The recomputation Section V step 1 prescribes for a pattern beyond the code:
   encode_a, encode_b once, then multiply, verify(fused), correct and a read-back
   of the reports -- this call waits for the stream after every attempt -- until no batch item
   reports GECC_UNCORRECTABLE or max_retries (>= 0) recomputations were made.  The whole batch is
   recomputed from the operands as the last attempt left them (an attempt patches located
   operand errors).  dev_faults / n_faults (may be null / 0) are planted into the first product
   only (transient faults, for tests).  host_report (out, host): batch entries of the last
   attempt; *attempts (out, host, may be null): products computed. */
int gecc_protected_gemm_retry(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, double* dev_A_par,
                              double* dev_B_par, double* dev_C_par, gecc_report* dev_report,
                              gecc_report* host_report, int32_t max_retries, const gecc_fault* dev_faults,
                              int32_t n_faults, int32_t* attempts, void* stream);

/* The same product kernel without parity work and without the syndrome epilogue:
   the denominator of the overhead figure. */
int gecc_plain_gemm(gecc_ctx* ctx, const void* dev_A, const void* dev_B, float* dev_C, void* stream);

/* Copies `count` reports device -> host on `stream` and waits for it. */
int gecc_report_to_host(gecc_ctx* ctx, const gecc_report* dev_report, gecc_report* host_report,
                        int32_t count, void* stream);

/* Copies the syndromes of the last gecc_verify (r1[n], r2[n], q1[m], q2[m] per batch item,
   doubles) device -> host and waits; for threshold calibration.  A gecc_correct that repaired
   an operand error has moved them to the syndromes of the repaired C-bar. */
int gecc_syndromes_to_host(gecc_ctx* ctx, double* host_syndromes, void* stream);

/* Per-launch timing, for roofline reports.  Every kernel launch of the library belongs to one of
   the classes below.  gecc_timing_enable(ctx, r, mask) with r > 0 makes the next r launches whose
   class has its bit set in mask (bit GECC_K_x) record a HIP event pair on their stream (host
   objects only, no device memory); r = 0 disables and frees them.  gecc_timing_read waits for the
   recorded pairs, writes their durations in milliseconds to host_ms[0..*count) and their classes
   to host_kind[0..*count) (at most cap each; host_kind may be null) and rearms.  The product
   class brackets everything gecc_multiply's product step enqueues (the k-split tail's zeroing
   and second launch included); a row scan that carries the second stage of a column scan is
   timed with it. */
enum {
  GECC_K_ENCODE_A = 0,  /* A_P = [P_n1; P_n2] A                          */
  GECC_K_ENCODE_B = 1,  /* B_P = B [P_m1^T P_m2^T]                       */
  GECC_K_PARITY_R = 2,  /* P_r = A B_P                                   */
  GECC_K_PARITY_C = 3,  /* P_c = A_P B                                   */
  GECC_K_PRODUCT = 4,   /* data block C (+ fused partial sums, P_g)      */
  GECC_K_THRESHOLD = 5, /* partial sums -> syndromes -> flags            */
  GECC_K_DECODE = 6,    /* report / Section V step 2                     */
  GECC_K_AUDIT_A = 7,   /* gated re-encoding of A                        */
  GECC_K_AUDIT_B = 8,   /* gated re-encoding of B                        */
  GECC_K_REPAIR = 9,    /* gated operand repair + second pass            */
  GECC_K_PARTIALS = 10, /* stand-alone partial sums of a C in memory     */
  GECC_K_STAGE2 = 11,   /* second stage of a scan, launched alone        */
  GECC_K_TILE_A = 12,   /* A_P and P_r in one pass over A                */
  GECC_K_TILE_B = 13,   /* B_P and P_c in one pass over B                */
  GECC_K_AUDIT_AB = 14, /* both gated re-encodings in one launch         */
  GECC_K_COUNT = 15
};
int gecc_timing_enable(gecc_ctx* ctx, int32_t max_records, uint32_t kinds_mask);
int gecc_timing_read(gecc_ctx* ctx, float* host_ms, int32_t* host_kind, int32_t cap, int32_t* count);

const char* gecc_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* GECC_H */
