// Internal declarations shared by the translation units of libgecc (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gecc.h"

namespace gecc {

// ----------------------------------------------------------------------------------------
// The product kernel and the stand-alone syndrome kernel both reduce C in tile_m x tile_n
// tiles (the product kernel's own blocking, fixed when the context is created).

// rows per chunk of the two-stage column reduction (scan kernels)
constexpr int SCAN_CHUNK_ROWS = 128;
// "Done" counters at the front of the workspace: one per column segment (or chunk of rows) of a scan
// whose last workgroup adds the partial results up itself.  Zero between launches (the last arrival
// wraps its counter), zeroed once when a workspace is attached.
constexpr int SCAN_DONE_WORDS = 16384;
// A column reduction finishes by itself when one workgroup can add a segment's chunks up quickly
constexpr int SCAN_FUSE_MAX_CHUNKS = 64;

// decoder phases kept in device memory (per batch item)
enum : int { PH_DONE = 0, PH_AUDIT = 1, PH_REVERIFY = 2 };

struct AuditHit {
  int32_t line;   // l: column of A / row of B the hit is in
  int32_t pos;    // located row of A / column of B (0-based); -1 = not explainable
  double e;       // magnitude (plain parity difference)
};

struct DecodeState {
  // filled by the threshold kernel (atomics; cleared by reset_state before each verify)
  int32_t s_cnt, t_cnt;
  int32_t nonfinite;          // some syndrome is NaN or infinite: nothing can be subtracted, recompute
  int32_t rows[GECC_MAX_ERR], cols[GECC_MAX_ERR];
  // decoder
  int32_t phase;
  int32_t n_err;              // operand errors already accepted by the audit
  gecc_err errs[GECC_MAX_ERR];
};

struct Layout {            // byte offsets into the caller's workspace
  size_t done;             // uint32 [SCAN_DONE_WORDS]      always first, whatever the shape: contexts that share a
                           //                               workspace in stream order share the counters too
  size_t rowpart;          // float  [batch][ntn][rp_ld][2]   per-tile row sums (plain, local-weighted)
  size_t colpart;          // float  [batch][ntm][cp_ld][2]   per-tile column sums
                           // (rp_ld, cp_ld: n, m padded so that the slab stride is no power of two)
  size_t synd;             // double [batch][2n + 2m]     r1, r2, q1, q2
  size_t allow;            // double [batch][2n + 2m]     threshold allowances of repaired lines
  size_t state;            // DecodeState [batch]
  size_t audit_a;          // double [batch][2][k]        re-formed parity of A
  size_t audit_b;          // double [batch][2][k]        re-formed parity of B
  size_t blockmax;         // double [batch][nblk][4]     max |syndrome| per family and threshold workgroup
  size_t scan_a;           // double scratch of the two-stage column reduction (A side)
  size_t scan_b;           // same, B side
  size_t scan_row;         // double scratch of the row part of the tile scan (the larger operand's)
  size_t ksplit;           // float [batch x tiles][ksplit][128 x 128]: partial tiles of a k-split product (0 bytes: none)
  // blocked mode only
  size_t w_a, w_b;         // parity rows of all row blocks of A / parity columns of all column blocks of B, as operands of the product
  size_t side_r, side_c;   // float: A x (parity columns), (parity rows) x B
  size_t gate;             // int32: some block asked for the operand audit
  size_t total;
};

}  // namespace gecc

struct gecc_ctx {
  gecc_params p;
  gecc::Layout lay;
  int tile_m, tile_n;      // blocking of the product kernel = granularity of the partials
  int ntm, ntn;            // partial tiles along n and m
  int rp_ld, cp_ld;        // lines per slab of the row / column partials (n, m plus padding)
  int nbi, nbj;            // blocked mode: blocks along n and m (0, 0: the whole product is one codeword)
  int pieces;              // blocked mode: operand-type pieces one fp64 parity is split into (bf16: 3, fp32: 1)
  int w_cols_a, w_cols_b;  // rows of W_A (2 * pieces * nbi) and of W_B, padded to a multiple of 8
  int tile_op;             // operand whose two reductions share one pass (GECC_MAT_A / GECC_MAT_B)
  int ksplit;              // workgroups per tile of the 128 x 128-tile product kernel (1: no split)
  int cu_hint;             // GECC_CU_COUNT (tests: plan the tile rounds as for that many CUs), else 0
  int64_t tile_min;        // operands of that many elements or more take the tile scan (2^25; GECC_TILE_MIN for tests)
  char* ws;                // device workspace (caller's)
  size_t ws_bytes;
  char* ws_zeroed;         // the workspace whose "done" counters this context knows to be zero between launches
  int fault_bias;          // see GemmArgs::fault_bias (nonzero only in a panel's context)
  gecc_ctx** panel;        // contexts of the k-panels of the last gecc_protected_gemm_panels call
  int n_panel;
  hipEvent_t* ev;          // optional timing records around kernel launches (start, stop pairs)
  int32_t* ev_kind;        // class (GECC_K_x) of each record
  uint32_t ev_mask;        // classes that are recorded
  int ev_cap, ev_n;
};

namespace gecc {

// ---- scan kernels (scan_kernels.hip) -----------------------------------------------------
// X is a row-major R x Cc matrix (leading dimension ld, batch stride xs) of dtype.
// rowdot: out[b][t][r] = sum_c w_t[c] X[r,c];  coldot: out[b][t][c] = sum_r w_t[r] X[r,c].
// w == nullptr selects the index weights of Section III: w_0 = 1, w_1 = index + 1.
// Otherwise w points at batch x [2][len] doubles.  gate (may be null): int per batch item at
// byte stride gate_stride; the kernels return at once for items whose gate != gate_value.
// Second stage of a column scan (chunks of rows) and / or of the row part of a tile scan (segments of
// columns) that has not been launched yet: either launch_stage2() runs it as a kernel of its own,
// or the next rowdot launch carries it (a dependent launch costs about 5 us of stream time
// whatever it does, and this stage is tiny).
struct Stage2Job {
  bool valid;
  const double* scratch;      // column part: [batch][nchunk][2][Cc] -> out [2][Cc]   (Cc = 0: none)
  double* out;
  int64_t out_stride;
  int Cc, nchunk;
  const double* row_scratch;  // row part: [batch][R][nseg][2] -> row_out [2][R]     (R = 0: none)
  double* row_out;
  int64_t row_out_stride;
  int R, nseg;
  int batch;
  const int32_t* gate;
  int64_t gate_stride;
  int gate_value;
};
struct ScanArgs {
  const void* X;
  int dtype;
  int R, Cc;
  int64_t ld, xs;
  int batch;
  const double* w;      // [2][len] per batch item (batch stride w_stride doubles), or null
  double* out;          // [2][len_out] per batch item (batch stride out_stride doubles)
  int64_t w_stride, out_stride;
  int vec_ok;           // set by the launcher: rows are 16-byte aligned, vector loads allowed
  double* scratch;      // coldot only: [batch][nchunk][2][Cc]
  uint32_t* done;       // coldot only: counters (coldot_done_words of them, all zero); the scan then finishes
                        // by itself.  null: the second stage is left to the caller (see launch_coldot_stage1)
  const int32_t* gate;
  int64_t gate_stride;  // in bytes
  int gate_value;
  // rowdot only: the second stage of an earlier launch, done by carry_blocks extra workgroups at
  // the end of the grid (same batch and gate as the carrier)
  Stage2Job carry;
  int carry_blocks;
};
// carry: null, or a pending second stage whose output this scan does not read
hipError_t launch_rowdot(const ScanArgs& a, const Stage2Job* carry, hipStream_t st);
// launches the first stage and describes the second in *pending (pending->valid = false when the
// scan finishes by itself: a.done set)
hipError_t launch_coldot_stage1(const ScanArgs& a, Stage2Job* pending, hipStream_t st);
// counters a column scan needs to finish by itself; 0: it cannot (too many chunks per segment)
int coldot_done_words(const ScanArgs& a);
hipError_t launch_stage2(const Stage2Job& j, hipStream_t st);
int stage2_blocks(const Stage2Job& j);
// words[0 .. count) = 0 (a kernel, so that a captured call stays free of memset nodes)
hipError_t launch_zero_words(uint32_t* words, int count, hipStream_t st);
size_t coldot_scratch_doubles(int R, int Cc, int batch);

// tile scan: column part (out_col[t][c] = sum_r wr_t[r] X[r,c]) and row part (out_row[t][r] =
// sum_c wc_t[c] X[r,c]) of one operand in one pass; null weights = Section III's index weights.
// Either part alone computes bit for bit what it computes beside the other.
struct TileScanJob {
  const void* X;
  int dtype;
  int R, Cc;
  int64_t ld, xs;
  int batch;
  bool col_on;
  const double* wr;         // [2][R] per batch item, or null
  int64_t wr_stride;
  double* col_out;          // [2][Cc] per batch item
  int64_t col_out_stride;
  bool row_on;
  const double* wc;         // [2][Cc] per batch item, or null
  int64_t wc_stride;
  double* row_out;          // [2][R] per batch item
  int64_t row_out_stride;
  double* col_scratch;      // coldot_scratch_doubles(R, Cc, batch)
  double* row_scratch;      // tile_scan_row_scratch_doubles(R, Cc, dtype, batch)
  uint32_t* done;           // SCAN_DONE_WORDS zeroed counters, or null: parts that can then finish by themselves
  const int32_t* gate;
  int64_t gate_stride;
  int gate_value;
};
bool tile_scan_ok(const TileScanJob& t);     // 16-byte aligned rows, Cc a multiple of the vector width
size_t tile_scan_row_scratch_doubles(int R, int Cc, int dtype, int batch);
// launches the first stage and describes in *pending what is left of the second (valid = false: nothing)
hipError_t launch_tile_scan(const TileScanJob& t, Stage2Job* pending, hipStream_t st);

// The two gated re-encodings of the operand audit in one launch.  kind: 0 rowdot (s), 1 coldot (s),
// 2 tile scan with one part on (t); index weights, same gate.  Every column reduction has to be able
// to finish by itself (audit_pair_ok says whether); done: SCAN_DONE_WORDS zeroed counters.
struct ScanPairItem { int kind; ScanArgs s; TileScanJob t; };
bool audit_pair_ok(const ScanPairItem& x0, const ScanPairItem& x1);
hipError_t launch_audit_pair(const ScanPairItem& x0, const ScanPairItem& x1, uint32_t* done, hipStream_t st);

// ---- product (gemm_kernels.hip) ------------------------------------------------------------
struct GemmArgs {
  const void* A;
  const void* B;
  float* C;
  int dtype, trans_a, trans_b;
  int n, k, m, batch;
  int64_t lda, ldb, ldc, sa, sb, sc;
  float* rowpart;       // null = no syndrome epilogue (plain product)
  float* colpart;
  int tile_m, tile_n, ntm, ntn;
  int rp_ld, cp_ld;     // lines per sub-tile slab of rowpart / colpart (n, m plus padding)
  const gecc_fault* faults;
  int n_faults;
  int fault_bias;       // a fault strikes batch item b when its `batch` field equals b + fault_bias
                        // (the per-panel call uses that field for the panel number)
  int cu_hint;          // compute units to plan the rounds of tiles for (0: ask the device)
  int split_first;      // set by the launcher of the bf16 256 x 256 kernel: first workgroup of the
                        // k-split tail (-1: none)
  int map_sr, map_sc;   // set by the same launcher: a round of 256 workgroups takes a block of
                        // map_sr x map_sc tiles (0: the default order)
  // 128 x 128-tile kernel only: ksplit workgroups share a tile, one per range of k (products with far
  // fewer tiles than compute units); the last to finish adds their partial tiles up in a fixed order
  int ksplit;           // 0 or 1: off
  int k_per;            // set by the launcher: k range of one workgroup
  float* split_part;    // [tiles x batch][ksplit][128 x 128]
  uint32_t* split_done; // [tiles x batch] counters, zero between launches (shared with the scans)
  // protected product only: P_g = A_P B_P goes to pg_out[b * pg_stride + 0..3], formed by the
  // workgroup of the first tile, which also resets the decoder state of its batch item
  const double* A_par;
  const double* B_par;
  double* pg_out;
  int64_t pg_stride;
  DecodeState* state;
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t st);

#if defined(__HIPCC__)
// "Last workgroup finishes" without cache flushes.  Results that another workgroup of the same launch
// will read are stored with store_dev (written through to device-coherent memory) and read with
// load_dev (never served from a cache that another compute die cannot see).  A device-wide fence
// would do as well, but it writes back and invalidates a whole L2, and one per workgroup multiplies
// the duration of a scan.
template <class T> static __device__ __forceinline__ void store_dev(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T> static __device__ __forceinline__ T load_dev(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Every thread of the workgroup has issued its store_dev()s; true in the workgroup that is the last
// of `count` to get here (its load_dev()s then see the stores of all the others).  The counter wraps
// to zero with the last arrival.  flag: an int of LDS that nobody else uses between the two barriers.
static __device__ __forceinline__ bool arrive_last(uint32_t* counter, uint32_t count, int* flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wavefront's stores have been written through
  __syncthreads();
  if (threadIdx.x == 0) *flag = atomicInc(counter, count - 1) == count - 1;
  __syncthreads();
  return *flag != 0;
}

// counters, phase and error list of one batch item, as before any verification
static __device__ __forceinline__ void reset_state(DecodeState* s) {
  s->s_cnt = 0; s->t_cnt = 0;
  s->nonfinite = 0;
  s->phase = PH_DONE;
  s->n_err = 0;
}

// Global parity block P_g = A_P B_P (Section III, 2 x 2) of batch item b, in fp64 and in a fixed
// order; thread 0 also resets the item's decoder state.  Called by every thread of one
// workgroup of at most 256 threads, after its last use of the 16 doubles at `lds`.
static __device__ __forceinline__ void form_pg(const GemmArgs& a, int b, double* lds) {
  const double* ap = a.A_par + (int64_t)b * 2 * a.k;
  const double* bp = a.B_par + (int64_t)b * 2 * a.k;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  for (int l = threadIdx.x; l < a.k; l += blockDim.x) {
    const double a0 = ap[l], a1 = ap[a.k + l], b0 = bp[l], b1 = bp[a.k + l];
    acc[0] = fma(a0, b0, acc[0]); acc[1] = fma(a0, b1, acc[1]);
    acc[2] = fma(a1, b0, acc[2]); acc[3] = fma(a1, b1, acc[3]);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc[q] += __shfl_down(acc[q], off, 64);
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0)
#pragma unroll
    for (int q = 0; q < 4; ++q) lds[wave * 4 + q] = acc[q];
  __syncthreads();
  if (threadIdx.x < 4) {
    double v = lds[threadIdx.x];
    for (int w = 1; w < nw; ++w) v += lds[w * 4 + threadIdx.x];
    a.pg_out[(int64_t)b * a.pg_stride + threadIdx.x] = v;
  }
  if (threadIdx.x == 0 && a.state) reset_state(a.state + b);
}
#endif
// 256 x 256-tile bf16 kernel for aligned operands (gemm_bf16_kernels.hip)
bool gemm_bf16_fast_ok(const GemmArgs& a);
hipError_t launch_gemm_bf16_fast(const GemmArgs& a, hipStream_t st);

// stand-alone syndrome partials from a C in HBM (same workspace layout as the fused epilogue)
struct PartialArgs {
  const float* C;
  int n, m, batch;
  int64_t ldc, sc;
  float* rowpart;
  float* colpart;
  int tile_m, tile_n, ntm, ntn;
  int rp_ld, cp_ld;
  const int32_t* gate;
  int64_t gate_stride;
  int gate_value;
};
hipError_t launch_partials(const PartialArgs& a, hipStream_t st);
// C += P (both n x m fp32, leading dimension ldc): the sum of per-panel partial products
hipError_t launch_accumulate(float* C, const float* P, int n, int m, int64_t ldc, hipStream_t st);

// ---- decoder (decode_kernels.hip) ----------------------------------------------------------
struct DecodeArgs {
  gecc_params p;
  int tile_m, tile_n, ntm, ntn;
  int rp_ld, cp_ld;
  void* A;
  void* B;
  float* C;
  const double* A_par;
  const double* B_par;
  double* C_par;
  const float* rowpart;
  const float* colpart;
  double* synd;
  double* allow;
  DecodeState* state;
  const double* audit_a;
  const double* audit_b;
  double* blockmax;     // [batch][nblk][4] family maxima per workgroup of the first threshold pass
  int nblk;             // (blocked mode: [items][4], nblk = 1, kept as bit patterns for atomicMax)
  gecc_report* report;
  // Item addressing.  An item is a batch item (nbj = 0: I = J = b) or a block of the blocked code
  // (I = b / nbj, J = b % nbj; p.n, p.m are then the block sizes and p.batch the number of blocks).
  // A and A_par go by I, B and B_par by J, C by both; everything else by b.
  int nbj;
  int64_t ia_stride, jb_stride, ic_stride, jc_stride;   // elements
  int32_t* gate_word;   // blocked mode: set to PH_AUDIT by the first block that needs the operand audit
};
// P_r, P_c, P_g of every block from the side products (blocked mode), plus the per-item resets
struct BlockedParityArgs {
  int nb, mb, k, nbi, nbj, pieces;
  const float* side_r; int64_t ld_r;     // n x (2 pieces nbj)
  const float* side_c; int64_t ld_c;     // (2 pieces nbi) x m
  const double* A_par; const double* B_par;
  double* C_par;
  DecodeState* state;
  double* itemmax;
  int32_t* gate_word;
};
hipError_t launch_blocked_parities(const BlockedParityArgs& a, hipStream_t st);
// fp64 parities [lines][2][k] -> operand-type rows [(line * 2 + t) * pieces + s][k] (k contiguous)
hipError_t launch_split_parities(const double* par, void* W, int dtype, int lines, int k, int pieces, int rows_padded, hipStream_t st);
// blocked mode: per-block syndromes and flags from the sub-tile partial sums
hipError_t launch_threshold_blocked(const DecodeArgs& a, int n_full, int m_full, hipStream_t st);
// blocked mode: the repair in three launches (own block of C-bar; operands; Section V on the rest)
hipError_t launch_repair_blocked(const DecodeArgs& a, int nbi, hipStream_t st);
hipError_t launch_reset_state(const DecodeArgs& a, hipStream_t st);
// partial sums -> syndromes -> threshold flags (Section V step 1) and max |syndrome| per family
hipError_t launch_threshold(const DecodeArgs& a, hipStream_t st);
// first report (s, t, maxima, CLEAN / DETECTED) from the counters of the first threshold pass
hipError_t launch_summarize(const DecodeArgs& a, hipStream_t st);
// Section V step 2 right after detection.  with_summary = 1: also writes the first report
hipError_t launch_decode_c(const DecodeArgs& a, int with_summary, hipStream_t st);
// audit differences, operand patches, rank-one repair of C-bar and of the syndromes, Section V on the rest
hipError_t launch_repair(const DecodeArgs& a, hipStream_t st);

}  // namespace gecc
