// C ABI of libgecc: argument checking, workspace layout and the stream-ordered launch
// sequences.  Host code only; all arithmetic of the path runs in the kernels.
#include <cstdlib>
#include <mutex>
#include <new>
#include "gecc_internal.h"

using namespace gecc;

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

size_t elem_size(int dtype) { return dtype == GECC_BF16 ? 2 : 4; }

bool blocked(const gecc_ctx* c) { return c->nbi > 0; }
int items_of(const gecc_ctx* c) { return blocked(c) ? c->nbi * c->nbj : c->p.batch; }

void make_layout(gecc_ctx* c) {
  const gecc_params& p = c->p;
  const size_t b = p.batch, n = p.n, k = p.k, m = p.m;
  const size_t ni = blocked(c) ? c->nbi : 1, nj = blocked(c) ? c->nbj : 1;   // (blocked mode has batch 1)
  Layout& L = c->lay;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  L.done = take(SCAN_DONE_WORDS * sizeof(uint32_t));
  L.rowpart = take(b * c->ntn * (size_t)c->rp_ld * 2 * sizeof(float));
  L.colpart = take(b * c->ntm * (size_t)c->cp_ld * 2 * sizeof(float));
  // (blocked mode: one record per block, nj * 2n + ni * 2m doubles in all; audits per operand line)
  L.synd = take(b * (nj * 2 * n + ni * 2 * m) * sizeof(double));
  L.allow = take(b * (nj * 2 * n + ni * 2 * m) * sizeof(double));
  L.state = take(b * ni * nj * sizeof(DecodeState));
  L.audit_a = take(b * ni * 2 * k * sizeof(double));
  L.audit_b = take(b * nj * 2 * k * sizeof(double));
  L.blockmax = take(b * (((n + m + 63) / 64) + ni * nj) * 4 * sizeof(double));
  // column reductions: A side reduces over n (A stored n x k) or over k (P_r with A stored
  // k x n); B side over k (P_c with B stored k x m) or over m (B stored m x k)
  const size_t sa = p.trans_a ? coldot_scratch_doubles(p.k, p.n, p.batch)
                              : coldot_scratch_doubles(p.n, p.k, p.batch);
  const size_t sb = p.trans_b ? coldot_scratch_doubles(p.m, p.k, p.batch)
                              : coldot_scratch_doubles(p.k, p.m, p.batch);
  L.scan_a = take(sa * sizeof(double));
  L.scan_b = take(sb * sizeof(double));
  // the operand that gets the one-pass tile scan, as stored: rows x contiguous columns
  const size_t ra = tile_scan_row_scratch_doubles(p.trans_a ? p.k : p.n, p.trans_a ? p.n : p.k, p.dtype, p.batch);
  const size_t rb = tile_scan_row_scratch_doubles(p.trans_b ? p.m : p.k, p.trans_b ? p.k : p.m, p.dtype, p.batch);
  L.scan_row = take((ra > rb ? ra : rb) * sizeof(double));
  L.ksplit = take(c->ksplit > 1 ? b * c->ntm * c->ntn * (size_t)c->ksplit * 128 * 128 * sizeof(float) : 0);
  L.w_a = L.w_b = L.side_r = L.side_c = L.gate = 0;
  if (blocked(c)) {
    const size_t esz = p.dtype == GECC_BF16 ? 2 : 4;
    L.w_a = take((size_t)c->w_cols_a * k * esz);
    L.w_b = take((size_t)c->w_cols_b * k * esz);
    L.side_r = take(n * (size_t)c->w_cols_b * sizeof(float));
    L.side_c = take((size_t)c->w_cols_a * m * sizeof(float));
    L.gate = take(256);
  }
  L.total = off;
}

int check_ws(const gecc_ctx* c) {
  if (!c) return GECC_ERR_ARG;
  if (!c->ws || c->ws_bytes < c->lay.total) return GECC_ERR_WORKSPACE;
  return GECC_OK;
}

int hip_rc(hipError_t e) { return e == hipSuccess ? GECC_OK : GECC_ERR_HIP; }

// The counters at the front of the workspace have to start at zero: done once per attached
// workspace, on the stream of the first call that launches scans.
int prep(gecc_ctx* c, hipStream_t st) {
  if (c->ws_zeroed == c->ws) return GECC_OK;
  if (launch_zero_words(reinterpret_cast<uint32_t*>(c->ws + c->lay.done), SCAN_DONE_WORDS, st) != hipSuccess)
    return GECC_ERR_HIP;
  c->ws_zeroed = c->ws;
  return GECC_OK;
}

// operands need only their natural alignment; 16-byte aligned rows get the vector paths
bool aligned_to(const void* p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

DecodeArgs decode_args(gecc_ctx* c, void* A, const double* A_par, void* B, const double* B_par,
                       float* C, double* C_par, gecc_report* rep) {
  DecodeArgs d;
  d.p = c->p;
  d.tile_m = c->tile_m; d.tile_n = c->tile_n; d.ntm = c->ntm; d.ntn = c->ntn;
  d.rp_ld = c->rp_ld; d.cp_ld = c->cp_ld;
  d.A = A; d.B = B; d.C = C;
  d.A_par = A_par; d.B_par = B_par; d.C_par = C_par;
  d.rowpart = reinterpret_cast<float*>(c->ws + c->lay.rowpart);
  d.colpart = reinterpret_cast<float*>(c->ws + c->lay.colpart);
  d.synd = reinterpret_cast<double*>(c->ws + c->lay.synd);
  d.allow = reinterpret_cast<double*>(c->ws + c->lay.allow);
  d.state = reinterpret_cast<DecodeState*>(c->ws + c->lay.state);
  d.blockmax = reinterpret_cast<double*>(c->ws + c->lay.blockmax);
  d.nblk = (c->p.n + c->p.m + 63) / 64;
  d.audit_a = reinterpret_cast<double*>(c->ws + c->lay.audit_a);
  d.audit_b = reinterpret_cast<double*>(c->ws + c->lay.audit_b);
  d.report = rep;
  d.nbj = 0;
  d.ia_stride = c->p.stride_a; d.jb_stride = c->p.stride_b; d.ic_stride = c->p.stride_c; d.jc_stride = 0;
  d.gate_word = nullptr;
  if (blocked(c)) {
    // the decoder sees every block as an item of its own: n, m are the block sizes
    const gecc_params& p = c->p;
    d.p.n = p.block_n; d.p.m = p.block_m; d.p.batch = c->nbi * c->nbj;
    d.nbj = c->nbj;
    d.ia_stride = p.trans_a ? (int64_t)p.block_n : (int64_t)p.block_n * p.lda;
    d.jb_stride = p.trans_b ? (int64_t)p.block_m * p.ldb : (int64_t)p.block_m;
    d.ic_stride = (int64_t)p.block_n * p.ldc; d.jc_stride = p.block_m;
    d.nblk = 1;
    d.blockmax += (size_t)((p.n + p.m + 63) / 64) * 4;     // the per-block maxima live behind the per-workgroup ones
    d.gate_word = reinterpret_cast<int32_t*>(c->ws + c->lay.gate);
  }
  return d;
}

// Blocked mode: the row blocks of A (column blocks of B) as batch items of the scans -- a copy of
// the context whose n (m) is the block size, whose batch is the number of blocks and whose batch
// stride walks from block to block.  Both views use the tile scan for their operand (encoding and
// audit alike) where it applies.
gecc_ctx view_a(const gecc_ctx* c) {
  gecc_ctx v = *c;
  v.p.n = c->p.block_n; v.p.batch = c->nbi;
  v.p.stride_a = c->p.trans_a ? (int64_t)c->p.block_n : (int64_t)c->p.block_n * c->p.lda;
  v.nbi = v.nbj = 0; v.tile_op = GECC_MAT_A;
  return v;
}
gecc_ctx view_b(const gecc_ctx* c) {
  gecc_ctx v = *c;
  v.p.m = c->p.block_m; v.p.batch = c->nbj;
  v.p.stride_b = c->p.trans_b ? (int64_t)c->p.block_m * c->p.ldb : (int64_t)c->p.block_m;
  v.nbi = v.nbj = 0; v.tile_op = GECC_MAT_B;
  return v;
}

ScanArgs scan_base(const gecc_ctx* c, const void* X, int64_t ld, int64_t xs) {
  ScanArgs s{};
  s.X = X; s.dtype = c->p.dtype; s.ld = ld; s.xs = xs; s.batch = c->p.batch;
  s.gate = nullptr; s.gate_stride = 0; s.gate_value = 0;
  return s;
}

// The four scans of the path.  Each operand is reduced once along its contiguous index (rowdot:
// one launch) and once along the other (coldot: two stages), whichever way it is stored.
struct ScanJob {
  ScanArgs s;
  bool rowdot;
  int kind;   // GECC_K_x, for the timing records
};

// Brackets the launches between its construction and done() with a timing record, when the
// context records launches of that class.
struct Timed {
  gecc_ctx* c;
  hipStream_t st;
  int kind;
  bool on;
  hipError_t err;
  Timed(gecc_ctx* ctx, int k, hipStream_t s) : c(ctx), st(s), kind(k), err(hipSuccess) {
    on = c->ev && ((c->ev_mask >> k) & 1u) && c->ev_n < c->ev_cap;
    if (on) err = hipEventRecord(c->ev[2 * c->ev_n], st);
  }
  hipError_t done(hipError_t launch_result) {
    if (launch_result != hipSuccess) return launch_result;
    if (err != hipSuccess) return err;
    if (on) {
      if ((err = hipEventRecord(c->ev[2 * c->ev_n + 1], st)) != hipSuccess) return err;
      c->ev_kind[c->ev_n] = kind;
      ++c->ev_n;
    }
    return hipSuccess;
  }
};

// reduce A over its row index i (length n) -> [2][k]; w = null: Section III's index weights
ScanJob scan_a_over_n(gecc_ctx* c, const void* A, const double* w, double* out, const int32_t* gate) {
  const gecc_params& p = c->p;
  ScanJob j{scan_base(c, A, p.lda, p.stride_a), p.trans_a != 0, gate ? GECC_K_AUDIT_A : GECC_K_ENCODE_A};
  ScanArgs& s = j.s;
  s.w = w; s.out = out; s.w_stride = 2 * (int64_t)p.n; s.out_stride = 2 * (int64_t)p.k;
  if (gate) { s.gate = gate; s.gate_stride = sizeof(DecodeState); s.gate_value = PH_AUDIT; }
  if (p.trans_a) { s.R = p.k; s.Cc = p.n; }   // stored k x n
  else { s.R = p.n; s.Cc = p.k; s.scratch = reinterpret_cast<double*>(c->ws + c->lay.scan_a); }
  return j;
}
// reduce A over its column index l (length k) -> [2][n]
ScanJob scan_a_over_k(gecc_ctx* c, const void* A, const double* w, double* out, int64_t out_stride) {
  const gecc_params& p = c->p;
  ScanJob j{scan_base(c, A, p.lda, p.stride_a), p.trans_a == 0, GECC_K_PARITY_R};
  ScanArgs& s = j.s;
  s.w = w; s.out = out; s.w_stride = 2 * (int64_t)p.k; s.out_stride = out_stride;
  if (p.trans_a) { s.R = p.k; s.Cc = p.n; s.scratch = reinterpret_cast<double*>(c->ws + c->lay.scan_a); }
  else { s.R = p.n; s.Cc = p.k; }
  return j;
}
// reduce B over its column index j (length m) -> [2][k]
ScanJob scan_b_over_m(gecc_ctx* c, const void* B, const double* w, double* out, const int32_t* gate) {
  const gecc_params& p = c->p;
  ScanJob j{scan_base(c, B, p.ldb, p.stride_b), p.trans_b == 0, gate ? GECC_K_AUDIT_B : GECC_K_ENCODE_B};
  ScanArgs& s = j.s;
  s.w = w; s.out = out; s.w_stride = 2 * (int64_t)p.m; s.out_stride = 2 * (int64_t)p.k;
  if (gate) { s.gate = gate; s.gate_stride = sizeof(DecodeState); s.gate_value = PH_AUDIT; }
  if (p.trans_b) { s.R = p.m; s.Cc = p.k; s.scratch = reinterpret_cast<double*>(c->ws + c->lay.scan_b); }   // stored m x k
  else { s.R = p.k; s.Cc = p.m; }
  return j;
}
// reduce B over its row index l (length k) -> [2][m]
ScanJob scan_b_over_k(gecc_ctx* c, const void* B, const double* w, double* out, int64_t out_stride) {
  const gecc_params& p = c->p;
  ScanJob j{scan_base(c, B, p.ldb, p.stride_b), p.trans_b != 0, GECC_K_PARITY_C};
  ScanArgs& s = j.s;
  s.w = w; s.out = out; s.w_stride = 2 * (int64_t)p.k; s.out_stride = out_stride;
  if (p.trans_b) { s.R = p.m; s.Cc = p.k; }
  else { s.R = p.k; s.Cc = p.m; s.scratch = reinterpret_cast<double*>(c->ws + c->lay.scan_b); }
  return j;
}

// The tile scan of operand `op` (as stored: rows x contiguous columns).  enc_out: where the
// index-weighted reduction of Section III goes (A_P or B_P, or an audit buffer), or null;
// par_w / par_out: weights and destination of the parity block of C-bar along the other axis
// (P_r = A B_P or P_c = A_P B), or null.
TileScanJob tile_job(gecc_ctx* c, int op, const void* X, double* enc_out, const double* par_w, double* par_out,
                     int64_t par_out_stride, const int32_t* gate) {
  const gecc_params& p = c->p;
  const bool is_a = op == GECC_MAT_A;
  const bool tr = is_a ? p.trans_a != 0 : p.trans_b != 0;
  TileScanJob t{};
  t.X = X; t.dtype = p.dtype; t.batch = p.batch;
  t.ld = is_a ? p.lda : p.ldb;
  t.xs = is_a ? p.stride_a : p.stride_b;
  const int len = is_a ? p.n : p.m;                 // the axis the encoding sums over
  t.R = is_a ? (tr ? p.k : p.n) : (tr ? p.m : p.k);
  t.Cc = is_a ? (tr ? p.n : p.k) : (tr ? p.k : p.m);
  (void)len;
  // A stored n x k and B stored m x k keep the encoded axis in the rows: column part.  The other
  // two layouts keep it in the columns: row part.
  const bool enc_is_col = is_a ? !tr : tr;
  t.col_scratch = reinterpret_cast<double*>(c->ws + (is_a ? c->lay.scan_a : c->lay.scan_b));
  t.row_scratch = reinterpret_cast<double*>(c->ws + c->lay.scan_row);
  const int64_t k2 = 2 * (int64_t)p.k;
  if (enc_out) {
    if (enc_is_col) { t.col_on = true; t.wr = nullptr; t.col_out = enc_out; t.col_out_stride = k2; }
    else            { t.row_on = true; t.wc = nullptr; t.row_out = enc_out; t.row_out_stride = k2; }
  }
  if (par_w) {
    if (enc_is_col) { t.row_on = true; t.wc = par_w; t.wc_stride = k2; t.row_out = par_out; t.row_out_stride = par_out_stride; }
    else            { t.col_on = true; t.wr = par_w; t.wr_stride = k2; t.col_out = par_out; t.col_out_stride = par_out_stride; }
  }
  if (gate) { t.gate = gate; t.gate_stride = sizeof(DecodeState); t.gate_value = PH_AUDIT; }
  return t;
}

// Whether the tile scan serves this operand: its rows have to allow it, and the operand has to be
// large enough for one pass to beat two (small operands are bound by the number of dependent
// launches, and the two separate scans need one launch less: a row scan carries the second stage
// of a column scan).  A function of shape and alignment alone, so that an encoding and the audit
// that re-forms it always take the same kernel.
bool use_tile(const gecc_ctx* c, const TileScanJob& t) {
  return tile_scan_ok(t) && (int64_t)t.R * t.Cc * t.batch >= c->tile_min;
}

// Scans in stream order.  The second stage of a coldot is held back: the next rowdot carries it in
// the same launch unless it reads that stage's output (or is gated differently); anything else
// flushes it first.  The caller flushes before the results are needed.
struct ScanQueue {
  gecc_ctx* c;
  hipStream_t st;
  Stage2Job pending{};
  uint32_t* done() const { return reinterpret_cast<uint32_t*>(c->ws + c->lay.done); }
  hipError_t flush() {
    if (!pending.valid) return hipSuccess;
    pending.valid = false;
    Timed t(c, GECC_K_STAGE2, st);
    return t.done(launch_stage2(pending, st));
  }
  hipError_t run(const ScanJob& j) {
    hipError_t e;
    const ScanArgs& s = j.s;
    const bool reads_pending = s.w != nullptr && (s.w == pending.out || s.w == pending.row_out);
    const bool can_carry = j.rowdot && pending.valid && !reads_pending && s.batch == pending.batch &&
                           s.gate == pending.gate && s.gate_stride == pending.gate_stride &&
                           s.gate_value == pending.gate_value;
    if (pending.valid && !can_carry && (e = flush()) != hipSuccess) return e;
    Timed t(c, j.kind, st);
    if (j.rowdot) {
      e = launch_rowdot(s, can_carry ? &pending : nullptr, st);
      pending.valid = false;
      return t.done(e);
    }
    // (a gated column scan finishes by itself where it can: the audits then need no launch for it)
    ScanArgs f = s;
    if (s.gate && coldot_done_words(f) > 0) f.done = done();
    return t.done(launch_coldot_stage1(f, &pending, st));
  }
  // a tile scan: what is left of its second stage becomes the pending one
  hipError_t run_tile(const TileScanJob& tj, int kind) {
    hipError_t e;
    if (pending.valid && (e = flush()) != hipSuccess) return e;
    TileScanJob f = tj;
    if (tj.gate) f.done = done();
    Timed t(c, kind, st);
    return t.done(launch_tile_scan(f, &pending, st));
  }
  // both gated audits in one launch, where every column reduction among them can finish by itself
  hipError_t run_audit_pair(const ScanPairItem& x0, const ScanPairItem& x1) {
    hipError_t e;
    if (pending.valid && (e = flush()) != hipSuccess) return e;
    Timed t(c, GECC_K_AUDIT_AB, st);
    return t.done(launch_audit_pair(x0, x1, done(), st));
  }
};

// P_r = A B_P (n x 2) and P_c = A_P B (2 x m) of C-bar; the coldot of the two goes first so that the
// rowdot can carry its second stage
hipError_t parity_products(gecc_ctx* c, ScanQueue& q, const void* A, const double* A_par, const void* B,
                           const double* B_par, double* C_par) {
  const gecc_params& p = c->p;
  const int64_t rec = 2 * (int64_t)p.n + 2 * (int64_t)p.m + 4;
  const ScanJob pr = scan_a_over_k(c, A, B_par, C_par, rec);
  const ScanJob pc = scan_b_over_k(c, B, A_par, C_par + 2 * (size_t)p.n, rec);
  hipError_t e;
  if (!pc.rowdot && pr.rowdot) {
    if ((e = q.run(pc)) != hipSuccess) return e;
    return q.run(pr);
  }
  if ((e = q.run(pr)) != hipSuccess) return e;
  return q.run(pc);
}

GemmArgs gemm_args(const gecc_ctx* c, const void* A, const void* B, float* C) {
  const gecc_params& p = c->p;
  GemmArgs g{};
  g.A = A; g.B = B; g.C = C;
  g.dtype = p.dtype; g.trans_a = p.trans_a; g.trans_b = p.trans_b;
  g.n = p.n; g.k = p.k; g.m = p.m; g.batch = p.batch;
  g.lda = p.lda; g.ldb = p.ldb; g.ldc = p.ldc;
  g.sa = p.stride_a; g.sb = p.stride_b; g.sc = p.stride_c;
  g.tile_m = c->tile_m; g.tile_n = c->tile_n; g.ntm = c->ntm; g.ntn = c->ntn;
  g.cu_hint = c->cu_hint; g.split_first = -1;
  if (c->ksplit > 1 && c->ws && c->ws_bytes >= c->lay.total) {
    g.ksplit = c->ksplit;
    g.split_part = reinterpret_cast<float*>(c->ws + c->lay.ksplit);
    g.split_done = reinterpret_cast<uint32_t*>(c->ws + c->lay.done);
  }
  g.rp_ld = c->rp_ld; g.cp_ld = c->cp_ld;
  return g;
}

// the product kernel(s), bracketed by a timing record when timing is enabled
hipError_t timed_gemm(gecc_ctx* c, const GemmArgs& g, hipStream_t st) {
  Timed t(c, GECC_K_PRODUCT, st);
  return t.done(launch_gemm(g, st));
}

}  // namespace

extern "C" {

int gecc_create(gecc_ctx** out, const gecc_params* p) {
  if (!out || !p) return GECC_ERR_ARG;
  *out = nullptr;
  if (p->n < 1 || p->k < 1 || p->m < 1 || p->batch < 1) return GECC_ERR_ARG;
  if (p->dtype != GECC_F32 && p->dtype != GECC_BF16) return GECC_ERR_ARG;
  if ((p->trans_a != 0 && p->trans_a != 1) || (p->trans_b != 0 && p->trans_b != 1)) return GECC_ERR_ARG;
  if (p->lda < (p->trans_a ? p->n : p->k)) return GECC_ERR_ARG;
  if (p->ldb < (p->trans_b ? p->k : p->m)) return GECC_ERR_ARG;
  if (p->ldc < p->m) return GECC_ERR_ARG;
  if (p->batch > 1) {
    const int64_t rows_a = p->trans_a ? p->k : p->n, rows_b = p->trans_b ? p->m : p->k;
    if (p->stride_a < rows_a * p->lda || p->stride_b < rows_b * p->ldb ||
        p->stride_c < (int64_t)p->n * p->ldc)
      return GECC_ERR_ARG;
  }
  if (!(p->tau_r1 >= 0) || !(p->tau_r2 >= 0) || !(p->tau_q1 >= 0) || !(p->tau_q2 >= 0) ||
      !(p->tau_op >= 0) || !(p->tau_rep >= 0) || !(p->tau_rel >= 0))
    return GECC_ERR_ARG;
  if (p->weighted != 0 && p->weighted != 1) return GECC_ERR_ARG;
  if ((p->block_n == 0) != (p->block_m == 0) || p->block_n < 0 || p->block_m < 0) return GECC_ERR_ARG;
  if (p->block_n > 0 && (p->block_n % 128 || p->block_m % 128 || p->n % p->block_n || p->m % p->block_m ||
                         p->batch != 1 || p->weighted != 1))
    return GECC_ERR_ARG;
  if ((int64_t)p->n + p->m > (int64_t)1 << 30) return GECC_ERR_ARG;
  gecc_ctx* c = new (std::nothrow) gecc_ctx;
  if (!c) return GECC_ERR_ARG;
  c->p = *p;
  {
    const char* e = getenv("GECC_CU_COUNT");       // test hook: see GemmArgs::cu_hint
    c->cu_hint = e ? atoi(e) : 0;
    if (c->cu_hint < 0) c->cu_hint = 0;
    const char* t = getenv("GECC_TILE_MIN");       // test hook: operands of that many elements or more take the one-pass scan
    c->tile_min = (t && atoll(t) > 0) ? atoll(t) : ((int64_t)1 << 25);
  }
  // the larger operand is read once for both of its reductions (tile scan), the other one twice
  c->tile_op = p->n >= p->m ? GECC_MAT_A : GECC_MAT_B;
  c->nbi = p->block_n > 0 ? p->n / p->block_n : 0;
  c->nbj = p->block_n > 0 ? p->m / p->block_m : 0;
  c->pieces = p->dtype == GECC_BF16 ? 3 : 1;
  c->w_cols_a = (2 * c->pieces * c->nbi + 7) / 8 * 8;
  c->w_cols_b = (2 * c->pieces * c->nbj + 7) / 8 * 8;
  c->tile_m = 128;
  c->tile_n = 128;
  c->ntm = (p->n + c->tile_m - 1) / c->tile_m;
  c->ntn = (p->m + c->tile_n - 1) / c->tile_n;
  {
    // products with far fewer tiles than compute units split k over several workgroups per tile
    // (128 x 128-tile kernel only; every range keeps at least 128 terms)
    const int64_t tiles = (int64_t)c->ntm * c->ntn * p->batch;
    int s = tiles * 2 <= 256 ? (int)(256 / tiles) : 1;
    if (s > 8) s = 8;
    while (s > 1 && p->k / s < 128) --s;
    c->ksplit = p->block_n > 0 ? 1 : s;
  }
  // slab strides of the partial sums: a multiple of 2 KiB would put the same line of every slab
  // into the same memory channel
  c->rp_ld = p->n % 256 == 0 ? p->n + 16 : p->n;
  c->cp_ld = p->m % 256 == 0 ? p->m + 16 : p->m;
  c->ws = nullptr;
  c->ws_bytes = 0;
  c->ws_zeroed = nullptr;
  c->panel = nullptr;
  c->n_panel = 0;
  c->fault_bias = 0;
  c->ev = nullptr;
  c->ev_kind = nullptr;
  c->ev_mask = 0;
  c->ev_cap = 0;
  c->ev_n = 0;
  make_layout(c);
  *out = c;
  return GECC_OK;
}

namespace {
void drop_panels(gecc_ctx* ctx) {
  for (int g = 0; g < ctx->n_panel; ++g) delete ctx->panel[g];
  delete[] ctx->panel;
  ctx->panel = nullptr;
  ctx->n_panel = 0;
}
}  // namespace

void gecc_destroy(gecc_ctx* ctx) {
  if (!ctx) return;
  drop_panels(ctx);
  gecc_timing_enable(ctx, 0, 0);
  delete ctx;
}

int gecc_timing_enable(gecc_ctx* ctx, int32_t max_records, uint32_t kinds_mask) {
  if (!ctx || max_records < 0) return GECC_ERR_ARG;
  for (int i = 0; i < 2 * ctx->ev_cap; ++i) (void)hipEventDestroy(ctx->ev[i]);
  delete[] ctx->ev;
  delete[] ctx->ev_kind;
  ctx->ev = nullptr;
  ctx->ev_kind = nullptr;
  ctx->ev_cap = 0;
  ctx->ev_n = 0;
  ctx->ev_mask = 0;
  if (max_records == 0) return GECC_OK;
  ctx->ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_records];
  ctx->ev_kind = new (std::nothrow) int32_t[(size_t)max_records];
  if (!ctx->ev || !ctx->ev_kind) {
    delete[] ctx->ev; delete[] ctx->ev_kind;
    ctx->ev = nullptr; ctx->ev_kind = nullptr;
    return GECC_ERR_ARG;
  }
  for (int i = 0; i < 2 * max_records; ++i)
    if (hipEventCreate(&ctx->ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(ctx->ev[j]);
      delete[] ctx->ev; delete[] ctx->ev_kind;
      ctx->ev = nullptr; ctx->ev_kind = nullptr;
      return GECC_ERR_HIP;
    }
  ctx->ev_cap = max_records;
  ctx->ev_mask = kinds_mask;
  return GECC_OK;
}

int gecc_timing_read(gecc_ctx* ctx, float* host_ms, int32_t* host_kind, int32_t cap, int32_t* count) {
  if (!ctx || !host_ms || !count || cap < 0) return GECC_ERR_ARG;
  const int n = ctx->ev_n < cap ? ctx->ev_n : cap;
  for (int i = 0; i < n; ++i) {
    if (hipEventSynchronize(ctx->ev[2 * i + 1]) != hipSuccess) return GECC_ERR_HIP;
    if (hipEventElapsedTime(&host_ms[i], ctx->ev[2 * i], ctx->ev[2 * i + 1]) != hipSuccess) return GECC_ERR_HIP;
    if (host_kind) host_kind[i] = ctx->ev_kind[i];
  }
  *count = n;
  ctx->ev_n = 0;
  return GECC_OK;
}

size_t gecc_workspace_bytes(const gecc_ctx* ctx) { return ctx ? ctx->lay.total : 0; }

int gecc_set_workspace(gecc_ctx* ctx, void* dev_workspace, size_t bytes) {
  if (!ctx || !dev_workspace) return GECC_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(dev_workspace) % 256) return GECC_ERR_ALIGN;
  if (bytes < ctx->lay.total) return GECC_ERR_WORKSPACE;
  ctx->ws = static_cast<char*>(dev_workspace);
  ctx->ws_bytes = bytes;
  ctx->ws_zeroed = nullptr;     // its counters are zeroed by the first call that launches something
  return GECC_OK;
}

size_t gecc_a_par_len(const gecc_ctx* ctx) {
  return ctx ? 2 * (size_t)ctx->p.k * (blocked(ctx) ? ctx->nbi : 1) : 0;
}
size_t gecc_b_par_len(const gecc_ctx* ctx) {
  return ctx ? 2 * (size_t)ctx->p.k * (blocked(ctx) ? ctx->nbj : 1) : 0;
}
size_t gecc_c_par_len(const gecc_ctx* ctx) {
  if (!ctx) return 0;
  if (blocked(ctx)) return (size_t)ctx->nbi * ctx->nbj * (2 * (size_t)ctx->p.block_n + 2 * (size_t)ctx->p.block_m + 4);
  return 2 * (size_t)ctx->p.n + 2 * (size_t)ctx->p.m + 4;
}
int32_t gecc_item_count(const gecc_ctx* ctx) { return ctx ? items_of(ctx) : 0; }

int gecc_encode_a(gecc_ctx* ctx, const void* dev_A, double* dev_A_par, void* stream) {
  int rc = check_ws(ctx);
  if (rc) return rc;
  if (!dev_A || !dev_A_par) return GECC_ERR_ARG;
  if (!aligned_to(dev_A, elem_size(ctx->p.dtype)) || !aligned_to(dev_A_par, 8)) return GECC_ERR_ALIGN;
  if ((rc = prep(ctx, (hipStream_t)stream))) return rc;
  if (blocked(ctx)) {
    gecc_ctx v = view_a(ctx);
    const int rc2 = gecc_encode_a(&v, dev_A, dev_A_par, stream);
    ctx->ev_n = v.ev_n;
    return rc2;
  }
  ScanQueue q{ctx, (hipStream_t)stream};
  const TileScanJob tj = tile_job(ctx, GECC_MAT_A, dev_A, dev_A_par, nullptr, nullptr, 0, nullptr);
  hipError_t e = ctx->tile_op == GECC_MAT_A && use_tile(ctx, tj) ? q.run_tile(tj, GECC_K_ENCODE_A)
                                                                : q.run(scan_a_over_n(ctx, dev_A, nullptr, dev_A_par, nullptr));
  return hip_rc(e != hipSuccess ? e : q.flush());
}

int gecc_encode_b(gecc_ctx* ctx, const void* dev_B, double* dev_B_par, void* stream) {
  int rc = check_ws(ctx);
  if (rc) return rc;
  if (!dev_B || !dev_B_par) return GECC_ERR_ARG;
  if (!aligned_to(dev_B, elem_size(ctx->p.dtype)) || !aligned_to(dev_B_par, 8)) return GECC_ERR_ALIGN;
  if ((rc = prep(ctx, (hipStream_t)stream))) return rc;
  if (blocked(ctx)) {
    gecc_ctx v = view_b(ctx);
    const int rc2 = gecc_encode_b(&v, dev_B, dev_B_par, stream);
    ctx->ev_n = v.ev_n;
    return rc2;
  }
  ScanQueue q{ctx, (hipStream_t)stream};
  const TileScanJob tj = tile_job(ctx, GECC_MAT_B, dev_B, dev_B_par, nullptr, nullptr, 0, nullptr);
  hipError_t e = ctx->tile_op == GECC_MAT_B && use_tile(ctx, tj) ? q.run_tile(tj, GECC_K_ENCODE_B)
                                                                : q.run(scan_b_over_m(ctx, dev_B, nullptr, dev_B_par, nullptr));
  return hip_rc(e != hipSuccess ? e : q.flush());
}

namespace {

int check_multiply_args(gecc_ctx* ctx, const void* dev_A, const double* dev_A_par, const void* dev_B,
                        const double* dev_B_par, float* dev_C, double* dev_C_par, const gecc_fault* dev_faults,
                        int32_t n_faults) {
  int rc = check_ws(ctx);
  if (rc) return rc;
  if (!dev_A || !dev_A_par || !dev_B || !dev_B_par || !dev_C || !dev_C_par) return GECC_ERR_ARG;
  if (n_faults < 0 || n_faults > GECC_MAX_FAULTS || (n_faults > 0 && !dev_faults)) return GECC_ERR_ARG;
  if (!aligned_to(dev_A, elem_size(ctx->p.dtype)) || !aligned_to(dev_B, elem_size(ctx->p.dtype)) ||
      !aligned_to(dev_C, 4) || !aligned_to(dev_C_par, 8) || !aligned_to(dev_A_par, 8) ||
      !aligned_to(dev_B_par, 8))
    return GECC_ERR_ALIGN;
  return GECC_OK;
}

// S3 after the parity products: the data block, the fused syndrome partial sums, P_g
hipError_t product(gecc_ctx* ctx, const void* dev_A, const double* dev_A_par, const void* dev_B,
                   const double* dev_B_par, float* dev_C, double* dev_C_par, const gecc_fault* dev_faults,
                   int32_t n_faults, hipStream_t st) {
  const gecc_params& p = ctx->p;
  GemmArgs g = gemm_args(ctx, dev_A, dev_B, dev_C);
  g.rowpart = reinterpret_cast<float*>(ctx->ws + ctx->lay.rowpart);
  g.colpart = reinterpret_cast<float*>(ctx->ws + ctx->lay.colpart);
  g.faults = dev_faults;
  g.n_faults = n_faults;
  g.fault_bias = ctx->fault_bias;
  // P_g is formed inside the product kernel, which also resets the decoder state for the
  // fused verification that follows
  g.A_par = dev_A_par; g.B_par = dev_B_par;
  g.pg_out = dev_C_par + 2 * (size_t)p.n + 2 * (size_t)p.m;
  g.pg_stride = 2 * (int64_t)p.n + 2 * (int64_t)p.m + 4;
  g.state = reinterpret_cast<DecodeState*>(ctx->ws + ctx->lay.state);
  return timed_gemm(ctx, g, st);
}

// Blocked mode, S3: the parity blocks of every block of C-bar on the matrix units -- the parity
// columns of all column blocks of B-bar, split into operand-type pieces, form one narrow operand
// W_B (and the parity rows of all row blocks of A-bar one flat operand W_A); A W_B^T and W_A B are
// two plain products of the same kernels -- then the data block with the fused partial sums.
hipError_t blocked_multiply(gecc_ctx* ctx, const void* dev_A, const double* dev_A_par, const void* dev_B,
                            const double* dev_B_par, float* dev_C, double* dev_C_par, const gecc_fault* dev_faults,
                            int32_t n_faults, hipStream_t st) {
  const gecc_params& p = ctx->p;
  void* WA = ctx->ws + ctx->lay.w_a;
  void* WB = ctx->ws + ctx->lay.w_b;
  float* side_r = reinterpret_cast<float*>(ctx->ws + ctx->lay.side_r);
  float* side_c = reinterpret_cast<float*>(ctx->ws + ctx->lay.side_c);
  hipError_t e;
  {
    Timed t(ctx, GECC_K_PARITY_R, st);
    if ((e = launch_split_parities(dev_B_par, WB, p.dtype, ctx->nbj, p.k, ctx->pieces, ctx->w_cols_b, st)) != hipSuccess) return e;
    GemmArgs g = gemm_args(ctx, dev_A, WB, side_r);
    g.trans_b = 1; g.m = ctx->w_cols_b; g.ldb = p.k; g.ldc = ctx->w_cols_b;
    g.ntn = (g.m + ctx->tile_n - 1) / ctx->tile_n;
    g.rowpart = nullptr; g.colpart = nullptr; g.faults = nullptr; g.n_faults = 0; g.ksplit = 1;
    if ((e = t.done(launch_gemm(g, st))) != hipSuccess) return e;
  }
  {
    Timed t(ctx, GECC_K_PARITY_C, st);
    if ((e = launch_split_parities(dev_A_par, WA, p.dtype, ctx->nbi, p.k, ctx->pieces, ctx->w_cols_a, st)) != hipSuccess) return e;
    GemmArgs g = gemm_args(ctx, WA, dev_B, side_c);
    g.trans_a = 0; g.n = ctx->w_cols_a; g.lda = p.k; g.ldc = p.m;
    g.ntm = (g.n + ctx->tile_m - 1) / ctx->tile_m;
    g.rowpart = nullptr; g.colpart = nullptr; g.faults = nullptr; g.n_faults = 0; g.ksplit = 1;
    if ((e = t.done(launch_gemm(g, st))) != hipSuccess) return e;
  }
  {
    BlockedParityArgs b{};
    b.nb = p.block_n; b.mb = p.block_m; b.k = p.k; b.nbi = ctx->nbi; b.nbj = ctx->nbj; b.pieces = ctx->pieces;
    b.side_r = side_r; b.ld_r = ctx->w_cols_b; b.side_c = side_c; b.ld_c = p.m;
    b.A_par = dev_A_par; b.B_par = dev_B_par; b.C_par = dev_C_par;
    b.state = reinterpret_cast<DecodeState*>(ctx->ws + ctx->lay.state);
    b.itemmax = reinterpret_cast<double*>(ctx->ws + ctx->lay.blockmax) + (size_t)((p.n + p.m + 63) / 64) * 4;
    b.gate_word = reinterpret_cast<int32_t*>(ctx->ws + ctx->lay.gate);
    Timed t(ctx, GECC_K_DECODE, st);
    if ((e = t.done(launch_blocked_parities(b, st))) != hipSuccess) return e;
  }
  GemmArgs g = gemm_args(ctx, dev_A, dev_B, dev_C);
  g.rowpart = reinterpret_cast<float*>(ctx->ws + ctx->lay.rowpart);
  g.colpart = reinterpret_cast<float*>(ctx->ws + ctx->lay.colpart);
  g.faults = dev_faults;
  g.n_faults = n_faults;
  g.pg_out = nullptr;      // P_g of every block and the resets are done above
  g.state = nullptr;
  return timed_gemm(ctx, g, st);
}

}  // namespace

int gecc_multiply(gecc_ctx* ctx, const void* dev_A, const double* dev_A_par, const void* dev_B,
                  const double* dev_B_par, float* dev_C, double* dev_C_par,
                  const gecc_fault* dev_faults, int32_t n_faults, void* stream) {
  int rc = check_multiply_args(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_faults, n_faults);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = prep(ctx, st))) return rc;
  if (blocked(ctx)) return hip_rc(blocked_multiply(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_faults, n_faults, st));
  ScanQueue q{ctx, st};
  hipError_t e;
  if ((e = parity_products(ctx, q, dev_A, dev_A_par, dev_B, dev_B_par, dev_C_par)) != hipSuccess) return hip_rc(e);
  if ((e = q.flush()) != hipSuccess) return hip_rc(e);
  return hip_rc(product(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_faults, n_faults, st));
}

namespace {

// S4 + S5.  summary = 0 leaves the first report to the decoder's first pass (saves a launch).
int verify_impl(gecc_ctx* ctx, const float* dev_C, const double* dev_C_par, gecc_report* dev_report,
                int32_t fused, int summary, hipStream_t st) {
  DecodeArgs d = decode_args(ctx, nullptr, nullptr, nullptr, nullptr, const_cast<float*>(dev_C),
                             const_cast<double*>(dev_C_par), dev_report);
  hipError_t e;
  if (!fused && blocked(ctx)) return GECC_ERR_ARG;   // (blocked mode verifies from the product's own partial sums)
  if (!fused) {
    // (the fused path had its state reset by gecc_multiply)
    {
      Timed t(ctx, GECC_K_DECODE, st);
      if ((e = t.done(launch_reset_state(d, st))) != hipSuccess) return hip_rc(e);
    }
    const gecc_params& p = ctx->p;
    PartialArgs pa{};
    pa.C = dev_C; pa.n = p.n; pa.m = p.m; pa.batch = p.batch; pa.ldc = p.ldc; pa.sc = p.stride_c;
    pa.rowpart = const_cast<float*>(d.rowpart); pa.colpart = const_cast<float*>(d.colpart);
    pa.tile_m = ctx->tile_m; pa.tile_n = ctx->tile_n; pa.ntm = ctx->ntm; pa.ntn = ctx->ntn;
    pa.rp_ld = ctx->rp_ld; pa.cp_ld = ctx->cp_ld;
    pa.gate = nullptr;
    Timed t(ctx, GECC_K_PARTIALS, st);
    if ((e = t.done(launch_partials(pa, st))) != hipSuccess) return hip_rc(e);
  }
  {
    Timed t(ctx, GECC_K_THRESHOLD, st);
    e = blocked(ctx) ? launch_threshold_blocked(d, ctx->p.n, ctx->p.m, st) : launch_threshold(d, st);
    if ((e = t.done(e)) != hipSuccess) return hip_rc(e);
  }
  if (!summary) return GECC_OK;
  Timed t(ctx, GECC_K_DECODE, st);
  return hip_rc(t.done(launch_summarize(d, st)));
}

// S6 + S7.  with_summary = 1: the first decoder pass also writes the first report.
int correct_impl(gecc_ctx* ctx, void* dev_A, const double* dev_A_par, void* dev_B, const double* dev_B_par,
                 float* dev_C, double* dev_C_par, gecc_report* dev_report, int with_summary, hipStream_t st) {
  DecodeArgs d = decode_args(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_report);
  const int32_t* gate = &d.state->phase;
  hipError_t e;
  // Section V step 2 on the flagged lines; on failure the phase becomes PH_AUDIT
  {
    Timed t(ctx, GECC_K_DECODE, st);
    if ((e = t.done(launch_decode_c(d, with_summary, st))) != hipSuccess) return hip_rc(e);
  }
  if (blocked(ctx)) {
    // the audits of all row blocks of A and all column blocks of B, gated on one word that the
    // first block in need sets; then the repair in three launches (see launch_repair_blocked)
    gecc_ctx va = view_a(ctx), vb = view_b(ctx);
    const int32_t* gw = d.gate_word;
    auto audit = [&](gecc_ctx& v, int op, const void* X, double* out, const ScanJob& old_job, int kind) -> hipError_t {
      ScanQueue qv{&v, st};
      TileScanJob tj = tile_job(&v, op, X, out, nullptr, nullptr, 0, gw);
      tj.gate_stride = 0;
      hipError_t ee;
      if (use_tile(&v, tj)) ee = qv.run_tile(tj, kind);
      else { ScanJob j = old_job; j.s.gate_stride = 0; ee = qv.run(j); }
      if (ee == hipSuccess) { qv.pending.gate_stride = 0; ee = qv.flush(); }
      ctx->ev_n = v.ev_n;
      return ee;
    };
    va.ev_n = ctx->ev_n;
    if ((e = audit(va, GECC_MAT_A, dev_A, const_cast<double*>(d.audit_a),
                   scan_a_over_n(&va, dev_A, nullptr, const_cast<double*>(d.audit_a), gw), GECC_K_AUDIT_A)) != hipSuccess)
      return hip_rc(e);
    vb.ev_n = ctx->ev_n;
    if ((e = audit(vb, GECC_MAT_B, dev_B, const_cast<double*>(d.audit_b),
                   scan_b_over_m(&vb, dev_B, nullptr, const_cast<double*>(d.audit_b), gw), GECC_K_AUDIT_B)) != hipSuccess)
      return hip_rc(e);
    Timed t(ctx, GECC_K_REPAIR, st);
    return hip_rc(t.done(launch_repair_blocked(d, ctx->nbi, st)));
  }
  // operand audit: re-form the parities of A and B as the product read them
  // (the coldot of the two first, so that the rowdot carries its second stage)
  // (an encoding made by the tile scan is re-formed by the tile scan: same sums, same order)
  ScanQueue q{ctx, st};
  const ScanJob ja = scan_a_over_n(ctx, dev_A, nullptr, const_cast<double*>(d.audit_a), gate);
  const ScanJob jb = scan_b_over_m(ctx, dev_B, nullptr, const_cast<double*>(d.audit_b), gate);
  const bool t_is_a = ctx->tile_op == GECC_MAT_A;
  const TileScanJob tj = tile_job(ctx, ctx->tile_op, t_is_a ? dev_A : dev_B,
                                  const_cast<double*>(t_is_a ? d.audit_a : d.audit_b), nullptr, nullptr, 0, gate);
  const bool tile = use_tile(ctx, tj);
  const ScanPairItem xa{tile && t_is_a ? 2 : (ja.rowdot ? 0 : 1), ja.s, tj};
  const ScanPairItem xb{tile && !t_is_a ? 2 : (jb.rowdot ? 0 : 1), jb.s, tj};
  if (audit_pair_ok(xa, xb)) {
    if ((e = q.run_audit_pair(xa, xb)) != hipSuccess) return hip_rc(e);
  } else if (tile) {
    if ((e = q.run_tile(tj, t_is_a ? GECC_K_AUDIT_A : GECC_K_AUDIT_B)) != hipSuccess) return hip_rc(e);
    if ((e = q.run(t_is_a ? jb : ja)) != hipSuccess) return hip_rc(e);
  } else {
    const bool b_first = ja.rowdot && !jb.rowdot;
    if ((e = q.run(b_first ? jb : ja)) != hipSuccess) return hip_rc(e);
    if ((e = q.run(b_first ? ja : jb)) != hipSuccess) return hip_rc(e);
  }
  if ((e = q.flush()) != hipSuccess) return hip_rc(e);
  // parity differences, operand patches, rank-one repair of C-bar with the residual syndromes
  // kept up to date, then Section V once more -- all in one workgroup per batch item
  Timed t(ctx, GECC_K_REPAIR, st);
  return hip_rc(t.done(launch_repair(d, st)));
}

}  // namespace

namespace {

// S1-S3 as one chain of scans.  The order of the four scans depends on how the operands are stored
// (which of them are rowdots) and on what reads what: P_r needs B_P, P_c needs A_P.
int encode_and_multiply(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, double* dev_A_par,
                        double* dev_B_par, double* dev_C_par, const gecc_fault* dev_faults, int32_t n_faults,
                        hipStream_t st) {
  int rc = check_multiply_args(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_faults, n_faults);
  if (rc) return rc;
  if ((rc = prep(ctx, st))) return rc;
  if (blocked(ctx)) {
    if ((rc = gecc_encode_a(ctx, dev_A, dev_A_par, st)) || (rc = gecc_encode_b(ctx, dev_B, dev_B_par, st))) return rc;
    return hip_rc(blocked_multiply(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_faults, n_faults, st));
  }
  const gecc_params& p = ctx->p;
  const int64_t rec = 2 * (int64_t)p.n + 2 * (int64_t)p.m + 4;
  const ScanJob ea = scan_a_over_n(ctx, dev_A, nullptr, dev_A_par, nullptr);
  const ScanJob eb = scan_b_over_m(ctx, dev_B, nullptr, dev_B_par, nullptr);
  const ScanJob pr = scan_a_over_k(ctx, dev_A, dev_B_par, dev_C_par, rec);
  const ScanJob pc = scan_b_over_k(ctx, dev_B, dev_A_par, dev_C_par + 2 * (size_t)p.n, rec);
  ScanQueue q{ctx, st};
  hipError_t e;
  const bool t_is_a = ctx->tile_op == GECC_MAT_A;
  const TileScanJob tj = t_is_a ? tile_job(ctx, GECC_MAT_A, dev_A, dev_A_par, dev_B_par, dev_C_par, rec, nullptr)
                                : tile_job(ctx, GECC_MAT_B, dev_B, dev_B_par, dev_A_par, dev_C_par + 2 * (size_t)p.n, rec, nullptr);
  if (use_tile(ctx, tj)) {
    // the larger operand in one pass: its encoding and its parity block of C-bar together.  That
    // pass reads the other operand's encoding, and the other operand's parity block reads this one's.
    if ((e = q.run(t_is_a ? eb : ea)) != hipSuccess) return hip_rc(e);
    if ((e = q.run_tile(tj, t_is_a ? GECC_K_TILE_A : GECC_K_TILE_B)) != hipSuccess) return hip_rc(e);
    // the other operand's parity block: a row scan over few, long rows (too few workgroups for the
    // row kernel) goes through the tile scan's row part instead
    const ScanJob& po = t_is_a ? pc : pr;
    const TileScanJob to = t_is_a ? tile_job(ctx, GECC_MAT_B, dev_B, nullptr, dev_A_par, dev_C_par + 2 * (size_t)p.n, rec, nullptr)
                                  : tile_job(ctx, GECC_MAT_A, dev_A, nullptr, dev_B_par, dev_C_par, rec, nullptr);
    if (po.rowdot && to.row_on && !to.col_on && po.s.R < 8192 && po.s.Cc >= 4096 && tile_scan_ok(to))
      e = q.run_tile(to, po.kind);
    else
      e = q.run(po);
    if (e != hipSuccess) return hip_rc(e);
  } else {
    // stored:        A n x k, B k x m   A n x k, B m x k   A k x n, B k x m   A k x n, B m x k
    // rowdots:       B_P, P_r           P_r, P_c           A_P, B_P           A_P, P_c
    const ScanJob* order[4];
    if (!p.trans_a) { order[0] = &ea; order[1] = &eb; order[2] = &pc; order[3] = &pr; }
    else if (!p.trans_b) { order[0] = &eb; order[1] = &pr; order[2] = &ea; order[3] = &pc; }
    else { order[0] = &eb; order[1] = &ea; order[2] = &pr; order[3] = &pc; }
    for (int x = 0; x < 4; ++x)
      if ((e = q.run(*order[x])) != hipSuccess) return hip_rc(e);
  }
  if ((e = q.flush()) != hipSuccess) return hip_rc(e);
  return hip_rc(product(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_faults, n_faults, st));
}

}  // namespace

int gecc_verify(gecc_ctx* ctx, const float* dev_C, const double* dev_C_par, gecc_report* dev_report,
                int32_t fused, void* stream) {
  int rc = check_ws(ctx);
  if (rc) return rc;
  if (!dev_C_par || !dev_report || (!fused && !dev_C)) return GECC_ERR_ARG;
  return verify_impl(ctx, dev_C, dev_C_par, dev_report, fused, 1, (hipStream_t)stream);
}

int gecc_correct(gecc_ctx* ctx, void* dev_A, const double* dev_A_par, void* dev_B,
                 const double* dev_B_par, float* dev_C, double* dev_C_par, gecc_report* dev_report,
                 void* stream) {
  int rc = check_ws(ctx);
  if (rc) return rc;
  if (!dev_A || !dev_A_par || !dev_B || !dev_B_par || !dev_C || !dev_C_par || !dev_report)
    return GECC_ERR_ARG;
  if ((rc = prep(ctx, (hipStream_t)stream))) return rc;
  return correct_impl(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_report, 0,
                      (hipStream_t)stream);
}

int gecc_protected_gemm(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, double* dev_A_par,
                        double* dev_B_par, double* dev_C_par, gecc_report* dev_report, void* stream) {
  int rc;
  if (!dev_report) return GECC_ERR_ARG;
  if ((rc = encode_and_multiply(ctx, dev_A, dev_B, dev_C, dev_A_par, dev_B_par, dev_C_par, nullptr, 0,
                                (hipStream_t)stream)))
    return rc;
  if ((rc = verify_impl(ctx, dev_C, dev_C_par, dev_report, 1, 0, (hipStream_t)stream))) return rc;
  return correct_impl(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_report, 1,
                      (hipStream_t)stream);
}

int gecc_protected_gemm_retry(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, double* dev_A_par,
                              double* dev_B_par, double* dev_C_par, gecc_report* dev_report,
                              gecc_report* host_report, int32_t max_retries, const gecc_fault* dev_faults,
                              int32_t n_faults, int32_t* attempts, void* stream) {
  int rc;
  if (!dev_report || !host_report || max_retries < 0) return GECC_ERR_ARG;
  if (attempts) *attempts = 0;
  for (int32_t a = 0; a <= max_retries; ++a) {
    // the planted faults are transient: they strike the first product only
    if (a == 0)
      rc = encode_and_multiply(ctx, dev_A, dev_B, dev_C, dev_A_par, dev_B_par, dev_C_par, dev_faults, n_faults,
                               (hipStream_t)stream);
    else
      rc = gecc_multiply(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, nullptr, 0, stream);
    if (rc) return rc;
    if ((rc = verify_impl(ctx, dev_C, dev_C_par, dev_report, 1, 0, (hipStream_t)stream))) return rc;
    if ((rc = correct_impl(ctx, dev_A, dev_A_par, dev_B, dev_B_par, dev_C, dev_C_par, dev_report, 1,
                           (hipStream_t)stream)))
      return rc;
    if ((rc = gecc_report_to_host(ctx, dev_report, host_report, items_of(ctx), stream))) return rc;
    if (attempts) *attempts = a + 1;
    bool again = false;
    for (int32_t b = 0; b < items_of(ctx); ++b) again = again || host_report[b].status == GECC_UNCORRECTABLE;
    if (!again) break;
  }
  return GECC_OK;
}

namespace {

// Scratch of gecc_protected_gemm_static: one array per GPU, placed by the code-object loader, held
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress; the
// device address it yields (one per device) is what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[GECC_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
char* scratch_addr[MAX_DEVICES] = {};
bool scratch_cleared[MAX_DEVICES] = {};

// device address of `scratch` on the current device, looked up once per device; *first: nobody has
// used the array on this device yet
int static_scratch(char** out, bool* first, int* device) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return GECC_ERR_HIP;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GECC_ERR_HIP;
    scratch_addr[dev] = static_cast<char*>(p);
  }
  *out = scratch_addr[dev];
  *first = !scratch_cleared[dev];
  *device = dev;
  return GECC_OK;
}

}  // namespace

int gecc_protected_gemm_static(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, double* dev_A_par,
                               double* dev_B_par, double* dev_C_par, gecc_report* dev_report,
                               void* stream) {
  if (!ctx || !dev_A || !dev_B || !dev_C || !dev_A_par || !dev_B_par || !dev_C_par || !dev_report)
    return GECC_ERR_ARG;
  if (ctx->lay.total > (size_t)GECC_STATIC_SCRATCH_BYTES) return GECC_ERR_SCRATCH;
  char* ws = nullptr;
  bool first = false;
  int dev = 0;
  int rc = static_scratch(&ws, &first, &dev);
  if (rc) return rc;
  // the context's own workspace (if any) is left alone: this call runs on the static one
  char* const keep_ws = ctx->ws;
  const size_t keep_bytes = ctx->ws_bytes;
  char* const keep_zeroed = ctx->ws_zeroed;
  ctx->ws = ws;
  ctx->ws_bytes = GECC_STATIC_SCRATCH_BYTES;
  // every launch leaves the counters at the front of the array at zero, whichever context used it
  // before; the first call on a device clears them (a kernel launch, not an allocation)
  ctx->ws_zeroed = first ? nullptr : ws;
  rc = gecc_protected_gemm(ctx, dev_A, dev_B, dev_C, dev_A_par, dev_B_par, dev_C_par, dev_report, stream);
  ctx->ws = keep_ws;
  ctx->ws_bytes = keep_bytes;
  ctx->ws_zeroed = keep_zeroed;
  if (rc == GECC_OK && first) {
    std::lock_guard<std::mutex> lock(scratch_mutex);
    scratch_cleared[dev] = true;
  }
  return rc;
}

namespace {
int panel_step(const gecc_ctx* ctx, int panels) {
  const int per = (ctx->p.k + panels - 1) / panels;
  return (per + 63) / 64 * 64;
}
}  // namespace

int32_t gecc_panel_count(const gecc_ctx* ctx, int32_t panels) {
  if (!ctx || panels < 1) return 0;
  const int step = panel_step(ctx, panels);
  return (ctx->p.k + step - 1) / step;
}

int gecc_protected_gemm_panels(gecc_ctx* ctx, void* dev_A, void* dev_B, float* dev_C, float* dev_C_partial,
                               double* dev_A_par, double* dev_B_par, double* dev_C_par,
                               gecc_report* dev_report, int32_t panels, const gecc_fault* dev_faults,
                               int32_t n_faults, void* stream) {
  int rc = check_ws(ctx);
  if (rc) return rc;
  if (panels < 1 || ctx->p.batch != 1 || !dev_report || blocked(ctx)) return GECC_ERR_ARG;
  const int P = gecc_panel_count(ctx, panels), step = panel_step(ctx, panels);
  if (P > 1 && !dev_C_partial) return GECC_ERR_ARG;
  if (dev_C_partial && !aligned_to(dev_C_partial, 4)) return GECC_ERR_ALIGN;
  // one context per panel: the same product with k_g terms (host objects, rebuilt when the panel count changes)
  if (ctx->n_panel != P || !ctx->panel || ctx->panel[0]->p.k != (P == 1 ? ctx->p.k : step)) {
    drop_panels(ctx);
    ctx->panel = new (std::nothrow) gecc_ctx*[P];
    if (!ctx->panel) return GECC_ERR_ARG;
    for (int g = 0; g < P; ++g) {
      gecc_params q = ctx->p;
      const int k0 = g * step;
      q.k = ctx->p.k - k0 < step ? ctx->p.k - k0 : step;
      const double f = (double)q.k / (double)ctx->p.k;
      q.tau_r1 *= f; q.tau_r2 *= f; q.tau_q1 *= f; q.tau_q2 *= f;
      gecc_ctx* child = nullptr;
      rc = gecc_create(&child, &q);
      if (rc || child->lay.total > ctx->lay.total) {
        if (child) gecc_destroy(child);
        ctx->n_panel = g;
        drop_panels(ctx);
        return rc ? rc : GECC_ERR_WORKSPACE;
      }
      child->cu_hint = ctx->cu_hint;
      ctx->panel[g] = child;
      ctx->n_panel = g + 1;
    }
  }
  hipStream_t st = (hipStream_t)stream;
  if ((rc = prep(ctx, st))) return rc;
  const gecc_params& p = ctx->p;
  const size_t esz = elem_size(p.dtype);
  const int64_t rec = 2 * (int64_t)p.n + 2 * (int64_t)p.m + 4;
  for (int g = 0; g < P; ++g) {
    gecc_ctx* c = ctx->panel[g];
    c->ws = ctx->ws; c->ws_bytes = ctx->ws_bytes; c->ws_zeroed = ctx->ws_zeroed;
    c->ev = ctx->ev; c->ev_kind = ctx->ev_kind; c->ev_mask = ctx->ev_mask; c->ev_cap = ctx->ev_cap; c->ev_n = ctx->ev_n;
    const int64_t k0 = (int64_t)g * step;
    char* Ag = static_cast<char*>(dev_A) + (p.trans_a ? k0 * p.lda : k0) * (int64_t)esz;
    char* Bg = static_cast<char*>(dev_B) + (p.trans_b ? k0 : k0 * p.ldb) * (int64_t)esz;
    float* Cg = g == 0 ? dev_C : dev_C_partial;
    double* Apg = dev_A_par + 2 * k0;
    double* Bpg = dev_B_par + 2 * k0;
    double* Cpg = dev_C_par + g * rec;
    c->fault_bias = g;
    rc = encode_and_multiply(c, Ag, Bg, Cg, Apg, Bpg, Cpg, dev_faults, n_faults, st);
    if (!rc) rc = verify_impl(c, Cg, Cpg, dev_report + g, 1, 0, st);
    if (!rc) rc = correct_impl(c, Ag, Apg, Bg, Bpg, Cg, Cpg, dev_report + g, 1, st);
    if (!rc && g > 0) rc = hip_rc(launch_accumulate(dev_C, dev_C_partial, p.n, p.m, p.ldc, st));
    ctx->ev_n = c->ev_n;
    c->ev = nullptr; c->ev_kind = nullptr; c->ev_cap = 0; c->ev_n = 0;     // the records stay the parent's
    if (rc) return rc;
  }
  return GECC_OK;
}

int gecc_plain_gemm(gecc_ctx* ctx, const void* dev_A, const void* dev_B, float* dev_C, void* stream) {
  if (!ctx || !dev_A || !dev_B || !dev_C) return GECC_ERR_ARG;
  if (!aligned_to(dev_A, elem_size(ctx->p.dtype)) || !aligned_to(dev_B, elem_size(ctx->p.dtype)) ||
      !aligned_to(dev_C, 4))
    return GECC_ERR_ALIGN;
  GemmArgs g = gemm_args(ctx, dev_A, dev_B, dev_C);
  g.rowpart = nullptr; g.colpart = nullptr; g.faults = nullptr; g.n_faults = 0;
  if (g.ksplit > 1) {
    const int rc = prep(ctx, (hipStream_t)stream);
    if (rc) return rc;
  }
  return hip_rc(timed_gemm(ctx, g, (hipStream_t)stream));
}

int gecc_report_to_host(gecc_ctx* ctx, const gecc_report* dev_report, gecc_report* host_report,
                        int32_t count, void* stream) {
  if (!ctx || !dev_report || !host_report || count < 1) return GECC_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = hipMemcpyAsync(host_report, dev_report, sizeof(gecc_report) * (size_t)count,
                                hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return GECC_ERR_HIP;
  return hip_rc(hipStreamSynchronize(st));
}

int gecc_syndromes_to_host(gecc_ctx* ctx, double* host_syndromes, void* stream) {
  int rc = check_ws(ctx);
  if (rc) return rc;
  if (!host_syndromes) return GECC_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  const size_t bytes = blocked(ctx) ? ((size_t)ctx->nbj * 2 * ctx->p.n + (size_t)ctx->nbi * 2 * ctx->p.m) * sizeof(double)
                                    : (size_t)ctx->p.batch * (2 * (size_t)ctx->p.n + 2 * (size_t)ctx->p.m) * sizeof(double);
  hipError_t e = hipMemcpyAsync(host_syndromes, ctx->ws + ctx->lay.synd, bytes, hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return GECC_ERR_HIP;
  return hip_rc(hipStreamSynchronize(st));
}

const char* gecc_strerror(int code) {
  switch (code) {
    case GECC_OK: return "ok";
    case GECC_ERR_ARG: return "invalid argument (null pointer, size, enum or leading dimension)";
    case GECC_ERR_WORKSPACE: return "workspace missing or too small";
    case GECC_ERR_HIP: return "HIP runtime error";
    case GECC_ERR_ALIGN: return "pointer or leading dimension breaks the alignment rule";
    case GECC_ERR_SCRATCH: return "problem needs more scratch than the library's static buffer holds "
                                  "(GECC_STATIC_SCRATCH_BYTES); use gecc_set_workspace and gecc_protected_gemm";
    default: return "unknown error code";
  }
}

}  // extern "C"
