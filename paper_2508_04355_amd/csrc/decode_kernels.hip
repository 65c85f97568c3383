// Section V on the device: syndromes from the per-tile partial sums, threshold tests, the
// correction rule for flagged rows/columns, and the operand audit that completes it for
// errors in A and B (each column of [A; A_P] and each row of [B B_P] is a codeword with two
// parity symbols, Section III).  All scalar decoding arithmetic is fp64; everything is
// stream-ordered and gated on state kept in device memory, so no host round trip is needed.
#include "gecc_internal.h"

namespace gecc {
namespace {

struct Est { int i, j; double x, u; };

__device__ __forceinline__ DecodeState* state_of(const DecodeArgs& a, int b) { return a.state + b; }
__device__ __forceinline__ double* synd_of(const DecodeArgs& a, int b) {
  return a.synd + (int64_t)b * (2 * a.p.n + 2 * a.p.m);
}
__device__ __forceinline__ double* allow_of(const DecodeArgs& a, int b) {
  return a.allow + (int64_t)b * (2 * a.p.n + 2 * a.p.m);
}
__device__ __forceinline__ double* cpar_of(const DecodeArgs& a, int b) {
  return a.C_par + (int64_t)b * (2 * a.p.n + 2 * a.p.m + 4);
}

__device__ __forceinline__ double load_elem(const void* P, int dtype, int64_t idx) {
  if (dtype == GECC_BF16)
    return (double)__uint_as_float(((uint32_t) reinterpret_cast<const uint16_t*>(P)[idx]) << 16);
  return (double)reinterpret_cast<const float*>(P)[idx];
}
// round-to-nearest-even store into the operand's storage type
__device__ __forceinline__ void store_elem(void* P, int dtype, int64_t idx, double v) {
  const float f = (float)v;
  if (dtype == GECC_BF16) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    reinterpret_cast<uint16_t*>(P)[idx] = (uint16_t)(u >> 16);
  } else {
    reinterpret_cast<float*>(P)[idx] = f;
  }
}
// item b -> its row block I (A, A_P) and column block J (B, B_P); batch items: I = J = b
__device__ __forceinline__ int item_i(const DecodeArgs& a, int b) { return a.nbj ? b / a.nbj : b; }
__device__ __forceinline__ int item_j(const DecodeArgs& a, int b) { return a.nbj ? b % a.nbj : b; }
__device__ __forceinline__ int64_t a_index(const DecodeArgs& a, int b, int i, int l) {
  const gecc_params& p = a.p;
  return (int64_t)item_i(a, b) * a.ia_stride + (p.trans_a ? (int64_t)l * p.lda + i : (int64_t)i * p.lda + l);
}
__device__ __forceinline__ int64_t b_index(const DecodeArgs& a, int b, int l, int j) {
  const gecc_params& p = a.p;
  return (int64_t)item_j(a, b) * a.jb_stride + (p.trans_b ? (int64_t)j * p.ldb + l : (int64_t)l * p.ldb + j);
}
__device__ __forceinline__ float* c_of(const DecodeArgs& a, int b) {
  return a.C + (int64_t)item_i(a, b) * a.ic_stride + (int64_t)item_j(a, b) * a.jc_stride;
}
__device__ __forceinline__ const double* apar_of(const DecodeArgs& a, int b) { return a.A_par + (int64_t)item_i(a, b) * 2 * a.p.k; }
__device__ __forceinline__ const double* bpar_of(const DecodeArgs& a, int b) { return a.B_par + (int64_t)item_j(a, b) * 2 * a.p.k; }

// Section V step 1 clears a line when |sum - parity| <= threshold holds; anything else, a NaN
// included, flags it.
__device__ __forceinline__ bool outside(double v, double tau) { return !(fabs(v) <= tau); }
__device__ __forceinline__ bool finite2(double a, double b) { return isfinite(a) && isfinite(b); }
// maximum that keeps a NaN (fmax would drop it)
__device__ __forceinline__ double max_nan(double a, double b) { return (a != a || a > b) ? a : b; }

// -------------------------------------------------------------------------------------------
__global__ void reset_state_kernel(DecodeArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.p.batch) return;
  reset_state(state_of(a, b));
}

// partial sums -> syndromes (sum - parity, Section V step 1) -> flags
constexpr int TH_SLICES = 4;    // wavefronts of a workgroup; each adds every 4th sub-tile of a line
constexpr int TH_MAXLOADS = 32; // loads a thread keeps in flight

__global__ __launch_bounds__(64 * TH_SLICES) void threshold_kernel(DecodeArgs a) {
  const int b = blockIdx.y;
  DecodeState* st = state_of(a, b);
  const int n = a.p.n, m = a.p.m;
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int o = blockIdx.x * 64 + lane;          // line: rows first, then columns
  const double* cpar = cpar_of(a, b);
  double* synd = synd_of(a, b);
  const bool is_row = o < n, valid = o < n + m;
  const bool wt = a.p.weighted != 0;     // single-checksum mode: the weighted sums are not read

  // partial sums of this line over the sub-tiles slice, slice + 4, ... (fixed order); all loads
  // of a thread are issued before the first is used
  double S = 0.0, W = 0.0;
  {
    // (lanes past the last line read the last line's data and drop the result; sub-tiles past
    // the last one are clamped and count as zero: no load depends on a branch)
    const int oo = min(o, n + m - 1);
    const bool rowline = oo < n;
    const int nt = rowline ? a.ntn : a.ntm, len = rowline ? a.rp_ld : a.cp_ld, tile = rowline ? a.tile_n : a.tile_m;
    const float2* pp = rowline ? reinterpret_cast<const float2*>(a.rowpart) + (int64_t)b * a.ntn * a.rp_ld + oo
                               : reinterpret_cast<const float2*>(a.colpart) + (int64_t)b * a.ntm * a.cp_ld + (oo - n);
    for (int t0 = slice; t0 < nt; t0 += TH_SLICES * TH_MAXLOADS) {
      float2 v[TH_MAXLOADS];
#pragma unroll
      for (int u = 0; u < TH_MAXLOADS; ++u) v[u] = pp[(int64_t)min(t0 + u * TH_SLICES, nt - 1) * len];
#pragma unroll
      for (int u = 0; u < TH_MAXLOADS; ++u) {
        const int t = t0 + u * TH_SLICES;
        const double x = t < nt ? (double)v[u].x : 0.0, y = t < nt ? (double)v[u].y : 0.0;
        S += x;
        W += y + (double)(t * tile) * x;
      }
    }
  }
  __shared__ double red[2][TH_SLICES][64];
  red[0][slice][lane] = S;
  red[1][slice][lane] = W;
  __syncthreads();
  if (slice != 0) return;
  double v1 = 0.0, v2 = 0.0;
  if (valid) {
    S = (red[0][0][lane] + red[0][1][lane]) + (red[0][2][lane] + red[0][3][lane]);
    W = (red[1][0][lane] + red[1][1][lane]) + (red[1][2][lane] + red[1][3][lane]);
    if (is_row) {
      const int i = o;
      v1 = S - cpar[i];
      v2 = W - cpar[n + i];
      synd[i] = v1;
      synd[n + i] = v2;
      if (outside(v1, a.p.tau_r1) || (wt && outside(v2, a.p.tau_r2))) {
        const int idx = atomicAdd(&st->s_cnt, 1);
        if (idx < GECC_MAX_ERR) st->rows[idx] = i;
      }
    } else {
      const int j = o - n;
      v1 = S - cpar[2 * n + j];
      v2 = W - cpar[2 * n + m + j];
      synd[2 * n + j] = v1;
      synd[2 * n + m + j] = v2;
      if (outside(v1, a.p.tau_q1) || (wt && outside(v2, a.p.tau_q2))) {
        const int idx = atomicAdd(&st->t_cnt, 1);
        if (idx < GECC_MAX_ERR) st->cols[idx] = j;
      }
    }
    if (!wt) v2 = 0.0;
    if (!finite2(v1, v2)) atomicOr(&st->nonfinite, 1);
  }
  {
    // family maxima of this workgroup (rows: [0], [1]; columns: [2], [3]); the summary reduces
    // them (atomics on one line from every workgroup would serialise in L2)
    double mr1 = (valid && is_row) ? fabs(v1) : 0.0, mr2 = (valid && is_row) ? fabs(v2) : 0.0;
    double mq1 = (valid && !is_row) ? fabs(v1) : 0.0, mq2 = (valid && !is_row) ? fabs(v2) : 0.0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      mr1 = max_nan(mr1, __shfl_down(mr1, off, 64));
      mr2 = max_nan(mr2, __shfl_down(mr2, off, 64));
      mq1 = max_nan(mq1, __shfl_down(mq1, off, 64));
      mq2 = max_nan(mq2, __shfl_down(mq2, off, 64));
    }
    if (lane == 0) {
      double* bm = a.blockmax + ((int64_t)b * gridDim.x + blockIdx.x) * 4;
      bm[0] = mr1; bm[1] = mr2; bm[2] = mq1; bm[3] = mq2;
    }
  }
}

// first report after detection: CLEAN or DETECTED.  Called by every thread of a workgroup of 1
// to 4 wavefronts (the family maxima are reduced over the threshold kernel's workgroups);
// returns the status to all of them.
__device__ int summarize(const DecodeArgs& a, int b, const DecodeState* st, gecc_report* rep) {
  __shared__ double smx[4][4];
  double mx[4] = {0.0, 0.0, 0.0, 0.0};
  const double* bm = a.blockmax + (int64_t)b * a.nblk * 4;
  for (int i = threadIdx.x; i < a.nblk; i += blockDim.x)
#pragma unroll
    for (int f = 0; f < 4; ++f) mx[f] = max_nan(mx[f], bm[(int64_t)i * 4 + f]);
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx[f] = max_nan(mx[f], __shfl_down(mx[f], off, 64));
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  if ((threadIdx.x & 63) == 0)
#pragma unroll
    for (int f = 0; f < 4; ++f) smx[wave][f] = mx[f];
  __syncthreads();
  const int status = (st->s_cnt == 0 && st->t_cnt == 0) ? GECC_CLEAN : GECC_DETECTED;
  if (threadIdx.x == 0) {
    rep->s = st->s_cnt;
    rep->t = st->t_cnt;
    rep->n_err = 0;
    rep->n_total = 0;
    rep->reserved = 0;
    for (int f = 0; f < 4; ++f) {
      double v = smx[0][f];
      for (int w = 1; w < nw; ++w) v = max_nan(v, smx[w][f]);
      rep->max_abs_synd[f] = v;
    }
    rep->status = status;
  }
  return status;
}
__global__ __launch_bounds__(64) void summarize_kernel(DecodeArgs a) {   // one wavefront per item
  const int b = blockIdx.x;
  summarize(a, b, state_of(a, b), a.report + b);
}

// ---- Section V step 2 ------------------------------------------------------------------------
// The decoder's workgroup-wide routines below are written for exactly DC_THREADS threads
// (threadIdx.x < DC_THREADS; a larger workgroup lets its other wavefronts end first).
constexpr int DC_THREADS = 256;

__device__ void sort_small(int* v, int cnt) {
  for (int x = 1; x < cnt; ++x) {
    const int key = v[x];
    int y = x - 1;
    while (y >= 0 && v[y] > key) { v[y + 1] = v[y]; --y; }
    v[y + 1] = key;
  }
}

struct Synd {
  const double *r1, *r2, *q1, *q2;
  double b_r1, b_r2, b_q1, b_q2;            // thresholds of the four families
  const double *a_r1, *a_r2, *a_q1, *a_q2;  // per-line allowances (null: none)
  double rel;                               // relative rounding allowance of a syndrome value
  bool wt;                                  // false: single-checksum mode, r2 / q2 are not read
  // how far each syndrome value is trusted when an estimate is verified
  __device__ double tr1(int i) const { return b_r1 + (a_r1 ? a_r1[i] : 0.0) + rel * fabs(r1[i]); }
  __device__ double tr2(int i) const { return b_r2 + (a_r2 ? a_r2[i] : 0.0) + rel * fabs(r2[i]); }
  __device__ double tq1(int j) const { return b_q1 + (a_q1 ? a_q1[j] : 0.0) + rel * fabs(q1[j]); }
  __device__ double tq2(int j) const { return b_q2 + (a_q2 ? a_q2[j] : 0.0) + rel * fabs(q2[j]); }
};

// every syndrome of a flagged line has to be explained by the estimate, within the thresholds
// widened by the uncertainty the estimate itself carries
__device__ bool residual_ok(const Est* est, int ne, const int* Er, int s, const int* Et, int t,
                            const Synd& y) {
  for (int a = 0; a < s; ++a) {
    const int i = Er[a];
    double sx = 0, su = 0, wx = 0, wu = 0;
    for (int e = 0; e < ne; ++e)
      if (est[e].i == i) {
        sx += est[e].x; su += est[e].u;
        wx += (est[e].j + 1) * est[e].x; wu += (est[e].j + 1) * est[e].u;
      }
    if (fabs(y.r1[i] - sx) > y.tr1(i) + su) return false;
    if (y.wt && fabs(y.r2[i] - wx) > y.tr2(i) + wu) return false;
  }
  for (int c = 0; c < t; ++c) {
    const int j = Et[c];
    double sx = 0, su = 0, wx = 0, wu = 0;
    for (int e = 0; e < ne; ++e)
      if (est[e].j == j) {
        sx += est[e].x; su += est[e].u;
        wx += (est[e].i + 1) * est[e].x; wu += (est[e].i + 1) * est[e].u;
      }
    if (fabs(y.q1[j] - sx) > y.tq1(j) + su) return false;
    if (y.wt && fabs(y.q2[j] - wx) > y.tq2(j) + wu) return false;
  }
  return true;
}

// drops insignificant parts, verifies, sorts by (i, j).  Returns the count or -1.
__device__ int accept(Est* est, int ne, const int* Er, int s, const int* Et, int t, const Synd& y) {
  int k = 0;
  for (int e = 0; e < ne; ++e)
    if (fabs(est[e].x) > est[e].u) est[k++] = est[e];
  if (!residual_ok(est, k, Er, s, Et, t, y)) return -1;
  for (int x = 1; x < k; ++x) {
    const Est key = est[x];
    int z = x - 1;
    while (z >= 0 && (est[z].i > key.i || (est[z].i == key.i && est[z].j > key.j))) {
      est[z + 1] = est[z];
      --z;
    }
    est[z + 1] = key;
  }
  return k;
}

// Correction rule for 1 <= s, t <= 2 (s <= t: columns carry the information; s > t mirrored).
__device__ int d0_correct(Est* out, const int* Er, int s, const int* Et, int t, const Synd& y) {
  Est est[4];
  if (s <= t) {
    if (s == 1) {
      for (int c = 0; c < t; ++c) est[c] = Est{Er[0], Et[c], y.q1[Et[c]], y.tq1(Et[c])};
      const int k = accept(est, t, Er, s, Et, t, y);
      for (int e = 0; e < k; ++e) out[e] = est[e];
      return k;
    }
    const int s1 = Er[0], s2 = Er[1], t1 = Et[0], t2 = Et[1];
    Est dg[4] = {Est{s1, t1, y.q1[t1], y.tq1(t1)}, Est{s2, t2, y.q1[t2], y.tq1(t2)}};
    Est an[4] = {Est{s1, t2, y.q1[t2], y.tq1(t2)}, Est{s2, t1, y.q1[t1], y.tq1(t1)}};
    const int kd = accept(dg, 2, Er, s, Et, t, y);
    const int ka = accept(an, 2, Er, s, Et, t, y);
    if (kd >= 0 && ka >= 0) return -1;   // cannot tell the two apart
    if (kd >= 0) { for (int e = 0; e < kd; ++e) out[e] = dg[e]; return kd; }
    if (ka >= 0) { for (int e = 0; e < ka; ++e) out[e] = an[e]; return ka; }
    const double w1 = s1 + 1.0, w2 = s2 + 1.0;
    int ne = 0;
    for (int c = 0; c < 2; ++c) {
      const int j = Et[c];
      const double e2 = (y.q2[j] - w1 * y.q1[j]) / (w2 - w1);
      const double e1 = y.q1[j] - e2;
      const double u2 = (y.tq2(j) + w1 * y.tq1(j)) / (w2 - w1);
      const double u1 = y.tq1(j) + u2;
      est[ne++] = Est{s1, j, e1, u1};
      est[ne++] = Est{s2, j, e2, u2};
    }
    const int k = accept(est, ne, Er, s, Et, t, y);
    for (int e = 0; e < k; ++e) out[e] = est[e];
    return k;
  }
  for (int r = 0; r < s; ++r) est[r] = Est{Er[r], Et[0], y.r1[Er[r]], y.tr1(Er[r])};
  const int k = accept(est, s, Er, s, Et, t, y);
  for (int e = 0; e < k; ++e) out[e] = est[e];
  return k;
}

// fp64 dot product of row i of A with column j of B over k, by the whole workgroup
__device__ double block_dot(const DecodeArgs& a, int b, int i, int j, double* red) {
  double s = 0.0;
  constexpr int U = 8;   // products per thread whose loads are issued together (one workgroup: latency-bound)
  for (int l0 = threadIdx.x; l0 < a.p.k; l0 += U * DC_THREADS) {
    double x[U], y[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int l = min(l0 + u * DC_THREADS, a.p.k - 1);
      x[u] = load_elem(a.A, a.p.dtype, a_index(a, b, i, l));
      y[u] = load_elem(a.B, a.p.dtype, b_index(a, b, l, j));
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (l0 + u * DC_THREADS < a.p.k) s = fma(x[u], y[u], s);
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = DC_THREADS / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  const double r = red[0];
  __syncthreads();
  return r;
}

// Theorem 2 (Appendix B): min(s, t) <= 2 < max(s, t).  The at most two flagged lines of the
// short side are the known lines; every flagged line c of the other kind is decoded on its own
// from its two syndromes (one known line: e = y1_c; two: the 2x2 system of Section V), the
// estimates are verified against every flagged line like those of d0_correct, and Section V's
// subtraction is applied.  All threads of the workgroup take part: thread x owns a contiguous
// chunk of the other-kind lines.  Returns the number of corrected symbols, or -1.
struct LineEst { double x[2], u[2]; bool sig[2], flagged; };

__device__ int known_lines_correct(const DecodeArgs& a, int b, DecodeState* st, gecc_report* rep,
                                   const Synd& y, int final_pass) {
  const int n = a.p.n, m = a.p.m;
  const int s = st->s_cnt, t = st->t_cnt;
  const bool rows_known = a.p.weighted ? s <= 2 : s == 1;
  const int nk = rows_known ? s : t;
  const int L = rows_known ? m : n;
  int K[2] = {0, 0};
  for (int q = 0; q < nk; ++q) K[q] = rows_known ? st->rows[q] : st->cols[q];
  if (nk == 2 && K[0] > K[1]) { const int z = K[0]; K[0] = K[1]; K[1] = z; }
  const double w1 = K[0] + 1.0, w2 = K[1] + 1.0;
  const double *y1 = rows_known ? y.q1 : y.r1, *y2 = rows_known ? y.q2 : y.r2;
  const double b1 = rows_known ? y.b_q1 : y.b_r1, b2 = rows_known ? y.b_q2 : y.b_r2;
  const double *a1 = rows_known ? y.a_q1 : y.a_r1, *a2 = rows_known ? y.a_q2 : y.a_r2;

  auto estimate = [&](int c) {
    LineEst e;
    e.flagged = fabs(y1[c]) > b1 + (a1 ? a1[c] : 0.0) || (y.wt && fabs(y2[c]) > b2 + (a2 ? a2[c] : 0.0));
    e.sig[0] = e.sig[1] = false; e.x[0] = e.x[1] = e.u[0] = e.u[1] = 0.0;
    if (!e.flagged) return e;
    const double u1 = rows_known ? y.tq1(c) : y.tr1(c), u2 = rows_known ? y.tq2(c) : y.tr2(c);
    if (nk == 1) {
      e.x[0] = y1[c]; e.u[0] = u1;
    } else {
      e.x[1] = (y2[c] - w1 * y1[c]) / (w2 - w1);
      e.x[0] = y1[c] - e.x[1];
      e.u[1] = (u2 + w1 * u1) / (w2 - w1);
      e.u[0] = u1 + e.u[1];
    }
    for (int q = 0; q < nk; ++q) e.sig[q] = fabs(e.x[q]) > e.u[q];   // insignificant parts are dropped
    return e;
  };

  __shared__ double t2_red[8][256];
  __shared__ int t2_cnt[2][256];
  __shared__ int t2_bad;
  const int tid = threadIdx.x, ch = (L + DC_THREADS - 1) / DC_THREADS;
  const int c0 = min(L, tid * ch), c1 = min(L, c0 + ch);
  if (tid == 0) t2_bad = 0;
  __syncthreads();
  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // per known line: sum x, sum u, weighted sum x, weighted sum u
  int cnt[2] = {0, 0};
  bool bad = false;
  for (int c = c0; c < c1; ++c) {
    const LineEst e = estimate(c);
    if (!e.flagged) continue;
    // this line's own two syndromes
    double sx = 0, su = 0, wx = 0, wu = 0;
    for (int q = 0; q < nk; ++q)
      if (e.sig[q]) {
        const double w = K[q] + 1.0;
        sx += e.x[q]; su += e.u[q]; wx += w * e.x[q]; wu += w * e.u[q];
        acc[4 * q + 0] += e.x[q]; acc[4 * q + 1] += e.u[q];
        acc[4 * q + 2] += (c + 1.0) * e.x[q]; acc[4 * q + 3] += (c + 1.0) * e.u[q];
        ++cnt[q];
      }
    const double u1 = rows_known ? y.tq1(c) : y.tr1(c), u2 = rows_known ? y.tq2(c) : y.tr2(c);
    bad = bad || fabs(y1[c] - sx) > u1 + su || (y.wt && fabs(y2[c] - wx) > u2 + wu);
  }
  for (int q = 0; q < 8; ++q) t2_red[q][tid] = acc[q];
  t2_cnt[0][tid] = cnt[0]; t2_cnt[1][tid] = cnt[1];
  if (bad) t2_bad = 1;
  __syncthreads();
  if (tid == 0) {
    // the known lines' own syndromes against everything attributed to them
    for (int q = 0; q < nk; ++q) {
      double v[4] = {0, 0, 0, 0};
      for (int x = 0; x < DC_THREADS; ++x)
        for (int f = 0; f < 4; ++f) v[f] += t2_red[4 * q + f][x];
      const int line = K[q];
      const double z1 = rows_known ? y.r1[line] : y.q1[line], z2 = rows_known ? y.r2[line] : y.q2[line];
      const double tz1 = rows_known ? y.tr1(line) : y.tq1(line), tz2 = rows_known ? y.tr2(line) : y.tq2(line);
      if (fabs(z1 - v[0]) > tz1 + v[1] || (y.wt && fabs(z2 - v[2]) > tz2 + v[3])) t2_bad = 1;
    }
  }
  __syncthreads();
  if (t2_bad) return -1;
  // position of this thread's entries in the list sorted by (row, column)
  int before[2] = {0, 0}, total[2] = {0, 0};
  for (int x = 0; x < DC_THREADS; ++x)
    for (int q = 0; q < 2; ++q) {
      if (x < tid) before[q] += t2_cnt[q][x];
      total[q] += t2_cnt[q][x];
    }
  const int ne0 = st->n_err;                  // operand errors of the audit come first
  int idx[2];
  if (rows_known) { idx[0] = before[0]; idx[1] = total[0] + before[1]; }     // row K0 first, then row K1
  else            { idx[0] = idx[1] = before[0] + before[1]; }               // row by row
  float* C = c_of(a, b);
  for (int c = c0; c < c1; ++c) {
    const LineEst e = estimate(c);
    if (!e.flagged) continue;
    for (int q = 0; q < nk; ++q)
      if (e.sig[q]) {
        const int i = rows_known ? K[q] : c, j = rows_known ? c : K[q];
        const int64_t ic = (int64_t)i * a.p.ldc + j;
        C[ic] = (float)((double)C[ic] - e.x[q]);
        const int pos = ne0 + (rows_known ? idx[q]++ : idx[0]++);
        if (pos < GECC_MAX_ERR) {
          gecc_err g;
          g.matrix = GECC_MAT_C; g.row = i; g.col = j; g.reserved = 0; g.magnitude = e.x[q];
          rep->err[pos] = g;
        }
      }
  }
  return total[0] + total[1];
}

// Section V step 2 for one batch item, by DC_THREADS threads.  final_pass = 0: right after
// detection; = 1: on the residual syndromes after an operand repair (per-line allowances apply,
// failure is final).
__device__ void decode_c_body(const DecodeArgs& a, int b, DecodeState* st, gecc_report* rep, int final_pass) {
  __shared__ Est fix[4];
  __shared__ int nfix;          // -1: the rule does not apply / failed
  __shared__ double red[256];
  const int n = a.p.n, m = a.p.m;
  if (st->nonfinite) {
    // a syndrome that is not a number: no estimate can be subtracted, the product is computed again
    if (threadIdx.x == 0) { rep->status = GECC_UNCORRECTABLE; rep->n_err = 0; rep->n_total = 0; st->phase = PH_DONE; }
    return;
  }
  {
    const int s = st->s_cnt, t = st->t_cnt, lo = min(s, t), hi = max(s, t);
    // Theorem 2: many lines of one kind, at most two of the other.  Its errors all lie in C-bar,
    // so it runs only after the operand audit (on what the repair leaves, or on the whole pattern
    // when both operands are intact): a wrong symbol of A a few rows from a flagged row would
    // otherwise pass for a row full of small errors of C.
    // (single-checksum mode: one known line only, any number of the other kind -- Appendix A, case s = 1)
    if (final_pass && (a.p.weighted ? (lo >= 1 && lo <= 2 && hi > 2) : (lo == 1 && hi >= 2))) {
      const double* sy = synd_of(a, b);
      const double* al = final_pass ? allow_of(a, b) : nullptr;
      const Synd y{sy, sy + n, sy + 2 * n, sy + 2 * n + m, a.p.tau_r1, a.p.tau_r2, a.p.tau_q1, a.p.tau_q2,
                   al, al ? al + n : nullptr, al ? al + 2 * n : nullptr, al ? al + 2 * n + m : nullptr,
                   a.p.tau_rel, a.p.weighted != 0};
      const int k = known_lines_correct(a, b, st, rep, y, final_pass);
      if (threadIdx.x == 0) {
        if (k < 0) {
          rep->status = GECC_UNCORRECTABLE; rep->n_err = 0; rep->n_total = 0; st->phase = PH_DONE;
        } else {
          for (int e = 0; e < st->n_err; ++e) rep->err[e] = st->errs[e];
          rep->n_total = st->n_err + k;
          rep->n_err = min(rep->n_total, GECC_MAX_ERR);
          rep->status = GECC_CORRECTED;
          st->phase = PH_DONE;
        }
      }
      return;
    }
  }
  if (threadIdx.x == 0) {
    const int s = st->s_cnt, t = st->t_cnt;
    nfix = -1;
    if (s == 0 && t == 0) {
      nfix = 0;
    } else if (s >= 1 && s <= 2 && t >= 1 && t <= 2 && (a.p.weighted || (s == 1 && t == 1))) {
      int Er[2], Et[2];
      for (int x = 0; x < s; ++x) Er[x] = st->rows[x];
      for (int x = 0; x < t; ++x) Et[x] = st->cols[x];
      sort_small(Er, s);
      sort_small(Et, t);
      const double* sy = synd_of(a, b);
      const double* al = final_pass ? allow_of(a, b) : nullptr;
      Synd y{sy, sy + n, sy + 2 * n, sy + 2 * n + m, a.p.tau_r1, a.p.tau_r2, a.p.tau_q1, a.p.tau_q2,
             al, al ? al + n : nullptr, al ? al + 2 * n : nullptr, al ? al + 2 * n + m : nullptr,
             a.p.tau_rel, a.p.weighted != 0};
      Est tmp[4];
      const int k = d0_correct(tmp, Er, s, Et, t, y);
      if (k >= 0) {
        for (int e = 0; e < k; ++e) fix[e] = tmp[e];
        nfix = k;
      }
    }
  }
  __syncthreads();
  const int k = nfix;
  if (k < 0) {
    if (threadIdx.x == 0) {
      if (final_pass) { rep->status = GECC_UNCORRECTABLE; rep->n_err = 0; rep->n_total = 0; st->phase = PH_DONE; }
      else            { st->phase = PH_AUDIT; if (a.gate_word) *a.gate_word = PH_AUDIT; }
    }
    return;
  }
  // patch C: Section V's subtraction, optionally followed by re-evaluating the symbol
  float* C = c_of(a, b);
  for (int e = 0; e < k; ++e) {
    const int64_t idx = (int64_t)fix[e].i * a.p.ldc + fix[e].j;
    if (a.p.refine) {
      const double d = block_dot(a, b, fix[e].i, fix[e].j, red);
      if (threadIdx.x == 0) C[idx] = (float)d;
    } else if (threadIdx.x == 0) {
      C[idx] = (float)((double)C[idx] - fix[e].x);
    }
  }
  if (threadIdx.x == 0) {
    int ne = 0;
    for (int e = 0; e < st->n_err; ++e) rep->err[ne++] = st->errs[e];   // A then B, sorted (at most 8)
    const int total = ne + k;
    for (int e = 0; e < k && ne < GECC_MAX_ERR; ++e) {
      gecc_err g;
      g.matrix = GECC_MAT_C; g.row = fix[e].i; g.col = fix[e].j; g.reserved = 0;
      g.magnitude = fix[e].x;
      rep->err[ne++] = g;
    }
    rep->n_total = total;
    rep->n_err = ne;
    rep->status = GECC_CORRECTED;
    st->phase = PH_DONE;
  }
}

// One workgroup per batch item, right after detection.  with_summary: this kernel also writes
// the first report (saves the summary launch).
__global__ __launch_bounds__(DC_THREADS) void decode_c_kernel(DecodeArgs a, int with_summary) {
  const int b = blockIdx.x;
  DecodeState* st = state_of(a, b);
  gecc_report* rep = a.report + b;
  if (with_summary) {
    if (summarize(a, b, st, rep) == GECC_CLEAN) return;
  } else {
    if (rep->status != GECC_DETECTED) return;
  }
  decode_c_body(a, b, st, rep, 0);
}

// ---- operand audit -----------------------------------------------------------------------------
// A single wrong symbol of a line (column l of A, row l of B) shows as (u1, u2) = (e, (pos+1) e)
// in the difference of re-formed and stored parities.
__device__ AuditHit audit_line(const double* cur, const double* ref, int k, int l, int len, double tau,
                               bool wt, bool* hit) {
  const double u1 = cur[l] - ref[l], u2 = cur[k + l] - ref[k + l];
  AuditHit h;
  h.line = l; h.pos = -1; h.e = u1;
  *hit = outside(u1, tau) || (wt && outside(u2, tau));
  if (*hit && fabs(u1) > tau && finite2(u1, u2)) {
    const double rho = u2 / u1, w = rint(rho);
    if (fabs(rho - w) < 0.25 && w >= 1.0 && w <= (double)len) h.pos = (int)w - 1;
  }
  return h;
}

__device__ void sort_hits(AuditHit* h, int cnt) {
  for (int x = 1; x < cnt; ++x) {
    const AuditHit key = h[x];
    int y = x - 1;
    while (y >= 0 && h[y].line > key.line) { h[y + 1] = h[y]; --y; }
    h[y + 1] = key;
  }
}

// Remove the rank-one footprint of every audit hit from C-bar, then patch the operands.
// Order (it absorbs the cross term when an A hit and a B hit share the index l): rows of the
// A hits first, using B as the product read it; then columns of the B hits, using the
// corrected A.  The operands themselves are written last, so nothing here depends on a
// store becoming visible to another wavefront.
constexpr int RP_THREADS = 1024;   // one workgroup per batch item: latency-bound loops, so a full one
constexpr int RP_U = 4;            // symbols (lines) a thread has in flight

// SPLIT (blocked mode: several blocks share an operand line): this launch leaves the operands alone
// and stops before Section V's second pass; patch_operands_kernel and final_decode_kernel follow.
template <bool SPLIT>
__global__ __launch_bounds__(RP_THREADS) void repair_kernel(DecodeArgs a) {
  const int b = blockIdx.x;
  DecodeState* st = state_of(a, b);
  if (st->phase != PH_AUDIT) return;
  gecc_report* rep = a.report + b;
  __shared__ int ok, cnt_a, cnt_b;
  __shared__ AuditHit ha[GECC_MAX_ERR], hb[GECC_MAX_ERR];
  const int n = a.p.n, m = a.p.m, k = a.p.k;
  if (threadIdx.x == 0) { cnt_a = 0; cnt_b = 0; }
  __syncthreads();
  {   // difference of the re-formed and the stored operand parities, line by line
    const double* cur_a = a.audit_a + (int64_t)item_i(a, b) * 2 * k;
    const double* cur_b = a.audit_b + (int64_t)item_j(a, b) * 2 * k;
    const double* ref_a = apar_of(a, b);
    const double* ref_b = bpar_of(a, b);
#pragma unroll 4
    for (int l = threadIdx.x; l < k; l += blockDim.x) {
      bool hit;
      AuditHit h = audit_line(cur_a, ref_a, k, l, n, a.p.tau_op, a.p.weighted != 0, &hit);
      if (hit) { const int idx = atomicAdd(&cnt_a, 1); if (idx < GECC_MAX_ERR) ha[idx] = h; }
      h = audit_line(cur_b, ref_b, k, l, m, a.p.tau_op, a.p.weighted != 0, &hit);
      if (hit) { const int idx = atomicAdd(&cnt_b, 1); if (idx < GECC_MAX_ERR) hb[idx] = h; }
    }
  }
  __syncthreads();
  const int na = cnt_a, nb = cnt_b;
  if (threadIdx.x == 0) {
    ok = na + nb <= GECC_MAX_ERR;       // no hit at all: the pattern lies in C-bar alone (second pass below)
    // single-checksum mode: one parity names the line of a wrong operand symbol, not its place in it
    if (!a.p.weighted && na + nb > 0) ok = 0;
    if (ok) {
      for (int x = 0; x < na; ++x) if (ha[x].pos < 0) ok = 0;
      for (int x = 0; x < nb; ++x) if (hb[x].pos < 0) ok = 0;
    }
    if (ok) { sort_hits(ha, na); sort_hits(hb, nb); }
  }
  __syncthreads();
  if (!ok) {
    if (threadIdx.x == 0) { rep->status = GECC_UNCORRECTABLE; rep->n_err = 0; rep->n_total = 0; st->phase = PH_DONE; }
    return;
  }
  float* C = c_of(a, b);
  double* cpar = cpar_of(a, b);
  const double* apar = apar_of(a, b);
  const double* bpar = bpar_of(a, b);
  // threshold allowances of the lines a repair touches (rounding noise of the corrupted terms)
  double* al_r1 = allow_of(a, b);
  double* al_r2 = al_r1 + n;
  double* al_q1 = al_r1 + 2 * n;
  double* al_q2 = al_r1 + 2 * n + m;
  const double cc = a.p.tau_rep * sqrt((double)k);
  // residual syndromes: every repair below also moves the syndromes by exactly what it changes
  // (the stored symbols' differences and the parity symbols), so that Section V can run again
  // without another pass over C
  double* sy_r1 = synd_of(a, b);
  double* sy_r2 = sy_r1 + n;
  double* sy_q1 = sy_r1 + 2 * n;
  double* sy_q2 = sy_r1 + 2 * n + m;
  __shared__ double red[4][RP_THREADS];
  for (int o = threadIdx.x; o < 2 * n + 2 * m; o += blockDim.x) al_r1[o] = 0.0;
  __syncthreads();
  for (int x = 0; x < na; ++x) {
    const int i = ha[x].pos, l = ha[x].line;
    const double e = ha[x].e;
    if (threadIdx.x == 0) {
      cpar[i] -= e * bpar[l];              // cbar_{i,m+1}
      cpar[n + i] -= e * bpar[k + l];      // cbar_{i,m+2}
    }
    double s2 = 0.0, w2 = 0.0, ds = 0.0, dw = 0.0;
    // (RP_U symbols per thread at a time: all their loads are issued before the first store, one
    // workgroup has nothing else to hide the memory latency with)
    for (int j0 = threadIdx.x; j0 < m; j0 += RP_U * RP_THREADS) {
      float cold[RP_U];
      double bv[RP_U], q1[RP_U], q2[RP_U], g1[RP_U], g2[RP_U];
#pragma unroll
      for (int u = 0; u < RP_U; ++u) {
        const int j = min(j0 + u * RP_THREADS, m - 1);
        cold[u] = C[(int64_t)i * a.p.ldc + j];
        bv[u] = load_elem(a.B, a.p.dtype, b_index(a, b, l, j));
        q1[u] = sy_q1[j]; q2[u] = sy_q2[j]; g1[u] = al_q1[j]; g2[u] = al_q2[j];
      }
#pragma unroll
      for (int u = 0; u < RP_U; ++u) {
        const int j = j0 + u * RP_THREADS;
        if (j >= m) break;
        const double f = e * bv[u];
        const float cnew = (float)((double)cold[u] - f);
        C[(int64_t)i * a.p.ldc + j] = cnew;
        const double d = (double)cold[u] - (double)cnew;   // what the sums of row i and column j lose
        sy_q1[j] = q1[u] - d;
        sy_q2[j] = q2[u] - (double)(i + 1) * d;
        ds += d;
        dw += (double)(j + 1) * d;
        s2 += f * f;
        w2 += (double)(j + 1) * (j + 1) * f * f;
        al_q1[j] = g1[u] + cc * fabs(f);
        al_q2[j] = g2[u] + cc * (double)(i + 1) * fabs(f);
      }
    }
    red[0][threadIdx.x] = s2; red[1][threadIdx.x] = w2; red[2][threadIdx.x] = ds; red[3][threadIdx.x] = dw;
    __syncthreads();
    for (int w = RP_THREADS / 2; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w)
        for (int q = 0; q < 4; ++q) red[q][threadIdx.x] += red[q][threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0) {
      al_r1[i] += cc * sqrt(red[0][0]); al_r2[i] += cc * sqrt(red[1][0]);
      sy_r1[i] += e * bpar[l] - red[2][0];          // sum - parity: both moved
      sy_r2[i] += e * bpar[k + l] - red[3][0];
    }
    __syncthreads();
  }
  for (int x = 0; x < nb; ++x) {
    const int l = hb[x].line, j = hb[x].pos;
    const double e = hb[x].e;
    if (threadIdx.x == 0) {
      cpar[2 * n + j] -= apar[l] * e;          // cbar_{n+1,j}
      cpar[2 * n + m + j] -= apar[k + l] * e;  // cbar_{n+2,j}
    }
    double s2 = 0.0, w2 = 0.0, ds = 0.0, dw = 0.0;
    for (int i0 = threadIdx.x; i0 < n; i0 += RP_U * RP_THREADS) {
      float cold[RP_U];
      double av[RP_U], r1[RP_U], r2[RP_U], g1[RP_U], g2[RP_U];
#pragma unroll
      for (int u = 0; u < RP_U; ++u) {
        const int i = min(i0 + u * RP_THREADS, n - 1);
        cold[u] = C[(int64_t)i * a.p.ldc + j];
        av[u] = load_elem(a.A, a.p.dtype, a_index(a, b, i, l));
        r1[u] = sy_r1[i]; r2[u] = sy_r2[i]; g1[u] = al_r1[i]; g2[u] = al_r2[i];
      }
#pragma unroll
      for (int u = 0; u < RP_U; ++u) {
        const int i = i0 + u * RP_THREADS;
        if (i >= n) break;
        double ai = av[u];
        for (int z = 0; z < na; ++z)
          if (ha[z].pos == i && ha[z].line == l) ai -= ha[z].e;   // corrected A
        const double f = ai * e;
        const float cnew = (float)((double)cold[u] - f);
        C[(int64_t)i * a.p.ldc + j] = cnew;
        const double d = (double)cold[u] - (double)cnew;
        sy_r1[i] = r1[u] - d;
        sy_r2[i] = r2[u] - (double)(j + 1) * d;
        ds += d;
        dw += (double)(i + 1) * d;
        s2 += f * f;
        w2 += (double)(i + 1) * (i + 1) * f * f;
        al_r1[i] = g1[u] + cc * fabs(f);
        al_r2[i] = g2[u] + cc * (double)(j + 1) * fabs(f);
      }
    }
    red[0][threadIdx.x] = s2; red[1][threadIdx.x] = w2; red[2][threadIdx.x] = ds; red[3][threadIdx.x] = dw;
    __syncthreads();
    for (int w = RP_THREADS / 2; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w)
        for (int q = 0; q < 4; ++q) red[q][threadIdx.x] += red[q][threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0) {
      al_q1[j] += cc * sqrt(red[0][0]); al_q2[j] += cc * sqrt(red[1][0]);
      sy_q1[j] += apar[l] * e - red[2][0];
      sy_q2[j] += apar[k + l] * e - red[3][0];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    for (int x = 0; x < na && !SPLIT; ++x) {
      const int64_t ia = a_index(a, b, ha[x].pos, ha[x].line);
      store_elem(a.A, a.p.dtype, ia, load_elem(a.A, a.p.dtype, ia) - ha[x].e);
    }
    for (int x = 0; x < nb && !SPLIT; ++x) {
      const int64_t ib = b_index(a, b, hb[x].line, hb[x].pos);
      store_elem(a.B, a.p.dtype, ib, load_elem(a.B, a.p.dtype, ib) - hb[x].e);
    }
    // located operand errors, sorted by (matrix, row, col)
    int ne = 0;
    for (int x = 0; x < na; ++x) {
      gecc_err g;
      g.matrix = GECC_MAT_A; g.row = ha[x].pos; g.col = ha[x].line; g.reserved = 0;
      g.magnitude = ha[x].e;
      st->errs[ne++] = g;
    }
    for (int x = 1; x < ne; ++x) {           // A hits were ordered by column: reorder by (row, col)
      const gecc_err key = st->errs[x];
      int y = x - 1;
      while (y >= 0 && (st->errs[y].row > key.row ||
                        (st->errs[y].row == key.row && st->errs[y].col > key.col))) {
        st->errs[y + 1] = st->errs[y];
        --y;
      }
      st->errs[y + 1] = key;
    }
    for (int x = 0; x < nb; ++x) {           // B hits are ordered by row l; one hit per row
      gecc_err g;
      g.matrix = GECC_MAT_B; g.row = hb[x].line; g.col = hb[x].pos; g.reserved = 0;
      g.magnitude = hb[x].e;
      st->errs[ne++] = g;
    }
    st->n_err = ne;
  }
  // Section V step 1 on the residual syndromes (thresholds widened by the allowances above) ...
  __shared__ int res_s, res_t, res_bad;
  const bool wt = a.p.weighted != 0;
  if (threadIdx.x == 0) { res_s = 0; res_t = 0; res_bad = 0; }
  __syncthreads();
  for (int o0 = threadIdx.x; o0 < n + m; o0 += 2 * RP_U * RP_THREADS) {
    double y1[2 * RP_U], y2[2 * RP_U], g1[2 * RP_U], g2[2 * RP_U];
#pragma unroll
    for (int u = 0; u < 2 * RP_U; ++u) {
      const int o = min(o0 + u * RP_THREADS, n + m - 1);
      // row line o: r1 at [o], r2 at [n + o]; column line j = o - n: q1 at [2n + j], q2 at [2n + m + j]
      const int p1 = o < n ? o : n + o, p2 = o < n ? n + o : n + m + o;
      y1[u] = sy_r1[p1]; y2[u] = sy_r1[p2]; g1[u] = al_r1[p1]; g2[u] = al_r1[p2];
    }
#pragma unroll
    for (int u = 0; u < 2 * RP_U; ++u) {
      const int o = o0 + u * RP_THREADS;
      if (o >= n + m) break;
      if (o < n) {
        if (outside(y1[u], a.p.tau_r1 + g1[u]) || (wt && outside(y2[u], a.p.tau_r2 + g2[u]))) {
          const int idx = atomicAdd(&res_s, 1);
          if (idx < GECC_MAX_ERR) st->rows[idx] = o;
        }
      } else if (outside(y1[u], a.p.tau_q1 + g1[u]) || (wt && outside(y2[u], a.p.tau_q2 + g2[u]))) {
        const int idx = atomicAdd(&res_t, 1);
        if (idx < GECC_MAX_ERR) st->cols[idx] = o - n;
      }
      if (!finite2(y1[u], wt ? y2[u] : 0.0)) res_bad = 1;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) { st->s_cnt = res_s; st->t_cnt = res_t; st->nonfinite = res_bad; st->phase = PH_REVERIFY; }
  __syncthreads();
  // ... and step 2, by the first DC_THREADS threads (the other wavefronts end here)
  if (SPLIT || threadIdx.x >= DC_THREADS) return;
  decode_c_body(a, b, st, rep, 1);
}

// Blocked mode, after repair_kernel<true>: the located operand symbols are put right, once per
// operand line (workgroup x < nbi: row block x of A; otherwise column block x - nbi of B), from
// the same parity differences the blocks used -- after every block has finished reading the
// operands as the product read them.
__global__ __launch_bounds__(256) void patch_operands_kernel(DecodeArgs a, int nbi) {
  if (*a.gate_word != PH_AUDIT) return;
  const bool is_a = (int)blockIdx.x < nbi;
  const int line_blk = is_a ? blockIdx.x : blockIdx.x - nbi;
  const int b = is_a ? line_blk * a.nbj : line_blk;           // an item of that line (item_i / item_j = line_blk)
  const int k = a.p.k, len = is_a ? a.p.n : a.p.m;
  const double* cur = (is_a ? a.audit_a : a.audit_b) + (int64_t)line_blk * 2 * k;
  const double* ref = (is_a ? a.A_par : a.B_par) + (int64_t)line_blk * 2 * k;
  __shared__ int cnt;
  __shared__ AuditHit h[GECC_MAX_ERR];
  if (threadIdx.x == 0) cnt = 0;
  __syncthreads();
  for (int l = threadIdx.x; l < k; l += blockDim.x) {
    bool hit;
    const AuditHit x = audit_line(cur, ref, k, l, len, a.p.tau_op, true, &hit);
    if (hit) { const int idx = atomicAdd(&cnt, 1); if (idx < GECC_MAX_ERR) h[idx] = x; }
  }
  __syncthreads();
  if (threadIdx.x != 0 || cnt == 0 || cnt > GECC_MAX_ERR) return;
  for (int x = 0; x < cnt; ++x) if (h[x].pos < 0) return;      // a line no single wrong symbol explains: hands off
  for (int x = 0; x < cnt; ++x) {
    const int64_t idx = is_a ? a_index(a, b, h[x].pos, h[x].line) : b_index(a, b, h[x].line, h[x].pos);
    void* M = is_a ? a.A : a.B;
    store_elem(M, a.p.dtype, idx, load_elem(M, a.p.dtype, idx) - h[x].e);
  }
}

// Blocked mode: Section V once more on what the repairs left, block by block.
__global__ __launch_bounds__(DC_THREADS) void final_decode_kernel(DecodeArgs a) {
  const int b = blockIdx.x;
  DecodeState* st = state_of(a, b);
  if (st->phase != PH_REVERIFY) return;
  decode_c_body(a, b, st, a.report + b, 1);
}

// Blocked mode: syndromes of every block from the partial sums of the 128 x 128 sub-tiles (a block
// is a whole number of them), one thread per line and block along it.  a.p.n, a.p.m: block sizes.
__global__ __launch_bounds__(256) void threshold_blocked_kernel(DecodeArgs a, int n_full, int m_full) {
  const int nb = a.p.n, mb = a.p.m, nbj = a.nbj, nbi = n_full / nb;
  // (n_full, m_full are multiples of 128: the 64 lines of a wavefront lie in one block, and every
  // wavefront of the grid is full)
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total_r = (int64_t)n_full * nbj, total = total_r + (int64_t)m_full * nbi;
  if (idx >= total) return;
  const bool is_row = idx < total_r;
  double S = 0.0, W = 0.0;
  int b, loc;
  if (is_row) {
    const int i = (int)(idx % n_full), J = (int)(idx / n_full);
    const float2* pp = reinterpret_cast<const float2*>(a.rowpart) + i;
    for (int t = J * (mb / 128); t < (J + 1) * (mb / 128); ++t) {
      const float2 v = pp[(int64_t)t * a.rp_ld];
      S += (double)v.x;
      W += (double)v.y + (double)(t * 128 - J * mb) * (double)v.x;
    }
    b = (i / nb) * nbj + J; loc = i % nb;
  } else {
    const int64_t o = idx - total_r;
    const int j = (int)(o % m_full), I = (int)(o / m_full);
    const float2* pp = reinterpret_cast<const float2*>(a.colpart) + j;
    for (int t = I * (nb / 128); t < (I + 1) * (nb / 128); ++t) {
      const float2 v = pp[(int64_t)t * a.cp_ld];
      S += (double)v.x;
      W += (double)v.y + (double)(t * 128 - I * nb) * (double)v.x;
    }
    b = I * nbj + j / mb; loc = j % mb;
  }
  DecodeState* st = state_of(a, b);
  const double* cpar = cpar_of(a, b);
  double* synd = synd_of(a, b);
  const int o1 = is_row ? loc : 2 * nb + loc, o2 = is_row ? nb + loc : 2 * nb + mb + loc;
  const double v1 = S - cpar[o1], v2 = W - cpar[o2];
  synd[o1] = v1;
  synd[o2] = v2;
  const double t1 = is_row ? a.p.tau_r1 : a.p.tau_q1, t2 = is_row ? a.p.tau_r2 : a.p.tau_q2;
  if (outside(v1, t1) || outside(v2, t2)) {
    const int x = atomicAdd(is_row ? &st->s_cnt : &st->t_cnt, 1);
    if (x < GECC_MAX_ERR) (is_row ? st->rows : st->cols)[x] = loc;
  }
  if (!finite2(v1, v2)) atomicOr(&st->nonfinite, 1);
  // family maxima of the block: first over the wavefront (one block, see above), then one atomic per
  // wavefront -- non-negative doubles order like their bit patterns, a NaN above all
  double m1 = fabs(v1), m2 = fabs(v2);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    m1 = max_nan(m1, __shfl_xor(m1, off, 64));
    m2 = max_nan(m2, __shfl_xor(m2, off, 64));
  }
  if ((threadIdx.x & 63) == 0) {
    unsigned long long* mx = reinterpret_cast<unsigned long long*>(a.blockmax) + (int64_t)b * 4 + (is_row ? 0 : 2);
    atomicMax(mx, (unsigned long long)__double_as_longlong(m1));
    atomicMax(mx + 1, (unsigned long long)__double_as_longlong(m2));
  }
}

// Blocked mode: the parity blocks of every block of C-bar from the two side products (A times the
// parity columns of all column blocks, the parity rows of all row blocks times B), P_g in fp64,
// and the per-block resets.  One workgroup per block.
__global__ __launch_bounds__(256) void blocked_parities_kernel(BlockedParityArgs a) {
  const int b = blockIdx.x, I = b / a.nbj, J = b % a.nbj;
  const int nb = a.nb, mb = a.mb, S = a.pieces;
  double* cpar = a.C_par + (int64_t)b * (2 * nb + 2 * mb + 4);
  for (int il = threadIdx.x; il < nb; il += blockDim.x) {      // 2 S consecutive floats of a row of the side product
    const float* p = a.side_r + (int64_t)(I * nb + il) * a.ld_r + J * 2 * S;
    double v0 = 0.0, v1 = 0.0;
    for (int s = 0; s < S; ++s) { v0 += (double)p[s]; v1 += (double)p[S + s]; }
    cpar[il] = v0;
    cpar[nb + il] = v1;
  }
  for (int o = threadIdx.x; o < 2 * mb; o += blockDim.x) {
    const int t = o / mb, jl = o % mb;
    const float* p = a.side_c + (int64_t)((I * 2 + t) * S) * a.ld_c + J * mb + jl;
    double v = 0.0;
    for (int s = 0; s < S; ++s) v += (double)p[(int64_t)s * a.ld_c];
    cpar[2 * nb + o] = v;
  }
  const double* ap = a.A_par + (int64_t)I * 2 * a.k;
  const double* bp = a.B_par + (int64_t)J * 2 * a.k;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  for (int l = threadIdx.x; l < a.k; l += blockDim.x) {
    const double a0 = ap[l], a1 = ap[a.k + l], b0 = bp[l], b1 = bp[a.k + l];
    acc[0] = fma(a0, b0, acc[0]); acc[1] = fma(a0, b1, acc[1]);
    acc[2] = fma(a1, b0, acc[2]); acc[3] = fma(a1, b1, acc[3]);
  }
  __shared__ double red[4][4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc[q] += __shfl_down(acc[q], off, 64);
  if ((threadIdx.x & 63) == 0)
#pragma unroll
    for (int q = 0; q < 4; ++q) red[threadIdx.x >> 6][q] = acc[q];
  __syncthreads();
  if (threadIdx.x < 4) cpar[2 * nb + 2 * mb + threadIdx.x] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
  if (threadIdx.x == 0) {
    reset_state(a.state + b);
    for (int f = 0; f < 4; ++f) a.itemmax[(int64_t)b * 4 + f] = 0.0;
    if (b == 0) *a.gate_word = PH_DONE;
  }
}

// fp64 parities -> rows of an operand of the product: `pieces` values of the operand's type per
// parity whose sum (in fp32 arithmetic of the product) restores 24 bits of it
__global__ __launch_bounds__(256) void split_parities_kernel(const double* par, void* W, int dtype, int lines, int k,
                                                             int pieces, int rows_padded) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)rows_padded * k) return;
  const int row = (int)(idx / k), l = (int)(idx % k);
  const int line_t = row / pieces, s = row % pieces;     // line_t = line * 2 + t
  double x = line_t < 2 * lines ? par[(int64_t)line_t * k + l] : 0.0;
  if (dtype == GECC_F32) {
    reinterpret_cast<float*>(W)[idx] = (float)x;
    return;
  }
  float piece = 0.f;
  for (int q = 0; q <= s; ++q) {          // hi, then what is left of it, then what is left of that
    uint32_t u = __float_as_uint((float)x);
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    piece = __uint_as_float(u);
    x -= (double)piece;
  }
  reinterpret_cast<uint16_t*>(W)[idx] = (uint16_t)(__float_as_uint(piece) >> 16);
}

}  // namespace

hipError_t launch_reset_state(const DecodeArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(reset_state_kernel, dim3((a.p.batch + 63) / 64), dim3(64), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_threshold(const DecodeArgs& a, hipStream_t st) {
  dim3 grid((a.p.n + a.p.m + 63) / 64, a.p.batch);   // 64 lines per workgroup: spreads over all CUs
  hipLaunchKernelGGL(threshold_kernel, grid, dim3(64 * TH_SLICES), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_summarize(const DecodeArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(summarize_kernel, dim3(a.p.batch), dim3(64), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_decode_c(const DecodeArgs& a, int with_summary, hipStream_t st) {
  hipLaunchKernelGGL(decode_c_kernel, dim3(a.p.batch), dim3(DC_THREADS), 0, st, a, with_summary);
  return hipGetLastError();
}

hipError_t launch_repair(const DecodeArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(repair_kernel<false>, dim3(a.p.batch), dim3(RP_THREADS), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_repair_blocked(const DecodeArgs& a, int nbi, hipStream_t st) {
  hipLaunchKernelGGL(repair_kernel<true>, dim3(a.p.batch), dim3(RP_THREADS), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(patch_operands_kernel, dim3(nbi + a.nbj), dim3(256), 0, st, a, nbi);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(final_decode_kernel, dim3(a.p.batch), dim3(DC_THREADS), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_threshold_blocked(const DecodeArgs& a, int n_full, int m_full, hipStream_t st) {
  const int64_t total = (int64_t)n_full * a.nbj + (int64_t)m_full * (n_full / a.p.n);
  hipLaunchKernelGGL(threshold_blocked_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, n_full, m_full);
  return hipGetLastError();
}

hipError_t launch_blocked_parities(const BlockedParityArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(blocked_parities_kernel, dim3(a.nbi * a.nbj), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_split_parities(const double* par, void* W, int dtype, int lines, int k, int pieces, int rows_padded,
                                 hipStream_t st) {
  const int64_t total = (int64_t)rows_padded * k;
  hipLaunchKernelGGL(split_parities_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, par, W, dtype, lines, k,
                     pieces, rows_padded);
  return hipGetLastError();
}


}  // namespace gecc
