// HBM-bound weighted reductions over an operand: parity encoding (Section III, A_P and B_P),
// the parity blocks of the encoded product (P_r = A B_P, P_c = A_P B) and the operand audit.
//
// Both kernels read the operand once with 16-byte loads that are contiguous across a
// wavefront, accumulate in fp64 and reduce in a fixed order (no floating-point atomics), so
// that re-forming a parity from an unchanged operand reproduces it bit for bit.
#include "gecc_internal.h"
#include <cstdlib>

namespace gecc {
namespace {

template <int DT> struct Elem;
template <> struct Elem<GECC_F32> {
  using type = float;
  static constexpr int VEC = 4;
  using raw = float4;
  static __device__ __forceinline__ raw load_raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
  static __device__ __forceinline__ void widen(const raw& x, double* v) {
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
  static __device__ __forceinline__ void load_vec(const float* p, double* v) { widen(load_raw(p), v); }
  static __device__ __forceinline__ double load_one(const float* p) { return (double)*p; }
};
template <> struct Elem<GECC_BF16> {
  using type = uint16_t;
  static constexpr int VEC = 8;
  using raw = uint4;
  static __device__ __forceinline__ raw load_raw(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  static __device__ __forceinline__ void widen(const raw& x, double* v) {
    uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = (double)__uint_as_float(w[i] << 16);
      v[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void load_vec(const uint16_t* p, double* v) { widen(load_raw(p), v); }
  static __device__ __forceinline__ double load_one(const uint16_t* p) {
    return (double)__uint_as_float(((uint32_t)*p) << 16);
  }
};

__device__ __forceinline__ bool gated_off(const int32_t* gate, int64_t stride, int b, int value) {
  if (!gate) return false;
  const int32_t g = *reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(gate) + stride * b);
  return g != value;
}

// The second stage of a column reduction adds the chunk partials of an output in one fixed order,
// whoever does it (a kernel of its own, workgroups carried by a row scan, or the last workgroup of
// the first stage): four slices, slice w over the chunks w, w + 4, ..., each with four running sums,
// combined as ((s0 + s1) + (s2 + s3)).
// One slice of G outputs at once (G independent chains of loads in flight); part[g]: chunk 0's
// partial of output g, stride: doubles between chunks.
// DEV: the partials were written by other workgroups of this launch (load_dev)
template <int G, bool DEV>
__device__ __forceinline__ void slice_sums(const double* const* part, int64_t stride, int nchunk, int w, double* s) {
  double t[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) { t[g][0] = 0.0; t[g][1] = 0.0; t[g][2] = 0.0; t[g][3] = 0.0; }
  int ch = w;
  for (; ch + 12 < nchunk; ch += 16) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const double* q = part[g] + (int64_t)(ch + 4 * u) * stride;
        t[g][u] += DEV ? load_dev(q) : *q;
      }
  }
  for (; ch < nchunk; ch += 4) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const double* q = part[g] + (int64_t)ch * stride;
      t[g][0] += DEV ? load_dev(q) : *q;
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) s[g] = (t[g][0] + t[g][1]) + (t[g][2] + t[g][3]);
}

// Stage 2 of coldot as workgroups of its own: 64 outputs per workgroup of 256 threads, wavefront w
// takes slice w.  scratch, out: of batch item b; red: 256 doubles of LDS.
__device__ __forceinline__ void coldot_stage2_body(const double* scratch, double* out, int Cc, int nchunk, int blk,
                                                   double* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int o = blk * 64 + lane;                   // index into [2][Cc]
  double s = 0.0;
  if (o < 2 * Cc) {
    const double* part = scratch + o;
    slice_sums<1, false>(&part, 2 * (int64_t)Cc, nchunk, wave, &s);
  }
  red[wave * 64 + lane] = s;
  __syncthreads();
  if (wave == 0 && o < 2 * Cc) out[o] = (red[lane] + red[64 + lane]) + (red[128 + lane] + red[192 + lane]);
}

// The same sums for the 2 * 64 * VEC outputs of one column segment, by the workgroup that finished
// the segment's last chunk.  col0: first column of the segment; red: 4 * 256 doubles of LDS.
template <int VEC>
__device__ __forceinline__ void coldot_finish_segment(const double* scratch, double* out, int Cc, int nchunk, int col0,
                                                      double* red) {
  constexpr int G = 4;                              // groups of 64 outputs a thread works on at once
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  static_assert((2 * VEC) % G == 0, "groups");
#pragma unroll 1
  for (int g0 = 0; g0 < 2 * VEC; g0 += G) {
    const double* part[G];
    int o[G];
    bool ok[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int t = (g0 + g) / VEC, col = col0 + ((g0 + g) % VEC) * 64 + lane;
      ok[g] = col < Cc;
      o[g] = t * Cc + min(col, Cc - 1);
      part[g] = scratch + o[g];
    }
    double s[G];
    slice_sums<G, true>(part, 2 * (int64_t)Cc, nchunk, wave, s);
#pragma unroll
    for (int g = 0; g < G; ++g) red[(g * 4 + wave) * 64 + lane] = s[g];
    __syncthreads();
    if (wave < G) {                                 // wavefront g writes group g
      const int g = wave;
      if (ok[g]) out[o[g]] = (red[(g * 4 + 0) * 64 + lane] + red[(g * 4 + 1) * 64 + lane]) +
                             (red[(g * 4 + 2) * 64 + lane] + red[(g * 4 + 3) * 64 + lane]);
    }
    __syncthreads();
  }
}

// Stage 2 of the row part of tile_scan (see below): the segments of a row added in order.
// part: [R][nseg][2], out: [2][R], both of batch item b.
template <bool DEV>
__device__ __forceinline__ void rowseg_sum(const double* part, double* out, int R, int nseg, int r) {
  const double* p = part + (int64_t)r * nseg * 2;
  double s0 = 0.0, s1 = 0.0;
  for (int g = 0; g < nseg; ++g) {
    s0 += DEV ? load_dev(p + 2 * g) : p[2 * g];
    s1 += DEV ? load_dev(p + 2 * g + 1) : p[2 * g + 1];
  }
  out[r] = s0;
  out[(int64_t)R + r] = s1;
}
// as workgroups of their own: 256 rows each
__device__ __forceinline__ void rowseg_stage2_body(const double* part, double* out, int R, int nseg, int blk) {
  const int r = blk * 256 + threadIdx.x;
  if (r < R) rowseg_sum<false>(part, out, R, nseg, r);
}

// a pending second stage (column chunks and / or row segments), by workgroup index
__device__ __forceinline__ void stage2_dispatch(const Stage2Job& j, int b, int blk, double* lds) {
  const int col_blocks = j.Cc > 0 ? (2 * j.Cc + 63) / 64 : 0;
  if (blk < col_blocks)
    coldot_stage2_body(j.scratch + (int64_t)b * j.nchunk * 2 * j.Cc, j.out + (int64_t)b * j.out_stride, j.Cc,
                       j.nchunk, blk, lds);
  else
    rowseg_stage2_body(j.row_scratch + (int64_t)b * j.R * j.nseg * 2, j.row_out + (int64_t)b * j.row_out_stride,
                       j.R, j.nseg, blk - col_blocks);
}

// -------------------------------------------------------------------------------------------
// rowdot: out[t][r] = sum_c w_t[c] X[r,c].   One workgroup owns RB rows and walks all columns;
// a thread keeps the weights of its VEC columns in registers and reuses them for the RB rows.
constexpr int RD_THREADS = 256;
constexpr int RD_BIG_RB = 16, RD_BIG_U = 1, RD_SMALL_RB = 4, RD_SMALL_U = 2;
constexpr int RD_BIG_RB_W = 8;   // with explicit weights (they take registers too)

// RD_RB rows per workgroup: 16 when there are rows enough to fill the chip, else 4.  RD_U column
// steps are taken together, so that a thread has RD_RB * RD_U independent 16-byte loads in
// flight before the first of them is used (the kernel is a stream over the operand: what it
// needs is memory-level parallelism, the arithmetic hides behind it).
// The rows bx * RD_RB ... of batch item b.  red: RD_RB * RD_THREADS doubles of LDS.  The sums of a row
// do not depend on RD_RB or RD_U (a thread adds its columns in ascending order either way).
template <int DT, bool IDXW, int RD_RB, int RD_U>
__device__ __forceinline__ void rowdot_body(const ScanArgs& a, int bx, int b, double* lds) {
  using E = Elem<DT>;
  using T = typename E::type;
  constexpr int VEC = E::VEC;
  constexpr int STEP = RD_THREADS * VEC;   // columns one pass of the workgroup covers
  const T* X = reinterpret_cast<const T*>(a.X) + (int64_t)b * a.xs;
  const double* w0 = IDXW ? nullptr : a.w + (int64_t)b * a.w_stride;
  const double* w1 = IDXW ? nullptr : w0 + a.Cc;
  double* out = a.out + (int64_t)b * a.out_stride;
  const int r0 = bx * RD_RB;
  const int tid = threadIdx.x;

  double acc0[RD_RB], acc1[RD_RB];
#pragma unroll
  for (int r = 0; r < RD_RB; ++r) { acc0[r] = 0.0; acc1[r] = 0.0; }

  // whole vectors for every thread: rows past the end are clamped to the last one (their sums
  // are computed and never stored), so the body has no branches
  int c0 = 0;
  if (a.vec_ok) {
    for (; c0 + RD_U * STEP <= a.Cc; c0 += RD_U * STEP) {
      typename E::raw x[RD_U][RD_RB];
      double wa[RD_U][VEC], wb[RD_U][VEC];
#pragma unroll
      for (int u = 0; u < RD_U; ++u) {
        const int c = c0 + u * STEP + tid * VEC;
#pragma unroll
        for (int r = 0; r < RD_RB; ++r)
          x[u][r] = E::load_raw(X + (int64_t)min(r0 + r, a.R - 1) * a.ld + (unsigned)c);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          if (IDXW) { wa[u][e] = 1.0; wb[u][e] = (double)(c + e + 1); }
          else      { wa[u][e] = w0[c + e]; wb[u][e] = w1[c + e]; }
        }
      }
#pragma unroll
      for (int u = 0; u < RD_U; ++u) {
#pragma unroll
        for (int r = 0; r < RD_RB; ++r) {
          double v[VEC];
          E::widen(x[u][r], v);
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            acc0[r] = IDXW ? acc0[r] + v[e] : fma(wa[u][e], v[e], acc0[r]);
            acc1[r] = fma(wb[u][e], v[e], acc1[r]);
          }
          __builtin_amdgcn_sched_barrier(0);   // widen one vector at a time (registers)
        }
      }
    }
  }
  // the remaining columns (and everything, if the rows are not 16-byte aligned)
  for (; c0 < a.Cc; c0 += STEP) {
    const int c = c0 + tid * VEC;
    if (c >= a.Cc) continue;
    const int nv = min(VEC, a.Cc - c);
    double wa[VEC], wb[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      if (IDXW) { wa[e] = 1.0; wb[e] = (double)(c + e + 1); }
      else      { wa[e] = e < nv ? w0[c + e] : 0.0; wb[e] = e < nv ? w1[c + e] : 0.0; }
    }
    if (nv == VEC && a.vec_ok) {
      typename E::raw x[RD_RB];
#pragma unroll
      for (int r = 0; r < RD_RB; ++r) x[r] = E::load_raw(X + (int64_t)min(r0 + r, a.R - 1) * a.ld + c);
#pragma unroll
      for (int r = 0; r < RD_RB; ++r) {
        double v[VEC];
        E::widen(x[r], v);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          acc0[r] = IDXW ? acc0[r] + v[e] : fma(wa[e], v[e], acc0[r]);
          acc1[r] = fma(wb[e], v[e], acc1[r]);
        }
      }
    } else {
      for (int r = 0; r < RD_RB; ++r) {
        const int row = r0 + r;
        if (row < a.R)
          for (int e = 0; e < nv; ++e) {
            const double v = E::load_one(X + (int64_t)row * a.ld + c + e);
            acc0[r] = fma(wa[e], v, acc0[r]);
            acc1[r] = fma(wb[e], v, acc1[r]);
          }
      }
    }
  }

  // fixed-order reduction over the 256 threads, one parity kind (t) at a time
  double (*red)[RD_THREADS] = reinterpret_cast<double (*)[RD_THREADS]>(lds);
  const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    if (t) __syncthreads();
#pragma unroll
    for (int r = 0; r < RD_RB; ++r) red[r][tid] = t ? acc1[r] : acc0[r];
    __syncthreads();
    for (int q = wave; q < RD_RB; q += RD_THREADS / 64) {
      double s = (red[q][lane] + red[q][lane + 64]) + (red[q][lane + 128] + red[q][lane + 192]);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
      const int row = r0 + q;
      if (lane == 0 && row < a.R) out[(int64_t)t * a.R + row] = s;
    }
  }
}

// GATED: the launch belongs to the operand audit and returns at once unless the decoder asked for
// it (a separate instantiation, so that profiles list encoding and audit launches apart).
template <int DT, bool IDXW, int RD_RB, int RD_U, bool GATED>
__global__ __launch_bounds__(RD_THREADS) void rowdot_kernel(ScanArgs a) {
  __shared__ double lds[RD_RB * RD_THREADS];
  const int b = blockIdx.y;
  if (GATED && gated_off(a.gate, a.gate_stride, b, a.gate_value)) return;
  const int own = (int)gridDim.x - a.carry_blocks;
  if ((int)blockIdx.x >= own) {   // carried second stage of an earlier column / tile scan
    stage2_dispatch(a.carry, b, (int)blockIdx.x - own, lds);
    return;
  }
  rowdot_body<DT, IDXW, RD_RB, RD_U>(a, blockIdx.x, b, lds);
}

// -------------------------------------------------------------------------------------------
// coldot: out[t][c] = sum_r w_t[r] X[r,c].   Stage 1: a workgroup owns 64*VEC columns and one
// chunk of SCAN_CHUNK_ROWS rows; its 4 wavefronts interleave the rows and are combined through
// LDS.  Stage 2 adds the chunks in order.
constexpr int CD_THREADS = 256;

// LDS of a coldot workgroup: the four wavefronts' sums, reused by the last workgroup of a segment
constexpr int CD_LDS_DOUBLES = 4 * 2 * 8 * 64;
constexpr int CD_FLAG_AT = 1024;     // (behind what coldot_finish_segment uses)

// Column segment bx, chunk `chunk` of batch item b.  With a.done set, the workgroup that finishes a
// segment's last chunk also adds the chunks up (no second stage to launch).
template <int DT, bool IDXW>
__device__ __forceinline__ void coldot_body(const ScanArgs& a, int nchunk, int nsegx, int bx, int chunk, int b,
                                            double* lds) {
  using E = Elem<DT>;
  using T = typename E::type;
  constexpr int VEC = E::VEC;
  const T* X = reinterpret_cast<const T*>(a.X) + (int64_t)b * a.xs;
  const double* w0 = IDXW ? nullptr : a.w + (int64_t)b * a.w_stride;
  const double* w1 = IDXW ? nullptr : w0 + a.R;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = (bx * 64 + lane) * VEC;
  const int rbeg = chunk * SCAN_CHUNK_ROWS;
  const int rend = min(a.R, rbeg + SCAN_CHUNK_ROWS);
  const int nv = min(VEC, a.Cc - c);   // <= 0: this lane owns no column

  double acc0[VEC], acc1[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { acc0[e] = 0.0; acc1[e] = 0.0; }

  if (nv == VEC && a.vec_ok) {
    // Batches of CD_NB rows per wavefront, double buffered: the loads of the next batch are in
    // flight while this one is added up (a wavefront walks its rows one batch after the other,
    // so without this every batch would pay the full memory latency).
    constexpr int CD_NB = 8;
    typename E::raw xa[CD_NB], xb[CD_NB];
    const T* col = X + c;
    auto load = [&](typename E::raw* x, int rr) {
#pragma unroll
      for (int u = 0; u < CD_NB; ++u) x[u] = E::load_raw(col + (int64_t)(rr + 4 * u) * a.ld);
    };
    auto add = [&](const typename E::raw* x, int rr) {
#pragma unroll
      for (int u = 0; u < CD_NB; ++u) {
        double v[VEC];
        E::widen(x[u], v);
        const int row = rr + 4 * u;
        const double wa = IDXW ? 1.0 : w0[row];
        const double wb = IDXW ? (double)(row + 1) : w1[row];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          acc0[e] = IDXW ? acc0[e] + v[e] : fma(wa, v[e], acc0[e]);
          acc1[e] = fma(wb, v[e], acc1[e]);
        }
      }
    };
    int r = rbeg + wave;
    const int cnt = r < rend ? (rend - r + 3) / 4 : 0;   // rows of this wavefront
    const int nb = cnt / CD_NB;
    constexpr int STEP = 4 * CD_NB;
    if (nb > 0) {
      load(xa, r);
      int bi = 0;
      for (; bi + 1 < nb; bi += 2) {
        load(xb, r + STEP);
        add(xa, r);
        if (bi + 2 < nb) load(xa, r + 2 * STEP);
        add(xb, r + STEP);
        r += 2 * STEP;
      }
      if (bi < nb) { add(xa, r); r += STEP; }
    }
    for (; r < rend; r += 4) {
      double v[VEC];
      E::load_vec(col + (int64_t)r * a.ld, v);
      const double wa = IDXW ? 1.0 : w0[r];
      const double wb = IDXW ? (double)(r + 1) : w1[r];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        acc0[e] = IDXW ? acc0[e] + v[e] : fma(wa, v[e], acc0[e]);
        acc1[e] = fma(wb, v[e], acc1[e]);
      }
    }
  } else if (nv > 0) {
    for (int r = rbeg + wave; r < rend; r += 4) {
      const double wa = IDXW ? 1.0 : w0[r];
      const double wb = IDXW ? (double)(r + 1) : w1[r];
      for (int e = 0; e < nv; ++e) {
        const double v = E::load_one(X + (int64_t)r * a.ld + c + e);
        acc0[e] = fma(wa, v, acc0[e]);
        acc1[e] = fma(wb, v, acc1[e]);
      }
    }
  }

  double (*red)[2][VEC][64] = reinterpret_cast<double (*)[2][VEC][64]>(lds);
#pragma unroll
  for (int e = 0; e < VEC; ++e) { red[wave][0][e][lane] = acc0[e]; red[wave][1][e][lane] = acc1[e]; }
  __syncthreads();
  // thread -> (t, e, lane'): 2*VEC*64 outputs, 256 threads
  double* part = a.scratch + ((int64_t)b * nchunk + chunk) * 2 * a.Cc;
  for (int o = tid; o < 2 * VEC * 64; o += CD_THREADS) {
    const int l = o & 63, e = (o >> 6) % VEC, t = o / (64 * VEC);
    const int col = (bx * 64 + l) * VEC + e;
    if (col < a.Cc) {
      const double s = (red[0][t][e][l] + red[1][t][e][l]) + (red[2][t][e][l] + red[3][t][e][l]);
      // (written through only when another workgroup of this launch reads it: such stores cost more)
      if (a.done) store_dev(part + (int64_t)t * a.Cc + col, s);
      else part[(int64_t)t * a.Cc + col] = s;
    }
  }
  if (a.done && arrive_last(a.done + (int64_t)b * nsegx + bx, (uint32_t)nchunk, reinterpret_cast<int*>(lds + CD_FLAG_AT)))
    coldot_finish_segment<VEC>(a.scratch + (int64_t)b * nchunk * 2 * a.Cc, a.out + (int64_t)b * a.out_stride, a.Cc,
                               nchunk, bx * 64 * VEC, lds);
}

template <int DT, bool IDXW, bool GATED>
__global__ __launch_bounds__(CD_THREADS) void coldot_stage1(ScanArgs a, int nchunk) {
  __shared__ double lds[CD_LDS_DOUBLES];
  const int b = blockIdx.z;
  if (GATED && gated_off(a.gate, a.gate_stride, b, a.gate_value)) return;
  coldot_body<DT, IDXW>(a, nchunk, gridDim.x, blockIdx.x, blockIdx.y, b, lds);
}

__global__ __launch_bounds__(256) void coldot_stage2(Stage2Job j) {
  __shared__ double lds[256];
  const int b = blockIdx.y;
  if (gated_off(j.gate, j.gate_stride, b, j.gate_value)) return;
  stage2_dispatch(j, b, blockIdx.x, lds);
}

// -------------------------------------------------------------------------------------------
// tile_scan: both reductions of an operand in ONE pass over it.
//   column part  out_col[t][c] = sum_r wr_t[r] X[r,c]      (two-stage, like coldot)
//   row part     out_row[t][r] = sum_c wc_t[c] X[r,c]      (two-stage: per 64*VEC-column segment)
// Each part has either the index weights of Section III (1, index + 1) or two fp64 vectors.  With
// both parts on, encoding an operand (A_P, index weights along one axis) and its parity block of
// C-bar (P_r = A B_P, vector weights along the other) cost one read of the operand instead of two.
// A part switched off costs nothing; a part computes the same sums in the same order whether the
// other one is on or not, so the gated audit (one part) reproduces an encoding (maybe both) bit for
// bit.  All products go through fma(), never a*b+c, for the same reason.
//
// A workgroup is four wavefronts on one segment of 64*VEC columns; each walks its own quarter of
// the chunk's rows, TS_RB rows (loads) at a time; three wavefronts share a SIMD and cover each
// other's waits.  The kernel is bound by its arithmetic as much as by memory: per 16 bytes a lane
// spends 8 conversions and 32 fp64 operations, which issue at half rate, about 380 cycles per row
// and wavefront (measured: its loads alone stream at 5.8 TB/s, the whole kernel at 4.4; more loads in
// flight, 8-byte lanes, rows DMA'd into an LDS ring or workgroups that read 4 KiB of every row
// change nothing).  A lane keeps the column sums of its VEC columns in registers for the whole walk.
// The row sums of a block of rows (TS_RB rows x 2 kinds, one partial per lane) are transposed through
// LDS and added by four lanes per output; only the wavefront's own LDS region is involved, so no
// workgroup barrier sits in the loop.
constexpr int TS_THREADS = 256;
constexpr int TS_RB = 8;            // rows per block of loads
constexpr int TS_LDS_LD = 65;       // doubles per output row of the transpose (64 lanes + 1: conflict-free)

struct TileScanArgs {
  const void* X;
  int dtype;
  int R, Cc;
  int64_t ld, xs;
  int batch;
  const double* wr;       // column part: row weights [2][R] per batch item (null: index weights)
  int64_t wr_stride;
  double* col_part;       // [batch][nchunk][2][Cc]
  const double* wc;       // row part: column weights [2][Cc] per batch item (null: index weights)
  int64_t wc_stride;
  double* row_part;       // [batch][R][nseg][2]
  int chunk_rows, nchunk, nseg;
  const int32_t* gate;
  int64_t gate_stride;
  int gate_value;
  // With done_col set, the last workgroup of a column segment adds the segment's chunks up; with
  // done_row set, the last one of a chunk of rows adds the row partials of its rows: that part
  // then has no second stage to launch.
  uint32_t* done_col;     // [batch][nseg]
  uint32_t* done_row;     // [batch][nchunk]
  double* col_out; int64_t col_out_stride;
  double* row_out; int64_t row_out_stride;
};
constexpr int TS_FLAG_AT = 1024;   // doubles into the LDS: behind what coldot_finish_segment uses

// wavefront-local ordering of LDS traffic: the hardware keeps a wavefront's LDS instructions in
// order; this keeps the compiler from moving them across
// (a compiler barrier only: a fence instruction would also wait for the wavefront's outstanding
// global loads and stores, which is exactly what the loop must not do)
__device__ __forceinline__ void wave_lds_fence() { asm volatile("" ::: "memory"); }

constexpr int TS_LDS_DOUBLES = 4 * 2 * TS_RB * TS_LDS_LD;

// segment `seg` of the columns, chunk `chunk` of the rows, batch item b; ts_lds: TS_LDS_DOUBLES of LDS
template <int DT, bool COL, bool ROW, bool COL_IDX, bool ROW_IDX>
__device__ __forceinline__ void tile_scan_body(const TileScanArgs& a, int seg, int chunk, int b, double* ts_lds) {
  using E = Elem<DT>;
  using T = typename E::type;
  constexpr int VEC = E::VEC;
  constexpr int SEG = 64 * VEC;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const T* X = reinterpret_cast<const T*>(a.X) + (int64_t)b * a.xs;
  // columns of this lane (Cc is a multiple of VEC; lanes past the end read the last vector and drop it)
  const int c_true = seg * SEG + lane * VEC;
  const bool lane_ok = c_true < a.Cc;
  const int c = lane_ok ? c_true : a.Cc - VEC;
  const T* col = X + c;
  // rows of this wavefront: a quarter of the chunk (multiple of TS_RB, so only the last has a tail)
  const int rbeg = chunk * a.chunk_rows;
  const int rend = min(a.R, rbeg + a.chunk_rows);
  const int quarter = a.chunk_rows >> 2;
  const int w_beg = min(rend, rbeg + wave * quarter), w_end = min(rend, w_beg + quarter);

  const double* wr0 = (COL && !COL_IDX) ? a.wr + (int64_t)b * a.wr_stride : nullptr;
  const double* wr1 = (COL && !COL_IDX) ? wr0 + a.R : nullptr;
  double wc0[VEC], wc1[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    if (ROW && !ROW_IDX) {
      const double* w = a.wc + (int64_t)b * a.wc_stride;
      wc0[e] = w[c + e]; wc1[e] = w[a.Cc + c + e];
    } else {
      wc0[e] = 1.0; wc1[e] = (double)(c + e + 1);
    }
  }
  double ca0[VEC], ca1[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { ca0[e] = 0.0; ca1[e] = 0.0; }

  double* tr = ts_lds + wave * (2 * TS_RB * TS_LDS_LD);     // this wavefront's transpose region
  double* rp_out = ROW ? a.row_part + ((int64_t)b * a.R * a.nseg + seg) * 2 : nullptr;

  // one row into the column sums; its two row partials go straight into the transpose region
  auto take = [&](const typename E::raw& x, int u, double u0, double u1) {
    double v[VEC];
    E::widen(x, v);
    if (COL) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        ca0[e] = COL_IDX ? ca0[e] + v[e] : fma(u0, v[e], ca0[e]);
        ca1[e] = fma(u1, v[e], ca1[e]);
        // (pins the update to this row: left alone, the compiler keeps the widened values of all
        // the rows of a block alive and adds them up at the end, at the cost of half the occupancy)
        asm volatile("" : "+v"(ca0[e]), "+v"(ca1[e]));
      }
    }
    if (ROW) {
      double s0 = 0.0, s1 = 0.0;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        s0 = ROW_IDX ? s0 + v[e] : fma(wc0[e], v[e], s0);
        s1 = fma(wc1[e], v[e], s1);
      }
      tr[(2 * u) * TS_LDS_LD + lane] = lane_ok ? s0 : 0.0;
      tr[(2 * u + 1) * TS_LDS_LD + lane] = lane_ok ? s1 : 0.0;
    }
  };
  // row partials of `cnt` rows starting at r0: LDS -> four lanes per output add 16 lanes' values each
  auto emit_rows = [&](int r0, int cnt) {
    wave_lds_fence();
    const int o = lane >> 2, q = lane & 3;      // output (row u = o / 2, kind t = o % 2), quarter of the lanes
    // (all sixteen reads are issued before the first is used: one wait instead of eight)
    double part[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) part[i] = tr[o * TS_LDS_LD + q * 16 + i];
    __builtin_amdgcn_sched_barrier(0);
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += part[i];
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);
    wave_lds_fence();
    const int u = o >> 1, t = o & 1;
    if (q == 0 && u < cnt) {
      double* dst = rp_out + (int64_t)(r0 + u) * a.nseg * 2 + t;
      if (a.done_row) store_dev(dst, s); else *dst = s;
    }
  };

  int r = w_beg;
  const int nfull = (w_end - w_beg) / TS_RB;
  if (nfull > 0) {
    typename E::raw xa[TS_RB];
    auto load = [&](typename E::raw* x, int rr) {
#pragma unroll
      for (int u = 0; u < TS_RB; ++u) x[u] = E::load_raw(col + (int64_t)(rr + u) * a.ld);
    };
    auto work = [&](const typename E::raw* x, int rr) {
      // the row weights of the whole block first (uniform loads: one wait, not one per row)
      double u0[TS_RB], u1[TS_RB];
#pragma unroll
      for (int u = 0; u < TS_RB; ++u) {
        u0[u] = (COL && !COL_IDX) ? wr0[rr + u] : 1.0;
        u1[u] = (COL && !COL_IDX) ? wr1[rr + u] : (double)(rr + u + 1);
      }
#pragma unroll
      for (int u = 0; u < TS_RB; ++u) {
        take(x[u], u, u0[u], u1[u]);
        __builtin_amdgcn_sched_barrier(0);   // one row at a time: widening all of them first costs the occupancy
      }
      if (ROW) emit_rows(rr, TS_RB);
    };
    for (int bi = 0; bi < nfull; ++bi) {
      load(xa, r);
      work(xa, r);
      r += TS_RB;
    }
  }
  if (r < w_end) {     // the last rows of the operand: fewer than TS_RB
    const int cnt = w_end - r;
    for (int u = 0; u < TS_RB; ++u) {
      if (u < cnt) {
        take(E::load_raw(col + (int64_t)(r + u) * a.ld), u, (COL && !COL_IDX) ? wr0[r + u] : 1.0,
             (COL && !COL_IDX) ? wr1[r + u] : (double)(r + u + 1));
      } else if (ROW) {
        tr[(2 * u) * TS_LDS_LD + lane] = 0.0;
        tr[(2 * u + 1) * TS_LDS_LD + lane] = 0.0;
      }
    }
    if (ROW) emit_rows(r, cnt);
  }

  if (COL) {
    // the four quarters of the chunk, combined in order
    __syncthreads();
    double* cb = ts_lds;                          // [4][2 * VEC][64]
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      cb[(wave * 2 * VEC + e) * 64 + lane] = ca0[e];
      cb[(wave * 2 * VEC + VEC + e) * 64 + lane] = ca1[e];
    }
    __syncthreads();
    double* part = a.col_part + ((int64_t)b * a.nchunk + chunk) * 2 * a.Cc;
    for (int o = threadIdx.x; o < 2 * VEC * 64; o += TS_THREADS) {
      const int l = o & 63, e = (o >> 6) % VEC, t = o / (64 * VEC);
      const int cc = seg * SEG + l * VEC + e;
      if (cc < a.Cc) {
        const int x = (t * VEC + e) * 64 + l;
        const double v = (cb[x] + cb[2 * VEC * 64 + x]) + (cb[2 * 2 * VEC * 64 + x] + cb[3 * 2 * VEC * 64 + x]);
        if (a.done_col) store_dev(part + (int64_t)t * a.Cc + cc, v);
        else part[(int64_t)t * a.Cc + cc] = v;
      }
    }
  }

  if ((COL && a.done_col) || (ROW && a.done_row)) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's partial results have been written through
    __syncthreads();
    int* flag = reinterpret_cast<int*>(ts_lds + TS_FLAG_AT);
    if (threadIdx.x == 0) {
      flag[0] = (COL && a.done_col) ? atomicInc(a.done_col + (int64_t)b * a.nseg + seg, (uint32_t)a.nchunk - 1) == (uint32_t)a.nchunk - 1 : 0;
      flag[1] = (ROW && a.done_row) ? atomicInc(a.done_row + (int64_t)b * a.nchunk + chunk, (uint32_t)a.nseg - 1) == (uint32_t)a.nseg - 1 : 0;
    }
    __syncthreads();
    const bool last_col = flag[0] != 0, last_row = flag[1] != 0;
    if (ROW && last_row) {
      const double* part = a.row_part + (int64_t)b * a.R * a.nseg * 2;
      double* out = a.row_out + (int64_t)b * a.row_out_stride;
      for (int rr = rbeg + (int)threadIdx.x; rr < rend; rr += TS_THREADS) rowseg_sum<true>(part, out, a.R, a.nseg, rr);
    }
    if (COL && last_col)
      coldot_finish_segment<VEC>(a.col_part + (int64_t)b * a.nchunk * 2 * a.Cc, a.col_out + (int64_t)b * a.col_out_stride,
                                 a.Cc, a.nchunk, seg * SEG, ts_lds);
  }
}

template <int DT, bool COL, bool ROW, bool COL_IDX, bool ROW_IDX, bool GATED>
__global__ __launch_bounds__(TS_THREADS) void tile_scan(TileScanArgs a) {
  extern __shared__ double ts_lds[];
  const int b = blockIdx.z;
  if (GATED && gated_off(a.gate, a.gate_stride, b, a.gate_value)) return;
  tile_scan_body<DT, COL, ROW, COL_IDX, ROW_IDX>(a, blockIdx.x, blockIdx.y, b, ts_lds);
}

// -------------------------------------------------------------------------------------------
// The two gated re-encodings of the operand audit in one launch: on a clean step each of them only
// finds its gate closed, and a dependent launch costs about 5 us of stream time whatever it does.
// When the audit does run, every column reduction in here is finished by the workgroup that comes
// last to its segment (a.done / done_col / done_row set): that tail costs about what the launch of a
// second stage would, so it is used here only, where it saves a launch on every clean step.
struct PairJob {
  int kind;          // PJ_x
  ScanArgs s;        // PJ_ROW, PJ_COL
  TileScanArgs t;    // PJ_TILE_COL, PJ_TILE_ROW
  int nblk;          // workgroups of this job
  int gx, gy;        // workgroups per batch item: gx (rowdot) or gx x gy (segments x chunks)
};
enum : int { PJ_ROW = 0, PJ_COL = 1, PJ_TILE_COL = 2, PJ_TILE_ROW = 3, PJ_ROW_BIG = 4 };
struct PairArgs { PairJob j[2]; };
constexpr int AUDIT_PAIR_MAX_BLOCKS = 5120;
constexpr int PAIR_LDS_DOUBLES = TS_LDS_DOUBLES > CD_LDS_DOUBLES ? TS_LDS_DOUBLES : CD_LDS_DOUBLES;

template <int DT>
__global__ __launch_bounds__(256) void audit_pair(PairArgs p) {
  __shared__ double lds[PAIR_LDS_DOUBLES];
  int v = blockIdx.x;
  const bool second = v >= p.j[0].nblk;
  if (second) v -= p.j[0].nblk;
  const PairJob& j = second ? p.j[1] : p.j[0];
  const int per_item = j.gx * j.gy;
  const int b = v / per_item, x = (v % per_item) % j.gx, y = (v % per_item) / j.gx;
  if (j.kind == PJ_ROW) {
    if (gated_off(j.s.gate, j.s.gate_stride, b, j.s.gate_value)) return;
    rowdot_body<DT, true, RD_SMALL_RB, RD_SMALL_U>(j.s, x, b, lds);
  } else if (j.kind == PJ_ROW_BIG) {
    if (gated_off(j.s.gate, j.s.gate_stride, b, j.s.gate_value)) return;
    rowdot_body<DT, true, RD_BIG_RB, RD_BIG_U>(j.s, x, b, lds);
  } else if (j.kind == PJ_COL) {
    if (gated_off(j.s.gate, j.s.gate_stride, b, j.s.gate_value)) return;
    coldot_body<DT, true>(j.s, j.gy, j.gx, x, y, b, lds);
  } else {
    if (gated_off(j.t.gate, j.t.gate_stride, b, j.t.gate_value)) return;
    if (j.kind == PJ_TILE_COL) tile_scan_body<DT, true, false, true, true>(j.t, x, y, b, lds);
    else tile_scan_body<DT, false, true, true, true>(j.t, x, y, b, lds);
  }
}

// vector loads need 16-byte aligned rows
bool vec_ok(const ScanArgs& a) {
  const int vec = a.dtype == GECC_BF16 ? 8 : 4;
  const size_t esz = a.dtype == GECC_BF16 ? 2 : 4;
  return (reinterpret_cast<uintptr_t>(a.X) % 16 == 0) && (a.ld % vec == 0) && ((a.xs * esz) % 16 == 0);
}

}  // namespace

size_t coldot_scratch_doubles(int R, int Cc, int batch) {
  const size_t nchunk = (R + SCAN_CHUNK_ROWS - 1) / SCAN_CHUNK_ROWS;
  return (size_t)batch * nchunk * 2 * (size_t)Cc;
}

hipError_t launch_rowdot(const ScanArgs& a0, const Stage2Job* carry, hipStream_t st) {
  ScanArgs a = a0;
  a.vec_ok = vec_ok(a0) ? 1 : 0;
  a.carry_blocks = 0;
  if (carry && carry->valid) {
    if (carry->batch != a.batch || carry->gate != a.gate || carry->gate_stride != a.gate_stride ||
        carry->gate_value != a.gate_value)
      return hipErrorInvalidValue;
    a.carry = *carry;
    a.carry_blocks = stage2_blocks(*carry);
  }
  const int extra = a.carry_blocks;
  const bool idx = a.w == nullptr;
  const bool small = (int64_t)((a.R + RD_BIG_RB - 1) / RD_BIG_RB) * a.batch < 1024;   // fewer than 4 workgroups per CU
  const bool gated = a.gate != nullptr;   // audits only, and audits use the index weights
#define GECC_LAUNCH_ROWDOT(DT, IDX, G)                                                               \
  do {                                                                                              \
    constexpr int BIG = IDX ? RD_BIG_RB : RD_BIG_RB_W;                                                \
    if (small) hipLaunchKernelGGL((rowdot_kernel<DT, IDX, RD_SMALL_RB, RD_SMALL_U, G>),               \
                                  dim3((a.R + RD_SMALL_RB - 1) / RD_SMALL_RB + extra, a.batch),       \
                                  dim3(RD_THREADS), 0, st, a);                                        \
    else       hipLaunchKernelGGL((rowdot_kernel<DT, IDX, BIG, RD_BIG_U, G>),                         \
                                  dim3((a.R + BIG - 1) / BIG + extra, a.batch),                       \
                                  dim3(RD_THREADS), 0, st, a);                                        \
  } while (0)
  if (gated && !idx) return hipErrorInvalidValue;
  if (a.dtype == GECC_BF16) {
    if (gated) GECC_LAUNCH_ROWDOT(GECC_BF16, true, true);
    else if (idx) GECC_LAUNCH_ROWDOT(GECC_BF16, true, false);
    else GECC_LAUNCH_ROWDOT(GECC_BF16, false, false);
  } else {
    if (gated) GECC_LAUNCH_ROWDOT(GECC_F32, true, true);
    else if (idx) GECC_LAUNCH_ROWDOT(GECC_F32, true, false);
    else GECC_LAUNCH_ROWDOT(GECC_F32, false, false);
  }
#undef GECC_LAUNCH_ROWDOT
  return hipGetLastError();
}

int coldot_done_words(const ScanArgs& a) {
  const int vec = a.dtype == GECC_BF16 ? 8 : 4;
  const int nchunk = (a.R + SCAN_CHUNK_ROWS - 1) / SCAN_CHUNK_ROWS;
  if (nchunk > SCAN_FUSE_MAX_CHUNKS) return 0;
  const int64_t words = (int64_t)((a.Cc + 64 * vec - 1) / (64 * vec)) * a.batch;
  return words <= SCAN_DONE_WORDS ? (int)words : 0;
}

hipError_t launch_coldot_stage1(const ScanArgs& a0, Stage2Job* pending, hipStream_t st) {
  ScanArgs a = a0;
  a.vec_ok = vec_ok(a0) ? 1 : 0;
  a.carry_blocks = 0;
  const int vec = a.dtype == GECC_BF16 ? 8 : 4;
  const int nchunk = (a.R + SCAN_CHUNK_ROWS - 1) / SCAN_CHUNK_ROWS;
  dim3 grid((a.Cc + 64 * vec - 1) / (64 * vec), nchunk, a.batch);
  const bool idx = a.w == nullptr, gated = a.gate != nullptr;
  if (gated && !idx) return hipErrorInvalidValue;
  if (a.done && coldot_done_words(a) == 0) return hipErrorInvalidValue;
  if (a.dtype == GECC_BF16) {
    if (gated)    hipLaunchKernelGGL((coldot_stage1<GECC_BF16, true, true>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else if (idx) hipLaunchKernelGGL((coldot_stage1<GECC_BF16, true, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else          hipLaunchKernelGGL((coldot_stage1<GECC_BF16, false, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
  } else {
    if (gated)    hipLaunchKernelGGL((coldot_stage1<GECC_F32, true, true>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else if (idx) hipLaunchKernelGGL((coldot_stage1<GECC_F32, true, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else          hipLaunchKernelGGL((coldot_stage1<GECC_F32, false, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
  }
  *pending = Stage2Job{};
  if (!a.done) {
    pending->valid = true;
    pending->scratch = a.scratch; pending->out = a.out; pending->out_stride = a.out_stride;
    pending->Cc = a.Cc; pending->nchunk = nchunk; pending->batch = a.batch;
    pending->gate = a.gate; pending->gate_stride = a.gate_stride; pending->gate_value = a.gate_value;
  }
  return hipGetLastError();
}

// ---- tile_scan ------------------------------------------------------------------------------
bool tile_scan_ok(const TileScanJob& t) {
  const int vec = t.dtype == GECC_BF16 ? 8 : 4;
  const size_t esz = t.dtype == GECC_BF16 ? 2 : 4;
  return reinterpret_cast<uintptr_t>(t.X) % 16 == 0 && t.ld % vec == 0 && (t.xs * esz) % 16 == 0 &&
         t.Cc % vec == 0 && t.Cc >= vec && t.R >= 1;
}

int tile_scan_segments(int Cc, int dtype) {
  const int seg = 64 * (dtype == GECC_BF16 ? 8 : 4);
  return (Cc + seg - 1) / seg;
}

size_t tile_scan_row_scratch_doubles(int R, int Cc, int dtype, int batch) {
  return (size_t)batch * (size_t)R * tile_scan_segments(Cc, dtype) * 2;
}

// rows per chunk: 128 (the chunk the column scratch is sized for) or, as long as two workgroups per
// compute unit remain, 256 or 512 (fewer column partial sums to write and read back; measured at
// 16384 x 4096: 30.3 us with 256-row chunks against 32.3 with 128)
static int tile_scan_chunk_rows(int R, int nseg, int batch) {
  int ch = SCAN_CHUNK_ROWS;
  while (ch < 512 && (int64_t)nseg * ((R + 2 * ch - 1) / (2 * ch)) * batch * 4 >= 2048) ch *= 2;
  return ch;
}

// kernel arguments of a tile scan; fuse_col / fuse_row: parts that finish by themselves (t.done set:
// the column part when a segment has few enough chunks for one workgroup to add up, the row part
// always -- as far as the counters reach).  done_words: counters used.
static bool make_tile_args(const TileScanJob& t, TileScanArgs& a, bool& fuse_col, bool& fuse_row, int& done_words) {
  if (!tile_scan_ok(t) || (!t.col_on && !t.row_on)) return false;
  a = TileScanArgs{};
  a.X = t.X; a.dtype = t.dtype; a.R = t.R; a.Cc = t.Cc; a.ld = t.ld; a.xs = t.xs; a.batch = t.batch;
  a.wr = t.wr; a.wr_stride = t.wr_stride; a.col_part = t.col_scratch;
  a.wc = t.wc; a.wc_stride = t.wc_stride; a.row_part = t.row_scratch;
  a.nseg = tile_scan_segments(t.Cc, t.dtype);
  // (larger chunks only save column partial sums: a row part alone takes the smallest, for the balance)
  a.chunk_rows = t.col_on ? tile_scan_chunk_rows(t.R, a.nseg, t.batch) : SCAN_CHUNK_ROWS;
  a.nchunk = (t.R + a.chunk_rows - 1) / a.chunk_rows;
  a.gate = t.gate; a.gate_stride = t.gate_stride; a.gate_value = t.gate_value;
  fuse_col = false; fuse_row = false;
  int64_t used = 0;
  if (t.done) {
    if (t.col_on && a.nchunk <= SCAN_FUSE_MAX_CHUNKS && (int64_t)t.batch * a.nseg <= SCAN_DONE_WORDS) {
      fuse_col = true; a.done_col = t.done; used = (int64_t)t.batch * a.nseg;
    }
    if (t.row_on && used + (int64_t)t.batch * a.nchunk <= SCAN_DONE_WORDS) {
      fuse_row = true; a.done_row = t.done + used; used += (int64_t)t.batch * a.nchunk;
    }
  }
  done_words = (int)used;
  a.col_out = t.col_out; a.col_out_stride = t.col_out_stride;
  a.row_out = t.row_out; a.row_out_stride = t.row_out_stride;
  return true;
}

hipError_t launch_tile_scan(const TileScanJob& t, Stage2Job* pending, hipStream_t st) {
  TileScanArgs a;
  bool fuse_col, fuse_row;
  int words;
  if (!make_tile_args(t, a, fuse_col, fuse_row, words)) return hipErrorInvalidValue;
  const dim3 grid(a.nseg, a.nchunk, a.batch), block(TS_THREADS);
  const size_t lds = TS_LDS_DOUBLES * sizeof(double);
  const bool gated = t.gate != nullptr;
  const bool cidx = t.wr == nullptr, ridx = t.wc == nullptr;
#define GECC_TS(DT, COL, ROW, CI, RI, G) \
  hipLaunchKernelGGL((tile_scan<DT, COL, ROW, CI, RI, G>), grid, block, lds, st, a)
#define GECC_TS_DT(DT)                                                                       \
  do {                                                                                       \
    if (t.col_on && t.row_on) {                                                              \
      if (gated) return hipErrorInvalidValue;                                                \
      if (cidx && !ridx) GECC_TS(DT, true, true, true, false, false);                        \
      else if (!cidx && ridx) GECC_TS(DT, true, true, false, true, false);                   \
      else return hipErrorInvalidValue;                                                      \
    } else if (t.col_on) {                                                                   \
      if (!cidx) return hipErrorInvalidValue;                                                \
      if (gated) GECC_TS(DT, true, false, true, true, true);                                 \
      else GECC_TS(DT, true, false, true, true, false);                                      \
    } else {                                                                                 \
      if (gated && !ridx) return hipErrorInvalidValue;                                       \
      if (gated) GECC_TS(DT, false, true, true, true, true);                                 \
      else if (ridx) GECC_TS(DT, false, true, true, true, false);                            \
      else GECC_TS(DT, false, true, true, false, false);                                     \
    }                                                                                        \
  } while (0)
  if (t.dtype == GECC_BF16) GECC_TS_DT(GECC_BF16); else GECC_TS_DT(GECC_F32);
#undef GECC_TS_DT
#undef GECC_TS
  *pending = Stage2Job{};
  pending->valid = (t.col_on && !fuse_col) || (t.row_on && !fuse_row);
  pending->batch = t.batch;
  pending->gate = t.gate; pending->gate_stride = t.gate_stride; pending->gate_value = t.gate_value;
  if (t.col_on && !fuse_col) {
    pending->scratch = t.col_scratch; pending->out = t.col_out; pending->out_stride = t.col_out_stride;
    pending->Cc = t.Cc; pending->nchunk = a.nchunk;
  }
  if (t.row_on && !fuse_row) {
    pending->row_scratch = t.row_scratch; pending->row_out = t.row_out; pending->row_out_stride = t.row_out_stride;
    pending->R = t.R; pending->nseg = a.nseg;
  }
  return hipGetLastError();
}

// ---- the two audits in one launch ---------------------------------------------------------------
// fills j from x; returns the counters it uses, or -1 when x cannot finish by itself
static int make_pair_job(const ScanPairItem& x, uint32_t* done, PairJob& j) {
  j = PairJob{};
  if (x.kind == 2) {
    TileScanJob t = x.t;
    if (t.col_on == t.row_on || !t.gate) return -1;                       // one part, gated
    if ((t.col_on && t.wr) || (t.row_on && t.wc)) return -1;              // index weights
    t.done = done;
    bool fc, fr;
    int words;
    if (!make_tile_args(t, j.t, fc, fr, words) || !(t.col_on ? fc : fr)) return -1;
    j.kind = t.col_on ? PJ_TILE_COL : PJ_TILE_ROW;
    j.gx = j.t.nseg; j.gy = j.t.nchunk;
    j.nblk = j.gx * j.gy * t.batch;
    return words;
  }
  j.s = x.s;
  j.s.vec_ok = vec_ok(x.s) ? 1 : 0;
  j.s.carry_blocks = 0;
  if (!j.s.gate || j.s.w) return -1;
  if (x.kind == 0) {
    // (rows per workgroup as in launch_rowdot; the sums of a row do not depend on it)
    const bool small = (int64_t)((j.s.R + RD_BIG_RB - 1) / RD_BIG_RB) * j.s.batch < 1024;
    const int rb = small ? RD_SMALL_RB : RD_BIG_RB;
    j.kind = small ? PJ_ROW : PJ_ROW_BIG;
    j.gx = (j.s.R + rb - 1) / rb; j.gy = 1;
    j.nblk = j.gx * j.s.batch;
    return 0;
  }
  const int words = coldot_done_words(j.s);
  if (words == 0) return -1;
  const int vec = j.s.dtype == GECC_BF16 ? 8 : 4;
  j.kind = PJ_COL;
  j.s.done = done;
  j.gx = (j.s.Cc + 64 * vec - 1) / (64 * vec);
  j.gy = (j.s.R + SCAN_CHUNK_ROWS - 1) / SCAN_CHUNK_ROWS;
  j.nblk = j.gx * j.gy * j.s.batch;
  return words;
}

static int pair_dtype(const ScanPairItem& x) { return x.kind == 2 ? x.t.dtype : x.s.dtype; }

bool audit_pair_ok(const ScanPairItem& x0, const ScanPairItem& x1) {
  static uint32_t dummy;   // (an address that is never used: only the counts matter here)
  PairJob j;
  const int w0 = make_pair_job(x0, &dummy, j);
  if (w0 < 0) return false;
  const int nblk0 = j.nblk;
  const int w1 = make_pair_job(x1, &dummy, j);
  // (a closed gate still costs the dispatch of every workgroup: about 2 us per thousand, so a pair of
  // very large grids is no cheaper than two launches)
  return w1 >= 0 && w0 + w1 <= SCAN_DONE_WORDS && pair_dtype(x0) == pair_dtype(x1) && nblk0 + j.nblk <= AUDIT_PAIR_MAX_BLOCKS;
}

hipError_t launch_audit_pair(const ScanPairItem& x0, const ScanPairItem& x1, uint32_t* done, hipStream_t st) {
  if (!done || !audit_pair_ok(x0, x1)) return hipErrorInvalidValue;
  PairArgs p;
  const int w0 = make_pair_job(x0, done, p.j[0]);
  make_pair_job(x1, done + w0, p.j[1]);
  const dim3 grid(p.j[0].nblk + p.j[1].nblk);
  if (pair_dtype(x0) == GECC_BF16) hipLaunchKernelGGL(audit_pair<GECC_BF16>, grid, dim3(256), 0, st, p);
  else                             hipLaunchKernelGGL(audit_pair<GECC_F32>, grid, dim3(256), 0, st, p);
  return hipGetLastError();
}

namespace {
__global__ void zero_words_kernel(uint32_t* w, int count) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) w[i] = 0u;
}
}  // namespace
hipError_t launch_zero_words(uint32_t* words, int count, hipStream_t st) {
  hipLaunchKernelGGL(zero_words_kernel, dim3((count + 255) / 256), dim3(256), 0, st, words, count);
  return hipGetLastError();
}

int stage2_blocks(const Stage2Job& j) {
  return (j.Cc > 0 ? (2 * j.Cc + 63) / 64 : 0) + (j.R > 0 ? (j.R + 255) / 256 : 0);
}

hipError_t launch_stage2(const Stage2Job& j, hipStream_t st) {
  dim3 g2(stage2_blocks(j), j.batch);
  hipLaunchKernelGGL(coldot_stage2, g2, dim3(256), 0, st, j);
  return hipGetLastError();
}

}  // namespace gecc
