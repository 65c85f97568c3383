// HBM-bound weighted reductions over an operand: parity encoding (Section III, A_P and B_P),
// the parity blocks of the encoded product (P_r = A B_P, P_c = A_P B) and the operand audit.
//
// Both kernels read the operand once with 16-byte loads that are contiguous across a
// wavefront, accumulate in fp64 and reduce in a fixed order (no floating-point atomics), so
// that re-forming a parity from an unchanged operand reproduces it bit for bit.
#include "gecc_internal.h"

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

// Stage 2 of coldot (see below): 64 outputs per workgroup of 256 threads; the 4 wavefronts take
// the chunks 4 apart and are combined in order.  scratch, out: of batch item b.
__device__ __forceinline__ void coldot_stage2_body(const double* scratch, double* out, int Cc, int nchunk, int blk) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int o = blk * 64 + lane;                   // index into [2][Cc]
  __shared__ double red[4][64];
  double s = 0.0;
  if (o < 2 * Cc) {
    const double* part = scratch + o;
    double t[4] = {0.0, 0.0, 0.0, 0.0};
    int ch = wave;
    for (; ch + 12 < nchunk; ch += 16) {           // 4 loads in flight
#pragma unroll
      for (int u = 0; u < 4; ++u) t[u] += part[(int64_t)(ch + 4 * u) * 2 * Cc];
    }
    for (; ch < nchunk; ch += 4) t[0] += part[(int64_t)ch * 2 * Cc];
    s = (t[0] + t[1]) + (t[2] + t[3]);
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && o < 2 * Cc) out[o] = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
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
// GATED: the launch belongs to the operand audit and returns at once unless the decoder asked for
// it (a separate instantiation, so that profiles list encoding and audit launches apart).
template <int DT, bool IDXW, int RD_RB, int RD_U, bool GATED>
__global__ __launch_bounds__(RD_THREADS) void rowdot_kernel(ScanArgs a) {
  using E = Elem<DT>;
  using T = typename E::type;
  constexpr int VEC = E::VEC;
  constexpr int STEP = RD_THREADS * VEC;   // columns one pass of the workgroup covers
  const int b = blockIdx.y;
  if (GATED && gated_off(a.gate, a.gate_stride, b, a.gate_value)) return;
  const int own = (int)gridDim.x - a.carry_blocks;
  if ((int)blockIdx.x >= own) {   // carried second stage of an earlier coldot
    coldot_stage2_body(a.carry_scratch + (int64_t)b * a.carry_nchunk * 2 * a.carry_Cc,
                       a.carry_out + (int64_t)b * a.carry_out_stride, a.carry_Cc, a.carry_nchunk,
                       (int)blockIdx.x - own);
    return;
  }
  const T* X = reinterpret_cast<const T*>(a.X) + (int64_t)b * a.xs;
  const double* w0 = IDXW ? nullptr : a.w + (int64_t)b * a.w_stride;
  const double* w1 = IDXW ? nullptr : w0 + a.Cc;
  double* out = a.out + (int64_t)b * a.out_stride;
  const int r0 = blockIdx.x * RD_RB;
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
  __shared__ double red[RD_RB][RD_THREADS];
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

// -------------------------------------------------------------------------------------------
// coldot: out[t][c] = sum_r w_t[r] X[r,c].   Stage 1: a workgroup owns 64*VEC columns and one
// chunk of SCAN_CHUNK_ROWS rows; its 4 wavefronts interleave the rows and are combined through
// LDS.  Stage 2 adds the chunks in order.
constexpr int CD_THREADS = 256;

template <int DT, bool IDXW, bool GATED>
__global__ __launch_bounds__(CD_THREADS) void coldot_stage1(ScanArgs a, int nchunk) {
  using E = Elem<DT>;
  using T = typename E::type;
  constexpr int VEC = E::VEC;
  const int b = blockIdx.z;
  if (GATED && gated_off(a.gate, a.gate_stride, b, a.gate_value)) return;
  const T* X = reinterpret_cast<const T*>(a.X) + (int64_t)b * a.xs;
  const double* w0 = IDXW ? nullptr : a.w + (int64_t)b * a.w_stride;
  const double* w1 = IDXW ? nullptr : w0 + a.R;
  const int chunk = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int c = (blockIdx.x * 64 + lane) * VEC;
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

  __shared__ double red[4][2][VEC][64];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { red[wave][0][e][lane] = acc0[e]; red[wave][1][e][lane] = acc1[e]; }
  __syncthreads();
  // thread -> (t, e, lane'): 2*VEC*64 outputs, 256 threads
  double* part = a.scratch + ((int64_t)b * nchunk + chunk) * 2 * a.Cc;
  for (int o = tid; o < 2 * VEC * 64; o += CD_THREADS) {
    const int l = o & 63, e = (o >> 6) % VEC, t = o / (64 * VEC);
    const int col = (blockIdx.x * 64 + l) * VEC + e;
    if (col < a.Cc) {
      const double s = (red[0][t][e][l] + red[1][t][e][l]) + (red[2][t][e][l] + red[3][t][e][l]);
      part[(int64_t)t * a.Cc + col] = s;
    }
  }
}

__global__ __launch_bounds__(256) void coldot_stage2(Stage2Job j) {
  const int b = blockIdx.y;
  if (gated_off(j.gate, j.gate_stride, b, j.gate_value)) return;
  coldot_stage2_body(j.scratch + (int64_t)b * j.nchunk * 2 * j.Cc, j.out + (int64_t)b * j.out_stride, j.Cc,
                     j.nchunk, blockIdx.x);
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
    a.carry_scratch = carry->scratch; a.carry_out = carry->out; a.carry_out_stride = carry->out_stride;
    a.carry_Cc = carry->Cc; a.carry_nchunk = carry->nchunk;
    a.carry_blocks = (2 * carry->Cc + 63) / 64;
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

hipError_t launch_coldot_stage1(const ScanArgs& a0, Stage2Job* pending, hipStream_t st) {
  ScanArgs a = a0;
  a.vec_ok = vec_ok(a0) ? 1 : 0;
  a.carry_blocks = 0;
  const int vec = a.dtype == GECC_BF16 ? 8 : 4;
  const int nchunk = (a.R + SCAN_CHUNK_ROWS - 1) / SCAN_CHUNK_ROWS;
  dim3 grid((a.Cc + 64 * vec - 1) / (64 * vec), nchunk, a.batch);
  const bool idx = a.w == nullptr, gated = a.gate != nullptr;
  if (gated && !idx) return hipErrorInvalidValue;
  if (a.dtype == GECC_BF16) {
    if (gated)    hipLaunchKernelGGL((coldot_stage1<GECC_BF16, true, true>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else if (idx) hipLaunchKernelGGL((coldot_stage1<GECC_BF16, true, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else          hipLaunchKernelGGL((coldot_stage1<GECC_BF16, false, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
  } else {
    if (gated)    hipLaunchKernelGGL((coldot_stage1<GECC_F32, true, true>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else if (idx) hipLaunchKernelGGL((coldot_stage1<GECC_F32, true, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
    else          hipLaunchKernelGGL((coldot_stage1<GECC_F32, false, false>), grid, dim3(CD_THREADS), 0, st, a, nchunk);
  }
  pending->valid = true;
  pending->scratch = a.scratch; pending->out = a.out; pending->out_stride = a.out_stride;
  pending->Cc = a.Cc; pending->nchunk = nchunk; pending->batch = a.batch;
  pending->gate = a.gate; pending->gate_stride = a.gate_stride; pending->gate_value = a.gate_value;
  return hipGetLastError();
}

hipError_t launch_stage2(const Stage2Job& j, hipStream_t st) {
  dim3 g2((2 * j.Cc + 63) / 64, j.batch);
  hipLaunchKernelGGL(coldot_stage2, g2, dim3(256), 0, st, j);
  return hipGetLastError();
}

}  // namespace gecc
