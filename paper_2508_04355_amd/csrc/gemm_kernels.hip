// The data block of the encoded product (Section III, C = A B) on the MFMA units, with the
// row/column sums that Section V's syndromes need taken from the accumulators before C
// leaves the compute unit, so that verification never re-reads C from HBM.
//
// Per workgroup: a BM x BN tile of C.  Operand tiles are staged through LDS in a
// k-contiguous layout (whatever the storage order of the operand is), MFMA fragments are read
// from there.  After the k loop the tile passes through LDS once more in slabs of rows:
// planted faults are applied, per-tile row sums (plain and weighted by the local column
// index + 1) and column sums (plain and weighted by the local row index + 1) are formed, and
// C is written with full-width stores.
#include "gecc_internal.h"

namespace gecc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int THREADS = 256;
constexpr int CPAD = 4;   // padding of the C slab rows (floats)

template <int DT> struct GT;
template <> struct GT<GECC_BF16> {
  using T = uint16_t;
  static constexpr int VEC = 8;    // elements per 16-byte load
  static constexpr int BK = 32;
  static constexpr int KPAD = 8;   // LDS row padding (elements)
};
template <> struct GT<GECC_F32> {
  using T = float;
  static constexpr int VEC = 4;
  static constexpr int BK = 16;
  static constexpr int KPAD = 1;
};

// ---- staging of one operand tile: ROWS (m- or n-index) x BK, into registers then LDS -------
// KCONTIG: element (r, kk) lives at P[r * ld + kk]; otherwise at P[kk * ld + r].
template <int DT, int ROWS, bool KCONTIG>
struct Stager {
  using G = GT<DT>;
  using T = typename G::T;
  static constexpr int VEC = G::VEC;
  static constexpr int BK = G::BK;
  static constexpr int LDK = BK + G::KPAD;
  static constexpr int CHUNKS = ROWS * BK / VEC;
  static constexpr int PER_THREAD = CHUNKS / THREADS;
  static_assert(CHUNKS % THREADS == 0, "tile must split evenly over the workgroup");
  __attribute__((aligned(16))) T reg[PER_THREAD][VEC];

  __device__ __forceinline__ void load(const T* P, int64_t ld, int r0, int k0, int rlim, int klim,
                                       bool vec_ok) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int c = threadIdx.x + THREADS * i;
      int r, kk;
      if (KCONTIG) { r = c / (BK / VEC); kk = (c % (BK / VEC)) * VEC; }
      else         { kk = c / (ROWS / VEC); r = (c % (ROWS / VEC)) * VEC; }
      const int gr = r0 + r, gk = k0 + kk;
      const T* src = KCONTIG ? P + (int64_t)gr * ld + gk : P + (int64_t)gk * ld + gr;
      const bool full = KCONTIG ? (gr < rlim && gk + VEC <= klim) : (gk < klim && gr + VEC <= rlim);
      if (full && vec_ok) {
        *reinterpret_cast<uint4*>(reg[i]) = *reinterpret_cast<const uint4*>(src);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const bool in = KCONTIG ? (gr < rlim && gk + e < klim) : (gk < klim && gr + e < rlim);
          reg[i][e] = in ? src[e] : (T)0;
        }
      }
    }
  }

  __device__ __forceinline__ void store(T (*S)[LDK]) const {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int c = threadIdx.x + THREADS * i;
      if (KCONTIG) {
        const int r = c / (BK / VEC), kk = (c % (BK / VEC)) * VEC;
        if (DT == GECC_BF16) {
          *reinterpret_cast<uint4*>(&S[r][kk]) = *reinterpret_cast<const uint4*>(reg[i]);
        } else {
#pragma unroll
          for (int e = 0; e < VEC; ++e) S[r][kk + e] = reg[i][e];
        }
      } else {
        const int kk = c / (ROWS / VEC), r = (c % (ROWS / VEC)) * VEC;
#pragma unroll
        for (int e = 0; e < VEC; ++e) S[r + e][kk] = reg[i][e];
      }
    }
  }
};

// ---- one row slab of the C tile, resident in LDS: faults, partial sums, store ---------------
// Cs holds SLAB rows x BN columns; rows slab_r0.. of the tile.  cs/cw accumulate the column
// sums of the thread's column (threads < BN) over the slabs.
template <int BN, int SLAB>
__device__ __forceinline__ void slab_reduce(float (*Cs)[BN + CPAD], int slab_r0, int tile_r0,
                                            int tile_c0, int n, int m, float* rowpart_tile,
                                            float& cs, float& cw) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // row sums: one wavefront per row, lanes stride the columns
  if (rowpart_tile) {
    for (int r = wave; r < SLAB; r += THREADS / 64) {
      float s = 0.f, w = 0.f;
#pragma unroll
      for (int c = lane; c < BN; c += 64) {
        const float v = Cs[r][c];
        s += v;
        w = fmaf((float)(c + 1), v, w);
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        s += __shfl_down(s, off, 64);
        w += __shfl_down(w, off, 64);
      }
      const int gi = tile_r0 + slab_r0 + r;
      if (lane == 0 && gi < n) {
        rowpart_tile[(int64_t)gi * 2] = s;
        rowpart_tile[(int64_t)gi * 2 + 1] = w;
      }
    }
    if (tid < BN) {
#pragma unroll 8
      for (int r = 0; r < SLAB; ++r) {
        const float v = Cs[r][tid];
        cs += v;
        cw = fmaf((float)(slab_r0 + r + 1), v, cw);
      }
    }
  }
}

template <int BN, int SLAB>
__device__ __forceinline__ void slab_store(float (*Cs)[BN + CPAD], int slab_r0, int tile_r0,
                                           int tile_c0, int n, int m, float* C, int64_t ldc,
                                           bool vec_ok) {
  constexpr int V4 = BN / 4;
  for (int o = threadIdx.x; o < SLAB * V4; o += THREADS) {
    const int r = o / V4, c = (o % V4) * 4;
    const int gi = tile_r0 + slab_r0 + r, gj = tile_c0 + c;
    if (gi >= n || gj >= m) continue;
    float* dst = C + (int64_t)gi * ldc + gj;
    if (vec_ok && gj + 4 <= m) {
      *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(&Cs[r][c]);
    } else {
      for (int e = 0; e < 4 && gj + e < m; ++e) dst[e] = Cs[r][c + e];
    }
  }
}

// planted faults (distinct positions): each thread takes a strided share of the list
__device__ __forceinline__ void apply_faults(const gecc_fault* faults, int n_faults, int b,
                                             int r_lo, int r_hi, int c_lo, int c_hi, float* Cs,
                                             int ldcs) {
  for (int f = threadIdx.x; f < n_faults; f += THREADS) {
    const gecc_fault ft = faults[f];
    if (ft.batch == b && ft.row >= r_lo && ft.row < r_hi && ft.col >= c_lo && ft.col < c_hi)
      Cs[(ft.row - r_lo) * ldcs + (ft.col - c_lo)] += ft.offset;
  }
}

// -------------------------------------------------------------------------------------------
template <int DT, bool KCA, bool KCB>
__global__ __launch_bounds__(THREADS) void gemm_kernel(GemmArgs a) {
  using G = GT<DT>;
  using T = typename G::T;
  constexpr int BM = 128, BN = 128, BK = G::BK, LDK = BK + G::KPAD, SLAB = 64;
  // k-split (products of few tiles): ksplit workgroups share a tile, one per range of k
  const int S = a.ksplit > 1 ? a.ksplit : 1;
  const int b = (int)blockIdx.z / S, split = (int)blockIdx.z % S;
  const int k_begin = S > 1 ? min(a.k, split * a.k_per) : 0;
  const int k_end = S > 1 ? min(a.k, k_begin + a.k_per) : a.k;
  const int tm = blockIdx.y, tn = blockIdx.x;
  const int tile_r0 = tm * BM, tile_c0 = tn * BN;
  const T* A = reinterpret_cast<const T*>(a.A) + (int64_t)b * a.sa;
  const T* B = reinterpret_cast<const T*>(a.B) + (int64_t)b * a.sb;
  float* C = a.C + (int64_t)b * a.sc;

  constexpr int AB_BYTES = (BM + BN) * LDK * (int)sizeof(T);
  constexpr int CS_BYTES = SLAB * (BN + CPAD) * (int)sizeof(float);
  __shared__ __attribute__((aligned(16))) char smem[AB_BYTES > CS_BYTES ? AB_BYTES : CS_BYTES];
  T (*As)[LDK] = reinterpret_cast<T (*)[LDK]>(smem);
  T (*Bs)[LDK] = reinterpret_cast<T (*)[LDK]>(smem + BM * LDK * sizeof(T));
  float (*Cs)[BN + CPAD] = reinterpret_cast<float (*)[BN + CPAD]>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;          // 2 x 2 wavefronts, 64 x 64 each
  const int l32 = lane & 31, lhi = lane >> 5;

  const bool vecA = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (a.lda % G::VEC == 0);
  const bool vecB = (reinterpret_cast<uintptr_t>(B) % 16 == 0) && (a.ldb % G::VEC == 0);

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  Stager<DT, BM, KCA> sa;
  Stager<DT, BN, KCB> sb;
  sa.load(A, a.lda, tile_r0, k_begin, a.n, k_end, vecA);
  sb.load(B, a.ldb, tile_c0, k_begin, a.m, k_end, vecB);

  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    __syncthreads();               // previous tile fully consumed
    sa.store(As);
    sb.store(Bs);
    __syncthreads();
    if (k0 + BK < k_end) {         // prefetch the next tile into registers
      sa.load(A, a.lda, tile_r0, k0 + BK, a.n, k_end, vecA);
      sb.load(B, a.ldb, tile_c0, k0 + BK, a.m, k_end, vecB);
    }
    if (DT == GECC_BF16) {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 16) {
        bf16x8_t fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
          fa[i] = *reinterpret_cast<const bf16x8_t*>(&As[wr * 64 + i * 32 + l32][ks + lhi * 8]);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fb[j] = *reinterpret_cast<const bf16x8_t*>(&Bs[wc * 64 + j * 32 + l32][ks + lhi * 8]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < BK; ks += 2) {
        float fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
          fa[i] = *reinterpret_cast<const float*>(&As[wr * 64 + i * 32 + l32][ks + lhi]);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fb[j] = *reinterpret_cast<const float*>(&Bs[wc * 64 + j * 32 + l32][ks + lhi]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
    }
  }

  if (S > 1) {
    // Every workgroup of the tile leaves its partial sums in memory; the one that arrives last adds
    // them all up in the order of the k ranges (so the result does not depend on which one that
    // is) and goes on with the tile.
    const int64_t tile_id = ((int64_t)b * gridDim.y + tm) * gridDim.x + tn;
    float* part = a.split_part + tile_id * S * (BM * BN);
    float* mine = part + (int64_t)split * (BM * BN);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = wr * 64 + i * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3);
          store_dev(mine + r * BN + wc * 64 + j * 32 + l32, acc[i][j][v]);
        }
    if (!arrive_last(a.split_done + tile_id, (uint32_t)S, reinterpret_cast<int*>(smem))) return;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int q = 0; q < S; ++q) {
      const float* src = part + (int64_t)q * (BM * BN);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int r = wr * 64 + i * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3);
            acc[i][j][v] += load_dev(src + r * BN + wc * 64 + j * 32 + l32);
          }
    }
  }

  // ---- epilogue: the tile goes through LDS in two slabs of 64 rows -------------------------
  const bool epi = a.rowpart != nullptr;
  float* rowpart_tile = epi ? a.rowpart + ((int64_t)b * a.ntn + tn) * a.rp_ld * 2 : nullptr;
  const bool vecC = (reinterpret_cast<uintptr_t>(C) % 16 == 0) && (a.ldc % 4 == 0);
  float cs = 0.f, cw = 0.f;
#pragma unroll
  for (int slab = 0; slab < BM / SLAB; ++slab) {
    __syncthreads();
    if (wr == slab) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int r = i * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3);
            Cs[r][wc * 64 + j * 32 + l32] = acc[i][j][v];
          }
    }
    __syncthreads();
    const int r_lo = tile_r0 + slab * SLAB;
    apply_faults(a.faults, a.n_faults, b + a.fault_bias, r_lo, min(r_lo + SLAB, a.n), tile_c0,
                 min(tile_c0 + BN, a.m), &Cs[0][0], BN + CPAD);
    if (a.n_faults > 0) __syncthreads();
    slab_reduce<BN, SLAB>(Cs, slab * SLAB, tile_r0, tile_c0, a.n, a.m, rowpart_tile, cs, cw);
    slab_store<BN, SLAB>(Cs, slab * SLAB, tile_r0, tile_c0, a.n, a.m, C, a.ldc, vecC);
  }
  if (epi && tid < BN && tile_c0 + tid < a.m) {
    float* cp = a.colpart + (((int64_t)b * a.ntm + tm) * a.cp_ld + tile_c0 + tid) * 2;
    cp[0] = cs;
    cp[1] = cw;
  }
  if (epi && tm == 0 && tn == 0 && a.pg_out) form_pg(a, b, reinterpret_cast<double*>(smem));   // P_g, once per batch item
}

// -------------------------------------------------------------------------------------------
// Stand-alone partial sums of a C that sits in HBM (same 128 x 128 tiling and workspace layout
// as the fused epilogues).  HBM-bound: every thread streams 16 rows x 4 columns with 16-byte
// loads (two full 512-byte tile rows per wavefront instruction), keeps its row and column
// partial sums in registers, and the workgroup combines them through LDS in a fixed order.
__global__ __launch_bounds__(THREADS) void partials_kernel(PartialArgs a) {
  const int b = blockIdx.z;
  if (a.gate) {
    const int32_t g = *reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(a.gate) +
                                                        a.gate_stride * b);
    if (g != a.gate_value) return;
  }
  const int tm = blockIdx.y, tn = blockIdx.x;
  const int tile_r0 = tm * 128, tile_c0 = tn * 128;
  const float* C = a.C + (int64_t)b * a.sc;
  const int tid = threadIdx.x;
  const int cg = tid & 31, rg = tid >> 5;          // 32 column groups of 4, 8 row groups of 16
  const int gj = tile_c0 + cg * 4;
  const bool vec = (reinterpret_cast<uintptr_t>(C) % 16 == 0) && (a.ldc % 4 == 0) && gj + 4 <= a.m;
  __shared__ float red_row[2][128][33];
  __shared__ float red_col[2][8][128];
  float cs[4] = {0.f, 0.f, 0.f, 0.f}, cw[4] = {0.f, 0.f, 0.f, 0.f};
  // the kernel is a stream over C: all 16 loads of a thread are issued before the first is used
  // (rows past the end are clamped, not branched on, and count as zero below)
  float4 pre[16];
  if (vec) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      pre[r] = *reinterpret_cast<const float4*>(C + (int64_t)min(tile_r0 + rg * 16 + r, a.n - 1) * a.ldc + gj);
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int rl = rg * 16 + r, gi = tile_r0 + rl;
    float x[4] = {0.f, 0.f, 0.f, 0.f};
    if (gi < a.n) {
      if (vec) {
        x[0] = pre[r].x; x[1] = pre[r].y; x[2] = pre[r].z; x[3] = pre[r].w;
      } else {
        const float* src = C + (int64_t)gi * a.ldc + gj;
        for (int e = 0; e < 4; ++e) if (gj + e < a.m) x[e] = src[e];
      }
    }
    float rs = 0.f, rw = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      cs[e] += x[e];
      cw[e] = fmaf((float)(rl + 1), x[e], cw[e]);
      rs += x[e];
      rw = fmaf((float)(cg * 4 + e + 1), x[e], rw);
    }
    red_row[0][rl][cg] = rs;
    red_row[1][rl][cg] = rw;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    red_col[0][rg][cg * 4 + e] = cs[e];
    red_col[1][rg][cg * 4 + e] = cw[e];
  }
  __syncthreads();
  if (tid < 128) {
    float s = 0.f, w = 0.f;
#pragma unroll
    for (int c = 0; c < 32; ++c) { s += red_row[0][tid][c]; w += red_row[1][tid][c]; }
    const int gi = tile_r0 + tid;
    if (gi < a.n) {
      float2* rp = reinterpret_cast<float2*>(a.rowpart + (((int64_t)b * a.ntn + tn) * a.rp_ld + gi) * 2);
      *rp = make_float2(s, w);
    }
  } else {
    const int c = tid - 128;
    float s = 0.f, w = 0.f;
#pragma unroll
    for (int g = 0; g < 8; ++g) { s += red_col[0][g][c]; w += red_col[1][g][c]; }
    const int gc = tile_c0 + c;
    if (gc < a.m) {
      float2* cp = reinterpret_cast<float2*>(a.colpart + (((int64_t)b * a.ntm + tm) * a.cp_ld + gc) * 2);
      *cp = make_float2(s, w);
    }
  }
}

template <int DT>
hipError_t launch_dt(const GemmArgs& a0, hipStream_t st) {
  GemmArgs a = a0;
  const int ntiles = ((a.m + 127) / 128) * ((a.n + 127) / 128);
  if (a.ksplit > 1 && a.split_part && a.split_done && (int64_t)ntiles * a.batch <= SCAN_DONE_WORDS) {
    const int bk = GT<DT>::BK;
    a.k_per = ((a.k + a.ksplit - 1) / a.ksplit + bk - 1) / bk * bk;
  } else {
    a.ksplit = 1;
  }
  dim3 grid((a.m + 127) / 128, (a.n + 127) / 128, a.batch * a.ksplit);
  // k-contiguous storage: A when not transposed, B when transposed
  const bool kca = a.trans_a == 0, kcb = a.trans_b != 0;
  if (kca && kcb)        hipLaunchKernelGGL((gemm_kernel<DT, true, true>), grid, dim3(THREADS), 0, st, a);
  else if (kca && !kcb)  hipLaunchKernelGGL((gemm_kernel<DT, true, false>), grid, dim3(THREADS), 0, st, a);
  else if (!kca && kcb)  hipLaunchKernelGGL((gemm_kernel<DT, false, true>), grid, dim3(THREADS), 0, st, a);
  else                   hipLaunchKernelGGL((gemm_kernel<DT, false, false>), grid, dim3(THREADS), 0, st, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, hipStream_t st) {
  if (a.tile_m != 128 || a.tile_n != 128) return hipErrorInvalidValue;
  if (gemm_bf16_fast_ok(a)) return launch_gemm_bf16_fast(a, st);
  return a.dtype == GECC_BF16 ? launch_dt<GECC_BF16>(a, st) : launch_dt<GECC_F32>(a, st);
}

namespace {
// C += P, 16 bytes per thread where the rows allow it
__global__ __launch_bounds__(256) void accumulate_kernel(float* C, const float* P, int n, int m, int64_t ldc, int vec_ok) {
  const int64_t total4 = (int64_t)n * ((m + 3) / 4);
  for (int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x; o < total4; o += (int64_t)gridDim.x * 256) {
    const int64_t i = o / ((m + 3) / 4);
    const int j = (int)(o - i * ((m + 3) / 4)) * 4;
    float* c = C + i * ldc + j;
    const float* p = P + i * ldc + j;
    if (vec_ok && j + 4 <= m) {
      float4 x = *reinterpret_cast<const float4*>(c);
      const float4 y = *reinterpret_cast<const float4*>(p);
      x.x += y.x; x.y += y.y; x.z += y.z; x.w += y.w;
      *reinterpret_cast<float4*>(c) = x;
    } else {
      for (int e = 0; e < 4 && j + e < m; ++e) c[e] += p[e];
    }
  }
}
}  // namespace

hipError_t launch_accumulate(float* C, const float* P, int n, int m, int64_t ldc, hipStream_t st) {
  const int vec_ok = ldc % 4 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && reinterpret_cast<uintptr_t>(P) % 16 == 0;
  const int64_t total4 = (int64_t)n * ((m + 3) / 4);
  const int blocks = (int)((total4 + 255) / 256 < 16384 ? (total4 + 255) / 256 : 16384);
  hipLaunchKernelGGL(accumulate_kernel, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, st, C, P, n, m, ldc, vec_ok);
  return hipGetLastError();
}

hipError_t launch_partials(const PartialArgs& a, hipStream_t st) {
  if (a.tile_m != 128 || a.tile_n != 128) return hipErrorInvalidValue;
  dim3 grid(a.ntn, a.ntm, a.batch);
  hipLaunchKernelGGL(partials_kernel, grid, dim3(THREADS), 0, st, a);
  return hipGetLastError();
}

}  // namespace gecc
