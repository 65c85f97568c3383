// bf16 x bf16 -> fp32 data block of the encoded product (Section III, C = A B), the kernel
// that holds nearly all flops of the path.
//
// Workgroup: 256 x 256 tile of C, 4 wavefronts (2 x 2), each owning a 128 x 128 sub-tile as
// 4 x 4 MFMA 32x32x16 accumulators (256 fp32 registers per lane).  k advances in steps of 64
// through two LDS buffers (2 x 64 KiB); the next operand tiles travel global -> registers
// while the current ones feed the MFMA units.
//
// LDS format (both operands, whatever their storage order): row = m- or n-index, 128 bytes
// = 64 k-values per row, stored as eight 16-byte chunks whose position is XOR-swizzled with
// the row index so that fragment reads (32 consecutive rows, one chunk each) and tile writes
// are free of bank conflicts without padding.  An operand that is contiguous along m or n in
// memory is loaded as 8 x 8 element blocks and transposed in registers on the way.
//
// Epilogue, from the accumulators (no pass through LDS for C itself): planted faults, per
// sub-tile column sums (in-lane) and row sums (through a small LDS transpose), then C.
#include "gecc_internal.h"

namespace gecc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int THREADS = 256;
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ROW_BYTES = BK * 2;                  // 128
constexpr int TILE_BYTES = BM * ROW_BYTES;         // 32 KiB per operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;        // A + B
constexpr int SMEM_BYTES = 2 * STAGE_BYTES;        // double buffered: 128 KiB
constexpr int GROUP_M = 8;                         // tile rows per L2-sharing group

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * ROW_BYTES + ((chunk ^ swz(row)) << 4);
}

// ---- operand tile: global -> registers -> LDS ------------------------------------------------
// KC = true : element (r, kk) at P[r * ld + kk]  (k contiguous)
// KC = false: element (r, kk) at P[kk * ld + r]  (r contiguous); 8 x 8 blocks, transposed here
template <bool KC>
struct TileStager {
  uint4 reg[8];

  __device__ __forceinline__ void load(const uint16_t* P, int64_t ld, int r0, int k0, int rlim, int klim) {
    const int tid = threadIdx.x;
    if (KC) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int q = tid + THREADS * i;
        const int gr = r0 + (q >> 3), gk = k0 + ((q & 7) << 3);
        const bool ok = gr < rlim && gk < klim;
        reg[i] = ok ? *reinterpret_cast<const uint4*>(P + (int64_t)gr * ld + gk) : make_uint4(0, 0, 0, 0);
      }
    } else {
      const int gr = r0 + ((tid & 31) << 3);
      const int gkb = k0 + ((tid >> 5) << 3);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const bool ok = gr < rlim && gkb + kk < klim;
        reg[kk] = ok ? *reinterpret_cast<const uint4*>(P + (int64_t)(gkb + kk) * ld + gr) : make_uint4(0, 0, 0, 0);
      }
    }
  }

  __device__ __forceinline__ void store(char* tile) const {
    const int tid = threadIdx.x;
    if (KC) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int q = tid + THREADS * i;
        *reinterpret_cast<uint4*>(tile + lds_off(q >> 3, q & 7)) = reg[i];
      }
    } else {
      // reg[kk] holds r = rb .. rb+7 at k = kb + kk.  Row (rb + e) of the tile needs the eight
      // k-values of column e: dword p of it = { reg[2p][e], reg[2p+1][e] }.
      const int rb = (tid & 31) << 3, g = tid >> 5;
      const uint32_t* w = reinterpret_cast<const uint32_t*>(reg);   // w[kk * 4 + d]
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint4 o;
        uint32_t* od = reinterpret_cast<uint32_t*>(&o);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const uint32_t x = w[(2 * p) * 4 + (e >> 1)], y = w[(2 * p + 1) * 4 + (e >> 1)];
          od[p] = (e & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
        }
        *reinterpret_cast<uint4*>(tile + lds_off(rb + e, g)) = o;
      }
    }
  }
};

template <bool KCA, bool KCB, bool EPI>
__global__ __launch_bounds__(THREADS, 1) void gemm_bf16_256(GemmArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int b = blockIdx.y;

  // ---- tile order: consecutive workgroups land on different XCDs (round robin), so give
  // every XCD a contiguous range of the tile sequence; inside it walk GROUP_M tile rows at a
  // time, column by column, so that co-resident tiles share A row panels and B column panels
  const int ntm = (a.n + BM - 1) / BM, ntn = (a.m + BN - 1) / BN;
  const int ntiles = ntm * ntn;
  int pid = blockIdx.x;
  {
    const int per = ntiles / 8, rem = ntiles - per * 8;     // XCD x gets per (+1 if x < rem)
    const int x = pid & 7, idx = pid >> 3;
    pid = x * per + min(x, rem) + idx;
  }
  const int gsz = GROUP_M * ntn;
  const int grp = pid / gsz;
  const int first_m = grp * GROUP_M;
  const int gm = min(GROUP_M, ntm - first_m);
  const int tm = first_m + (pid - grp * gsz) % gm;
  const int tn = (pid - grp * gsz) / gm;
  const int tile_r0 = tm * BM, tile_c0 = tn * BN;

  const uint16_t* A = reinterpret_cast<const uint16_t*>(a.A) + (int64_t)b * a.sa;
  const uint16_t* B = reinterpret_cast<const uint16_t*>(a.B) + (int64_t)b * a.sb;
  float* C = a.C + (int64_t)b * a.sc;

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // fragment addresses inside a tile: row = sub-tile base + 32 * i + l32, chunk = 2 * ks + lhi
  int a_row[4], b_row[4], a_sw[4], b_sw[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a_row[i] = (wr * 128 + i * 32 + l32) * ROW_BYTES;
    b_row[i] = (wc * 128 + i * 32 + l32) * ROW_BYTES;
    a_sw[i] = swz(wr * 128 + i * 32 + l32);
    b_sw[i] = swz(wc * 128 + i * 32 + l32);
  }

  TileStager<KCA> sa;
  TileStager<KCB> sb;
  const int KT = (a.k + BK - 1) / BK;
  sa.load(A, a.lda, tile_r0, 0, a.n, a.k);
  sb.load(B, a.ldb, tile_c0, 0, a.m, a.k);
  sa.store(smem);
  sb.store(smem + TILE_BYTES);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    char* cur = smem + (kt & 1) * STAGE_BYTES;
    char* nxt = smem + ((kt & 1) ^ 1) * STAGE_BYTES;
    const bool more = kt + 1 < KT;
    if (more) {
      sa.load(A, a.lda, tile_r0, (kt + 1) * BK, a.n, a.k);
      sb.load(B, a.ldb, tile_c0, (kt + 1) * BK, a.m, a.k);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8_t fa[4], fb[4];
      const int ch = 2 * ks + lhi;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8_t*>(cur + a_row[i] + ((ch ^ a_sw[i]) << 4));
        fb[i] = *reinterpret_cast<const bf16x8_t*>(cur + TILE_BYTES + b_row[i] + ((ch ^ b_sw[i]) << 4));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      sa.store(nxt);
      sb.store(nxt + TILE_BYTES);
    }
    __syncthreads();
  }

  // ---- epilogue -------------------------------------------------------------------------------
  const int R0 = tile_r0 + wr * 128, C0 = tile_c0 + wc * 128;   // origin of this wavefront's sub-tile
  if (R0 >= a.n || C0 >= a.m) {
    // nothing of this sub-tile is inside C; still take part in the barriers below
  }
  if (a.n_faults > 0) {
    for (int f = 0; f < a.n_faults; ++f) {
      const gecc_fault ft = a.faults[f];
      if (ft.batch != b || ft.row < R0 || ft.row >= R0 + 128 || ft.col < C0 || ft.col >= C0 + 128) continue;
      const int dr = ft.row - R0, dc = ft.col - C0;
      const int fi = dr >> 5, rr = dr & 31, fj = dc >> 5;
      const int fv = ((rr >> 3) << 2) | (rr & 3);
      const bool mine = (((rr >> 2) & 1) == lhi) && ((dc & 31) == l32);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (mine && i == fi && j == fj && v == fv) acc[i][j][v] += ft.offset;
    }
  }

  if (EPI) {
    const int tm128 = R0 >> 7, tn128 = C0 >> 7;
    // column sums of the 128 x 128 sub-tile: plain and weighted by (local row + 1)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float cs = 0.f, cw = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float x = acc[i][j][v];
          cs += x;
          cw = fmaf((float)(i * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3) + 1), x, cw);
        }
      cs += __shfl_xor(cs, 32, 64);
      cw += __shfl_xor(cw, 32, 64);
      const int col = C0 + j * 32 + l32;
      if (lhi == 0 && col < a.m && R0 < a.n) {
        float2* cp = reinterpret_cast<float2*>(a.colpart + (((int64_t)b * a.ntm + tm128) * a.m + col) * 2);
        *cp = make_float2(cs, cw);
      }
    }
    // row sums: per lane over its 4 columns (one per 32-wide block), then across the 32 lanes
    // of a half wavefront through LDS; plain first, then weighted by (local column + 1)
    float* red = reinterpret_cast<float*>(smem) + wave * (128 * 33);
#pragma unroll
    for (int kind = 0; kind < 2; ++kind) {
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float s = 0.f;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            s = kind ? fmaf((float)(j * 32 + l32 + 1), acc[i][j][v], s) : s + acc[i][j][v];
          red[(i * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3)) * 33 + l32] = s;
        }
      __syncthreads();
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int r = lane + 64 * h;
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < 32; ++c) s += red[r * 33 + c];
        const int row = R0 + r;
        if (row < a.n && C0 < a.m)
          a.rowpart[(((int64_t)b * a.ntn + tn128) * a.n + row) * 2 + kind] = s;
      }
    }
  }

  // C, straight from the accumulators: one store covers 2 rows x 32 consecutive columns
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = R0 + i * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3);
      if (row < a.n) {
        float* crow = C + (int64_t)row * a.ldc + C0 + l32;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (C0 + j * 32 + l32 < a.m) crow[j * 32] = acc[i][j][v];
      }
    }
}

template <bool KCA, bool KCB, bool EPI>
hipError_t launch_one(const GemmArgs& a, hipStream_t st) {
  static bool configured = false;   // per instantiation
  auto kern = gemm_bf16_256<KCA, KCB, EPI>;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int ntm = (a.n + BM - 1) / BM, ntn = (a.m + BN - 1) / BN;
  dim3 grid(ntm * ntn, a.batch);
  hipLaunchKernelGGL(kern, grid, dim3(THREADS), SMEM_BYTES, st, a);
  return hipGetLastError();
}

template <bool EPI>
hipError_t launch_epi(const GemmArgs& a, hipStream_t st) {
  const bool kca = a.trans_a == 0, kcb = a.trans_b != 0;
  if (kca && kcb) return launch_one<true, true, EPI>(a, st);
  if (kca && !kcb) return launch_one<true, false, EPI>(a, st);
  if (!kca && kcb) return launch_one<false, true, EPI>(a, st);
  return launch_one<false, false, EPI>(a, st);
}

}  // namespace

// The fast kernel needs 16-byte aligned operand rows and whole 8-element chunks:
// k % 8 == 0, leading dimensions % 8 == 0, and n (m) % 8 == 0 for an operand stored with n (m)
// contiguous.  Partial sums are produced per 128 x 128 sub-tile.
bool gemm_bf16_fast_ok(const GemmArgs& a) {
  if (a.dtype != GECC_BF16 || a.tile_m != 128 || a.tile_n != 128) return false;
  if (a.k % 8 || a.lda % 8 || a.ldb % 8) return false;
  if (reinterpret_cast<uintptr_t>(a.A) % 16 || reinterpret_cast<uintptr_t>(a.B) % 16) return false;
  if (a.batch > 1 && (a.sa % 8 || a.sb % 8)) return false;
  if (a.trans_a && a.n % 8) return false;
  if (!a.trans_b && a.m % 8) return false;
  return (int64_t)a.n * a.m >= (int64_t)BM * BN;   // smaller problems: the 128 x 128 kernel
}

hipError_t launch_gemm_bf16_fast(const GemmArgs& a, hipStream_t st) {
  return a.rowpart ? launch_epi<true>(a, st) : launch_epi<false>(a, st);
}

}  // namespace gecc
