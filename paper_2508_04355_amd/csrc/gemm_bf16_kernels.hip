// bf16 x bf16 -> fp32 data block of the encoded product (Section III, C = A B), the kernel
// that holds nearly all flops of the path.
//
// Workgroup: 256 x 256 tile of C, 4 wavefronts (2 x 2), each owning a 128 x 128 sub-tile as
// 4 x 4 MFMA 32x32x16 accumulators (256 fp32 registers per lane).  k advances in steps of 32
// through a ring of four LDS stages (4 x 32 KiB).  Operand tiles travel HBM -> LDS directly
// (buffer loads with the LDS bit set: no registers in between, out-of-range rows read as
// zero), three stages ahead of the one the MFMA units are consuming, which is what hides the
// memory latency with a single workgroup per compute unit.
//
// LDS formats, chosen so that neither the DMA writes (64 consecutive 16-byte slots per
// wavefront instruction) nor the fragment reads hit a bank twice:
//   operand contiguous along k in memory:  tile[row][32 k], 64 bytes per row, the four 16-byte
//     chunks of a row XOR-swizzled with (row >> 1) & 3; fragments by ds_read_b128.
//   operand contiguous along m (or n):     tile[32 k][256 m], 512 bytes per k-row, the sixteen
//     32-byte chunks of a row XOR-swizzled with k & 3; fragments by the transposing LDS read
//     (two ds_read_b64_tr_b16 per fragment: 16 lanes fetch 4 k-rows x 16 columns and each
//     lane receives the 4 k-values of its own column).
//
// Epilogue, from the accumulators (C itself never passes through LDS): per sub-tile column
// sums (in-lane) and row sums (through a small LDS transpose) for Section V's syndromes, then
// C.  A second instantiation additionally plants test faults into the accumulators first.
#include <type_traits>
#include "gecc_internal.h"

namespace gecc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

constexpr int THREADS = 256;
constexpr int BM = 256, BN = 256, BK = 32;
constexpr int TILE_BYTES = BM * BK * 2;            // 16 KiB per operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;        // A + B
constexpr int NSTAGE = 4;
constexpr int SMEM_BYTES = NSTAGE * STAGE_BYTES;   // 128 KiB
constexpr int GROUP_M = 8;                         // tile rows per L2-sharing group
constexpr unsigned OOB = 0x80000000u;              // voffset beyond any num_records: reads zero

// one LDS-DMA instruction: 64 lanes x 16 bytes from buffer `rsrc` at (voff + soff) into the
// 1 KiB of LDS starting at lds_addr (lane L lands at lds_addr + 16 L).  Invisible to the
// compiler's memory-counter bookkeeping on purpose: the waits are placed by hand below.
__device__ __forceinline__ void dma16(unsigned lds_addr, unsigned voff, i32x4_t rsrc, unsigned soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}

__device__ __forceinline__ i32x4_t make_rsrc(const void* base, unsigned bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  i32x4_t r;
  r[0] = (int)(p & 0xffffffffu);
  r[1] = (int)((p >> 32) & 0xffffu);       // stride 0: raw buffer, offsets in bytes
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}

// ---- per-operand addressing ---------------------------------------------------------------
// KC = true : element (r, kk) at P[r * ld + kk]  (k contiguous)
// KC = false: element (r, kk) at P[kk * ld + r]  (r contiguous)
template <bool KC>
struct Operand {
  i32x4_t rsrc;
  unsigned voff[4];     // byte offsets of this lane's four 16-byte slots, loop invariant
  unsigned sstep;       // soffset advance per k-tile
  int frag[4];          // LDS byte offset of this lane's fragment address for i = 0..3 (ks = 0)

  // P: operand base for this batch item; r0: first row (m- or n-index) of the tile;
  // rlim: number of valid rows; sub: first row of this wavefront's sub-tile inside the tile
  __device__ __forceinline__ void init(const uint16_t* P, int64_t ld, int r0, int rlim, int klim, int sub) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (KC) {
      const int64_t rows_left = rlim - r0;
      const int64_t bytes = rows_left > 0 ? rows_left * ld * 2 : 0;
      rsrc = make_rsrc(P + (int64_t)r0 * ld, (unsigned)(bytes > 0x7fffffff ? 0x7fffffff : bytes));
      sstep = BK * 2;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s = (wave * 4 + i) * 64 + lane;          // slot in the tile
        const int row = s >> 2, c = (s & 3) ^ ((row >> 1) & 3);
        voff[i] = (unsigned)(row * ld * 2 + c * 16);
      }
      const int l32 = lane & 31, lhi = lane >> 5;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = sub + i * 32 + l32;
        frag[i] = row * 64 + ((lhi ^ ((row >> 1) & 3)) << 4);   // chunk = 2 ks + lhi; ks toggles bit 1
      }
    } else {
      const int64_t bytes = ((int64_t)klim * ld - r0) * 2;
      rsrc = make_rsrc(P + r0, (unsigned)(bytes > 0x7fffffff ? 0x7fffffff : (bytes > 0 ? bytes : 0)));
      sstep = (unsigned)(BK * ld * 2);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s = (wave * 4 + i) * 64 + lane;
        const int krow = s >> 5, p = s & 31;
        const int u = ((((p >> 1) ^ (krow & 3)) << 1) | (p & 1));   // logical 16-byte unit along r
        voff[i] = (r0 + u * 8 < rlim) ? (unsigned)(krow * ld * 2 + u * 16) : OOB;
      }
      // transposing read: in each group of 16 lanes, lane 4 j + q supplies k-row j, columns 4 q..4 q + 3
      const int g = lane >> 4, j = (lane >> 2) & 3, q = lane & 3;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int col = sub + i * 32 + 16 * (g & 1) + 4 * q;        // first of the 4 columns
        const int krow = 8 * (g >> 1) + j;                          // + 16 ks, + 4 for the second read
        const int u = col >> 3;
        frag[i] = krow * 512 + (((((u >> 1) ^ j) << 1) | (u & 1)) << 4) + (col & 7) * 2;
      }
    }
  }

  __device__ __forceinline__ void issue(unsigned lds_tile, unsigned soff) const {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int i = 0; i < 4; ++i) dma16(lds_tile + (wave * 4 + i) * 1024, voff[i], rsrc, soff);
  }

  __device__ __forceinline__ bf16x8_t fragment(const char* tile, int i, int ks) const {
    if (KC) {
      return *reinterpret_cast<const bf16x8_t*>(tile + (frag[i] ^ (ks << 5)));
    } else {
      const char* p = tile + frag[i] + ks * (16 * 512);
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p + 4 * 512));
      const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8_t, v);
    }
  }
};

// Scheduling hint for one quarter (4 MFMAs) of a half k-tile: the NDS LDS reads issued in that
// quarter are placed one or two at a time behind the MFMAs instead of in front of them.
template <int NDS>
__device__ __forceinline__ void hint_quarter() {
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA
    if (r == 0 && (NDS + 3) / 4 > 0) __builtin_amdgcn_sched_group_barrier(0x100, (NDS + 3) / 4, 0);
    if (r == 1 && (NDS + 2) / 4 > 0) __builtin_amdgcn_sched_group_barrier(0x100, (NDS + 2) / 4, 0);
    if (r == 2 && (NDS + 1) / 4 > 0) __builtin_amdgcn_sched_group_barrier(0x100, (NDS + 1) / 4, 0);
    if (r == 3 && NDS / 4 > 0)       __builtin_amdgcn_sched_group_barrier(0x100, NDS / 4, 0);
  }
}
// reads per quarter: B fragments 0-2 | B fragment 3 and A fragments 0-1 | A fragments 2-3 | none
template <bool KCA, bool KCB>
__device__ __forceinline__ void interleave(int quarter, bool reads) {
  constexpr int NA = KCA ? 1 : 2, NB = KCB ? 1 : 2;   // LDS instructions per fragment
  if (!reads || quarter == 3) hint_quarter<0>();
  else if (quarter == 0)      hint_quarter<3 * NB>();
  else if (quarter == 1)      hint_quarter<NB + 2 * NA>();
  else                        hint_quarter<2 * NA>();
}

template <bool KCA, bool KCB, bool EPI, bool FAULTS>
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

  Operand<KCA> oa;
  Operand<KCB> ob;
  oa.init(A, a.lda, tile_r0, a.n, a.k, wr * 128);
  ob.init(B, a.ldb, tile_c0, a.m, a.k, wc * 128);

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // LDS byte address of the ring (the address-space-3 pointer value, not the flat address)
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const int KT = a.k / BK;                           // k % 32 == 0 (checked by the launcher)
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);

  // Software pipeline.  Stage t = k-tile t in ring slot t & 3.  Two fragment sets: fr0 for the
  // first 16 k of a stage, fr1 for the second.  Steady state of iteration kt:
  //     read fr1 of stage kt | 16 MFMAs on fr0 | stage kt+1 landed? barrier | start the DMA of
  //     stage kt+4 into the slot stage kt just left, read fr0 of stage kt+1 | 16 MFMAs on fr1
  // so every LDS read and every DMA issue has 16 MFMAs (512 cycles) of cover.
#pragma unroll
  for (int s = 0; s < NSTAGE; ++s)
    if (s < KT) {
      oa.issue(lds0 + s * STAGE_BYTES, s * oa.sstep);
      ob.issue(lds0 + s * STAGE_BYTES + TILE_BYTES, s * ob.sstep);
    }
  {
    const int younger = min(NSTAGE - 1, KT - 1);
    if (younger >= 3)      asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    else if (younger == 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (younger == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else                   asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  bf16x8_t fa0[4], fb0[4], fa1[4], fb1[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    fa0[i] = oa.fragment(smem, i, 0);
    fb0[i] = ob.fragment(smem + TILE_BYTES, i, 0);
  }

  // one k-tile; REFILL / NEXT are compile-time in the steady state so that the body is one
  // basic block the scheduler can interleave freely
  auto k_tile = [&](auto refill_c, auto next_c, const int kt) {
    constexpr bool REFILL = decltype(refill_c)::value, NEXT = decltype(next_c)::value;
    const char* cur = smem + (kt & (NSTAGE - 1)) * STAGE_BYTES;
    const char* nxt = smem + ((kt + 1) & (NSTAGE - 1)) * STAGE_BYTES;
    // first half: 16 MFMAs on fr0; the reads of fr1 (second 16 k of stage kt) are spread over
    // the first three quarters, B fragments first (every quarter of the next half needs all of
    // them, but only one A fragment)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i == 0) { fb1[0] = ob.fragment(cur + TILE_BYTES, 0, 1); fb1[1] = ob.fragment(cur + TILE_BYTES, 1, 1);
                    fb1[2] = ob.fragment(cur + TILE_BYTES, 2, 1); }
      if (i == 1) { fb1[3] = ob.fragment(cur + TILE_BYTES, 3, 1); fa1[0] = oa.fragment(cur, 0, 1);
                    fa1[1] = oa.fragment(cur, 1, 1); }
      if (i == 2) { fa1[2] = oa.fragment(cur, 2, 1); fa1[3] = oa.fragment(cur, 3, 1); }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0[i], fb0[j], acc[i][j], 0, 0, 0);
      interleave<KCA, KCB>(i, true);
    }
    __builtin_amdgcn_sched_barrier(0);

    if (NEXT) {
      // stage kt+1 has landed once only the (up to two) younger stages are still pending
      const int younger = REFILL ? NSTAGE - 2 : min(NSTAGE - 2, KT - 2 - kt);
      if (younger >= 2)      asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      else if (younger == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else                   asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own reads of stage kt are back
    __builtin_amdgcn_s_barrier();        // stage kt+1 complete for everyone; stage kt released
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // second half: 16 MFMAs on fr1; between them the reads of fr0 of stage kt+1 and the DMA of
    // stage kt+4 into the slot stage kt just left
    const unsigned slot = lds0 + (kt & (NSTAGE - 1)) * STAGE_BYTES + (wave_u * 4) * 1024;
    const unsigned sa_off = (kt + NSTAGE) * oa.sstep, sb_off = (kt + NSTAGE) * ob.sstep;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (NEXT) {
        if (i == 0) { fb0[0] = ob.fragment(nxt + TILE_BYTES, 0, 0); fb0[1] = ob.fragment(nxt + TILE_BYTES, 1, 0);
                      fb0[2] = ob.fragment(nxt + TILE_BYTES, 2, 0); }
        if (i == 1) { fb0[3] = ob.fragment(nxt + TILE_BYTES, 3, 0); fa0[0] = oa.fragment(nxt, 0, 0);
                      fa0[1] = oa.fragment(nxt, 1, 0); }
        if (i == 2) { fa0[2] = oa.fragment(nxt, 2, 0); fa0[3] = oa.fragment(nxt, 3, 0); }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1[i], fb1[j], acc[i][j], 0, 0, 0);
      interleave<KCA, KCB>(i, NEXT);
      __builtin_amdgcn_sched_barrier(0);
      if (REFILL) {
        dma16(slot + i * 1024, oa.voff[i], oa.rsrc, sa_off);
        dma16(slot + TILE_BYTES + i * 1024, ob.voff[i], ob.rsrc, sb_off);
      }
    }
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  int kt = 0;
  for (; kt + NSTAGE < KT; ++kt) k_tile(T_{}, T_{}, kt);   // steady state
  for (; kt + 1 < KT; ++kt) k_tile(F_{}, T_{}, kt);        // drain: nothing left to fetch
  k_tile(F_{}, F_{}, kt);                                  // last k-tile
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // ---- epilogue -------------------------------------------------------------------------------
  const int R0 = tile_r0 + wr * 128, C0 = tile_c0 + wc * 128;   // origin of this wavefront's sub-tile
  if (FAULTS) {
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

template <bool KCA, bool KCB, bool EPI, bool FAULTS>
hipError_t launch_one(const GemmArgs& a, hipStream_t st) {
  static bool configured = false;   // per instantiation
  auto kern = gemm_bf16_256<KCA, KCB, EPI, FAULTS>;
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

template <bool EPI, bool FAULTS>
hipError_t launch_layout(const GemmArgs& a, hipStream_t st) {
  const bool kca = a.trans_a == 0, kcb = a.trans_b != 0;
  if (kca && kcb) return launch_one<true, true, EPI, FAULTS>(a, st);
  if (kca && !kcb) return launch_one<true, false, EPI, FAULTS>(a, st);
  if (!kca && kcb) return launch_one<false, true, EPI, FAULTS>(a, st);
  return launch_one<false, false, EPI, FAULTS>(a, st);
}

}  // namespace

// The fast kernel needs 16-byte aligned operand rows, whole 16-byte chunks and whole k-tiles:
// k % 32 == 0, leading dimensions % 8 == 0, n (m) % 8 == 0 for an operand stored with n (m)
// contiguous, and operand panels that 32-bit byte offsets can address.  Partial sums are
// produced per 128 x 128 sub-tile.  Everything else goes to the generic 128 x 128 kernel.
bool gemm_bf16_fast_ok(const GemmArgs& a) {
  if (a.dtype != GECC_BF16 || a.tile_m != 128 || a.tile_n != 128) return false;
  if (a.k % BK || a.lda % 8 || a.ldb % 8) return false;
  if (reinterpret_cast<uintptr_t>(a.A) % 16 || reinterpret_cast<uintptr_t>(a.B) % 16) return false;
  if (a.batch > 1 && (a.sa % 8 || a.sb % 8)) return false;
  if (a.trans_a && a.n % 8) return false;
  if (!a.trans_b && a.m % 8) return false;
  // byte offsets inside a tile panel (k-contiguous: 256 rows; otherwise the whole k extent)
  const int64_t span_a = (a.trans_a ? (int64_t)a.k : (int64_t)BM) * a.lda * 2;
  const int64_t span_b = (a.trans_b ? (int64_t)BN : (int64_t)a.k) * a.ldb * 2;
  if (span_a >= 0x7fffffff || span_b >= 0x7fffffff) return false;
  return (int64_t)a.n * a.m >= (int64_t)BM * BN;   // smaller problems: the 128 x 128 kernel
}

hipError_t launch_gemm_bf16_fast(const GemmArgs& a, hipStream_t st) {
  if (!a.rowpart) return launch_layout<false, false>(a, st);
  return a.n_faults > 0 ? launch_layout<true, true>(a, st) : launch_layout<true, false>(a, st);
}

}  // namespace gecc
