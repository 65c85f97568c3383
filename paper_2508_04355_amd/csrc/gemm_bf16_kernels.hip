// bf16 x bf16 -> fp32 data block of the encoded product (Section III, C = A B), the kernel
// that holds nearly all flops of the path.
//
// Workgroup: 256 x 256 tile of C, 4 wavefronts (2 x 2), each owning a 128 x 128 sub-tile as
// 8 x 8 MFMA 16x16x32 accumulators (256 fp32 registers per lane).  k advances in tiles of 32.
// (Both bf16 MFMA shapes deliver 1024 flop per cycle and SIMD, but the chip is power-limited
// under this load and sustains a 15 % higher clock on 16x16x32 than on 32x32x16.)
// Operand tiles travel HBM -> LDS directly (buffer loads with the LDS bit set: no registers in
// between, out-of-range rows read as zero) and several k-tiles ahead of the one the MFMA units
// are consuming, which is what hides the memory latency with one workgroup per compute unit.
// Every request asks L2 for whole 128-byte lines: the L2 request rate, not its bandwidth, is
// what 32 compute units per XCD saturate first.
//
// LDS (64 KiB per operand), laid out so that neither the DMA writes (64 consecutive 16-byte
// slots per wavefront instruction) nor the fragment reads hit a bank twice:
// (the LDS serves 256 bytes per cycle from 64 banks: 16 lanes of a 16-byte read, 32 lanes of
// an 8-byte read):
//   operand contiguous along k in memory:  two slots, each a PAIR of k-tiles: tile[row][64 k],
//     128 bytes per row (one full line per row and request), the eight 16-byte chunks of a row
//     XOR-swizzled with (row >> 1) & 7; fragments (16 rows x 32 k) by ds_read_b128.
//   operand contiguous along m (or n):     four slots of one k-tile: tile[32 k][256 m], 512
//     bytes per k-row, the eight 64-byte chunks of a row XOR-swizzled with k & 3 and the two
//     32-byte halves of a chunk swapped when k & 8; fragments by the transposing LDS read (two
//     ds_read_b64_tr_b16 per fragment: 16 lanes fetch 4 k-rows x 16 columns and each lane
//     receives the 4 k-values of its own column).
//
// Epilogue, from the accumulators (C itself never passes through LDS): one branch-free pass that
// stores C through a range-checked raw buffer (rows and columns outside C are dropped by the
// hardware) and forms, per 128 x 128 sub-tile, the column sums (in-lane) and row sums (through
// a small LDS transpose) for Section V's syndromes.  Test faults, when a list is given, are
// planted into the accumulators first.
//
// Every tile walks k cyclically from its own start (a few k-tiles apart for neighbouring
// tiles), so that the compute units sharing an operand panel do not ask L2 for the same line
// in the same cycle: the first one misses, the others hit.
#include <mutex>
#include <type_traits>
#include "gecc_internal.h"

namespace gecc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

constexpr int THREADS = 256;
constexpr int BM = 256, BN = 256, BK = 32;
constexpr int TILE_BYTES = BM * BK * 2;            // 16 KiB: one k-tile of one operand
constexpr int NSTAGE = 4;                          // k-tiles of one operand resident in LDS
constexpr int REGION_BYTES = NSTAGE * TILE_BYTES;  // 64 KiB per operand
constexpr int SMEM_BYTES = 2 * REGION_BYTES;       // 128 KiB
constexpr int EPI_SMEM_BYTES = 4 * 2 * 128 * 17 * 4;  // 68 KiB: row-sum transpose of the epilogue
// DMA spread (see the schedule in the kernel): the 8 instructions of a pair go out as early as its
// slot allows (all in the half after the slot is released when there is one k-contiguous operand,
// 5 + 3 over two halves when there are two: a burst of 16 makes the address unit push back); the
// 4 instructions of a single k-tile go into its first half
constexpr int MX = 0;
constexpr int SKEW_M = 1, SKEW_N = 1;              // k start offset (pairs of k-tiles) per tile row / column
constexpr int GROUP_M = 8;                         // tile rows per L2-sharing group
constexpr unsigned OOB = 0x80000000u;              // voffset beyond any num_records: reads zero

// one LDS-DMA instruction: 64 lanes x 16 bytes from buffer `rsrc` at (voff + soff) into the
// 1 KiB of LDS starting at lds_addr (lane L lands at lds_addr + 16 L).  Invisible to the
// compiler's memory-counter bookkeeping on purpose: the waits are placed by hand below.
__device__ __forceinline__ void dma16(unsigned lds_addr, unsigned voff, i32x4_t rsrc, unsigned soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
// The same in two parts, for the main loop, where an MFMA goes between them (M0 must be written
// at least one instruction before the load that reads it; nothing else in the loop writes M0)
template <unsigned LDS_OFF>
__device__ __forceinline__ void dma16_dest(unsigned lds_base) {
  asm volatile("s_add_u32 m0, %0, %1" :: "s"(lds_base), "n"(LDS_OFF) : "memory", "scc");
}
__device__ __forceinline__ void dma16_load(unsigned voff, i32x4_t rsrc, unsigned soff) {
  asm volatile("buffer_load_dwordx4 %0, %1, %2 offen lds" :: "v"(voff), "s"(rsrc), "s"(soff) : "memory");
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
// KC = true : element (r, kk) at P[r * ld + kk]  (k contiguous);  LDS: 2 slots x pair of k-tiles
// KC = false: element (r, kk) at P[kk * ld + r]  (r contiguous);  LDS: 4 slots x one k-tile
template <bool KC>
struct Operand {
  static constexpr int NV = KC ? 8 : 4;   // DMA instructions of this wavefront per pair / per k-tile
  i32x4_t rsrc;
  unsigned voff[NV];    // byte offsets of this lane's 16-byte slots, loop invariant
  unsigned sstep;       // soffset advance per pair (KC) / per k-tile
  int frag[8];          // LDS byte offset of this lane's fragment address for i = 0..7 (16 rows each)

  // P: operand base for this batch item; r0: first row (m- or n-index) of the tile;
  // rlim: number of valid rows; sub: first row of this wavefront's sub-tile inside the tile
  __device__ __forceinline__ void init(const uint16_t* P, int64_t ld, int r0, int rlim, int klim, int sub) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (KC) {
      const int64_t rows_left = rlim - r0;
      const int64_t bytes = rows_left > 0 ? rows_left * ld * 2 : 0;
      rsrc = make_rsrc(P + (int64_t)r0 * ld, (unsigned)(bytes > 0x7fffffff ? 0x7fffffff : bytes));
      sstep = 2 * BK * 2;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int s = (wave * NV + i) * 64 + lane;          // slot in the pair tile
        const int row = s >> 3, c = (s & 7) ^ ((row >> 1) & 7);   // 8 lanes = one 128-byte line
        voff[i] = (unsigned)(row * ld * 2 + c * 16);
      }
      const int l16 = lane & 15, g = lane >> 4;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = sub + i * 16 + l16;
        // chunk = 4 (k-tile parity) + g: lane group g holds k = 8 g .. 8 g + 7 of the k-tile; the
        // parity toggles bit 6 of the offset
        frag[i] = row * 128 + ((g ^ ((row >> 1) & 7)) << 4);
      }
    } else {
      const int64_t bytes = ((int64_t)klim * ld - r0) * 2;
      rsrc = make_rsrc(P + r0, (unsigned)(bytes > 0x7fffffff ? 0x7fffffff : (bytes > 0 ? bytes : 0)));
      sstep = (unsigned)(BK * ld * 2);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int s = (wave * NV + i) * 64 + lane;
        const int krow = s >> 5, p = s & 31;
        const int u = ((((p >> 2) ^ (krow & 3)) << 2) | ((p & 3) ^ (((krow >> 3) & 1) << 1)));   // logical 16-byte unit along r
        voff[i] = (r0 + u * 8 < rlim) ? (unsigned)(krow * ld * 2 + u * 16) : OOB;
      }
      // transposing read: in each group of 16 lanes, lane 4 j + q supplies k-row j, columns
      // 4 q..4 q + 3, and lane t receives the 4 k-values of column t; group g reads k-rows 8 g + j
      // (+ 4 for the second read), which makes lane (t, g) hold k = 8 g .. 8 g + 7 of row t
      const int g = lane >> 4, j = (lane >> 2) & 3, q = lane & 3;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int col = sub + i * 16 + 4 * q;                       // first of the 4 columns
        const int krow = 8 * g + j;
        const int u = col >> 3;
        frag[i] = krow * 512 + (((((u >> 2) ^ j) << 2) | ((u & 3) ^ ((g & 1) << 1))) << 4) + (col & 7) * 2;
      }
    }
  }

  // LDS byte offset (inside this operand's region) of the slot that holds k-tile kt
  static __device__ __forceinline__ int slot_of(int kt) {
    return KC ? ((kt >> 1) & 1) * (2 * TILE_BYTES) : (kt & (NSTAGE - 1)) * TILE_BYTES;
  }

  // DMA instruction i (0 .. NV-1) of this wavefront: unit (pair or k-tile) number `src` into the
  // slot that unit number `unit` owns
  __device__ __forceinline__ void issue_one(unsigned lds_region, int wave_u, int unit, int src, int i) const {
    const unsigned slot = KC ? (unit & 1) * (2 * TILE_BYTES) : (unit & (NSTAGE - 1)) * TILE_BYTES;
    dma16(lds_region + slot + (wave_u * NV + i) * 1024, voff[i], rsrc, src * sstep);
  }
  // ... in two parts (PART 0: destination into M0, PART 1: the load)
  // UNIT: the unit's number modulo the slots (a compile-time constant in the main loop)
  template <int PART, int UNIT>
  __device__ __forceinline__ void issue_part(unsigned lds_region, int wave_u, int src, int i) const {
    constexpr unsigned slot = KC ? (UNIT & 1) * (2 * TILE_BYTES) : (UNIT & (NSTAGE - 1)) * TILE_BYTES;
    if (PART == 0) dma16_dest<slot>(lds_region + (wave_u * NV + i) * 1024);
    else if (PART == 1) dma16_load(voff[i], rsrc, src * sstep);
    else dma16(lds_region + slot + (wave_u * NV + i) * 1024, voff[i], rsrc, src * sstep);
  }
  __device__ __forceinline__ void issue_range(unsigned lds_region, int wave_u, int unit, int src, int first, int count) const {
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (i >= first && i < first + count) issue_one(lds_region, wave_u, unit, src, i);
  }

  // fragment i (16 rows x the 32 k) of k-tile kt, as two halves of 4 k-values per lane (a
  // transposing read fetches one half; the main loop puts them behind different MFMAs);
  // region = this operand's LDS region
  struct Frag {
    s16x4_t lo, hi;
    __device__ __forceinline__ bf16x8_t get() const {
      return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };
  // PART 0: all of a k-contiguous operand's fragment (one ds_read_b128), else the first half;
  // PART 1: the second half of the other kind
  // KT4: the k-tile's number modulo 4 (a compile-time constant in the main loop, so that slot
  // and fragment become the immediate offset of the read: the address registers are loop invariant)
  template <int PART, int KT4>
  __device__ __forceinline__ void fragment_part(Frag& f, const char* region, int i) const {
    if (KC) {
      if (PART == 0) {
        // frag[i] = frag[0] + 2048 i, and the parity only toggles bit 6 of frag[0]
        const char* p = region + (frag[0] ^ ((KT4 & 1) << 6)) + (((KT4 >> 1) & 1) * (2 * TILE_BYTES) + i * 2048);
        const s16x8_t v = *reinterpret_cast<const s16x8_t*>(p);
        f.lo = __builtin_shufflevector(v, v, 0, 1, 2, 3);
        f.hi = __builtin_shufflevector(v, v, 4, 5, 6, 7);
      }
    } else {
      const char* p = region + frag[i] + (KT4 & (NSTAGE - 1)) * TILE_BYTES;
      if (PART == 0) f.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p));
      else           f.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p + 4 * 512));
    }
  }
  // k-tile 0 (prologue)
  __device__ __forceinline__ void fragment(Frag& f, const char* region, int i) const {
    fragment_part<0, 0>(f, region, i);
    fragment_part<1, 0>(f, region, i);
  }
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// What goes behind each of the 32 MFMAs of a half.  Measured on the chip with one wavefront per
// SIMD: behind a 16-cycle MFMA one other instruction issues for free, a second costs 4 cycles,
// a third 8 more.  So the D DMA instructions of the half (two instructions each: destination
// into M0, then -- behind the next MFMA, which also is the wait state M0 needs -- the load) and
// its R LDS reads are dealt out one per MFMA, DMA instructions evenly over the half, reads from
// MFMA number G0 on and over the first four fifths of it (their data is needed when the half ends).
// With more than 32 of them some MFMAs get two.  S further scalar instructions (the bookkeeping
// of the cyclic k order) go behind MFMAs that have nothing yet, from the end of the half
// backwards, then next to LDS reads (a read and a scalar instruction together still cost nothing).
enum { OP_NONE = 0, OP_READ = 1, OP_DEST = 2, OP_LOAD = 3, OP_DMA = 4 /* both parts, with the wait state */ };
struct HalfPlan {
  signed char kind[32][2], idx[32][2], scalar[32];
};
template <int D, int R, int G0, int S>
constexpr HalfPlan make_half_plan() {
  HalfPlan p{};
  for (int g = 0; g < 32; ++g) p.scalar[g] = -1;
  int sk[80] = {}, si[80] = {}, T = 0;
  int d = 0, r = 0;
  while (d < D || r < R) {   // merge by position: DMA d at (d + 1/2) / D, read r at 4/5 (r + 1/2) / R
    const bool dma = d < D && (r >= R || 5 * (2 * d + 1) * R <= 4 * (2 * r + 1) * D);
    if (dma) { sk[T] = OP_DEST; si[T] = d; ++T; sk[T] = OP_LOAD; si[T] = d; ++T; ++d; }
    else { sk[T] = OP_READ; si[T] = r; ++T; ++r; }
  }
  const int cap = 32 - G0, den = T > cap ? T : cap;
  int fill[32] = {};
  for (int k = 0; k < T; ++k) {
    int g = G0 + k * cap / den;
    while (fill[g] >= 2) ++g;                       // (never past 31: T <= 64 - 2 G0 is asserted by the caller)
    if (fill[g] == 1 && p.kind[g][0] == OP_DEST && sk[k] == OP_LOAD) { p.kind[g][0] = OP_DMA; continue; }
    p.kind[g][fill[g]] = (signed char)sk[k];
    p.idx[g][fill[g]] = (signed char)si[k];
    ++fill[g];
  }
  int left = S;     // scalar instruction number S - left goes ...
  for (int g = 31; g >= 0 && left > 0; --g)
    if (fill[g] == 0) { p.scalar[g] = (signed char)(left - 1); --left; }
  for (int g = 31; g >= 0 && left > 0; --g)
    if (p.scalar[g] < 0 && fill[g] == 1 && p.kind[g][0] == OP_READ) { p.scalar[g] = (signed char)(left - 1); --left; }
  for (int g = 31; g >= 0 && left > 0; --g)
    if (p.scalar[g] < 0) { p.scalar[g] = (signed char)(left - 1); --left; }
  return p;
}
// What the kernel relies on: every read and every scalar instruction once and in order of their
// numbers (the scalar ones depend on each other); every DMA instruction once, its load behind a
// later MFMA than its destination (or both together, with the wait state), and no other
// destination in between (there is one M0)
template <int D, int R, int G0, int S>
constexpr bool half_plan_ok(const HalfPlan& p) {
  int next_read = 0, next_scalar = 0, next_dest = 0, next_load = 0;
  for (int g = 0; g < 32; ++g) {
    for (int sl = 0; sl < 2; ++sl) {
      const int k = p.kind[g][sl], i = p.idx[g][sl];
      if (k == OP_NONE) continue;
      if (g < G0) return false;
      if (k == OP_READ) { if (i != next_read) return false; ++next_read; }
      else if (k == OP_DEST) { if (i != next_dest || next_load != next_dest) return false; ++next_dest; }
      else if (k == OP_LOAD) { if (i != next_load || next_dest != next_load + 1 || (sl != 0 && p.kind[g][0] == OP_DEST)) return false; ++next_load; }
      else if (k == OP_DMA) { if (i != next_dest || next_load != next_dest) return false; ++next_dest; ++next_load; }
      else return false;
    }
    if (p.scalar[g] >= 0) { if (p.scalar[g] != next_scalar) return false; ++next_scalar; }
  }
  return next_read == R && next_dest == D && next_load == D && next_scalar == S;
}
template <int D, int R, int G0, int S>
inline constexpr HalfPlan kHalfPlan = make_half_plan<D, R, G0, S>();

// s_waitcnt vmcnt(N), N a compile-time constant below 64
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// ---- tile order: consecutive workgroups land on different XCDs (round robin), so give every
// XCD a contiguous range of the tile sequence; inside it walk GROUP_M tile rows at a time, column
// by column, so that co-resident tiles share A row panels and B column panels.
// Where the tile counts allow it (sr > 0, chosen by the launcher), a whole round of 256 workgroups
// takes a block of sr x sc tiles instead, XCD x an 8 x 4 sub-block of it: sr + sc operand
// panels per round instead of 64 + 4, which keeps a round's panels inside the 256 MiB memory-side
// cache when k is long (cfg4-dgrad: 234 MB instead of 500 MB per round, product +6 %).
__device__ __forceinline__ void tile_of(int pid, int ntm, int ntn, int sr, int sc, int& tm, int& tn) {
  const int ntiles = ntm * ntn;
  if (sr > 0) {
    const int q = pid >> 8, w = pid & 255, x = w & 7, idx = w >> 3;
    const int nsn = ntn / sc, xc = sc >> 2;
    const int sbm = q / nsn, sbn = q - sbm * nsn;
    tm = sbm * sr + (x / xc) * 8 + (idx & 7);
    tn = sbn * sc + (x % xc) * 4 + (idx >> 3);
    return;
  }
  {
    const int per = ntiles / 8, rem = ntiles - per * 8;     // XCD x gets per (+1 if x < rem)
    const int x = pid & 7, idx = pid >> 3;
    pid = x * per + min(x, rem) + idx;
  }
  const int gsz = GROUP_M * ntn;
  const int grp = pid / gsz;
  const int first_m = grp * GROUP_M;
  const int gm = min(GROUP_M, ntm - first_m);
  tm = first_m + (pid - grp * gsz) % gm;
  tn = (pid - grp * gsz) / gm;
}

// The k-split tail (see launch_one): a tile of the last, at most half filled round is computed
// by two workgroups, one per half of k, which add their halves into C and into the partial sums.
// Both are zeroed first, by the first workgroups of the launch that computes the full rounds
// (one tail tile each, before their own tile: that launch ends before the split one starts).
__device__ __forceinline__ void zero_tail_tile(const GemmArgs& a, int tile) {
  const int ntm = (a.n + BM - 1) / BM, ntn = (a.m + BN - 1) / BN;
  int tm, tn;
  tile_of(tile, ntm, ntn, a.map_sr, a.map_sc, tm, tn);
  const int r0 = tm * BM, c0 = tn * BN;
  const int rows = min(BM, a.n - r0), cols = min(BN, a.m - c0);
  for (int o = threadIdx.x; o < rows * BN; o += 256) {
    const int r = o / BN, c = o % BN;
    if (c < cols) a.C[(int64_t)(r0 + r) * a.ldc + c0 + c] = 0.f;
  }
  if (a.rowpart) {
    for (int o = threadIdx.x; o < 2 * BM; o += 256) {          // two 128-column slabs x 256 rows
      const int tn128 = 2 * tn + o / BM, row = r0 + o % BM;
      if (row < a.n && tn128 * 128 < a.m) {
        float2* rp = reinterpret_cast<float2*>(a.rowpart + ((int64_t)tn128 * a.rp_ld + row) * 2);
        *rp = make_float2(0.f, 0.f);
      }
    }
    for (int o = threadIdx.x; o < 2 * BN; o += 256) {
      const int tm128 = 2 * tm + o / BN, col = c0 + o % BN;
      if (col < a.m && tm128 * 128 < a.n) {
        float2* cp = reinterpret_cast<float2*>(a.colpart + ((int64_t)tm128 * a.cp_ld + col) * 2);
        *cp = make_float2(0.f, 0.f);
      }
    }
  }
}

template <bool KCA, bool KCB, bool EPI, bool SP>
__global__ __launch_bounds__(THREADS, 1) void gemm_bf16_256(GemmArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int l16 = lane & 15, lg = lane >> 4;
  const int b = blockIdx.y;
  if (!SP && a.split_first >= 0) {
    const int ntiles_all = ((a.n + BM - 1) / BM) * ((a.m + BN - 1) / BN);
    if (a.split_first + (int)blockIdx.x < ntiles_all) zero_tail_tile(a, a.split_first + (int)blockIdx.x);
  }

  const int ntm = (a.n + BM - 1) / BM, ntn = (a.m + BN - 1) / BN;
  // SP (the k-split launch, see launch_one): the workgroups share the tiles from split_first on
  // in pairs, khalf = 0 / 1 takes the first / second half of k.  Otherwise: one tile, all of k.
  const int khalf = SP ? (int)(blockIdx.x & 1) : -1;
  int tm, tn;
  tile_of(SP ? a.split_first + (int)(blockIdx.x >> 1) : (int)blockIdx.x, ntm, ntn, a.map_sr, a.map_sc, tm, tn);
  const int tile_r0 = tm * BM, tile_c0 = tn * BN;
  const int KT = SP ? a.k / (2 * BK) : a.k / BK;                 // even (checked by the launcher)
  const int k0 = khalf == 1 ? KT * BK : 0;

  const uint16_t* A = reinterpret_cast<const uint16_t*>(a.A) + (int64_t)b * a.sa + (KCA ? (int64_t)k0 : (int64_t)k0 * a.lda);
  const uint16_t* B = reinterpret_cast<const uint16_t*>(a.B) + (int64_t)b * a.sb + (KCB ? (int64_t)k0 : (int64_t)k0 * a.ldb);
  float* C = a.C + (int64_t)b * a.sc;

  Operand<KCA> oa;
  Operand<KCB> ob;
  oa.init(A, a.lda, tile_r0, a.n, KT * BK, wr * 128);
  ob.init(B, a.ldb, tile_c0, a.m, KT * BK, wc * 128);

  // acc[i][j][v] = C[16 i + 4 g + v][16 j + l16] of the sub-tile (g = lane >> 4, l16 = lane & 15)
  f32x4_t acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

  // LDS byte addresses of the two operand regions (address-space-3 values, not flat addresses)
  const unsigned ldsA = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  const unsigned ldsB = ldsA + REGION_BYTES;
  const char* regA = smem;
  const char* regB = smem + REGION_BYTES;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);

  // ---- DMA schedule ---------------------------------------------------------------------------
  // A "unit" is what one LDS slot holds: a pair of k-tiles for a k-contiguous operand (nK of
  // them, 8 instructions per wavefront and unit), one k-tile otherwise (nM of them, 4
  // instructions).  An iteration (one k-tile) has two halves of 16 steps (two MFMAs each) with
  // the workgroup barrier between them; that barrier releases the slot of k-tile kt (and of its pair when kt
  // is odd) and is where k-tile kt+1 must have landed.  Where the loads go is a trade between
  // lead time (a pair's slot is free from the barrier of k-tile 2q+1 on and its data is needed
  // at the barrier of 2q+3; with two k-contiguous operands the wavefronts used to wait there for
  // a sixth of the loop) and bursts (the address unit takes one instruction per 16 cycles):
  //   pair q+2:      PA instructions in the 2nd half of k-tile 2q+1, PB in the 1st half of
  //                  2q+2, PC = 8 - PA - PB in the 2nd half of 2q+2   (needed at barrier 2q+3)
  //   k-tile kt+4:   MX instructions in the 2nd half of kt, the rest in the 1st half of kt+1
  // Inside a half the k-contiguous operands go first.  The memory counter retires in order, so
  // "k-tile kt+1 has landed" becomes "at most W instructions are pending", W = at most what the
  // schedule issues after the last instruction of that k-tile's units (for any PA, PB, PC):
  //   kt even: (PA + PB) nK + 8 nM        kt odd: 4 nM  (8 nM without a k-contiguous operand)
  // Units past the end of k wrap around to the start of the tile's cyclic order (a harmless
  // reload into a free slot that nobody reads), which keeps every iteration identical.
  constexpr int nK = (KCA ? 1 : 0) + (KCB ? 1 : 0), nM = 2 - nK;
  constexpr int PA = nK == 2 ? 5 : 8, PB = 8 - PA, PC = 8 - PA - PB;
  constexpr int W_EVEN = (PA + PB) * nK + 8 * nM, W_ODD = nK > 0 ? 4 * nM : 8 * nM;
  const int NP = KT / 2;
  // k order of this tile: cyclic, starting at pair p0 (see SKEW_M, SKEW_N)
  const int p0 = __builtin_amdgcn_readfirstlane(((tm & 7) * SKEW_M + (tn & 3) * SKEW_N) % NP);
  auto src_pair = [&](int pair) { int x = pair + p0; x -= x >= NP ? NP : 0; x -= x >= NP ? NP : 0; return x; };
  auto src_kt = [&](int t) { int x = t + 2 * p0; x -= x >= KT ? KT : 0; x -= x >= KT ? KT : 0; return x; };

  // Sources (cyclic k order) of what the loop requests next, kept as running scalars: cp = pair
  // kt/2 + 1 and cn = pair kt/2 + 2 of the current even kt, cm0 = k-tile kt + 3, cm1 = kt + 4
  int cp = src_pair(1), cn = src_pair(2), cm0 = src_kt(3), cm1 = src_kt(4);
  // DMA instructions of half PH (0: 1st of even kt, 1: 2nd of even, 2: 1st of odd, 3: 2nd of odd)
  // that belong behind step number `step` of the half
  // DMA instruction number ORD of half PH of the main loop (PH = 0..3: the halves of k-tiles kt,
  // kt + 1 with kt = 0 mod 4; 4..7: those of kt + 2, kt + 3), PART 0: destination, 1: load, 2: both
  auto dma_op = [&](auto ph_c, auto part_c, auto ord_c) {
    constexpr int PH8 = decltype(ph_c)::value, PH = PH8 & 3, KT0 = (PH8 >> 2) * 2 + (PH >> 1);   // k-tile mod 4
    constexpr int PART = decltype(part_c)::value, ORD = decltype(ord_c)::value;
    constexpr int k_cnt = PH == 3 ? PA : PH == 0 ? PB : PH == 1 ? PC : 0;       // per operand
    constexpr int k_first = PH == 3 ? 0 : PH == 0 ? PA : PA + PB;
    constexpr int m_cnt = (PH & 1) ? MX : 4 - MX;
    constexpr int m_first = (PH & 1) ? 0 : MX;
    constexpr int pair = PH == 3 ? (KT0 + 3) >> 1 : (KT0 + 2) >> 1;   // slot
    constexpr int mt = (PH & 1) ? KT0 + 4 : KT0 + 3;
    static_assert(MX == 0, "the running sources cover the k-tiles requested in first halves only");
    const int spair = PH == 3 ? cn : cp, smt = PH == 2 ? cm1 : cm0;
    int r = 0;
#pragma unroll
    for (int x = 0; x < k_cnt; ++x) {
      if (KCA) { if (r == ORD) oa.template issue_part<PART, pair>(ldsA, wave_u, spair, k_first + x); ++r; }
      if (KCB) { if (r == ORD) ob.template issue_part<PART, pair>(ldsB, wave_u, spair, k_first + x); ++r; }
    }
#pragma unroll
    for (int x = 0; x < m_cnt; ++x) {
      if (!KCA) { if (r == ORD) oa.template issue_part<PART, mt>(ldsA, wave_u, smt, m_first + x); ++r; }
      if (!KCB) { if (r == ORD) ob.template issue_part<PART, mt>(ldsB, wave_u, smt, m_first + x); ++r; }
    }
  };

  // prologue, in the order the waits assume: pair 0, k-tile 0 | k-tile 1 | start of pair 1,
  // k-tile 2, start of k-tile 3
  if (KCA) oa.issue_range(ldsA, wave_u, 0, src_pair(0), 0, 8);
  if (KCB) ob.issue_range(ldsB, wave_u, 0, src_pair(0), 0, 8);
  if (!KCA) oa.issue_range(ldsA, wave_u, 0, src_kt(0), 0, 4);
  if (!KCB) ob.issue_range(ldsB, wave_u, 0, src_kt(0), 0, 4);
  if (!KCA) oa.issue_range(ldsA, wave_u, 1, src_kt(1), 0, 4);
  if (!KCB) ob.issue_range(ldsB, wave_u, 1, src_kt(1), 0, 4);
  if (KCA) oa.issue_range(ldsA, wave_u, 1, src_pair(1), 0, PA);
  if (KCB) ob.issue_range(ldsB, wave_u, 1, src_pair(1), 0, PA);
  if (!KCA) oa.issue_range(ldsA, wave_u, 2, src_kt(2), 0, 4);
  if (!KCB) ob.issue_range(ldsB, wave_u, 2, src_kt(2), 0, 4);
  if (!KCA) oa.issue_range(ldsA, wave_u, 3, src_kt(3), 0, MX);
  if (!KCB) ob.issue_range(ldsB, wave_u, 3, src_kt(3), 0, MX);
  wait_vm<PA * nK + (8 + MX) * nM>();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // Software pipeline.  A k-tile is 8 x 8 MFMA 16x16x32 per wavefront (the 16-row shape runs at
  // a higher sustained clock than 32x32x16 at the same flops per cycle), in two halves of 32:
  // rows 0..63 of the sub-tile (A fragments 0..3), then rows 64..127 (fragments 4..7), each
  // against the 8 B fragments of the k-tile.  A "step" is two MFMAs.  1st half of kt: the reads
  // of A fragments 4..7 of kt behind its first four steps; barrier; 2nd half: the reads of the 8
  // B fragments (into the other of two sets) and of A fragments 0..3 of k-tile kt+1 behind its
  // first twelve.  A step carries at most one fragment read and one DMA instruction, dealt out
  // over its two MFMAs in exactly the order written below (every position is fenced), so each
  // of them has an MFMA in flight as cover.
  typename Operand<KCA>::Frag fal[4], fah[4];     // A low / high rows
  typename Operand<KCB>::Frag fbe[8], fbo[8];     // B of the even / odd k-tile
#pragma unroll
  for (int i = 0; i < 4; ++i) oa.fragment(fal[i], regA, i);
#pragma unroll
  for (int j = 0; j < 8; ++j) ob.fragment(fbe[j], regB, j);

  // The sources of the next two k-tiles' requests, one scalar instruction at a time (x + 1
  // modulo N as min(x + 1, x + 1 - N) in unsigned arithmetic); they replace cp, cn, cm0, cm1
  // when the two k-tiles are done
  unsigned nx0 = 0, nx1 = 0, ncn = 0, ncm0 = 0, ncm1 = 0;
  constexpr int N_SCALAR = 9;
  auto scalar_op = [&](auto op_c) {
    constexpr int op = decltype(op_c)::value;
    if constexpr (op == 0) nx0 = (unsigned)cn + 1u;
    else if constexpr (op == 1) nx1 = nx0 - (unsigned)NP;
    else if constexpr (op == 2) ncn = nx0 < nx1 ? nx0 : nx1;
    else if constexpr (op == 3) nx0 = (unsigned)cm1 + 1u;
    else if constexpr (op == 4) nx1 = nx0 - (unsigned)KT;
    else if constexpr (op == 5) ncm0 = nx0 < nx1 ? nx0 : nx1;
    else if constexpr (op == 6) nx0 = ncm0 + 1u;
    else if constexpr (op == 7) nx1 = nx0 - (unsigned)KT;
    else if constexpr (op == 8) ncm1 = nx0 < nx1 ? nx0 : nx1;
  };
  auto half = [&](auto ph_c) {
    constexpr int PH8 = decltype(ph_c)::value, PH = PH8 & 3, KT0 = (PH8 >> 2) * 2 + (PH >> 1);   // k-tile mod 4
    constexpr bool SECOND = PH & 1, ODD = (PH >> 1) & 1;
    constexpr int OA = KCA ? 1 : 2, OB = KCB ? 1 : 2;     // LDS instructions per fragment
    constexpr int D = (PH == 3 ? PA : PH == 0 ? PB : PH == 1 ? PC : 0) * nK + ((PH & 1) ? MX : 4 - MX) * nM;
    constexpr int R = SECOND ? 8 * OB + 4 * OA : 4 * OA;
    constexpr int G0 = SECOND ? 0 : 2;   // (1st half: not behind the first MFMAs, or the wait for the previous half's reads takes them along)
    static_assert(2 * D + R <= 64 - 2 * G0, "two instructions per MFMA at most");
    constexpr int S = PH == 1 ? N_SCALAR : 0;   // the 2nd half of the even k-tile requests nothing: room for the bookkeeping
    static_assert(half_plan_ok<D, R, G0, S>(kHalfPlan<D, R, G0, S>), "instruction plan of the half");
    // LDS instruction number OP of the half: 2nd half: the 8 B fragments, then A fragments 0..3, of
    // the next k-tile (past the last k-tile this reads a slot nobody filled: in range, never
    // used); 1st half: A fragments 4..7 of this k-tile
    auto read_op = [&](auto op_c) {
      constexpr int op = decltype(op_c)::value;
      if constexpr (SECOND) {
        if constexpr (op < 8 * OB) {
          constexpr int f = op / OB, part = op % OB;
          if (ODD) ob.template fragment_part<part, (KT0 + 1) & 3>(fbe[f], regB, f);
          else     ob.template fragment_part<part, (KT0 + 1) & 3>(fbo[f], regB, f);
        } else {
          constexpr int f = (op - 8 * OB) / OA, part = (op - 8 * OB) % OA;
          oa.template fragment_part<part, (KT0 + 1) & 3>(fal[f], regA, f);
        }
      } else {
        constexpr int f = op / OA, part = op % OA;
        oa.template fragment_part<part, KT0>(fah[f], regA, 4 + f);
      }
    };
    static_for<32>([&](auto g_c) {
      constexpr int g = decltype(g_c)::value, i = g >> 3, j = g & 7;
      const bf16x8_t fb = ODD ? fbo[j].get() : fbe[j].get();
      // (inline, with the accumulator tied to the accumulation registers: left to itself the
      // compiler moves hundreds of accumulators between register files in every round of the loop)
      if (SECOND) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[4 + i][j]) : "v"(fah[i].get()), "v"(fb));
      else        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fal[i].get()), "v"(fb));
      __builtin_amdgcn_sched_barrier(0);
      static_for<2>([&](auto s_c) {
        constexpr int sl = decltype(s_c)::value;
        constexpr int kind = kHalfPlan<D, R, G0, S>.kind[g][sl], idx = kHalfPlan<D, R, G0, S>.idx[g][sl];
        if constexpr (kind == OP_READ) read_op(std::integral_constant<int, idx>{});
        else if constexpr (kind == OP_DEST) dma_op(ph_c, std::integral_constant<int, 0>{}, std::integral_constant<int, idx>{});
        else if constexpr (kind == OP_LOAD) dma_op(ph_c, std::integral_constant<int, 1>{}, std::integral_constant<int, idx>{});
        else if constexpr (kind == OP_DMA)  dma_op(ph_c, std::integral_constant<int, 2>{}, std::integral_constant<int, idx>{});
      });
      if constexpr (kHalfPlan<D, R, G0, S>.scalar[g] >= 0) scalar_op(std::integral_constant<int, kHalfPlan<D, R, G0, S>.scalar[g]>{});
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  auto barrier = [&](auto w_c) {
    wait_vm<decltype(w_c)::value>();                     // k-tile kt+1 of this wavefront's loads
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // own reads of k-tile kt are back
    __builtin_amdgcn_s_barrier();        // k-tile kt+1 complete for everyone; k-tile kt released
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
  };
  // two k-tiles, the first of them number 2 Q modulo 4
  auto two_ktiles = [&](auto q_c) {
    constexpr int Q = decltype(q_c)::value;
    half(std::integral_constant<int, 4 * Q + 0>{});
    barrier(std::integral_constant<int, W_EVEN>{});
    half(std::integral_constant<int, 4 * Q + 1>{});
    half(std::integral_constant<int, 4 * Q + 2>{});
    barrier(std::integral_constant<int, W_ODD>{});
    half(std::integral_constant<int, 4 * Q + 3>{});
    cp = cn;
    cn = (int)ncn;
    cm0 = (int)ncm0;
    cm1 = (int)ncm1;
  };
  // four k-tiles per round of the loop, so that every LDS slot is a compile-time constant (KT is even)
  for (int kt = 0; kt + 4 <= KT; kt += 4) {
    two_ktiles(std::integral_constant<int, 0>{});
    two_ktiles(std::integral_constant<int, 1>{});
  }
  if (KT & 2) two_ktiles(std::integral_constant<int, 0>{});
  // (the wait states between the last MFMA and the first read of its result: the compiler does
  // not see the instruction inside the assembly statement)
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();            // nobody's clamped reloads still land in LDS

  // ---- epilogue -------------------------------------------------------------------------------
  const int R0 = tile_r0 + wr * 128, C0 = tile_c0 + wc * 128;   // origin of this wavefront's sub-tile
  // Test faults (none in production calls: then this is one scalar compare).
  if (khalf <= 0) {     // (of a split tile: planted into the first half)
    for (int f = 0; f < a.n_faults; ++f) {
      const gecc_fault ft = a.faults[f];
      if (ft.batch != b + a.fault_bias || ft.row < R0 || ft.row >= R0 + 128 || ft.col < C0 || ft.col >= C0 + 128) continue;
      const int dr = ft.row - R0, dc = ft.col - C0;
      const int fi = dr >> 4, fv = dr & 3, fj = dc >> 4;
      const bool mine = (((dr >> 2) & 3) == lg) && ((dc & 15) == l16);
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (mine && i == fi && j == fj && v == fv) acc[i][j][v] += ft.offset;
    }
  }

  // One pass over the accumulators, no branches.  C goes straight to memory through a raw
  // buffer whose base is the sub-tile origin and whose size ends with the last valid row: rows
  // beyond n fail the hardware range check and are dropped, and a lane whose column is beyond m
  // carries an offset that is out of range by itself.  An accumulator register holds 4 rows x
  // 16 columns (64-byte pieces, which the memory system takes a third slower than whole
  // lines), so the registers of two neighbouring column blocks first trade their odd / even
  // groups of 16 lanes (v_permlane16_swap): each then holds 2 rows x 32 consecutive columns, two
  // full lines per store.  (Stores are marked non-temporal: C is written once and is larger
  // than the memory-side cache, which is better spent on the operands the parity kernels read
  // again.)
  // The accumulators of such rows and columns are exact zeros (their
  // operand rows were read as zeros), so the sums below need no predicates.
  // Column sums build up in 16 registers with the lane-independent part of the row weight (the
  // lane part, 4 g, is added at the end); of every row the lane keeps the sum of its 8
  // columns (one per 16-wide block) and u = x1 + 2 x2 + .. + 7 x7, the block part of the column
  // weight -- both go through LDS, where the 16 lanes of a group are added and the lane part of
  // the weight is applied.
  // (SP: this workgroup has one half of k of a split tile; its partner has the other.  Both add
  // into zeroed memory instead of storing: two terms, so the result does not depend on who is
  // first.)
  {
    const int tm128 = R0 >> 7, tn128 = C0 >> 7;
    const int R0u = tile_r0 + (wave_u >> 1) * 128, C0u = tile_c0 + (wave_u & 1) * 128;   // scalar copies
    const int rows_left = min(a.n - R0u, 128), cols_left = a.m - C0u;
    const __amdgpu_buffer_rsrc_t crsrc = __builtin_amdgcn_make_buffer_rsrc(
        C + (int64_t)R0u * a.ldc + C0u, 0, rows_left > 0 && cols_left > 0 ? rows_left * a.ldc * 4 : 0, 0x00020000);
    auto put = [&](float x, int off) {
      if (SP) __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(x, crsrc, off, 0, 0);
      else __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, x), crsrc, off, 0, 2);
    };
    // after the swap lane (l16, g) of the first register of a pair has row 8 (g >> 1), column
    // 16 (g & 1) + l16 of the 32-wide block (the second register: 4 rows further down)
    int vo[4];   // byte offset of this lane in the sub-tile, per 32-wide block
#pragma unroll
    for (int jp = 0; jp < 4; ++jp) {
      const int col = jp * 32 + (lg & 1) * 16 + l16;
      vo[jp] = col < cols_left ? ((lg >> 1) * 8 * a.ldc + col) * 4 : (int)OOB;
    }
    float cs[8], cw[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) cs[j] = cw[j] = 0.f;
    float2* red2 = reinterpret_cast<float2*>(smem) + wave_u * (128 * 17) + (lg * 4) * 17 + l16;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int ru = i * 16 + v;                        // row inside the sub-tile, without 4 g
        const int rowoff = ru * a.ldc * 4;                // scalar; < 2^31 (ldc < 2^22, checked by the launcher)
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = acc[i][j][v];
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) {
          // (inline: this compiler's builtin for the swap loses its second result; the wait
          // states are the ones a swap needs after a vector instruction wrote its operands)
          float t0 = x[2 * jp], t1 = x[2 * jp + 1];
          asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(t0), "+v"(t1));
          put(t0, vo[jp] + rowoff);
          put(t1, vo[jp] + rowoff + 4 * a.ldc * 4);
        }
        if (EPI) {
          // s = x0 + .. + x7 and u = x1 + 2 x2 + .. + 7 x7 from suffix sums: u = t1 + t2 + .. + t7
          const float t7 = x[7], t6 = x[6] + t7, t5 = x[5] + t6, t4 = x[4] + t5;
          const float t3 = x[3] + t4, t2 = x[2] + t3, t1 = x[1] + t2;
          red2[ru * 17] = make_float2(x[0] + t1, ((t1 + t2) + (t3 + t4)) + ((t5 + t6) + t7));
          const float wr_ = (float)(ru + 1);
#pragma unroll
          for (int j = 0; j < 8; ++j) { cs[j] += x[j]; cw[j] = fmaf(x[j], wr_, cw[j]); }
        }
      }
    }
    if (EPI) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float w1 = fmaf((float)(lg * 4), cs[j], cw[j]);
        float s = cs[j] + __shfl_xor(cs[j], 16, 64), w = w1 + __shfl_xor(w1, 16, 64);
        s += __shfl_xor(s, 32, 64);
        w += __shfl_xor(w, 32, 64);
        const int col = C0 + j * 16 + l16;
        if (lg == 0 && col < a.m && R0 < a.n) {
          float* cp = a.colpart + (((int64_t)b * a.ntm + tm128) * a.cp_ld + col) * 2;
          if (SP) { atomicAdd(cp, s); atomicAdd(cp + 1, w); }
          else *reinterpret_cast<float2*>(cp) = make_float2(s, w);
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the region is this wavefront's own
      const float2* mine = reinterpret_cast<const float2*>(smem) + wave_u * (128 * 17);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int r = lane + 64 * h;
        float s = 0.f, w = 0.f, u = 0.f;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          const float2 t = mine[r * 17 + c];
          s += t.x;
          w = fmaf((float)(c + 1), t.x, w);
          u += t.y;
        }
        const int row = R0 + r;
        if (row < a.n && C0 < a.m) {
          float* rp = a.rowpart + (((int64_t)b * a.ntn + tn128) * a.rp_ld + row) * 2;
          if (SP) { atomicAdd(rp, s); atomicAdd(rp + 1, fmaf(16.f, u, w)); }
          else *reinterpret_cast<float2*>(rp) = make_float2(s, fmaf(16.f, u, w));
        }
      }
    if (!SP && blockIdx.x == 0 && a.pg_out) form_pg(a, b, reinterpret_cast<double*>(smem));   // P_g, once per batch item
    }
  }
}

constexpr int MAX_DEVICES = 64;
// compute units of a device, asked once per device
int device_cus(int dev) {
  static std::mutex mu;
  static int cus_of[MAX_DEVICES] = {};
  std::lock_guard<std::mutex> lock(mu);
  if (cus_of[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    cus_of[dev] = cus;
  }
  return cus_of[dev];
}

template <bool KCA, bool KCB, bool EPI>
hipError_t launch_one(const GemmArgs& a0, hipStream_t st) {
  constexpr int lds_bytes = EPI && EPI_SMEM_BYTES > SMEM_BYTES ? EPI_SMEM_BYTES : SMEM_BYTES;
  auto kern = gemm_bf16_256<KCA, KCB, EPI, false>;
  auto kern_split = gemm_bf16_256<KCA, KCB, EPI, true>;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  {
    // the LDS limit of the two kernels of this instantiation and the CU count, once per device,
    // whichever host thread comes first
    static std::mutex mu;
    static bool configured[MAX_DEVICES] = {};
    std::lock_guard<std::mutex> lock(mu);
    if (!configured[dev]) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
      if (e != hipSuccess) return e;
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern_split),
                              hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
      if (e != hipSuccess) return e;
      configured[dev] = true;
    }
  }
  GemmArgs a = a0;
  const int ntm = (a.n + BM - 1) / BM, ntn = (a.m + BN - 1) / BN, ntiles = ntm * ntn;
  // Tiles run in rounds of one per compute unit.  When the last round is at most half full, its
  // tiles go to a launch of their own in which two workgroups share a tile, one per half of k,
  // so that the round takes half as long (cfg4-wgrad: 896 tiles on 256 CUs -> the time of 3.5
  // rounds instead of 4).  The halves add into C and the partial sums, zeroed beforehand.
  const int cus = a.cu_hint > 0 ? a.cu_hint : device_cus(dev);
  // rounds as blocks of tiles (see tile_of): 16 x 16 or 32 x 8, whichever fits
  // exactly -- where the panels a round of the default order touches (64 tile rows + 4 tile
  // columns) would not fit the 256 MiB memory-side cache; where they do, the default order is as
  // fast or a little faster
  a.map_sr = a.map_sc = 0;
  const int64_t default_round_bytes = (int64_t)((ntm < 64 ? ntm : 64) + 4) * BM * a.k * 2;
  if (cus == 256 && a.batch == 1 && default_round_bytes > ((int64_t)192 << 20)) {
    if (ntm % 16 == 0 && ntn % 16 == 0) { a.map_sr = 16; a.map_sc = 16; }
    else if (ntm % 32 == 0 && ntn % 8 == 0) { a.map_sr = 32; a.map_sc = 8; }
  }
  const int tail = ntiles % cus;
  a.split_first = -1;
  if (a.batch == 1 && ntiles > cus && tail > 0 && 2 * tail <= cus && a.k % (4 * BK) == 0) {
    a.split_first = ntiles - tail;      // (tail <= ntiles - tail: every tail tile has a workgroup to zero it)
    hipLaunchKernelGGL(kern, dim3(ntiles - tail, 1), dim3(THREADS), lds_bytes, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern_split, dim3(2 * tail, 1), dim3(THREADS), lds_bytes, st, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(kern, dim3(ntiles, a.batch), dim3(THREADS), lds_bytes, st, a);
  return hipGetLastError();
}

template <bool EPI>
hipError_t launch_layout(const GemmArgs& a, hipStream_t st) {
  const bool kca = a.trans_a == 0, kcb = a.trans_b != 0;
  if (kca && kcb) return launch_one<true, true, EPI>(a, st);
  if (kca && !kcb) return launch_one<true, false, EPI>(a, st);
  if (!kca && kcb) return launch_one<false, true, EPI>(a, st);
  return launch_one<false, false, EPI>(a, st);
}

}  // namespace

// The fast kernel needs 16-byte aligned operand rows, whole 16-byte chunks and whole pairs of
// k-tiles: k % 64 == 0, leading dimensions % 8 == 0, n (m) % 8 == 0 for an operand stored with n (m)
// contiguous, and operand panels that 32-bit byte offsets can address.  Partial sums are
// produced per 128 x 128 sub-tile.  Everything else goes to the generic 128 x 128 kernel.
bool gemm_bf16_fast_ok(const GemmArgs& a) {
  if (a.dtype != GECC_BF16 || a.tile_m != 128 || a.tile_n != 128) return false;
  if (a.k % (2 * BK) || a.lda % 8 || a.ldb % 8) return false;
  if (reinterpret_cast<uintptr_t>(a.A) % 16 || reinterpret_cast<uintptr_t>(a.B) % 16) return false;
  if (a.batch > 1 && (a.sa % 8 || a.sb % 8)) return false;
  if (a.trans_a && a.n % 8) return false;
  if (!a.trans_b && a.m % 8) return false;
  // byte offsets inside a tile panel (k-contiguous: 256 rows; otherwise the whole k extent)
  const int64_t span_a = (a.trans_a ? (int64_t)a.k : (int64_t)BM) * a.lda * 2;
  const int64_t span_b = (a.trans_b ? (int64_t)BN : (int64_t)a.k) * a.ldb * 2;
  if (span_a >= 0x7fffffff || span_b >= 0x7fffffff || a.ldc >= (1 << 22)) return false;
  return (int64_t)a.n * a.m >= (int64_t)BM * BN;   // smaller problems: the 128 x 128 kernel
}

hipError_t launch_gemm_bf16_fast(const GemmArgs& a, hipStream_t st) {
  return a.rowpart ? launch_layout<true>(a, st) : launch_layout<false>(a, st);
}

}  // namespace gecc
