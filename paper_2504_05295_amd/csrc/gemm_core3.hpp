// bf16 x bf16 MFMA GEMM core for gfx950 whose operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: no staging registers, no LDS store instructions), for the products of the Dion
// step whose operands are both bf16 matrices with k contiguous:
//   the Gram matrix and the triangular multiply of Cholesky-QR (up to three split-bf16 operand pairs),
//   Z = (M+G) Q and R = (M+G)^T P from the bf16 copy of M + G that one pass writes first (R reads it with k as the
//   slow index),
//   the fused rank-r updates of M and X (A = P, B = R, B2 = Q_new).
// Conventions as in gemm_core2.hpp: C[i,j] = sum_k A(i,k) B(j,k), same GemmArgs, same epilogues.
//
// LDS tile layout.  A direct load writes the 64 lanes' 16-byte chunks to 1 KB of consecutive LDS, so rows cannot
// be padded; instead chunk kc of row r sits at chunk position kc ^ ((r >> 1) & 7) of its 128-byte row (BK = 64;
// with BK = 32 a row has 64 bytes and the position is kc ^ ((r >> 2) & 3)).
// The lane decides which global chunk it fetches, so the permutation costs nothing on the way in, and on the way
// out the 16 lanes that read one chunk column of 16 consecutive rows hit 16 different 16-byte bank groups.
//
// Pipeline: two LDS stages.  The loads of slab s+1 are issued when slab s starts; each wave waits for its own
// loads before the one barrier per slab, which sits before the last k-step's MFMAs so that these and the first
// fragment reads of the next slab cover it.  The waits on the loads are written by hand (s_waitcnt vmcnt): left
// to the compiler, every LDS read would wait for all loads in flight, since it cannot tell their LDS
// destinations apart.
#pragma once
#include <algorithm>

#include "gemm_core.hpp"

namespace dion {

// BK_: 64, or 32 for tiles small enough that two workgroups share a compute unit (MINW_ = waves per SIMD the
// register budget is cut for: 2 means two four-wave workgroups per compute unit).
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int BK_ = 64, int MINW_ = 1>
struct TileCfg3 {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, MINW = MINW_;
  static constexpr int CPR = BK_ / 8;     // 16-byte chunks per LDS row
  static constexpr int ROWB = BK_ * 2;    // bytes per LDS row
  static_assert(BK_ == 64 || BK_ == 32, "slab depth");
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, NW = WAVES_M_ * WAVES_N_;
  static constexpr int NT = 64 * NW;
  static constexpr int WTM = BM_ / WAVES_M_, WTN = BN_ / WAVES_N_;
  static constexpr int MI = WTM / 32, NI = WTN / 32;
  static constexpr int A_BYTES = BM_ * BK * 2, B_BYTES = BN_ * BK * 2;
  static constexpr int A_LOADS = A_BYTES / 1024 / NW, B_LOADS = B_BYTES / 1024 / NW;   // 1 KB loads per wave and slab
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
  static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile does not divide over the waves");
};

// 64 lanes x 16 bytes: global (one address per lane) -> LDS [lds_addr, lds_addr + 1024).  The instruction takes
// its LDS address from M0; lds_addr has to be in a scalar register when it gets here (the build fails otherwise).
// Nothing in the statement writes a register that code outside it reads: the compiler does not look into an asm
// statement, so it could not keep a dependent instruction the required number of wait states away.  (A
// v_readfirstlane_b32 written here right after the compiler's own v_mov_b32 into its source read the old value.)
__device__ __forceinline__ void load_to_lds_16_raw(unsigned lds_addr, const void* lane_addr) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, off"
      :
      : "s"(lds_addr), "v"(lane_addr)
      : "memory");
}
#ifdef DION_GEMM3_BOUNDS
// Checking build (the program tests/native/gemm3_check.hip only): a lane whose 16 bytes do not lie inside
// [lo, hi) is counted and loads nothing.
__device__ unsigned long long dion_gemm3_bounds[2];
__device__ unsigned int dion_gemm3_violations;
__device__ unsigned long long dion_gemm3_first[64];
__device__ __forceinline__ void load_to_lds_16(unsigned lds_addr, const void* lane_addr) {
  const unsigned long long a = (unsigned long long)lane_addr;
  const bool ok = a >= dion_gemm3_bounds[0] && a + 16 <= dion_gemm3_bounds[1] && lds_addr + 1024 <= 160 * 1024;
  if (!ok) {
    const unsigned n = atomicAdd(&dion_gemm3_violations, 1u);
    if (n < 16) {
      dion_gemm3_first[4 * n + 0] = a;
      dion_gemm3_first[4 * n + 1] = 0;
      dion_gemm3_first[4 * n + 2] = lds_addr;
      dion_gemm3_first[4 * n + 3] = blockIdx.x * 1024ull + threadIdx.x;
    }
  }
  if (ok) load_to_lds_16_raw(lds_addr, lane_addr);
}
#else
__device__ __forceinline__ void load_to_lds_16(unsigned lds_addr, const void* lane_addr) { load_to_lds_16_raw(lds_addr, lane_addr); }
#endif
__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int CPR>
__device__ __forceinline__ int lds_swizzle(int row) {
  return CPR == 8 ? (row >> 1) & 7 : (row >> 2) & 3;
}

// Tile (row, column) of the `tile`-th tile in the order in which a launch visits them.
template <int BM, int BN>
__device__ __forceinline__ void gemm3_tile_coords(const GemmArgs& g, int tile, int& tm, int& tn) {
  tn = tile % g.tiles_n;
  tm = tile / g.tiles_n;
  if (g.tri_grid) {
    tm = (int)((__builtin_sqrtf(8.f * (float)tile + 1.f) - 1.f) * 0.5f);
    while (tm * (tm + 1) / 2 > tile) --tm;
    while ((tm + 1) * (tm + 2) / 2 <= tile) ++tm;
    tn = tile - tm * (tm + 1) / 2;
  } else if (g.heavy_first) {
    const int rows_per_xcd = g.tiles_m >> 3, per = rows_per_xcd * g.tiles_n;   // bid = xcd * per + position in the XCD
    const int xcd = tile / per, pos = tile - xcd * per;
    tm = xcd * rows_per_xcd + pos % rows_per_xcd;
    tn = g.tiles_n - 1 - pos / rows_per_xcd;
  } else if (g.group_n > 0) {
    const int gw = g.group_n * g.tiles_m;
    const int cg = tile / gw;
    const int first = cg * g.group_n;
    const int width = min(g.group_n, g.tiles_n - first);
    const int rem = tile - cg * gw;
    tm = rem / width;
    tn = first + rem % width;
  }
}

// Transposing LDS read of gfx950 (ds_read_b64_tr_b16).  Within every group of 16 lanes, with chunk[j] the four 16-bit
// elements at lane j's address and M[r][c] = chunk[4 r + c / 4][c % 4] (4 x 16), lane i of the group receives
// (M[0][i], M[1][i], M[2][i], M[3][i]).  With lane 4 r + q pointing at elements 4 q .. 4 q + 3 of row k0 + r of a
// [k][row] tile, lane i ends up with k0 .. k0 + 3 of matrix row i: four consecutive k of one row, which is what the
// matrix instruction wants, from an operand that is stored with k as the slow index.
typedef short v4s_t __attribute__((ext_vector_type(4)));
typedef short v8s_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4s_t lds_v4s_t;
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
__device__ __forceinline__ bf16x8_t lds_read_tr_pair(const lds_byte_t* p0, const lds_byte_t* p1) {
  const v4s_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_t*)p0);
  const v4s_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_t*)p1);
  return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ __forceinline__ void gemm3_store_split(uint16_t* hi, uint16_t* lo, long long idx, const f32x4_t v);

// Scheduling hint "one MFMA, then its share of READS LDS reads", MMAS times (the counts must be compile-time constants)
template <int Q, int MMAS, int READS>
__device__ __forceinline__ void gemm3_sched_pairs() {
  if constexpr (Q < MMAS) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, READS / MMAS + (Q < READS % MMAS ? 1 : 0), 0);
    gemm3_sched_pairs<Q + 1, MMAS, READS>();
  }
}

// AKS / BKS: that operand is stored with k as the slow index, element (row, k) at p[k * ld + row] (a row-major matrix
// used as the left operand of X^T Y, say).  Its slab is then BK rows of the tile's BM (BN) elements; chunk c of k-row kr
// sits at chunk position c ^ (4 (kr & 3)) of its row, and fragments come out through the transposing LDS read: the 32
// lanes of a half-wave then touch 16 different 16-byte bank groups, two lanes each on their own halves.
template <class Cfg, bool GBF16, int EPI, bool DUAL, bool AKS = false, bool BKS = false>
__global__ void __launch_bounds__(Cfg::NT, Cfg::MINW) gemm3_kernel(const GemmArgs g) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, NW = Cfg::NW, CPR = Cfg::CPR, ROWB = Cfg::ROWB;
  static_assert(!(AKS || BKS) || (BK == 64 && !DUAL), "k-slow operands: 64-deep slabs, single product");
  static_assert(!AKS || BM % 128 == 0, "k-slow A: tile rows");
  static_assert(!BKS || BN % 128 == 0, "k-slow B: tile columns");
  constexpr int MI = Cfg::MI, NI = Cfg::NI, KSTEPS = BK / 16;
  constexpr int A_BYTES = Cfg::A_BYTES, B_BYTES = Cfg::B_BYTES;
  constexpr int STAGE_BYTES = A_BYTES + B_BYTES * (DUAL ? 2 : 1);
  constexpr int SP = 36;   // epilogue patch row stride in floats
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  int bid = blockIdx.x;
  if (g.xcd_remap) {
    // (with a split last round the remapping covers the full rounds only: the tail keeps its place at the end)
    const int main_blocks = g.tail_split > 1 ? g.tail_first : (int)gridDim.x;
    if (bid < main_blocks) {
      const int per = main_blocks >> 3;
      bid = (bid & 7) * per + (bid >> 3);
    }
  }
  // tri_grid: the grid holds the tiles on and below the diagonal only (tile t -> row tm, column tn <= tm), so that
  // no workgroup is launched just to return and the live ones spread evenly over the XCDs
  const int ntile = g.tri_grid ? g.tiles_m * (g.tiles_m + 1) / 2 : g.tiles_m * g.tiles_n;
  int tile = bid % ntile;
  int rest = bid / ntile;
  int ks = rest % g.splitk;
  int b = rest / g.splitk;
  // a tile of the last, short round: tail_split workgroups share its contraction (one matrix, splitk == 1; the grid
  // then holds tail_first + tail_tiles * tail_split workgroups, more than there are tiles)
  int tail_q = -1;
  if (g.tail_split > 1 && bid >= g.tail_first) {
    tail_q = bid - g.tail_first;
    tile = g.tail_first + tail_q / g.tail_split;
    ks = tail_q % g.tail_split;
    b = 0;
  }
  int tn, tm;
  gemm3_tile_coords<BM, BN>(g, tile, tm, tn);
  if (g.lower_only && tn * BN > tm * BM + BM - 1) return;

  void* const* tab = g.table + (size_t)b * g.nslots;
  if (g.status_slot >= 0 && *(const int*)tab[g.status_slot] != 0) return;

  const int row0 = tm * BM, col0 = tn * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave % Cfg::WAVES_M, wn = wave / Cfg::WAVES_M;
  const int lr = lane & 31, lk = lane >> 5;

  // byte offset, inside its matrix, of the chunk this lane fetches in each of the wave's loads of a slab
  unsigned aoff[Cfg::A_LOADS], boff[Cfg::B_LOADS];
#pragma unroll
  for (int q = 0; q < Cfg::A_LOADS; ++q) {
    const int pos = (q * NW + wave) * 64 + lane;
    if constexpr (AKS) {
      const int kr = pos / (BM / 8), c = (pos % (BM / 8)) ^ (4 * (kr & 3));
      aoff[q] = (unsigned)(((long long)kr * g.A.ld + row0 + c * 8) * 2);
    } else {
      const int row = pos / CPR, kc = (pos % CPR) ^ lds_swizzle<CPR>(row);
      aoff[q] = (unsigned)(((long long)(row0 + row) * g.A.ld + kc * 8) * 2);
    }
  }
#pragma unroll
  for (int q = 0; q < Cfg::B_LOADS; ++q) {
    const int pos = (q * NW + wave) * 64 + lane;
    if constexpr (BKS) {
      const int kr = pos / (BN / 8), c = (pos % (BN / 8)) ^ (4 * (kr & 3));
      boff[q] = (unsigned)(((long long)kr * g.B.ld + col0 + c * 8) * 2);
    } else {
      const int row = pos / CPR, kc = (pos % CPR) ^ lds_swizzle<CPR>(row);
      boff[q] = (unsigned)(((long long)(col0 + row) * g.B.ld + kc * 8) * 2);
    }
  }
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem);
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);

  // The contraction is a list of k-slabs: nseg operand pairs, each contributing kseg_eff / BK slabs.
  if (g.noop_slot >= 0 && __builtin_amdgcn_readfirstlane(*(const int*)tab[g.noop_slot]) != 0) return;   // uniform, before any barrier
  const int nseg = g.nseg > 0 ? g.nseg : 1;
  const int kseg = g.nseg > 0 ? g.kseg : g.K;
  const int kseg_eff = g.tri_k ? min(kseg, (tn + 1) * BN) : kseg;
  const int slabs_per_seg = kseg_eff / BK;
  const int total = nseg * slabs_per_seg;
  const int kps = tail_q >= 0 ? (total + g.tail_split - 1) / g.tail_split : g.k_per_split;
  const int s_begin = g.slab_count > 0 ? g.slab_first : ks * kps;
  const int s_end = min(total, s_begin + (g.slab_count > 0 ? g.slab_count : kps));
  // Operand base addresses of the (up to three) operand pairs, read once and kept in scalar registers: a look-up
  // in the pointer table inside the loop is a memory load, and the wait for it would also wait for every tile
  // load in flight.  (Separate variables: an array indexed by the pair number would live in scratch memory.)
  const int b_fixed = g.nseg > 0 ? -1 : g.B.slot0;
  // (a single operand pair may start at a row of its left matrix: A.off elements in, for a product over a block of rows)
  const unsigned char* const A0 = (const unsigned char*)(tab[g.nseg > 0 ? g.segA[0] : g.A.slot0]) + (g.nseg > 0 ? 0 : g.A.off * 2);
  const unsigned char* const A1 = nseg > 1 ? (const unsigned char*)(tab[g.segA[1]]) : A0;
  const unsigned char* const A2 = nseg > 2 ? (const unsigned char*)(tab[g.segA[2]]) : A0;
  const unsigned char* const B0 = (const unsigned char*)(tab[b_fixed >= 0 ? b_fixed : g.segB[0]]);
  const unsigned char* const B1 = nseg > 1 ? (const unsigned char*)(tab[g.segB[1]]) : B0;
  const unsigned char* const B2 = nseg > 2 ? (const unsigned char*)(tab[g.segB[2]]) : B0;
  // running addresses of the next slab to be loaded, advanced by one slab per load
  int ld_seg = slabs_per_seg > 0 ? s_begin / slabs_per_seg : 0;
  int ld_k0 = (s_begin - ld_seg * slabs_per_seg) * BK;
  // bytes from one k to the next in either operand
  const size_t a_kstep = AKS ? (size_t)g.A.ld * 2 : 2, b_kstep = BKS ? (size_t)g.B.ld * 2 : 2;
  const unsigned char* a_run = (ld_seg <= 0 ? A0 : ld_seg == 1 ? A1 : A2) + (size_t)ld_k0 * a_kstep;
  const unsigned char* b_run = (ld_seg <= 0 ? B0 : ld_seg == 1 ? B1 : B2) + (size_t)ld_k0 * b_kstep;
  const unsigned char* b2_run = DUAL ? (const unsigned char*)(tab[g.B2.slot0]) + (size_t)ld_k0 * 2 : nullptr;

  auto issue = [&](int stage, const unsigned char* Ap, const unsigned char* Bp, const unsigned char* B2k) __attribute__((always_inline)) {
    const unsigned la = lds0 + stage * STAGE_BYTES + wave_s * 1024;
#pragma unroll
    for (int q = 0; q < Cfg::A_LOADS; ++q) load_to_lds_16(la + q * NW * 1024, Ap + aoff[q]);
#pragma unroll
    for (int q = 0; q < Cfg::B_LOADS; ++q) load_to_lds_16(la + A_BYTES + q * NW * 1024, Bp + boff[q]);
    if constexpr (DUAL) {
#pragma unroll
      for (int q = 0; q < Cfg::B_LOADS; ++q) load_to_lds_16(la + A_BYTES + B_BYTES + q * NW * 1024, B2k + boff[q]);
    }
  };

  f32x16_t acc[MI][NI];
  f32x16_t acc2[DUAL ? MI : 1][DUAL ? NI : 1];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
      if constexpr (DUAL) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc2[i][j][v] = 0.f;
      }
    }

  // fragment of k-step kk: row r, chunk 2 kk + lk, at r * ROWB + ((2 kk + lk) ^ swizzle(r)) * 16; the rows
  // i * 32 + lr of one lane all have the swizzle of lr
  const int sw = lds_swizzle<CPR>(lr);
  const int a_row_off = (wm * Cfg::WTM + lr) * ROWB, b_row_off = A_BYTES + (wn * Cfg::WTN + lr) * ROWB;
  bf16x8_t af[2][MI], bf[2][NI], bf2[2][DUAL ? NI : 1];
  // k-slow operands: lane 4 r + q of a group of 16 lanes reads elements 4 q .. 4 q + 3 of the group's 16 tile rows
  // at k-row 8 lk + r (+ 16 kk, + 4 for the second half of the fragment)
  const int tr_r = (lane >> 2) & 3, tr_q = lane & 3, tr_g = (lane >> 4) & 1;
  const lds_byte_t* const smem_lds = (const lds_byte_t*)smem;
  auto ks_off = [&](int tile_row0, int row_bytes) __attribute__((always_inline)) {   // tile_row0: multiple of 32
    const int chunk = (((tile_row0 + 16 * tr_g) >> 3) + (tr_q >> 1)) ^ (4 * tr_r);
    return (8 * lk + tr_r) * row_bytes + chunk * 16 + (tr_q & 1) * 8;
  };
  auto fetch = [&](int stage, int set, int kk) __attribute__((always_inline)) {
    const unsigned char* sa = smem + stage * STAGE_BYTES + a_row_off;
    const unsigned char* sb = smem + stage * STAGE_BYTES + b_row_off;
    const int co = ((kk * 2 + lk) ^ sw) * 16;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      if constexpr (AKS) {
        const lds_byte_t* p = smem_lds + stage * STAGE_BYTES + kk * 16 * (BM * 2) + ks_off(wm * Cfg::WTM + i * 32, BM * 2);
        af[set][i] = lds_read_tr_pair(p, p + 4 * (BM * 2));
      } else {
        af[set][i] = *(const bf16x8_t*)(sa + i * 32 * ROWB + co);
      }
    }
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      if constexpr (BKS) {
        const lds_byte_t* p = smem_lds + stage * STAGE_BYTES + A_BYTES + kk * 16 * (BN * 2) + ks_off(wn * Cfg::WTN + j * 32, BN * 2);
        bf[set][j] = lds_read_tr_pair(p, p + 4 * (BN * 2));
      } else {
        bf[set][j] = *(const bf16x8_t*)(sb + j * 32 * ROWB + co);
      }
      if constexpr (DUAL) bf2[set][j] = *(const bf16x8_t*)(sb + B_BYTES + j * 32 * ROWB + co);
    }
  };
  auto mma = [&](int set) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bf[set][j], acc[i][j], 0, 0, 0);
        if constexpr (DUAL) acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bf2[set][j], acc2[i][j], 0, 0, 0);
      }
  };
  // schedule of one k-step: MFMA, LDS read, MFMA, LDS read, ... so that the fragments of the next k-step trickle
  // in behind the MFMAs of this one
  auto interleave = [&]() __attribute__((always_inline)) {
    constexpr int READS = MI * (AKS ? 2 : 1) + NI * (BKS ? 2 : 1) * (DUAL ? 2 : 1), MMAS = MI * NI * (DUAL ? 2 : 1);
    if constexpr (MMAS >= READS) {
#pragma unroll
      for (int q = 0; q < READS; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      if constexpr (MMAS > READS) __builtin_amdgcn_sched_group_barrier(0x008, MMAS - READS, 0);
    } else {
      // more reads than MFMAs (k-slow operands take two reads per fragment): the surplus goes to the first MFMAs
      gemm3_sched_pairs<0, MMAS, READS>();
    }
  };

  // loads of the next slab into the given stage; then the running addresses move on
#define DION_GEMM3_ISSUE(stage)                                                                        \
  do {                                                                                                 \
    issue((stage), a_run, b_run, b2_run);                                                              \
    a_run += BK * a_kstep;                                                                             \
    b_run += BK * b_kstep;                                                                             \
    if constexpr (DUAL) b2_run += BK * 2;                                                              \
    ld_k0 += BK;                                                                                       \
    if (ld_k0 == kseg_eff && ld_seg + 1 < nseg) {                                                      \
      ld_k0 = 0;                                                                                       \
      ++ld_seg;                                                                                        \
      a_run = ld_seg == 1 ? A1 : A2;                                                                   \
      b_run = ld_seg == 1 ? B1 : B2;                                                                   \
    }                                                                                                  \
  } while (0)
  if (s_begin < s_end) {
    DION_GEMM3_ISSUE(0);
    wait_all_loads();
  }
  __syncthreads();
  if (s_begin < s_end) {
    fetch(0, 0, 0);
    int cur = 0;
    for (int sl = s_begin; sl < s_end; ++sl) {
      if (sl + 1 < s_end) DION_GEMM3_ISSUE(cur ^ 1);
#pragma unroll
      for (int kk = 0; kk + 1 < KSTEPS; ++kk) {
        fetch(cur, (kk + 1) & 1, kk + 1);
        mma(kk & 1);
        interleave();
      }
      wait_all_loads();        // this wave's part of the next slab has landed
      __syncthreads();         // ... everybody's has, and everybody has read the last fragments of this slab
      fetch(cur ^ 1, KSTEPS & 1, 0);   // (after the last slab this reads stale data that nobody uses)
      mma((KSTEPS - 1) & 1);
      interleave();
      cur ^= 1;
    }
  }
#undef DION_GEMM3_ISSUE
  __syncthreads();   // the operand tiles are dead from here on: the epilogue reuses their LDS

  // ---- epilogue (as in gemm_core2.hpp): each 32x32 accumulator tile goes through a wave-private LDS patch so
  // that a lane ends up with four consecutive columns of one row.
  float* patch = (float*)smem + wave * 32 * SP;
  const int prow = lane >> 3, pcol = (lane & 7) * 4;
  auto to_patch = [&](const f32x16_t& t) {
#pragma unroll
    for (int v = 0; v < 16; ++v) patch[(8 * (v / 4) + 4 * lk + (v % 4)) * SP + lr] = t[v];
  };
  if constexpr (EPI == EPI_STORE) {
    float* C = (float*)tab[g.E.slot] + g.E.off + (long long)ks * g.E.split_stride;
    long long c_ld = g.E.ld;
    int c_row0 = row0, c_col0 = col0;
    if (tail_q >= 0) {   // a partial tile of the last round: to the buffer of partial tiles, a BM x BN block of its own
      C = (float*)tab[g.tail_slot] + (long long)tail_q * (BM * BN);
      c_ld = BN;
      c_row0 = 0;
      c_col0 = 0;
    }
    uint16_t* const split_hi = (g.E.split_hi1 > 0 && tail_q < 0) ? (uint16_t*)tab[g.E.split_hi1 - 1] + g.E.off : nullptr;
    uint16_t* const split_lo = (g.E.split_hi1 > 0 && tail_q < 0) ? (uint16_t*)tab[g.E.split_lo1 - 1] + g.E.off : nullptr;
    float colsq[NI];   // sums of squares of this wave's WTM rows, per column (lane & 31) of each column block
#pragma unroll
    for (int j = 0; j < NI; ++j) colsq[j] = 0.f;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
#pragma unroll
        for (int v = 0; v < 16; ++v) colsq[j] += acc[i][j][v] * acc[i][j][v];
        to_patch(acc[i][j]);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int row = c_row0 + wm * Cfg::WTM + i * 32 + prow + 8 * p;
          const int col = c_col0 + wn * Cfg::WTN + j * 32 + pcol;
          f32x4_t v4 = *(const f32x4_t*)(patch + (prow + 8 * p) * SP + pcol);
          if (g.E.beta != 0.f) v4 += gload<f32x4_t>(C + (long long)row * c_ld + col);   // a later part of a contraction spread over launches
          gstore<f32x4_t>(C + (long long)row * c_ld + col, v4);
          if (split_hi) gemm3_store_split(split_hi, split_lo, (long long)row * c_ld + col, v4);
        }
      }
    // Column norms of the result (ColNorm of the update rule) without another pass over it: one partial sum of
    // squares per column and block of WTM rows, chunk (tile row, wave row) at part[chunk * N + column]; whoever
    // finishes adds the chunks up in their order.  Only for whole products (no split over k).
    if (g.E.colsq_slot >= 0 && tail_q < 0) {
      float* part = (float*)tab[g.E.colsq_slot] + (long long)(tm * Cfg::WAVES_M + wm) * g.N + col0 + wn * Cfg::WTN;
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const float both = colsq[j] + __shfl_xor(colsq[j], 32);   // the lane halves hold different rows
        if (lk == 0) part[j * 32 + lr] = both;
      }
    }
  } else {
    // M <- (M + G) - (1-mu) (P R^T);   X <- X - eta sqrt(m/n) (P Q_new^T)
    // The old M, X and G of the next 32x32 block are requested before the current block is written, so that a
    // wave always has loads in flight: with one block at a time the pass is a chain of load latencies.
    float* Xp = (float*)tab[g.E.slotX];
    float* Mp = (float*)tab[g.E.slotM];
    const void* Gp = tab[g.E.slotG];
    struct BlockIn {
      f32x4_t mv[4], xv[4];
      u32x4_t gw[4];   // G as loaded: four fp32 values, or four bf16 values in the first two words
    };
    auto block_index = [&](int t, int p) __attribute__((always_inline)) {
      const int i = t / NI, j = t % NI;
      const int row = row0 + wm * Cfg::WTM + i * 32 + prow + 8 * p;
      const int col = col0 + wn * Cfg::WTN + j * 32 + pcol;
      return (long long)row * g.E.ld + col;
    };
    auto g_value = [&](const u32x4_t& w) __attribute__((always_inline)) {
      if constexpr (GBF16) return f32x4_t{bf16_lo(w[0]), bf16_hi(w[0]), bf16_lo(w[1]), bf16_hi(w[1])};
      else return __builtin_bit_cast(f32x4_t, w);
    };
    // (the hint is a compile-time choice: a select between a hinted and a plain load would issue both, and two copies
    // of the pass inside one kernel cost registers)
    {
      constexpr bool NTH = EPI == EPI_UPDATE_STREAM;
      auto load_block = [&](int t, BlockIn& in) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const long long idx = block_index(t, p);
          in.mv[p] = NTH ? gload_nt<f32x4_t>(Mp + idx) : gload<f32x4_t>(Mp + idx);
          if constexpr (DUAL) {
            if (g.E.x_overwrite) in.xv[p] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            else in.xv[p] = NTH ? gload_nt<f32x4_t>(Xp + idx) : gload<f32x4_t>(Xp + idx);
          }
          if constexpr (GBF16) {
            const u32x2_t w = NTH ? gload_nt<u32x2_t>((const uint16_t*)Gp + idx) : gload<u32x2_t>((const uint16_t*)Gp + idx);
            in.gw[p] = u32x4_t{w[0], w[1], 0u, 0u};
          } else {
            in.gw[p] = NTH ? gload_nt<u32x4_t>((const float*)Gp + idx) : gload<u32x4_t>((const float*)Gp + idx);
          }
        }
      };
      constexpr int NBLK = MI * NI;
      BlockIn in[2];
      load_block(0, in[0]);
#pragma unroll
      for (int t = 0; t < NBLK; ++t) {
        if (t + 1 < NBLK) load_block(t + 1, in[(t + 1) & 1]);
        const BlockIn& c = in[t & 1];
        to_patch(acc[t / NI][t % NI]);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const f32x4_t a4 = *(const f32x4_t*)(patch + (prow + 8 * p) * SP + pcol);
          const f32x4_t mn = (c.mv[p] + g_value(c.gw[p])) - g.E.c_m * a4;
          if constexpr (NTH) gstore_nt<f32x4_t>(Mp + block_index(t, p), mn);
          else gstore<f32x4_t>(Mp + block_index(t, p), mn);
        }
        if constexpr (DUAL) {
          to_patch(acc2[t / NI][t % NI]);
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const f32x4_t a4 = *(const f32x4_t*)(patch + (prow + 8 * p) * SP + pcol);
            const f32x4_t xn = c.xv[p] - g.E.c_x * a4;
            if constexpr (NTH) gstore_nt<f32x4_t>(Xp + block_index(t, p), xn);
            else gstore<f32x4_t>(Xp + block_index(t, p), xn);
          }
        }
      }
    }
  }
}

// x = hi + lo with hi = bf16(x), lo = bf16(x - hi), four consecutive elements
__device__ __forceinline__ void gemm3_store_split(uint16_t* hi, uint16_t* lo, long long idx, const f32x4_t v) {
  const uint32_t h01 = pack_bf16x2(v[0], v[1]), h23 = pack_bf16x2(v[2], v[3]);
  const uint32_t l01 = pack_bf16x2(v[0] - bf16_lo(h01), v[1] - bf16_hi(h01)), l23 = pack_bf16x2(v[2] - bf16_lo(h23), v[3] - bf16_hi(h23));
  gstore<u32x2_t>(hi + idx, u32x2_t{h01, h23});
  gstore<u32x2_t>(lo + idx, u32x2_t{l01, l23});
}

// Adds up the partial tiles of a launch's last round (GemmArgs::tail_*) into the result, in a fixed order, and forms
// the per-column sums of squares that the main kernel's epilogue forms for whole tiles.  One workgroup of 1024 threads
// per tail tile and block of WTM rows (there are few such blocks, and each has half a megabyte to read): a thread owns four consecutive columns of every RPP-th row.
template <class Cfg>
__global__ void __launch_bounds__(1024) gemm3_tail_reduce_kernel(const GemmArgs g) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, WTM = Cfg::WTM;
  constexpr int TPR = BN / 4, RPP = 1024 / TPR;   // threads per row, rows per pass
  static_assert(1024 % TPR == 0 && WTM % RPP == 0, "tile shape");
  void* const* tab = g.table;
  if (g.status_slot >= 0 && *(const int*)tab[g.status_slot] != 0) return;
  if (g.noop_slot >= 0 && *(const int*)tab[g.noop_slot] != 0) return;
  const int t = blockIdx.x, chunk = blockIdx.y;
  const int cx = threadIdx.x % TPR, ry = threadIdx.x / TPR;
  int tm, tn;
  gemm3_tile_coords<BM, BN>(g, g.tail_first + t, tm, tn);
  const float* part = (const float*)tab[g.tail_slot] + (long long)t * g.tail_split * (BM * BN) + (long long)chunk * WTM * BN + cx * 4;
  float* C = (float*)tab[g.E.slot] + g.E.off + (long long)(tm * BM + chunk * WTM) * g.E.ld + tn * BN + cx * 4;
  const long long c_first = (long long)(tm * BM + chunk * WTM) * g.E.ld + tn * BN + cx * 4;
  uint16_t* const split_hi = g.E.split_hi1 > 0 ? (uint16_t*)tab[g.E.split_hi1 - 1] + g.E.off : nullptr;
  uint16_t* const split_lo = g.E.split_hi1 > 0 ? (uint16_t*)tab[g.E.split_lo1 - 1] + g.E.off : nullptr;
  f32x4_t sq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int row = ry; row < WTM; row += RPP) {
    f32x4_t acc = gload<f32x4_t>(part + (long long)row * BN);
    for (int sp = 1; sp < g.tail_split; ++sp) acc += gload<f32x4_t>(part + (long long)sp * (BM * BN) + (long long)row * BN);
    gstore<f32x4_t>(C + (long long)row * g.E.ld, acc);
    if (split_hi) gemm3_store_split(split_hi, split_lo, c_first + (long long)row * g.E.ld, acc);
    sq += acc * acc;
  }
  if (g.E.colsq_slot >= 0) {
    __shared__ f32x4_t red[RPP][TPR];
    red[ry][cx] = sq;
    __syncthreads();
    if (ry == 0) {
      f32x4_t tot = red[0][cx];
      for (int q = 1; q < RPP; ++q) tot += red[q][cx];
      gstore<f32x4_t>((float*)tab[g.E.colsq_slot] + (long long)(tm * Cfg::WAVES_M + chunk) * g.N + tn * BN + cx * 4, tot);
    }
  }
}

// True when launch_gemm3 can take these arguments: tile-aligned shapes and operands small enough for the
// 32-bit byte offsets of the direct loads.
template <class Cfg, bool AKS = false, bool BKS = false>
inline bool gemm3_fits(const GemmArgs& g) {
  const int kseg = g.nseg > 0 ? g.kseg : g.K;
  if (g.M % Cfg::BM || g.N % Cfg::BN || kseg % Cfg::BK || kseg <= 0) return false;
  if (g.tri_k && Cfg::BN % Cfg::BK) return false;
  if (g.A.ld % 8 || g.B.ld % 8) return false;                         // 16-byte aligned chunks
  const long long lim = 1ll << 32;
  // (a lane's offset stays inside one matrix for a k-fast operand, inside one slab of BK k-rows for a k-slow one)
  const long long a_span = AKS ? ((long long)Cfg::BK * g.A.ld + g.M) * 2 : (long long)g.M * g.A.ld * 2;
  const long long b_span = BKS ? ((long long)Cfg::BK * g.B.ld + g.N) * 2 : (long long)g.N * g.B.ld * 2;
  if (AKS && g.A.ld < g.M) return false;
  if (BKS && g.B.ld < g.N) return false;
  return a_span < lim && b_span < lim;
}

template <class Cfg, bool DUAL>
constexpr int gemm3_lds_bytes() {
  constexpr int STAGE_BYTES = Cfg::A_BYTES + Cfg::B_BYTES * (DUAL ? 2 : 1);
  constexpr int PATCH_BYTES = Cfg::NW * 32 * 36 * (int)sizeof(float);
  constexpr int LDS_BYTES = 2 * STAGE_BYTES > PATCH_BYTES ? 2 * STAGE_BYTES : PATCH_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "tile does not fit the LDS");
  return LDS_BYTES;
}

// More than 64 KB of dynamic LDS has to be allowed once per kernel and device.  The library does it for all its
// instantiations when a state is created (that call must not end up inside a stream capture); the launcher
// repeats it for a device it has not seen.
template <class Cfg, bool GBF16, int EPI, bool DUAL, bool AKS = false, bool BKS = false>
inline hipError_t gemm3_prepare() {
  static bool allowed[16] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
  if (!allowed[dev]) {
    e = hipFuncSetAttribute((const void*)gemm3_kernel<Cfg, GBF16, EPI, DUAL, AKS, BKS>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            gemm3_lds_bytes<Cfg, DUAL>());
    if (e != hipSuccess) return e;
    allowed[dev] = true;
  }
  return hipSuccess;
}

template <class Cfg, bool GBF16, int EPI, bool DUAL, bool AKS = false, bool BKS = false>
inline hipError_t launch_gemm3(GemmArgs g, int batch, hipStream_t stream) {
  if (!gemm3_fits<Cfg, AKS, BKS>(g)) return hipErrorInvalidValue;
  if (DUAL && g.B2.ld != g.B.ld) return hipErrorInvalidValue;          // B2 is fetched with B's offsets
  if (g.slab_count > 0 && (EPI != EPI_STORE || DUAL || g.nseg > 0 || g.splitk > 1 || g.slab_first < 0 ||
                           g.slab_first + g.slab_count > g.K / Cfg::BK))
    return hipErrorInvalidValue;
  if (g.E.beta != 0.f && (g.E.beta != 1.f || g.slab_count <= 0)) return hipErrorInvalidValue;
  if (g.A.off != 0 && (AKS || g.nseg > 0 || g.A.off < 0 || g.A.off % 8)) return hipErrorInvalidValue;   // (k-fast single pair, 16-byte aligned)
  if (g.slab_count > 0) g.tail_slot = -1;   // (no split last round for a part of a contraction)
  const int kseg = g.nseg > 0 ? g.kseg : g.K;
  g.tiles_m = g.M / Cfg::BM;
  g.tiles_n = g.N / Cfg::BN;
  if (g.splitk < 1) g.splitk = 1;
  const int total = (g.nseg > 0 ? g.nseg : 1) * (kseg / Cfg::BK);
  if (g.splitk > total) g.splitk = total;
  g.k_per_split = (total + g.splitk - 1) / g.splitk;
  g.splitk = (total + g.k_per_split - 1) / g.k_per_split;
  g.tri_grid = (g.lower_only && Cfg::BM == Cfg::BN && g.tiles_m == g.tiles_n && g.group_n == 0) ? 1 : 0;
  const long long ntile = g.tri_grid ? (long long)g.tiles_m * (g.tiles_m + 1) / 2 : (long long)g.tiles_m * g.tiles_n;
  const long long blocks = ntile * g.splitk * batch;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  // last round: when its tiles would occupy fewer than half the compute units, split each over k
  long long grid = blocks;
  g.tail_tiles = 0; g.tail_split = 1; g.tail_first = 0;
  if (EPI == EPI_STORE && !DUAL && g.cus > 0 && g.tail_slot >= 0 && batch == 1 && g.splitk == 1 && !g.tri_grid && !g.lower_only &&
      !g.heavy_first && ntile > g.cus) {
    const int tail = (int)(ntile % g.cus);
    const int sp = tail > 0 ? std::min(8, g.cus / tail) : 1;
    if (sp >= 2 && total / sp >= 16) {
      g.tail_tiles = tail; g.tail_split = sp; g.tail_first = (int)(ntile - tail);
      grid = (ntile - tail) + (long long)tail * sp;
    }
  }
  // (the XCD remapping permutes the workgroups of the full rounds; a split tail keeps its place at the end)
  g.xcd_remap = (g.xcd_remap && ((g.tail_split > 1 ? (long long)g.tail_first : grid) % 8 == 0)) ? 1 : 0;
  g.heavy_first = (g.heavy_first && g.xcd_remap && !g.tri_grid && g.group_n == 0 && g.splitk == 1 && batch == 1 && g.tiles_m % 8 == 0) ? 1 : 0;
  constexpr int LDS_BYTES = gemm3_lds_bytes<Cfg, DUAL>();
  hipError_t e = gemm3_prepare<Cfg, GBF16, EPI, DUAL, AKS, BKS>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm3_kernel<Cfg, GBF16, EPI, DUAL, AKS, BKS>), dim3((unsigned)grid), dim3(Cfg::NT), LDS_BYTES, stream, g);
  e = hipGetLastError();
  if (e != hipSuccess || g.tail_split < 2) return e;
  if constexpr (EPI == EPI_STORE && !DUAL) {
    hipLaunchKernelGGL((gemm3_tail_reduce_kernel<Cfg>), dim3(g.tail_tiles, Cfg::BM / Cfg::WTM), dim3(1024), 0, stream, g);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace dion
