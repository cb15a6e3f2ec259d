// Tiled MFMA GEMM core for gfx950, shared by every dense product of the Dion step.
//
// All products are brought to the form  C[i,j] (op)= sum_k A(i,k) * B(j,k)  over LDS tiles that
// hold k contiguously per row.  What differs between the uses is only
//   - where an operand element comes from (fp32 matrix read along k, fp32 matrix read across k
//     and transposed on the way into LDS, or the fused sum M + G that forms the paper's
//     accumulated buffer B = M + G without ever storing it), and
//   - what happens to the accumulators (plain store, or the fused error-feedback + weight
//     update of the unsharded update rule).
// MMA flavours: bf16 operands (v_mfma_f32_32x32x16_bf16) or fp32 operands
// (v_mfma_f32_32x32x2_f32); accumulation is fp32 in both.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace dion {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// Operand sources.  KC: element (row,k) at p[row*ld + k].  KS: element (row,k) at p[k*ld + row].
enum { SRC_F32_KC = 0, SRC_F32_KS = 1, SRC_SUM_KC = 2, SRC_SUM_KS = 3 };
// Epilogues.
enum { EPI_STORE = 0, EPI_UPDATE = 1, EPI_UPDATE_STREAM = 2 };   // the last: direct-load core only, non-temporal M, X, G

struct Operand {
  int slot0;            // pointer-table slot of the fp32 matrix
  int slot1;            // slot of G (SUM sources only)
  long long off;        // element offset of the sub-matrix
  long long ld;         // leading dimension in elements
  long long sub_stride; // extra element offset per sub-problem
};

struct EpilogueDesc {
  int slot;             // output matrix (EPI_STORE)
  long long off, ld, sub_stride, split_stride;
  float alpha, beta;    // C = alpha*acc + beta*C
  // EPI_UPDATE: M = (M+G) - c_m*acc ; X = X - c_x*acc2      (ld is the leading dimension n)
  int slotX, slotG, slotM;
  float c_m, c_x;
  int x_overwrite;      // EPI_UPDATE: X = -c_x*acc2, the old contents of X are not read
  int colsq_slot;       // EPI_STORE of the direct-load core, whole products only: >= 0: per-column partial sums of squares
                        // of the result go there, one row of N floats per block of Cfg::WTM result rows
  int split_hi1, split_lo1;   // EPI_STORE of the direct-load core, whole products only: slot + 1 (0: none) of two bf16
                        // matrices of the result's shape and leading dimension that receive the result split as
                        // x = hi + lo, hi = bf16(x), lo = bf16(x - hi): the operands of a split-bf16 product that follows
  int stream_hint;      // host side: take the EPI_UPDATE_STREAM kernel (M, X and G loaded and stored with the
                        // non-temporal hint; for working sets far beyond the last-level cache)
};

struct GemmArgs {
  void* const* table;   // device pointer table, nslots entries per batch member
  int nslots;
  int M, N, K;
  int tiles_m, tiles_n, splitk, k_per_split, sub_count;
  int lower_only;       // skip tiles strictly above the diagonal
  int status_slot;      // >= 0: skip the whole problem when *status != 0
  int xcd_remap;        // spread consecutive logical tiles over one XCD (grid must be a multiple of 8)
  // Large-tile kernels only: the contraction may run over up to three (A, B) operand pairs of length kseg
  // each (split-bf16 products: hi*hi + hi*lo + lo*hi), all sharing A.ld / B.ld.  nseg == 0 means one pair.
  int nseg, kseg;
  int segA[3], segB[3];
  int tri_k;            // B is lower triangular: column tile tn only needs k < (tn+1)*BN of every segment
  int group_n;          // > 0: tiles are visited column group by column group (group_n column tiles wide, all row
                        // tiles inside a group before the next group), so the B panels of a group stay in L2
  int noop_slot;        // large-tile kernels: >= 0 and the int32 there non-zero: the launch does nothing (like status_slot)
  int slab_first, slab_count;   // direct-load core, slab_count > 0: this launch contracts over the k-slabs [slab_first, slab_first +
                        // slab_count) only (plain products: one operand pair, no split over k, no split tail); with E.beta = 1
                        // it adds to what is in the output, so that a contraction can be spread over launches
  int heavy_first;      // direct-load core, triangular B (tri_k): column tiles cost (tn + 1) units each; every XCD gets
                        // tiles_m / 8 tile rows and visits their column tiles from the costliest down, so that the
                        // second round of workgroups fills in behind the first (needs xcd_remap, one matrix, split-K 1)
  int tri_grid;         // set by the direct-load launcher: lower_only grids hold the lower-triangle tiles only
  int side_slot;        // large-tile K1 only, >= 0: bf16(M + G) is also written there ([M][K] row-major, bf16)
  // Direct-load core, plain store, one matrix, no split over k: when the tiles make a last round that would leave most
  // compute units idle (tail_tiles of them, fewer than half the compute units), each of those tiles is split over k by
  // tail_split workgroups whose partial tiles go to tail_slot ([tail tile][split][BM][BN] floats); launch_gemm3 follows
  // up with a kernel that adds them into the result (and forms the column sums of squares the main kernel would have).
  int cus;              // host side: compute units of the device (0: no tail split)
  int tail_slot;        // >= 0: buffer for the partial tiles, at least 256 tiles of BM x BN floats (-1: no tail split)
  int tail_tiles, tail_split, tail_first;   // set by the launcher
  Operand A, B, B2;
  EpilogueDesc E;
};

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NT = 64 * WAVES_M_ * WAVES_N_;
  static constexpr int WTM = BM_ / WAVES_M_, WTN = BN_ / WAVES_N_;
  static constexpr int MI = WTM / 32, NI = WTN / 32;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
};

// Accesses through the global address space: the compiler then emits global_load / global_store, which count
// only against vmcnt.  A generic (flat) access also counts against lgkmcnt, so every wait for an LDS read
// would wait for all outstanding global prefetches as well and nothing would overlap.
template <class T>
__device__ __forceinline__ T gload(const void* p) {
  return *(const __attribute__((address_space(1))) T*)(p);
}
template <class T>
__device__ __forceinline__ void gstore(void* p, T v) {
  *(__attribute__((address_space(1))) T*)(p) = v;
}

// The same with the non-temporal hint, for data that is read or written once per step and is far too large to be
// found in a cache the next time: a pass that updates M and X in place streams about 10 % faster with the hint on both
// its loads and its stores (5.5-5.8 against 4.9-5.2 TB/s for the 18-byte-per-element update; either alone gains nothing).
template <class T>
__device__ __forceinline__ T gload_nt(const void* p) {
  return __builtin_nontemporal_load((const __attribute__((address_space(1))) T*)(p));
}
template <class T>
__device__ __forceinline__ void gstore_nt(void* p, T v) {
  __builtin_nontemporal_store(v, (__attribute__((address_space(1))) T*)(p));
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t v = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }

// ---------------------------------------------------------------------------------------------
// Global -> registers -> LDS tile mover for one operand tile of ROWS x BK.
// LDS layout: [row][k], row stride BKP elements (BK + 16 bytes of padding), element = bf16 or fp32.
template <class Cfg, int ROWS, bool BF16, int SRC, bool GBF16, bool CHECKED>
struct TileMover {
  static constexpr int BK = Cfg::BK, NT = Cfg::NT;
  static constexpr int VEC = BF16 ? 8 : 4;  // elements per 16-byte LDS vector
  static constexpr bool KS = (SRC == SRC_F32_KS || SRC == SRC_SUM_KS);
  static constexpr bool SUM = (SRC == SRC_SUM_KC || SRC == SRC_SUM_KS);
  static constexpr int BKP = BK + (BF16 ? 8 : 4);
  // KC: an item is one row x VEC k.  KS: an item is a patch of 4 k x 4 rows.
  static constexpr int ITEMS = KS ? (ROWS / 4) * (BK / 4) : ROWS * (BK / VEC);
  static constexpr int PER = ITEMS / NT;
  static constexpr int EL = KS ? 16 : VEC;
  static constexpr int GW = !SUM ? 1 : (CHECKED ? EL : (GBF16 ? EL / 2 : EL));
  static_assert(ITEMS % NT == 0 && PER >= 1, "tile does not divide over the workgroup");
  static_assert(ROWS % 4 == 0 && BK % VEC == 0, "tile shape");

  float a[PER][EL];
  uint32_t g[PER][GW];

  // p0: fp32 matrix, p1: G (bf16 or fp32) for SUM sources.  row0/k0: tile origin.
  // rows_total/k_end: bounds (used when CHECKED).
  __device__ __forceinline__ void load(const float* __restrict__ p0, const void* __restrict__ p1,
                                       long long ld, int row0, int k0, int rows_total, int k_end) {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int item = t + i * NT;
      if constexpr (!KS) {
        const int row = item / (BK / VEC), kc = item % (BK / VEC);
        const long long idx = (long long)(row0 + row) * ld + (k0 + kc * VEC);
        if constexpr (!CHECKED) {
#pragma unroll
          for (int v = 0; v < VEC / 4; ++v) {
            f32x4_t x = gload<f32x4_t>(p0 + idx + 4 * v);
            a[i][4 * v + 0] = x[0]; a[i][4 * v + 1] = x[1]; a[i][4 * v + 2] = x[2]; a[i][4 * v + 3] = x[3];
          }
          if constexpr (SUM) {
            if constexpr (GBF16) {
              const uint16_t* gp = (const uint16_t*)p1 + idx;
              if constexpr (VEC == 8) {
                u32x4_t x = gload<u32x4_t>(gp);
                g[i][0] = x[0]; g[i][1] = x[1]; g[i][2] = x[2]; g[i][3] = x[3];
              } else {
                u32x2_t x = gload<u32x2_t>(gp);
                g[i][0] = x[0]; g[i][1] = x[1];
              }
            } else {
              const float* gp = (const float*)p1 + idx;
#pragma unroll
              for (int v = 0; v < VEC / 4; ++v) {
                u32x4_t x = gload<u32x4_t>(gp + 4 * v);
                g[i][4 * v + 0] = x[0]; g[i][4 * v + 1] = x[1]; g[i][4 * v + 2] = x[2]; g[i][4 * v + 3] = x[3];
              }
            }
          }
        } else {
          const bool rok = (row0 + row) < rows_total;
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            const bool ok = rok && (k0 + kc * VEC + e) < k_end;
            a[i][e] = ok ? gload<float>(p0 + idx + e) : 0.f;
            if constexpr (SUM) {
              float gv = 0.f;
              if (ok) gv = GBF16 ? bf16_to_f32(gload<uint16_t>((const uint16_t*)p1 + idx + e)) : gload<float>((const float*)p1 + idx + e);
              g[i][e] = __builtin_bit_cast(uint32_t, gv);
            }
          }
        }
      } else {
        const int rg = item % (ROWS / 4), kc = item / (ROWS / 4);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const long long idx = (long long)(k0 + kc * 4 + kk) * ld + (row0 + rg * 4);
          if constexpr (!CHECKED) {
            f32x4_t x = gload<f32x4_t>(p0 + idx);
            a[i][4 * kk + 0] = x[0]; a[i][4 * kk + 1] = x[1]; a[i][4 * kk + 2] = x[2]; a[i][4 * kk + 3] = x[3];
            if constexpr (SUM) {
              if constexpr (GBF16) {
                u32x2_t y = gload<u32x2_t>((const uint16_t*)p1 + idx);
                g[i][2 * kk + 0] = y[0]; g[i][2 * kk + 1] = y[1];
              } else {
                u32x4_t y = gload<u32x4_t>((const float*)p1 + idx);
                g[i][4 * kk + 0] = y[0]; g[i][4 * kk + 1] = y[1]; g[i][4 * kk + 2] = y[2]; g[i][4 * kk + 3] = y[3];
              }
            }
          } else {
            const bool kok = (k0 + kc * 4 + kk) < k_end;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
              const bool ok = kok && (row0 + rg * 4 + rr) < rows_total;
              a[i][4 * kk + rr] = ok ? gload<float>(p0 + idx + rr) : 0.f;
              if constexpr (SUM) {
                float gv = 0.f;
                if (ok) gv = GBF16 ? bf16_to_f32(gload<uint16_t>((const uint16_t*)p1 + idx + rr)) : gload<float>((const float*)p1 + idx + rr);
                g[i][4 * kk + rr] = __builtin_bit_cast(uint32_t, gv);
              }
            }
          }
        }
      }
    }
  }

  // value e of item i, with G added for SUM sources (fp32 add, as the accumulate line M <- M + G)
  __device__ __forceinline__ float val(int i, int e) const {
    float x = a[i][e];
    if constexpr (SUM) {
      if constexpr (CHECKED || !GBF16) x += __builtin_bit_cast(float, g[i][e]);
      else x += (e & 1) ? bf16_hi(g[i][e >> 1]) : bf16_lo(g[i][e >> 1]);
    }
    return x;
  }

  template <class LT>
  __device__ __forceinline__ void store(LT* __restrict__ lds) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int item = t + i * NT;
      if constexpr (!KS) {
        const int row = item / (BK / VEC), kc = item % (BK / VEC);
        LT* dst = lds + row * BKP + kc * VEC;
        if constexpr (BF16) {
          u32x4_t w;
          w[0] = pack_bf16x2(val(i, 0), val(i, 1)); w[1] = pack_bf16x2(val(i, 2), val(i, 3));
          w[2] = pack_bf16x2(val(i, 4), val(i, 5)); w[3] = pack_bf16x2(val(i, 6), val(i, 7));
          *(u32x4_t*)dst = w;
        } else {
          f32x4_t w = {val(i, 0), val(i, 1), val(i, 2), val(i, 3)};
          *(f32x4_t*)dst = w;
        }
      } else {
        const int rg = item % (ROWS / 4), kc = item / (ROWS / 4);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          LT* dst = lds + (rg * 4 + rr) * BKP + kc * 4;
          if constexpr (BF16) {
            u32x2_t w;
            w[0] = pack_bf16x2(val(i, 0 * 4 + rr), val(i, 1 * 4 + rr));
            w[1] = pack_bf16x2(val(i, 2 * 4 + rr), val(i, 3 * 4 + rr));
            *(u32x2_t*)dst = w;
          } else {
            f32x4_t w = {val(i, 0 * 4 + rr), val(i, 1 * 4 + rr), val(i, 2 * 4 + rr), val(i, 3 * 4 + rr)};
            *(f32x4_t*)dst = w;
          }
        }
      }
    }
  }
};

// ---------------------------------------------------------------------------------------------
template <class Cfg, bool BF16, int ASRC, int BSRC, bool GBF16, int EPI, bool DUAL, bool CHECKED>
__global__ void __launch_bounds__(Cfg::NT) gemm_kernel(const GemmArgs g) {
  using LT = typename std::conditional<BF16, uint16_t, float>::type;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
  constexpr int BKP = BK + (BF16 ? 8 : 4);
  constexpr int MI = Cfg::MI, NI = Cfg::NI;
  __shared__ __attribute__((aligned(16))) LT As[BM * BKP];
  __shared__ __attribute__((aligned(16))) LT Bs[BN * BKP];
  __shared__ __attribute__((aligned(16))) LT B2s[DUAL ? BN * BKP : 4];

  int bid = blockIdx.x;
  if (g.xcd_remap) {
    const int per = gridDim.x >> 3;
    bid = (bid & 7) * per + (bid >> 3);
  }
  const int ntile = g.tiles_m * g.tiles_n;
  const int tile = bid % ntile;
  int rest = bid / ntile;
  const int ks = rest % g.splitk;
  rest /= g.splitk;
  const int sub = rest % g.sub_count;
  const int b = rest / g.sub_count;
  const int tn = tile % g.tiles_n, tm = tile / g.tiles_n;
  if (g.lower_only && tn * BN > tm * BM + BM - 1) return;

  void* const* tab = g.table + (size_t)b * g.nslots;
  if (g.status_slot >= 0 && *(const int*)tab[g.status_slot] != 0) return;

  const float* A0 = (const float*)tab[g.A.slot0] + g.A.off + sub * g.A.sub_stride;
  const float* B0 = (const float*)tab[g.B.slot0] + g.B.off + sub * g.B.sub_stride;
  const void* A1 = nullptr;
  const void* B1 = nullptr;
  if constexpr (ASRC == SRC_SUM_KC || ASRC == SRC_SUM_KS) {
    const long long o = g.A.off + sub * g.A.sub_stride;
    A1 = GBF16 ? (const void*)((const uint16_t*)tab[g.A.slot1] + o) : (const void*)((const float*)tab[g.A.slot1] + o);
  }
  if constexpr (BSRC == SRC_SUM_KC || BSRC == SRC_SUM_KS) {
    const long long o = g.B.off + sub * g.B.sub_stride;
    B1 = GBF16 ? (const void*)((const uint16_t*)tab[g.B.slot1] + o) : (const void*)((const float*)tab[g.B.slot1] + o);
  }
  const float* B20 = nullptr;
  if constexpr (DUAL) B20 = (const float*)tab[g.B2.slot0] + g.B2.off + sub * g.B2.sub_stride;

  const int row0 = tm * BM, col0 = tn * BN;
  const int k_begin = ks * g.k_per_split;
  const int k_end = min(g.K, k_begin + g.k_per_split);

  TileMover<Cfg, BM, BF16, ASRC, GBF16, CHECKED> ma;
  TileMover<Cfg, BN, BF16, BSRC, GBF16, CHECKED> mb;
  TileMover<Cfg, BN, BF16, SRC_F32_KC, false, CHECKED> mb2;

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

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave % Cfg::WAVES_M, wn = wave / Cfg::WAVES_M;
  const int lr = lane & 31, lk = lane >> 5;

  if (k_begin < k_end) {
    ma.load(A0, A1, g.A.ld, row0, k_begin, g.M, k_end);
    mb.load(B0, B1, g.B.ld, col0, k_begin, g.N, k_end);
    if constexpr (DUAL) mb2.load(B20, nullptr, g.B2.ld, col0, k_begin, g.N, k_end);
  }
  for (int k0 = k_begin; k0 < k_end; k0 += BK) {
    ma.store(As);
    mb.store(Bs);
    if constexpr (DUAL) mb2.store(B2s);
    __syncthreads();
    if (k0 + BK < k_end) {
      ma.load(A0, A1, g.A.ld, row0, k0 + BK, g.M, k_end);
      mb.load(B0, B1, g.B.ld, col0, k0 + BK, g.N, k_end);
      if constexpr (DUAL) mb2.load(B20, nullptr, g.B2.ld, col0, k0 + BK, g.N, k_end);
    }
    if constexpr (BF16) {
#pragma unroll
      for (int kk = 0; kk < BK; kk += 16) {
        bf16x8_t af[MI], bf[NI], bf2[DUAL ? NI : 1];
#pragma unroll
        for (int i = 0; i < MI; ++i)
          af[i] = *(const bf16x8_t*)(As + (wm * Cfg::WTM + i * 32 + lr) * BKP + kk + lk * 8);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          bf[j] = *(const bf16x8_t*)(Bs + (wn * Cfg::WTN + j * 32 + lr) * BKP + kk + lk * 8);
          if constexpr (DUAL) bf2[j] = *(const bf16x8_t*)(B2s + (wn * Cfg::WTN + j * 32 + lr) * BKP + kk + lk * 8);
        }
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
            if constexpr (DUAL) acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf2[j], acc2[i][j], 0, 0, 0);
          }
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < BK; kk += 8) {
        f32x4_t af[MI], bf[NI], bf2[DUAL ? NI : 1];
#pragma unroll
        for (int i = 0; i < MI; ++i)
          af[i] = *(const f32x4_t*)(As + (wm * Cfg::WTM + i * 32 + lr) * BKP + kk + lk * 4);
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          bf[j] = *(const f32x4_t*)(Bs + (wn * Cfg::WTN + j * 32 + lr) * BKP + kk + lk * 4);
          if constexpr (DUAL) bf2[j] = *(const f32x4_t*)(B2s + (wn * Cfg::WTN + j * 32 + lr) * BKP + kk + lk * 4);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][s], bf[j][s], acc[i][j], 0, 0, 0);
              if constexpr (DUAL) acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][s], bf2[j][s], acc2[i][j], 0, 0, 0);
            }
      }
    }
    __syncthreads();
  }

  // ---- epilogue.  Accumulator register v of lane l holds C[8*(v/4) + 4*(l/32) + v%4][l%32] of its 32x32 tile.
  if constexpr (EPI == EPI_STORE) {
    float* C = (float*)tab[g.E.slot] + g.E.off + sub * g.E.sub_stride + (long long)ks * g.E.split_stride;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row0 + wm * Cfg::WTM + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
          const int col = col0 + wn * Cfg::WTN + j * 32 + lr;
          if (CHECKED && (row >= g.M || col >= g.N)) continue;
          float* c = C + (long long)row * g.E.ld + col;
          float out = g.E.alpha * acc[i][j][v];
          if (g.E.beta != 0.f) out += g.E.beta * gload<float>(c);
          gstore<float>(c, out);
        }
  } else {
    // Fused error feedback and weight update (unsharded update rule):
    //   M <- (M + G) - (1-mu) * (P R^T)        X <- X - eta*sqrt(m/n) * (P Q_new^T)
    float* Xp = (float*)tab[g.E.slotX];
    float* Mp = (float*)tab[g.E.slotM];
    const void* Gp = tab[g.E.slotG];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = row0 + wm * Cfg::WTM + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
          const int col = col0 + wn * Cfg::WTN + j * 32 + lr;
          if (CHECKED && (row >= g.M || col >= g.N)) continue;
          const long long idx = (long long)row * g.E.ld + col;
          const float gv = GBF16 ? bf16_to_f32(gload<uint16_t>((const uint16_t*)Gp + idx)) : gload<float>((const float*)Gp + idx);
          const float bv = gload<float>(Mp + idx) + gv;
          gstore<float>(Mp + idx, bv - g.E.c_m * acc[i][j][v]);
          if constexpr (DUAL) gstore<float>(Xp + idx, (g.E.x_overwrite ? 0.f : gload<float>(Xp + idx)) - g.E.c_x * acc2[i][j][v]);
        }
  }
}

// Host-side launcher.  The caller has validated shapes; `fast` kernels need every dimension to be
// a multiple of its tile and 16-byte aligned rows.
template <class Cfg, bool BF16, int ASRC, int BSRC, bool GBF16, int EPI, bool DUAL, bool CHECKED>
inline hipError_t launch_gemm(GemmArgs g, int batch, hipStream_t stream) {
  g.tiles_m = (g.M + Cfg::BM - 1) / Cfg::BM;
  g.tiles_n = (g.N + Cfg::BN - 1) / Cfg::BN;
  if (g.splitk < 1) g.splitk = 1;
  if (g.sub_count < 1) g.sub_count = 1;
  if (g.splitk == 1) g.k_per_split = g.K;
  const long long blocks = (long long)g.tiles_m * g.tiles_n * g.splitk * g.sub_count * batch;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  g.xcd_remap = (g.xcd_remap && (blocks % 8 == 0)) ? 1 : 0;
  hipLaunchKernelGGL((gemm_kernel<Cfg, BF16, ASRC, BSRC, GBF16, EPI, DUAL, CHECKED>), dim3((unsigned)blocks), dim3(Cfg::NT), 0,
                     stream, g);
  return hipGetLastError();
}

}  // namespace dion
