// Register-staged bf16 MFMA GEMM core for gfx950 (v_mfma_f32_32x32x16_bf16): operand tiles go global ->
// registers -> LDS, which lets an operand be transformed on the way (the fused sum M + G, a transposition).
// Serves the big products of the Dion step when the shapes are multiples of the tile but the output has too few
// 256-wide tiles to fill the GPU (128 x 128 tiles, split-K), and any shape the direct-load core
// (gemm_core3.hpp) cannot take:
//   K1  Z = (M+G) Q          A = fused sum read along k (its bf16 values can be kept in memory on the way),
//                            B = Q^T  (bf16 copy, k contiguous)
//   K2  R = (M+G)^T P        A = that bf16 copy (or the fused sum itself) transposed into LDS,
//                            B = P^T  (bf16 copy, k contiguous)
//   K5  M, X updates         A = P (bf16 copy), B = R, B2 = Q_new (bf16 copies), fused epilogue
// Same conventions as gemm_core.hpp: C[i,j] = sum_k A(i,k) B(j,k), LDS tiles [row][k] with 16 bytes
// of padding per row, register prefetch of the next k-slab while the MFMAs of the current one run.
#pragma once
#include "gemm_core.hpp"

namespace dion {

// Operand sources: bf16 matrix read along k; fused fp32 sum M + G read along k; the same sum read across k
// (transposed on its way into LDS); bf16 matrix read across k.
enum { SRC2_BF16_KC = 0, SRC2_SUM_KC = 1, SRC2_SUM_KS = 2, SRC2_BF16_KS = 3 };

template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_, int MINW_>
struct TileCfg2 {
  static constexpr int BM = BM_, BN = BN_, BK = BK_;
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NT = 64 * WAVES_M_ * WAVES_N_;
  static constexpr int WTM = BM_ / WAVES_M_, WTN = BN_ / WAVES_N_;
  static constexpr int MI = WTM / 32, NI = WTN / 32;
  static constexpr int STAGES = STAGES_, MINW = MINW_;
  static constexpr int BKP = BK_ + 8;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK_ % 16 == 0, "tile shape");
};

// Global -> registers -> LDS mover of one ROWS x BK bf16 operand tile.
template <class Cfg, int ROWS, int SRC, bool GBF16>
struct Mover2 {
  static constexpr int BK = Cfg::BK, NT = Cfg::NT, BKP = Cfg::BKP;
  static constexpr bool KS = (SRC == SRC2_SUM_KS || SRC == SRC2_BF16_KS);
  static constexpr bool SUM = (SRC == SRC2_SUM_KC || SRC == SRC2_SUM_KS);
  // KC: item = 1 row x 8 k.   KS: item = 8 k x 4 rows.
  static constexpr int ITEMS = KS ? (ROWS / 4) * (BK / 8) : ROWS * (BK / 8);
  static constexpr int PER = ITEMS / NT;
  static_assert(ITEMS % NT == 0 && PER >= 1, "tile does not divide over the workgroup");
  static constexpr int AW = SUM ? (KS ? 32 : 8) : (KS ? 16 : 4);      // 32-bit words of the main operand per item
  static constexpr int GW = !SUM ? 1 : (GBF16 ? AW / 2 : AW);         // words of G per item

  uint32_t a[PER][AW];
  uint32_t g[PER][GW];
  int k0_;   // k offset of the slab in the registers (for the side copy)

  __device__ __forceinline__ void load(const void* __restrict__ p0, const void* __restrict__ p1, long long ld, int row0, int k0) {
    const int t = threadIdx.x;
    k0_ = k0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int item = t + i * NT;
      if constexpr (!KS) {
        const int row = item / (BK / 8), kc = item % (BK / 8);
        const long long idx = (long long)(row0 + row) * ld + (k0 + kc * 8);
        if constexpr (!SUM) {
          const u32x4_t x = gload<u32x4_t>((const uint16_t*)p0 + idx);
          a[i][0] = x[0]; a[i][1] = x[1]; a[i][2] = x[2]; a[i][3] = x[3];
        } else {
          const u32x4_t x0 = gload<u32x4_t>((const float*)p0 + idx);
          const u32x4_t x1 = gload<u32x4_t>((const float*)p0 + idx + 4);
          a[i][0] = x0[0]; a[i][1] = x0[1]; a[i][2] = x0[2]; a[i][3] = x0[3];
          a[i][4] = x1[0]; a[i][5] = x1[1]; a[i][6] = x1[2]; a[i][7] = x1[3];
          if constexpr (GBF16) {
            const u32x4_t y = gload<u32x4_t>((const uint16_t*)p1 + idx);
            g[i][0] = y[0]; g[i][1] = y[1]; g[i][2] = y[2]; g[i][3] = y[3];
          } else {
            const u32x4_t y0 = gload<u32x4_t>((const float*)p1 + idx);
            const u32x4_t y1 = gload<u32x4_t>((const float*)p1 + idx + 4);
            g[i][0] = y0[0]; g[i][1] = y0[1]; g[i][2] = y0[2]; g[i][3] = y0[3];
            g[i][4] = y1[0]; g[i][5] = y1[1]; g[i][6] = y1[2]; g[i][7] = y1[3];
          }
        }
      } else {
        const int rg = item % (ROWS / 4), kc = item / (ROWS / 4);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const long long idx = (long long)(k0 + kc * 8 + kk) * ld + (row0 + rg * 4);
          if constexpr (!SUM) {
            const u32x2_t x = gload<u32x2_t>((const uint16_t*)p0 + idx);
            a[i][2 * kk + 0] = x[0]; a[i][2 * kk + 1] = x[1];
            continue;
          }
          const u32x4_t x = gload<u32x4_t>((const float*)p0 + idx);
          a[i][4 * kk + 0] = x[0]; a[i][4 * kk + 1] = x[1]; a[i][4 * kk + 2] = x[2]; a[i][4 * kk + 3] = x[3];
          if constexpr (GBF16) {
            const u32x2_t y = gload<u32x2_t>((const uint16_t*)p1 + idx);
            g[i][2 * kk + 0] = y[0]; g[i][2 * kk + 1] = y[1];
          } else {
            const u32x4_t y = gload<u32x4_t>((const float*)p1 + idx);
            g[i][4 * kk + 0] = y[0]; g[i][4 * kk + 1] = y[1]; g[i][4 * kk + 2] = y[2]; g[i][4 * kk + 3] = y[3];
          }
        }
      }
    }
  }

  // fp32 value e of item i of the fused sum M + G
  __device__ __forceinline__ float sum(int i, int e) const {
    float x = __builtin_bit_cast(float, a[i][e]);
    if constexpr (GBF16) x += (e & 1) ? bf16_hi(g[i][e >> 1]) : bf16_lo(g[i][e >> 1]);
    else x += __builtin_bit_cast(float, g[i][e]);
    return x;
  }

  // side != nullptr (fused sum read along k only): the bf16 values also go to side[row][k], leading dimension ld
  __device__ __forceinline__ void store(uint16_t* __restrict__ lds, uint16_t* __restrict__ side = nullptr, long long ld = 0,
                                        int row0 = 0) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int item = t + i * NT;
      if constexpr (!KS) {
        const int row = item / (BK / 8), kc = item % (BK / 8);
        u32x4_t w;
        if constexpr (!SUM) {
          w[0] = a[i][0]; w[1] = a[i][1]; w[2] = a[i][2]; w[3] = a[i][3];
        } else {
          w[0] = pack_bf16x2(sum(i, 0), sum(i, 1)); w[1] = pack_bf16x2(sum(i, 2), sum(i, 3));
          w[2] = pack_bf16x2(sum(i, 4), sum(i, 5)); w[3] = pack_bf16x2(sum(i, 6), sum(i, 7));
          if (side) gstore<u32x4_t>(side + (long long)(row0 + row) * ld + (k0_ + kc * 8), w);
        }
        *(u32x4_t*)(lds + row * BKP + kc * 8) = w;
      } else {
        const int rg = item % (ROWS / 4), kc = item / (ROWS / 4);
        if constexpr (!SUM) {
          // element (k, row rr) is the (rr & 1) half of word a[2 k + rr / 2]: gather the halves of two k per word
          constexpr unsigned SEL_LO = 0x05040100u, SEL_HI = 0x07060302u;
          u32x4_t wr[4];
#pragma unroll
          for (int rr = 0; rr < 4; ++rr)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              wr[rr][j] = __builtin_amdgcn_perm(a[i][2 * (2 * j + 1) + rr / 2], a[i][2 * (2 * j) + rr / 2], (rr & 1) ? SEL_HI : SEL_LO);
          // Lanes that are neighbours hold rows 4 apart, which with this row stride fall on the same banks four at
          // a time; so in each of the four rounds a lane writes a different one of its rows, chosen so that any 16
          // consecutive lanes hit 16 different residues of the row number modulo 16.
          const int rot = (rg >> 2) & 3;
#pragma unroll
          for (int rnd = 0; rnd < 4; ++rnd) {
            const int rr = (rnd + rot) & 3;
            u32x4_t w;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const uint32_t lo = (rr & 1) ? wr[1][j] : wr[0][j], hi = (rr & 1) ? wr[3][j] : wr[2][j];
              w[j] = (rr & 2) ? hi : lo;
            }
            *(u32x4_t*)(lds + (rg * 4 + rr) * BKP + kc * 8) = w;
          }
          continue;
        }
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          u32x4_t w;
          w[0] = pack_bf16x2(sum(i, 0 * 4 + rr), sum(i, 1 * 4 + rr));
          w[1] = pack_bf16x2(sum(i, 2 * 4 + rr), sum(i, 3 * 4 + rr));
          w[2] = pack_bf16x2(sum(i, 4 * 4 + rr), sum(i, 5 * 4 + rr));
          w[3] = pack_bf16x2(sum(i, 6 * 4 + rr), sum(i, 7 * 4 + rr));
          *(u32x4_t*)(lds + (rg * 4 + rr) * BKP + kc * 8) = w;
        }
      }
    }
  }
};

template <class Cfg, int ASRC, bool GBF16, int EPI, bool DUAL>
__global__ void __launch_bounds__(Cfg::NT, Cfg::MINW) gemm2_kernel(const GemmArgs g) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, BKP = Cfg::BKP;
  // STAGES: 1 = one LDS buffer, 2 = two LDS buffers, 3 = two LDS buffers and two register sets (the global
  // loads of k-slab s+2 are issued while slab s is multiplied: two slabs in flight instead of one)
  constexpr int MI = Cfg::MI, NI = Cfg::NI, ST = Cfg::STAGES >= 2 ? 2 : 1;
  constexpr bool DEEP = Cfg::STAGES == 3;
  constexpr int SP = 36;   // epilogue patch row stride in floats (16-byte aligned rows, conflict-free)
  constexpr size_t OPER_BYTES = (size_t)(ST * BM * BKP + ST * BN * BKP + (DUAL ? ST * BN * BKP : 0)) * sizeof(uint16_t);
  constexpr size_t PATCH_BYTES = (size_t)(Cfg::NT / 64) * 32 * SP * sizeof(float);
  __shared__ __attribute__((aligned(16))) unsigned char smem[OPER_BYTES > PATCH_BYTES ? OPER_BYTES : PATCH_BYTES];
  uint16_t* const As = (uint16_t*)smem;
  uint16_t* const Bs = As + ST * BM * BKP;
  uint16_t* const B2s = Bs + ST * BN * BKP;

  int bid = blockIdx.x;
  if (g.xcd_remap) {
    const int per = gridDim.x >> 3;
    bid = (bid & 7) * per + (bid >> 3);
  }
  const int ntile = g.tiles_m * g.tiles_n;
  const int tile = bid % ntile;
  int rest = bid / ntile;
  const int ks = rest % g.splitk;
  const int b = rest / g.splitk;
  int tn = tile % g.tiles_n, tm = tile / g.tiles_n;
  if (g.group_n > 0) {
    const int gw = g.group_n * g.tiles_m;                   // tiles of one full column group
    const int cg = tile / gw;
    const int first = cg * g.group_n;
    const int width = min(g.group_n, g.tiles_n - first);    // the last group may be narrower
    const int rem = tile - cg * gw;
    tm = rem / width;
    tn = first + rem % width;
  }
  if (g.lower_only && tn * BN > tm * BM + BM - 1) return;

  void* const* tab = g.table + (size_t)b * g.nslots;
  if (g.status_slot >= 0 && *(const int*)tab[g.status_slot] != 0) return;

  const void* A1 = (ASRC == SRC2_SUM_KC || ASRC == SRC2_SUM_KS) ? tab[g.A.slot1] : nullptr;
  // the bf16 values of the fused sum are also left in memory: the workgroups of one tile row all hold the same
  // k-slabs of it, so they take turns (slab s is written by tile column s mod tiles_n)
  uint16_t* sideA = nullptr;
  if constexpr (ASRC == SRC2_SUM_KC) sideA = g.side_slot >= 0 ? (uint16_t*)tab[g.side_slot] : nullptr;
  const void* B20 = DUAL ? tab[g.B2.slot0] : nullptr;

  const int row0 = tm * BM, col0 = tn * BN;

  Mover2<Cfg, BM, ASRC, GBF16> ma, ma1;
  Mover2<Cfg, BN, SRC2_BF16_KC, false> mb, mb1;
  Mover2<Cfg, BN, SRC2_BF16_KC, false> mb2, mb21;

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

  // The contraction is a list of k-slabs: nseg operand pairs, each contributing kseg_eff / BK slabs.
  if (g.noop_slot >= 0 && *(const int*)tab[g.noop_slot] != 0) return;   // uniform, before any barrier
  const int nseg = g.nseg > 0 ? g.nseg : 1;
  const int kseg = g.nseg > 0 ? g.kseg : g.K;
  const int kseg_eff = g.tri_k ? min(kseg, (tn + 1) * BN) : kseg;
  const int slabs_per_seg = kseg_eff / BK;
  const int total = nseg * slabs_per_seg;
  const int s_begin = ks * g.k_per_split;                     // k_per_split counts slabs here
  const int s_end = min(total, s_begin + g.k_per_split);
  auto issue = [&](int sl, auto& xa, auto& xb, auto& xb2) __attribute__((always_inline)) {
    const int seg = sl / slabs_per_seg, k0 = (sl - seg * slabs_per_seg) * BK;
    const void* Ap = tab[g.nseg > 0 ? g.segA[seg] : g.A.slot0];
    const void* Bp = tab[g.nseg > 0 ? g.segB[seg] : g.B.slot0];
    xa.load(Ap, A1, g.A.ld, row0, k0);
    xb.load(Bp, nullptr, g.B.ld, col0, k0);
    if constexpr (DUAL) xb2.load(B20, nullptr, g.B2.ld, col0, k0);
  };
  auto stash = [&](int stage, const auto& xa, const auto& xb, const auto& xb2) __attribute__((always_inline)) {
    xa.store(As + stage * BM * BKP, (sideA && (xa.k0_ / BK) % g.tiles_n == tn) ? sideA : nullptr, g.A.ld, row0);
    xb.store(Bs + stage * BN * BKP);
    if constexpr (DUAL) xb2.store(B2s + stage * BN * BKP);
  };
  // MFMAs of one k-slab.  The fragments of k-step s+1 are requested from LDS before the MFMAs of step s are
  // issued (two fragment sets), so the LDS latency hides behind the matrix pipe instead of in front of it.
  auto multiply = [&](int stage) __attribute__((always_inline)) {
    const uint16_t* Ac = As + stage * BM * BKP + (wm * Cfg::WTM + lr) * BKP + lk * 8;
    const uint16_t* Bc = Bs + stage * BN * BKP + (wn * Cfg::WTN + lr) * BKP + lk * 8;
    const uint16_t* B2c = B2s + (DUAL ? stage * BN * BKP + (wn * Cfg::WTN + lr) * BKP + lk * 8 : 0);
    constexpr int KS = BK / 16;
    bf16x8_t af[2][MI], bf[2][NI], bf2[2][DUAL ? NI : 1];
    auto fetch = [&](int set, int kk) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < MI; ++i) af[set][i] = *(const bf16x8_t*)(Ac + i * 32 * BKP + kk);
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        bf[set][j] = *(const bf16x8_t*)(Bc + j * 32 * BKP + kk);
        if constexpr (DUAL) bf2[set][j] = *(const bf16x8_t*)(B2c + j * 32 * BKP + kk);
      }
    };
    fetch(0, 0);
#pragma unroll
    for (int st = 0; st < KS; ++st) {
      if (st + 1 < KS) fetch((st + 1) & 1, (st + 1) * 16);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st & 1][i], bf[st & 1][j], acc[i][j], 0, 0, 0);
          if constexpr (DUAL) acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[st & 1][i], bf2[st & 1][j], acc2[i][j], 0, 0, 0);
        }
    }
  };

  if constexpr (!DEEP) {
    if (s_begin < s_end) {
      issue(s_begin, ma, mb, mb2);
      stash(0, ma, mb, mb2);
    }
    __syncthreads();
    int cur = 0;
    for (int sl = s_begin; sl < s_end; ++sl) {
      const bool more = sl + 1 < s_end;
      if (more) issue(sl + 1, ma, mb, mb2);
      multiply(cur);
      if constexpr (ST == 1) __syncthreads();
      const int nxt = (ST == 2) ? (cur ^ 1) : 0;
      if (more) stash(nxt, ma, mb, mb2);
      __syncthreads();
      cur = nxt;
    }
  } else {
    // register set 0 carries even slabs (relative to s_begin), set 1 odd ones; LDS stage = slab parity
    if (s_begin < s_end) {
      issue(s_begin, ma, mb, mb2);
      if (s_begin + 1 < s_end) issue(s_begin + 1, ma1, mb1, mb21);
      stash(0, ma, mb, mb2);
    }
    __syncthreads();
    int sl = s_begin;
    for (; sl + 1 < s_end; sl += 2) {
      if (sl + 2 < s_end) issue(sl + 2, ma, mb, mb2);
      multiply(0);
      stash(1, ma1, mb1, mb21);
      __syncthreads();
      if (sl + 3 < s_end) issue(sl + 3, ma1, mb1, mb21);
      multiply(1);
      if (sl + 2 < s_end) stash(0, ma, mb, mb2);
      __syncthreads();
    }
    if (sl < s_end) multiply(0);   // odd slab count: the last slab is already in LDS buffer 0
    __syncthreads();
  }

  // ---- epilogue.  Each 32x32 accumulator tile goes through a wave-private LDS patch so that a lane ends
  // up with four consecutive columns of one row: global accesses are then 16 bytes per lane, 128 bytes per
  // row segment.  (The operand tiles in LDS are dead here: the k loop ended with a barrier.)
  float* patch = (float*)smem + wave * 32 * SP;
  const int prow = lane >> 3, pcol = (lane & 7) * 4;
  auto to_patch = [&](const f32x16_t& t) {
#pragma unroll
    for (int v = 0; v < 16; ++v) patch[(8 * (v / 4) + 4 * lk + (v % 4)) * SP + lr] = t[v];
  };
  if constexpr (EPI == EPI_STORE) {
    float* C = (float*)tab[g.E.slot] + g.E.off + (long long)ks * g.E.split_stride;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        to_patch(acc[i][j]);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int row = row0 + wm * Cfg::WTM + i * 32 + prow + 8 * p;
          const int col = col0 + wn * Cfg::WTN + j * 32 + pcol;
          f32x4_t v = *(const f32x4_t*)(patch + (prow + 8 * p) * SP + pcol);
          gstore<f32x4_t>(C + (long long)row * g.E.ld + col, v);
        }
      }
  } else {
    // M <- (M + G) - (1-mu) (P R^T);   X <- X - eta sqrt(m/n) (P Q_new^T)
    float* Xp = (float*)tab[g.E.slotX];
    float* Mp = (float*)tab[g.E.slotM];
    const void* Gp = tab[g.E.slotG];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        long long idx[4];
        f32x4_t mv[4], xv[4], gv[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int row = row0 + wm * Cfg::WTM + i * 32 + prow + 8 * p;
          const int col = col0 + wn * Cfg::WTN + j * 32 + pcol;
          idx[p] = (long long)row * g.E.ld + col;
          mv[p] = gload<f32x4_t>(Mp + idx[p]);
          if constexpr (DUAL) xv[p] = g.E.x_overwrite ? f32x4_t{0.f, 0.f, 0.f, 0.f} : gload<f32x4_t>(Xp + idx[p]);
          if constexpr (GBF16) {
            const u32x2_t w = gload<u32x2_t>((const uint16_t*)Gp + idx[p]);
            gv[p] = f32x4_t{bf16_lo(w[0]), bf16_hi(w[0]), bf16_lo(w[1]), bf16_hi(w[1])};
          } else {
            gv[p] = gload<f32x4_t>((const float*)Gp + idx[p]);
          }
        }
        to_patch(acc[i][j]);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const f32x4_t a4 = *(const f32x4_t*)(patch + (prow + 8 * p) * SP + pcol);
          gstore<f32x4_t>(Mp + idx[p], (mv[p] + gv[p]) - g.E.c_m * a4);
        }
        if constexpr (DUAL) {
          to_patch(acc2[i][j]);
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const f32x4_t a4 = *(const f32x4_t*)(patch + (prow + 8 * p) * SP + pcol);
            gstore<f32x4_t>(Xp + idx[p], xv[p] - g.E.c_x * a4);
          }
        }
      }
  }
}

template <class Cfg, int ASRC, bool GBF16, int EPI, bool DUAL>
inline hipError_t launch_gemm2(GemmArgs g, int batch, hipStream_t stream) {
  const int kseg = g.nseg > 0 ? g.kseg : g.K;
  if (g.M % Cfg::BM || g.N % Cfg::BN || kseg % Cfg::BK || kseg <= 0) return hipErrorInvalidValue;
  if (g.tri_k && Cfg::BN % Cfg::BK) return hipErrorInvalidValue;
  g.tiles_m = g.M / Cfg::BM;
  g.tiles_n = g.N / Cfg::BN;
  if (g.splitk < 1) g.splitk = 1;
  // k_per_split counts k-slabs of the longest column tile; every split gets at least one slab
  const int total = (g.nseg > 0 ? g.nseg : 1) * (kseg / Cfg::BK);
  if (g.splitk > total) g.splitk = total;
  g.k_per_split = (total + g.splitk - 1) / g.splitk;
  g.splitk = (total + g.k_per_split - 1) / g.k_per_split;
  const long long blocks = (long long)g.tiles_m * g.tiles_n * g.splitk * batch;
  if (blocks <= 0) return hipSuccess;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  g.xcd_remap = (g.xcd_remap && (blocks % 8 == 0)) ? 1 : 0;
  hipLaunchKernelGGL((gemm2_kernel<Cfg, ASRC, GBF16, EPI, DUAL>), dim3((unsigned)blocks), dim3(Cfg::NT), 0, stream, g);
  return hipGetLastError();
}

// Number of split-K partial results launch_gemm2 will produce for these arguments (needed to size and
// reduce the partial buffers).
template <class Cfg>
inline int gemm2_effective_splitk(const GemmArgs& g) {
  const int kseg = g.nseg > 0 ? g.kseg : g.K;
  const int total = (g.nseg > 0 ? g.nseg : 1) * (kseg / Cfg::BK);
  int sk = g.splitk < 1 ? 1 : g.splitk;
  if (sk > total) sk = total;
  const int per = (total + sk - 1) / sk;
  return (total + per - 1) / per;
}

}  // namespace dion
