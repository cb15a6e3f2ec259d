// One panel step of the blocked right-looking Cholesky factorisation used by Cholesky-QR (Appendix A),
// fused into a single launch with no dependency between workgroups.
//
// For the 64-wide panel starting at row/column k0 of the rp x rp Gram matrix C (lower triangle):
//   L11 = chol(C11),  W11 = L11^-1                       (64 x 64)
//   L21 = C21 W11^T                                       (rows below the diagonal block)
//   C22 -= L21 L21^T                                      (trailing matrix, lower tiles)
// Workgroup 0 writes L11 and W11.  Every other workgroup owns one 64x64 tile (i, j) of the trailing
// matrix; it redoes the small diagonal factorisation itself (cheaper than a grid-wide wait), forms
// the two panel blocks L21_i and L21_j it needs with fp32 MFMA, and updates its tile.  The workgroups
// of column j = 1 also store their L21_i into L.
//
// Inside a workgroup the diagonal block is the latency-critical part, so it is spread over the waves:
//   wave 0  factors C11 column by column (row i of the block lives in the registers of lane i),
//   wave 1  follows one column behind and builds W11 = L11^-1 by forward substitution,
//   waves 2,3 meanwhile fetch the two panel blocks C21_i, C21_j into LDS.
// Waves 0 and 1 talk through LDS: broadcast reads (all lanes read one address) replace cross-lane
// shuffles, and a progress counter tells wave 1 which columns are final.  LDS operations of one wave
// are processed in issue order, so data stored before the counter is visible to whoever sees the counter.
#include <type_traits>
#include <utility>

#include "internal.hpp"

namespace dion {

namespace {
// compile-time loop: the body sees its index as a constant, so register arrays are indexed statically
template <int B, int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, B + Is>{}), ...);
}
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) static_for_impl<B>(std::make_integer_sequence<int, E - B>{}, f);
}
constexpr int CB = CHOL_NB;   // 64
constexpr int CBP = CB + 4;   // LDS row stride (floats): conflict-free 16-byte reads

// acc = As[64 x 64] * Bs[64 x 64]^T for this wave's 32x32 quadrant (LDS tiles, k contiguous).
__device__ __forceinline__ f32x16_t mma_64(const float* As, const float* Bs, int wm, int wn, int lr, int lk) {
  f32x16_t acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
  for (int kk = 0; kk < CB; kk += 8) {
    const f32x4_t a = *(const f32x4_t*)(As + (wm * 32 + lr) * CBP + kk + lk * 4);
    const f32x4_t b = *(const f32x4_t*)(Bs + (wn * 32 + lr) * CBP + kk + lk * 4);
#pragma unroll
    for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[s], acc, 0, 0, 0);
  }
  return acc;
}
}  // namespace

// Wave 0: factors the 64x64 block held in S0 (row i in lane i).  Publishes every finished column to
// LT / rsv and bumps *progress.  When Lout is given (writer workgroup) also stores L11 and the status.
__device__ __noinline__ void factor_wave(const float* S0, float* LT, float* col, float* rsv, volatile int* progress, int lane,
                                         float piv_lo, float piv_hi, float* Lout, long long ld, int* status) {
    float a[CB];
    static_for<0, CB>([&](auto kc) __attribute__((always_inline)) { a[decltype(kc)::value] = S0[lane * CBP + decltype(kc)::value]; });
    bool bad = false;
    static_for<0, CB>([&](auto jc) __attribute__((always_inline)) {
      constexpr int jj = decltype(jc)::value;
      f32x4_t cv[CB / 4];
      col[lane] = a[jj];
      float piv = col[jj];
      static_for<(jj + 1) / 4, CB / 4>([&](auto qc) __attribute__((always_inline)) {
        constexpr int q = decltype(qc)::value;
        cv[q] = *(const f32x4_t*)(col + 4 * q);
      });
      asm volatile("" ::: "memory");
      if (!(piv > piv_lo) || !(piv < piv_hi)) { bad = true; piv = 1.f; }
      float rs = __builtin_amdgcn_rsqf(piv);
      rs = rs * (1.5f - 0.5f * piv * rs * rs);                 // one Newton step on the hardware estimate
      const float lij = (lane == jj) ? piv * rs : a[jj] * rs;  // L[i][j]
      const float gj = a[jj] * (rs * rs);                      // L[i][j] / L[j][j]
      a[jj] = lij;
      LT[lane * CBP + jj] = lij;
      rsv[jj] = rs;   // every lane stores the same value: no branch in the column loop
      asm volatile("" ::: "memory");
      *progress = jj + 1;
      // trailing update inside the block: a[k] -= L[i][j] * L[k][j] = gj * col[k]
      static_for<(jj + 1) / 4, CB / 4>([&](auto qc) __attribute__((always_inline)) {
        constexpr int q = decltype(qc)::value;
        if constexpr (4 * q + 0 > jj) a[4 * q + 0] -= gj * cv[q][0];
        if constexpr (4 * q + 1 > jj) a[4 * q + 1] -= gj * cv[q][1];
        if constexpr (4 * q + 2 > jj) a[4 * q + 2] -= gj * cv[q][2];
        if constexpr (4 * q + 3 > jj) a[4 * q + 3] -= gj * cv[q][3];
      });
    });
    if (Lout) {
      static_for<0, CB>([&](auto kc) __attribute__((always_inline)) {
        constexpr int k = decltype(kc)::value;
        Lout[(long long)lane * ld + k] = (k <= lane) ? a[k] : 0.f;
      });
      if (bad && lane == 0) *status = 1;
    }
}

// Wave 1: W11 = L11^-1, following wave 0 column by column; leaves W11 (row-major) in S0.
__device__ __noinline__ void invert_wave(float* S0, const float* LT, const float* rsv, volatile int* progress, int lane) {
    // lane c builds column c of W = L^-1:  w_i = (delta_ic - sum_{k<i} L[i][k] w_k) / L[i][i]
    float w[CB];
    static_for<0, CB>([&](auto ic) __attribute__((always_inline)) {
      constexpr int ii = decltype(ic)::value;
      while (*progress <= ii) __builtin_amdgcn_s_sleep(1);   // wave 0 always gets there: it waits for nobody
      asm volatile("" ::: "memory");
      f32x4_t lv[CB / 4];
      static_for<0, (ii + 3) / 4>([&](auto qc) __attribute__((always_inline)) {
        constexpr int q = decltype(qc)::value;
        lv[q] = *(const f32x4_t*)(LT + ii * CBP + 4 * q);
      });
      const float rs = rsv[ii];
      asm volatile("" ::: "memory");
      float acc0 = (lane == ii) ? 1.f : 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
      static_for<0, (ii + 3) / 4>([&](auto qc) __attribute__((always_inline)) {
        constexpr int q = decltype(qc)::value;
        if constexpr (4 * q + 0 < ii) acc0 -= lv[q][0] * w[4 * q + 0];
        if constexpr (4 * q + 1 < ii) acc1 -= lv[q][1] * w[4 * q + 1];
        if constexpr (4 * q + 2 < ii) acc2 -= lv[q][2] * w[4 * q + 2];
        if constexpr (4 * q + 3 < ii) acc3 -= lv[q][3] * w[4 * q + 3];
      });
      w[ii] = ((acc0 + acc1) + (acc2 + acc3)) * rs;
      asm volatile("" : "+v"(w[ii]));   // keeps this row's arithmetic ahead of the next wait loop
    });
    static_for<0, CB>([&](auto rc) __attribute__((always_inline)) { S0[decltype(rc)::value * CBP + lane] = w[decltype(rc)::value]; });  // wave 0 read S0 only before it started
}

__global__ void __launch_bounds__(256, 2) chol_panel_kernel(void* const* table, int nslots, int slotC, int slotL, int slotW,
                                                            int k0, int rp, float piv_lo, float piv_hi, int mode, int skip_slot) {
  // mode 0: fused (workgroup 0 writes L11/W11, the others own tiles and redo the factorisation)
  // mode 1: diagonal block only (one workgroup per matrix)      mode 2: tiles only, W11 read back from memory
  // Modes 1+2 are used when there are so many tiles (large batches) that redoing the factorisation in
  // every workgroup would cost more than a second launch.
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  if (skip_slot >= 0 && *(const int*)tab[skip_slot] != 0) return;   // uniform for the whole workgroup
  float* C = (float*)tab[slotC];
  float* L = (float*)tab[slotL];
  float* W = (float*)tab[slotW];
  const long long ld = rp;
  __shared__ __attribute__((aligned(16))) float S0[CB * CBP];   // C11, later W11
  __shared__ __attribute__((aligned(16))) float S1[CB * CBP];   // C21_i, later L21_i
  __shared__ __attribute__((aligned(16))) float S2[CB * CBP];   // C21_j, later L21_j
  __shared__ __attribute__((aligned(16))) float LT[CB * CBP];   // finished rows of L11
  __shared__ __attribute__((aligned(16))) float col[CB];        // current column, shared by the lanes of wave 0
  __shared__ float rsv[CB];                                     // 1 / L[j][j]
  __shared__ volatile int progress;                             // number of factored columns
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave & 1, wn = wave >> 1, lr = lane & 31, lk = lane >> 5;

  // tile (i, j), 1 <= j <= i, in units of 64 rows/columns below/right of the diagonal block
  const bool writer = mode != 2 && blockIdx.x == 0;
  int i = 1, j = 1;
  if (!writer) {
    const int q = (mode == 2) ? blockIdx.x : blockIdx.x - 1;
    i = (int)((sqrtf(8.f * q + 1.f) - 1.f) * 0.5f) + 1;
    while ((i - 1) * i / 2 > q) --i;
    while (i * (i + 1) / 2 <= q) ++i;
    j = q - (i - 1) * i / 2 + 1;
  }
  const long long rowi = k0 + (long long)CB * i, rowj = k0 + (long long)CB * j;

  for (int idx = t; idx < CB * CB; idx += 256) {
    const int rr = idx >> 6, cc = idx & 63;
    const long long at = (long long)(k0 + rr) * ld + k0 + cc;
    S0[rr * CBP + cc] = (mode == 2) ? W[at] : ((cc <= rr) ? C[at] : 0.f);
  }
  if (t == 0) progress = 0;
  // this thread's 16 entries of the trailing tile, fetched now so that they arrive during the factorisation
  float cold[16];
  if (!writer) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wm * 32 + 8 * (v / 4) + 4 * lk + (v % 4), cc = wn * 32 + lr;
      cold[v] = C[(rowi + row) * ld + rowj + cc];
    }
  }
  __syncthreads();

  if (mode == 2) {
    for (int idx = t; idx < CB * CB; idx += 256) {
      const int rr = idx >> 6, cc = idx & 63;
      S1[rr * CBP + cc] = C[(rowi + rr) * ld + k0 + cc];
      if (j != i) S2[rr * CBP + cc] = C[(rowj + rr) * ld + k0 + cc];
    }
  } else if (wave == 0) {
    factor_wave(S0, LT, col, rsv, &progress, lane, piv_lo, piv_hi, writer ? L + (long long)k0 * ld + k0 : nullptr, ld,
                (int*)tab[SLOT_STATUS]);
  } else if (wave == 1) {
    invert_wave(S0, LT, rsv, &progress, lane);
  } else if (!writer) {
    for (int idx = t - 128; idx < CB * CB; idx += 128) {
      const int rr = idx >> 6, cc = idx & 63;
      S1[rr * CBP + cc] = C[(rowi + rr) * ld + k0 + cc];
      if (j != i) S2[rr * CBP + cc] = C[(rowj + rr) * ld + k0 + cc];
    }
  }
  __syncthreads();
  if (writer) {
    for (int idx = t; idx < CB * CB; idx += 256) {
      const int rr = idx >> 6, cc = idx & 63;
      W[(long long)(k0 + rr) * ld + k0 + cc] = S0[rr * CBP + cc];
    }
    return;
  }
  const f32x16_t li = mma_64(S1, S0, wm, wn, lr, lk);   // L21_i = C21_i W11^T
  f32x16_t lj = li;
  if (j != i) lj = mma_64(S2, S0, wm, wn, lr, lk);
  __syncthreads();
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = wm * 32 + 8 * (v / 4) + 4 * lk + (v % 4), cc = wn * 32 + lr;
    S1[row * CBP + cc] = li[v];
    if (j != i) S2[row * CBP + cc] = lj[v];
    if (j == 1) L[(rowi + row) * ld + k0 + cc] = li[v];
  }
  __syncthreads();
  const f32x16_t up = mma_64(S1, (j != i) ? S2 : S1, wm, wn, lr, lk);   // L21_i L21_j^T
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = wm * 32 + 8 * (v / 4) + 4 * lk + (v % 4), cc = wn * 32 + lr;
    C[(rowi + row) * ld + rowj + cc] = cold[v] - up[v];
  }
}

hipError_t launch_chol_panel(void* const* table, int nslots, int batch, int slotC, int slotL, int slotW, int k0, int rp,
                             float piv_lo, float piv_hi, int skip_slot, hipStream_t s) {
  const int nb = (rp - k0 - CB) / CB;
  const int tiles = nb * (nb + 1) / 2;
  if ((long long)(1 + tiles) * batch <= 1024 || tiles == 0) {
    hipLaunchKernelGGL(chol_panel_kernel, dim3(1 + tiles, batch), dim3(256), 0, s, table, nslots, slotC, slotL, slotW, k0, rp,
                       piv_lo, piv_hi, 0, skip_slot);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(chol_panel_kernel, dim3(1, batch), dim3(256), 0, s, table, nslots, slotC, slotL, slotW, k0, rp, piv_lo, piv_hi, 1, skip_slot);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(chol_panel_kernel, dim3(tiles, batch), dim3(256), 0, s, table, nslots, slotC, slotL, slotW, k0, rp, piv_lo,
                     piv_hi, 2, skip_slot);
  return hipGetLastError();
}

}  // namespace dion
