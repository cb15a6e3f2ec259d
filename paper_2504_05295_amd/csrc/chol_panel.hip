// One panel step of the blocked right-looking Cholesky factorisation used by Cholesky-QR (Appendix A),
// fused into a single launch with no dependency between workgroups.
//
// For the 64-wide panel starting at row/column k0 of the rp x rp Gram matrix C (lower triangle):
//   L11 = chol(C11),  W11 = L11^-1                       (64 x 64, one wavefront, registers only)
//   L21 = C21 W11^T                                       (rows below the diagonal block)
//   C22 -= L21 L21^T                                      (trailing matrix, lower tiles)
// Workgroup 0 writes L11 and W11.  Every other workgroup owns one 64x64 tile (i, j) of the trailing
// matrix; it redoes the tiny diagonal factorisation itself (that is cheaper than a grid-wide wait),
// forms the two panel blocks L21_i and L21_j it needs with fp32 MFMA, and updates its tile.  The
// workgroups of column j = 1 also store their L21_i into L.
#include "internal.hpp"

namespace dion {

namespace {
constexpr int CB = CHOL_NB;   // 64
constexpr int CBP = CB + 4;   // LDS row stride (floats): conflict-free 16-byte reads

// acc (+)= As[64 x 64] * Bs[64 x 64]^T for this wave's 32x32 quadrant (LDS tiles, k contiguous).
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

__global__ void __launch_bounds__(256) chol_panel_kernel(void* const* table, int nslots, int slotC, int slotL, int slotW,
                                                         int k0, int rp, float piv_lo, float piv_hi) {
  void* const* tab = table + (size_t)blockIdx.y * nslots;
  float* C = (float*)tab[slotC];
  float* L = (float*)tab[slotL];
  float* W = (float*)tab[slotW];
  const long long ld = rp;
  __shared__ __attribute__((aligned(16))) float S0[CB * CBP];
  __shared__ __attribute__((aligned(16))) float S1[CB * CBP];
  __shared__ __attribute__((aligned(16))) float S2[CB * CBP];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;

  for (int idx = t; idx < CB * CB; idx += 256) {
    const int rr = idx >> 6, cc = idx & 63;
    S0[rr * CBP + cc] = (cc <= rr) ? C[(long long)(k0 + rr) * ld + k0 + cc] : 0.f;
  }
  __syncthreads();
  if (wave == 0) {
    // Lane i holds row i of the block in a[].  Cross-lane traffic goes through LDS broadcast reads
    // (every lane reads the same address): `col` carries the current column to all lanes, `LT` keeps
    // the finished rows of L for the inverse.  LDS operations of one wavefront complete in order, so no
    // barrier is needed inside this section.
    float a[CB], w[CB];
#pragma unroll
    for (int k = 0; k < CB; ++k) a[k] = S0[lane * CBP + k];
    float* col = S1;
    float* LT = S2;
    bool bad = false;
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      col[lane] = a[j];
      float piv = col[j];
      if (!(piv > piv_lo) || !(piv < piv_hi)) { bad = true; piv = 1.f; }
      float rs = __builtin_amdgcn_rsqf(piv);
      rs = rs * (1.5f - 0.5f * piv * rs * rs);   // one Newton step on the hardware estimate
      const float lij = (lane == j) ? piv * rs : a[j] * rs;   // L[i][j]
      const float gj = a[j] * (rs * rs);                      // L[i][j] / L[j][j]
      a[j] = lij;
      // trailing update inside the block: a[k] -= L[i][j] * L[k][j] = gj * col[k]
#pragma unroll
      for (int q = (j + 1) / 4; q < CB / 4; ++q) {
        const f32x4_t c4 = *(const f32x4_t*)(col + 4 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (4 * q + e > j) a[4 * q + e] -= gj * c4[e];
      }
      LT[lane * CBP + j] = lij;
      // row j of W = L^-1 (lane c holds column c): w_j = (delta_jc - sum_{k<j} L[j][k] w_k) / L[j][j]
      float acc = (lane == j) ? 1.f : 0.f;
#pragma unroll
      for (int q = 0; q < (j + 3) / 4; ++q) {
        const f32x4_t l4 = *(const f32x4_t*)(LT + j * CBP + 4 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (4 * q + e < j) acc -= l4[e] * w[4 * q + e];
      }
      w[j] = acc * rs;
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) S0[i * CBP + lane] = w[i];
    if (blockIdx.x == 0) {
#pragma unroll
      for (int k = 0; k < CB; ++k) L[(long long)(k0 + lane) * ld + k0 + k] = (k <= lane) ? a[k] : 0.f;
      if (bad && lane == 0) *(int*)tab[SLOT_STATUS] = 1;
    }
  }
  __syncthreads();
  if (blockIdx.x == 0) {
    for (int idx = t; idx < CB * CB; idx += 256) {
      const int rr = idx >> 6, cc = idx & 63;
      W[(long long)(k0 + rr) * ld + k0 + cc] = S0[rr * CBP + cc];
    }
    return;
  }
  // tile (i, j), 1 <= j <= i, in units of 64 rows/columns below/right of the diagonal block
  const int q = blockIdx.x - 1;
  int i = (int)((sqrtf(8.f * q + 1.f) - 1.f) * 0.5f) + 1;
  while ((i - 1) * i / 2 > q) --i;
  while (i * (i + 1) / 2 <= q) ++i;
  const int j = q - (i - 1) * i / 2 + 1;
  const long long rowi = k0 + (long long)CB * i, rowj = k0 + (long long)CB * j;
  for (int idx = t; idx < CB * CB; idx += 256) {
    const int rr = idx >> 6, cc = idx & 63;
    S1[rr * CBP + cc] = C[(rowi + rr) * ld + k0 + cc];
    if (j != i) S2[rr * CBP + cc] = C[(rowj + rr) * ld + k0 + cc];
  }
  __syncthreads();
  const int wm = wave & 1, wn = wave >> 1, lr = lane & 31, lk = lane >> 5;
  const f32x16_t li = mma_64(S1, S0, wm, wn, lr, lk);   // L21_i = C21_i W11^T
  f32x16_t lj = li;
  if (j != i) lj = mma_64(S2, S0, wm, wn, lr, lk);
  __syncthreads();
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = wm * 32 + 8 * (v / 4) + 4 * lk + (v % 4), col = wn * 32 + lr;
    S1[row * CBP + col] = li[v];
    if (j != i) S2[row * CBP + col] = lj[v];
    if (j == 1) L[(rowi + row) * ld + k0 + col] = li[v];
  }
  __syncthreads();
  const f32x16_t up = mma_64(S1, (j != i) ? S2 : S1, wm, wn, lr, lk);   // L21_i L21_j^T
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = wm * 32 + 8 * (v / 4) + 4 * lk + (v % 4), col = wn * 32 + lr;
    float* c = C + (rowi + row) * ld + rowj + col;
    *c -= up[v];
  }
}

hipError_t launch_chol_panel(void* const* table, int nslots, int batch, int slotC, int slotL, int slotW, int k0, int rp,
                             float piv_lo, float piv_hi, hipStream_t s) {
  const int nb = (rp - k0 - CB) / CB;
  const int tiles = nb * (nb + 1) / 2;
  hipLaunchKernelGGL(chol_panel_kernel, dim3(1 + tiles, batch), dim3(256), 0, s, table, nslots, slotC, slotL, slotW, k0, rp, piv_lo,
                     piv_hi);
  return hipGetLastError();
}

}  // namespace dion
